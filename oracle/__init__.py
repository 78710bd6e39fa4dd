"""CPU oracle of the Tucker-2 convolution layer.  Test infrastructure only; see tdc_oracle.c."""
