// CHAIN kernel instances whose stage-1 register tiles are 4 channel blocks high (see tdc_chain_kernel.h).
#include "tdc_chain_kernel.h"

hipError_t tdc_launch_chain_mb4(const TdcChainArgs &a, int nb2, int pb, bool weights_in_lds, int lay, dim3 grid, dim3 block,
                                size_t lds_bytes, hipStream_t s, bool prepare_only)
{
    return tdc_launch_chain_instance<4>(a, nb2, pb, weights_in_lds, lay, grid, block, lds_bytes, s, prepare_only);
}
