#ifndef TDC_DIV_H
#define TDC_DIV_H

// Division by a launch-time constant (this header is free of HIP, so host-only code can check it).  An integer division costs a lone wavefront some 300 cycles
// (a dependent chain of ~25 VALU instructions), and a kernel prologue here has half a dozen of
// them between its first instruction and its first load: at microsecond kernel durations that is
// measurable (0.15 us each).  The host precomputes a multiplier instead (Granlund & Montgomery):
//   m = floor(2^32 * (2^L - d) / d) + 1,  L = ceil(log2 d),  q = (t + ((x - t) >> min(L,1))) >> max(L-1,0),
//   t = mulhi(m, x); exact for every 0 <= x < 2^32 and 1 <= d < 2^31.
struct TdcDiv {
    unsigned m, sh1, sh2;
};

inline TdcDiv tdc_make_div(unsigned d)
{
    unsigned L = 0;
    while ((1ull << L) < d) ++L;
    TdcDiv r;
    r.m = (unsigned)((((1ull << 32) * ((1ull << L) - d)) / d) + 1);
    r.sh1 = L < 1 ? L : 1;
    r.sh2 = L > 1 ? L - 1 : 0;
    return r;
}

// The quotient x / d from t = high 32 bits of m * x (the device takes t from __umulhi).
#ifdef __HIPCC__
__host__ __device__
#endif
inline unsigned tdc_div_from_hi(unsigned x, unsigned t, const TdcDiv &d)
{
    return (t + ((x - t) >> d.sh1)) >> d.sh2;
}

#endif
