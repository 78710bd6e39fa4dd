// Hardware-aware rank selection (host only): the first step of the paper's Algorithm 1 with the
// rules of section 6.  For every layer in network order:
//   1. the FLOPs budget B (a target reduction ratio over all listed layers) gives the layer a cap:
//      it may keep at most (1 - b) * F MACs, where b is the reduction still owed by this and the
//      following layers divided by their dense MACs -- so a layer that stays dense passes its share
//      on to the rest, as the paper describes, and one that removes more than its share relaxes it;
//   2. among the table entries within the cap, those of minimal measured latency (within the
//      caller's tie tolerance, since measured plateaus never tie exactly) are kept and the largest
//      ranks among them win (Algorithm 1: max of the argmin);
//   3. the layer is decomposed only if that latency beats (1 - theta) times the latency of its
//      original convolution.
// MACs follow the complexity formula of section 3, batch included.
#include <cstddef>

#include "tdc.h"

namespace {

struct Macs {
    double dense, in_px, core_px, out_px;   // P(D1, D2) = in_px*D1 + core_px*D1*D2 + out_px*D2
};

Macs macs_of(const tdc_shape &s)
{
    const double Ho = tdc_out_size(s.H, s.K, s.stride, s.pad), Wo = tdc_out_size(s.W, s.K, s.stride, s.pad);
    Macs m;
    m.dense = (double)s.batch * Ho * Wo * s.K * s.K * s.C * s.N;
    m.in_px = (double)s.batch * s.H * s.W * s.C;
    m.core_px = (double)s.batch * Ho * Wo * s.K * s.K;
    m.out_px = (double)s.batch * Ho * Wo * s.N;
    return m;
}

bool larger_ranks(const tdc_rank_entry &a, const tdc_rank_entry &b)
{
    const long pa = (long)a.R1 * a.R2, pb = (long)b.R1 * b.R2;
    if (pa != pb) return pa > pb;
    if (a.R1 + a.R2 != b.R1 + b.R2) return a.R1 + a.R2 > b.R1 + b.R2;
    return a.R1 > b.R1;
}

}  // namespace

extern "C" int tdc_select_ranks(const tdc_rank_layer *layers, int n_layers, double budget, double theta,
                                double tie_tol, tdc_rank_choice *out)
{
    if (!layers || !out) return TDC_ERR_NULL;
    if (n_layers < 1 || !(budget >= 0.0) || !(budget < 1.0) || !(theta >= 0.0) || !(theta < 1.0) || !(tie_tol >= 0.0))
        return TDC_ERR_BAD_SHAPE;
    double total = 0.0;
    for (int l = 0; l < n_layers; ++l) {
        const tdc_shape &s = layers[l].shape;
        if (s.batch < 1 || s.C < 1 || s.N < 1 || s.H < 1 || s.W < 1 || s.K < 1 || s.stride < 1 || s.pad < 0) return TDC_ERR_BAD_SHAPE;
        if (tdc_out_size(s.H, s.K, s.stride, s.pad) < 1 || tdc_out_size(s.W, s.K, s.stride, s.pad) < 1) return TDC_ERR_BAD_SHAPE;
        if (layers[l].n_entries < 0 || (layers[l].n_entries > 0 && !layers[l].table)) return TDC_ERR_NULL;
        if (!(layers[l].dense_latency_us > 0.0)) return TDC_ERR_BAD_SHAPE;
        for (int e = 0; e < layers[l].n_entries; ++e)
            if (layers[l].table[e].R1 < 1 || layers[l].table[e].R2 < 1 || !(layers[l].table[e].latency_us > 0.0)) return TDC_ERR_BAD_SHAPE;
        total += macs_of(s).dense;
    }
    const double need = budget * total;
    double removed = 0.0, remaining = total;
    for (int l = 0; l < n_layers; ++l) {
        const tdc_rank_layer &L = layers[l];
        const Macs m = macs_of(L.shape);
        double b = (need - removed) / remaining;
        if (b < 0.0) b = 0.0;
        const double cap = (1.0 - b) * m.dense;
        double t_min = -1.0;
        for (int e = 0; e < L.n_entries; ++e) {
            const tdc_rank_entry &c = L.table[e];
            const double P = m.in_px * c.R1 + m.core_px * c.R1 * c.R2 + m.out_px * c.R2;
            if (P <= cap && (t_min < 0.0 || c.latency_us < t_min)) t_min = c.latency_us;
        }
        const tdc_rank_entry *best = nullptr;
        if (t_min >= 0.0)
            for (int e = 0; e < L.n_entries; ++e) {
                const tdc_rank_entry &c = L.table[e];
                const double P = m.in_px * c.R1 + m.core_px * c.R1 * c.R2 + m.out_px * c.R2;
                if (P <= cap && c.latency_us <= (1.0 + tie_tol) * t_min && (!best || larger_ranks(c, *best))) best = &c;
            }
        if (best && best->latency_us >= (1.0 - theta) * L.dense_latency_us) best = nullptr;
        tdc_rank_choice &o = out[l];
        if (best) {
            const double P = m.in_px * best->R1 + m.core_px * best->R1 * best->R2 + m.out_px * best->R2;
            o.decomposed = 1; o.R1 = best->R1; o.R2 = best->R2; o.latency_us = best->latency_us; o.macs = P;
            removed += m.dense - P;
        } else {
            o.decomposed = 0; o.R1 = 0; o.R2 = 0; o.latency_us = L.dense_latency_us; o.macs = m.dense;
        }
        remaining -= m.dense;
    }
    return TDC_OK;
}
