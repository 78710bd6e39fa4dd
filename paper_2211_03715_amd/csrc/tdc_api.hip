// C ABI of libtdc.so: plans, validation, weight re-layout bookkeeping and launch dispatch.
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "tdc_internal.h"

struct tdc_plan {
    tdc_shape shape;
    TdcDims dims;
    tdc_tuning tuning;
    TdcFusedGeom geom;
    int device;
    float *z1, *z2;                    // intermediates (NAIVE, SPLIT)
    float *uin_p, *core_p, *uout_p;    // re-laid-out weights (SPLIT, FUSED, CHAIN; MERGED keeps the merged kernel in core_p)
    float *wm;                         // MERGED: core x_2 U_out in the caller's layout, before re-layout
    const float *packed_from[3];       // caller pointers the stored copy was made from, or NULLs
    unsigned *arrive = nullptr;        // MERGED_XCD: arrival words, 8 XCDs x 32 roles, then the count of waits that gave up
    unsigned *status = nullptr;        // MERGED_XCD: one word of pinned host memory the kernel writes when it cannot run here
    unsigned wait_limit = 512;
    size_t ws_bytes;
    double model_us;                   // the selector's latency estimate for this tuning
    char desc[320];
};

namespace {

__global__ void tdc_null_kernel() {}

struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) return;
        ok = (prev == dev) || (hipSetDevice(dev) == hipSuccess);
        if (prev == dev) prev = -1;
    }
    ~DeviceGuard()
    {
        if (prev >= 0) (void)hipSetDevice(prev);
    }
};

// NHWC kernels move x, y and the residual in 16-byte pieces
bool misaligned16(const void *x, const void *y, const void *residual)
{
    return (((uintptr_t)x | (uintptr_t)y | (uintptr_t)residual) & 15u) != 0;
}

bool same_shape(const tdc_shape &a, const tdc_shape &b)
{
    return a.batch == b.batch && a.C == b.C && a.N == b.N && a.H == b.H && a.W == b.W && a.R1 == b.R1 &&
           a.R2 == b.R2 && a.K == b.K && a.stride == b.stride && a.pad == b.pad && a.layout == b.layout;
}

int validate(const tdc_shape &s)
{
    if (s.batch < 1 || s.C < 1 || s.N < 1 || s.H < 1 || s.W < 1 || s.R1 < 1 || s.R2 < 1 || s.K < 1) return TDC_ERR_BAD_SHAPE;
    if (s.stride < 1 || s.pad < 0) return TDC_ERR_BAD_SHAPE;
    if ((long)s.H + 2L * s.pad < s.K || (long)s.W + 2L * s.pad < s.K) return TDC_ERR_BAD_SHAPE;
    if (s.layout != 0 && s.layout != 1) return TDC_ERR_UNSUPPORTED;
    if (s.layout == 1 && (s.C % 4 || s.N % 4)) return TDC_ERR_UNSUPPORTED;   // NHWC moves channels four at a time
    if (s.K > 7 || s.stride > 4 || s.pad > s.K - 1) return TDC_ERR_UNSUPPORTED;
    const long Ho = tdc_out_size(s.H, s.K, s.stride, s.pad), Wo = tdc_out_size(s.W, s.K, s.stride, s.pad);
    const long lim = 0x7fffffffL;
    const long r1p = (s.R1 + 15L) / 16 * 16, r2p = (s.R2 + 15L) / 16 * 16, np = (s.N + 15L) / 16 * 16;
    const long cp = (s.C + 15L) / 16 * 16;
    if ((double)s.batch * s.C * s.H * s.W >= lim || (double)s.batch * np * Ho * Wo >= lim) return TDC_ERR_UNSUPPORTED;
    if ((double)s.batch * r1p * s.H * s.W >= lim || (double)s.batch * r2p * Ho * Wo >= lim) return TDC_ERR_UNSUPPORTED;
    if ((double)cp * r1p >= lim || (double)r1p * r2p * s.K * s.K >= lim || (double)r2p * np >= lim) return TDC_ERR_UNSUPPORTED;
    // one image of any activation and each re-laid-out weight array must fit a 2 GiB buffer descriptor
    const double lim4 = (double)lim / 4;
    if ((double)cp * s.H * s.W >= lim4 || (double)r1p * s.H * s.W >= lim4 || (double)r2p * Ho * Wo >= lim4) return TDC_ERR_UNSUPPORTED;
    if ((double)np * Ho * Wo >= lim4) return TDC_ERR_UNSUPPORTED;
    if ((double)cp * r1p >= lim4 || (double)r1p * r2p * s.K * s.K >= lim4 || (double)r2p * np >= lim4) return TDC_ERR_UNSUPPORTED;
    if (s.batch > 65535) return TDC_ERR_UNSUPPORTED;   // images ride in the grid's y dimension
    return TDC_OK;
}

// The shape the kernels see: a DENSE plan runs the stage-2 kernel with the layer's own channel
// counts standing in for the ranks.
tdc_shape kernel_shape(const tdc_shape &s, int variant)
{
    tdc_shape k = s;
    if (variant == TDC_VARIANT_DENSE) {
        k.R1 = s.C;
        k.R2 = s.N;
    }
    return k;
}

TdcDims make_dims(const tdc_shape &s)
{
    TdcDims d;
    d.B = s.batch; d.C = s.C; d.N = s.N; d.H = s.H; d.W = s.W; d.R1 = s.R1; d.R2 = s.R2; d.K = s.K;
    d.stride = s.stride; d.pad = s.pad;
    d.Ho = tdc_out_size(s.H, s.K, s.stride, s.pad);
    d.Wo = tdc_out_size(s.W, s.K, s.stride, s.pad);
    d.NB1 = (s.R1 + 15) / 16; d.NB2 = (s.R2 + 15) / 16; d.NB3 = (s.N + 15) / 16;
    d.KG1 = (s.C + 15) / 16;
    d.nhwc = s.layout == 1;
    d.s1_runs = 0;       // decided with the variant, see tdc_plan_create_tuned
    return d;
}

int check_tuning(const tdc_plan &p, const TdcDeviceInfo &dev)
{
    const tdc_tuning &t = p.tuning;
    if (t.variant == TDC_VARIANT_NAIVE) return TDC_OK;
    for (int i = 0; i < 3; ++i)
        if (t.waves[i] < 1 || t.waves[i] > 8) return TDC_ERR_BAD_TUNING;
    const bool dense = t.variant == TDC_VARIANT_DENSE;   // one kernel, tiled over the blocks of N
    // MERGED, FUSED_MERGED: the second field tiles the blocks of N
    const bool merged = t.variant == TDC_VARIANT_MERGED || t.variant == TDC_VARIANT_FUSED_MERGED ||
                        t.variant == TDC_VARIANT_MERGED_XCD;
    const int nb[3] = {dense ? p.dims.NB2 : p.dims.NB1, merged ? p.dims.NB3 : p.dims.NB2, dense ? p.dims.NB2 : p.dims.NB3};
    for (int i = 0; i < 3; ++i)
        if (t.mb[i] < 1 || nb[i] % t.mb[i]) return TDC_ERR_BAD_TUNING;   // whole register tiles only
    if (t.variant == TDC_VARIANT_DENSE) {
        if (!tdc_gemm_unit_supported(t.mb[1], t.pb[1])) return TDC_ERR_BAD_TUNING;
        if (t.waves[1] > 1 && (size_t)t.waves[1] * t.mb[1] * t.pb[1] * 1024 > 64 * 1024) return TDC_ERR_BAD_TUNING;
        return TDC_OK;
    }
    if (t.variant == TDC_VARIANT_FUSED_MERGED) {
        if (t.tile_h < 1 || t.tile_w < 1 || t.tile_h * t.tile_w > 64) return TDC_ERR_BAD_TUNING;
        if (!tdc_fm_supported(p.dims, t.tile_h, t.tile_w, t.waves[0], t.mb[0], t.mb[1])) return TDC_ERR_BAD_TUNING;
        if ((long)p.geom.lds_bytes > dev.lds_per_wg) return TDC_ERR_BAD_TUNING;
        return TDC_OK;
    }
    if (t.variant == TDC_VARIANT_MERGED) {
        for (int i = 0; i < 2; ++i) {
            if (!tdc_gemm_unit_supported(t.mb[i], t.pb[i])) return TDC_ERR_BAD_TUNING;
            if (t.waves[i] > 1 && (size_t)t.waves[i] * t.mb[i] * t.pb[i] * 1024 > 64 * 1024) return TDC_ERR_BAD_TUNING;
        }
        return TDC_OK;
    }
    if (t.variant == TDC_VARIANT_MERGED_XCD) {
        if (!tdc_merged_xcd_supported(t)) return TDC_ERR_BAD_TUNING;
        // eight copies of z1, each behind a buffer descriptor and a 32-bit stride
        if ((size_t)p.dims.B * 16 * p.dims.NB1 * p.dims.H * p.dims.W * sizeof(float) >= (1ull << 28)) return TDC_ERR_BAD_TUNING;
        // the whole grid must be resident for its barrier to open: one workgroup per compute unit is what is counted on
        if (dev.cus % 8 || tdc_merged_xcd_grid(p.dims, t) > dev.cus) return TDC_ERR_BAD_TUNING;
        return TDC_OK;
    }
    if (t.variant == TDC_VARIANT_SPLIT) {
        for (int i = 0; i < 3; ++i) {
            if (!tdc_gemm_unit_supported(t.mb[i], t.pb[i])) return TDC_ERR_BAD_TUNING;
            if (t.waves[i] > 1 && (size_t)t.waves[i] * t.mb[i] * t.pb[i] * 1024 > 64 * 1024) return TDC_ERR_BAD_TUNING;
        }
        return TDC_OK;
    }
    if (t.variant == TDC_VARIANT_FUSED) {
        if (t.tile_h < 1 || t.tile_w < 1 || t.tile_h * t.tile_w > 4096) return TDC_ERR_BAD_TUNING;
        if (!tdc_fused_unit_supported(t.mb[0], t.mb[1], t.mb[2], t.pb[0])) return TDC_ERR_BAD_TUNING;
        if ((long)p.geom.lds_bytes > dev.lds_per_wg) return TDC_ERR_BAD_TUNING;
        // the kernels number their workgroups over the whole grid, batch included, in 32-bit arithmetic
        if ((long long)p.geom.tiles_x * p.geom.tiles_y * p.dims.B > 0x7fffffffLL) return TDC_ERR_BAD_TUNING;
        return TDC_OK;
    }
    if (t.variant == TDC_VARIANT_CHAIN) {
        if (t.tile_h < 1 || t.tile_w < 1 || t.tile_h * t.tile_w > 4096) return TDC_ERR_BAD_TUNING;
        if (!tdc_chain_supported(p.dims.NB2, t.mb[0], t.pb[0])) return TDC_ERR_BAD_TUNING;
        if ((long)p.geom.lds_bytes > dev.lds_per_wg) return TDC_ERR_BAD_TUNING;
        if ((long long)p.geom.tiles_x * p.geom.tiles_y * p.dims.B > 0x7fffffffLL) return TDC_ERR_BAD_TUNING;
        return TDC_OK;
    }
    return TDC_ERR_BAD_TUNING;
}

void describe(tdc_plan &p)
{
    const tdc_tuning &t = p.tuning;
    const char *names[] = {"auto", "naive", "split", "fused"};
    if (t.variant == TDC_VARIANT_CHAIN)
        snprintf(p.desc, sizeof(p.desc),
                 "chain tile=%dx%d in=%dx%d waves=%d units(mb1,pb)=(%d,%d) grid=%dx%d lds=%zuB%s model=%.1fus",
                 t.tile_h, t.tile_w, p.geom.QH, p.geom.QW, t.waves[0], t.mb[0], t.pb[0],
                 p.geom.tiles_x * p.geom.tiles_y, p.dims.B, p.geom.lds_bytes, p.geom.weights_in_lds ? " wlds" : "", p.model_us);
    else if (t.variant == TDC_VARIANT_FUSED)
        snprintf(p.desc, sizeof(p.desc),
                 "fused tile=%dx%d in=%dx%d waves=%d units(mb1,mb2,mb3,pb)=(%d,%d,%d,%d) grid=%dx%d lds=%zuB%s model=%.1fus",
                 t.tile_h, t.tile_w, p.geom.QH, p.geom.QW, t.waves[0], t.mb[0], t.mb[1], t.mb[2], t.pb[0],
                 p.geom.tiles_x * p.geom.tiles_y, p.dims.B, p.geom.lds_bytes, p.geom.weights_in_lds ? " wlds" : "", p.model_us);
    else if (t.variant == TDC_VARIANT_FUSED_MERGED)
        snprintf(p.desc, sizeof(p.desc),
                 "fused-merged tile=%dx%d in=%dx%d waves=%d mb1=%d n-blocks/wg=%d k-slices=%d grid=%dx%d lds=%zuB model=%.1fus",
                 t.tile_h, t.tile_w, p.geom.QH, p.geom.QW, t.waves[0], t.mb[0], t.mb[1], t.waves[0] / t.mb[1],
                 p.geom.tiles_x * p.geom.tiles_y * (p.dims.NB3 / t.mb[1]), p.dims.B, p.geom.lds_bytes, p.model_us);
    else if (t.variant == TDC_VARIANT_MERGED)
        snprintf(p.desc, sizeof(p.desc), "merged stage(mb,pb,waves)= s1(%d,%d,%d) s23(%d,%d,%d) model=%.1fus", t.mb[0], t.pb[0],
                 t.waves[0], t.mb[1], t.pb[1], t.waves[1], p.model_us);
    else if (t.variant == TDC_VARIANT_MERGED_XCD)
        snprintf(p.desc, sizeof(p.desc), "merged-xcd split-k(s1,s23)=(%d,%d) grid=%d model=%.1fus", t.waves[0], t.waves[1],
                 tdc_merged_xcd_grid(p.dims, t), p.model_us);
    else if (t.variant == TDC_VARIANT_DENSE)
        snprintf(p.desc, sizeof(p.desc), "dense %dx%d conv (mb,pb,waves)=(%d,%d,%d) model=%.1fus", p.dims.K, p.dims.K,
                 t.mb[1], t.pb[1], t.waves[1], p.model_us);
    else if (t.variant == TDC_VARIANT_SPLIT)
        snprintf(p.desc, sizeof(p.desc), "split stage(mb,pb,waves)= s1(%d,%d,%d) s2(%d,%d,%d) s3(%d,%d,%d) model=%.1fus",
                 t.mb[0], t.pb[0], t.waves[0], t.mb[1], t.pb[1], t.waves[1], t.mb[2], t.pb[2], t.waves[2], p.model_us);
    else
        snprintf(p.desc, sizeof(p.desc), "%s", names[t.variant & 3]);
}

}  // namespace

hipError_t tdc_allow_lds(const void *fn, size_t bytes)
{
    if (bytes <= 48 * 1024) return hipSuccess;
    struct Granted {
        const void *fn;
        int device;
        size_t bytes;
    };
    static std::mutex lock;
    static std::vector<Granted> table;
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> hold(lock);
    for (Granted &g : table)
        if (g.fn == fn && g.device == device) {
            if (g.bytes >= bytes) return hipSuccess;
            e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
            if (e == hipSuccess) g.bytes = bytes;
            return e;
        }
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) table.push_back(Granted{fn, device, bytes});
    return e;
}

extern "C" {

int tdc_version(void) { return 100; }

int tdc_out_size(int in, int K, int stride, int pad)
{
    if (in < 1 || K < 1 || stride < 1 || pad < 0 || in + 2 * pad < K) return 0;
    return (in + 2 * pad - K) / stride + 1;
}

const char *tdc_status_string(int status)
{
    switch (status) {
        case TDC_OK: return "ok";
        case TDC_ERR_NULL: return "null pointer argument";
        case TDC_ERR_BAD_SHAPE: return "invalid layer shape";
        case TDC_ERR_SHAPE_MISMATCH: return "shape differs from the plan's shape";
        case TDC_ERR_UNSUPPORTED: return "layer outside the supported domain";
        case TDC_ERR_ALLOC: return "allocation failed";
        case TDC_ERR_HIP: return "HIP runtime or kernel launch error";
        case TDC_ERR_BAD_TUNING: return "forced tuning does not fit the shape or the device";
        case TDC_ERR_TOO_LARGE: return "layer needs more scratch memory than the static buffer holds";
        case TDC_ERR_NO_CONVERGENCE: return "eigen-decomposition did not converge within the sweep limit";
        case TDC_ERR_WAIT: return "a one-launch kernel found XCD or workgroup numbers it was not written for";
        default: return "unknown status";
    }
}

int tdc_plan_create_tuned(tdc_plan **out, const tdc_shape *shape, int device, const tdc_tuning *forced)
{
    if (!out || !shape) return TDC_ERR_NULL;
    *out = nullptr;
    int rc = validate(*shape);
    if (rc != TDC_OK) return rc;
    const int want = forced ? forced->variant : TDC_VARIANT_AUTO;
    if (want < TDC_VARIANT_AUTO || want > TDC_VARIANT_MERGED_XCD) return TDC_ERR_BAD_TUNING;
    const tdc_shape kshape = kernel_shape(*shape, want);
    rc = validate(kshape);
    if (rc != TDC_OK) return rc;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return TDC_ERR_HIP;
    DeviceGuard guard(device);
    if (!guard.ok) return TDC_ERR_HIP;

    TdcDeviceInfo dev;
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) return TDC_ERR_HIP;
    dev.cus = v > 0 ? v : 256;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, device) != hipSuccess) return TDC_ERR_HIP;
    dev.lds_per_wg = v > 0 ? v : 65536;

    tdc_plan *p = new (std::nothrow) tdc_plan();
    if (!p) return TDC_ERR_ALLOC;
    memset(p, 0, sizeof(*p));
    p->wait_limit = 512;
    p->shape = *shape;
    p->dims = make_dims(kshape);
    p->device = device;
    if (forced) p->tuning = *forced;
    rc = tdc_select(p->dims, dev, &p->tuning, &p->model_us);
    if (rc == TDC_OK && tdc_runs_apply(p->dims, dev.cus) &&
        (p->tuning.variant == TDC_VARIANT_FUSED || p->tuning.variant == TDC_VARIANT_CHAIN))
        p->dims.s1_runs = 1;
    if (rc == TDC_OK && p->tuning.variant == TDC_VARIANT_FUSED)
        p->geom = tdc_fused_geometry(p->dims, p->tuning.tile_h, p->tuning.tile_w, dev.lds_per_wg);
    if (rc == TDC_OK && p->tuning.variant == TDC_VARIANT_CHAIN)
        p->geom = tdc_chain_geometry(p->dims, p->tuning.tile_h, p->tuning.tile_w, p->tuning.waves[0], p->tuning.pb[0], dev.lds_per_wg);
    if (rc == TDC_OK && p->tuning.variant == TDC_VARIANT_FUSED_MERGED)
        p->geom = tdc_fm_geometry(p->dims, p->tuning.tile_h, p->tuning.tile_w, p->tuning.waves[0], p->tuning.mb[1]);
    if (rc == TDC_OK) rc = check_tuning(*p, dev);
    if (rc == TDC_OK && p->tuning.variant == TDC_VARIANT_MERGED_XCD) {
        bool fits = false;
        if (tdc_merged_xcd_resident(tdc_merged_xcd_grid(p->dims, p->tuning), p->dims.nhwc, &fits) != hipSuccess) rc = TDC_ERR_HIP;
        else if (!fits) rc = TDC_ERR_BAD_TUNING;
    }
    if (rc != TDC_OK) {
        delete p;
        return rc;
    }

    const TdcDims &d = p->dims;
    const size_t n_z1 = (size_t)d.B * 16 * d.NB1 * d.H * d.W, n_z2 = (size_t)d.B * 16 * d.NB2 * d.Ho * d.Wo;
    const size_t n_w1 = tdc_packed_floats_uin(d), n_w2 = tdc_packed_floats_core(d), n_w3 = tdc_packed_floats_uout(d);
    bool ok = true;
    const bool dense = p->tuning.variant == TDC_VARIANT_DENSE;
    const bool fm = p->tuning.variant == TDC_VARIANT_FUSED_MERGED;
    const bool xcd = p->tuning.variant == TDC_VARIANT_MERGED_XCD;
    const bool merged = p->tuning.variant == TDC_VARIANT_MERGED || fm || xcd;
    if (merged) {
        const size_t n_wm = (size_t)d.R1 * d.N * d.K * d.K, n_wmp = (size_t)d.NB3 * d.K * d.K * d.NB1 * 256;
        if (!fm) {
            const size_t copies = xcd ? 8 : 1;
            ok = ok && hipMalloc((void **)&p->z1, copies * n_z1 * sizeof(float)) == hipSuccess;
            p->ws_bytes += copies * n_z1 * sizeof(float);
        }
        if (xcd) {
            ok = ok && hipMalloc((void **)&p->arrive, (8 * 32 + 8) * sizeof(unsigned)) == hipSuccess;
            ok = ok && hipMemset(p->arrive, 0, (8 * 32 + 8) * sizeof(unsigned)) == hipSuccess;
            ok = ok && hipHostMalloc((void **)&p->status, sizeof(unsigned), hipHostMallocDefault) == hipSuccess;
            if (ok) *p->status = 0;
            p->ws_bytes += (8 * 32 + 8) * sizeof(unsigned);
        }
        ok = ok && hipMalloc((void **)&p->uin_p, n_w1 * sizeof(float)) == hipSuccess;
        ok = ok && hipMalloc((void **)&p->wm, n_wm * sizeof(float)) == hipSuccess;
        ok = ok && hipMalloc((void **)&p->core_p, n_wmp * sizeof(float)) == hipSuccess;
        p->ws_bytes += (n_w1 + n_wm + n_wmp) * sizeof(float);
    }
    if (dense) {
        ok = ok && hipMalloc((void **)&p->core_p, n_w2 * sizeof(float)) == hipSuccess;
        p->ws_bytes += n_w2 * sizeof(float);
    }
    if (!dense && !merged && p->tuning.variant != TDC_VARIANT_FUSED && p->tuning.variant != TDC_VARIANT_CHAIN) {
        ok = ok && hipMalloc((void **)&p->z1, n_z1 * sizeof(float)) == hipSuccess;
        ok = ok && hipMalloc((void **)&p->z2, n_z2 * sizeof(float)) == hipSuccess;
        p->ws_bytes += (n_z1 + n_z2) * sizeof(float);
    }
    if (!dense && !merged && p->tuning.variant != TDC_VARIANT_NAIVE) {
        ok = ok && hipMalloc((void **)&p->uin_p, n_w1 * sizeof(float)) == hipSuccess;
        ok = ok && hipMalloc((void **)&p->core_p, n_w2 * sizeof(float)) == hipSuccess;
        ok = ok && hipMalloc((void **)&p->uout_p, n_w3 * sizeof(float)) == hipSuccess;
        p->ws_bytes += (n_w1 + n_w2 + n_w3) * sizeof(float);
    }
    if (!ok) {
        (void)hipGetLastError();
        tdc_plan_destroy(p);
        return TDC_ERR_ALLOC;
    }
    // whatever a first launch would have to set up, now: a conv call may be the first thing a capturing stream sees
    {
        const TdcEpi none{nullptr, nullptr, 0};
        hipError_t e = hipSuccess;
        if (p->tuning.variant == TDC_VARIANT_FUSED)
            e = tdc_launch_fused(d, p->tuning, p->geom, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, none, true);
        else if (p->tuning.variant == TDC_VARIANT_CHAIN)
            e = tdc_launch_chain(d, p->tuning, p->geom, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, none, true);
        else if (p->tuning.variant == TDC_VARIANT_FUSED_MERGED)
            e = tdc_launch_fm(d, p->tuning, p->geom, nullptr, nullptr, nullptr, nullptr, nullptr, none, true);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            tdc_plan_destroy(p);
            return TDC_ERR_HIP;
        }
    }
    describe(*p);
    *out = p;
    return TDC_OK;
}

int tdc_select_tuning(const tdc_shape *shape, int compute_units, int lds_bytes, tdc_tuning *inout)
{
    if (!shape || !inout) return TDC_ERR_NULL;
    int rc = validate(*shape);
    if (rc != TDC_OK) return rc;
    if (compute_units < 1 || lds_bytes < 1024) return TDC_ERR_BAD_TUNING;
    if (inout->variant < TDC_VARIANT_AUTO || inout->variant > TDC_VARIANT_MERGED_XCD) return TDC_ERR_BAD_TUNING;
    const tdc_shape kshape = kernel_shape(*shape, inout->variant);
    rc = validate(kshape);
    if (rc != TDC_OK) return rc;
    TdcDeviceInfo dev;
    dev.cus = compute_units;
    dev.lds_per_wg = lds_bytes;
    tdc_plan tmp;
    memset(&tmp, 0, sizeof(tmp));
    tmp.dims = make_dims(kshape);
    tmp.tuning = *inout;
    rc = tdc_select(tmp.dims, dev, &tmp.tuning, nullptr);
    if (rc == TDC_OK && tmp.tuning.variant == TDC_VARIANT_FUSED)
        tmp.geom = tdc_fused_geometry(tmp.dims, tmp.tuning.tile_h, tmp.tuning.tile_w, dev.lds_per_wg);
    if (rc == TDC_OK && tmp.tuning.variant == TDC_VARIANT_CHAIN)
        tmp.geom = tdc_chain_geometry(tmp.dims, tmp.tuning.tile_h, tmp.tuning.tile_w, tmp.tuning.waves[0], tmp.tuning.pb[0], dev.lds_per_wg);
    if (rc == TDC_OK && tmp.tuning.variant == TDC_VARIANT_FUSED_MERGED)
        tmp.geom = tdc_fm_geometry(tmp.dims, tmp.tuning.tile_h, tmp.tuning.tile_w, tmp.tuning.waves[0], tmp.tuning.mb[1]);
    if (rc == TDC_OK) rc = check_tuning(tmp, dev);
    if (rc == TDC_OK) *inout = tmp.tuning;
    return rc;
}

int tdc_model_terms(const tdc_shape *shape, const tdc_tuning *tuning, int compute_units, int lds_bytes, double *terms,
                    const char **names, int max_terms, int *n_terms, const char **model)
{
    if (!shape || !tuning || !terms || !n_terms) return TDC_ERR_NULL;
    int rc = validate(*shape);
    if (rc != TDC_OK) return rc;
    if (compute_units < 1 || lds_bytes < 1024) return TDC_ERR_BAD_TUNING;
    if (tuning->variant <= TDC_VARIANT_NAIVE || tuning->variant > TDC_VARIANT_MERGED_XCD) return TDC_ERR_BAD_TUNING;
    const tdc_shape kshape = kernel_shape(*shape, tuning->variant);
    rc = validate(kshape);
    if (rc != TDC_OK) return rc;
    TdcDeviceInfo dev;
    dev.cus = compute_units;
    dev.lds_per_wg = lds_bytes;
    tdc_plan tmp;
    memset(&tmp, 0, sizeof(tmp));
    tmp.dims = make_dims(kshape);
    tmp.tuning = *tuning;
    if (tuning->variant == TDC_VARIANT_FUSED)
        tmp.geom = tdc_fused_geometry(tmp.dims, tuning->tile_h, tuning->tile_w, lds_bytes);
    if (tuning->variant == TDC_VARIANT_CHAIN)
        tmp.geom = tdc_chain_geometry(tmp.dims, tuning->tile_h, tuning->tile_w, tuning->waves[0], tuning->pb[0], lds_bytes);
    if (tuning->variant == TDC_VARIANT_FUSED_MERGED)
        tmp.geom = tdc_fm_geometry(tmp.dims, tuning->tile_h, tuning->tile_w, tuning->waves[0], tuning->mb[1]);
    rc = check_tuning(tmp, dev);
    if (rc != TDC_OK) return rc;
    return tdc_select_terms(tmp.dims, dev, tmp.tuning, terms, names, max_terms, n_terms, model);
}

int tdc_plan_create(tdc_plan **out, const tdc_shape *shape, int device)
{
    return tdc_plan_create_tuned(out, shape, device, nullptr);
}

int tdc_plan_destroy(tdc_plan *p)
{
    if (!p) return TDC_OK;
    DeviceGuard guard(p->device);
    int rc = TDC_OK;
    float *bufs[] = {p->z1, p->z2, p->uin_p, p->core_p, p->uout_p, p->wm};
    for (float *b : bufs)
        if (b && hipFree(b) != hipSuccess) rc = TDC_ERR_HIP;
    if (p->arrive && hipFree(p->arrive) != hipSuccess) rc = TDC_ERR_HIP;
    if (p->status && hipHostFree(p->status) != hipSuccess) rc = TDC_ERR_HIP;
    delete p;
    return rc;
}

int tdc_plan_pack_weights(tdc_plan *p, void *hip_stream, const float *U_in, const float *core, const float *U_out)
{
    if (!p || !U_in || !core || !U_out) return TDC_ERR_NULL;
    if (p->tuning.variant == TDC_VARIANT_DENSE) return TDC_ERR_BAD_TUNING;
    p->packed_from[0] = p->packed_from[1] = p->packed_from[2] = nullptr;
    if (p->tuning.variant == TDC_VARIANT_NAIVE) {   // reads the caller's layouts directly
        p->packed_from[0] = U_in; p->packed_from[1] = core; p->packed_from[2] = U_out;
        return TDC_OK;
    }
    DeviceGuard guard(p->device);
    if (!guard.ok) return TDC_ERR_HIP;
    const bool merged_weights = p->tuning.variant == TDC_VARIANT_MERGED || p->tuning.variant == TDC_VARIANT_FUSED_MERGED ||
                                p->tuning.variant == TDC_VARIANT_MERGED_XCD;
    const hipError_t e = merged_weights
                             ? tdc_launch_pack_merged(p->dims, (hipStream_t)hip_stream, U_in, core, U_out, p->uin_p, p->wm, p->core_p)
                             : tdc_launch_pack(p->dims, (hipStream_t)hip_stream, U_in, core, U_out, p->uin_p, p->core_p, p->uout_p);
    if (e != hipSuccess) return TDC_ERR_HIP;
    p->packed_from[0] = U_in; p->packed_from[1] = core; p->packed_from[2] = U_out;
    return TDC_OK;
}

int tdc_conv_tucker2(tdc_plan *p, void *hip_stream, const float *x, const float *U_in, const float *core,
                     const float *U_out, float *y, const tdc_shape *shape)
{
    return tdc_conv_tucker2_ex(p, hip_stream, x, U_in, core, U_out, y, shape, nullptr);
}

int tdc_conv_tucker2_ex(tdc_plan *p, void *hip_stream, const float *x, const float *U_in, const float *core,
                        const float *U_out, float *y, const tdc_shape *shape, const tdc_epilogue *epilogue)
{
    if (!p || !x || !U_in || !core || !U_out || !y || !shape) return TDC_ERR_NULL;
    const TdcEpi epi = epilogue ? TdcEpi{epilogue->bias, epilogue->residual, epilogue->relu} : TdcEpi{nullptr, nullptr, 0};
    if (!same_shape(*shape, p->shape)) return TDC_ERR_SHAPE_MISMATCH;
    if (p->tuning.variant == TDC_VARIANT_DENSE) return TDC_ERR_BAD_TUNING;
    if (p->dims.nhwc && misaligned16(x, y, epi.residual)) return TDC_ERR_UNSUPPORTED;
    if (p->dims.s1_runs && misaligned16(x, nullptr, nullptr)) return TDC_ERR_UNSUPPORTED;
    if (p->status && *(volatile unsigned *)p->status) return TDC_ERR_WAIT;
    DeviceGuard guard(p->device);
    if (!guard.ok) return TDC_ERR_HIP;
    hipStream_t s = (hipStream_t)hip_stream;
    const TdcDims &d = p->dims;
    hipError_t e;
    if (p->tuning.variant == TDC_VARIANT_NAIVE) {
        e = tdc_launch_naive(d, s, x, U_in, core, U_out, p->z1, p->z2, y, epi);
        return e == hipSuccess ? TDC_OK : TDC_ERR_HIP;
    }
    const bool packed = p->packed_from[0] == U_in && p->packed_from[1] == core && p->packed_from[2] == U_out;
    if (!packed) {   // no stored copy for these pointers: re-lay out on the stream, remember nothing
        p->packed_from[0] = p->packed_from[1] = p->packed_from[2] = nullptr;
        e = (p->tuning.variant == TDC_VARIANT_MERGED || p->tuning.variant == TDC_VARIANT_FUSED_MERGED ||
             p->tuning.variant == TDC_VARIANT_MERGED_XCD)
                ? tdc_launch_pack_merged(d, s, U_in, core, U_out, p->uin_p, p->wm, p->core_p)
                : tdc_launch_pack(d, s, U_in, core, U_out, p->uin_p, p->core_p, p->uout_p);
        if (e != hipSuccess) return TDC_ERR_HIP;
    }
    if (p->tuning.variant == TDC_VARIANT_FUSED_MERGED)
        e = tdc_launch_fm(d, p->tuning, p->geom, s, x, p->uin_p, p->core_p, y, epi);
    else if (p->tuning.variant == TDC_VARIANT_MERGED)
        e = tdc_launch_merged(d, p->tuning, s, x, p->uin_p, p->core_p, p->z1, y, epi);
    else if (p->tuning.variant == TDC_VARIANT_MERGED_XCD)
        e = tdc_launch_merged_xcd(d, p->tuning, s, x, p->uin_p, p->core_p, p->z1, p->arrive, p->status, p->wait_limit, y, epi);
    else if (p->tuning.variant == TDC_VARIANT_SPLIT)
        e = tdc_launch_split(d, p->tuning, s, x, p->uin_p, p->core_p, p->uout_p, p->z1, p->z2, y, epi);
    else if (p->tuning.variant == TDC_VARIANT_CHAIN)
        e = tdc_launch_chain(d, p->tuning, p->geom, s, x, p->uin_p, p->core_p, p->uout_p, y, epi);
    else
        e = tdc_launch_fused(d, p->tuning, p->geom, s, x, p->uin_p, p->core_p, p->uout_p, y, epi);
    return e == hipSuccess ? TDC_OK : TDC_ERR_HIP;
}

int tdc_plan_pack_dense(tdc_plan *p, void *hip_stream, const float *W)
{
    if (!p || !W) return TDC_ERR_NULL;
    if (p->tuning.variant != TDC_VARIANT_DENSE) return TDC_ERR_BAD_TUNING;
    p->packed_from[1] = nullptr;
    DeviceGuard guard(p->device);
    if (!guard.ok) return TDC_ERR_HIP;
    if (tdc_launch_pack_core(p->dims, (hipStream_t)hip_stream, W, p->core_p) != hipSuccess) return TDC_ERR_HIP;
    p->packed_from[1] = W;
    return TDC_OK;
}

int tdc_conv_dense(tdc_plan *p, void *hip_stream, const float *x, const float *W, float *y, const tdc_shape *shape)
{
    return tdc_conv_dense_ex(p, hip_stream, x, W, y, shape, nullptr);
}

int tdc_conv_dense_ex(tdc_plan *p, void *hip_stream, const float *x, const float *W, float *y, const tdc_shape *shape,
                      const tdc_epilogue *epilogue)
{
    if (!p || !x || !W || !y || !shape) return TDC_ERR_NULL;
    const TdcEpi epi = epilogue ? TdcEpi{epilogue->bias, epilogue->residual, epilogue->relu} : TdcEpi{nullptr, nullptr, 0};
    if (!same_shape(*shape, p->shape)) return TDC_ERR_SHAPE_MISMATCH;
    if (p->tuning.variant != TDC_VARIANT_DENSE) return TDC_ERR_BAD_TUNING;
    if (p->dims.nhwc && misaligned16(x, y, epi.residual)) return TDC_ERR_UNSUPPORTED;
    DeviceGuard guard(p->device);
    if (!guard.ok) return TDC_ERR_HIP;
    hipStream_t s = (hipStream_t)hip_stream;
    if (p->packed_from[1] != W) {   // no stored copy for this pointer: re-lay out on the stream, remember nothing
        p->packed_from[1] = nullptr;
        if (tdc_launch_pack_core(p->dims, s, W, p->core_p) != hipSuccess) return TDC_ERR_HIP;
    }
    return tdc_launch_dense(p->dims, p->tuning, s, x, p->core_p, y, epi) == hipSuccess ? TDC_OK : TDC_ERR_HIP;
}

int tdc_plan_get_tuning(const tdc_plan *p, tdc_tuning *out)
{
    if (!p || !out) return TDC_ERR_NULL;
    *out = p->tuning;
    return TDC_OK;
}

int tdc_plan_describe(const tdc_plan *p, char *buf, size_t buf_len)
{
    if (!p || !buf || buf_len == 0) return TDC_ERR_NULL;
    snprintf(buf, buf_len, "%s", p->desc);
    return TDC_OK;
}

size_t tdc_plan_workspace_bytes(const tdc_plan *p) { return p ? p->ws_bytes : 0; }

int tdc_plan_kernel_count(const tdc_plan *p)
{
    if (!p) return 0;
    const int v = p->tuning.variant;
    if (v == TDC_VARIANT_MERGED) return 2;
    if (v == TDC_VARIANT_MERGED_XCD) return 1;
    return (v == TDC_VARIANT_FUSED || v == TDC_VARIANT_CHAIN || v == TDC_VARIANT_DENSE || v == TDC_VARIANT_FUSED_MERGED) ? 1 : 3;
}

int tdc_plan_status(const tdc_plan *p)
{
    if (!p) return TDC_ERR_NULL;
    return p->status && *(volatile unsigned *)p->status ? TDC_ERR_WAIT : TDC_OK;
}

int tdc_plan_set_wait_limit(tdc_plan *p, unsigned polls)
{
    if (!p) return TDC_ERR_NULL;
    if (p->tuning.variant != TDC_VARIANT_MERGED_XCD) return TDC_ERR_BAD_TUNING;
    p->wait_limit = polls;
    return TDC_OK;
}

int tdc_plan_waits_given_up(tdc_plan *p, unsigned *count)
{
    if (!p || !count) return TDC_ERR_NULL;
    if (p->tuning.variant != TDC_VARIANT_MERGED_XCD) return TDC_ERR_BAD_TUNING;
    DeviceGuard guard(p->device);
    if (!guard.ok) return TDC_ERR_HIP;
    return hipMemcpy(count, p->arrive + 8 * 32, sizeof(unsigned), hipMemcpyDeviceToHost) == hipSuccess ? TDC_OK : TDC_ERR_HIP;
}

int tdc_launch_null(void *hip_stream)
{
    hipLaunchKernelGGL(tdc_null_kernel, dim3(1), dim3(64), 0, (hipStream_t)hip_stream);
    return hipGetLastError() == hipSuccess ? TDC_OK : TDC_ERR_HIP;
}

}  // extern "C"

// ---- the entry point that allocates nothing.  Its scratch memory (re-laid-out weights, z1, z2: what a SPLIT
// plan keeps in hipMalloc'ed workspace) is this file-scope device array.  The name is a host-side stand-in,
// not a device address: host code only ever uses the per-device pointer hipGetSymbolAddress returns for it.
static __device__ __align__(256) float tdc_static_scratch[TDC_STATIC_SCRATCH_BYTES / sizeof(float)];

namespace {

struct StaticDevice {
    float *scratch;      // this device's copy of tdc_static_scratch, or null before the first call on it
    TdcDeviceInfo info;
};
constexpr int kMaxStaticDevices = 64;
StaticDevice static_devices[kMaxStaticDevices];
std::mutex static_lock;

// Looks the calling thread's current device up, resolving the array's address the first time that device is seen.
int static_device(StaticDevice *out)
{
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return TDC_ERR_HIP;
    if (device < 0 || device >= kMaxStaticDevices) return TDC_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> hold(static_lock);
    StaticDevice &sd = static_devices[device];
    if (!sd.scratch) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(tdc_static_scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return TDC_ERR_HIP;
        }
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) return TDC_ERR_HIP;
        sd.info.cus = v > 0 ? v : 256;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, device) != hipSuccess) return TDC_ERR_HIP;
        sd.info.lds_per_wg = v > 0 ? v : 65536;
        sd.scratch = static_cast<float *>(ptr);
    }
    *out = sd;
    return TDC_OK;
}

size_t round64(size_t floats) { return (floats + 63) / 64 * 64; }   // regions start on 256-byte boundaries

}  // namespace

extern "C" int tdc_conv_tucker2_static(void *hip_stream, const float *x, const float *U_in, const float *core,
                            const float *U_out, float *y, const tdc_shape *shape)
{
    if (!x || !U_in || !core || !U_out || !y || !shape) return TDC_ERR_NULL;
    int rc = validate(*shape);
    if (rc != TDC_OK) return rc;
    TdcDims d = make_dims(*shape);
    if (d.nhwc && misaligned16(x, y, nullptr)) return TDC_ERR_UNSUPPORTED;
    // scratch regions: packed U_in | packed core | packed U_out | z1 | z2
    const size_t n_w1 = round64(tdc_packed_floats_uin(d)), n_w2 = round64(tdc_packed_floats_core(d));
    const size_t n_w3 = round64(tdc_packed_floats_uout(d));
    const size_t n_z1 = round64((size_t)d.B * 16 * d.NB1 * d.H * d.W), n_z2 = round64((size_t)d.B * 16 * d.NB2 * d.Ho * d.Wo);
    if (n_w1 + n_w2 + n_w3 + n_z1 + n_z2 > TDC_STATIC_SCRATCH_BYTES / sizeof(float)) return TDC_ERR_TOO_LARGE;
    StaticDevice sd;
    rc = static_device(&sd);
    if (rc != TDC_OK) return rc;
    tdc_tuning t;
    memset(&t, 0, sizeof(t));
    t.variant = TDC_VARIANT_SPLIT;
    rc = tdc_select(d, sd.info, &t, nullptr);
    if (rc != TDC_OK) return rc;
    float *uin_p = sd.scratch, *core_p = uin_p + n_w1, *uout_p = core_p + n_w2, *z1 = uout_p + n_w3, *z2 = z1 + n_z1;
    hipStream_t s = (hipStream_t)hip_stream;
    // every element of the five regions is written before it is read (the re-layout kernels write their zero
    // padding themselves, each GEMM stage writes all of its output), so nothing has to be cleared between calls
    if (tdc_launch_pack(d, s, U_in, core, U_out, uin_p, core_p, uout_p) != hipSuccess) return TDC_ERR_HIP;
    const TdcEpi none{nullptr, nullptr, 0};
    return tdc_launch_split(d, t, s, x, uin_p, core_p, uout_p, z1, z2, y, none) == hipSuccess ? TDC_OK : TDC_ERR_HIP;
}
