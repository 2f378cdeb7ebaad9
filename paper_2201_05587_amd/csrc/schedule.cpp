// Host-side schedule logic: default records, re-application of a record to a
// target kernel (paper Sections 4.1, 4.2), the host mirror of the index map,
// the selection rule of the sweep (Section 4.3) and the enumerated space.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

#include "tt_internal.h"

namespace tt {

namespace {

struct Extents {
    int batch, M, N, K;
};

inline int cdiv(int a, int b) { return (a + b - 1) / b; }
inline bool pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }
inline int pow2_floor(int v)
{
    int p = 1;
    while (p <= v / 2) p <<= 1;
    return p;
}
// Vector-width reformulation: the widest power of two not above vmax that divides the extent.
inline int widest_dividing(int vmax, int64_t extent)
{
    int v = 1;
    while (v * 2 <= vmax && extent % (v * 2) == 0) v *= 2;
    return v;
}
inline int conv_out(int in, int f, int stride, int pad) { return (in + 2 * pad - f) / stride + 1; }

bool extents_of(int cls, const void *shape, Extents *e, int *dtype)
{
    if (is_conv_class(cls) || cls == TT_DWCONV_BIAS_RELU6) {
        const tt_conv_shape *s = static_cast<const tt_conv_shape *>(shape);
        if (s->n < 1 || s->c < 1 || s->h < 1 || s->w < 1 || s->k < 1 || s->r < 1 || s->s < 1) return false;
        if (s->stride_h < 1 || s->stride_w < 1 || s->pad_h < 0 || s->pad_w < 0) return false;
        if (s->h + 2 * s->pad_h < s->r || s->w + 2 * s->pad_w < s->s) return false;
        const int ho = conv_out(s->h, s->r, s->stride_h, s->pad_h);
        const int wo = conv_out(s->w, s->s, s->stride_w, s->pad_w);
        *dtype = s->dtype;
        if (cls == TT_DWCONV_BIAS_RELU6) {
            if (s->k != s->c) return false;
            const int64_t planes = (int64_t)s->n * s->c;
            if (planes > INT32_MAX) return false;
            *e = {1, ho, wo, (int)planes};
            return true;
        }
        // The fused GEMM view of Algorithm 2's loop nest: rows are output pixels, the reduction runs
        // over c * r * s.  (The gathering loaders walk it in padded runs; that walk, which is at most
        // 8 / 7 of the reduction plus 7 elements per filter row, must also fit 32 bits.)
        const int64_t m = (int64_t)s->n * ho * wo, k = (int64_t)s->c * s->r * s->s;
        if (m > INT32_MAX || k + k / 4 + 8ll * s->r > INT32_MAX) return false;
        *e = {1, (int)m, s->k, (int)k};
        return true;
    }
    const tt_gemm_shape *g = static_cast<const tt_gemm_shape *>(shape);
    if (g->batch < 1 || g->m < 1 || g->n < 1 || g->k < 1) return false;
    if (g->trans_b != 0 && g->trans_b != 1) return false;
    if (is_dense_class(cls) && (g->batch != 1 || g->trans_b != 1)) return false;
    *dtype = g->dtype;
    *e = {g->batch, g->m, g->n, g->k};
    return true;
}

bool record_well_formed(const tt_schedule &r)
{
    if (r.cls < 0 || r.cls >= TT_NUM_CLASSES) return false;
    if (r.sketch < TT_SK_MFMA || r.sketch > TT_SK_DIRECT) return false;
    if (r.split_k < 1 || r.order < 0 || r.order >= 6) return false;
    if (r.vec != 1 && r.vec != 2 && r.vec != 4 && r.vec != 8) return false;
    if (r.unroll < 1 || r.stages < 1 || r.stages > (r.sketch == TT_SK_MFMA ? 7 : 2)) return false;
    switch (r.sketch) {
    case TT_SK_MFMA: {
        if (r.mfma != 16 && r.mfma != 32) return false;
        if (!pow2(r.tile_m) || !pow2(r.tile_n)) return false;
        if (r.tile_m < 16 || r.tile_m > 256 || r.tile_n < 16 || r.tile_n > 256) return false;
        if (r.tile_k != 16 && r.tile_k != 32 && r.tile_k != 64 && r.tile_k != 128) return false;
        if (r.wave_m < r.mfma || r.wave_n < r.mfma) return false;
        if (r.tile_m % r.wave_m || r.tile_n % r.wave_n || r.wave_m % r.mfma || r.wave_n % r.mfma) return false;
        const int waves = (r.tile_m / r.wave_m) * (r.tile_n / r.wave_n);
        if (!pow2(waves) || waves > 16) return false;
        return r.wave_m * r.wave_n / 64 <= 256;
    }
    case TT_SK_GEMV: {
        if (r.mfma != 0 || r.split_k != 1) return false;
        if (r.tile_m < 1 || r.tile_m > 8 || r.wave_m != r.tile_m) return false;
        if (r.wave_n < 1 || r.wave_n > 8 || r.tile_n % r.wave_n) return false;
        const int waves = r.tile_n / r.wave_n;
        if (!pow2(waves) || waves > 16) return false;
        if (r.tile_k % 64) return false;
        const int chunk = r.tile_k / 64;
        return chunk == 1 || chunk == 2 || chunk == 4 || chunk == 8;
    }
    case TT_SK_DWCONV: {
        if (r.mfma != 0 || r.split_k != 1) return false;
        if (r.tile_m < 1 || r.tile_n < 1 || r.tile_k < 1 || r.wave_m < 1 || r.wave_n < 1) return false;
        if (r.tile_m % r.wave_m || r.tile_n % r.wave_n || r.wave_m > 8 || r.wave_n > 8) return false;
        const int64_t threads = (int64_t)r.tile_k * (r.tile_m / r.wave_m) * (r.tile_n / r.wave_n);
        return threads % 64 == 0 && threads >= 64 && threads <= 1024;
    }
    default:
        return r.mfma == 0 && r.tile_m == 1 && r.tile_n == 1 && r.tile_k == 1 && r.wave_m == 1 && r.wave_n == 1 &&
               r.split_k == 1;
    }
}

// Pixels of the padded input that the tile_m output pixels of one workgroup touch under a 3x3 filter,
// the largest over all tiles: the index range [base(first), base(last) + 2 PW + 2] of flat padded pixel
// indices, base(img, p, q) = img * PH * PW + p * stride * PW + q * stride.
int64_t patch_pixels(const tt_conv_shape &s, int tile_m, int M)
{
    const int ho = conv_out(s.h, s.r, s.stride_h, s.pad_h), wo = conv_out(s.w, s.s, s.stride_w, s.pad_w);
    const int64_t pw = s.w + 2 * s.pad_w, phw = (int64_t)(s.h + 2 * s.pad_h) * pw;
    const auto base = [&](int64_t m) {
        const int64_t img = m / ((int64_t)ho * wo), rem = m % ((int64_t)ho * wo);
        return img * phw + (rem / wo) * s.stride_h * pw + (rem % wo) * s.stride_w;
    };
    int64_t worst = 0;
    for (int64_t m0 = 0; m0 < M; m0 += tile_m) {
        const int64_t last = std::min<int64_t>(m0 + tile_m, M) - 1;
        worst = std::max(worst, base(last) - base(m0) + 2 * pw + 3);
    }
    return worst;
}

int fail(tt_plan *plan, int status, int reason)
{
    std::memset(plan, 0, sizeof *plan);
    plan->status = status;
    plan->reason = reason;
    plan->variant_id = -1;
    return status;
}

tt_schedule make_record(int cls, int sketch, int tm, int tn, int tk, int wm, int wn, int mf, int split_k, int order,
                        int vec, int unroll, int stages)
{
    tt_schedule r;
    std::memset(&r, 0, sizeof r);
    r.cls = cls;
    r.sketch = sketch;
    r.tile_m = tm;
    r.tile_n = tn;
    r.tile_k = tk;
    r.wave_m = wm;
    r.wave_n = wn;
    r.mfma = mf;
    r.split_k = split_k;
    r.order = order;
    r.vec = vec;
    r.unroll = unroll;
    r.stages = stages;
    r.id = -1;
    return r;
}

} // namespace

int family_of(int cls, int trans_b)
{
    if (is_conv_class(cls)) return FAM_CONV;
    if (cls == TT_BATCH_MATMUL && !trans_b) return FAM_GEMM_NN;
    return FAM_GEMM_TN;
}

int find_variant(int dtype, int family, int tm, int tn, int tk, int wm, int wn, int mf, int amode, int pipe, int stride)
{
    for (int i = 0; i < kNumVariants; ++i) {
        const Variant &v = kVariants[i];
        if (v.dtype == dtype && v.family == family && v.tile_m == tm && v.tile_n == tn && v.tile_k == tk &&
            v.wave_m == wm && v.wave_n == wn && v.mfma == mf && v.amode == amode && v.pipe == pipe && v.stride == stride)
            return i;
    }
    return -1;
}

} // namespace tt

using namespace tt;

extern "C" int tt_version(void) { return 100; }

extern "C" const char *tt_status_name(int status)
{
    switch (status) {
    case TT_OK: return "TT_OK";
    case TT_ERR_INVALID_SCHEDULE: return "TT_ERR_INVALID_SCHEDULE";
    case TT_ERR_CLASS_MISMATCH: return "TT_ERR_CLASS_MISMATCH";
    case TT_ERR_BAD_ARG: return "TT_ERR_BAD_ARG";
    case TT_ERR_WORKSPACE: return "TT_ERR_WORKSPACE";
    case TT_ERR_UNSUPPORTED: return "TT_ERR_UNSUPPORTED";
    case TT_ERR_HIP: return "TT_ERR_HIP";
    default: return "TT_ERR_UNKNOWN";
    }
}

extern "C" int tt_schedule_default(int cls, const void *shape, tt_schedule *out)
{
    if (!shape || !out || cls < 0 || cls >= TT_NUM_CLASSES) return TT_ERR_BAD_ARG;
    Extents e;
    int dt;
    if (!extents_of(cls, shape, &e, &dt) || (dt != TT_F32 && dt != TT_BF16)) return TT_ERR_BAD_ARG;
    const tt_schedule direct = make_record(cls, TT_SK_DIRECT, 1, 1, 1, 1, 1, 0, 1, 0, 1, 1, 1);
    *out = direct;
    if (cls == TT_DWCONV_BIAS_RELU6) {
        if (dt != TT_F32) return TT_OK;
        // planes (channels) are the contiguous axis: give them to the lanes first
        const int tk = std::min(64, pow2_floor(e.K));
        const int tn = std::min(256 / tk, pow2_floor(e.N)), tm = std::min(256 / (tk * tn), pow2_floor(e.M));
        const int threads = tk * tm * tn;
        if (threads % 64 || threads < 64) return TT_OK;
        *out = make_record(cls, TT_SK_DWCONV, tm, tn, tk, 1, 1, 0, 1, 0, 1, 1, 1);
        return TT_OK;
    }
    const int kmin = dt == TT_F32 ? 16 : 32;
    if (e.M >= 16 && e.N >= 16 && e.K >= kmin) {
        const int tm = std::min(64, pow2_floor(e.M)), tn = std::min(64, pow2_floor(e.N));
        *out = make_record(cls, TT_SK_MFMA, tm, tn, kmin, std::min(tm, 32), std::min(tn, 32), 16, 1, 0,
                           dt == TT_F32 ? 4 : 8, 1, 2);
        return TT_OK;
    }
    if (is_dense_class(cls) && e.K >= 64 && e.N >= 4)
        *out = make_record(cls, TT_SK_GEMV, 1, 4, e.K >= 256 ? 256 : 64, 1, 1, 0, 1, 0, 4, 1, 1);
    return TT_OK;
}

extern "C" int tt_schedule_apply(const tt_schedule *sched, int cls, const void *shape, int flags, tt_plan *plan)
{
    if (!plan) return TT_ERR_BAD_ARG;
    if (!sched || !shape || cls < 0 || cls >= TT_NUM_CLASSES || !record_well_formed(*sched))
        return fail(plan, TT_ERR_BAD_ARG, TT_R_NONE);
    Extents e;
    int dt;
    if (!extents_of(cls, shape, &e, &dt) || (dt != TT_F32 && dt != TT_BF16))
        return fail(plan, TT_ERR_BAD_ARG, TT_R_NONE);
    const tt_schedule &r = *sched;
    // A record of another class would transform loops this kernel does not have (Section 4.2).
    if (r.cls != cls) return fail(plan, TT_ERR_CLASS_MISMATCH, TT_R_NONE);
    const bool dw = cls == TT_DWCONV_BIAS_RELU6;
    if (r.sketch != TT_SK_DIRECT && (r.sketch == TT_SK_DWCONV) != dw)
        return fail(plan, TT_ERR_INVALID_SCHEDULE, TT_R_SKETCH_CLASS);
    if (r.sketch == TT_SK_GEMV && !is_dense_class(cls)) return fail(plan, TT_ERR_INVALID_SCHEDULE, TT_R_SKETCH_CLASS);

    const bool strict = (flags & TT_STRICT_DIVISIBLE) != 0;
    const int elem = dt == TT_F32 ? 4 : 2;
    const int vmax = std::min(r.vec, 16 / elem);
    tt_plan p;
    std::memset(&p, 0, sizeof p);
    p.variant_id = -1;
    p.sketch = r.sketch;
    p.batch = e.batch;
    p.M = e.M;
    p.N = e.N;
    p.K = e.K;
    p.order = r.order;
    p.stages = r.stages;
    p.mfma = r.mfma;

    if (r.sketch == TT_SK_DIRECT) {
        const int64_t total = (int64_t)e.batch * e.M * e.N * (dw ? e.K : 1);
        const int64_t grid = (total + 255) / 256;
        if (grid > INT32_MAX) return fail(plan, TT_ERR_INVALID_SCHEDULE, TT_R_GRID);
        p.tile_m = p.tile_n = p.tile_k = p.wave_m = p.wave_n = 1;
        p.tiles_m = e.M;
        p.tiles_n = e.N;
        p.k_tiles = e.K;
        p.tail_m = p.tail_n = p.tail_k = 1;
        p.eff_split_k = 1;
        p.k_iters = dw ? 1 : e.K;
        p.slabs = dw ? e.K : e.batch;
        p.eff_vec_a = p.eff_vec_b = p.eff_vec_c = p.eff_unroll = 1;
        p.grid = (int)grid;
        p.block = 256;
        p.variant_id = 0;
        *plan = p;
        return TT_OK;
    }

    // Depthwise: Vectorize applies to the plane axis and is reformulated to the target (Section 4.1):
    // a lane owns the widest group of channel-contiguous planes, not above the record's width, that
    // divides the channel count, so the tile_k lanes a workgroup has along that axis cover tile_k * ev
    // planes.
    int ev_planes = 1;
    if (r.sketch == TT_SK_DWCONV) ev_planes = widest_dividing(vmax, static_cast<const tt_conv_shape *>(shape)->c);
    const int64_t tile_k_eff = (int64_t)r.tile_k * ev_planes;
    if (tile_k_eff > INT32_MAX) return fail(plan, TT_ERR_INVALID_SCHEDULE, TT_R_FACTOR_GT_K);
    // Inner factors are kept as recorded; a factor larger than the loop it splits cannot be applied.
    const int factor[3] = {r.tile_m, r.tile_n, (int)tile_k_eff};
    const int extent[3] = {e.M, e.N, e.K};
    for (int i = 0; i < 3; ++i) {
        if (factor[i] > extent[i]) return fail(plan, TT_ERR_INVALID_SCHEDULE, TT_R_FACTOR_GT_M + i);
        if (strict && extent[i] % factor[i]) return fail(plan, TT_ERR_INVALID_SCHEDULE, TT_R_NOT_DIVISIBLE);
    }
    // Outer extents come from the target shape; the last tile is guarded.
    p.tile_m = r.tile_m;
    p.tile_n = r.tile_n;
    p.tile_k = (int)tile_k_eff;
    p.wave_m = r.wave_m;
    p.wave_n = r.wave_n;
    p.tiles_m = cdiv(e.M, r.tile_m);
    p.tiles_n = cdiv(e.N, r.tile_n);
    p.k_tiles = cdiv(e.K, p.tile_k);
    p.tail_m = e.M - (p.tiles_m - 1) * r.tile_m;
    p.tail_n = e.N - (p.tiles_n - 1) * r.tile_n;
    p.tail_k = e.K - (p.k_tiles - 1) * p.tile_k;

    if (r.sketch == TT_SK_DWCONV) {
        const tt_conv_shape *s = static_cast<const tt_conv_shape *>(shape);
        const int64_t grid = (int64_t)p.tiles_m * p.tiles_n * p.k_tiles;
        if (grid > INT32_MAX) return fail(plan, TT_ERR_INVALID_SCHEDULE, TT_R_GRID);
        // The library's own part: the input patch the two-stage kernel keeps in LDS, and which kernel runs.
        int64_t lds = 0;
        if (r.stages == 2) {
            const int64_t rows = (int64_t)(r.tile_m - 1) * s->stride_h + s->r;
            const int64_t cols = (int64_t)(r.tile_n - 1) * s->stride_w + s->s;
            lds = p.tile_k * rows * cols * elem;
        }
        if (lds > kLdsBudget) return fail(plan, TT_ERR_INVALID_SCHEDULE, TT_R_LDS);
        // Several planes per lane exist in the register kernel only (one stage, equal strides of 1 or 2,
        // input below 2 GiB); elsewhere such a plan has no kernel.
        const bool rows_kernel = r.stages == 1 && s->stride_h == s->stride_w && (s->stride_h == 1 || s->stride_h == 2) &&
                                 (int64_t)s->n * s->h * s->w * s->c * elem < (1ll << 31);
        const int block = r.tile_k * (r.tile_m / r.wave_m) * (r.tile_n / r.wave_n);
        const bool fits = block <= dw_max_block(r.wave_m, r.wave_n, ev_planes, s->stride_w, rows_kernel);
        p.variant_id = (ev_planes == 1 || rows_kernel) && s->r == 3 && s->s == 3 && dt == TT_F32 && fits ? 0 : -1;
        p.eff_split_k = 1;
        p.k_iters = 1;
        p.slabs = p.k_tiles;
        p.eff_vec_a = p.eff_vec_c = ev_planes;
        p.eff_vec_b = 1;
        p.eff_unroll = std::min(r.unroll, r.wave_m);
        p.grid = (int)grid;
        p.block = block;
        p.lds_bytes = (int)lds;
        *plan = p;
        return TT_OK;
    }

    if (r.sketch == TT_SK_GEMV) {
        const int64_t grid = (int64_t)p.tiles_m * p.tiles_n * e.batch;
        if (grid > INT32_MAX) return fail(plan, TT_ERR_INVALID_SCHEDULE, TT_R_GRID);
        const int ev = widest_dividing(std::min(vmax, r.tile_k / 64), e.K);
        p.eff_split_k = 1;
        p.k_iters = p.k_tiles;
        p.slabs = e.batch;
        p.eff_vec_a = p.eff_vec_b = ev;
        p.eff_vec_c = 1;
        p.eff_unroll = std::min(r.unroll, p.k_tiles);
        p.grid = (int)grid;
        p.block = 64 * (r.tile_n / r.wave_n);
        p.variant_id = 0;
        *plan = p;
        return TT_OK;
    }

    // Matrix-core sketch.  First what the method defines: the parallel split of the reduction and the grid.
    if (r.split_k > p.k_tiles) return fail(plan, TT_ERR_INVALID_SCHEDULE, TT_R_SPLIT_K);
    if (strict && p.k_tiles % r.split_k) return fail(plan, TT_ERR_INVALID_SCHEDULE, TT_R_NOT_DIVISIBLE);
    p.k_iters = cdiv(p.k_tiles, r.split_k);
    p.eff_split_k = cdiv(p.k_tiles, p.k_iters);
    p.block = 64 * (r.tile_m / r.wave_m) * (r.tile_n / r.wave_n);
    p.slabs = e.batch * p.eff_split_k;
    const int64_t grid = (int64_t)p.tiles_m * p.tiles_n * p.slabs;
    if (grid > INT32_MAX) return fail(plan, TT_ERR_INVALID_SCHEDULE, TT_R_GRID);
    p.grid = (int)grid;
    p.workspace_bytes = p.eff_split_k > 1 ? 4ll * p.eff_split_k * e.batch * e.M * e.N : 0;

    // From here on: this library's kernels (how the operands are fetched and staged).  None of it is
    // part of the method; the constants come from the compiled kernels themselves.
    const int granule = k_granule(dt, r.mfma);
    if (r.tile_k % granule) return fail(plan, TT_ERR_INVALID_SCHEDULE, TT_R_K_GRANULE);
    int trans_b = 1;
    if (!is_conv_class(cls)) trans_b = static_cast<const tt_gemm_shape *>(shape)->trans_b;
    if (is_conv_class(cls)) {
        // vectors run along the channel axis of both operands and along the output channels
        const tt_conv_shape *s = static_cast<const tt_conv_shape *>(shape);
        p.eff_vec_a = p.eff_vec_b = widest_dividing(vmax, s->c);
        p.eff_vec_c = widest_dividing(vmax, e.N);
    } else {
        p.eff_vec_a = widest_dividing(vmax, e.K);
        p.eff_vec_b = trans_b ? widest_dividing(vmax, e.K) : widest_dividing(vmax, e.N);
        p.eff_vec_c = widest_dividing(vmax, e.N);
    }
    // Conv: 16-byte gathers when the effective vector width fills an item, else element by element;
    // a unit-stride 1x1 convolution without padding reads the activations as a plain [M][C] matrix
    // and runs on the dense family.
    int amode = 0, family = family_of(cls, trans_b);
    bool whole_items = false; // both operands are fetched as whole 16-byte items along K
    if (is_conv_class(cls)) {
        const tt_conv_shape *s = static_cast<const tt_conv_shape *>(shape);
        const bool pointwise = s->r == 1 && s->s == 1 && s->pad_h == 0 && s->pad_w == 0 && s->stride_h == 1 &&
                               s->stride_w == 1;
        amode = p.eff_vec_a * elem == 16 ? 16 : elem;
        whole_items = amode == 16;
        if (pointwise && amode == 16) {
            family = FAM_GEMM_TN;
            amode = 0;
        }
    } else if (trans_b) {
        whole_items = p.eff_vec_a * elem == 16;
    }
    // Three or four stages ask for the asynchronous pipeline (16-byte loads straight into a ring of
    // LDS buffers).  It exists for tiles its loader can fill (a compiled ring variant), whole items
    // and operands within 2 GiB; a record that asks for it elsewhere is reformulated to the two-stage
    // register pipeline (Section 4.1 treats unroll depths the same way).
    // (the conv entry point refuses tensors of 2 GiB and more for every matrix-core record)
    const bool in_range = is_conv_class(cls) ||
                          ((int64_t)e.M * e.K * elem < (1ll << 31) && (int64_t)e.N * e.K * elem < (1ll << 31));
    // Five or six stages ask for the 3x3 convolution kernel that keeps the padded input patch of the
    // workgroup's tile in LDS and streams the filters through a ring of three or four buffers.  It exists
    // for bf16, 32-blocks, equal strides of 1 or 2, channel counts that tile_k divides, splits of the
    // reduction that fall on channel-slice boundaries, and tiles whose patch fits the compiled buffer;
    // elsewhere the record is reformulated to the plain ring of stages - 2 buffers.
    int want = r.stages;
    // Seven stages ask for the persistent kernel of the dense family: the whole [tile_n][K] panel of B stays
    // in LDS, a workgroup walks down M with the next tile's A rows requested a tile ahead.  It exists for
    // reductions of a few whole slices (the panel, two A buffers and the epilogue's staging must fit the LDS,
    // the requests the vector-memory counter), one batch, no split of the reduction, whole 16-byte items;
    // elsewhere the record is reformulated to the ring of four buffers.
    if (want == 7) {
        int stream_id = -1;
        if (family == FAM_GEMM_TN && whole_items && in_range && e.batch == 1 && p.eff_split_k == 1 && e.K % r.tile_k == 0)
            stream_id = find_variant(dt, FAM_GEMM_TN, r.tile_m, r.tile_n, r.tile_k, r.wave_m, r.wave_n, r.mfma, 0, 3);
        if (stream_id >= 0) {
            const Variant &v = kVariants[stream_id];
            if (v.lds_bytes(p.k_tiles) > kLdsBudget || (int64_t)p.k_tiles * v.stage_bytes() + 8 > 63) stream_id = -1;
        }
        if (stream_id >= 0) {
            p.stages = 7;
            p.eff_unroll = std::min(r.unroll, r.tile_k / granule);
            p.variant_id = stream_id;
            p.lds_bytes = kVariants[stream_id].lds_bytes(p.k_tiles);
            *plan = p;
            return TT_OK;
        }
        want = 4;
    }
    if (want >= 5) {
        int patch_id = -1;
        if (is_conv_class(cls) && dt == TT_BF16 && r.mfma == 32 && whole_items && amode == 16) {
            const tt_conv_shape *s = static_cast<const tt_conv_shape *>(shape);
            if (s->r == 3 && s->s == 3 && s->stride_h == s->stride_w && (s->stride_h == 1 || s->stride_h == 2) &&
                s->c % r.tile_k == 0 && p.k_iters % 9 == 0) {
                const int id = find_variant(dt, FAM_CONV, r.tile_m, r.tile_n, r.tile_k, r.wave_m, r.wave_n, r.mfma, 16, 2,
                                            s->stride_h);
                if (id >= 0 && patch_pixels(*s, r.tile_m, e.M) <= kVariants[id].stage_bytes()) patch_id = id;
            }
        }
        if (patch_id >= 0) {
            const int64_t lds = kVariants[patch_id].lds_bytes(want);
            if (lds > kLdsBudget) return fail(plan, TT_ERR_INVALID_SCHEDULE, TT_R_LDS);
            p.stages = want;
            p.eff_unroll = std::min(r.unroll, r.tile_k / granule);
            p.variant_id = patch_id;
            p.lds_bytes = (int)lds;
            *plan = p;
            return TT_OK;
        }
        want -= 2;
    }
    const int ring_id = whole_items && in_range
                            ? find_variant(dt, family, r.tile_m, r.tile_n, r.tile_k, r.wave_m, r.wave_n, r.mfma, amode, 1)
                            : -1;
    p.stages = want;
    if (want >= 3 && ring_id < 0) p.stages = 2;
    p.eff_unroll = std::min(r.unroll, r.tile_k / granule);
    p.variant_id = p.stages >= 3 ? ring_id
                                 : find_variant(dt, family, r.tile_m, r.tile_n, r.tile_k, r.wave_m, r.wave_n, r.mfma,
                                                amode, 0);
    if (p.variant_id >= 0) {
        const int64_t lds = kVariants[p.variant_id].lds_bytes(p.stages);
        if (lds > kLdsBudget) return fail(plan, TT_ERR_INVALID_SCHEDULE, TT_R_LDS);
        p.lds_bytes = (int)lds;
    }
    *plan = p;
    return TT_OK;
}

extern "C" int tt_plan_tile(const tt_plan *plan, int64_t wg, int32_t out[8])
{
    if (!plan || !out || plan->status != TT_OK || plan->sketch == TT_SK_DIRECT) return TT_ERR_BAD_ARG;
    if (wg < 0 || wg >= plan->grid) return TT_ERR_BAD_ARG;
    const TileCoord c = decode_tile(tile_map_of(*plan), (int32_t)wg);
    out[0] = c.hi;
    out[1] = c.lo;
    out[2] = c.m0;
    out[3] = c.m_ext;
    out[4] = c.n0;
    out[5] = c.n_ext;
    out[6] = c.k0;
    out[7] = c.k_ext;
    return TT_OK;
}

extern "C" int64_t tt_debug_fast_div(uint32_t n, uint32_t d)
{
    if (d < 1 || d >= (1u << 31) || n >= (1u << 31)) return -1;
    return (int64_t)fast_div(n, make_fastdiv(d));
}

extern "C" int tt_variant_info(int variant_id, int32_t out[12])
{
    if (!out || variant_id < 0 || variant_id >= kNumVariants) return TT_ERR_BAD_ARG;
    const Variant &v = kVariants[variant_id];
    const int32_t vals[12] = {v.dtype, v.family, v.tile_m, v.tile_n, v.tile_k, v.wave_m, v.wave_n, v.mfma, v.amode, v.pipe,
                              v.stage_bytes(),
                              k_granule(v.dtype, v.mfma)};
    std::copy(vals, vals + 12, out);
    return TT_OK;
}

extern "C" int tt_num_variants(void) { return kNumVariants; }

extern "C" int tt_sweep_select(const int32_t *kernel_cls, int nk, const int32_t *pool_cls, int np,
                               const double *pair_us, const double *default_us, int allow_slower, tt_sweep_row *rows)
{
    if (nk < 0 || np < 0 || !rows || (nk && (!kernel_cls || !default_us)) || (np && (!pool_cls || !pair_us)))
        return TT_ERR_BAD_ARG;
    for (int k = 0; k < nk; ++k) {
        tt_sweep_row row;
        std::memset(&row, 0, sizeof row);
        row.kernel = k;
        row.chosen = -1;
        row.default_us = default_us[k];
        bool have = !allow_slower;
        double best = default_us[k];
        for (int p = 0; p < np; ++p) {
            if (pool_cls[p] != kernel_cls[k]) {
                ++row.n_other_class;
                continue;
            }
            const double t = pair_us[(size_t)k * np + p];
            if (t == -3.0) {
                ++row.n_not_tried; // left out by the sweep's budget
                continue;
            }
            if (t < 0) {
                ++row.n_invalid; // does not apply to this kernel: skipped
                continue;
            }
            ++row.n_valid;
            if (!have || t < best) { // strict '<': the default, then the lowest index, win ties
                best = t;
                row.chosen = p;
                have = true;
            }
        }
        row.best_us = row.chosen < 0 ? default_us[k] : best;
        rows[k] = row;
    }
    return TT_OK;
}

// SplitMix64 (Steele, Lea, Flood: "Fast splittable pseudorandom number generators", 2014): the output
// function applied to a counter; used as a counter-based generator of sampling keys.
static uint64_t splitmix64(uint64_t x)
{
    x += 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}

extern "C" int tt_sweep_plan(const int32_t *kernel_cls, const double *weight, int nk, const int32_t *pool_cls, int np,
                             int pair_budget, int prioritise, uint64_t seed, uint8_t *mask, int64_t *selected)
{
    if (nk < 0 || np < 0 || !mask || (nk && !kernel_cls) || (np && !pool_cls) || (prioritise && nk && !weight))
        return TT_ERR_BAD_ARG;
    struct Pair {
        uint64_t key;
        int64_t index;
    };
    std::vector<std::vector<Pair>> per_kernel(nk);
    int64_t total = 0;
    for (int k = 0; k < nk; ++k)
        for (int p = 0; p < np; ++p) {
            const int64_t i = (int64_t)k * np + p;
            mask[i] = 0;
            if (pool_cls[p] != kernel_cls[k]) continue;
            per_kernel[k].push_back({splitmix64(seed + (uint64_t)i + 1), i});
            ++total;
        }
    const auto by_key = [](const Pair &a, const Pair &b) { return a.key != b.key ? a.key < b.key : a.index < b.index; };
    int64_t chosen = 0;
    if (pair_budget <= 0 || pair_budget >= total) {
        for (auto &v : per_kernel)
            for (const Pair &q : v) mask[q.index] = 1;
        chosen = total;
    } else if (!prioritise) {
        std::vector<Pair> all;
        for (auto &v : per_kernel) all.insert(all.end(), v.begin(), v.end());
        std::sort(all.begin(), all.end(), by_key);
        for (int64_t i = 0; i < pair_budget; ++i) mask[all[i].index] = 1;
        chosen = pair_budget;
    } else {
        std::vector<int> order(nk);
        for (int k = 0; k < nk; ++k) order[k] = k;
        std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return weight[a] > weight[b]; });
        int64_t left = pair_budget;
        for (int k : order) {
            auto &v = per_kernel[k];
            if (left <= 0) break;
            if ((int64_t)v.size() > left) std::sort(v.begin(), v.end(), by_key);
            const int64_t take = std::min<int64_t>(left, (int64_t)v.size());
            for (int64_t i = 0; i < take; ++i) mask[v[i].index] = 1;
            left -= take;
            chosen += take;
        }
    }
    if (selected) *selected = chosen;
    return TT_OK;
}

extern "C" int tt_refine_space(const tt_schedule *base, tt_schedule *out, int cap)
{
    if (!base || cap < 0 || (cap && !out) || !record_well_formed(*base)) return TT_ERR_BAD_ARG;
    std::vector<tt_schedule> recs;
    const auto consider = [&](tt_schedule r) {
        if (!record_well_formed(r)) return;
        if (std::memcmp(&r, base, sizeof(int32_t) * 13) == 0) return; // the thirteen knobs lead the record
        r.id = (int32_t)recs.size();
        recs.push_back(r);
    };
    const tt_schedule &b = *base;
    if (b.sketch == TT_SK_MFMA || b.sketch == TT_SK_DWCONV) {
        int32_t tt_schedule::*factors[] = {&tt_schedule::tile_m, &tt_schedule::tile_n, &tt_schedule::tile_k,
                                           &tt_schedule::wave_m, &tt_schedule::wave_n, &tt_schedule::vec};
        for (auto f : factors)
            for (int up = 0; up < 2; ++up) {
                tt_schedule r = b;
                r.*f = up ? b.*f * 2 : b.*f / 2;
                if (r.*f >= 1 && (up || b.*f % 2 == 0)) consider(r);
            }
        for (int order = 0; order < 6; ++order) {
            tt_schedule r = b;
            r.order = order;
            consider(r);
        }
        for (int d = -1; d <= 1; d += 2) {
            tt_schedule r = b;
            r.stages = b.stages + d;
            consider(r);
        }
        tt_schedule u = b;
        u.unroll = b.unroll >= 2 ? 1 : 8;
        consider(u);
    }
    if (b.sketch == TT_SK_MFMA) {
        tt_schedule r = b;
        r.mfma = b.mfma == 16 ? 32 : 16;
        consider(r);
        static const int splits[] = {1, 2, 3, 4, 6, 8, 12, 16, 32};
        int at = -1;
        for (int i = 0; i < 9; ++i)
            if (splits[i] == b.split_k) at = i;
        if (at >= 0)
            for (int d = -1; d <= 1; d += 2)
                if (at + d >= 0 && at + d < 9) {
                    tt_schedule q = b;
                    q.split_k = splits[at + d];
                    consider(q);
                }
    }
    for (size_t i = 0; i < recs.size() && (int)i < cap; ++i) out[i] = recs[i];
    return (int)recs.size();
}

extern "C" int tt_select_donor(const double *class_cost, int num_classes, const int32_t *donor_class_count,
                               int n_donors, double *scores, int32_t *best)
{
    if (!class_cost || num_classes < 1 || n_donors < 0 || !best || (n_donors && !donor_class_count)) return TT_ERR_BAD_ARG;
    double total = 0.0;
    for (int c = 0; c < num_classes; ++c) {
        if (!(class_cost[c] >= 0.0)) return TT_ERR_BAD_ARG;
        total += class_cost[c];
    }
    if (!(total > 0.0)) return TT_ERR_BAD_ARG;
    *best = -1;
    double best_score = 0.0;
    for (int t = 0; t < n_donors; ++t) {
        double score = 0.0;
        for (int c = 0; c < num_classes; ++c) {
            const int32_t count = donor_class_count[(size_t)t * num_classes + c];
            if (count < 0) return TT_ERR_BAD_ARG;
            const double share = class_cost[c] / total;
            score += share * share * std::sqrt((double)count);
        }
        if (scores) scores[t] = score;
        if (*best < 0 || score > best_score) { // strict '>': the lowest index wins ties
            *best = t;
            best_score = score;
        }
    }
    return TT_OK;
}

extern "C" int tt_schedule_space(int cls, int dtype, int level, tt_schedule *out, int cap)
{
    if (cls < 0 || cls >= TT_NUM_CLASSES || (dtype != TT_F32 && dtype != TT_BF16) || cap < 0 || (cap && !out))
        return TT_ERR_BAD_ARG;
    std::vector<tt_schedule> recs;
    const int vfull = dtype == TT_F32 ? 4 : 8;
    if (cls == TT_DWCONV_BIAS_RELU6) {
        // planes (channels) are the contiguous axis: tiles are wide in planes and small in rows x cols
        static const int tms[] = {1, 2, 4, 7, 8, 14}, tns[] = {1, 2, 4, 7, 8, 14, 16, 28};
        static const int tks[] = {8, 16, 32, 64, 128, 256}, wms[] = {1, 2, 4, 7}, wns[] = {1, 2, 4, 7};
        for (int tm : tms)
            for (int tn : tns)
                for (int tk : tks)
                    for (int wm : wms)
                        for (int wn : wns)
                            for (int stages = 1; stages <= (level >= 2 ? 2 : 1); ++stages) {
                                // several planes per lane exist in the one-stage kernel only
                                for (int vec : {1, 2, 4}) {
                                    if (stages == 2 && vec != 1) continue;
                                    tt_schedule r = make_record(cls, TT_SK_DWCONV, tm, tn, tk, wm, wn, 0, 1, 0, vec, wm, stages);
                                    if (record_well_formed(r)) recs.push_back(r);
                                }
                            }
    } else {
        // families this class can run on: conv classes one, dense one, batch matmul both layouts
        for (int i = 0; i < kNumVariants; ++i) {
            const Variant &v = kVariants[i];
            if (v.dtype != dtype) continue;
            const bool fam_ok = is_conv_class(cls) ? v.family == FAM_CONV
                                : cls == TT_BATCH_MATMUL ? (v.family == FAM_GEMM_TN || v.family == FAM_GEMM_NN)
                                                         : v.family == FAM_GEMM_TN;
            if (!fam_ok) continue;
            // batch matmul records do not carry the layout: list each tile once (TN and NN tables are the same)
            if (cls == TT_BATCH_MATMUL && v.family == FAM_GEMM_NN) continue;
            // One pass per tile: the register-pipeline instance stands for the tile.  A tile that only the patch
            // kernel is compiled for (its first instance stands for it) contributes its stages 5 and 6 alone.
            bool patch_only = false;
            if (v.pipe == 2) {
                if (find_variant(v.dtype, v.family, v.tile_m, v.tile_n, v.tile_k, v.wave_m, v.wave_n, v.mfma, 16, 0) >= 0)
                    continue;
                bool first = true;
                for (int j = 0; j < i; ++j) {
                    const Variant &u = kVariants[j];
                    if (u.pipe == 2 && u.dtype == v.dtype && u.tile_m == v.tile_m && u.tile_n == v.tile_n &&
                        u.tile_k == v.tile_k && u.wave_m == v.wave_m && u.wave_n == v.wave_n && u.mfma == v.mfma)
                        first = false;
                }
                if (!first) continue;
                patch_only = true;
            } else if (v.pipe != 0 || (v.family == FAM_CONV && v.amode != 16)) {
                continue;
            }
            static const int splits[] = {1, 2, 3, 4, 6, 8, 12, 16, 32};
            const int n_split = level >= 1 ? 9 : 1;
            const int n_order = level >= 2 ? 6 : (level >= 1 ? 2 : 1);
            for (int si = 0; si < n_split; ++si)
                for (int order = 0; order < n_order; ++order)
                    for (int stages = (level >= 1 ? 1 : 2); stages <= (level >= 1 ? 7 : 2); ++stages) {
                        if (patch_only && (stages < 5 || stages > 6)) continue;
                        // seven stages only for tiles the persistent kernel is compiled for, unsplit
                        if (stages == 7 &&
                            (splits[si] != 1 ||
                             find_variant(v.dtype, FAM_GEMM_TN, v.tile_m, v.tile_n, v.tile_k, v.wave_m, v.wave_n, v.mfma, 0, 3) < 0))
                            continue;
                        // three and four stages only for tiles the asynchronous pipeline can load, five and six
                        // only for tiles the patch kernel is compiled for
                        if ((stages == 3 || stages == 4) &&
                            find_variant(v.dtype, v.family, v.tile_m, v.tile_n, v.tile_k, v.wave_m, v.wave_n, v.mfma, v.amode, 1) < 0)
                            continue;
                        if ((stages == 5 || stages == 6) &&
                            find_variant(v.dtype, v.family, v.tile_m, v.tile_n, v.tile_k, v.wave_m, v.wave_n, v.mfma, 16, 2, 1) < 0 &&
                            find_variant(v.dtype, v.family, v.tile_m, v.tile_n, v.tile_k, v.wave_m, v.wave_n, v.mfma, 16, 2, 2) < 0)
                            continue;
                        tt_schedule r = make_record(cls, TT_SK_MFMA, v.tile_m, v.tile_n, v.tile_k, v.wave_m, v.wave_n,
                                                    v.mfma, splits[si], order, vfull, 8, stages);
                        if (record_well_formed(r)) recs.push_back(r);
                    }
        }
        if (is_dense_class(cls)) {
            static const int tks[] = {64, 128, 256, 512};
            for (int tm : {1, 2, 4})
                for (int wn : {1, 2, 4})
                    for (int waves : {1, 2, 4, 8})
                        for (int tk : tks) {
                            tt_schedule r = make_record(cls, TT_SK_GEMV, tm, wn * waves, tk, tm, wn, 0, 1, 0, 4, 1, 1);
                            if (record_well_formed(r)) recs.push_back(r);
                        }
        }
    }
    for (size_t i = 0; i < recs.size(); ++i) {
        recs[i].id = (int)i;
        if ((int)i < cap) out[i] = recs[i];
    }
    return (int)recs.size();
}
