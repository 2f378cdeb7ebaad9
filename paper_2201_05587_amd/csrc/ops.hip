// C-ABI operator entry points, standalone pair timing and the transfer-tuning sweep.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <atomic>
#include <cstring>
#include <mutex>
#include <vector>

#include "tt_internal.h"

using namespace tt;

namespace tt {
static thread_local char g_last_error[256] = "";
int note_hip_error(int code, const char *where)
{
    snprintf(g_last_error, sizeof g_last_error, "%s: %s (%d)", where, hipGetErrorString((hipError_t)code), code);
    return TT_ERR_HIP;
}
} // namespace tt

extern "C" const char *tt_last_error(void) { return tt::g_last_error; }

namespace {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int conv_out(int in, int f, int stride, int pad) { return (in + 2 * pad - f) / stride + 1; }

// Resolve the record (NULL = default), re-apply it to the shape, check the workspace.
int make_plan(const tt_schedule *sched, int cls, const void *shape, const void *ws, size_t ws_bytes, tt_plan *plan)
{
    tt_schedule def;
    if (!sched) {
        const int rc = tt_schedule_default(cls, shape, &def);
        if (rc != TT_OK) return rc;
        sched = &def;
    }
    const int rc = tt_schedule_apply(sched, cls, shape, 0, plan);
    if (rc != TT_OK) return rc;
    if (plan->workspace_bytes > 0 && (!ws || (int64_t)ws_bytes < plan->workspace_bytes || !aligned16(ws)))
        return TT_ERR_WORKSPACE;
    return TT_OK;
}

void fill_common(ContractArgs &g, const tt_plan &plan, const tt_schedule *sched, int cls, int dtype)
{
    g.map = tile_map_of(plan);
    g.batch = plan.batch;
    g.M = plan.M;
    g.N = plan.N;
    g.K = plan.K;
    g.eff_vec_a = plan.eff_vec_a;
    g.eff_vec_b = plan.eff_vec_b;
    g.eff_vec_c = plan.eff_vec_c;
    g.stages = plan.stages;
    g.unroll = plan.eff_unroll;
    g.act = act_of_class(cls);
    g.dtype = dtype;
    (void)sched;
}

int run_contraction(ContractArgs &g, const tt_plan &plan, int family, void *stream)
{
    switch (plan.sketch) {
    case TT_SK_DIRECT:
        return launch_direct(g, family, plan.grid, stream);
    case TT_SK_GEMV:
        return launch_gemv(g, plan, stream);
    case TT_SK_MFMA: {
        if (plan.variant_id < 0 || plan.variant_id >= kNumVariants) return TT_ERR_UNSUPPORTED;
        const int rc = kVariants[plan.variant_id].launch(g, plan.grid, plan.lds_bytes, stream);
        if (rc != TT_OK) return rc;
        if (plan.eff_split_k > 1) return launch_splitk_reduce(g, family, stream);
        return TT_OK;
    }
    default:
        return TT_ERR_UNSUPPORTED;
    }
}

} // namespace

// ---- split-K partial sums without a caller's workspace ----------------------------------------------
// One array per GPU, part of the library's code object: it exists from the moment the library is loaded
// on a device until the process ends.  In host code the array's name is only a handle; the address the
// kernels get comes from hipGetSymbolAddress, asked for once per device with that device current.
static __device__ __align__(256) unsigned char scratch[TT_STATIC_WORKSPACE_BYTES];

namespace {

constexpr int kMaxDevices = 64;

int static_workspace(void **ptr)
{
    static std::mutex guard;
    static void *per_device[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return note_hip_error((int)e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return TT_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(guard);
    if (!per_device[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return note_hip_error((int)e, "hipGetSymbolAddress(scratch)");
        per_device[dev] = p;
    }
    *ptr = per_device[dev];
    return TT_OK;
}

} // namespace

extern "C" int tt_conv2d_bias_relu_noalloc(const void *x, const void *w, const void *bias, const void *residual,
                                           void *y, const tt_conv_shape *shape, int cls, const tt_schedule *sched,
                                           void *stream)
{
    void *ws = nullptr;
    if (const int rc = static_workspace(&ws); rc != TT_OK) return rc;
    const int rc = tt_conv2d_bias_relu(x, w, bias, residual, y, shape, cls, sched, ws, TT_STATIC_WORKSPACE_BYTES, stream);
    if (rc == TT_ERR_WORKSPACE)
        snprintf(tt::g_last_error, sizeof tt::g_last_error,
                 "tt_conv2d_bias_relu_noalloc: the split-K partial sums of this (schedule, shape) exceed the "
                 "library's static workspace of %d bytes", (int)TT_STATIC_WORKSPACE_BYTES);
    return rc;
}

extern "C" int tt_conv2d_bias_relu(const void *x, const void *w, const void *bias, const void *residual, void *y,
                                   const tt_conv_shape *shape, int cls, const tt_schedule *sched, void *ws,
                                   size_t ws_bytes, void *stream)
{
    if (!x || !w || !y || !shape || !is_conv_class(cls)) return TT_ERR_BAD_ARG;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y) || !aligned16(bias) || !aligned16(residual))
        return TT_ERR_BAD_ARG;
    if ((cls == TT_CONV2D_BIAS_ADD_RELU) != (residual != nullptr)) return TT_ERR_BAD_ARG;
    tt_plan plan;
    const int rc = make_plan(sched, cls, shape, ws, ws_bytes, &plan);
    if (rc != TT_OK) return rc;
    // the matrix-core kernels address both tensors with 32-bit byte offsets below 2^31 and keep one
    // bit per filter row
    const int elem = shape->dtype == TT_F32 ? 4 : 2;
    const int64_t x_bytes = (int64_t)shape->n * shape->h * shape->w * shape->c * elem;
    const int64_t w_bytes = (int64_t)shape->k * shape->r * shape->s * shape->c * elem;
    if (plan.sketch == TT_SK_MFMA && (x_bytes >= (1ll << 31) || w_bytes >= (1ll << 31) || shape->r > 32))
        return TT_ERR_UNSUPPORTED;
    ContractArgs g;
    std::memset(&g, 0, sizeof g);
    fill_common(g, plan, sched, cls, shape->dtype);
    g.a = x;
    g.b = w;
    g.bias = bias;
    g.res = residual;
    g.out = y;
    g.ws = static_cast<float *>(ws);
    g.has_bias = bias != nullptr;
    g.has_res = residual != nullptr;
    g.C = shape->c;
    g.H = shape->h;
    g.W = shape->w;
    g.R = shape->r;
    g.S = shape->s;
    g.stride_h = shape->stride_h;
    g.stride_w = shape->stride_w;
    g.pad_h = shape->pad_h;
    g.pad_w = shape->pad_w;
    g.Ho = conv_out(shape->h, shape->r, shape->stride_h, shape->pad_h);
    g.Wo = conv_out(shape->w, shape->s, shape->stride_w, shape->pad_w);
    const int per_item = 16 / elem;
    g.run = shape->s * shape->c;
    g.runp = (g.run + per_item - 1) / per_item * per_item;
    g.k_walk = shape->r * g.runp;
    g.div_hw = make_fastdiv((uint32_t)(g.Ho * g.Wo));
    g.div_wo = make_fastdiv((uint32_t)g.Wo);
    g.PW = shape->w + 2 * shape->pad_w;
    g.PHW = (shape->h + 2 * shape->pad_h) * g.PW;
    g.div_phw = make_fastdiv((uint32_t)g.PHW);
    g.div_pw = make_fastdiv((uint32_t)g.PW);
    g.a_bytes = (uint32_t)x_bytes;
    g.b_bytes = (uint32_t)w_bytes;
    int family = FAM_CONV;
    if (plan.sketch == TT_SK_MFMA && plan.variant_id >= 0 && plan.variant_id < kNumVariants)
        family = kVariants[plan.variant_id].family; // the dense family for unit-stride 1x1 filters
    return run_contraction(g, plan, family, stream);
}

static int gemm_entry(const void *a, const void *b, const void *bias, void *c, const tt_gemm_shape *shape, int cls,
                      const tt_schedule *sched, void *ws, size_t ws_bytes, void *stream)
{
    if (!a || !b || !c || !shape) return TT_ERR_BAD_ARG;
    if (!aligned16(a) || !aligned16(b) || !aligned16(c) || !aligned16(bias)) return TT_ERR_BAD_ARG;
    tt_plan plan;
    const int rc = make_plan(sched, cls, shape, ws, ws_bytes, &plan);
    if (rc != TT_OK) return rc;
    ContractArgs g;
    std::memset(&g, 0, sizeof g);
    fill_common(g, plan, sched, cls, shape->dtype);
    g.a = a;
    g.b = b;
    g.bias = bias;
    g.out = c;
    g.ws = static_cast<float *>(ws);
    g.has_bias = bias != nullptr;
    g.Ho = g.Wo = 1;
    return run_contraction(g, plan, family_of(cls, shape->trans_b), stream);
}

extern "C" int tt_dense_bias_relu(const void *x, const void *w, const void *bias, void *y,
                                  const tt_gemm_shape *shape, int cls, const tt_schedule *sched, void *ws,
                                  size_t ws_bytes, void *stream)
{
    if (!is_dense_class(cls)) return TT_ERR_BAD_ARG;
    return gemm_entry(x, w, bias, y, shape, cls, sched, ws, ws_bytes, stream);
}

extern "C" int tt_batch_matmul(const void *a, const void *b, void *c, const tt_gemm_shape *shape,
                               const tt_schedule *sched, void *ws, size_t ws_bytes, void *stream)
{
    return gemm_entry(a, b, nullptr, c, shape, TT_BATCH_MATMUL, sched, ws, ws_bytes, stream);
}

extern "C" int tt_dwconv(const void *x, const void *w, const void *bias, void *y, const tt_conv_shape *shape,
                         const tt_schedule *sched, void *stream)
{
    if (!x || !w || !y || !shape) return TT_ERR_BAD_ARG;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y) || !aligned16(bias)) return TT_ERR_BAD_ARG;
    tt_plan plan;
    const int rc = make_plan(sched, TT_DWCONV_BIAS_RELU6, shape, nullptr, 0, &plan);
    if (rc != TT_OK) return rc;
    if (shape->dtype != TT_F32 || shape->r != 3 || shape->s != 3) return TT_ERR_UNSUPPORTED;
    DwArgs g;
    std::memset(&g, 0, sizeof g);
    g.x = static_cast<const float *>(x);
    g.w = static_cast<const float *>(w);
    g.bias = static_cast<const float *>(bias);
    g.y = static_cast<float *>(y);
    g.map = tile_map_of(plan);
    g.planes = shape->n * shape->c;
    g.C = shape->c;
    g.H = shape->h;
    g.W = shape->w;
    g.Ho = plan.M;
    g.Wo = plan.N;
    g.stride_h = shape->stride_h;
    g.stride_w = shape->stride_w;
    g.pad_h = shape->pad_h;
    g.pad_w = shape->pad_w;
    g.wave_m = plan.wave_m;
    g.wave_n = plan.wave_n;
    g.stages = plan.stages;
    g.unroll = plan.eff_unroll;
    g.eff_vec = plan.eff_vec_a;
    const int64_t x_bytes = (int64_t)shape->n * shape->h * shape->w * shape->c * 4;
    g.x_bytes = x_bytes < (1ll << 31) ? (uint32_t)x_bytes : 0u;
    if (plan.sketch == TT_SK_DIRECT) return launch_dw_direct(g, plan.grid, stream);
    return launch_dwconv(g, plan, stream);
}

extern "C" int tt_debug_tile_map(const tt_plan *plan, int32_t *out_dev, void *stream)
{
    if (!plan || !out_dev || plan->status != TT_OK || plan->sketch == TT_SK_DIRECT || plan->grid < 1)
        return TT_ERR_BAD_ARG;
    return launch_tile_map_dump(tile_map_of(*plan), out_dev, stream);
}

// ---- standalone timing of one (kernel, schedule) pair (Section 4.3: pairs run as distinct programs) ----------

namespace {

// `turn` picks the tensor set: 0 = bufs, then the alternatives in order, round and round.
int launch_kernel_desc(const tt_kernel_desc &k, const tt_schedule *sched, void *stream, int64_t turn = 0)
{
    void *const *b = k.bufs;
    if (k.n_alt > 0) {
        const int set = (int)(turn % (k.n_alt + 1));
        if (set > 0) b = k.alt_bufs + (size_t)(set - 1) * 5;
    }
    if (is_conv_class(k.cls))
        return tt_conv2d_bias_relu(b[0], b[1], b[2], b[3], b[4], static_cast<const tt_conv_shape *>(k.shape), k.cls, sched,
                                   k.ws, k.ws_bytes, stream);
    if (is_dense_class(k.cls))
        return tt_dense_bias_relu(b[0], b[1], b[2], b[3], static_cast<const tt_gemm_shape *>(k.shape), k.cls, sched, k.ws,
                                  k.ws_bytes, stream);
    if (k.cls == TT_BATCH_MATMUL)
        return tt_batch_matmul(b[0], b[1], b[2], static_cast<const tt_gemm_shape *>(k.shape), sched, k.ws, k.ws_bytes,
                               stream);
    if (k.cls == TT_DWCONV_BIAS_RELU6)
        return tt_dwconv(b[0], b[1], b[2], b[3], static_cast<const tt_conv_shape *>(k.shape), sched, stream);
    return TT_ERR_BAD_ARG;
}

struct Timer {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    bool ok = false;
    Timer() { ok = hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess; }
    ~Timer()
    {
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    }
};

tt_sweep_opts resolve(const tt_sweep_opts *o)
{
    tt_sweep_opts r;
    r.warmup = 3;
    r.samples = 10;
    r.min_sample_us = 200;
    r.max_launches = 64;
    r.flags = 0;
    r.allow_slower_than_default = 0;
    r.pair_budget = 0;
    r.prioritise = 0;
    r.seed = 0;
    if (o) {
        r.pair_budget = o->pair_budget;
        r.prioritise = o->prioritise;
        r.seed = o->seed;
        if (o->warmup >= 0) r.warmup = o->warmup;
        if (o->samples > 0) r.samples = o->samples;
        if (o->min_sample_us > 0) r.min_sample_us = o->min_sample_us;
        if (o->max_launches > 0) r.max_launches = o->max_launches;
        r.flags = o->flags;
        r.allow_slower_than_default = o->allow_slower_than_default;
    }
    return r;
}

int time_pair(const tt_kernel_desc &k, const tt_schedule *sched, const tt_sweep_opts &o, hipStream_t s, Timer &t,
              double *median_us, double *min_us)
{
    // Validity first: nothing is launched for a record that does not apply.
    tt_schedule def;
    const tt_schedule *rec = sched;
    if (!rec) {
        const int rc = tt_schedule_default(k.cls, k.shape, &def);
        if (rc != TT_OK) return rc;
        rec = &def;
    }
    if (k.n_alt < 0 || (k.n_alt > 0 && !k.alt_bufs)) return TT_ERR_BAD_ARG;
    tt_plan plan;
    int rc = tt_schedule_apply(rec, k.cls, k.shape, o.flags, &plan);
    if (rc != TT_OK) return rc;
    // Launches so far, over all timed pairs of the process: every launch moves on to the next tensor set, and
    // the next pair carries on where this one stops (a pair that started over at the first set would find it,
    // and the few sets a short measurement touches, still in the memory-side cache from the pair before).
    static std::atomic<int64_t> turns{0};
    auto next_turn = [&]() { return turns.fetch_add(1, std::memory_order_relaxed); };
    for (int i = 0; i < std::max(1, o.warmup); ++i) {
        rc = launch_kernel_desc(k, rec, s, next_turn());
        if (rc != TT_OK) return rc;
    }
    // Size a sample: time one launch, then batch enough launches to fill min_sample_us.
    float ms = 0.0f;
    if (hipEventRecord(t.e0, s) != hipSuccess) return TT_ERR_HIP;
    rc = launch_kernel_desc(k, rec, s, next_turn());
    if (rc != TT_OK) return rc;
    if (hipEventRecord(t.e1, s) != hipSuccess || hipEventSynchronize(t.e1) != hipSuccess ||
        hipEventElapsedTime(&ms, t.e0, t.e1) != hipSuccess)
        return TT_ERR_HIP;
    const double one_us = std::max(1.0, (double)ms * 1000.0);
    const int launches = (int)std::min<double>(o.max_launches, std::max(1.0, o.min_sample_us / one_us + 0.999));
    std::vector<double> us(o.samples);
    for (int smp = 0; smp < o.samples; ++smp) {
        if (hipEventRecord(t.e0, s) != hipSuccess) return TT_ERR_HIP;
        for (int l = 0; l < launches; ++l) {
            rc = launch_kernel_desc(k, rec, s, next_turn());
            if (rc != TT_OK) return rc;
        }
        if (hipEventRecord(t.e1, s) != hipSuccess || hipEventSynchronize(t.e1) != hipSuccess ||
            hipEventElapsedTime(&ms, t.e0, t.e1) != hipSuccess)
            return TT_ERR_HIP;
        us[smp] = (double)ms * 1000.0 / launches;
    }
    std::sort(us.begin(), us.end());
    const int n = (int)us.size();
    if (median_us) *median_us = n % 2 ? us[n / 2] : 0.5 * (us[n / 2 - 1] + us[n / 2]);
    if (min_us) *min_us = us[0];
    return TT_OK;
}

} // namespace

extern "C" int tt_time_pair(const tt_kernel_desc *kernel, const tt_schedule *sched, const tt_sweep_opts *opts,
                            void *stream, double *median_us, double *min_us)
{
    if (!kernel || !kernel->shape) return TT_ERR_BAD_ARG;
    Timer t;
    if (!t.ok) return TT_ERR_HIP;
    return time_pair(*kernel, sched, resolve(opts), static_cast<hipStream_t>(stream), t, median_us, min_us);
}

extern "C" int tt_run_kernels(const tt_kernel_desc *kernels, const tt_schedule *const *scheds, int nk, int repeat,
                              void *stream)
{
    if (nk < 0 || repeat < 0 || (nk && !kernels)) return TT_ERR_BAD_ARG;
    for (int r = 0; r < repeat; ++r)
        for (int k = 0; k < nk; ++k) {
            if (!kernels[k].shape) return TT_ERR_BAD_ARG;
            for (int u = 0; u < kernels[k].use_count; ++u) {
                const int rc = launch_kernel_desc(kernels[k], scheds ? scheds[k] : nullptr, stream);
                if (rc != TT_OK) return rc;
            }
        }
    return TT_OK;
}

extern "C" int tt_transfer_sweep(const tt_kernel_desc *kernels, int nk, const tt_schedule *pool, int np,
                                 const tt_sweep_opts *opts, void *stream, tt_sweep_row *rows, double *pair_us,
                                 int64_t *evaluations, double *wall_seconds)
{
    if (nk < 0 || np < 0 || (nk && (!kernels || !rows)) || (np && !pool)) return TT_ERR_BAD_ARG;
    const auto t0 = std::chrono::steady_clock::now();
    const tt_sweep_opts o = resolve(opts);
    hipStream_t s = static_cast<hipStream_t>(stream);
    Timer timer;
    if (!timer.ok) return TT_ERR_HIP;
    std::vector<double> local((size_t)nk * np, -2.0), defaults(nk, 0.0), weight(nk, 0.0);
    std::vector<int32_t> kcls(nk), pcls(np);
    for (int p = 0; p < np; ++p) pcls[p] = pool[p].cls;
    int64_t evals = 0;
    // the default ("untuned") schedule is always evaluated: it is the baseline and the fallback
    for (int k = 0; k < nk; ++k) {
        if (!kernels[k].shape) return TT_ERR_BAD_ARG;
        kcls[k] = kernels[k].cls;
        const int rc = time_pair(kernels[k], nullptr, o, s, timer, &defaults[k], nullptr);
        if (rc != TT_OK) return rc;
        weight[k] = defaults[k] * std::max(1, kernels[k].use_count);
        ++evals;
    }
    // which same-class pairs are tried: all of them, or the budgeted subset
    std::vector<uint8_t> mask((size_t)nk * np + 1, 0);
    if (const int rc = tt_sweep_plan(kcls.data(), weight.data(), nk, pcls.data(), np, o.pair_budget, o.prioritise, o.seed,
                                     mask.data(), nullptr);
        rc != TT_OK)
        return rc;
    for (int k = 0; k < nk; ++k)
        for (int p = 0; p < np; ++p) {
            if (pool[p].cls != kernels[k].cls) continue; // other classes are never tried (Section 4.2)
            if (!mask[(size_t)k * np + p]) {
                local[(size_t)k * np + p] = -3.0;
                continue;
            }
            ++evals;
            double us = -1.0;
            const int rc = time_pair(kernels[k], &pool[p], o, s, timer, &us, nullptr);
            if (rc == TT_ERR_HIP) return rc;
            // every other failure means "this record does not fit this kernel": the paper's -1
            local[(size_t)k * np + p] = rc == TT_OK ? us : -1.0;
        }
    if (hipStreamSynchronize(s) != hipSuccess) return TT_ERR_HIP;
    const int rc = tt_sweep_select(kcls.data(), nk, pcls.data(), np, local.data(), defaults.data(),
                                   o.allow_slower_than_default, rows);
    if (rc != TT_OK) return rc;
    if (pair_us) std::copy(local.begin(), local.end(), pair_us);
    if (evaluations) *evaluations = evals;
    if (wall_seconds) *wall_seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    return TT_OK;
}

// ---- local refinement of a record (Section 6's outlook) and the native sweep of one kernel -----------------

extern "C" int tt_refine(const tt_kernel_desc *kernel, const tt_schedule *base, int rounds, const tt_sweep_opts *opts,
                         void *stream, tt_schedule *best, double *best_us, double *base_us, int32_t *tried)
{
    if (!kernel || !kernel->shape || !base || !best || rounds < 0) return TT_ERR_BAD_ARG;
    const tt_sweep_opts o = resolve(opts);
    hipStream_t s = static_cast<hipStream_t>(stream);
    Timer timer;
    if (!timer.ok) return TT_ERR_HIP;
    double cur_us = 0.0;
    int rc = time_pair(*kernel, base, o, s, timer, &cur_us, nullptr);
    if (rc != TT_OK) return rc;
    int32_t n = 1;
    tt_schedule cur = *base;
    if (base_us) *base_us = cur_us;
    for (int r = 0; r < rounds; ++r) {
        const int count = tt_refine_space(&cur, nullptr, 0);
        if (count <= 0) break;
        std::vector<tt_schedule> near(count);
        tt_refine_space(&cur, near.data(), count);
        int win = -1;
        double win_us = cur_us;
        for (int i = 0; i < count; ++i) {
            double us = 0.0;
            rc = time_pair(*kernel, &near[i], o, s, timer, &us, nullptr);
            if (rc == TT_ERR_HIP) return rc;
            if (rc != TT_OK) continue; // does not apply to this kernel, or no kernel implements it
            ++n;
            if (us < win_us) { // strict: the current record, then the lowest index, win ties
                win_us = us;
                win = i;
            }
        }
        if (win < 0) break;
        const int32_t keep_id = cur.id;
        cur = near[win];
        cur.id = keep_id;
        cur_us = win_us;
    }
    if (hipStreamSynchronize(s) != hipSuccess) return TT_ERR_HIP;
    *best = cur;
    if (best_us) *best_us = cur_us;
    if (tried) *tried = n;
    return TT_OK;
}

extern "C" int tt_native_sweep(const tt_kernel_desc *kernel, int level, int finalists, const tt_sweep_opts *explore,
                               const tt_sweep_opts *full, void *stream, tt_schedule *best, double *best_us,
                               double *default_us, int32_t *n_valid, int32_t *n_records)
{
    if (!kernel || !kernel->shape || !best || finalists < 1) return TT_ERR_BAD_ARG;
    tt_sweep_opts quick;
    std::memset(&quick, 0, sizeof quick);
    quick.warmup = 1;
    quick.samples = 3;
    quick.min_sample_us = 60;
    quick.max_launches = 16;
    const tt_sweep_opts ex = explore ? resolve(explore) : quick, fu = resolve(full);
    const bool conv = is_conv_class(kernel->cls) || kernel->cls == TT_DWCONV_BIAS_RELU6;
    const int dtype = conv ? static_cast<const tt_conv_shape *>(kernel->shape)->dtype
                           : static_cast<const tt_gemm_shape *>(kernel->shape)->dtype;
    const int count = tt_schedule_space(kernel->cls, dtype, level, nullptr, 0);
    if (count < 0) return count;
    std::vector<tt_schedule> space(std::max(count, 1));
    tt_schedule_space(kernel->cls, dtype, level, space.data(), count);
    hipStream_t s = static_cast<hipStream_t>(stream);
    Timer timer;
    if (!timer.ok) return TT_ERR_HIP;

    // the `keep` fastest records of a list under one protocol, fastest first (ties: list order)
    struct Timed {
        double us;
        int index;
    };
    int valid = 0;
    const auto fastest = [&](const std::vector<tt_schedule> &list, int n, const tt_sweep_opts &o, size_t keep, bool count_valid,
                             std::vector<tt_schedule> *out, std::vector<double> *out_us) -> int {
        std::vector<Timed> t;
        for (int i = 0; i < n; ++i) {
            double us = 0.0;
            const int rc = time_pair(*kernel, &list[i], o, s, timer, &us, nullptr);
            if (rc == TT_ERR_HIP) return rc;
            if (rc != TT_OK) continue;
            if (count_valid) ++valid;
            t.push_back({us, i});
        }
        std::stable_sort(t.begin(), t.end(), [](const Timed &a, const Timed &b) { return a.us < b.us; });
        out->clear();
        if (out_us) out_us->clear();
        for (size_t i = 0; i < t.size() && i < keep; ++i) {
            out->push_back(list[t[i].index]);
            if (out_us) out_us->push_back(t[i].us);
        }
        return TT_OK;
    };
    std::vector<tt_schedule> top;
    int rc = fastest(space, count, ex, (size_t)finalists, true, &top, nullptr);
    if (rc != TT_OK) return rc;
    if (!top.empty() && top[0].sketch == TT_SK_MFMA) {
        // the enumerated space carries one unroll setting and (below level 2) two workgroup orders: the
        // finalists are re-tried under all of them
        std::vector<tt_schedule> wide;
        for (const tt_schedule &f : top)
            for (int order = 0; order < 6; ++order)
                for (int unroll : {8, 1}) {
                    tt_schedule r = f;
                    r.order = order;
                    r.unroll = unroll;
                    bool seen = false;
                    for (const tt_schedule &w : wide) seen = seen || std::memcmp(&w, &r, sizeof(int32_t) * 13) == 0;
                    if (!seen) wide.push_back(r);
                }
        rc = fastest(wide, (int)wide.size(), ex, (size_t)finalists, false, &top, nullptr);
        if (rc != TT_OK) return rc;
    }
    std::vector<double> top_us;
    rc = fastest(top, (int)top.size(), fu, 1, false, &top, &top_us);
    if (rc != TT_OK) return rc;
    double def_us = 0.0;
    rc = time_pair(*kernel, nullptr, fu, s, timer, &def_us, nullptr);
    if (rc != TT_OK) return rc;
    if (hipStreamSynchronize(s) != hipSuccess) return TT_ERR_HIP;
    if (!top.empty() && top_us[0] < def_us) { // the default wins ties
        *best = top[0];
        if (best_us) *best_us = top_us[0];
    } else {
        rc = tt_schedule_default(kernel->cls, kernel->shape, best);
        if (rc != TT_OK) return rc;
        if (best_us) *best_us = def_us;
    }
    if (default_us) *default_us = def_us;
    if (n_valid) *n_valid = valid;
    if (n_records) *n_records = count;
    return TT_OK;
}
