// Kernels that do not use the matrix cores: the one-thread-per-output "direct"
// sketch (the unscheduled loop nest, always valid), the split-K reduction with
// the fused epilogue, the wave-reduction GEMV sketch for small-M dense kernels,
// the depthwise 3x3 tile kernel, and the index-map dump.
#include <hip/hip_runtime.h>

#include "contract.hip.h"
#include "tt_internal.h"

namespace tt {

namespace {

inline int launched()
{
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : note_hip_error((int)e, "kernel launch");
}

// ---- direct sketch: one thread per output element ------------------------------------------------
template <int DT, int FAM> __global__ void __launch_bounds__(256) direct_kernel(const ContractArgs g)
{
    using E = typename ElemOf<DT>::type;
    const int64_t total = (int64_t)g.batch * g.M * g.N;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const E *a = static_cast<const E *>(g.a), *b = static_cast<const E *>(g.b);
    float acc = 0.0f;
    int n;
    if constexpr (FAM == FAM_CONV) {
        // idx walks the NHWC output: (img, p, q, n); activations NHWC, filters KRSC
        n = (int)(idx % g.N);
        const int64_t pix = idx / g.N;
        const int q = (int)(pix % g.Wo), p = (int)((pix / g.Wo) % g.Ho);
        const int img = (int)(pix / ((int64_t)g.Ho * g.Wo));
        for (int r = 0; r < g.R; ++r) {
            const int ih = p * g.stride_h + r - g.pad_h;
            if (ih < 0 || ih >= g.H) continue;
            for (int s = 0; s < g.S; ++s) {
                const int iw = q * g.stride_w + s - g.pad_w;
                if (iw < 0 || iw >= g.W) continue;
                const E *xp = a + (((int64_t)img * g.H + ih) * g.W + iw) * g.C;
                const E *wp = b + (((int64_t)n * g.R + r) * g.S + s) * g.C;
                for (int c = 0; c < g.C; ++c) acc = fmaf(load_as_float<DT>(xp, c), load_as_float<DT>(wp, c), acc);
            }
        }
    } else {
        n = (int)(idx % g.N);
        const int m = (int)((idx / g.N) % g.M);
        const int bi = (int)(idx / ((int64_t)g.M * g.N));
        const E *ar = a + ((int64_t)bi * g.M + m) * g.K;
        const E *bb = b + (int64_t)bi * g.N * g.K;
        for (int k = 0; k < g.K; ++k) {
            const float bv = FAM == FAM_GEMM_TN ? load_as_float<DT>(bb, (int64_t)n * g.K + k)
                                                : load_as_float<DT>(bb, (int64_t)k * g.N + n);
            acc = fmaf(load_as_float<DT>(ar, k), bv, acc);
        }
    }
    if (g.has_bias) acc += load_as_float<DT>(g.bias, n);
    if (g.has_res) acc += load_as_float<DT>(g.res, idx);
    store_from_float<DT>(g.out, idx, apply_act(acc, g.act));
}

// ---- split-K: sum the partial tiles in split order, then the fused epilogue -----------------------
template <int DT> __global__ void __launch_bounds__(256) splitk_reduce_kernel(const ContractArgs g)
{
    const int64_t total = (int64_t)g.batch * g.M * g.N;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    float acc = 0.0f;
    for (int z = 0; z < g.map.eff_split_k; ++z) acc += g.ws[(int64_t)z * total + idx];
    const int n = (int)(idx % g.N);
    if (g.has_bias) acc += load_as_float<DT>(g.bias, n);
    if (g.has_res) acc += load_as_float<DT>(g.res, idx);
    store_from_float<DT>(g.out, idx, apply_act(acc, g.act));
}

// ---- GEMV sketch: a wave owns WN outputs of TMR rows; lanes split K; butterfly reduction ---------
template <int DT> __global__ void __launch_bounds__(1024) gemv_kernel(const ContractArgs g, int tile_m, int wave_n, int chunk)
{
    using E = typename ElemOf<DT>::type;
    const TileCoord tc = decode_tile(g.map, (int32_t)blockIdx.x);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n_first = tc.n0 + wave * wave_n;
    const E *x = static_cast<const E *>(g.a), *w = static_cast<const E *>(g.b);
    const int ev = g.eff_vec_a;
    // Every array below is indexed by unrolled loop counters only (rows and outputs beyond tile_m and
    // wave_n are skipped by wave-uniform tests), so all of it stays in registers.
    float acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0.0f;
    const int step = 64 * chunk;
    for (int kb = 0; kb < g.K; kb += step) {
        const int k = kb + lane * chunk;
        for (int c0 = 0; c0 < chunk; c0 += ev) {
            // ev consecutive K per access; K % ev == 0 so a group is all in or all out
            if (k + c0 >= g.K) break;
            for (int e = 0; e < ev; ++e) {
                const int64_t kk = k + c0 + e;
                float xv[8], wv[8];
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    xv[i] = (i < tile_m && tc.m0 + i < g.M) ? load_as_float<DT>(x, (int64_t)(tc.m0 + i) * g.K + kk) : 0.0f;
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    wv[j] = (j < wave_n && n_first + j < g.N) ? load_as_float<DT>(w, (int64_t)(n_first + j) * g.K + kk) : 0.0f;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    if (i >= tile_m) break;
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[i][j] = fmaf(xv[i], wv[j], acc[i][j]);
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if (i >= tile_m) break;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (j >= wave_n) break;
            float v = acc[i][j];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
            const int m = tc.m0 + i, n = n_first + j;
            if (lane == 0 && m < g.M && n < g.N && n < tc.n0 + tc.n_ext) {
                if (g.has_bias) v += load_as_float<DT>(g.bias, n);
                store_from_float<DT>(g.out, (int64_t)m * g.N + n, apply_act(v, g.act));
            }
        }
    }
}

// ---- depthwise 3x3 over NHWC: (rows, cols, planes) tile per workgroup, WM x WN outputs per thread ---
// A plane is one (image, channel) pair, numbered image * C + channel.  Threads are laid out planes
// fastest, then cols, then rows, so the lanes of a wave read and write neighbouring channels of one
// pixel.  With two stages the input patch of the tile is first copied to LDS (planes fastest too).
template <int WM, int WN, int MAXT> __global__ void __launch_bounds__(MAXT) dwconv3x3_kernel(const DwArgs g)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    float *patch = reinterpret_cast<float *>(smem_raw);
    const TileCoord tc = decode_tile(g.map, (int32_t)blockIdx.x);
    const int tk = g.map.tile_k;
    const int tcols = g.map.tile_n / WN;
    const int tid = threadIdx.x;
    const int tp = tid % tk, tx = (tid / tk) % tcols, ty = tid / (tk * tcols);
    const int plane = tc.k0 + tp;
    const int p0 = tc.m0 + ty * WM, q0 = tc.n0 + tx * WN;
    const int prow = (g.map.tile_m - 1) * g.stride_h + 3, pcol = (g.map.tile_n - 1) * g.stride_w + 3;
    const int ih_org = tc.m0 * g.stride_h - g.pad_h, iw_org = tc.n0 * g.stride_w - g.pad_w;
    if (g.stages == 2) {
        const int total = prow * pcol * tk;
        for (int e = tid; e < total; e += blockDim.x) {
            const int pl = e % tk, cell = e / tk;
            const int rr = cell / pcol, cc = cell - rr * pcol;
            const int ih = ih_org + rr, iw = iw_org + cc;
            float v = 0.0f;
            if (pl < tc.k_ext && ih >= 0 && ih < g.H && iw >= 0 && iw < g.W) {
                const int pn = (tc.k0 + pl) / g.C, pc = (tc.k0 + pl) - pn * g.C;
                v = g.x[(((int64_t)pn * g.H + ih) * g.W + iw) * g.C + pc];
            }
            patch[e] = v;
        }
        __syncthreads();
    }
    if (tp >= tc.k_ext) return;
    const int img = plane / g.C, ch = plane - img * g.C;
    float wgt[9];
#pragma unroll
    for (int i = 0; i < 9; ++i) wgt[i] = g.w[i * g.C + ch];
    const float bias = g.bias ? g.bias[ch] : 0.0f;
    const float *xp = g.x + (int64_t)img * g.H * g.W * g.C + ch;
    float *yp = g.y + (int64_t)img * g.Ho * g.Wo * g.C + ch;
    auto body = [&](int i) {
        const int p = p0 + i;
        if (p >= g.Ho || p >= tc.m0 + tc.m_ext) return;
        float out[WN];
#pragma unroll
        for (int j = 0; j < WN; ++j) out[j] = bias;
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const int ih = p * g.stride_h + r - g.pad_h;
#pragma unroll
            for (int j = 0; j < WN; ++j) {
#pragma unroll
                for (int s = 0; s < 3; ++s) {
                    const int iw = (q0 + j) * g.stride_w + s - g.pad_w;
                    float v = 0.0f;
                    if (g.stages == 2) {
                        v = patch[((ih - ih_org) * pcol + (iw - iw_org)) * tk + tp];
                    } else if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W) {
                        v = xp[((int64_t)ih * g.W + iw) * g.C];
                    }
                    out[j] = fmaf(v, wgt[r * 3 + s], out[j]);
                }
            }
        }
        const int qlim = min(g.Wo, tc.n0 + tc.n_ext);
#pragma unroll
        for (int j = 0; j < WN; ++j)
            if (q0 + j < qlim) yp[((int64_t)p * g.Wo + q0 + j) * g.C] = fminf(fmaxf(out[j], 0.0f), 6.0f);
    };
    if (g.unroll >= WM) {
#pragma unroll
        for (int i = 0; i < WM; ++i) body(i);
    } else {
#pragma unroll 1
        for (int i = 0; i < WM; ++i) body(i);
    }
}

// ---- depthwise 3x3, register version: VC channel-contiguous planes per lane, unit or double stride ---
// The same tile and thread layout as above, without LDS.  For each of its WM output rows a thread
// fetches the three input rows it needs, each input pixel once, as VC-wide vectors through
// bounds-checked buffer loads (an offset outside the tensor reads as zero, which is the padding),
// then forms its WN outputs.  Lanes of a wave hold neighbouring channel groups of one pixel, so
// every load and store instruction covers one contiguous run of memory.
template <int WM, int WN, int VC, int STR, int MAXT>
__global__ void __launch_bounds__(MAXT) dwconv3x3_rows_kernel(const DwArgs g)
{
    typedef __attribute__((ext_vector_type(VC))) float vec_t;
    constexpr int COLS = (WN - 1) * STR + 3;
    const TileCoord tc = decode_tile(g.map, (int32_t)blockIdx.x);
    const int lanes_k = g.map.tile_k / VC; // lanes along the plane axis
    const int tcols = g.map.tile_n / WN;
    const int tid = threadIdx.x;
    const int tp = tid % lanes_k, tx = (tid / lanes_k) % tcols, ty = tid / (lanes_k * tcols);
    const int plane = tc.k0 + tp * VC;
    if (plane >= tc.k0 + tc.k_ext) return;
    const int img = plane / g.C, ch = plane - img * g.C;
    const int p0 = tc.m0 + ty * WM, q0 = tc.n0 + tx * WN;
    const __amdgpu_buffer_rsrc_t xr = make_rsrc(g.x, g.x_bytes);

    vec_t wgt[9], bias;
#pragma unroll
    for (int i = 0; i < 9; ++i) wgt[i] = *reinterpret_cast<const vec_t *>(g.w + i * g.C + ch);
#pragma unroll
    for (int v = 0; v < VC; ++v) bias[v] = g.bias ? g.bias[ch + v] : 0.0f;

    // byte offset of input column c of this thread's window, or out of range
    const int iw0 = q0 * STR - g.pad_w;
    uint32_t col_off[COLS];
#pragma unroll
    for (int c = 0; c < COLS; ++c) {
        const int iw = iw0 + c;
        col_off[c] = (iw >= 0 && iw < g.W) ? (uint32_t)((iw * g.C + ch) * 4) : kOutOfRange;
    }
    const int plim = min(g.Ho, tc.m0 + tc.m_ext), qlim = min(g.Wo, tc.n0 + tc.n_ext);
    float *yp = g.y + (int64_t)img * g.Ho * g.Wo * g.C + ch;

    auto body = [&](int i) {
        const int p = p0 + i;
        if (p >= plim) return;
        vec_t out[WN];
#pragma unroll
        for (int j = 0; j < WN; ++j) out[j] = bias;
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const int ih = p * STR + r - g.pad_h;
            const bool row_ok = ih >= 0 && ih < g.H;
            const uint32_t row_off = (uint32_t)((img * g.H + ih) * g.W * g.C * 4);
            vec_t in[COLS];
#pragma unroll
            for (int c = 0; c < COLS; ++c) {
                // an out-of-range column keeps its sentinel: the sum below stays out of range for every row offset
                const uint32_t off = (row_ok && col_off[c] != kOutOfRange) ? row_off + col_off[c] : kOutOfRange;
                if constexpr (VC == 4) {
                    const u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(xr, off, 0, 0);
                    in[c] = __builtin_bit_cast(vec_t, t);
                } else if constexpr (VC == 2) {
                    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
                    const u32x2 t = __builtin_amdgcn_raw_buffer_load_b64(xr, off, 0, 0);
                    in[c] = __builtin_bit_cast(vec_t, t);
                } else {
                    in[c][0] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(xr, off, 0, 0));
                }
            }
#pragma unroll
            for (int j = 0; j < WN; ++j)
#pragma unroll
                for (int s = 0; s < 3; ++s)
#pragma unroll
                    for (int v = 0; v < VC; ++v) out[j][v] = fmaf(in[j * STR + s][v], wgt[r * 3 + s][v], out[j][v]);
        }
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            if (q0 + j >= qlim) continue;
            vec_t o;
#pragma unroll
            for (int v = 0; v < VC; ++v) o[v] = fminf(fmaxf(out[j][v], 0.0f), 6.0f);
            __builtin_nontemporal_store(o, reinterpret_cast<vec_t *>(yp + ((int64_t)p * g.Wo + q0 + j) * g.C)); // streamed
        }
    };
    if (g.unroll >= WM) {
#pragma unroll
        for (int i = 0; i < WM; ++i) body(i);
    } else {
#pragma unroll 1
        for (int i = 0; i < WM; ++i) body(i);
    }
}

__global__ void __launch_bounds__(256) dw_direct_kernel(const DwArgs g)
{
    // idx walks the NHWC output: (image, p, q, channel)
    const int64_t total = (int64_t)g.planes * g.Ho * g.Wo;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int ch = (int)(idx % g.C);
    const int64_t pix = idx / g.C;
    const int q = (int)(pix % g.Wo), p = (int)((pix / g.Wo) % g.Ho);
    const int img = (int)(pix / ((int64_t)g.Ho * g.Wo));
    float acc = 0.0f;
    for (int r = 0; r < 3; ++r) {
        const int ih = p * g.stride_h + r - g.pad_h;
        if (ih < 0 || ih >= g.H) continue;
        for (int s = 0; s < 3; ++s) {
            const int iw = q * g.stride_w + s - g.pad_w;
            if (iw < 0 || iw >= g.W) continue;
            acc = fmaf(g.x[(((int64_t)img * g.H + ih) * g.W + iw) * g.C + ch], g.w[(r * 3 + s) * g.C + ch], acc);
        }
    }
    if (g.bias) acc += g.bias[ch];
    g.y[idx] = fminf(fmaxf(acc, 0.0f), 6.0f);
}

__global__ void __launch_bounds__(256) tile_map_dump_kernel(const TileMap map, int32_t *out)
{
    const int wg = blockIdx.x * 256 + threadIdx.x;
    if (wg >= map.grid) return;
    const TileCoord c = decode_tile(map, wg);
    int32_t *o = out + (int64_t)wg * 8;
    o[0] = c.hi;
    o[1] = c.lo;
    o[2] = c.m0;
    o[3] = c.m_ext;
    o[4] = c.n0;
    o[5] = c.n_ext;
    o[6] = c.k0;
    o[7] = c.k_ext;
}

template <int DT> int launch_direct_dt(const ContractArgs &a, int family, int grid, hipStream_t s)
{
    switch (family) {
    case FAM_CONV: hipLaunchKernelGGL((direct_kernel<DT, FAM_CONV>), dim3(grid), dim3(256), 0, s, a); break;
    case FAM_GEMM_TN: hipLaunchKernelGGL((direct_kernel<DT, FAM_GEMM_TN>), dim3(grid), dim3(256), 0, s, a); break;
    default: hipLaunchKernelGGL((direct_kernel<DT, FAM_GEMM_NN>), dim3(grid), dim3(256), 0, s, a); break;
    }
    return launched();
}

} // namespace

int launch_direct(const ContractArgs &args, int family, int grid, void *stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    return args.dtype == TT_F32 ? launch_direct_dt<TT_F32>(args, family, grid, s)
                                : launch_direct_dt<TT_BF16>(args, family, grid, s);
}

int launch_splitk_reduce(const ContractArgs &args, int family, void *stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t total = (int64_t)args.batch * args.M * args.N;
    const int grid = (int)((total + 255) / 256);
    (void)family; // every family writes a row-major [M][N] output
    if (args.dtype == TT_F32)
        hipLaunchKernelGGL((splitk_reduce_kernel<TT_F32>), dim3(grid), dim3(256), 0, s, args);
    else
        hipLaunchKernelGGL((splitk_reduce_kernel<TT_BF16>), dim3(grid), dim3(256), 0, s, args);
    return launched();
}

int launch_gemv(const ContractArgs &args, const tt_plan &plan, void *stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int chunk = plan.tile_k / 64;
    if (args.dtype == TT_F32)
        hipLaunchKernelGGL((gemv_kernel<TT_F32>), dim3(plan.grid), dim3(plan.block), 0, s, args, plan.tile_m,
                           plan.wave_n, chunk);
    else
        hipLaunchKernelGGL((gemv_kernel<TT_BF16>), dim3(plan.grid), dim3(plan.block), 0, s, args, plan.tile_m,
                           plan.wave_n, chunk);
    return launched();
}

// The depthwise kernels are compiled for workgroups of at most 256, 512 and 1024 threads, which leaves a
// lane 512, 256 and 128 registers.  What a lane keeps in flight grows with the input columns of its
// window times the planes per access (register kernel) or with its outputs per row (general kernel); the
// bounds below are the sizes the compiler keeps in registers (the build's resource report: no instance
// that these bounds admit uses scratch memory).
constexpr int dw_block_limit(int wave_m, int wave_n, int planes_per_lane, int stride, bool rows_kernel)
{
    const auto built = [](int w) { return w == 1 || w == 2 || w == 4 || w == 7; };
    if (!built(wave_m) || !built(wave_n)) return 0; // no instance for other outputs per thread
    if (rows_kernel) {
        const int in_flight = ((wave_n - 1) * stride + 3) * planes_per_lane;
        return in_flight <= 9 || (in_flight <= 16 && wave_n < 7) ? 1024 : in_flight <= 36 ? 512 : 256;
    }
    return wave_n <= 2 ? 1024 : wave_n <= 4 ? 512 : 256;
}

int dw_max_block(int wave_m, int wave_n, int planes_per_lane, int stride, bool rows_kernel)
{
    return dw_block_limit(wave_m, wave_n, planes_per_lane, stride, rows_kernel);
}

namespace {

template <int WM, int WN> int launch_dw_rows(const DwArgs &a, dim3 grid, dim3 block, hipStream_t s)
{
    const int str = a.stride_h;
#define TT_DW_ROWS(VC_, STR_)                                                                                        \
    if (a.eff_vec == VC_ && str == STR_) {                                                                           \
        constexpr int LIMIT = dw_block_limit(WM, WN, VC_, STR_, true);                                               \
        if ((int)block.x > LIMIT) return TT_ERR_UNSUPPORTED;                                                         \
        if (block.x <= 256) {                                                                                        \
            hipLaunchKernelGGL((dwconv3x3_rows_kernel<WM, WN, VC_, STR_, 256>), grid, block, 0, s, a);               \
        } else if (block.x <= 512) {                                                                                 \
            if constexpr (LIMIT >= 512)                                                                              \
                hipLaunchKernelGGL((dwconv3x3_rows_kernel<WM, WN, VC_, STR_, 512>), grid, block, 0, s, a);           \
        } else {                                                                                                     \
            if constexpr (LIMIT >= 1024)                                                                             \
                hipLaunchKernelGGL((dwconv3x3_rows_kernel<WM, WN, VC_, STR_, 1024>), grid, block, 0, s, a);          \
        }                                                                                                            \
        return launched();                                                                                           \
    }
    TT_DW_ROWS(1, 1) TT_DW_ROWS(2, 1) TT_DW_ROWS(4, 1) TT_DW_ROWS(1, 2) TT_DW_ROWS(2, 2) TT_DW_ROWS(4, 2)
#undef TT_DW_ROWS
    return TT_ERR_UNSUPPORTED;
}

} // namespace

int launch_dwconv(const DwArgs &a, const tt_plan &plan, void *stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid(plan.grid), block(plan.block);
    const int lds = plan.lds_bytes;
    // One stage, strides 1 or 2 and a tensor within the 2 GiB offset range: the register kernel.
    // Everything else (the LDS patch of two stages, other strides): the general kernel, one plane per lane.
    const bool rows_kernel = a.stages == 1 && a.stride_h == a.stride_w && (a.stride_h == 1 || a.stride_h == 2) &&
                             a.x_bytes != 0;
    if (!rows_kernel && a.eff_vec != 1) return TT_ERR_UNSUPPORTED;
#define TT_DW_CASE(WM_, WN_)                                                                                         \
    if (a.wave_m == WM_ && a.wave_n == WN_) {                                                                        \
        if (rows_kernel) return launch_dw_rows<WM_, WN_>(a, grid, block, s);                                         \
        constexpr int LIMIT = dw_block_limit(WM_, WN_, 1, 1, false);                                                 \
        if ((int)block.x > LIMIT) return TT_ERR_UNSUPPORTED;                                                         \
        const int bc = block.x <= 256 ? 0 : block.x <= 512 ? 1 : 2;                                                  \
        auto kern = dwconv3x3_kernel<WM_, WN_, 256>;                                                                 \
        if constexpr (LIMIT >= 512)                                                                                  \
            if (bc == 1) kern = dwconv3x3_kernel<WM_, WN_, 512>;                                                     \
        if constexpr (LIMIT >= 1024)                                                                                 \
            if (bc == 2) kern = dwconv3x3_kernel<WM_, WN_, 1024>;                                                    \
        static DynamicLdsLimit limits[3]; /* per kernel instance; host threads may launch concurrently */           \
        if (const int rc = limits[bc].raise_to(reinterpret_cast<const void *>(kern), lds); rc != TT_OK) return rc;   \
        hipLaunchKernelGGL(kern, grid, block, lds, s, a);                                                            \
        return launched();                                                                                           \
    }
    TT_DW_CASE(1, 1) TT_DW_CASE(1, 2) TT_DW_CASE(1, 4) TT_DW_CASE(1, 7)
    TT_DW_CASE(2, 1) TT_DW_CASE(2, 2) TT_DW_CASE(2, 4) TT_DW_CASE(2, 7)
    TT_DW_CASE(4, 1) TT_DW_CASE(4, 2) TT_DW_CASE(4, 4) TT_DW_CASE(4, 7)
    TT_DW_CASE(7, 1) TT_DW_CASE(7, 2) TT_DW_CASE(7, 4) TT_DW_CASE(7, 7)
#undef TT_DW_CASE
    return TT_ERR_UNSUPPORTED;
}

int launch_dw_direct(const DwArgs &a, int grid, void *stream)
{
    hipLaunchKernelGGL(dw_direct_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream), a);
    return launched();
}

int launch_tile_map_dump(const TileMap &map, int32_t *out_dev, void *stream)
{
    const int grid = (map.grid + 255) / 256;
    hipLaunchKernelGGL(tile_map_dump_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream), map, out_dev);
    return launched();
}

} // namespace tt
