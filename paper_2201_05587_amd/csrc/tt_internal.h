// Internal declarations shared by the host code and the HIP kernels of libtt.
#pragma once

#include <stdint.h>

#include "tt.h"

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define TT_HD __host__ __device__ __forceinline__
#else
#define TT_HD inline
#endif

namespace tt {

constexpr int kXcds = 8;           // accelerator complex dies; workgroups are dealt to them round-robin
constexpr int kGroupM = 8;         // band height of raster order 2
constexpr int kLdsBudget = 160 * 1024;

enum Act { ACT_NONE = 0, ACT_RELU = 1, ACT_RELU6 = 2, ACT_GELU = 3 };

// Exact n / d for 0 <= n < 2^31 and 1 <= d < 2^31 by one widening multiply:
// magic = ceil(2^(31+shift) / d) with shift = ceil(log2 d) fits 32 bits, and the
// error n * (magic * d - 2^(31+shift)) / (d * 2^(31+shift)) stays below 1/d.
struct FastDiv {
    uint32_t magic, shift;
};
inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    f.shift = 0;
    while ((1ull << f.shift) < d) ++f.shift;
    const uint64_t pw = 1ull << (31 + f.shift);
    f.magic = (uint32_t)((pw + d - 1) / d);
    return f;
}
TT_HD uint32_t fast_div(uint32_t n, const FastDiv &f) { return (uint32_t)((((uint64_t)n * f.magic) >> 31) >> f.shift); }

// What a workgroup needs to find its tile: the integer fields of the plan the index map reads.
struct TileMap {
    int32_t sketch, order, grid;
    int32_t tiles_m, tiles_n, tile_m, tile_n, tile_k;
    int32_t M, N, K;
    int32_t eff_split_k, k_iters, k_tiles;
    // reciprocals of the map's divisors (a workgroup's first instructions; integer division is emulated
    // on the GPU): tiles_m * tiles_n, tiles_m, tiles_n, kGroupM * tiles_n, eff_split_k
    FastDiv div_tiles, div_m, div_n, div_band, div_split;
};

struct TileCoord {
    int32_t hi, lo;        // (batch, k-split); depthwise: (plane tile, 0)
    int32_t m0, m_ext, n0, n_ext, k0, k_ext;
};

// Workgroup id -> tile.  One implementation for the host mirror (tt_plan_tile) and every kernel.
TT_HD TileCoord decode_tile(const TileMap &p, int32_t wg)
{
    int32_t L = wg;
    if (p.order >= 3) {
        // XCD x receives workgroups x, x + 8, ...: give it one contiguous run of logical ids.
        const int32_t per = p.grid / kXcds, rem = p.grid % kXcds;
        const int32_t x = wg % kXcds, j = wg / kXcds;
        L = x * per + (x < rem ? x : rem) + j;
    }
    const int32_t T = p.tiles_m * p.tiles_n;
    const int32_t slab = (int32_t)fast_div((uint32_t)L, p.div_tiles), t = L - slab * T;
    const int32_t base = p.order % 3;
    int32_t im, in;
    if (base == 0) {
        in = (int32_t)fast_div((uint32_t)t, p.div_m);
        im = t - in * p.tiles_m;
    } else if (base == 1) {
        im = (int32_t)fast_div((uint32_t)t, p.div_n);
        in = t - im * p.tiles_n;
    } else {
        const int32_t width = kGroupM * p.tiles_n;
        const int32_t band = (int32_t)fast_div((uint32_t)t, p.div_band);
        const int32_t first = band * kGroupM, at = t - band * width;
        const int32_t left = p.tiles_m - first;
        if (left >= kGroupM) {
            in = at / kGroupM;
            im = first + at % kGroupM;
        } else { // the last, lower band
            in = at / left;
            im = first + at % left;
        }
    }
    TileCoord c;
    c.m0 = im * p.tile_m;
    c.n0 = in * p.tile_n;
    c.m_ext = (p.M - c.m0) < p.tile_m ? (p.M - c.m0) : p.tile_m;
    c.n_ext = (p.N - c.n0) < p.tile_n ? (p.N - c.n0) : p.tile_n;
    if (p.sketch == TT_SK_DWCONV) {
        c.hi = slab;
        c.lo = 0;
        c.k0 = slab * p.tile_k;
        c.k_ext = (p.K - c.k0) < p.tile_k ? (p.K - c.k0) : p.tile_k;
    } else if (p.sketch == TT_SK_GEMV) {
        c.hi = slab;
        c.lo = 0;
        c.k0 = 0;
        c.k_ext = p.K;
    } else {
        c.hi = (int32_t)fast_div((uint32_t)slab, p.div_split);
        c.lo = slab - c.hi * p.eff_split_k;
        const int32_t kt0 = c.lo * p.k_iters;
        int32_t kt1 = kt0 + p.k_iters;
        if (kt1 > p.k_tiles) kt1 = p.k_tiles;
        c.k0 = kt0 * p.tile_k;
        const int32_t kend = kt1 * p.tile_k < p.K ? kt1 * p.tile_k : p.K;
        c.k_ext = kend - c.k0;
    }
    return c;
}

inline TileMap tile_map_of(const tt_plan &pl)
{
    TileMap m;
    m.sketch = pl.sketch;
    m.order = pl.order;
    m.grid = pl.grid;
    m.tiles_m = pl.tiles_m;
    m.tiles_n = pl.tiles_n;
    m.tile_m = pl.tile_m;
    m.tile_n = pl.tile_n;
    m.tile_k = pl.tile_k;
    m.M = pl.M;
    m.N = pl.N;
    m.K = pl.K;
    m.eff_split_k = pl.eff_split_k;
    m.k_iters = pl.k_iters;
    m.k_tiles = pl.k_tiles;
    const auto at_least_one = [](int32_t v) { return (uint32_t)(v > 0 ? v : 1); };
    m.div_tiles = make_fastdiv(at_least_one(pl.tiles_m * pl.tiles_n));
    m.div_m = make_fastdiv(at_least_one(pl.tiles_m));
    m.div_n = make_fastdiv(at_least_one(pl.tiles_n));
    m.div_band = make_fastdiv(at_least_one(kGroupM * pl.tiles_n));
    m.div_split = make_fastdiv(at_least_one(pl.eff_split_k));
    return m;
}

// Operand families of the matrix-core contraction kernel.
enum Family {
    FAM_CONV = 0,    // A = NHWC activations gathered as an implicit GEMM, B = KRSC filters ([N][K])
    FAM_GEMM_TN = 1, // A = [M][K], B = [N][K] (dense; batch matmul with trans_b = 1; unit-stride 1x1 conv)
    FAM_GEMM_NN = 2  // A = [M][K], B = [K][N] (batch matmul with trans_b = 0)
};

// Everything a contraction kernel (matrix-core, direct or split-K reduce) needs, passed by value.
struct ContractArgs {
    const void *a, *b, *bias, *res;
    void *out;
    float *ws;
    TileMap map;
    int32_t batch, M, N, K;
    // FAM_CONV: the extent of the reduction as the gathering loaders walk it, R * runp >= K (see below);
    // the split of the reduction that ends at K runs on to k_walk
    int32_t k_walk;
    // convolution geometry (FAM_CONV).  The reduction index is k = r * runp + j: filter row r and
    // position j inside the run of S * C elements that one filter row covers contiguously in an
    // NHWC image row (and in a KRSC filter); runp is the run rounded up to whole 16-byte items.
    int32_t C, H, W, R, S, stride_h, stride_w, pad_h, pad_w, Ho, Wo;
    int32_t run, runp;
    FastDiv div_hw, div_wo; // output pixel index -> (image, row, column)
    // padded image geometry of the patch kernel: PW = W + 2 pad_w, PHW = (H + 2 pad_h) * PW
    int32_t PW, PHW;
    FastDiv div_phw, div_pw; // flat padded pixel index -> (image, padded row, padded column)
    uint32_t a_bytes, b_bytes; // sizes of the activation and filter tensors (bounds of the gathering loads)
    int32_t eff_vec_a, eff_vec_b, eff_vec_c, stages, unroll, act, has_bias, has_res, dtype;
};

struct DwArgs {
    const float *x, *w, *bias;
    float *y;
    TileMap map;
    int32_t planes, C, H, W, Ho, Wo, stride_h, stride_w, pad_h, pad_w;
    int32_t wave_m, wave_n, stages, unroll;
    int32_t eff_vec;   // channel-contiguous planes per lane (1, 2 or 4)
    uint32_t x_bytes;  // size of the input tensor when it is below 2 GiB, else 0
};

struct Variant {
    int32_t dtype, family, tile_m, tile_n, tile_k, wave_m, wave_n, mfma;
    int32_t amode; // conv family: bytes per gathered load (16 or the element size); 0 otherwise
    int32_t pipe;  // 0: register-staged loads, 1 or 2 LDS stages; 1: asynchronous loads into a ring of 3 or 4;
                   // 2: 3x3 conv with the padded input patch in LDS and a filter ring of 3 or 4 (stages 5 or 6)
                   // 3: persistent dense kernel, the B panel resident in LDS and two A buffers (stages 7)
    int32_t stride; // pipe 2: the convolution stride the kernel is compiled for; 0 otherwise
    int (*launch)(const ContractArgs &args, int grid, int lds_bytes, void *stream);
    int (*stage_bytes)();        // pipes 0, 1: LDS bytes of one pipeline stage; pipe 2: pixels a patch buffer holds;
                                 // pipe 3: request instructions per lane and K slice
    int (*lds_bytes)(int stages); // LDS bytes for a plan's number of stages (pipe 3: for its number of K slices), as
                                  // the compiled kernel lays LDS out
};

// Reduction elements one 16-byte operand fragment per lane feeds to the matrix cores: a block of MF rows
// leaves 64 / MF lane groups along K, each holding 16 bytes.  tile_k must be a multiple of it.
constexpr int k_granule(int dtype, int mfma) { return (dtype == TT_F32 ? 4 : 8) * (64 / mfma); }

// variant table (generated) and lookups
extern const Variant kVariants[];
extern const int kNumVariants;
int find_variant(int dtype, int family, int tm, int tn, int tk, int wm, int wn, int mf, int amode, int pipe,
                 int stride = 0);
int family_of(int cls, int trans_b);

// launchers of the non-matrix-core kernels (simple_kernels.hip)
int launch_direct(const ContractArgs &args, int family, int grid, void *stream);
int launch_splitk_reduce(const ContractArgs &args, int family, void *stream);
int launch_gemv(const ContractArgs &args, const tt_plan &plan, void *stream);
int dw_max_block(int wave_m, int wave_n, int planes_per_lane, int stride, bool rows_kernel);
int launch_dwconv(const DwArgs &args, const tt_plan &plan, void *stream);
int launch_dw_direct(const DwArgs &args, int grid, void *stream);
int launch_tile_map_dump(const TileMap &map, int32_t *out_dev, void *stream);

// Remember the text of a failed HIP call for tt_last_error(); returns TT_ERR_HIP.
int note_hip_error(int hip_error_code, const char *where);

inline int act_of_class(int cls)
{
    switch (cls) {
    case TT_CONV2D_BIAS_RELU:
    case TT_CONV2D_BIAS_ADD_RELU:
    case TT_DENSE_BIAS_RELU:
        return ACT_RELU;
    case TT_CONV2D_BIAS_RELU6:
    case TT_DWCONV_BIAS_RELU6:
        return ACT_RELU6;
    case TT_DENSE_BIAS_GELU:
        return ACT_GELU;
    default:
        return ACT_NONE;
    }
}

inline bool is_conv_class(int cls) { return cls >= TT_CONV2D_ADD && cls <= TT_CONV2D_BIAS_RELU6; }
inline bool is_dense_class(int cls) { return cls >= TT_DENSE_ADD && cls <= TT_DENSE_BIAS_GELU; }

} // namespace tt
