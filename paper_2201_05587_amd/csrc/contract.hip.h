// Matrix-core contraction kernel for gfx950: conv2d as implicit GEMM, dense and
// batch matmul, with the fused epilogue (bias, residual, activation, down-convert).
//
// One workgroup owns a tile_m x tile_n output tile (and one split of K); its
// waves own wave_m x wave_n sub-tiles made of MF x MF matrix-core blocks.
// The K loop stages tile_k-wide slices of both operands through LDS, rows
// K-contiguous and padded by 16 bytes, so every lane fetches its operand
// fragment with one 16-byte LDS read.  Global loads of slice t+1 are issued
// before the matrix work of slice t (register prefetch); with two LDS stages one
// barrier per slice is enough.
//
// The order of K inside a 16-byte fragment fetch is permuted (lane group g
// takes elements [g*CH, g*CH+CH) of each K granule); both operands use the same
// permutation, so the sum is unchanged.
//
// Matrix-core rows are mapped to the axis that is NOT contiguous in the output
// and columns to the contiguous one, so the 32 (16) lanes of a block row write
// neighbouring addresses: conv (NCHW) -> rows = output channels, columns =
// pixels; dense / batch matmul (row-major [M][N]) -> rows = M, columns = N.
#pragma once

#include <hip/hip_runtime.h>

#include "tt_internal.h"

namespace tt {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

template <int DT> struct ElemOf;
template <> struct ElemOf<TT_F32> {
    using type = float;
    static constexpr int CH = 4; // elements per 16 bytes
};
template <> struct ElemOf<TT_BF16> {
    using type = uint16_t;
    static constexpr int CH = 8;
};

__device__ __forceinline__ float bf16_bits_to_float(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// float -> bf16, round to nearest, ties to even; NaN stays a quiet NaN.
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <int DT> __device__ __forceinline__ float load_as_float(const void *p, int64_t i)
{
    if constexpr (DT == TT_F32)
        return static_cast<const float *>(p)[i];
    else
        return bf16_bits_to_float(static_cast<const uint16_t *>(p)[i]);
}

template <int DT> __device__ __forceinline__ void store_from_float(void *p, int64_t i, float v)
{
    if constexpr (DT == TT_F32)
        static_cast<float *>(p)[i] = v;
    else
        static_cast<uint16_t *>(p)[i] = float_to_bf16_bits(v);
}

__device__ __forceinline__ float apply_act(float v, int act)
{
    switch (act) {
    case ACT_RELU: return fmaxf(v, 0.0f);
    case ACT_RELU6: return fminf(fmaxf(v, 0.0f), 6.0f);
    case ACT_GELU: return 0.5f * v * (1.0f + erff(v * 0.70710678118654752f));
    default: return v;
    }
}

// One matrix-core step on a 16-byte fragment per operand.
template <int DT, int MF> struct Mma;
template <> struct Mma<TT_BF16, 32> {
    using Acc = f32x16;
    static __device__ __forceinline__ void run(Acc &c, const u32x4 &a, const u32x4 &b)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                    0, 0);
    }
};
template <> struct Mma<TT_BF16, 16> {
    using Acc = f32x4;
    static __device__ __forceinline__ void run(Acc &c, const u32x4 &a, const u32x4 &b)
    {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                    0, 0);
    }
};
template <> struct Mma<TT_F32, 32> {
    using Acc = f32x16;
    static __device__ __forceinline__ void run(Acc &c, const u32x4 &a, const u32x4 &b)
    {
#pragma unroll
        for (int t = 0; t < 4; ++t)
            c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[t]), __uint_as_float(b[t]), c, 0, 0, 0);
    }
};
template <> struct Mma<TT_F32, 16> {
    using Acc = f32x4;
    static __device__ __forceinline__ void run(Acc &c, const u32x4 &a, const u32x4 &b)
    {
#pragma unroll
        for (int t = 0; t < 4; ++t)
            c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a[t]), __uint_as_float(b[t]), c, 0, 0, 0);
    }
};

// ---- global -> register loaders ---------------------------------------------------------------------------------

// Rows of a K-contiguous matrix [rows_total][ld]: each thread fetches 16-byte chunks along K.
template <int DT, int ROWS, int TK, int THREADS> struct RowKLoader {
    using E = typename ElemOf<DT>::type;
    static constexpr int CH = ElemOf<DT>::CH, CPR = TK / CH, TOTAL = ROWS * CPR;
    static constexpr int NL = (TOTAL + THREADS - 1) / THREADS;
    static constexpr int ROWB = (TK + CH) * (int)sizeof(E);

    static __device__ __forceinline__ void load(u32x4 (&regs)[NL], const E *base, int64_t ld, int row0, int rows_total,
                                                int k0, int k_end, int ev, int tid)
    {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int c = tid + i * THREADS;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (TOTAL % THREADS == 0 || c < TOTAL) {
                const int r = c / CPR, kc = c % CPR;
                const int gr = row0 + r, gk = k0 + kc * CH;
                if (gr < rows_total && gk < k_end) {
                    const E *p = base + (int64_t)gr * ld + gk;
                    if (ev == CH && gk + CH <= k_end) {
                        v = *reinterpret_cast<const u32x4 *>(p);
                    } else if (ev * (int)sizeof(E) == 8) {
#pragma unroll
                        for (int h = 0; h < 2; ++h)
                            if (gk + (h + 1) * (CH / 2) <= k_end) {
                                const uint2 t = *reinterpret_cast<const uint2 *>(p + h * (CH / 2));
                                v[2 * h] = t.x;
                                v[2 * h + 1] = t.y;
                            }
                    } else if (ev * (int)sizeof(E) == 4) {
#pragma unroll
                        for (int h = 0; h < 4; ++h)
                            if (gk + (h + 1) * (CH / 4) <= k_end)
                                v[h] = *reinterpret_cast<const uint32_t *>(p + h * (CH / 4));
                    } else {
                        // element-wise (bf16 with odd K)
#pragma unroll
                        for (int j = 0; j < CH; ++j)
                            if (gk + j < k_end) {
                                if constexpr (DT == TT_F32)
                                    v[j] = __float_as_uint(p[j]);
                                else
                                    v[j / 2] |= (uint32_t)p[j] << (16 * (j & 1));
                            }
                    }
                }
            }
            regs[i] = v;
        }
    }

    static __device__ __forceinline__ void store(const u32x4 (&regs)[NL], unsigned char *lds, int tid)
    {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int c = tid + i * THREADS;
            if (TOTAL % THREADS == 0 || c < TOTAL) {
                const int r = c / CPR, kc = c % CPR;
                *reinterpret_cast<u32x4 *>(lds + r * ROWB + kc * 16) = regs[i];
            }
        }
    }
};

// Rows whose elements along K are NOT contiguous in memory: the implicit-GEMM view of NCHW
// activations (K = (c, r, s)) and the [K][N] operand of a non-transposed batch matmul.  Lanes
// take neighbouring rows (contiguous in memory), each thread assembles CH consecutive K of its row.
template <int DT, int FAM, int ROWS, int TK, int THREADS> struct GatherLoader {
    using E = typename ElemOf<DT>::type;
    static constexpr int CH = ElemOf<DT>::CH, CPR = TK / CH, TOTAL = ROWS * CPR;
    static constexpr int NL = (TOTAL + THREADS - 1) / THREADS;
    static constexpr int NR = ROWS > THREADS ? ROWS / THREADS : 1; // distinct rows a thread serves
    static constexpr int ROWB = (TK + CH) * (int)sizeof(E);

    struct Row {
        int64_t base; // element offset of the row's image (conv) / the row index itself (NN)
        int ih0, iw0;
        bool valid;
    };

    static __device__ __forceinline__ int row_of(int slot, int tid)
    {
        return ROWS > THREADS ? tid + slot * THREADS : tid % ROWS;
    }

    static __device__ __forceinline__ void init(Row (&rows)[NR], const ContractArgs &g, int row0, int tid)
    {
#pragma unroll
        for (int s = 0; s < NR; ++s) {
            const int gr = row0 + row_of(s, tid);
            Row r;
            if constexpr (FAM == FAM_CONV) {
                r.valid = gr < g.M;
                const int hw = g.Ho * g.Wo;
                const int img = gr / hw, pix = gr - img * hw;
                const int p = pix / g.Wo, q = pix - p * g.Wo;
                r.ih0 = p * g.stride_h - g.pad_h;
                r.iw0 = q * g.stride_w - g.pad_w;
                r.base = (int64_t)img * g.C * g.H * g.W;
            } else {
                r.valid = gr < g.N;
                r.base = gr;
                r.ih0 = r.iw0 = 0;
            }
            rows[s] = r;
        }
    }

    static __device__ __forceinline__ void load(u32x4 (&regs)[NL], const Row (&rows)[NR], const E *base,
                                                const ContractArgs &g, int k0, int k_end, int tid)
    {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int c = tid + i * THREADS;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (TOTAL % THREADS == 0 || c < TOTAL) {
                const int slot = ROWS > THREADS ? i % NR : 0;
                const int kc = ROWS > THREADS ? i / NR : tid / ROWS + i * (THREADS / ROWS);
                const Row &r = rows[slot];
                const int k = k0 + kc * CH;
                if (r.valid && k < k_end) {
                    if constexpr (FAM == FAM_CONV) {
                        const int rs = g.R * g.S;
                        int cin = k / rs;
                        const int rem = k - cin * rs;
                        int fr = rem / g.S, fs = rem - fr * g.S;
#pragma unroll
                        for (int j = 0; j < CH; ++j) {
                            const int ih = r.ih0 + fr, iw = r.iw0 + fs;
                            if (k + j < k_end && ih >= 0 && ih < g.H && iw >= 0 && iw < g.W) {
                                const E e = base[r.base + ((int64_t)cin * g.H + ih) * g.W + iw];
                                if constexpr (DT == TT_F32)
                                    v[j] = __float_as_uint(e);
                                else
                                    v[j / 2] |= (uint32_t)e << (16 * (j & 1));
                            }
                            if (++fs == g.S) {
                                fs = 0;
                                if (++fr == g.R) {
                                    fr = 0;
                                    ++cin;
                                }
                            }
                        }
                    } else {
#pragma unroll
                        for (int j = 0; j < CH; ++j)
                            if (k + j < k_end) {
                                const E e = base[(int64_t)(k + j) * g.N + r.base];
                                if constexpr (DT == TT_F32)
                                    v[j] = __float_as_uint(e);
                                else
                                    v[j / 2] |= (uint32_t)e << (16 * (j & 1));
                            }
                    }
                }
            }
            regs[i] = v;
        }
    }

    static __device__ __forceinline__ void store(const u32x4 (&regs)[NL], unsigned char *lds, int tid)
    {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int c = tid + i * THREADS;
            if (TOTAL % THREADS == 0 || c < TOTAL) {
                const int slot = ROWS > THREADS ? i % NR : 0;
                const int kc = ROWS > THREADS ? i / NR : tid / ROWS + i * (THREADS / ROWS);
                *reinterpret_cast<u32x4 *>(lds + row_of(slot, tid) * ROWB + kc * 16) = regs[i];
            }
        }
    }
};

template <int DT, int FAM, int TM, int TN, int TK, int WM, int WN, int MF>
__global__ void __launch_bounds__((TM / WM) * (TN / WN) * 64) contract_kernel(const ContractArgs g)
{
    using E = typename ElemOf<DT>::type;
    constexpr int CH = ElemOf<DT>::CH, ES = (int)sizeof(E);
    constexpr int THREADS = (TM / WM) * (TN / WN) * 64;
    constexpr int ROWB = (TK + CH) * ES;
    constexpr int A_BYTES = TM * ROWB, B_BYTES = TN * ROWB, STAGE_BYTES = A_BYTES + B_BYTES;
    constexpr bool SWAP = FAM == FAM_CONV; // matrix-core rows = N side
    constexpr int WR = SWAP ? WN : WM, WC = SWAP ? WM : WN;
    constexpr int NWR = SWAP ? TN / WN : TM / WM; // waves along the matrix-core row axis
    constexpr int NI = WR / MF, NJ = WC / MF;
    constexpr int LG = 64 / MF, KS = CH * LG, NKS = TK / KS;
    constexpr int ACC = MF * MF / 64;
    static_assert(TK % KS == 0, "tile_k must be a multiple of the K granule");
    using M = Mma<DT, MF>;
    using ALoad = RowKLoader<DT, TM, TK, THREADS>;
    using AGather = GatherLoader<DT, FAM_CONV, TM, TK, THREADS>;
    using BLoad = RowKLoader<DT, TN, TK, THREADS>;
    using BGather = GatherLoader<DT, FAM_GEMM_NN, TN, TK, THREADS>;
    constexpr int NLA = FAM == FAM_CONV ? AGather::NL : ALoad::NL;
    constexpr int NLB = FAM == FAM_GEMM_NN ? BGather::NL : BLoad::NL;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const TileCoord tc = decode_tile(g.map, (int32_t)blockIdx.x);
    const int k_end = tc.k0 + tc.k_ext;
    const int kt_count = (tc.k_ext + TK - 1) / TK;
    const int bidx = tc.hi;

    const E *a_base = static_cast<const E *>(g.a);
    const E *b_base = static_cast<const E *>(g.b);
    if constexpr (FAM != FAM_CONV) {
        a_base += (int64_t)bidx * g.M * g.K;
        b_base += (int64_t)bidx * g.N * g.K;
    }

    typename AGather::Row a_rows[AGather::NR];
    typename BGather::Row b_rows[BGather::NR];
    if constexpr (FAM == FAM_CONV) AGather::init(a_rows, g, tc.m0, tid);
    if constexpr (FAM == FAM_GEMM_NN) BGather::init(b_rows, g, tc.n0, tid);

    u32x4 ra[NLA], rb[NLB];
    auto fetch = [&](int kt) {
        const int k0 = tc.k0 + kt * TK;
        if constexpr (FAM == FAM_CONV)
            AGather::load(ra, a_rows, a_base, g, k0, k_end, tid);
        else
            ALoad::load(ra, a_base, g.K, tc.m0, g.M, k0, k_end, g.eff_vec_a, tid);
        if constexpr (FAM == FAM_GEMM_NN)
            BGather::load(rb, b_rows, b_base, g, k0, k_end, tid);
        else
            BLoad::load(rb, b_base, g.K, tc.n0, g.N, k0, k_end, g.eff_vec_b, tid);
    };
    auto stash = [&](int stage) {
        unsigned char *sa = smem + stage * STAGE_BYTES, *sb = sa + A_BYTES;
        if constexpr (FAM == FAM_CONV)
            AGather::store(ra, sa, tid);
        else
            ALoad::store(ra, sa, tid);
        if constexpr (FAM == FAM_GEMM_NN)
            BGather::store(rb, sb, tid);
        else
            BLoad::store(rb, sb, tid);
    };

    typename M::Acc acc[NI][NJ];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int v = 0; v < ACC; ++v) acc[i][j][v] = 0.0f;

    const int wr = wave % NWR, wc = wave / NWR;
    const int lane_r = lane % MF, lane_g = lane / MF;
    const int r_off = (wr * WR + lane_r) * ROWB + lane_g * 16;
    const int c_off = (wc * WC + lane_r) * ROWB + lane_g * 16;

    auto k_step = [&](const unsigned char *sr, const unsigned char *sc, int ks) {
        u32x4 rf[NI], cf[NJ];
#pragma unroll
        for (int i = 0; i < NI; ++i)
            rf[i] = *reinterpret_cast<const u32x4 *>(sr + r_off + i * MF * ROWB + ks * KS * ES);
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            cf[j] = *reinterpret_cast<const u32x4 *>(sc + c_off + j * MF * ROWB + ks * KS * ES);
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) M::run(acc[i][j], rf[i], cf[j]);
    };

    fetch(0);
    stash(0);
    __syncthreads();
    int cur = 0;
    const bool two_stage = g.stages == 2;
    const bool unrolled = g.unroll >= 2;
    for (int it = 0; it < kt_count; ++it) {
        const bool more = it + 1 < kt_count;
        if (more) fetch(it + 1);
        const unsigned char *sa = smem + cur * STAGE_BYTES, *sb = sa + A_BYTES;
        const unsigned char *sr = SWAP ? sb : sa, *sc = SWAP ? sa : sb;
        if (unrolled || NKS == 1) {
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) k_step(sr, sc, ks);
        } else {
#pragma unroll 1
            for (int ks = 0; ks < NKS; ++ks) k_step(sr, sc, ks);
        }
        if (more) {
            if (!two_stage) __syncthreads();
            stash(two_stage ? cur ^ 1 : 0);
        }
        __syncthreads();
        if (two_stage) cur ^= 1;
    }

    // ---- epilogue: bias, residual, activation, down-convert, store (or raw partial sums for split-K) ----
    const bool partial = g.map.eff_split_k > 1;
    const int64_t mn = (int64_t)g.M * g.N;
    float *ws = g.ws + ((int64_t)tc.lo * g.batch) * mn;
    const int hw = g.Ho * g.Wo;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int col = wc * WC + j * MF + lane_r;
        int64_t col_base; // output offset contributed by the contiguous-axis coordinate
        bool col_ok;
        int n_of_col = 0;
        if constexpr (SWAP) {
            const int m = tc.m0 + col;
            col_ok = m < g.M;
            const int img = m / hw, pix = m - img * hw;
            col_base = (int64_t)img * g.N * hw + pix;
        } else {
            n_of_col = tc.n0 + col;
            col_ok = n_of_col < g.N;
            col_base = (int64_t)bidx * mn + n_of_col;
        }
        float bias_c = 0.0f;
        if constexpr (!SWAP)
            if (g.has_bias && col_ok && !partial) bias_c = load_as_float<DT>(g.bias, n_of_col);
#pragma unroll
        for (int i = 0; i < NI; ++i) {
#pragma unroll
            for (int v = 0; v < ACC; ++v) {
                const int row_l = MF == 32 ? (v / 4) * 8 + lane_g * 4 + (v % 4) : lane_g * 4 + v;
                const int row = wr * WR + i * MF + row_l;
                int64_t idx;
                bool ok = col_ok;
                float bias_v = bias_c;
                if constexpr (SWAP) {
                    const int n = tc.n0 + row;
                    ok = ok && n < g.N;
                    idx = col_base + (int64_t)n * hw;
                    if (g.has_bias && ok && !partial) bias_v = load_as_float<DT>(g.bias, n);
                } else {
                    const int m = tc.m0 + row;
                    ok = ok && m < g.M;
                    idx = col_base + (int64_t)m * g.N;
                }
                if (!ok) continue;
                float val = acc[i][j][v];
                if (partial) {
                    ws[idx] = val;
                } else {
                    val += bias_v;
                    if (g.has_res) val += load_as_float<DT>(g.res, idx);
                    store_from_float<DT>(g.out, idx, apply_act(val, g.act));
                }
            }
        }
    }
}

template <int DT, int FAM, int TM, int TN, int TK, int WM, int WN, int MF>
int launch_contract(const ContractArgs &args, int grid, int lds_bytes, void *stream)
{
    auto kern = contract_kernel<DT, FAM, TM, TN, TK, WM, WN, MF>;
    static int raised = 0; // largest dynamic-LDS size this kernel has been enabled for
    if (lds_bytes > 48 * 1024 && lds_bytes > raised) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return note_hip_error((int)e, "hipFuncSetAttribute(MaxDynamicSharedMemorySize)");
        raised = lds_bytes;
    }
    constexpr int THREADS = (TM / WM) * (TN / WN) * 64;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(THREADS), lds_bytes, static_cast<hipStream_t>(stream), args);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : note_hip_error((int)e, "contract_kernel launch");
}

} // namespace tt
