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
//
// All loaders follow one rule: a fetch only ISSUES loads.  Every load is unconditional (an
// address that would fall outside the tensor is replaced by a safe one inside it) and lands in a
// register nothing reads until the slice is written to LDS, so the loads of slice t+1 stay in
// flight during the matrix work of slice t.  Zero padding, tails and edge repair are applied by
// the store step, which recomputes (or has kept) which parts of each 16-byte item are real.
// There is one straight-line code path per kernel: how the activations are fetched is a
// template parameter, not a run-time branch.

// Unconditional loads into registers (addresses need only element alignment).
__device__ __forceinline__ void load16(u32x4 &dst, const void *p) { __builtin_memcpy(&dst, p, 16); }
__device__ __forceinline__ void load4(u32x4 &v, int at, const void *p)
{
    uint32_t t;
    __builtin_memcpy(&t, p, 4);
    v[at] = t;
}

// Shift the 16-byte value by whole elements: positive = towards higher element indices; zero fill.
template <int DT> __device__ __forceinline__ u32x4 shift_elems(const u32x4 &v, int elems)
{
    constexpr int EB = DT == TT_F32 ? 32 : 16;
    unsigned __int128 x = ((unsigned __int128)v[3] << 96) | ((unsigned __int128)v[2] << 64) |
                          ((unsigned __int128)v[1] << 32) | (unsigned __int128)v[0];
    x = elems >= 0 ? (x << (EB * elems)) : (x >> (EB * -elems));
    u32x4 r = {(uint32_t)x, (uint32_t)(x >> 32), (uint32_t)(x >> 64), (uint32_t)(x >> 96)};
    return r;
}
__device__ __forceinline__ uint32_t shift32(uint32_t x, int bits) { return bits >= 0 ? x << bits : x >> -bits; }

// shift_elems for the repair of a vector that hung over a row edge: one element either way is the
// common case (3x3 filters with padding 1) and costs four byte-align operations; wider shifts take
// the general path.
template <int DT> __device__ __forceinline__ u32x4 shift_edge(const u32x4 &v, int elems)
{
    if constexpr (DT == TT_F32) {
        if (elems == 1) return u32x4{0u, v[0], v[1], v[2]};
        if (elems == -1) return u32x4{v[1], v[2], v[3], 0u};
    } else {
        if (elems == 1)
            return u32x4{v[0] << 16, __builtin_amdgcn_alignbyte(v[1], v[0], 2), __builtin_amdgcn_alignbyte(v[2], v[1], 2),
                         __builtin_amdgcn_alignbyte(v[3], v[2], 2)};
        if (elems == -1)
            return u32x4{__builtin_amdgcn_alignbyte(v[1], v[0], 2), __builtin_amdgcn_alignbyte(v[2], v[1], 2),
                         __builtin_amdgcn_alignbyte(v[3], v[2], 2), v[3] >> 16};
    }
    return shift_elems<DT>(v, elems);
}

// Zero the elements of a 16-byte item at positions >= keep (0 <= keep; keep >= CH keeps all).
template <int DT> __device__ __forceinline__ u32x4 keep_first(u32x4 v, int keep)
{
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        if constexpr (DT == TT_F32) {
            v[h] = h < keep ? v[h] : 0u;
        } else {
            const uint32_t lo = 2 * h < keep ? 0xffffu : 0u, hi = 2 * h + 1 < keep ? 0xffff0000u : 0u;
            v[h] &= lo | hi;
        }
    }
    return v;
}

// Rows of a K-contiguous matrix [rows_total][K], K >= CH: each thread fetches 16-byte chunks along
// K.  A chunk that would run past the end of its row is read CH elements back from the row end
// and shifted down afterwards, so the access never leaves the matrix.
template <int DT, int ROWS, int TK, int THREADS> struct RowKLoader {
    using E = typename ElemOf<DT>::type;
    static constexpr int CH = ElemOf<DT>::CH, CPR = TK / CH, TOTAL = ROWS * CPR;
    static constexpr int NL = (TOTAL + THREADS - 1) / THREADS;
    static constexpr int ROWB = (TK + CH) * (int)sizeof(E);
    struct State {
        u32x4 raw[NL];
    };

    static __device__ __forceinline__ void load(State &st, const E *base, int K, int row0, int rows_total, int k0,
                                                int tid)
    {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            int c = tid + i * THREADS;
            if (TOTAL % THREADS != 0) c = min(c, TOTAL - 1);
            const int r = c / CPR, kc = c % CPR;
            const int gr = min(row0 + r, rows_total - 1);
            const int gk = min(k0 + kc * CH, K - CH);
            load16(st.raw[i], base + (int64_t)gr * K + gk);
        }
    }

    static __device__ __forceinline__ void store(const State &st, unsigned char *lds, int K, int row0, int rows_total,
                                                 int k0, int k_end, int tid)
    {
        // Whole tile inside the matrix and the slice inside the K range (the usual case, the same for
        // every thread of the workgroup): the registers go to LDS as they are.
        const bool interior = row0 + ROWS <= rows_total && k0 + TK <= k_end;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int c = tid + i * THREADS;
            if (TOTAL % THREADS != 0 && c >= TOTAL) continue;
            const int r = c / CPR, kc = c % CPR;
            u32x4 v = st.raw[i];
            if (!interior) {
                const int gk = k0 + kc * CH;
                const int back = gk - min(gk, K - CH); // how far the load was moved back
                if (back > 0 || gk + CH > k_end) v = keep_first<DT>(shift_elems<DT>(v, -back), k_end - gk);
                if (row0 + r >= rows_total) v = u32x4{0u, 0u, 0u, 0u};
            }
            *reinterpret_cast<u32x4 *>(lds + r * ROWB + kc * 16) = v;
        }
    }
};

// ---- K-major tiles: operands whose memory is contiguous along the OUTPUT axis, not along K -----------------------
//
// NCHW activations seen as the implicit-GEMM matrix (K = (c, r, s); consecutive output pixels of
// a row are consecutive input pixels) and the [K][N] operand of a non-transposed batch matmul.
// The tile is kept in LDS as T[k][x], x contiguous, so global vectors are copied as they are.
// Matrix-core fragments (8 consecutive K per lane for bf16) come out of the transposing LDS read
// of gfx950: within 16 lanes, lane i supplies the address of 4 consecutive x of K-row i/4 and
// receives the 4 K-rows of column i.  fp32 fragments are four 4-byte reads.

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// Padded row length (elements) of a K-major tile: keeps the fragment reads free of bank conflicts.
template <int DT, int ROWS, int MF> struct KMajorRow {
    static constexpr int PAD = DT == TT_BF16 ? (32 + 64 - ROWS % 64) % 64 : (MF == 32 ? 8 : 4);
    static constexpr int LEN = ROWS + PAD;
};

// Implicit-GEMM activation tile, K-major.  An item is one K-row times G = 16 bytes of consecutive
// output pixels, fetched as 16 / VB loads of VB bytes: the whole item when a row of output
// pixels is a multiple of G and the stride is 1 (VB = 16), pairs of bf16 pixels when rows are
// even (VB = 4), else single pixels (VB = element size).
//
// Address generation is kept off the critical path.  What depends only on the thread's pixels is
// computed once per workgroup: the element offset of filter tap (0, 0), one bit per filter row
// saying whether that row falls inside the image, and one 4-bit code per filter column saying
// whether the sub-vector is inside the row, outside, or hangs over its left or right end (then
// the load is moved back inside and the code is the element shift that repairs it).  What depends
// only on K - (channel, filter row, filter column) - advances by add-and-carry, never by division.
template <int DT, int TM, int TK, int THREADS, int LEN, int VB> struct ConvTileLoader {
    using E = typename ElemOf<DT>::type;
    static constexpr int ES = (int)sizeof(E);
    static constexpr int G = ElemOf<DT>::CH;              // pixels per item
    static constexpr int V = VB / ES;                      // pixels per load
    static constexpr int NS = 16 / VB;                     // loads per item
    static constexpr int MG = TM / G;                      // items per K-row
    static constexpr int KSTEP = THREADS / MG;             // K-rows between a thread's items
    static constexpr int NL = (TK + KSTEP - 1) / KSTEP;    // items per thread and slice
    static_assert(MG >= 1 && MG <= THREADS, "tile_m does not fit the workgroup");
    static_assert(VB == 16 || VB == 4 || VB == ES, "unsupported activation fetch width");

    struct Mixed { // a K index as (channel, filter row, filter column)
        int c, r, s;
    };
    struct State {
        int32_t off[NS];     // per sub-vector: element offset of tap (0, 0) of its first pixel
        uint32_t rows[NS];   // bit r: filter row r is inside the image
        uint32_t cols[NS];   // nibble s: 0 = outside, else 8 + element shift to apply after the load
        uint32_t raw[NL][VB == 2 ? 8 : 4];
        uint32_t fix[NL];    // nibble j: the code sub-vector j was loaded with
        Mixed kpos;          // decomposition of the first K-row this thread serves in the next slice
        Mixed step_item, step_tile;
    };

    static __device__ __forceinline__ Mixed decompose(int k, int R, int S)
    {
        Mixed m;
        m.c = k / (R * S);
        const int rem = k - m.c * R * S;
        m.r = rem / S;
        m.s = rem - m.r * S;
        return m;
    }
    static __device__ __forceinline__ Mixed advance(Mixed a, const Mixed &d, int R, int S)
    {
        a.s += d.s;
        const int cs = a.s >= S;
        a.s -= cs ? S : 0;
        a.r += d.r + cs;
        const int cr = a.r >= R;
        a.r -= cr ? R : 0;
        a.c += d.c + cr;
        return a;
    }

    static __device__ __forceinline__ void init(State &st, const ContractArgs &g, int m0, int k_first, int tid)
    {
        const int mg = tid % MG;
        const int hw = g.Ho * g.Wo;
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            st.off[j] = 0;
            st.rows[j] = 0u;
            st.cols[j] = 0u;
            const int m = m0 + mg * G + j * V;
            if (m >= g.M) continue;
            const int img = m / hw, pix = m - img * hw;
            const int p = pix / g.Wo, q = pix - p * g.Wo;
            const int ih0 = p * g.stride_h - g.pad_h, iw0 = q * g.stride_w - g.pad_w;
            st.off[j] = (img * g.C * g.H + ih0) * g.W + iw0;
            uint32_t rows = 0u, cols = 0u;
            for (int r = 0; r < g.R; ++r)
                if (ih0 + r >= 0 && ih0 + r < g.H) rows |= 1u << r;
            for (int s = 0; s < g.S; ++s) {
                const int iw = iw0 + s;
                if (iw > -V && iw < g.W) {
                    const int shift = iw < 0 ? -iw : (iw + V > g.W ? g.W - V - iw : 0);
                    cols |= (uint32_t)(shift + 8) << (4 * s);
                }
            }
            st.rows[j] = rows;
            st.cols[j] = cols;
        }
        st.kpos = decompose(k_first + tid / MG, g.R, g.S);
        st.step_item = decompose(KSTEP, g.R, g.S);
        st.step_tile = decompose(TK, g.R, g.S);
    }

    // Issue the loads of the slice whose first K index is k0 (slices must be fetched in order).
    static __device__ __forceinline__ void load(State &st, const E *x, const ContractArgs &g, int k0, int k_end, int tid)
    {
        const int kl0 = tid / MG;
        const int hw_in = g.H * g.W;
        Mixed kp = st.kpos;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int kl = kl0 + i * KSTEP;
            const uint32_t k_ok = (kl < TK) & (k0 + kl < k_end);
            const int koff = kp.c * hw_in + kp.r * g.W + kp.s;
            uint32_t fix = 0u;
#pragma unroll
            for (int j = 0; j < NS; ++j) {
                const uint32_t present = k_ok & (st.rows[j] >> kp.r) & 1u;
                const uint32_t code = present ? (st.cols[j] >> (4 * kp.s)) & 15u : 0u;
                // nothing to read: point at the start of the tensor, which is always readable
                const int idx = code ? st.off[j] + koff + (int)code - 8 : 0;
                fix |= code << (4 * j);
                const E *p = x + idx;
                if constexpr (VB == 16) {
                    u32x4 t;
                    load16(t, p);
                    st.raw[i][0] = t[0];
                    st.raw[i][1] = t[1];
                    st.raw[i][2] = t[2];
                    st.raw[i][3] = t[3];
                } else if constexpr (VB == 4) {
                    uint32_t t;
                    __builtin_memcpy(&t, p, 4);
                    st.raw[i][j] = t;
                } else {
                    st.raw[i][j] = *reinterpret_cast<const uint16_t *>(p);
                }
            }
            st.fix[i] = fix;
            kp = advance(kp, st.step_item, g.R, g.S);
        }
        st.kpos = advance(st.kpos, st.step_tile, g.R, g.S);
    }

    static __device__ __forceinline__ void store(const State &st, unsigned char *lds, int tid)
    {
        const int mg = tid % MG, kl0 = tid / MG;
        constexpr int EB = 8 * ES;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int kl = kl0 + i * KSTEP;
            if (KSTEP * NL > TK && kl >= TK) continue;
            u32x4 v;
            const uint32_t fix = st.fix[i];
            if constexpr (VB == 16) {
                const int code = (int)(fix & 15u);
                v = u32x4{st.raw[i][0], st.raw[i][1], st.raw[i][2], st.raw[i][3]};
                if (code == 0) v = u32x4{0u, 0u, 0u, 0u};
                if (code != 0 && code != 8) v = shift_edge<DT>(v, code - 8); // only lanes at a row edge
            } else if constexpr (VB == 4) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int code = (int)((fix >> (4 * j)) & 15u);
                    // fp32: a single element, present or not; bf16: a pair that may need a one-element shift
                    if constexpr (DT == TT_F32)
                        v[j] = code != 0 ? st.raw[i][j] : 0u;
                    else
                        v[j] = code != 0 ? shift32(st.raw[i][j], EB * (code - 8)) : 0u;
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t lo = ((fix >> (8 * j)) & 15u) != 0u ? (st.raw[i][2 * j] & 0xffffu) : 0u;
                    const uint32_t hi = ((fix >> (8 * j + 4)) & 15u) != 0u ? (st.raw[i][2 * j + 1] << 16) : 0u;
                    v[j] = lo | hi;
                }
            }
            *reinterpret_cast<u32x4 *>(lds + ((size_t)kl * LEN + mg * G) * sizeof(E)) = v;
        }
    }
};

// [K][N] operand of a non-transposed batch matmul (N >= G): rows of the matrix are rows of the
// K-major tile.  A 16-byte item that would run past the end of its row is read G elements back
// from the row end and shifted down afterwards.
template <int DT, int TN, int TK, int THREADS, int LEN> struct KRowTileLoader {
    using E = typename ElemOf<DT>::type;
    static constexpr int G = ElemOf<DT>::CH, NG = TN / G;
    static constexpr int KSTEP = THREADS / NG;
    static constexpr int NL = (TK + KSTEP - 1) / KSTEP;
    static_assert(NG >= 1 && NG <= THREADS, "tile_n does not fit the workgroup");
    struct State {
        u32x4 raw[NL];
    };

    static __device__ __forceinline__ void load(State &st, const E *b, int N, int K, int n0, int k0, int tid)
    {
        const int ng = tid % NG, kl0 = tid / NG;
        const int n = min(n0 + ng * G, N - G);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int k = min(k0 + kl0 + i * KSTEP, K - 1);
            load16(st.raw[i], b + (int64_t)k * N + n);
        }
    }

    static __device__ __forceinline__ void store(const State &st, unsigned char *lds, int N, int n0, int k0, int k_end,
                                                 int tid)
    {
        const int ng = tid % NG, kl0 = tid / NG;
        const int n = n0 + ng * G;
        const bool interior = n0 + TN <= N && k0 + TK <= k_end; // same for every thread of the workgroup
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int kl = kl0 + i * KSTEP;
            if (KSTEP * NL > TK && kl >= TK) continue;
            u32x4 v = st.raw[i];
            if (!interior) {
                const int back = n - min(n, N - G);
                if (back > 0) v = keep_first<DT>(shift_elems<DT>(v, -back), N - n);
                if (k0 + kl >= k_end || n >= N) v = u32x4{0u, 0u, 0u, 0u};
            }
            *reinterpret_cast<u32x4 *>(lds + ((size_t)kl * LEN + ng * G) * sizeof(E)) = v;
        }
    }
};

// Fragment of a K-major tile for lane (column x = x_base + lane % MF, K group = lane / MF) at K offset kk.
template <int DT, int MF, int LEN> __device__ __forceinline__ u32x4 kmajor_fragment(const unsigned char *tile, int x_base,
                                                                                     int kk, int lane)
{
    if constexpr (DT == TT_BF16) {
        const int i = lane & 15, xblk = (lane % MF) / 16, kg = lane / MF;
        const int row = kk + kg * 8 + (i >> 2), col = x_base + xblk * 16 + 4 * (i & 3);
        const unsigned char *p = tile + ((size_t)row * LEN + col) * 2;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)p);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + (size_t)4 * LEN * 2));
        const uint2 l = __builtin_bit_cast(uint2, lo), h = __builtin_bit_cast(uint2, hi);
        return u32x4{l.x, l.y, h.x, h.y};
    } else {
        const int x = x_base + lane % MF, kg = lane / MF;
        const float *p = reinterpret_cast<const float *>(tile) + (size_t)(kk + kg * 4) * LEN + x;
        return u32x4{__float_as_uint(p[0]), __float_as_uint(p[LEN]), __float_as_uint(p[2 * LEN]),
                     __float_as_uint(p[3 * LEN])};
    }
}

// LDS bytes of one pipeline stage: the A tile followed by the B tile.
template <int DT, int FAM, int TM, int TN, int TK, int MF> struct StageLayout {
    using E = typename ElemOf<DT>::type;
    static constexpr int CH = ElemOf<DT>::CH, ES = (int)sizeof(E);
    static constexpr int ROWB = (TK + CH) * ES; // row of a K-contiguous tile, padded by 16 bytes
    static constexpr int LEN_A = KMajorRow<DT, TM, MF>::LEN, LEN_B = KMajorRow<DT, TN, MF>::LEN;
    static constexpr int A_BYTES = FAM == FAM_CONV ? TK * LEN_A * ES : TM * ROWB;
    static constexpr int B_BYTES = FAM == FAM_GEMM_NN ? TK * LEN_B * ES : TN * ROWB;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
};

// AM = bytes per activation load of the conv family (16, 4 or the element size); 0 for the others.
template <int DT, int FAM, int TM, int TN, int TK, int WM, int WN, int MF, int AM>
__global__ void __launch_bounds__((TM / WM) * (TN / WN) * 64) contract_kernel(const ContractArgs g)
{
    using E = typename ElemOf<DT>::type;
    using L = StageLayout<DT, FAM, TM, TN, TK, MF>;
    constexpr int CH = ElemOf<DT>::CH, ES = (int)sizeof(E);
    constexpr int THREADS = (TM / WM) * (TN / WN) * 64;
    constexpr int ROWB = L::ROWB, A_BYTES = L::A_BYTES, STAGE_BYTES = L::STAGE_BYTES;
    constexpr bool SWAP = FAM == FAM_CONV; // matrix-core rows = N side, columns = M side
    constexpr int WR = SWAP ? WN : WM, WC = SWAP ? WM : WN;
    constexpr int NWR = SWAP ? TN / WN : TM / WM; // waves along the matrix-core row axis
    constexpr int NI = WR / MF, NJ = WC / MF;
    constexpr int LG = 64 / MF, KS = CH * LG, NKS = TK / KS;
    constexpr int ACC = MF * MF / 64;
    constexpr bool C_KMAJOR = FAM != FAM_GEMM_TN;     // the column-side tile is K-major
    constexpr int LEN_C = SWAP ? L::LEN_A : L::LEN_B; // its padded row length
    static_assert(TK % KS == 0, "tile_k must be a multiple of the K granule");
    using M = Mma<DT, MF>;
    using ALoad = RowKLoader<DT, TM, TK, THREADS>;
    using AConv = ConvTileLoader<DT, TM, TK, THREADS, L::LEN_A, FAM == FAM_CONV ? AM : 16>;
    using BLoad = RowKLoader<DT, TN, TK, THREADS>;
    using BKRow = KRowTileLoader<DT, TN, TK, THREADS, L::LEN_B>;

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

    // registers holding the slice in flight (only the members of the family in use are live)
    typename AConv::State a_conv;
    typename BKRow::State b_krow;
    typename ALoad::State a_rows;
    typename BLoad::State b_rows;
    if constexpr (FAM == FAM_CONV) AConv::init(a_conv, g, tc.m0, tc.k0, tid);

    auto fetch = [&](int kt) {
        const int k0 = tc.k0 + kt * TK;
        if constexpr (FAM == FAM_CONV)
            AConv::load(a_conv, a_base, g, k0, k_end, tid);
        else
            ALoad::load(a_rows, a_base, g.K, tc.m0, g.M, k0, tid);
        if constexpr (FAM == FAM_GEMM_NN)
            BKRow::load(b_krow, b_base, g.N, g.K, tc.n0, k0, tid);
        else
            BLoad::load(b_rows, b_base, g.K, tc.n0, g.N, k0, tid);
    };
    auto stash = [&](int stage, int kt) {
        const int k0 = tc.k0 + kt * TK;
        unsigned char *sa = smem + stage * STAGE_BYTES, *sb = sa + A_BYTES;
        if constexpr (FAM == FAM_CONV)
            AConv::store(a_conv, sa, tid);
        else
            ALoad::store(a_rows, sa, g.K, tc.m0, g.M, k0, k_end, tid);
        if constexpr (FAM == FAM_GEMM_NN)
            BKRow::store(b_krow, sb, g.N, tc.n0, k0, k_end, tid);
        else
            BLoad::store(b_rows, sb, g.K, tc.n0, g.N, k0, k_end, tid);
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
        for (int j = 0; j < NJ; ++j) {
            if constexpr (C_KMAJOR)
                cf[j] = kmajor_fragment<DT, MF, LEN_C>(sc, wc * WC + j * MF, ks * KS, lane);
            else
                cf[j] = *reinterpret_cast<const u32x4 *>(sc + c_off + j * MF * ROWB + ks * KS * ES);
        }
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) M::run(acc[i][j], rf[i], cf[j]);
    };

    fetch(0);
    stash(0, 0);
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
            stash(two_stage ? cur ^ 1 : 0, it + 1);
        }
        __syncthreads();
        if (two_stage) cur ^= 1;
    }

    // ---- epilogue ------------------------------------------------------------------------------------------
    // The accumulators hold, per lane, 4 consecutive ROWS of one column, while memory is contiguous
    // along COLUMNS.  Each wave therefore passes its tile through a private LDS region, one band of
    // MF rows at a time, and reads it back so that a lane owns 8 consecutive columns of one row:
    // bias, residual, activation and down-conversion then work on 16-byte vectors (or on the widest
    // sub-vectors the output's row length allows), and stores are fully coalesced.  With split-K
    // the raw partial sums go to the workspace in the same pattern.
    {
        constexpr int ESTRIDE = WC + (MF == 32 ? 8 : 4);      // floats per staged row (bank-conflict padding)
        constexpr int CG = WC / 8;                            // 8-column groups per row
        constexpr int ROWS_PER_PASS = 64 / CG;                // rows the 64 lanes cover at once
        constexpr int PASSES = (MF + ROWS_PER_PASS - 1) / ROWS_PER_PASS;
        float *stage = reinterpret_cast<float *>(smem) + wave * (MF * ESTRIDE);
        const bool partial = g.map.eff_split_k > 1;
        const int64_t mn = (int64_t)g.M * g.N;
        float *ws = g.ws + ((int64_t)tc.lo * g.batch) * mn;
        const int hw = g.Ho * g.Wo;
        int vc = g.eff_vec_c; // consecutive outputs that are contiguous in memory and all inside or all outside
        const int cg = lane % CG, row_in_pass = lane / CG;
        const int c0 = wc * WC + cg * 8; // first of this lane's 8 columns inside the workgroup tile

#pragma unroll
        for (int i = 0; i < NI; ++i) {
            __syncthreads(); // the band before this one has been read (and the K loop is over)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int v = 0; v < ACC; ++v) {
                    const int row_l = MF == 32 ? (v / 4) * 8 + lane_g * 4 + (v % 4) : lane_g * 4 + v;
                    stage[row_l * ESTRIDE + j * MF + lane_r] = acc[i][j][v];
                }
            __syncthreads();
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps) {
                const int row_l = ps * ROWS_PER_PASS + row_in_pass;
                if (ROWS_PER_PASS * PASSES > MF && row_l >= MF) continue;
                const f32x4 lo = *reinterpret_cast<const f32x4 *>(stage + row_l * ESTRIDE + cg * 8);
                const f32x4 hi = *reinterpret_cast<const f32x4 *>(stage + row_l * ESTRIDE + cg * 8 + 4);
                float val[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                const int row = wr * WR + i * MF + row_l;
                // coordinates: SWAP (conv): row -> output channel n, columns -> pixels m; else row -> m, columns -> n
                const int fixed = (SWAP ? tc.n0 : tc.m0) + row;
                if (fixed >= (SWAP ? g.N : g.M)) continue;
                const int first = (SWAP ? tc.m0 : tc.n0) + c0;
                const int limit = SWAP ? g.M : g.N;
                const float bias_row = (SWAP && g.has_bias && !partial) ? load_as_float<DT>(g.bias, fixed) : 0.0f;
                // groups of vc consecutive columns
                for (int e0 = 0; e0 < 8; e0 += vc) {
                    const int colg = first + e0;
                    if (colg >= limit) break;
                    int64_t idx;
                    if constexpr (SWAP) {
                        const int img = colg / hw, pix = colg - img * hw;
                        idx = ((int64_t)img * g.N + fixed) * hw + pix;
                    } else {
                        idx = (int64_t)bidx * mn + (int64_t)fixed * g.N + colg;
                    }
                    if (partial) {
                        if (vc == 8) {
                            *reinterpret_cast<f32x4 *>(ws + idx) = lo;
                            *reinterpret_cast<f32x4 *>(ws + idx + 4) = hi;
                        } else if (vc == 4) {
                            *reinterpret_cast<f32x4 *>(ws + idx) = e0 == 0 ? lo : hi;
                        } else {
                            for (int e = 0; e < vc; ++e) ws[idx + e] = val[e0 + e];
                        }
                        continue;
                    }
                    if (vc == 8 && DT == TT_BF16) {
                        u32x4 resv = {0u, 0u, 0u, 0u}, biasv = {0u, 0u, 0u, 0u};
                        if (g.has_res) resv = *reinterpret_cast<const u32x4 *>(static_cast<const uint16_t *>(g.res) + idx);
                        if (!SWAP && g.has_bias)
                            biasv = *reinterpret_cast<const u32x4 *>(static_cast<const uint16_t *>(g.bias) + colg);
                        u32x4 outv;
#pragma unroll
                        for (int h = 0; h < 4; ++h) {
                            float a = val[2 * h] + bias_row + __uint_as_float(biasv[h] << 16) +
                                      __uint_as_float(resv[h] << 16);
                            float b = val[2 * h + 1] + bias_row + __uint_as_float(biasv[h] & 0xffff0000u) +
                                      __uint_as_float(resv[h] & 0xffff0000u);
                            outv[h] = (uint32_t)float_to_bf16_bits(apply_act(a, g.act)) |
                                      ((uint32_t)float_to_bf16_bits(apply_act(b, g.act)) << 16);
                        }
                        *reinterpret_cast<u32x4 *>(static_cast<uint16_t *>(g.out) + idx) = outv;
                    } else if (vc >= 4 && DT == TT_F32) {
#pragma unroll
                        for (int q4 = 0; q4 < 2; ++q4) {
                            if (q4 * 4 < e0 || q4 * 4 >= e0 + vc) continue;
                            f32x4 r = q4 == 0 ? lo : hi;
                            const int64_t at = idx + (q4 * 4 - e0);
                            f32x4 add = {bias_row, bias_row, bias_row, bias_row};
                            if (!SWAP && g.has_bias)
                                add += *reinterpret_cast<const f32x4 *>(static_cast<const float *>(g.bias) + colg + (q4 * 4 - e0));
                            if (g.has_res) add += *reinterpret_cast<const f32x4 *>(static_cast<const float *>(g.res) + at);
#pragma unroll
                            for (int e = 0; e < 4; ++e) r[e] = apply_act(r[e] + add[e], g.act);
                            *reinterpret_cast<f32x4 *>(static_cast<float *>(g.out) + at) = r;
                        }
                    } else {
                        for (int e = 0; e < vc; ++e) {
                            float a = val[e0 + e] + bias_row;
                            if (!SWAP && g.has_bias) a += load_as_float<DT>(g.bias, colg + e);
                            if (g.has_res) a += load_as_float<DT>(g.res, idx + e);
                            store_from_float<DT>(g.out, idx + e, apply_act(a, g.act));
                        }
                    }
                }
            }
        }
    }
}

template <int DT, int FAM, int TM, int TN, int TK, int WM, int WN, int MF, int AM>
int launch_contract(const ContractArgs &args, int grid, int lds_bytes, void *stream)
{
    auto kern = contract_kernel<DT, FAM, TM, TN, TK, WM, WN, MF, AM>;
    // the epilogue stages one band of MF rows per wave in the same LDS
    constexpr int WC_ = FAM == FAM_CONV ? WM : WN;
    constexpr int EPI_BYTES = (TM / WM) * (TN / WN) * MF * (WC_ + (MF == 32 ? 8 : 4)) * 4;
    if (lds_bytes < EPI_BYTES) lds_bytes = EPI_BYTES;
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
