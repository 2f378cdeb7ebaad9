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
// Every output is a row-major [M][N] matrix: dense and batch matmul as they are,
// conv2d because activations are NHWC, so the flattened pixel index is M and the
// output channel is N.  Matrix-core rows map to M and columns to N.
#pragma once

#include <hip/hip_runtime.h>

#include <mutex>
#include <type_traits>

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

// two floats -> two bf16 in one register (first in the low half), round to nearest, ties to even; NaN stays
// a quiet NaN.  gfx950 converts a pair in one instruction.
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
__device__ __forceinline__ uint32_t pack_bf16x2(float first, float second)
{
    const f32x2 v = {first, second};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) { return (uint16_t)pack_bf16x2(f, 0.0f); }

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

// The same on N values with one (uniform) branch for all of them.
template <int N> __device__ __forceinline__ void apply_act_all(float (&v)[N], int act)
{
    switch (act) {
    case ACT_RELU:
#pragma unroll
        for (int e = 0; e < N; ++e) v[e] = fmaxf(v[e], 0.0f);
        break;
    case ACT_RELU6:
#pragma unroll
        for (int e = 0; e < N; ++e) v[e] = fminf(fmaxf(v[e], 0.0f), 6.0f);
        break;
    case ACT_GELU:
#pragma unroll
        for (int e = 0; e < N; ++e) v[e] = 0.5f * v[e] * (1.0f + erff(v[e] * 0.70710678118654752f));
        break;
    default: break;
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
// All loaders follow one rule: a fetch only ISSUES loads.  Every load is unconditional and lands
// in a register nothing reads until the slice is written to LDS, so the loads of slice t+1 stay
// in flight during the matrix work of slice t.  The row loader replaces an address that would fall
// outside the matrix by a safe one inside it and repairs tails in the store step; the gathering
// loader uses bounds-checked buffer loads, which return zero for an offset outside the tensor, so
// padding and tails cost one select on the offset and nothing afterwards.  There is one
// straight-line code path per kernel: how the operands are fetched is a template parameter.

// Unconditional loads into registers (addresses need only element alignment).
__device__ __forceinline__ void load16(u32x4 &dst, const void *p) { __builtin_memcpy(&dst, p, 16); }

// Shift the 16-byte value by whole elements: positive = towards higher element indices; zero fill.
// |elems| must be below the item's element count (a shift by the whole width is undefined).
template <int DT> __device__ __forceinline__ u32x4 shift_elems(const u32x4 &v, int elems)
{
    constexpr int EB = DT == TT_F32 ? 32 : 16;
    unsigned __int128 x = ((unsigned __int128)v[3] << 96) | ((unsigned __int128)v[2] << 64) |
                          ((unsigned __int128)v[1] << 32) | (unsigned __int128)v[0];
    x = elems >= 0 ? (x << (EB * elems)) : (x >> (EB * -elems));
    u32x4 r = {(uint32_t)x, (uint32_t)(x >> 32), (uint32_t)(x >> 64), (uint32_t)(x >> 96)};
    return r;
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

// Masks that zero the elements of a 16-byte item at positions outside [lo, hi), 0 <= lo <= hi <= elements
// per item, as a table in device memory indexed by lo * (CH + 1) + hi.  The element-wise gather is bound by
// vector instructions: it asks for an item's mask when it requests the item (one more load in flight, from
// a table of a few cache lines) and applies it with four ANDs when the item goes to LDS, where building the
// mask from range compares took about 25 instructions per item.
template <int DT> struct RangeMasks {
    static constexpr int CH = DT == TT_BF16 ? 8 : 4;
    uint32_t w[(CH + 1) * (CH + 1)][4];
    constexpr RangeMasks() : w{}
    {
        for (int lo = 0; lo <= CH; ++lo)
            for (int hi = lo; hi <= CH; ++hi)
                for (int e = lo; e < hi; ++e) {
                    if (DT == TT_BF16)
                        w[lo * (CH + 1) + hi][e / 2] |= 0xffffu << (16 * (e % 2));
                    else
                        w[lo * (CH + 1) + hi][e] = 0xffffffffu;
                }
    }
};
static __device__ const RangeMasks<TT_BF16> kRangeMasksBf16{};
static __device__ const RangeMasks<TT_F32> kRangeMasksF32{};
template <int DT> __device__ __forceinline__ u32x4 range_mask(int lo, int hi)
{
    if constexpr (DT == TT_BF16)
        return *reinterpret_cast<const u32x4 *>(kRangeMasksBf16.w[lo * 9 + hi]);
    else
        return *reinterpret_cast<const u32x4 *>(kRangeMasksF32.w[lo * 5 + hi]);
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
                if (back > 0 || gk + CH > k_end) v = keep_first<DT>(shift_elems<DT>(v, -min(back, CH - 1)), k_end - gk);
                // a chunk that starts at or past the end of the row or of the slice holds nothing
                if (row0 + r >= rows_total || back >= CH || gk >= k_end) v = u32x4{0u, 0u, 0u, 0u};
            }
            *reinterpret_cast<u32x4 *>(lds + r * ROWB + kc * 16) = v;
        }
    }
};


// ---- gathered tiles: conv2d as an implicit GEMM over NHWC activations -------------------------------------------
//
// Row m of the implicit matrix is output pixel (image, p, q); the reduction index is
// k = r * runp + j, with r the filter row and j the position inside the RUN of S * C elements that
// one filter row covers.  In an NHWC image row those S * C elements are contiguous, and so they are
// in a KRSC filter, so element (m, k) sits at  origin(m) + r * row_stride + j  where origin(m) is
// the (possibly negative) element offset of tap (0, 0), channel 0.  It is real when filter row r
// falls inside the image (one bit per r, kept per row of the tile) and j inside [jlo, jhi), the
// part of the run that falls inside the image row; everything else is zero padding.
//
// With VEC an item is one 16-byte load: C is a multiple of the items' element count, so an item
// lies inside one pixel and is real or padding as a whole.  Without VEC (the 3-channel stem) the
// run is padded up to whole items (runp > run) and an item may be real in part: it is still one
// 16-byte load, at element alignment, and the store step zeroes the elements outside [jlo, jhi).
// Only an item that would begin before the tensor or end after it (where the bounds check works on
// whole 4-byte words) is gathered element by element.  The same loader reads the filter matrix
// in that case (WEIGHTS): rows are output channels, origin = n * R * run, every filter row is real
// and j < run.
//
// All rows a thread loads share one chunk of the slice (THREADS is a multiple of the chunks per
// row), so (r, j) is one pair per thread, advanced by add-and-carry from slice to slice.

constexpr uint32_t kOutOfRange = 0x80000000u; // byte offset no tensor reaches: such a load returns zero

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes)
{
    // raw buffer (stride 0), 32-bit data format: offsets are bytes, checked against `bytes`
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, bytes, 0x00020000);
}

template <int DT, int ROWS, int TK, int THREADS, bool VEC, bool WEIGHTS> struct GatherLoader {
    using E = typename ElemOf<DT>::type;
    static constexpr int CH = ElemOf<DT>::CH, ES = (int)sizeof(E), CPR = TK / CH, TOTAL = ROWS * CPR;
    static constexpr int NL = (TOTAL + THREADS - 1) / THREADS, STEP = THREADS / CPR;
    static constexpr int ROWB = (TK + CH) * ES;
    static_assert(THREADS % CPR == 0, "a thread's items must share one chunk of the slice");
    struct State {
        int32_t origin[NL];  // element offset of (tap (0,0), channel 0) / of the filter's first element
        uint32_t rmask[NL];  // bit r set: filter row r of this tile row is real (0 for rows past the matrix)
        int32_t jlo[NL], jhi[NL];
        int32_t r, j, dr, dj, runp, row_stride, numel;
        u32x4 raw[NL];
        int32_t span[NL]; // without VEC, bf16: 2 if the item in flight starts in the upper half of its first
                          // 32-bit word (the bytes to shift it down by), else 0
        u32x4 mask[NL];   // without VEC: ones over the real elements of the item in flight
        uint32_t tail[NL]; // bf16 without VEC: the 32-bit word after raw (the item's last element if it starts odd)
    };

    static __device__ __forceinline__ void init(State &st, const ContractArgs &g, int row0, int k0, int tid)
    {
        const int chunk = tid % CPR, first = tid / CPR;
        const int kk = k0 + chunk * CH;
        st.numel = (int32_t)((WEIGHTS ? g.b_bytes : g.a_bytes) / (uint32_t)ES);
        st.runp = g.runp;
        st.r = kk / g.runp;
        st.j = kk - st.r * g.runp;
        st.dr = TK / g.runp;
        st.dj = TK - st.dr * g.runp;
        st.row_stride = WEIGHTS ? g.run : g.W * g.C;
        const uint32_t all_rows = g.R >= 32 ? 0xffffffffu : ((1u << g.R) - 1u);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int row = first + i * STEP;
            const int m = row0 + row;
            const bool live = (TOTAL % THREADS == 0 || row < ROWS) && m < (WEIGHTS ? g.N : g.M);
            if constexpr (WEIGHTS) {
                st.origin[i] = live ? m * g.R * g.run : 0;
                st.rmask[i] = live ? all_rows : 0u;
                st.jlo[i] = 0;
                st.jhi[i] = g.run;
            } else {
                const uint32_t um = live ? (uint32_t)m : 0u;
                const uint32_t img = fast_div(um, g.div_hw);
                const uint32_t rem = um - img * (uint32_t)(g.Ho * g.Wo);
                const uint32_t p = fast_div(rem, g.div_wo), q = rem - p * (uint32_t)g.Wo;
                const int ih0 = (int)p * g.stride_h - g.pad_h, iw0 = (int)q * g.stride_w - g.pad_w;
                st.origin[i] = (((int)img * g.H + ih0) * g.W + iw0) * g.C;
                // filter rows [lo, hi) read inside the image
                const int lo = max(0, -ih0), hi = min(g.R, g.H - ih0);
                const uint32_t below_hi = hi >= 32 ? 0xffffffffu : ((1u << max(hi, 0)) - 1u);
                const uint32_t below_lo = (1u << min(lo, 31)) - 1u;
                st.rmask[i] = (live && hi > lo) ? (below_hi & ~below_lo) : 0u;
                st.jlo[i] = max(0, -iw0) * g.C;
                st.jhi[i] = min(g.S, g.W - iw0) * g.C;
            }
        }
    }

    // Issue the loads of the current slice, then step (r, j) to the next one.
    static __device__ __forceinline__ void load(State &st, __amdgpu_buffer_rsrc_t rsrc, int R)
    {
        const int kterm = st.r * st.row_stride + st.j;
        const bool r_ok = st.r < R;
        const int rbit = st.r & 31;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const bool row_ok = r_ok & (((st.rmask[i] >> rbit) & 1u) != 0);
            const uint32_t at = (uint32_t)(st.origin[i] + kterm) * (uint32_t)ES;
            if constexpr (VEC) {
                const bool ok = row_ok & (st.j >= st.jlo[i]) & (st.j < st.jhi[i]);
                st.raw[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, ok ? at : kOutOfRange, 0, 0);
            } else {
                // real elements of this item: [lo, hi) relative to its first element
                const int lo = min(max(st.jlo[i] - st.j, 0), CH), hi = min(max(st.jhi[i] - st.j, 0), CH);
                const bool any = row_ok & (hi > lo);
                const int start = st.origin[i] + kterm;
                st.span[i] = 0;
                st.mask[i] = range_mask<DT>(any ? lo : 0, any ? hi : 0);
                if constexpr (DT == TT_BF16) st.tail[i] = 0u;
                if (!any || (start >= 0 && start + CH + 2 <= st.numel)) {
                    if constexpr (DT == TT_BF16) {
                        // Items start at any even byte.  Fetch the five 32-bit words that cover the item from
                        // its word-aligned start (a 16-byte load that is not word-aligned is split into
                        // many requests) and shift them into place when the slice is written to LDS.
                        const uint32_t at4 = at & ~3u;
                        st.raw[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, any ? at4 : kOutOfRange, 0, 0);
                        st.tail[i] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, any ? at4 + 16u : kOutOfRange, 0, 0);
                        st.span[i] = (int32_t)(at & 2u);
                    } else {
                        st.raw[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, any ? at : kOutOfRange, 0, 0);
                    }
                } else {
                    // the first or the last item of the whole tensor: element by element
#pragma unroll
                    for (int e = 0; e < CH; ++e) {
                        const uint32_t off = ((e >= lo) & (e < hi)) ? at + (uint32_t)(e * ES) : kOutOfRange;
                        if constexpr (DT == TT_F32) {
                            st.raw[i][e] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, off, 0, 0);
                        } else {
                            const uint32_t v = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rsrc, off, 0, 0);
                            if (e % 2 == 0)
                                st.raw[i][e / 2] = v;
                            else
                                st.raw[i][e / 2] |= v << 16;
                        }
                    }
                }
            }
        }
        st.j += st.dj;
        st.r += st.dr;
        if (st.j >= st.runp) {
            st.j -= st.runp;
            st.r += 1;
        }
    }

    static __device__ __forceinline__ void store(const State &st, unsigned char *lds, int tid)
    {
        const int chunk = tid % CPR, first = tid / CPR;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int row = first + i * STEP;
            if (TOTAL % THREADS != 0 && row >= ROWS) continue;
            u32x4 v = st.raw[i];
            if constexpr (!VEC) {
                if constexpr (DT == TT_BF16) {
                    const uint32_t sh = (uint32_t)st.span[i]; // 0 leaves the words as they are
                    v = u32x4{__builtin_amdgcn_alignbyte(v[1], v[0], sh), __builtin_amdgcn_alignbyte(v[2], v[1], sh),
                              __builtin_amdgcn_alignbyte(v[3], v[2], sh), __builtin_amdgcn_alignbyte(st.tail[i], v[3], sh)};
                }
                v &= st.mask[i];
            }
            *reinterpret_cast<u32x4 *>(lds + row * ROWB + chunk * 16) = v;
        }
    }
};

// ---- K-major tiles: the [K][N] operand of a non-transposed batch matmul ------------------------------------------
//
// Memory is contiguous along the output axis N, not along K.  The tile is kept in LDS as T[k][n],
// n contiguous, so global vectors are copied as they are.  Matrix-core fragments (8 consecutive K
// per lane for bf16) come out of the transposing LDS read of gfx950: within 16 lanes, lane i
// supplies the address of 4 consecutive n of K-row i/4 and receives the 4 K-rows of column i.
// fp32 fragments are four 4-byte reads.

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// Padded row length (elements) of a K-major tile: keeps the fragment reads free of bank conflicts.
template <int DT, int ROWS, int MF> struct KMajorRow {
    static constexpr int PAD = DT == TT_BF16 ? (32 + 64 - ROWS % 64) % 64 : (MF == 32 ? 8 : 4);
    static constexpr int LEN = ROWS + PAD;
};

// Loader of that operand (N >= G): rows of the matrix are rows of the K-major tile.  A 16-byte item that would run past the end of its row is read G elements back
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
                if (back > 0) v = keep_first<DT>(shift_elems<DT>(v, -min(back, G - 1)), N - n);
                if (k0 + kl >= k_end || n >= N || back >= G) v = u32x4{0u, 0u, 0u, 0u};
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


// ---- epilogue ---------------------------------------------------------------------------------------------------
// The accumulators hold, per lane, 4 consecutive ROWS of one column, while memory is contiguous
// along COLUMNS.  Each wave therefore passes its tile through a private LDS region, one band of
// MF rows at a time, and reads it back so that a lane owns 8 consecutive columns of one row:
// bias, residual, activation and down-conversion then work on 16-byte vectors (or on the widest
// sub-vectors the output's row length allows), and stores are fully coalesced.  With split-K
// the raw partial sums go to the workspace in the same pattern.
// Which outputs a lane owns after that transposition.
template <int TM, int WM, int WN, int MF> struct TileOut {
    static constexpr int NWR = TM / WM, NI = WM / MF, NJ = WN / MF, ACC = MF * MF / 64;
    static constexpr int ESTRIDE = WN + (MF == 32 ? 8 : 4);      // floats per staged row (bank-conflict padding)
    static constexpr int CG = WN / 8;                            // 8-column groups per row
    static constexpr int ROWS_PER_PASS = 64 / CG;                // rows the 64 lanes cover at once
    static constexpr int PASSES = (MF + ROWS_PER_PASS - 1) / ROWS_PER_PASS;
    // row of the workgroup tile / first of the 8 columns this lane handles in band i, pass ps
    static __device__ __forceinline__ int row(int wave, int lane, int i, int ps)
    {
        return (wave % NWR) * WM + i * MF + ps * ROWS_PER_PASS + lane / CG;
    }
    static __device__ __forceinline__ int col(int wave, int lane) { return (wave / NWR) * WN + (lane % CG) * 8; }
    static __device__ __forceinline__ bool pass_live(int lane, int ps)
    {
        return ROWS_PER_PASS * PASSES == MF || ps * ROWS_PER_PASS + lane / CG < MF;
    }
};

// `count` (1..8) consecutive outputs of one row, starting at element `at` of the output (column `n`), from
// the 8 staged sums lo, hi: bias, residual, activation, conversion and store one element at a time, or the
// raw sums into the split-K workspace.  Everything is passed by value so that the call needs no stack.
template <int DT>
__device__ __noinline__ void write_row_elements(float *ws, void *out, const void *bias, const void *res, bool partial,
                                                bool has_bias, bool has_res, int act, int64_t at, int n, int count,
                                                f32x4 lo, f32x4 hi)
{
#pragma unroll 1
    for (int e = 0; e < count; ++e) {
        float a = lo[0];
#pragma unroll
        for (int t = 1; t < 8; ++t) a = e == t ? (t < 4 ? lo[t] : hi[t - 4]) : a; // (registers cannot be indexed)
        if (partial) {
            ws[at + e] = a;
            continue;
        }
        if (has_bias) a += load_as_float<DT>(bias, n + e);
        if (has_res) a += load_as_float<DT>(res, at + e);
        store_from_float<DT>(out, at + e, apply_act(a, act));
    }
}

// The bias of the 8 output columns a lane finishes in the epilogue (the same for every row), as raw
// bits.  Requested at the start of a kernel, so that its memory latency runs under the K loop; a load
// inside the epilogue's loops would be repeated per pass at full latency, because the compiler cannot
// move it across the stores.  Zero where the vector path does not apply (no bias, split-K partials,
// rows that are not whole 16-byte vectors long: that path reads the bias element by element).
template <int DT> struct BiasRegs {
    u32x4 raw[DT == TT_BF16 ? 1 : 2];
};
template <int DT, int TM, int WM, int WN, int MF>
__device__ __forceinline__ BiasRegs<DT> load_bias_early(const ContractArgs &g, const TileCoord &tc, int wave, int lane)
{
    using T = TileOut<TM, WM, WN, MF>;
    BiasRegs<DT> b;
    b.raw[0] = u32x4{0u, 0u, 0u, 0u};
    if constexpr (DT == TT_F32) b.raw[1] = u32x4{0u, 0u, 0u, 0u};
    const int first = tc.n0 + T::col(wave, lane);
    const bool whole = DT == TT_BF16 ? g.eff_vec_c == 8 : g.eff_vec_c >= 4;
    if (whole && g.map.eff_split_k == 1 && g.has_bias && first < g.N) {
        if constexpr (DT == TT_BF16) {
            b.raw[0] = *reinterpret_cast<const u32x4 *>(static_cast<const uint16_t *>(g.bias) + first);
        } else {
            b.raw[0] = *reinterpret_cast<const u32x4 *>(static_cast<const float *>(g.bias) + first);
            if (first + 4 < g.N) b.raw[1] = *reinterpret_cast<const u32x4 *>(static_cast<const float *>(g.bias) + first + 4);
        }
    }
    return b;
}

// The residual values a lane adds in the epilogue, for ALL bands and passes, requested at the start of a
// kernel (right after the first operand slices) where that costs at most 16 registers and the kernel
// allows it (16-wave workgroups have 128 registers per lane and none to spare).  A streaming
// layer (short reduction, long rows of outputs) otherwise pays two memory round trips in a row, operands
// and then residuals; with this they overlap.  Wave tiles with more rows fetch band by band in the epilogue.
template <int DT, int TM, int WM, int WN, int MF, bool ALLOW = true> struct ResRegs {
    using T = TileOut<TM, WM, WN, MF>;
    static constexpr int W = DT == TT_BF16 ? 1 : 2; // 16-byte items per lane and pass
    static constexpr bool EARLY = ALLOW && T::NI * T::PASSES * W <= 4;
    u32x4 v[EARLY ? T::NI : 1][EARLY ? T::PASSES : 1][W];
};
// One pass's residual items of a lane (rows past the matrix read the tile's first row: any valid address).
template <int DT, int TM, int WM, int WN, int MF>
__device__ __forceinline__ void load_res_pass(u32x4 (&dst)[DT == TT_BF16 ? 1 : 2], const ContractArgs &g, const TileCoord &tc,
                                              int wave, int lane, int i, int ps)
{
    using T = TileOut<TM, WM, WN, MF>;
    const int first = tc.n0 + T::col(wave, lane);
    const int m = tc.m0 + T::row(wave, lane, i, ps);
    const bool live = T::pass_live(lane, ps) && m < g.M && first < g.N;
    const int64_t row_at = (int64_t)tc.hi * g.M * g.N + (int64_t)(live ? m : tc.m0) * g.N + (live ? first : tc.n0);
    if constexpr (DT == TT_BF16) {
        dst[0] = *reinterpret_cast<const u32x4 *>(static_cast<const uint16_t *>(g.res) + row_at);
    } else {
        dst[0] = *reinterpret_cast<const u32x4 *>(static_cast<const float *>(g.res) + row_at);
        dst[1] = (live && first + 4 < g.N) ? *reinterpret_cast<const u32x4 *>(static_cast<const float *>(g.res) + row_at + 4)
                                           : u32x4{0u, 0u, 0u, 0u};
    }
}
template <int DT, int TM, int WM, int WN, int MF, bool ALLOW>
__device__ __forceinline__ void load_res_early(ResRegs<DT, TM, WM, WN, MF, ALLOW> &r, const ContractArgs &g,
                                               const TileCoord &tc, int wave, int lane)
{
    using R = ResRegs<DT, TM, WM, WN, MF, ALLOW>;
    if constexpr (R::EARLY) {
        const bool whole = DT == TT_BF16 ? g.eff_vec_c == 8 : g.eff_vec_c >= 4;
        if (whole && g.map.eff_split_k == 1 && g.has_res) {
#pragma unroll
            for (int i = 0; i < R::T::NI; ++i)
#pragma unroll
                for (int ps = 0; ps < R::T::PASSES; ++ps) load_res_pass<DT, TM, WM, WN, MF>(r.v[i][ps], g, tc, wave, lane, i, ps);
        }
    }
}

template <int N> __device__ __forceinline__ void wait_loads_outstanding(); // (defined with the asynchronous loaders)

// WAIT_LOADS: the caller has asynchronous requests in flight that must have landed before the first store
// is issued (a persistent kernel's next tile); the wait sits behind the staging of the first band.
template <int DT, int TM, int WM, int WN, int MF, typename Acc, bool ALLOW, bool WAIT_LOADS = false>
__device__ __forceinline__ void write_tile(Acc (&acc)[WM / MF][WN / MF], const ContractArgs &g, const TileCoord &tc,
                                           unsigned char *smem, int wave, int lane, const BiasRegs<DT> &bias,
                                           const ResRegs<DT, TM, WM, WN, MF, ALLOW> &early)
{
    using R = ResRegs<DT, TM, WM, WN, MF, ALLOW>;
    using T = TileOut<TM, WM, WN, MF>;
    constexpr int NI = T::NI, NJ = T::NJ, ACC = T::ACC, ESTRIDE = T::ESTRIDE, CG = T::CG, PASSES = T::PASSES;
    const int lane_r = lane % MF, lane_g = lane / MF;
    const int bidx = tc.hi;
    float *stage = reinterpret_cast<float *>(smem) + wave * (MF * ESTRIDE);
    const bool partial = g.map.eff_split_k > 1;
    const int64_t mn = (int64_t)g.M * g.N;
    float *ws = g.ws + ((int64_t)tc.lo * g.batch) * mn;
    const int vc = g.eff_vec_c; // consecutive outputs of a row that are all inside or all outside the matrix
    const bool whole = DT == TT_BF16 ? vc == 8 : vc >= 4; // rows are whole 16-byte vectors long
    const int64_t out_base = (int64_t)bidx * mn;
    const int cg = lane % CG;
    const int first = tc.n0 + T::col(wave, lane);

    float biasf[8];
    if constexpr (DT == TT_BF16) {
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            biasf[2 * h] = __uint_as_float(bias.raw[0][h] << 16);
            biasf[2 * h + 1] = __uint_as_float(bias.raw[0][h] & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) biasf[e] = __uint_as_float(bias.raw[0][e]), biasf[4 + e] = __uint_as_float(bias.raw[1][e]);
    }

    // Every wave is done reading the operand tiles.  From here on a wave only touches its own staging
    // region, and the LDS executes one wave's accesses in order: no further barrier is needed, only
    // the compiler must keep the staging writes and reads in program order.
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        // the residuals of this band's rows (where they were not requested at kernel start): all passes
        // before the staging, so that their latency runs in parallel instead of once per pass
        u32x4 resv[PASSES][R::W];
        if (whole && !partial && g.has_res) {
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps) {
                if constexpr (R::EARLY) {
#pragma unroll
                    for (int w = 0; w < R::W; ++w) resv[ps][w] = early.v[i][ps][w];
                } else {
                    load_res_pass<DT, TM, WM, WN, MF>(resv[ps], g, tc, wave, lane, i, ps);
                }
            }
        }
        asm volatile("" ::: "memory"); // the reads of the band before stay ahead of these writes
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int v = 0; v < ACC; ++v) {
                const int row_l = MF == 32 ? (v / 4) * 8 + lane_g * 4 + (v % 4) : lane_g * 4 + v;
                stage[row_l * ESTRIDE + j * MF + lane_r] = acc[i][j][v];
            }
        asm volatile("" ::: "memory"); // and the reads below stay behind them
        if constexpr (WAIT_LOADS)
            if (i == 0) wait_loads_outstanding<0>();
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
            if (!T::pass_live(lane, ps)) continue;
            const int row_l = ps * T::ROWS_PER_PASS + lane / CG;
            const f32x4 lo = *reinterpret_cast<const f32x4 *>(stage + row_l * ESTRIDE + cg * 8);
            const f32x4 hi = *reinterpret_cast<const f32x4 *>(stage + row_l * ESTRIDE + cg * 8 + 4);
            float val[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            const int m = tc.m0 + T::row(wave, lane, i, ps);
            if (m >= g.M || first >= g.N) continue;
            const int64_t row_at = out_base + (int64_t)m * g.N + first;
            if (whole) {
                // Rows are whole vectors long: the lane's 8 columns (fp32: its two groups of 4) need no
                // further checks and no loop.  Bias first, then the residual (the order of the
                // element-wise path).
                if (partial) {
                    *reinterpret_cast<f32x4 *>(ws + row_at) = lo;
                    if (DT == TT_BF16 || first + 4 < g.N) *reinterpret_cast<f32x4 *>(ws + row_at + 4) = hi;
                } else if constexpr (DT == TT_BF16) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) val[e] += biasf[e];
                    if (g.has_res) {
#pragma unroll
                        for (int h = 0; h < 4; ++h) {
                            val[2 * h] += __uint_as_float(resv[ps][0][h] << 16);
                            val[2 * h + 1] += __uint_as_float(resv[ps][0][h] & 0xffff0000u);
                        }
                    }
                    apply_act_all(val, g.act);
                    u32x4 outv;
#pragma unroll
                    for (int h = 0; h < 4; ++h) outv[h] = pack_bf16x2(val[2 * h], val[2 * h + 1]);
                    // streaming store: the output is not read again by this launch, and lines that leave
                    // the L2 as they are written do not wait for the write-back at the end of the kernel
                    __builtin_nontemporal_store(outv, reinterpret_cast<u32x4 *>(static_cast<uint16_t *>(g.out) + row_at));
                } else {
#pragma unroll
                    for (int q4 = 0; q4 < 2; ++q4) {
                        if (q4 == 1 && first + 4 >= g.N) break;
                        const int64_t at = row_at + 4 * q4;
                        float sum[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            sum[e] = val[4 * q4 + e] + biasf[4 * q4 + e];
                            if (g.has_res) sum[e] += __uint_as_float(resv[ps][q4][e]);
                        }
                        apply_act_all(sum, g.act);
                        __builtin_nontemporal_store(f32x4{sum[0], sum[1], sum[2], sum[3]},
                                                    reinterpret_cast<f32x4 *>(static_cast<float *>(g.out) + at));
                    }
                }
                continue;
            }
            // any other row length: element by element, out of line (rare, and it must not cost the
            // path above registers)
            write_row_elements<DT>(ws, g.out, g.bias, g.res, partial, g.has_bias, g.has_res, g.act, row_at, first,
                                   min(8, g.N - first), lo, hi);
        }
    }
}

// How many consecutive steps of a slice have their fragment reads issued together, ahead of the first
// product: the largest power of two dividing `steps` whose fragments (4 registers each) fit `budget`
// registers.  A wave then pays the LDS latency once per group instead of once per step, which the few
// waves of a workgroup that owns a CU alone cannot hide otherwise.
constexpr int steps_per_group(int fragments_per_step, int steps, int budget = 64)
{
    int g = 1;
    while (g * 2 <= steps && steps % (g * 2) == 0 && fragments_per_step * 4 * g * 2 <= budget) g *= 2;
    return g;
}

// LDS bytes of one pipeline stage: the A tile followed by the B tile.
template <int DT, int FAM, int TM, int TN, int TK, int MF> struct StageLayout {
    using E = typename ElemOf<DT>::type;
    static constexpr int CH = ElemOf<DT>::CH, ES = (int)sizeof(E);
    static constexpr int ROWB = (TK + CH) * ES; // row of a K-contiguous tile, padded by 16 bytes
    static constexpr int LEN_B = KMajorRow<DT, TN, MF>::LEN;
    static constexpr int A_BYTES = TM * ROWB;
    static constexpr int B_BYTES = FAM == FAM_GEMM_NN ? TK * LEN_B * ES : TN * ROWB;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
};

// AM = bytes per gathered load of the conv family (16 or the element size); 0 for the others.
template <int DT, int FAM, int TM, int TN, int TK, int WM, int WN, int MF, int AM>
__global__ void __launch_bounds__((TM / WM) * (TN / WN) * 64) contract_kernel(const ContractArgs g)
{
    using E = typename ElemOf<DT>::type;
    using L = StageLayout<DT, FAM, TM, TN, TK, MF>;
    constexpr int CH = ElemOf<DT>::CH, ES = (int)sizeof(E);
    constexpr int THREADS = (TM / WM) * (TN / WN) * 64;
    constexpr int ROWB = L::ROWB, A_BYTES = L::A_BYTES, STAGE_BYTES = L::STAGE_BYTES;
    constexpr int NWR = TM / WM; // waves along M
    constexpr int NI = WM / MF, NJ = WN / MF;
    constexpr int LG = 64 / MF, KS = k_granule(DT, MF), NKS = TK / KS;
    static_assert(KS == CH * LG, "one 16-byte fragment per lane group");
    constexpr int ACC = MF * MF / 64;
    constexpr bool B_KMAJOR = FAM == FAM_GEMM_NN;
    constexpr bool CONV = FAM == FAM_CONV;
    constexpr bool CONV_VEC = CONV && AM == 16; // 16-byte gathers of activations, plain rows of filters
    constexpr bool CONV_ELEM = CONV && AM != 16; // both operands gathered element by element
    static_assert(TK % KS == 0, "tile_k must be a multiple of the K granule");
    using M = Mma<DT, MF>;
    using ALoad = RowKLoader<DT, TM, TK, THREADS>;
    using AGather = GatherLoader<DT, TM, TK, THREADS, CONV_VEC, false>;
    using BLoad = RowKLoader<DT, TN, TK, THREADS>;
    using BGather = GatherLoader<DT, TN, TK, THREADS, false, true>;
    using BKRow = KRowTileLoader<DT, TN, TK, THREADS, L::LEN_B>;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const TileCoord tc = decode_tile(g.map, (int32_t)blockIdx.x);
    const BiasRegs<DT> bias = load_bias_early<DT, TM, WM, WN, MF>(g, tc, wave, lane);
    // The gathering loaders walk the reduction in runs padded to whole 16-byte items (k_walk >= K):
    // the split that ends at K runs on to the end of that walk.
    const int k_end = (CONV && tc.k0 + tc.k_ext == g.K) ? g.k_walk : tc.k0 + tc.k_ext;
    const int kt_count = (k_end - tc.k0 + TK - 1) / TK;
    const int bidx = tc.hi;

    const E *a_base = static_cast<const E *>(g.a);
    const E *b_base = static_cast<const E *>(g.b);
    if constexpr (!CONV) {
        a_base += (int64_t)bidx * g.M * g.K;
        b_base += (int64_t)bidx * g.N * g.K;
    }

    // registers holding the slice in flight (only the members of the family in use are live)
    typename AGather::State a_gat;
    typename BGather::State b_gat;
    typename BKRow::State b_krow;
    typename ALoad::State a_rows;
    typename BLoad::State b_rows;
    __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(g.a, CONV ? g.a_bytes : 0u);
    __amdgpu_buffer_rsrc_t b_rsrc = make_rsrc(g.b, CONV_ELEM ? g.b_bytes : 0u);
    if constexpr (CONV) AGather::init(a_gat, g, tc.m0, tc.k0, tid);
    if constexpr (CONV_ELEM) BGather::init(b_gat, g, tc.n0, tc.k0, tid);

    // slices are fetched in order: the gathering loaders step their own position
    auto fetch = [&](int kt) {
        const int k0 = tc.k0 + kt * TK;
        if constexpr (CONV)
            AGather::load(a_gat, a_rsrc, g.R);
        else
            ALoad::load(a_rows, a_base, g.K, tc.m0, g.M, k0, tid);
        if constexpr (B_KMAJOR)
            BKRow::load(b_krow, b_base, g.N, g.K, tc.n0, k0, tid);
        else if constexpr (CONV_ELEM)
            BGather::load(b_gat, b_rsrc, g.R);
        else
            BLoad::load(b_rows, b_base, g.K, tc.n0, g.N, k0, tid);
    };
    auto stash = [&](int stage, int kt) {
        const int k0 = tc.k0 + kt * TK;
        unsigned char *sa = smem + stage * STAGE_BYTES, *sb = sa + A_BYTES;
        if constexpr (CONV)
            AGather::store(a_gat, sa, tid);
        else
            ALoad::store(a_rows, sa, g.K, tc.m0, g.M, k0, k_end, tid);
        if constexpr (B_KMAJOR)
            BKRow::store(b_krow, sb, g.N, tc.n0, k0, k_end, tid);
        else if constexpr (CONV_ELEM)
            BGather::store(b_gat, sb, tid);
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
    const int r_off = (wr * WM + lane_r) * ROWB + lane_g * 16;
    const int c_off = (wc * WN + lane_r) * ROWB + lane_g * 16;

    auto k_step = [&](const unsigned char *sr, const unsigned char *sc, int ks) {
        u32x4 rf[NI], cf[NJ];
#pragma unroll
        for (int i = 0; i < NI; ++i)
            rf[i] = *reinterpret_cast<const u32x4 *>(sr + r_off + i * MF * ROWB + ks * KS * ES);
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            if constexpr (B_KMAJOR)
                cf[j] = kmajor_fragment<DT, MF, L::LEN_B>(sc, wc * WN + j * MF, ks * KS, lane);
            else
                cf[j] = *reinterpret_cast<const u32x4 *>(sc + c_off + j * MF * ROWB + ks * KS * ES);
        }
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) M::run(acc[i][j], rf[i], cf[j]);
    };

    // a slice's global loads are held in registers here as well: a smaller budget, and none to spare
    // for the workgroups of 16 waves (128 registers per lane)
    constexpr int GROUP = steps_per_group(NI + NJ, NKS, THREADS > 512 ? 16 : 48);
    auto k_group = [&](const unsigned char *sr, const unsigned char *sc, int ks0) {
        u32x4 rf[GROUP][NI], cf[GROUP][NJ];
#pragma unroll
        for (int s = 0; s < GROUP; ++s) {
#pragma unroll
            for (int i = 0; i < NI; ++i)
                rf[s][i] = *reinterpret_cast<const u32x4 *>(sr + r_off + i * MF * ROWB + (ks0 + s) * KS * ES);
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                if constexpr (B_KMAJOR)
                    cf[s][j] = kmajor_fragment<DT, MF, L::LEN_B>(sc, wc * WN + j * MF, (ks0 + s) * KS, lane);
                else
                    cf[s][j] = *reinterpret_cast<const u32x4 *>(sc + c_off + j * MF * ROWB + (ks0 + s) * KS * ES);
            }
        }
        __builtin_amdgcn_sched_barrier(0); // keep the reads ahead of the products
#pragma unroll
        for (int s = 0; s < GROUP; ++s)
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j) M::run(acc[i][j], rf[s][i], cf[s][j]);
    };

    fetch(0);
    ResRegs<DT, TM, WM, WN, MF, (THREADS <= 512)> res_early;
    load_res_early(res_early, g, tc, wave, lane); // behind the first slice's loads, which the stash below waits for alone
    stash(0, 0);
    __syncthreads();
    const bool two_stage = g.stages == 2;
    // The unroll knob picks one of two complete K loops: a choice inside the loop would make the
    // compiler shuttle the accumulators between the register sets of the two paths on every slice.
    auto k_loop = [&](auto unroll_steps) {
        int cur = 0;
        for (int it = 0; it < kt_count; ++it) {
            const bool more = it + 1 < kt_count;
            if (more) fetch(it + 1);
            const unsigned char *sa = smem + cur * STAGE_BYTES, *sb = sa + A_BYTES;
            if constexpr (decltype(unroll_steps)::value) {
#pragma unroll
                for (int ks = 0; ks < NKS; ks += GROUP) k_group(sa, sb, ks);
            } else {
#pragma unroll 1
                for (int ks = 0; ks < NKS; ++ks) k_step(sa, sb, ks);
            }
            if (more) {
                if (!two_stage) __syncthreads();
                stash(two_stage ? cur ^ 1 : 0, it + 1);
            }
            __syncthreads();
            if (two_stage) cur ^= 1;
        }
    };
    if (NKS == 1 || g.unroll >= 2)
        k_loop(std::true_type{});
    else
        k_loop(std::false_type{});

    write_tile<DT, TM, WM, WN, MF>(acc, g, tc, smem, wave, lane, bias, res_early);
}

// ---- asynchronous pipeline: global -> LDS without passing through registers --------------------------------------
//
// gfx950 buffer loads can deposit 16 bytes per lane straight into LDS (lane i of the wave writes
// at M0 + 16 * i; an out-of-range offset deposits zeros).  Nothing of a slice lives in registers, so
// several slices can be in flight: the K loop keeps a ring of `stages` LDS buffers, requests slice
// t + stages - 1 while computing on slice t, and waits only for the oldest outstanding slice (the
// vector-memory counter retires in order).  One barrier per slice both publishes the arrived
// slice and frees the buffer that was computed on before it.
//
// A wave's 64 items land in 1 KB of consecutive LDS, so rows cannot be padded.  Bank conflicts of
// the 16-byte fragment reads are avoided by a swizzle instead: the item holding K-chunk c of row r
// is stored at chunk position c ^ swizzle(r), which spreads 16 consecutive rows of one chunk over
// all banks.  The lane that fills LDS position p of a row simply fetches chunk p ^ swizzle(r).
//
// These loads are issued from inline assembly: the compiler would otherwise order every LDS read
// after ALL outstanding loads.  They have no register results, and the kernel waits for them
// explicitly (s_waitcnt vmcnt) before the barrier that precedes any read of their buffer.

// chunk swizzle of row r for rows of CPR 16-byte chunks (CPR = 4, 8 or 16): depends on r mod 16 only
template <int CPR> __device__ __forceinline__ int chunk_swizzle(int r) { return (r / (16 / CPR)) % CPR; }

// M0 is named as clobbered so that the compiler never places this statement between a write of M0 of
// its own and the instruction that reads it (M0 is a reserved register, which the allocator does not
// hand out; the compiler's generic warning about reserved registers in clobber lists is switched off).
__device__ __forceinline__ void load16_to_lds(__amdgpu_buffer_rsrc_t rsrc, uint32_t byte_offset, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(byte_offset), "s"(rsrc)
                 : "memory", "m0");
}

template <int N> __device__ __forceinline__ void wait_loads_outstanding()
{
    static_assert(N >= 0 && N < 64, "vector-memory counter range");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const unsigned char *)p;
}

// Rows of a K-contiguous matrix [rows_total][K], K a multiple of the items' element count.
template <int DT, int ROWS, int TK, int THREADS> struct AsyncRows {
    static constexpr int CH = ElemOf<DT>::CH, ES = 16 / CH, CPR = TK / CH, TOTAL = ROWS * CPR, NL = TOTAL / THREADS;
    static_assert(TOTAL % THREADS == 0 && (THREADS / 16) % CPR == 0, "tile does not fit the asynchronous loader");
    struct State {
        uint32_t at[NL]; // byte offset of this thread's chunk of the row at k = 0; out of range for rows past the matrix
        int32_t kc;      // element offset of the chunk inside a slice
    };
    static __device__ __forceinline__ void init(State &st, int K, int row0, int rows_total, int tid)
    {
        const int first = tid / CPR, pos = tid % CPR;
        st.kc = (pos ^ chunk_swizzle<CPR>(first)) * CH;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int row = row0 + first + i * (THREADS / CPR);
            st.at[i] = row < rows_total ? (uint32_t)(row * K + st.kc) * (uint32_t)ES : kOutOfRange;
        }
    }
    static __device__ __forceinline__ void issue(const State &st, __amdgpu_buffer_rsrc_t rsrc, uint32_t lds_tile, int k0,
                                                 int k_end, int wave)
    {
        const bool k_ok = k0 + st.kc < k_end;
#pragma unroll
        for (int i = 0; i < NL; ++i)
            load16_to_lds(rsrc, k_ok ? st.at[i] + (uint32_t)(k0 * ES) : kOutOfRange,
                          lds_tile + (uint32_t)((i * THREADS + wave * 64) * 16));
    }
};

// Implicit-GEMM rows of NHWC activations (see GatherLoader for the addressing), 16-byte items.
template <int DT, int ROWS, int TK, int THREADS> struct AsyncGather {
    static constexpr int CH = ElemOf<DT>::CH, ES = 16 / CH, CPR = TK / CH, TOTAL = ROWS * CPR, NL = TOTAL / THREADS;
    static_assert(TOTAL % THREADS == 0 && (THREADS / 16) % CPR == 0, "tile does not fit the asynchronous loader");
    struct State {
        int32_t origin[NL];
        uint32_t rmask[NL];
        int32_t jlo[NL], jhi[NL];
        int32_t r, j, dr, dj, runp, row_stride;
    };
    static __device__ __forceinline__ void init(State &st, const ContractArgs &g, int row0, int k0, int tid)
    {
        const int first = tid / CPR, pos = tid % CPR;
        const int kk = k0 + (pos ^ chunk_swizzle<CPR>(first)) * CH;
        st.runp = g.runp;
        st.r = kk / g.runp;
        st.j = kk - st.r * g.runp;
        st.dr = TK / g.runp;
        st.dj = TK - st.dr * g.runp;
        st.row_stride = g.W * g.C;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int m = row0 + first + i * (THREADS / CPR);
            const bool live = m < g.M;
            const uint32_t um = live ? (uint32_t)m : 0u;
            const uint32_t img = fast_div(um, g.div_hw);
            const uint32_t rem = um - img * (uint32_t)(g.Ho * g.Wo);
            const uint32_t p = fast_div(rem, g.div_wo), q = rem - p * (uint32_t)g.Wo;
            const int ih0 = (int)p * g.stride_h - g.pad_h, iw0 = (int)q * g.stride_w - g.pad_w;
            st.origin[i] = (((int)img * g.H + ih0) * g.W + iw0) * g.C;
            const int lo = max(0, -ih0), hi = min(g.R, g.H - ih0);
            const uint32_t below_hi = hi >= 32 ? 0xffffffffu : ((1u << max(hi, 0)) - 1u);
            const uint32_t below_lo = (1u << min(lo, 31)) - 1u;
            st.rmask[i] = (live && hi > lo) ? (below_hi & ~below_lo) : 0u;
            st.jlo[i] = max(0, -iw0) * g.C;
            st.jhi[i] = min(g.S, g.W - iw0) * g.C;
        }
    }
    // Request the current slice, then step (r, j) to the next one.
    static __device__ __forceinline__ void issue(State &st, __amdgpu_buffer_rsrc_t rsrc, uint32_t lds_tile, int R, int wave)
    {
        const int kterm = st.r * st.row_stride + st.j;
        const bool r_ok = st.r < R;
        const int rbit = st.r & 31;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const bool ok = r_ok & (((st.rmask[i] >> rbit) & 1u) != 0) & (st.j >= st.jlo[i]) & (st.j < st.jhi[i]);
            load16_to_lds(rsrc, ok ? (uint32_t)(st.origin[i] + kterm) * (uint32_t)ES : kOutOfRange,
                          lds_tile + (uint32_t)((i * THREADS + wave * 64) * 16));
        }
        st.j += st.dj;
        st.r += st.dr;
        if (st.j >= st.runp) {
            st.j -= st.runp;
            st.r += 1;
        }
    }
};

// One buffer of the ring: the A tile followed by the B tile, rows unpadded.
template <int DT, int TM, int TN, int TK> struct RingLayout {
    static constexpr int RB = TK * (int)sizeof(typename ElemOf<DT>::type);
    static constexpr int A_BYTES = TM * RB, STAGE_BYTES = (TM + TN) * RB;
};

// Conv (16-byte gathers) and dense family with the asynchronous pipeline; g.stages = 3 or 4 buffers.
template <int DT, int FAM, int TM, int TN, int TK, int WM, int WN, int MF>
__global__ void __launch_bounds__((TM / WM) * (TN / WN) * 64) contract_async_kernel(const ContractArgs g)
{
    static_assert(FAM == FAM_CONV || FAM == FAM_GEMM_TN, "family without an asynchronous loader");
    using E = typename ElemOf<DT>::type;
    constexpr int CH = ElemOf<DT>::CH, ES = (int)sizeof(E);
    constexpr int THREADS = (TM / WM) * (TN / WN) * 64;
    using L = RingLayout<DT, TM, TN, TK>;
    constexpr int RB = L::RB, CPR = TK / CH;
    constexpr int A_BYTES = L::A_BYTES, STAGE_BYTES = L::STAGE_BYTES;
    constexpr int NWR = TM / WM;
    constexpr int NI = WM / MF, NJ = WN / MF;
    constexpr int LG = 64 / MF, KS = CH * LG, NKS = TK / KS;
    constexpr int ACC = MF * MF / 64;
    constexpr bool CONV = FAM == FAM_CONV;
    using M = Mma<DT, MF>;
    using ARows = AsyncRows<DT, TM, TK, THREADS>;
    using AGat = AsyncGather<DT, TM, TK, THREADS>;
    using BRows = AsyncRows<DT, TN, TK, THREADS>;
    constexpr int LPS = ARows::NL + BRows::NL; // loads per slice and thread
    static_assert(2 * LPS < 64, "too many loads in flight for the counter");
    constexpr int GROUP = steps_per_group(NI + NJ, NKS);

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const uint32_t lds0 = lds_address(smem);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const TileCoord tc = decode_tile(g.map, (int32_t)blockIdx.x);
    const BiasRegs<DT> bias = load_bias_early<DT, TM, WM, WN, MF>(g, tc, wave, lane);
    const int k_end = tc.k0 + tc.k_ext; // (whole items only: the gather's walk is the reduction itself)
    const int kt_count = (tc.k_ext + TK - 1) / TK;
    const int bidx = tc.hi;
    const int nst = g.stages;

    // per-batch views of the operands; the caller has checked that each fits the 2 GiB offset range
    const E *a_base = static_cast<const E *>(g.a), *b_base = static_cast<const E *>(g.b);
    if constexpr (!CONV) {
        a_base += (int64_t)bidx * g.M * g.K;
        b_base += (int64_t)bidx * g.N * g.K;
    }
    const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(a_base, CONV ? g.a_bytes : (uint32_t)(g.M * g.K * ES));
    const __amdgpu_buffer_rsrc_t b_rsrc = make_rsrc(b_base, (uint32_t)(g.N * g.K * ES));

    typename ARows::State a_rows;
    typename AGat::State a_gat;
    typename BRows::State b_rows;
    if constexpr (CONV)
        AGat::init(a_gat, g, tc.m0, tc.k0, tid);
    else
        ARows::init(a_rows, g.K, tc.m0, g.M, tid);
    BRows::init(b_rows, g.K, tc.n0, g.N, tid);

    // slices are requested in order
    auto request = [&](int kt, int stage) {
        const int k0 = tc.k0 + kt * TK;
        const uint32_t sa = lds0 + (uint32_t)(stage * STAGE_BYTES);
        if constexpr (CONV)
            AGat::issue(a_gat, a_rsrc, sa, g.R, wave);
        else
            ARows::issue(a_rows, a_rsrc, sa, k0, k_end, wave);
        BRows::issue(b_rows, b_rsrc, sa + A_BYTES, k0, k_end, wave);
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
    const int swz = chunk_swizzle<CPR>(lane_r);
    const int a_row = (wr * WM + lane_r) * RB, b_row = (wc * WN + lane_r) * RB;

    auto k_step = [&](const unsigned char *sa, const unsigned char *sb, int ks) {
        const int at = ((ks * LG + lane_g) ^ swz) * 16;
        u32x4 rf[NI], cf[NJ];
#pragma unroll
        for (int i = 0; i < NI; ++i) rf[i] = *reinterpret_cast<const u32x4 *>(sa + a_row + i * MF * RB + at);
#pragma unroll
        for (int j = 0; j < NJ; ++j) cf[j] = *reinterpret_cast<const u32x4 *>(sb + b_row + j * MF * RB + at);
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) M::run(acc[i][j], rf[i], cf[j]);
    };

    // GROUP consecutive steps: all their fragment reads are issued before the first product
    struct Fragments {
        u32x4 rf[GROUP][NI], cf[GROUP][NJ];
    };
    auto read_group = [&](Fragments &f, const unsigned char *sa, const unsigned char *sb, int ks0) {
#pragma unroll
        for (int s = 0; s < GROUP; ++s) {
            const int at = (((ks0 + s) * LG + lane_g) ^ swz) * 16;
#pragma unroll
            for (int i = 0; i < NI; ++i) f.rf[s][i] = *reinterpret_cast<const u32x4 *>(sa + a_row + i * MF * RB + at);
#pragma unroll
            for (int j = 0; j < NJ; ++j) f.cf[s][j] = *reinterpret_cast<const u32x4 *>(sb + b_row + j * MF * RB + at);
        }
        __builtin_amdgcn_sched_barrier(0); // keep the reads ahead of what follows
    };
    auto multiply_group = [&](const Fragments &f) {
#pragma unroll
        for (int s = 0; s < GROUP; ++s)
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j) M::run(acc[i][j], f.rf[s][i], f.cf[s][j]);
    };

    // prologue: fill all but one buffer
    int requested = 0;
    for (; requested < nst - 1 && requested < kt_count; ++requested) request(requested, requested);
    // The residuals go out behind the first slices.  They are ordinary loads into registers, so the
    // counter arithmetic of the loop below sees them as further loads in flight: the first waits then also
    // wait for them to start arriving in order, which costs nothing a slice from the same memory would not.
    ResRegs<DT, TM, WM, WN, MF, (THREADS <= 512)> res_early;
    load_res_early(res_early, g, tc, wave, lane);
    // The unroll knob picks one of two complete K loops (a choice inside the loop would make the
    // compiler shuttle the accumulators between the register sets of the two paths on every slice).
    auto k_loop = [&](auto unroll_steps) {
        int cur = 0, fill = requested == nst - 1 ? nst - 1 : 0; // buffer to compute on / buffer the next request fills
        // One slice: wait until at most `younger` later slices are outstanding, publish it, compute on it;
        // `requesting` iterations also ask for slice it + stages - 1.
        auto wait_for_slice = [&](int younger) {
            if (younger >= 2)
                wait_loads_outstanding<2 * LPS>();
            else if (younger == 1)
                wait_loads_outstanding<LPS>();
            else
                wait_loads_outstanding<0>();
        };
        auto slice = [&](auto requesting) {
            __syncthreads(); // the slice is visible to all waves, and all waves are done with the one before it
            const unsigned char *sa = smem + cur * STAGE_BYTES, *sb = sa + A_BYTES;
            auto request_next = [&]() {
                if constexpr (decltype(requesting)::value) {
                    request(requested, fill); // into the buffer that held the slice before this one
                    ++requested;
                    fill = fill + 1 == nst ? 0 : fill + 1;
                }
            };
            if constexpr (decltype(unroll_steps)::value) {
                // The first fragment reads go out before the next slice is requested: the address
                // arithmetic of the requests then runs while the LDS answers, instead of after it (a wave
                // executes in order, and a workgroup that owns its CU has few waves to fill the gap).
                Fragments f;
                read_group(f, sa, sb, 0);
                request_next();
                multiply_group(f);
#pragma unroll
                for (int ks = GROUP; ks < NKS; ks += GROUP) {
                    read_group(f, sa, sb, ks);
                    multiply_group(f);
                }
            } else {
                request_next();
#pragma unroll 1
                for (int ks = 0; ks < NKS; ++ks) k_step(sa, sb, ks);
            }
            cur = cur + 1 == nst ? 0 : cur + 1;
        };
        // Steady state: while slices remain to be requested, stages - 2 younger slices are in flight at the
        // top of every iteration (the prologue requested stages - 1 of them), so the wait is the same each time.
        int it = 0;
        for (; requested < kt_count; ++it) {
            if (nst == 4)
                wait_loads_outstanding<2 * LPS>();
            else
                wait_loads_outstanding<LPS>();
            slice(std::true_type{});
        }
        // Drain: everything is requested; slice `it` has arrived once at most kt_count - it - 1 younger ones are outstanding.
        for (; it < kt_count; ++it) {
            wait_for_slice(kt_count - it - 1);
            slice(std::false_type{});
        }
    };
    if (NKS == 1 || g.unroll >= 2)
        k_loop(std::true_type{});
    else
        k_loop(std::false_type{});
    write_tile<DT, TM, WM, WN, MF>(acc, g, tc, smem, wave, lane, bias, res_early);
}

// More than 48 KB of dynamic LDS has to be enabled per kernel.  Remembers the largest size enabled so far
// (one device per process); host threads may launch the same kernel concurrently.
struct DynamicLdsLimit {
    std::mutex guard;
    int raised = 0;
    int raise_to(const void *kernel, int lds_bytes)
    {
        if (lds_bytes <= 48 * 1024) return TT_OK;
        std::lock_guard<std::mutex> lock(guard);
        if (lds_bytes > raised) {
            const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
            if (e != hipSuccess) return note_hip_error((int)e, "hipFuncSetAttribute(MaxDynamicSharedMemorySize)");
            raised = lds_bytes;
        }
        return TT_OK;
    }
};

template <int DT, int FAM, int TM, int TN, int TK, int WM, int WN, int MF, int AM>
int launch_contract(const ContractArgs &args, int grid, int lds_bytes, void *stream)
{
    auto kern = contract_kernel<DT, FAM, TM, TN, TK, WM, WN, MF, AM>;
    // the epilogue stages one band of MF rows per wave in the same LDS
    constexpr int EPI_BYTES = (TM / WM) * (TN / WN) * MF * (WN + (MF == 32 ? 8 : 4)) * 4;
    if (lds_bytes < EPI_BYTES) lds_bytes = EPI_BYTES;
    static DynamicLdsLimit limit; // per kernel instance
    if (const int rc = limit.raise_to(reinterpret_cast<const void *>(kern), lds_bytes); rc != TT_OK) return rc;
    constexpr int THREADS = (TM / WM) * (TN / WN) * 64;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(THREADS), lds_bytes, static_cast<hipStream_t>(stream), args);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : note_hip_error((int)e, "contract_kernel launch");
}

// What the host's resource check multiplies by the number of stages.
template <int DT, int FAM, int TM, int TN, int TK, int WM, int WN, int MF, int AM> int stage_bytes_contract()
{
    return StageLayout<DT, FAM, TM, TN, TK, MF>::STAGE_BYTES;
}
template <int DT, int FAM, int TM, int TN, int TK, int WM, int WN, int MF> int stage_bytes_contract_async()
{
    return RingLayout<DT, TM, TN, TK>::STAGE_BYTES;
}
template <int DT, int FAM, int TM, int TN, int TK, int WM, int WN, int MF, int AM> int lds_bytes_contract(int stages)
{
    return stages * StageLayout<DT, FAM, TM, TN, TK, MF>::STAGE_BYTES;
}
template <int DT, int FAM, int TM, int TN, int TK, int WM, int WN, int MF> int lds_bytes_contract_async(int stages)
{
    return stages * RingLayout<DT, TM, TN, TK>::STAGE_BYTES;
}

template <int DT, int FAM, int TM, int TN, int TK, int WM, int WN, int MF>
int launch_contract_async(const ContractArgs &args, int grid, int lds_bytes, void *stream)
{
    auto kern = contract_async_kernel<DT, FAM, TM, TN, TK, WM, WN, MF>;
    constexpr int EPI_BYTES = (TM / WM) * (TN / WN) * MF * (WN + (MF == 32 ? 8 : 4)) * 4;
    if (lds_bytes < EPI_BYTES) lds_bytes = EPI_BYTES;
    static DynamicLdsLimit limit; // per kernel instance
    if (const int rc = limit.raise_to(reinterpret_cast<const void *>(kern), lds_bytes); rc != TT_OK) return rc;
    constexpr int THREADS = (TM / WM) * (TN / WN) * 64;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(THREADS), lds_bytes, static_cast<hipStream_t>(stream), args);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : note_hip_error((int)e, "contract_async_kernel launch");
}

} // namespace tt
