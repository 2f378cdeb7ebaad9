// 3x3 convolution with the padded input of the workgroup's tile cached in LDS (bf16, 32x32x16 matrix cores).
//
// Algorithm 2 of the paper has a padding stage in front of the convolution, and where that stage is
// computed is a scheduling decision (ComputeAt).  The implicit-GEMM kernels compute it "inline": every
// element of the im2col matrix is fetched from global memory when a K slice needs it, so each input
// pixel passes the CU's memory pipeline R * S = 9 times.  That pipeline (about 45 bytes per clock and CU
// from the L2) is what bounds those kernels on the deep layers.  Here the padded input is computed at
// the workgroup tile instead: for a slice of CK input channels, every padded pixel that the tile's
// TM output pixels touch under any of the nine taps is brought to LDS ONCE (the "patch"; zeros for
// the padding come from out-of-range buffer loads), and the A fragments of all nine taps are read from
// it with per-lane addresses.  Only the filters are streamed, tap by tap, through a ring of LDS
// buffers, exactly as in the asynchronous GEMM pipeline.
//
// Reduction order: channel slices outermost, then the nine taps, then the CK channels of the slice
// (a permutation of the (r, s, c) order of the definition; a sum does not depend on it beyond rounding).
// A "K tile" of the schedule record (tile_k = CK) is one tap of one channel slice, so a split of the
// reduction must fall on slice boundaries (k_iters a multiple of 9).
//
// Workgroup: (TM / WM) * (TN / WN) wave positions times KG = 2 "K groups".  The two waves of a position
// share the output tile and take alternate 16-element K steps of every tap, so each SIMD holds two
// waves whose LDS reads and matrix products overlap; at the end each wave hands half of its partial
// tile to its partner through LDS and finishes the other half (bias, residual, activation, store).
//
// Padded coordinates: pixel (img, ph, pw) with ph = ih + pad_h, pw = iw + pad_w has the flat index
// pp = img * PH * PW + ph * PW + pw (PH = H + 2 pad_h, PW = W + 2 pad_w).  Tap (r, s) of output pixel
// m = (img, p, q) is pp = base(m) + r * PW + s with base(m) = img * PH * PW + p * stride * PW + q * stride,
// and base is increasing in m, so a tile's patch is the index range [base(m0), base(m_last) + 2 PW + 2].
#pragma once

#include "contract.hip.h"

namespace tt {

// f(integral_constant<int, 0>), ..., f(integral_constant<int, N - 1>): a loop whose index is a constant expression.
template <int I, int N, typename F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// Loads of one iteration of the tap loop: the filter tile, and at the taps below `pieces` one patch item.
// younger_loads = what was requested after the filters of tap `tap` (ring of `depth` buffers): the
// iterations of the depth - 2 taps before it.
constexpr int patch_younger_loads(int tap, int depth, int filter_loads, int pieces, int taps)
{
    int n = 0;
    for (int d = 1; d <= depth - 2; ++d) n += filter_loads + (((tap - d + taps) % taps) < pieces ? 1 : 0);
    return n;
}

// Geometry of the patch buffer of one channel slice.
template <int CK, int STRIDE, int PL, int THREADS> struct PatchLayout {
    static constexpr int CPP = CK / 8;                  // 16-byte items per pixel
    static constexpr int ITEMS = PL * THREADS;          // items the workgroup loads per slice
    static constexpr int PIXELS = ITEMS / CPP;          // capacity in pixels
    static constexpr int PLANE = PIXELS / STRIDE;       // pixels per parity plane (stride 2 keeps even and odd
                                                        // patch pixels apart, so that the 16 lanes of a fragment
                                                        // read, which are STRIDE pixels apart, sit side by side)
    static constexpr int BYTES = ITEMS * 16;
    static_assert(ITEMS % CPP == 0 && PIXELS % STRIDE == 0, "patch capacity");
    // Patch pixel j is stored at pixel position (j % STRIDE) * PLANE + j / STRIDE; inside it, channel chunk c
    // sits at chunk position c ^ chunk_swizzle(key), where key = (padded row / STRIDE) * Wo + padded
    // column / STRIDE counts pixels with the OUTPUT row length as its pitch.  Under a fixed tap the 16
    // lanes of a fragment read (16 consecutive output pixels) then have 16 consecutive keys also where
    // the run wraps to the next image row, while the storage index jumps over the padding there: the
    // pair (storage parity, swizzle) stays distinct across the group, and the read free of bank conflicts.
    static __device__ __forceinline__ int key(int img, int ph, int pw, int key_rows, int wo)
    {
        return (img * key_rows + ph / STRIDE) * wo + pw / STRIDE;
    }
};

// (CK, WM x WN wave tile of 32-blocks, PL patch items per thread and slice)
template <int TM, int TN, int CK, int WM, int WN, int STRIDE, int PL>
__global__ void __launch_bounds__((TM / WM) * (TN / WN) * 128) conv3x3_patch_kernel(const ContractArgs g)
{
    constexpr int DT = TT_BF16, MF = 32, KG = 2, TAPS = 9;
    constexpr int POS = (TM / WM) * (TN / WN), THREADS = POS * KG * 64;
    constexpr int NWR = TM / WM;
    constexpr int NI = WM / MF, NJ = WN / MF, ACC = 16;
    constexpr int CPP = CK / 8, KSTEPS = CK / 16, MY_STEPS = KSTEPS / KG;
    static_assert(KSTEPS % KG == 0, "every K group needs whole steps");
    static_assert(NI % 2 == 0 || NJ % 2 == 0, "the K groups exchange halves of the wave tile");
    // the epilogue's view: POS * 2 waves with half-size tiles (the K groups split the wave tile along the
    // dimension with an even number of 32-blocks, rows first)
    constexpr bool SPLIT_ROWS = NI % 2 == 0;
    constexpr int HI = SPLIT_ROWS ? NI / 2 : NI, HJ = SPLIT_ROWS ? NJ : NJ / 2;
    constexpr int EWM = SPLIT_ROWS ? WM / 2 : WM, EWN = SPLIT_ROWS ? WN : WN / 2;
    constexpr int ENWR = TM / EWM;
    using P = PatchLayout<CK, STRIDE, PL, THREADS>;
    using BRows = AsyncRows<DT, TN, CK, THREADS>;
    constexpr int LB = BRows::NL;
    constexpr int B_BYTES = TN * CK * 2;
    using M = Mma<DT, MF>;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const uint32_t lds0 = lds_address(smem);
    // layout: patch buffer 0, patch buffer 1, then the ring of filter tiles
    constexpr int RING0 = 2 * P::BYTES;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int pos = wave % POS, kgroup = wave / POS;
    const TileCoord tc = decode_tile(g.map, (int32_t)blockIdx.x);
    // position (wr, wc), half h -> row block wr * 2 + h (or column block wc * 2 + h) of the epilogue
    const int ewave = SPLIT_ROWS ? ((pos % NWR) * 2 + kgroup) + ENWR * (pos / NWR) : (pos % NWR) + ENWR * ((pos / NWR) * 2 + kgroup);
    const BiasRegs<DT> bias = load_bias_early<DT, TM, EWM, EWN, MF>(g, tc, ewave, lane);
    const int nst = g.stages - 2;                      // ring depth: 3 or 4
    const int slice0 = tc.k0 / (TAPS * CK);            // first channel slice of this split
    const int n_slices = tc.k_ext / (TAPS * CK);

    const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(g.a, g.a_bytes);
    const __amdgpu_buffer_rsrc_t b_rsrc = make_rsrc(g.b, g.b_bytes);

    // ---- filters: rows of the [N][9 * C] matrix, CK columns of tap t and slice s at column (t * C + s * CK) ----
    // Their first tiles are requested before anything else, so that the address arithmetic of the patch
    // below runs while they are on their way.
    typename BRows::State b_rows;
    BRows::init(b_rows, g.K, tc.n0, g.N, tid);
    const int k_total = g.K;
    auto request_filters = [&](int slice, int tap, int stage) {
        const bool live = slice < slice0 + n_slices;
        BRows::issue(b_rows, b_rsrc, lds0 + (uint32_t)(RING0 + stage * B_BYTES), tap * g.C + slice * CK, live ? k_total : 0, wave);
    };
    {
        int s = slice0, t = 0;
        for (int r = 0; r < nst - 1; ++r) {
            request_filters(s, t, r);
            if (++t == TAPS) t = 0, ++s;
        }
    }

    // ---- patch addressing: what each of this thread's PL items fetches (the same for every slice) ----
    const int PW = g.PW, PHW = g.PHW;
    const int key_rows = (g.H + 2 * g.pad_h) / STRIDE + 1;
    struct Pix {
        int base, key; // flat padded index of tap (0, 0) / swizzle key of tap (0, 0)
    };
    auto pixel_of = [&](int m) {
        const uint32_t um = (uint32_t)m;
        const uint32_t img = fast_div(um, g.div_hw);
        const uint32_t rem = um - img * (uint32_t)(g.Ho * g.Wo);
        const uint32_t p = fast_div(rem, g.div_wo), q = rem - p * (uint32_t)g.Wo;
        Pix x;
        x.base = (int)img * PHW + (int)p * STRIDE * PW + (int)q * STRIDE;
        x.key = ((int)img * key_rows + (int)p) * g.Wo + (int)q; // (p * STRIDE + r) / STRIDE = p + r / STRIDE
        return x;
    };
    const int pp_lo = pixel_of(tc.m0).base;
    const int last_m = min(tc.m0 + TM, g.M) - 1;
    const int np = pixel_of(last_m).base + 2 * PW + 2 - pp_lo + 1; // patch pixels of this tile
    // one piece = one item per thread; pieces 0 .. PL-1 of a slice are requested at taps 0 .. PL-1 of the
    // slice before it, those of the first slice here, each as soon as its address is known
    uint32_t patch_at[PL];
    auto request_patch_piece = [&](int l, int slice, int buffer) {
        const bool live = slice < slice0 + n_slices;
        load16_to_lds(a_rsrc, live && patch_at[l] != kOutOfRange ? patch_at[l] + (uint32_t)(slice * CK * 2) : kOutOfRange,
                      lds0 + (uint32_t)(buffer * P::BYTES + (l * THREADS + wave * 64) * 16));
    };
#pragma unroll
    for (int l = 0; l < PL; ++l) {
        const int item = l * THREADS + tid;
        const int slot = item % CPP, upix = item / CPP;
        const int phase = upix / P::PLANE, u = upix % P::PLANE;
        const int j = u * STRIDE + phase;
        const uint32_t pp = (uint32_t)(pp_lo + j);
        const uint32_t img = fast_div(pp, g.div_phw);
        const uint32_t rem = pp - img * (uint32_t)PHW;
        const uint32_t ph = fast_div(rem, g.div_pw), pw = rem - ph * (uint32_t)PW;
        const int c = slot ^ chunk_swizzle<CPP>(P::key((int)img, (int)ph, (int)pw, key_rows, g.Wo));
        const int ih = (int)ph - g.pad_h, iw = (int)pw - g.pad_w;
        const bool real = j < np && ih >= 0 && ih < g.H && iw >= 0 && iw < g.W;
        patch_at[l] = real ? (uint32_t)(((((int)img * g.H + ih) * g.W + iw) * g.C + c * 8) * 2) : kOutOfRange;
        request_patch_piece(l, slice0, 0);
    }

    ResRegs<DT, TM, EWM, EWN, MF, false> res_early; // (a long reduction: the residuals are fetched in the epilogue)

    // ---- this lane's rows of the patch (per 32-row block of the wave tile) ----
    const int wr = pos % NWR, wc = pos / NWR;
    const int lane_r = lane % MF, lane_g = lane / MF;
    Pix px[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        px[i] = pixel_of(min(tc.m0 + wr * WM + i * MF + lane_r, g.M - 1));
        px[i].base -= pp_lo;
    }
    const int b_row = (wc * WN + lane_r) * (CK * 2);
    const int b_swz = chunk_swizzle<CPP>(lane_r);

    typename M::Acc acc[NI][NJ];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int v = 0; v < ACC; ++v) acc[i][j][v] = 0.0f;

    // ---- LDS addresses of this lane's fragments ----
    // A: byte offset inside a patch buffer of (tap, 32-row block, K step), computed in the iteration
    // before the tap's (a dozen integer operations that run beside the other wave's matrix products);
    // B: inside a filter tile of (K step), the same for every tap.
    uint32_t b_addr[MY_STEPS];
#pragma unroll
    for (int s = 0; s < MY_STEPS; ++s) b_addr[s] = (uint32_t)(b_row + ((((s * KG + kgroup) * 2 + lane_g)) ^ b_swz) * 16);
    const int my_chunk0 = kgroup * 2 + lane_g; // chunk of this lane's first K step; step s adds 2 * KG * s

    struct Frags {
        u32x4 a[MY_STEPS][NI], b[MY_STEPS][NJ];
    };
    // fragments of tap `tap` from patch buffer `pbuf` (a constant) and ring buffer `slot`
    auto read_frags = [&](Frags &f, auto tap_c, auto pbuf_c, int slot) {
        constexpr int tap = decltype(tap_c)::value, pbuf = decltype(pbuf_c)::value;
        const unsigned char *pa = smem + pbuf * P::BYTES, *pb = smem + RING0 + slot * B_BYTES;
        uint32_t a_pos[NI];
        int a_swz[NI];
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int j = px[i].base + (tap / 3) * PW + (tap % 3);
            const int u = j / STRIDE, phase = j % STRIDE;
            a_pos[i] = (uint32_t)((phase * P::PLANE + u) * (CPP * 16));
            a_swz[i] = chunk_swizzle<CPP>(px[i].key + ((tap / 3) / STRIDE) * g.Wo + (tap % 3) / STRIDE);
        }
#pragma unroll
        for (int s = 0; s < MY_STEPS; ++s) {
#pragma unroll
            for (int i = 0; i < NI; ++i) f.a[s][i] = *reinterpret_cast<const u32x4 *>(pa + a_pos[i] + ((((my_chunk0 + 2 * KG * s)) ^ a_swz[i]) * 16));
#pragma unroll
            for (int j = 0; j < NJ; ++j) f.b[s][j] = *reinterpret_cast<const u32x4 *>(pb + b_addr[s] + j * MF * (CK * 2));
        }
    };
    auto multiply = [&](const Frags &f) {
#pragma unroll
        for (int s = 0; s < MY_STEPS; ++s)
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j) M::run(acc[i][j], f.a[s][i], f.b[s][j]);
    };

    // ---- software pipeline ----
    // Iteration g (tap g mod 9 of slice g / 9) multiplies the fragments it finds in registers and, before
    // that, reads the fragments of iteration g + 1 from LDS and requests the loads of later iterations:
    // a wave's LDS reads and global requests are in flight while its matrix products run.
    //   requests of iteration g: piece `tap` of the NEXT slice's patch (taps below PL), and the filter
    //   tile of iteration g + nst - 1 into the ring buffer of iteration g - 1 (whose fragments every wave
    //   had in registers before it passed this iteration's barrier);
    //   before the reads of iteration g + 1: wait until its filter tile, requested at iteration
    //   g + 2 - nst, has landed (only the nst - 3 request groups after it may be in flight), and a barrier.
    // Every iteration requests the same number of loads (past the end they are out-of-range requests
    // that deposit zeros where nothing reads), so the waits are constants of the tap.
    static_assert(PL <= TAPS - 2, "the last patch piece must land before the next slice's first fragments are read");
    const int total = n_slices * TAPS;
    int fill = nst - 1; // ring buffer the next request fills (iteration g: the buffer of iteration g - 1)
    int next = 1;       // ring buffer of iteration g + 1
    Frags f0, f1;       // fragments of even / odd iterations
    // the first fragments: the first slice's patch was requested last, so everything has to land
    wait_loads_outstanding<0>();
    __syncthreads();
    read_frags(f0, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, 0);

    auto slice_body = [&](auto parity_c, int sl) {
        constexpr int parity = decltype(parity_c)::value; // of the slice index: patch buffer, and which fragment set holds tap 0
        const int slice = slice0 + sl;
        static_for<0, TAPS>([&](auto tap_c) {
            constexpr int tap = decltype(tap_c)::value;
            constexpr bool even = (parity * TAPS + tap) % 2 == 0; // iteration index g = 9 sl + tap
            const int g = sl * TAPS + tap;
            if (nst == 4)
                wait_loads_outstanding<patch_younger_loads(tap, 3, LB, PL, TAPS)>();
            else
                wait_loads_outstanding<0>();
            __syncthreads();
            if (g + 1 < total) {
                constexpr int ntap = (tap + 1) % TAPS, nbuf = tap + 1 == TAPS ? 1 - parity : parity;
                if constexpr (even)
                    read_frags(f1, std::integral_constant<int, ntap>{}, std::integral_constant<int, nbuf>{}, next);
                else
                    read_frags(f0, std::integral_constant<int, ntap>{}, std::integral_constant<int, nbuf>{}, next);
            }
            __builtin_amdgcn_sched_barrier(0); // the reads go out before the requests' address arithmetic
            if constexpr (tap < PL) request_patch_piece(tap, slice + 1, 1 - parity);
            {
                int t2 = tap + nst - 1, s2 = slice;
                if (t2 >= TAPS) t2 -= TAPS, ++s2;
                request_filters(s2, t2, fill);
            }
            fill = fill + 1 == nst ? 0 : fill + 1;
            next = next + 1 == nst ? 0 : next + 1;
            if constexpr (even)
                multiply(f0);
            else
                multiply(f1);
        });
    };
    for (int sl = 0; sl < n_slices; sl += 2) {
        slice_body(std::integral_constant<int, 0>{}, sl);
        if (sl + 1 < n_slices) slice_body(std::integral_constant<int, 1>{}, sl + 1);
    }
    wait_loads_outstanding<0>(); // the out-of-range tail requests: nothing may still write LDS below
    __syncthreads();

    // ---- the two K groups of a position add their halves: each wave keeps one half of the wave tile ----
    float *xchg = reinterpret_cast<float *>(smem) + (size_t)wave * (HI * HJ * ACC * 64);
    // (register arrays must be indexed by constants: one copy of the code per K group)
    auto give = [&](auto half_c) { // store the half `half` of the wave tile
        constexpr int half = decltype(half_c)::value;
#pragma unroll
        for (int i = 0; i < HI; ++i)
#pragma unroll
            for (int j = 0; j < HJ; ++j) {
                constexpr int oi = SPLIT_ROWS ? half * HI : 0, oj = SPLIT_ROWS ? 0 : half * HJ;
#pragma unroll
                for (int v4 = 0; v4 < ACC / 4; ++v4)
                    *reinterpret_cast<f32x4 *>(xchg + ((size_t)((i * HJ + j) * (ACC / 4) + v4) * 64 + lane) * 4) =
                        f32x4{acc[oi + i][oj + j][4 * v4], acc[oi + i][oj + j][4 * v4 + 1], acc[oi + i][oj + j][4 * v4 + 2],
                              acc[oi + i][oj + j][4 * v4 + 3]};
            }
    };
    if (kgroup == 0)
        give(std::integral_constant<int, 1>{}); // group 0 keeps half 0
    else
        give(std::integral_constant<int, 0>{});
    __syncthreads();
    typename M::Acc mine[HI][HJ];
    const int partner = kgroup == 0 ? wave + POS : wave - POS;
    const float *from = reinterpret_cast<const float *>(smem) + (size_t)partner * (HI * HJ * ACC * 64);
    auto take = [&](auto half_c) { // add the partner's copy of the half this wave keeps
        constexpr int half = decltype(half_c)::value;
#pragma unroll
        for (int i = 0; i < HI; ++i)
#pragma unroll
            for (int j = 0; j < HJ; ++j) {
                constexpr int oi = SPLIT_ROWS ? half * HI : 0, oj = SPLIT_ROWS ? 0 : half * HJ;
#pragma unroll
                for (int v4 = 0; v4 < ACC / 4; ++v4) {
                    const f32x4 o = *reinterpret_cast<const f32x4 *>(from + ((size_t)((i * HJ + j) * (ACC / 4) + v4) * 64 + lane) * 4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) mine[i][j][4 * v4 + e] = acc[oi + i][oj + j][4 * v4 + e] + o[e];
                }
            }
    };
    if (kgroup == 0)
        take(std::integral_constant<int, 0>{});
    else
        take(std::integral_constant<int, 1>{});
    write_tile<DT, TM, EWM, EWN, MF>(mine, g, tc, smem, ewave, lane, bias, res_early);
}

// LDS bytes: two patch buffers and the filter ring; never less than the exchange of the K groups (the whole
// tile in fp32) or the epilogue's staging (one band of 32 rows per wave).
template <int TM, int TN, int CK, int WM, int WN, int STRIDE, int PL> struct PatchKernelLds {
    static constexpr int THREADS = (TM / WM) * (TN / WN) * 128;
    using P = PatchLayout<CK, STRIDE, PL, THREADS>;
    static constexpr int XCHG = TM * TN * 4;
    static constexpr int EWN = (WM / 32) % 2 == 0 ? WN : WN / 2;
    static constexpr int EPI = (THREADS / 64) * 32 * (EWN + 8) * 4;
    static constexpr int bytes(int stages)
    {
        const int run = 2 * P::BYTES + (stages - 2) * TN * CK * 2;
        const int tail = XCHG > EPI ? XCHG : EPI;
        return run > tail ? run : tail;
    }
};

template <int TM, int TN, int CK, int WM, int WN, int STRIDE, int PL>
int launch_conv_patch(const ContractArgs &args, int grid, int lds_bytes, void *stream)
{
    auto kern = conv3x3_patch_kernel<TM, TN, CK, WM, WN, STRIDE, PL>;
    using L = PatchKernelLds<TM, TN, CK, WM, WN, STRIDE, PL>;
    if (lds_bytes < L::bytes(args.stages)) lds_bytes = L::bytes(args.stages);
    static DynamicLdsLimit limit; // per kernel instance
    if (const int rc = limit.raise_to(reinterpret_cast<const void *>(kern), lds_bytes); rc != TT_OK) return rc;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(L::THREADS), lds_bytes, static_cast<hipStream_t>(stream), args);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : note_hip_error((int)e, "conv3x3_patch_kernel launch");
}

// capacity of a patch buffer in pixels, and LDS bytes for a record's `stages` (5 or 6)
template <int TM, int TN, int CK, int WM, int WN, int STRIDE, int PL> int capacity_conv_patch()
{
    return PatchLayout<CK, STRIDE, PL, (TM / WM) * (TN / WN) * 128>::PIXELS;
}
template <int TM, int TN, int CK, int WM, int WN, int STRIDE, int PL> int lds_bytes_conv_patch(int stages)
{
    return PatchKernelLds<TM, TN, CK, WM, WN, STRIDE, PL>::bytes(stages);
}

} // namespace tt
