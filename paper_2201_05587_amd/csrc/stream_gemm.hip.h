// Persistent contraction for short reductions: out[M][N] = act(A[M][K] . B[N][K]^T + bias + residual).
//
// Where K is a few slices long, a workgroup of the tile kernels spends its life in prologue and epilogue:
// the operands' memory latency, then the residuals' and the stores, one tile per workgroup.  Here a
// workgroup keeps the whole [TN][K] panel of B in LDS and walks down the M axis: the A rows of the next
// tile are requested (asynchronously, into the other of two LDS buffers) before the current tile is
// multiplied and written, so their latency runs under the epilogue of the tile before, and neither B nor
// the set-up is repeated per tile.
#pragma once
#include "contract.hip.h"

#include <algorithm>

namespace tt {

// LDS: B panel (k_tiles slices of TN rows), two A buffers (k_tiles slices of TM rows each), epilogue staging.
template <int DT, int TM, int TN, int TK, int WM, int WN, int MF> struct StreamLayout {
    using RL = RingLayout<DT, TM, TN, TK>;
    static constexpr int RB = RL::RB;
    static constexpr int WAVES = (TM / WM) * (TN / WN);
    static constexpr int EPI_BYTES = WAVES * MF * TileOut<TM, WM, WN, MF>::ESTRIDE * 4;
    static constexpr int bytes(int k_tiles) { return k_tiles * (TN + 2 * TM) * RB + EPI_BYTES; }
};

template <int DT, int TM, int TN, int TK, int WM, int WN, int MF>
__global__ void __launch_bounds__((TM / WM) * (TN / WN) * 64) gemm_stream_kernel(const ContractArgs g)
{
    using E = typename ElemOf<DT>::type;
    constexpr int CH = ElemOf<DT>::CH, ES = (int)sizeof(E);
    constexpr int THREADS = (TM / WM) * (TN / WN) * 64;
    using SL = StreamLayout<DT, TM, TN, TK, WM, WN, MF>;
    constexpr int RB = SL::RB, CPR = TK / CH;
    constexpr int NWR = TM / WM;
    constexpr int NI = WM / MF, NJ = WN / MF;
    constexpr int LG = 64 / MF, KS = CH * LG, NKS = TK / KS;
    constexpr int ACC = MF * MF / 64;
    using M = Mma<DT, MF>;
    using ARows = AsyncRows<DT, TM, TK, THREADS>;
    using BRows = AsyncRows<DT, TN, TK, THREADS>;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int kt_count = g.map.k_tiles; // K is a whole number of slices (the host checks)
    const int b_bytes = kt_count * TN * RB, a_bytes = kt_count * TM * RB;
    unsigned char *const lds_b = smem, *const lds_a = smem + b_bytes, *const lds_stage = lds_a + 2 * a_bytes;
    const uint32_t lds_b0 = lds_address(lds_b), lds_a0 = lds_address(lds_a);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // workgroup -> (panel of B, first tile and stride along M); the grid is a multiple of the panel count
    const int panels = g.map.tiles_n;
    const int panel = (int)blockIdx.x % panels, first = (int)blockIdx.x / panels, per = (int)gridDim.x / panels;
    TileCoord tc;
    tc.hi = 0, tc.lo = 0;
    tc.n0 = panel * TN, tc.n_ext = min(TN, g.N - tc.n0);
    tc.k0 = 0, tc.k_ext = g.K;
    tc.m0 = first * TM, tc.m_ext = min(TM, g.M - tc.m0);

    const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(g.a, (uint32_t)(g.M * g.K * ES));
    const __amdgpu_buffer_rsrc_t b_rsrc = make_rsrc(g.b, (uint32_t)(g.N * g.K * ES));
    typename ARows::State a_rows;
    typename BRows::State b_rows;
    BRows::init(b_rows, g.K, tc.n0, g.N, tid);
    for (int kt = 0; kt < kt_count; ++kt) BRows::issue(b_rows, b_rsrc, lds_b0 + (uint32_t)(kt * TN * RB), kt * TK, g.K, wave);
    auto request_a = [&](int tile_m, int buf) {
        ARows::init(a_rows, g.K, tile_m * TM, g.M, tid); // rows past the matrix (and tiles past the end) read as zeros
        for (int kt = 0; kt < kt_count; ++kt)
            ARows::issue(a_rows, a_rsrc, lds_a0 + (uint32_t)(buf * a_bytes + kt * TM * RB), kt * TK, g.K, wave);
    };
    request_a(first, 0);
    const BiasRegs<DT> bias = load_bias_early<DT, TM, WM, WN, MF>(g, tc, wave, lane);

    const int wr = wave % NWR, wc = wave / NWR;
    const int lane_r = lane % MF, lane_g = lane / MF;
    const int swz = chunk_swizzle<CPR>(lane_r);
    const int a_row = (wr * WM + lane_r) * RB, b_row = (wc * WN + lane_r) * RB;

    int buf = 0;
    for (int tile_m = first; tile_m < g.map.tiles_m; tile_m += per, buf ^= 1) {
        tc.m0 = tile_m * TM, tc.m_ext = min(TM, g.M - tc.m0);
        // This wave's pieces of the tile (and, the first time, of the B panel) have landed: the epilogue
        // of the tile before waited for them.  The barrier makes that true of every wave's pieces, and says
        // that every wave is done multiplying the tile before, whose buffer the next request overwrites.
        wait_loads_outstanding<0>();
        __syncthreads();
        request_a(tile_m + per, buf ^ 1);
        ResRegs<DT, TM, WM, WN, MF, true> res_early;
        load_res_early(res_early, g, tc, wave, lane);

        typename M::Acc acc[NI][NJ];
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int v = 0; v < ACC; ++v) acc[i][j][v] = 0.0f;
        for (int kt = 0; kt < kt_count; ++kt) {
            const unsigned char *sa = lds_a + buf * a_bytes + kt * TM * RB, *sb = lds_b + kt * TN * RB;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
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
            }
        }
        // the staging region is this kernel's own; the requests of the next tile are waited for inside,
        // before the first store (stores issued after a request would hide it from the counter)
        write_tile<DT, TM, WM, WN, MF, typename M::Acc, true, true>(acc, g, tc, lds_stage, wave, lane, bias, res_early);
    }
}

// Compute units of the current device (asked once; one device per process).
inline int compute_units()
{
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
            n = 256;
        return n;
    }();
    return cus;
}

// `tiles` is the plan's grid (one entry per output tile); the launch itself is persistent: as many
// workgroups as fit the chip (at most four per CU, as the LDS allows), a whole number per panel of B.
template <int DT, int TM, int TN, int TK, int WM, int WN, int MF>
int launch_gemm_stream(const ContractArgs &args, int tiles, int lds_bytes, void *stream)
{
    auto kern = gemm_stream_kernel<DT, TM, TN, TK, WM, WN, MF>;
    (void)tiles;
    if (args.batch != 1 || args.map.eff_split_k != 1 || args.K % TK || args.map.k_tiles != args.K / TK || lds_bytes <= 0 ||
        lds_bytes > 160 * 1024)
        return TT_ERR_UNSUPPORTED;
    static DynamicLdsLimit limit; // per kernel instance
    if (const int rc = limit.raise_to(reinterpret_cast<const void *>(kern), lds_bytes); rc != TT_OK) return rc;
    constexpr int THREADS = (TM / WM) * (TN / WN) * 64;
    const int fit = std::min(4, 160 * 1024 / lds_bytes);
    const int per = std::max(1, std::min(args.map.tiles_m, compute_units() * fit / args.map.tiles_n));
    hipLaunchKernelGGL(kern, dim3(per * args.map.tiles_n), dim3(THREADS), lds_bytes, static_cast<hipStream_t>(stream), args);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : note_hip_error((int)e, "gemm_stream_kernel launch");
}

// What the host's resource check needs: request instructions per lane and K slice (both operands; the
// vector-memory counter holds 63), and the LDS bytes for a reduction of k_tiles slices.
template <int DT, int TM, int TN, int TK, int WM, int WN, int MF> int requests_gemm_stream()
{
    constexpr int THREADS = (TM / WM) * (TN / WN) * 64;
    return AsyncRows<DT, TM, TK, THREADS>::NL + AsyncRows<DT, TN, TK, THREADS>::NL;
}
template <int DT, int TM, int TN, int TK, int WM, int WN, int MF> int lds_bytes_gemm_stream(int k_tiles)
{
    return StreamLayout<DT, TM, TN, TK, WM, WN, MF>::bytes(k_tiles);
}

} // namespace tt
