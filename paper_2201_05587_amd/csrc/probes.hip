// Hardware-rate probes: what this GPU gives a plain kernel, measured the way the operators are timed
// (HIP events on the caller's stream around back-to-back launches).  They put a kernel's roofline
// fraction next to the rate a kernel of the simplest kind reaches on the same machine; no operator
// uses them.
#include "tt_internal.h"

#include <hip/hip_runtime.h>

namespace tt {
namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

__global__ void probe_empty_kernel() {}

// 16 bytes per thread and step, grid-stride: every load and store instruction of a wave covers 1 KB.
__global__ void __launch_bounds__(256) probe_copy_linear_kernel(const u32x4 *src, u32x4 *dst, size_t items)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < items; i += stride)
        __builtin_nontemporal_store(src[i], dst + i);
}

// The same bytes seen as a row-major matrix of 512-byte rows and walked the way the contraction kernels'
// epilogues walk an output: a workgroup owns 64 rows x 128 bytes, a lane a 16-byte piece of a row, the four
// waves 16 rows each.
__global__ void __launch_bounds__(256) probe_copy_tiled_kernel(const u32x4 *src, u32x4 *dst, int rows)
{
    constexpr int ROW_ITEMS = 32, TILE_ITEMS = 8, TILE_ROWS = 64;
    const int tiles_n = ROW_ITEMS / TILE_ITEMS;
    const int tm = blockIdx.x / tiles_n, tn = blockIdx.x % tiles_n;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int col = tn * TILE_ITEMS + lane % TILE_ITEMS;
    u32x4 v[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int m = tm * TILE_ROWS + wave * 16 + p * 8 + lane / TILE_ITEMS;
        v[p] = m < rows ? src[(size_t)m * ROW_ITEMS + col] : u32x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int m = tm * TILE_ROWS + wave * 16 + p * 8 + lane / TILE_ITEMS;
        if (m < rows) __builtin_nontemporal_store(v[p], dst + (size_t)m * ROW_ITEMS + col);
    }
}

// Four independent accumulators per wave, 16 products of 32x32x16 per iteration: nothing but the matrix pipe.
__global__ void __launch_bounds__(256) probe_mfma_kernel(float *out, int iters)
{
    f32x16 acc[4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][v] = 0.0f;
    const u32x4 af = {threadIdx.x, 1u, 2u, 3u}, bf = {4u, 5u, 6u, threadIdx.x};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int a = 0; a < 4; ++a)
                acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af),
                                                                 __builtin_bit_cast(bf16x8, bf), acc[a], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int a = 0; a < 4; ++a) s += acc[a][0];
    if (s == 123.456f) out[threadIdx.x] = s; // keeps the products alive; never true for these operands
}

// Every workgroup pulls `span` bytes of a small source (one that stays in the L2) into registers, eight
// 16-byte loads in flight per lane: the rate at which a CU can be fed from the L2.
__global__ void __launch_bounds__(256) probe_l2_read_kernel(const unsigned char *src, uint32_t bytes, uint32_t span,
                                                            uint32_t *out)
{
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(src), 0, bytes,
                                                                          0x00020000);
    uint32_t off = (blockIdx.x * 65536u + threadIdx.x * 16u) % bytes;
    const uint32_t step = 256u * 16u;
    u32x4 acc = {0, 0, 0, 0};
    for (uint32_t done = 0; done < span; done += step * 8) {
        u32x4 v[8];
#pragma unroll
        for (int l = 0; l < 8; ++l) {
            v[l] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 0);
            off += step;
            if (off >= bytes) off -= bytes;
        }
#pragma unroll
        for (int l = 0; l < 8; ++l) acc ^= v[l];
    }
    if (acc[0] == 0x12345678u && acc[1] == 0x9abcdef0u) out[threadIdx.x] = acc[2];
}

// Microseconds per repetition of `launch`, after one untimed repetition.
template <typename F> int time_us(hipStream_t s, int reps, F launch, double *us)
{
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
        return note_hip_error((int)hipGetLastError(), "probe: hipEventCreate");
    launch();
    hipError_t e = hipEventRecord(e0, s);
    for (int r = 0; r < reps; ++r) launch();
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.0f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) return note_hip_error((int)e, "probe");
    *us = (double)ms * 1e3 / reps;
    return TT_OK;
}

} // namespace
} // namespace tt

using namespace tt;

extern "C" int tt_debug_probe(int which, const void *src, void *dst, size_t bytes, int reps, void *stream, double *result)
{
    if (!result || reps < 1 || reps > 100000) return TT_ERR_BAD_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    double us = 0.0;
    switch (which) {
    case TT_PROBE_LAUNCH_GAP_US: {
        const int rc = time_us(s, reps, [&] { hipLaunchKernelGGL(probe_empty_kernel, dim3(1), dim3(64), 0, s); }, &us);
        if (rc != TT_OK) return rc;
        *result = us;
        return TT_OK;
    }
    case TT_PROBE_MFMA_BF16_TFLOPS: {
        if (!dst || bytes < 256 * sizeof(float)) return TT_ERR_BAD_ARG;
        const int iters = 256, grid = 256 * 4; // four waves per workgroup, four workgroups per CU
        const int rc = time_us(
            s, reps, [&] { hipLaunchKernelGGL(probe_mfma_kernel, dim3(grid), dim3(256), 0, s, static_cast<float *>(dst), iters); },
            &us);
        if (rc != TT_OK) return rc;
        *result = (double)grid * 4 * iters * 16 * (2.0 * 32 * 32 * 16) / us / 1e6;
        return TT_OK;
    }
    case TT_PROBE_COPY_LINEAR_GBPS:
    case TT_PROBE_COPY_TILED_GBPS: {
        // read + write bytes per second over buffers the caller sizes (beyond the caches for a cold figure)
        if (!src || !dst || bytes < 32768 || bytes % 32768 || bytes > ((size_t)1 << 40)) return TT_ERR_BAD_ARG;
        if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) return TT_ERR_BAD_ARG;
        const size_t items = bytes / 16;
        const int rows = (int)(bytes / 512);
        if (bytes / 512 > (size_t)INT32_MAX / 4) return TT_ERR_BAD_ARG;
        int rc;
        if (which == TT_PROBE_COPY_LINEAR_GBPS)
            rc = time_us(
                s, reps,
                [&] {
                    hipLaunchKernelGGL(probe_copy_linear_kernel, dim3(8192), dim3(256), 0, s, static_cast<const u32x4 *>(src),
                                       static_cast<u32x4 *>(dst), items);
                },
                &us);
        else
            rc = time_us(
                s, reps,
                [&] {
                    hipLaunchKernelGGL(probe_copy_tiled_kernel, dim3((unsigned)((rows + 63) / 64 * 4)), dim3(256), 0, s,
                                       static_cast<const u32x4 *>(src), static_cast<u32x4 *>(dst), rows);
                },
                &us);
        if (rc != TT_OK) return rc;
        *result = 2.0 * (double)bytes / us / 1e3;
        return TT_OK;
    }
    case TT_PROBE_L2_READ_GBPS: {
        if (!src || !dst || bytes < (1u << 20) || bytes > (2u << 20) || (reinterpret_cast<uintptr_t>(src) & 15))
            return TT_ERR_BAD_ARG;
        const uint32_t span = 4u << 20; // per workgroup
        const int grid = 256 * 4;
        const int rc = time_us(
            s, reps,
            [&] {
                hipLaunchKernelGGL(probe_l2_read_kernel, dim3(grid), dim3(256), 0, s, static_cast<const unsigned char *>(src),
                                   (uint32_t)bytes, span, static_cast<uint32_t *>(dst));
            },
            &us);
        if (rc != TT_OK) return rc;
        *result = (double)grid * span / us / 1e3;
        return TT_OK;
    }
    default: return TT_ERR_BAD_ARG;
    }
}
