// Measured ceilings of the machine, for the benchmark only: what fraction of a kernel's nominal
// roofline is reachable at all on this chip at this problem size.  Neither kernel is part of the
// method; both are plain textbook probes.
//
//  - paro_diag_read_stream: every lane reads 16 bytes per step, non-temporal, grid-stride, four
//    independent loads in flight per lane; nothing is written.  The time of this launch on N bytes
//    is the floor of any kernel that must read N bytes from HBM once.
//  - paro_diag_mfma_f16: every wave issues `iters` x 16 independent v_mfma_f32_32x32x16_f16 on
//    register operands (no memory traffic): the matrix-pipe rate the chip sustains, with constant
//    operands or with random ones (random operands draw more power and clock lower).
#include "paro_internal.h"

namespace paro {

typedef uint32_t u32x4c __attribute__((ext_vector_type(4)));
typedef _Float16 half8c __attribute__((ext_vector_type(8)));
typedef float float16c __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void read_stream_kernel(const u32x4c *__restrict__ src, size_t n16, uint32_t *sink)
{
    constexpr int U = 4;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    u32x4c acc = {0, 0, 0, 0};
    for (; i + (U - 1) * stride < n16; i += U * stride) {
        u32x4c v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u];
    }
    for (; i < n16; i += stride) acc ^= __builtin_nontemporal_load(src + i);
    const uint32_t r = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    if (r == 0x12345678u && sink) *sink = r;      // keeps the loads alive; practically never taken
}

__global__ __launch_bounds__(256) void mfma_f16_kernel(float *out, int iters, int random_operands)
{
    half8c a = {1, 1, 1, 1, 1, 1, 1, 1}, b = {1, 0, 1, 0, 1, 0, 1, 0};
    a[0] = (_Float16)(threadIdx.x & 3);
    if (random_operands) {
        uint32_t h = threadIdx.x * 2654435761u + blockIdx.x * 40503u;
        for (int e = 0; e < 8; ++e) {
            h = h * 1664525u + 1013904223u; a[e] = (_Float16)((int)(h >> 20) % 2000 / 500.0f - 2.0f);
            h = h * 1664525u + 1013904223u; b[e] = (_Float16)((int)(h >> 20) % 2000 / 50000.0f - 0.02f);
        }
    }
    float16c acc[16];
    for (int i = 0; i < 16; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[i], 0, 0, 0);
    float s = 0;
    for (int i = 0; i < 16; ++i) s += acc[i][0];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// The block-scaled FP4 instruction of the MXFP4 linear, on register operands: 32 independent 16x16x128 MFMAs per
// iteration and wave (as many accumulators as one K-step of that kernel's wave tile).
typedef int v8ic __attribute__((ext_vector_type(8)));
typedef float float4c __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(512) void mfma_fp4_kernel(float *out, int iters, int random_operands)
{
    v8ic a = {0x22222222, 0x22222222, 0x22222222, 0x22222222, 0, 0, 0, 0}, b = a;      // all 1.0
    int sa = 127, sb = 127;
    if (random_operands) {
        uint32_t h = threadIdx.x * 2654435761u + blockIdx.x * 40503u;
        for (int e = 0; e < 4; ++e) {
            h = h * 1664525u + 1013904223u; a[e] = (int)(h ^ (h >> 13));
            h = h * 1664525u + 1013904223u; b[e] = (int)(h ^ (h >> 11));
        }
        sa = 120 + (int)(h & 7); sb = 118 + (int)((h >> 8) & 7);
    }
    float4c acc[32];
    for (int i = 0; i < 32; ++i) acc[i] = float4c{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int i = 0; i < 32; ++i) acc[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, acc[i], 4, 4, 0, sa, 0, sb);
    float s = 0;
    for (int i = 0; i < 32; ++i) s += acc[i][0];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace paro

extern "C" {

paro_status paro_diag_read_stream(const void *src, size_t bytes, void *sink, int32_t blocks, void *stream)
{
    if (!src) return PARO_ERR_NULL;
    if (bytes < 16 || blocks < 1 || blocks > 65536) return PARO_ERR_SHAPE;
    if ((uintptr_t)src % 16 || (uintptr_t)sink % 4) return PARO_ERR_ALIGN;
    hipLaunchKernelGGL(paro::read_stream_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                       (const paro::u32x4c *)src, bytes / 16, (uint32_t *)sink);
    return hipGetLastError() == hipSuccess ? PARO_OK : PARO_ERR_HIP;
}

double paro_diag_mfma_f16_flops(int32_t blocks, int32_t iters)
{
    // 4 waves per block, 16 MFMAs per iteration, 2 * 32 * 32 * 16 flop each
    return (double)blocks * 4.0 * (double)iters * 16.0 * 32768.0;
}

paro_status paro_diag_mfma_f16(void *out, size_t out_bytes, int32_t blocks, int32_t iters, int32_t random_operands,
                               void *stream)
{
    if (!out) return PARO_ERR_NULL;
    if (blocks < 1 || blocks > 65536 || iters < 1 || out_bytes < (size_t)blocks * 256 * sizeof(float)) return PARO_ERR_SHAPE;
    if ((uintptr_t)out % 4) return PARO_ERR_ALIGN;
    hipLaunchKernelGGL(paro::mfma_f16_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (float *)out, iters,
                       random_operands);
    return hipGetLastError() == hipSuccess ? PARO_OK : PARO_ERR_HIP;
}

double paro_diag_mfma_fp4_flops(int32_t blocks, int32_t iters)
{
    // 8 waves per block, 32 MFMAs per iteration, 2 * 16 * 16 * 128 flop each
    return (double)blocks * 8.0 * (double)iters * 32.0 * 65536.0;
}

paro_status paro_diag_mfma_fp4(void *out, size_t out_bytes, int32_t blocks, int32_t iters, int32_t random_operands,
                               void *stream)
{
    if (!out) return PARO_ERR_NULL;
    if (blocks < 1 || blocks > 65536 || iters < 1 || out_bytes < (size_t)blocks * 512 * sizeof(float)) return PARO_ERR_SHAPE;
    if ((uintptr_t)out % 4) return PARO_ERR_ALIGN;
    hipLaunchKernelGGL(paro::mfma_fp4_kernel, dim3(blocks), dim3(512), 0, (hipStream_t)stream, (float *)out, iters,
                       random_operands);
    return hipGetLastError() == hipSuccess ? PARO_OK : PARO_ERR_HIP;
}

}  // extern "C"
