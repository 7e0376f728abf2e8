// INT4 weight layouts: repack into the streamed tile layout, and the bit-exact test hooks
// (unpack codes / zero points, dequantise to fp16).  Dequantisation is Eq. 1 read backwards
// with one (s, z) per 128 input channels of an output column (Section 2.1):
//      w^ = (q - z) * s
#include "paro_internal.h"

namespace paro {

// move code e (nibble e of `w`) to nibble packed_nibble_pos(e)
__device__ inline uint32_t permute_nibbles_fwd(uint32_t w)
{
    uint32_t r = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) r |= ((w >> (4 * e)) & 15u) << (4 * packed_nibble_pos(e));
    return r;
}
__device__ inline uint32_t permute_nibbles_inv(uint32_t w)
{
    uint32_t r = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) r |= ((w >> (4 * packed_nibble_pos(e))) & 15u) << (4 * e);
    return r;
}

// One thread per 32-bit word of the tile section.
__global__ void repack_tiles_kernel(const uint32_t *__restrict__ qweight, int C, int N, uint32_t *__restrict__ tiles)
{
    const int G = C / kGroup;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)(N / kTileN) * G * 256;
    if (idx >= total) return;
    int j = idx & 3;
    int lane = (idx >> 2) & 63;
    size_t tg = idx >> 8;
    int g = (int)(tg % G);
    size_t nt = tg / G;
    int n = lane & 15, kb = lane >> 4;
    size_t row = nt * kTileN + n;
    uint32_t w = qweight[row * (C / 8) + (size_t)g * 16 + kb * 4 + j];
    tiles[idx] = permute_nibbles_fwd(w);
}

// One thread per (nt, slice, n): 4 scales and 4 zero nibbles.
__global__ void repack_params_kernel(const _Float16 *__restrict__ scales, const uint32_t *__restrict__ qzeros, int C,
                                     int N, _Float16 *__restrict__ pscales, uint16_t *__restrict__ pzeros)
{
    const int G = C / kGroup, S = G / kSliceGroups;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)(N / kTileN) * S * kTileN;
    if (idx >= total) return;
    int n = idx & 15;
    size_t ts = idx >> 4;
    int s = (int)(ts % S);
    size_t nt = ts / S;
    size_t row = nt * kTileN + n;
    uint32_t zz = 0;
#pragma unroll
    for (int gi = 0; gi < kSliceGroups; ++gi) {
        int g = s * kSliceGroups + gi;
        pscales[idx * kSliceGroups + gi] = scales[(size_t)g * N + row];
        uint32_t z = (qzeros[(size_t)g * (N / 8) + row / 8] >> (4 * (row % 8))) & 15u;
        zz |= z << (4 * gi);
    }
    pzeros[idx] = (uint16_t)zz;
}

hipError_t launch_repack(const paro_w4_weight &w, void *packed_out, hipStream_t s)
{
    PackedView v = packed_view(packed_out, w.c_in, w.c_out);
    size_t words = packed_tiles_bytes(w.c_in, w.c_out) / 4;
    hipLaunchKernelGGL(repack_tiles_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, s, w.qweight, w.c_in,
                       w.c_out, (uint32_t *)v.tiles);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    size_t items = (size_t)(w.c_out / kTileN) * (w.c_in / kGroup / kSliceGroups) * kTileN;
    hipLaunchKernelGGL(repack_params_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, s,
                       (const _Float16 *)w.scales, w.qzeros, w.c_in, w.c_out, (_Float16 *)v.scales,
                       (uint16_t *)v.zeros);
    return hipGetLastError();
}

// ---- hooks ---------------------------------------------------------------------------------

// word (n, wi) of the logical [N][C/8] matrix, in interchange nibble order, from either layout
__device__ inline uint32_t logical_word(const uint32_t *qweight, const uint32_t *tiles, int C, size_t n, int wi)
{
    if (tiles == nullptr) return qweight[n * (C / 8) + wi];
    const int G = C / kGroup;
    int g = wi >> 4, kb = (wi >> 2) & 3, j = wi & 3;
    size_t nt = n / kTileN;
    int lane = kb * 16 + (int)(n % kTileN);
    return permute_nibbles_inv(tiles[((nt * G + g) * 64 + lane) * 4 + j]);
}

__device__ inline int logical_zero(const uint32_t *qzeros, const PackedView &pv, bool packed, int C, int N, int g,
                                   size_t n)
{
    if (!packed) return (int)((qzeros[(size_t)g * (N / 8) + n / 8] >> (4 * (n % 8))) & 15u);
    const int S = C / kGroup / kSliceGroups;
    size_t idx = ((n / kTileN) * S + g / kSliceGroups) * kTileN + n % kTileN;
    return (pv.zeros[idx] >> (4 * (g % kSliceGroups))) & 15;
}

__device__ inline float logical_scale(const _Float16 *scales, const PackedView &pv, bool packed, int C, int N, int g,
                                      size_t n)
{
    if (!packed) return (float)scales[(size_t)g * N + n];
    const int S = C / kGroup / kSliceGroups;
    size_t idx = ((n / kTileN) * S + g / kSliceGroups) * kTileN + n % kTileN;
    return (float)((const _Float16 *)pv.scales)[idx * kSliceGroups + (g % kSliceGroups)];
}

__global__ void unpack_codes_kernel(const uint32_t *__restrict__ qweight, const uint32_t *__restrict__ tiles, int C,
                                    int N, uint8_t *__restrict__ codes)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)N * (C / 8);
    if (idx >= total) return;
    size_t n = idx / (C / 8);
    int wi = (int)(idx % (C / 8));
    uint32_t w = logical_word(qweight, tiles, C, n, wi);
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        lo |= ((w >> (4 * e)) & 15u) << (8 * e);
        hi |= ((w >> (4 * (e + 4))) & 15u) << (8 * e);
    }
    ((uint2 *)codes)[idx] = make_uint2(lo, hi);
}

__global__ void unpack_zeros_kernel(const uint32_t *__restrict__ qzeros, PackedView pv, bool packed, int C, int N,
                                    uint8_t *__restrict__ zeros)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int G = C / kGroup;
    if (idx >= (size_t)G * N) return;
    int g = (int)(idx / N);
    size_t n = idx % N;
    zeros[idx] = (uint8_t)logical_zero(qzeros, pv, packed, C, N, g, n);
}

__global__ void dequant_kernel(const uint32_t *__restrict__ qweight, const _Float16 *__restrict__ scales,
                               const uint32_t *__restrict__ qzeros, PackedView pv, bool packed, int C, int N,
                               _Float16 *__restrict__ W)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)N * (C / 8);
    if (idx >= total) return;
    size_t n = idx / (C / 8);
    int wi = (int)(idx % (C / 8));
    uint32_t w = logical_word(qweight, packed ? (const uint32_t *)pv.tiles : nullptr, C, n, wi);
    const float s = logical_scale(scales, pv, packed, C, N, wi / 16, n);
    const int z = logical_zero(qzeros, pv, packed, C, N, wi / 16, n);
    union { _Float16 h[8]; uint4 v; } o;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        int q = (int)((w >> (4 * e)) & 15u);
        // (q - z) is an integer of magnitude <= 15 and s has an 11-bit significand: the fp32
        // product is exact, so the fp16 conversion is the only rounding (nearest-even)
        o.h[e] = (_Float16)((float)(q - z) * s);
    }
    ((uint4 *)W)[idx] = o.v;
}

hipError_t launch_unpack_codes(const paro_w4_weight &w, uint8_t *codes, hipStream_t s)
{
    size_t total = (size_t)w.c_out * (w.c_in / 8);
    const uint32_t *tiles = w.packed ? (const uint32_t *)packed_view(w.packed, w.c_in, w.c_out).tiles : nullptr;
    hipLaunchKernelGGL(unpack_codes_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, w.qweight, tiles,
                       w.c_in, w.c_out, codes);
    return hipGetLastError();
}

hipError_t launch_unpack_zeros(const paro_w4_weight &w, uint8_t *zeros, hipStream_t s)
{
    size_t total = (size_t)(w.c_in / kGroup) * w.c_out;
    PackedView pv = packed_view(w.packed, w.c_in, w.c_out);
    hipLaunchKernelGGL(unpack_zeros_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, w.qzeros, pv,
                       w.packed != nullptr, w.c_in, w.c_out, zeros);
    return hipGetLastError();
}

hipError_t launch_dequant(const paro_w4_weight &w, paro_half_t *W, hipStream_t s)
{
    size_t total = (size_t)w.c_out * (w.c_in / 8);
    PackedView pv = packed_view(w.packed, w.c_in, w.c_out);
    hipLaunchKernelGGL(dequant_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, w.qweight,
                       (const _Float16 *)w.scales, w.qzeros, pv, w.packed != nullptr, w.c_in, w.c_out, (_Float16 *)W);
    return hipGetLastError();
}

}  // namespace paro
