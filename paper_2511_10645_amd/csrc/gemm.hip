// Prefill-side W4A16 linear: Y[T x N] = X'[T x C] . W^[N x C]^T for many tokens (Eq. 2), the one
// dense contraction of the path, on fp16 MFMA with fp32 accumulation.
//
// Block tile 256 (tokens) x 256 (outputs) x 64 (channels), 4 wavefronts as 2 x 2, each wave a
// 128 x 128 sub-tile = 4 x 4 v_mfma_f32_32x32x16_f16 tiles (256 accumulator registers).
// Per K-step a block fetches 32 KB of activations and 8 KB of packed INT4 codes; the codes are
// dequantised ONCE per block into an fp16 LDS tile
//      w^ = fp16( (q - z) * s )        ((q - z) exact in fp16, one rounding in the multiply:
//                                        the same value paro_w4_dequant produces)
// so the VALU cost per weight is amortised over the 256 token rows.  LDS is double-buffered
// (2 x (36 + 36) KB): global loads for step s+1 are issued before the MFMAs of step s and
// land in LDS after them, one barrier per K-step.  Rows are padded by 16 bytes so that the
// 16-byte fragment reads of 32 consecutive rows spread over all banks.
//
// Blocks are numbered so that the 32 blocks resident on one XCD (block id mod 8) form an
// 8 (token tiles) x 4 (output tiles) patch that walks K in step: they share activation and
// weight panels through that XCD's L2.
#include "paro_internal.h"

namespace paro {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kLdsRow = kBK + 8;                    // halfs per padded LDS row
constexpr int kGemmThreads = 256;
constexpr int kPatchM = 8, kPatchN = 4;             // blocks of one XCD patch

constexpr uint32_t kOobG = 0x80000000u;
__device__ inline __amdgpu_buffer_rsrc_t make_rsrc_g(const void *p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}
__device__ inline half2v g_as_h2(uint32_t u) { union { uint32_t u; half2v h; } c; c.u = u; return c.h; }
__device__ inline uint32_t g_as_u32(half2v h) { union { uint32_t u; half2v h; } c; c.h = h; return c.u; }

struct GemmArgs {
    const void *blob; uint32_t blob_bytes, scales_off, zeros_off;
    const _Float16 *X; int64_t ldx;
    _Float16 *Y; int64_t ldy;
    const _Float16 *bias;
    int T, C, N, G, S;          // S = G / 4 K-slices of the scales/zeros tiling
    int m_tiles, n_tiles;
};

struct BStage {       // packed codes and parameters of one K-step for this thread
    u32x4 w[2];
    uint32_t sc[2];   // fp16 scale (low half)
    uint32_t zq[2];   // 4 zero nibbles of the slice
};

__global__ __launch_bounds__(kGemmThreads) void gemm_w4a16_kernel(GemmArgs a)
{
    extern __shared__ __attribute__((aligned(16))) _Float16 smem[];
    _Float16 *As = smem;                                   // [2][kBM][kLdsRow]
    _Float16 *Bs = smem + 2 * kBM * kLdsRow;               // [2][kBN][kLdsRow]

    // ---- block -> (m tile, n tile), XCD-aware --------------------------------------------------
    const int bid = blockIdx.x;
    const int xcd = bid & 7, j = bid >> 3;
    const int patch = j / (kPatchM * kPatchN), q = j % (kPatchM * kPatchN);
    const int m_patches = (a.m_tiles + kPatchM - 1) / kPatchM;
    const int gp = patch * 8 + xcd;                        // global patch index
    const int pm = gp % m_patches, pn = gp / m_patches;
    const int mt = pm * kPatchM + q % kPatchM, ntile = pn * kPatchN + q / kPatchM;
    if (mt >= a.m_tiles || ntile >= a.n_tiles) return;
    const int m0 = mt * kBM, n0 = ntile * kBN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    const __amdgpu_buffer_rsrc_t xr = make_rsrc_g(a.X, (uint32_t)(((size_t)(a.T - 1) * a.ldx + a.C) * 2));
    const __amdgpu_buffer_rsrc_t br = make_rsrc_g(a.blob, a.blob_bytes);

    // per-thread load coordinates
    // A: 8 x 16 B per thread: idx = tid + 256 p -> row idx/8, 16-byte column idx%8
    // B: 2 x 16 B per thread: idx = tid + 256 p -> 16-row tile idx/32, lane-in-half idx%32
    const int a_c16 = tid & 7, a_row = tid >> 3;           // + 32 p rows
    const int b_l32 = tid & 31, b_rt = tid >> 5;           // + 8 p row tiles
    const int b_n = b_l32 & 15, b_kq = b_l32 >> 4;         // row in tile, 32-channel quarter within the half

    u32x4 areg[8];
    BStage bst;
    auto load_global = [&](int ks) {
        const int k0 = ks * kBK;
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int row = m0 + a_row + 32 * p;
            const uint32_t off = row < a.T ? (uint32_t)(((size_t)row * a.ldx + k0 + a_c16 * 8) * 2) : kOobG;
            areg[p] = __builtin_amdgcn_raw_buffer_load_b128(xr, (int)off, 0, 0);
        }
        const int g = k0 / kGroup, half = (k0 / kBK) & 1;
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int nt = n0 / kTileN + b_rt + 8 * p;                  // 16-row tile of the weight
            const bool ok = nt * kTileN < a.N;
            const int ln = (half * 2 + b_kq) * 16 + b_n;                 // lane inside the 1 KB tile
            const uint32_t off = ok ? (((uint32_t)nt * a.G + g) * 64u + ln) * 16u : kOobG;
            bst.w[p] = __builtin_amdgcn_raw_buffer_load_b128(br, (int)off, 0, 0);
            const uint32_t sidx = ((uint32_t)nt * a.S + g / kSliceGroups) * kTileN + b_n;
            bst.sc[p] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(
                br, ok ? (int)(a.scales_off + (sidx * 4u + (g % kSliceGroups)) * 2u) : (int)kOobG, 0, 0);
            bst.zq[p] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(
                br, ok ? (int)(a.zeros_off + sidx * 2u) : (int)kOobG, 0, 0);
        }
    };
    auto store_lds = [&](int buf, int ks) {
        _Float16 *Ab = As + (size_t)buf * kBM * kLdsRow, *Bb = Bs + (size_t)buf * kBN * kLdsRow;
#pragma unroll
        for (int p = 0; p < 8; ++p) *(u32x4 *)&Ab[(a_row + 32 * p) * kLdsRow + a_c16 * 8] = areg[p];
        const int g = (ks * kBK) / kGroup;
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const uint32_t z = (bst.zq[p] >> (4 * (g % kSliceGroups))) & 15u;
            const half2v nlo = g_as_h2((0xE400u + z) * 0x00010001u);          // -(1024 + z), twice
            const half2v nhi = g_as_h2((0xD400u + (z << 4)) * 0x00010001u);   // -(64 + z), twice
            const half2v s2 = g_as_h2(bst.sc[p] * 0x00010001u);
            _Float16 *dst = &Bb[((b_rt + 8 * p) * kTileN + b_n) * kLdsRow + b_kq * 32];
#pragma unroll
            for (int w4 = 0; w4 < 4; ++w4) {
                uint32_t u = bst.w[p][w4];
                u32x4 o;
                o[0] = g_as_u32((g_as_h2((u & 0x000F000Fu) | 0x64006400u) + nlo) * s2);
                o[1] = g_as_u32((g_as_h2((u & 0x00F000F0u) | 0x54005400u) + nhi) * s2);
                u >>= 8;
                o[2] = g_as_u32((g_as_h2((u & 0x000F000Fu) | 0x64006400u) + nlo) * s2);
                o[3] = g_as_u32((g_as_h2((u & 0x00F000F0u) | 0x54005400u) + nhi) * s2);
                *(u32x4 *)&dst[w4 * 8] = o;
            }
        }
    };

    float16v acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jn = 0; jn < 4; ++jn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jn][v] = 0.f;

    const int n_ks = a.C / kBK;
    load_global(0);
    store_lds(0, 0);
    __syncthreads();

    const int fr = lane & 31, fh = lane >> 5;
    for (int ks = 0; ks < n_ks; ++ks) {
        const int buf = ks & 1;
        if (ks + 1 < n_ks) load_global(ks + 1);
        const _Float16 *Ab = As + (size_t)buf * kBM * kLdsRow + (wm * 128 + fr) * kLdsRow + fh * 8;
        const _Float16 *Bb = Bs + (size_t)buf * kBN * kLdsRow + (wn * 128 + fr) * kLdsRow + fh * 8;
#pragma unroll
        for (int kk = 0; kk < kBK / 16; ++kk) {
            half8 af[4], bf[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) af[i] = *(const half8 *)&Ab[i * 32 * kLdsRow + kk * 16];
#pragma unroll
            for (int jn = 0; jn < 4; ++jn) bf[jn] = *(const half8 *)&Bb[jn * 32 * kLdsRow + kk * 16];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jn = 0; jn < 4; ++jn)
                    acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[jn], acc[i][jn], 0, 0, 0);
        }
        if (ks + 1 < n_ks) store_lds(buf ^ 1, ks + 1);
        __syncthreads();
    }

    // ---- epilogue: + bias, fp16 store.  Lane (column fr, half fh) holds rows 8b + 4 fh + r. ------
    const __amdgpu_buffer_rsrc_t yr = make_rsrc_g(a.Y, (uint32_t)(((size_t)(a.T - 1) * a.ldy + a.N) * 2));
#pragma unroll
    for (int jn = 0; jn < 4; ++jn) {
        const int n = n0 + wn * 128 + jn * 32 + fr;
        const float bv = (a.bias && n < a.N) ? (float)a.bias[n] : 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * 128 + i * 32 + (v >> 2) * 8 + fh * 4 + (v & 3);
                union { _Float16 h; uint16_t u; } o; o.h = (_Float16)(acc[i][jn][v] + bv);
                const uint32_t off = (m < a.T && n < a.N) ? (uint32_t)(((size_t)m * a.ldy + n) * 2) : kOobG;
                __builtin_amdgcn_raw_buffer_store_b16(o.u, yr, (int)off, 0, 0);
            }
    }
}

bool gemm_supported(const paro_w4_weight &w, int64_t ldx, int64_t ldy, int T)
{
    size_t blob = packed_tiles_bytes(w.c_in, w.c_out) + packed_scales_bytes(w.c_in, w.c_out) +
                  packed_zeros_bytes(w.c_in, w.c_out);
    return blob < (1ull << 31) && ((size_t)T * ldx) * 2 < (1ull << 31) && ((size_t)T * ldy) * 2 < (1ull << 31) &&
           w.c_in % kBK == 0;
}

hipError_t launch_gemm(const paro_w4_weight &w, const paro_half_t *X, int64_t ldx, paro_half_t *Y, int64_t ldy, int T,
                       hipStream_t s)
{
    GemmArgs a;
    a.blob = w.packed;
    a.scales_off = (uint32_t)packed_tiles_bytes(w.c_in, w.c_out);
    a.zeros_off = a.scales_off + (uint32_t)packed_scales_bytes(w.c_in, w.c_out);
    a.blob_bytes = a.zeros_off + (uint32_t)packed_zeros_bytes(w.c_in, w.c_out);
    a.X = (const _Float16 *)X; a.ldx = ldx; a.Y = (_Float16 *)Y; a.ldy = ldy;
    a.bias = (const _Float16 *)w.bias;
    a.T = T; a.C = w.c_in; a.N = w.c_out; a.G = w.c_in / kGroup; a.S = a.G / kSliceGroups;
    a.m_tiles = (T + kBM - 1) / kBM; a.n_tiles = (w.c_out + kBN - 1) / kBN;
    const int m_patches = (a.m_tiles + kPatchM - 1) / kPatchM, n_patches = (a.n_tiles + kPatchN - 1) / kPatchN;
    const int patches = m_patches * n_patches;
    const int rounds = (patches + 7) / 8;                 // patches per XCD
    const int blocks = rounds * 8 * kPatchM * kPatchN;
    const size_t lds = (size_t)2 * (kBM + kBN) * kLdsRow * sizeof(_Float16);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_w4a16_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(gemm_w4a16_kernel, dim3(blocks), dim3(kGemmThreads), lds, s, a);
    return hipGetLastError();
}

}  // namespace paro
