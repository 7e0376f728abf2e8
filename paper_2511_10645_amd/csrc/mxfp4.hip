// Weight-activation form of the linear layer with both operands in MXFP4 (App. A.3, first equation):
//      Y' = Q(X T^-1) . Q(T W) + b
// on the block-scaled FP4 matrix instruction of this chip, which takes E2M1 codes and one E8M0 scale per
// 32 elements of each operand directly: nothing is dequantised, the codes go from memory to the matrix
// core as they are and the products are accumulated in fp32.
//
// v_mfma_scale_f32_16x16x128_f8f6f4 (FP4 x FP4): lane l of the A operand holds row l % 16, elements
// 32 (l / 16) .. + 31 of the 128-wide K-step as 16 bytes (element k in nibble k % 8 of dword k / 8), and
// ONE scale byte for those 32 elements - an MX block is exactly a lane's share; B likewise with column
// l % 16; D as for the other 16x16 shapes (lane: column l % 16, rows 4 (l / 16) + r).  The scale operand
// is a dword of which an immediate picks the byte, so one register serves four K-steps.
//
// Weights are repacked once into that operand order ("tiles" of 16 rows x 128 channels = 1 KB, then
// per 16 rows x 512 channels one dword per lane with the four K-steps' scale bytes), so a wave's load of
// a tile is one contiguous kilobyte.  Activations stay in the plain row order their quantiser writes:
// a lane's 32 elements are 16 contiguous bytes of its token's row.
//
// Two kernels.  Up to 16 tokens: HBM-bound stream of the weight tiles (0.53 B per weight), one
// 512-channel slice per wave and pass, all slices of K inside one block (a wave takes SPW slices when
// there are more than 12), partial tiles summed through LDS; no exchange between blocks.  More tokens:
// a tiled GEMM whose operands go through LDS (see below).
#include "paro_internal.h"
#include <type_traits>

namespace paro {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

constexpr uint32_t kOobM = 0x80000000u;
__device__ inline __amdgpu_buffer_rsrc_t mx_rsrc(const void *p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}
__device__ inline v8i as_operand(u32x4 v) { return v8i{(int)v[0], (int)v[1], (int)v[2], (int)v[3], 0, 0, 0, 0}; }

template <int N, class F, int I = 0>
__device__ __forceinline__ void mx_static_while(F &&f)
{
    if constexpr (I < N) {
        if (f(std::integral_constant<int, I>{})) mx_static_while<N, F, I + 1>(static_cast<F &&>(f));
    }
}

// ------------------------------------------------------------------------------------------
// Layout: plain [N][C/8] words + [N][C/32] bytes  <->  blob = tiles | scale dwords
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void mxfp4_repack_kernel(const uint32_t *__restrict__ codes,
                                                           const uint8_t *__restrict__ scales, int N, int C,
                                                           u32x4 *__restrict__ tiles, uint32_t *__restrict__ sdw)
{
    const int K128 = C / 128, KS = C / 512;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t n_tiles16 = (size_t)(N / 16) * K128 * 64;
    if (idx < n_tiles16) {
        const int lane = (int)(idx & 63);
        const size_t tk = idx >> 6;
        const int k128 = (int)(tk % K128);
        const size_t nt = tk / K128;
        const size_t row = nt * 16 + (lane & 15);
        tiles[idx] = *(const u32x4 *)(codes + row * (C / 8) + (size_t)k128 * 16 + (lane >> 4) * 4);
    }
    const size_t n_sdw = (size_t)(N / 16) * KS * 64;
    if (idx < n_sdw) {
        const int lane = (int)(idx & 63);
        const size_t ts = idx >> 6;
        const int ks = (int)(ts % KS);
        const size_t nt = ts / KS;
        const uint8_t *sr = scales + (nt * 16 + (lane & 15)) * (size_t)(C / 32) + (size_t)ks * 16 + (lane >> 4);
        sdw[idx] = (uint32_t)sr[0] | ((uint32_t)sr[4] << 8) | ((uint32_t)sr[8] << 16) | ((uint32_t)sr[12] << 24);
    }
}

// one thread per (row, 32-channel block): 32 code bytes and the scale byte, from either layout
__global__ __launch_bounds__(256) void mxfp4_unpack_kernel(const uint32_t *__restrict__ codes,
                                                           const uint8_t *__restrict__ scales,
                                                           const u32x4 *__restrict__ tiles,
                                                           const uint32_t *__restrict__ sdw, int N, int C,
                                                           uint8_t *__restrict__ out_codes, uint8_t *__restrict__ out_scales)
{
    const int B = C / 32;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)N * B) return;
    const size_t row = idx / B;
    const int b = (int)(idx % B);
    u32x4 v;
    uint32_t sc;
    if (tiles) {
        const int lane = (int)(row & 15) + 16 * (b & 3);
        v = tiles[((row / 16) * (C / 128) + b / 4) * 64 + lane];
        sc = (sdw[((row / 16) * (C / 512) + b / 16) * 64 + lane] >> (8 * ((b / 4) & 3))) & 0xffu;
    } else {
        v = *(const u32x4 *)(codes + row * (C / 8) + (size_t)b * 4);
        sc = scales[row * B + b];
    }
    uint8_t *o = out_codes + row * C + (size_t)b * 32;
#pragma unroll
    for (int j = 0; j < 32; ++j) o[j] = (uint8_t)((v[j / 8] >> (4 * (j % 8))) & 15u);
    out_scales[idx] = (uint8_t)sc;
}

hipError_t launch_mxfp4_repack(const paro_mxfp4_weight &w, void *packed_out, hipStream_t s)
{
    const size_t n = (size_t)w.c_out * w.c_in / 32;                   // 16-byte chunks of codes
    hipLaunchKernelGGL(mxfp4_repack_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, w.codes, w.scales,
                       w.c_out, w.c_in, (u32x4 *)packed_out,
                       (uint32_t *)((char *)packed_out + (size_t)w.c_out * w.c_in / 2));
    return hipGetLastError();
}

hipError_t launch_mxfp4_unpack(const paro_mxfp4_weight &w, uint8_t *codes, uint8_t *scales, hipStream_t s)
{
    const size_t n = (size_t)w.c_out * w.c_in / 32;
    const u32x4 *tiles = (const u32x4 *)w.packed;
    const uint32_t *sdw = w.packed ? (const uint32_t *)((const char *)w.packed + (size_t)w.c_out * w.c_in / 2) : nullptr;
    hipLaunchKernelGGL(mxfp4_unpack_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, w.codes, w.scales, tiles,
                       sdw, w.c_out, w.c_in, codes, scales);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Up to 16 tokens
// ------------------------------------------------------------------------------------------
struct MxArgs {
    const void *blob; uint32_t blob_bytes, scales_off;
    const uint32_t *xc; const uint8_t *xs;          // activations of this pass: [T][C/8] words, [T][C/32] bytes
    _Float16 *Y; int64_t ldy;
    const _Float16 *bias;
    int T, C, N, NT, KS, tiles_per_block;
};

constexpr int kMxStages = 3;
constexpr int kMxMaxUnits = 16;                      // (tile, slice) units per wave: the stream is unrolled
constexpr int kMxMaxWaves = 12;                      // 3 waves per SIMD: 170 registers each

struct MxStage { u32x4 w[4]; uint32_t sc; };

// SPW: 512-channel slices per wave (wave w takes slices w, w + waves, ...).  TB: blocks of 16 tokens per wave
// (the weight tile of a unit is multiplied with each; the 4 MFMAs per token block are a small part of a unit's
// time, so up to 64 tokens cost little more than 16).  SPW * TB sets of activation fragments live in registers:
// up to 5 with 12 waves per block, up to 8 with 8.
template <int SPW, int TB>
__global__ __launch_bounds__((SPW * TB <= 5 ? kMxMaxWaves : 8) * 64) void mxfp4_decode_kernel(MxArgs a)
{
    constexpr int NS = kMxStages;
    extern __shared__ __attribute__((aligned(16))) float s_part[];       // [tiles per block][waves][TB][256]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw = blockDim.x >> 6;
    const int tile_lo = blockIdx.x * a.tiles_per_block;
    const int tile_hi = min(a.NT, tile_lo + a.tiles_per_block);
    const int n_iter = tile_hi - tile_lo;
    const int K128 = a.C / 128;
    const __amdgpu_buffer_rsrc_t blob = mx_rsrc(a.blob, a.blob_bytes);

    // ---- activations of the wave's slices as A operands: lane = (token l % 16 of its block, 32-channel block l / 16) ----
    const int ft = lane & 15, fkb = lane >> 4;
    u32x4 xf[SPW][TB][4];
    uint32_t xsc[SPW][TB];
    {
        const __amdgpu_buffer_rsrc_t xr = mx_rsrc(a.xc, (uint32_t)((size_t)a.T * a.C / 2));
        const __amdgpu_buffer_rsrc_t sr = mx_rsrc(a.xs, (uint32_t)((size_t)a.T * a.C / 32));
#pragma unroll
        for (int q = 0; q < SPW; ++q)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                const int ks = wave + q * nw, t = tb * 16 + ft;
                const bool ok = ks < a.KS && t < a.T;
                const uint32_t xo = ok ? (uint32_t)((size_t)t * (a.C / 2) + (size_t)ks * 256 + fkb * 16) : kOobM;
#pragma unroll
                for (int m = 0; m < 4; ++m) xf[q][tb][m] = __builtin_amdgcn_raw_buffer_load_b128(xr, (int)(xo + m * 64), 0, 0);
                // the slice's 16 scale bytes: dword m = K-step m, byte kb = the lane's block
                const u32x4 sc = __builtin_amdgcn_raw_buffer_load_b128(sr, ok ? (int)((size_t)t * (a.C / 32) + (size_t)ks * 16) : (int)kOobM, 0, 0);
                const int sh = 8 * fkb;
                xsc[q][tb] = ((sc[0] >> sh) & 0xffu) | (((sc[1] >> sh) & 0xffu) << 8) | (((sc[2] >> sh) & 0xffu) << 16) |
                             (((sc[3] >> sh) & 0xffu) << 24);
            }
    }
    // unit i = (tile tile_lo + i / SPW, slice wave + (i % SPW) waves); nothing to load beyond the range: zeros
    MxStage st[NS];
    auto load_unit = [&](int i, MxStage &s) {
        const int ti = i / SPW, ks = wave + (i % SPW) * nw;
        const bool ok = ti < n_iter && ks < a.KS;
        const uint32_t tile = (uint32_t)(tile_lo + ti);
        const uint32_t off = ok ? ((tile * K128 + ks * 4) * 64u + lane) * 16u : kOobM;
#pragma unroll
        for (int m = 0; m < 4; ++m) s.w[m] = __builtin_amdgcn_raw_buffer_load_b128(blob, (int)(off + m * 1024u), 0, 2);
        s.sc = __builtin_amdgcn_raw_buffer_load_b32(blob, ok ? (int)(a.scales_off + ((tile * a.KS + ks) * 64u + lane) * 4u) : (int)kOobM, 0, 0);
    };
#pragma unroll
    for (int i = 0; i + 1 < NS; ++i) load_unit(i, st[i]);

    float4v acc[TB];
    mx_static_while<kMxMaxUnits>([&](auto I) {
        constexpr int i = I;
        constexpr int q = i % SPW;
        if (i / SPW >= n_iter) return false;
        load_unit(i + NS - 1, st[(i + NS - 1) % NS]);
        const MxStage &s = st[i % NS];
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            if constexpr (q == 0) acc[tb] = float4v{0.f, 0.f, 0.f, 0.f};
            acc[tb] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(as_operand(xf[q][tb][0]), as_operand(s.w[0]), acc[tb], 4, 4, 0, (int)xsc[q][tb], 0, (int)s.sc);
            acc[tb] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(as_operand(xf[q][tb][1]), as_operand(s.w[1]), acc[tb], 4, 4, 1, (int)xsc[q][tb], 1, (int)s.sc);
            acc[tb] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(as_operand(xf[q][tb][2]), as_operand(s.w[2]), acc[tb], 4, 4, 2, (int)xsc[q][tb], 2, (int)s.sc);
            acc[tb] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(as_operand(xf[q][tb][3]), as_operand(s.w[3]), acc[tb], 4, 4, 3, (int)xsc[q][tb], 3, (int)s.sc);
            if constexpr (q == SPW - 1) *(float4v *)(s_part + (((size_t)(i / SPW) * nw + wave) * TB + tb) * 256 + lane * 4) = acc[tb];
        }
        return true;
    });
    __syncthreads();
    // ---- sum the waves' partial tiles: element lane * 4 + r <-> token 4 (lane / 16) + r of its block, row lane % 16 ----
    const int per_tile = a.T * kTileN;
    for (int idx = threadIdx.x; idx < n_iter * per_tile; idx += blockDim.x) {
        const int i = idx / per_tile, rem = idx % per_tile;
        const int t = rem / kTileN, nn = rem % kTileN;
        const int e = (t >> 4) * 256 + (((t & 15) >> 2) * 16 + nn) * 4 + (t & 3);
        float sum = 0.f;
        for (int w = 0; w < nw; ++w) sum += s_part[((size_t)i * nw + w) * (TB * 256) + e];
        const size_t n = (size_t)(tile_lo + i) * kTileN + nn;
        if (a.bias) sum += (float)a.bias[n];
        a.Y[(size_t)t * a.ldy + n] = (_Float16)sum;
    }
}

// Geometry of a pass of T tokens: TB token blocks per wave, as many as the registers allow for this K.
struct MxGeometry { int spw, tb, waves, tiles_per_block, blocks; size_t lds; };
static bool mx_geometry(int c_in, int c_out, int T, MxGeometry &g)
{
    const int KS = c_in / 512, NT = c_out / kTileN;
    const int want = T > 32 ? 4 : T > 16 ? 2 : 1;
    g.tb = 0;
    for (int tb = want; tb >= 1 && !g.tb; tb >>= 1) {
        // sets of fragments = SPW * TB: up to 5 with 12 waves per block, up to 8 with 8 waves
        const int spw12 = (KS + kMxMaxWaves - 1) / kMxMaxWaves, spw8 = (KS + 7) / 8;
        if (spw12 * tb <= 5) { g.tb = tb; g.spw = spw12; }
        else if (spw8 * tb <= 8) { g.tb = tb; g.spw = spw8; }
    }
    if (!g.tb || g.spw > 5) return false;
    g.waves = (KS + g.spw - 1) / g.spw;
    int tpb = (NT + 255) / 256;                               // one block per compute unit
    if (tpb > kMxMaxUnits / g.spw) tpb = kMxMaxUnits / g.spw;
    if (tpb * g.waves * g.tb > 144) tpb = 144 / (g.waves * g.tb);   // TB KB of LDS per (tile, wave)
    if (tpb < 1) return false;
    g.tiles_per_block = tpb;
    g.blocks = (NT + tpb - 1) / tpb;
    g.lds = (size_t)tpb * g.waves * g.tb * 1024;
    return true;
}

bool mxfp4_linear_supported(const paro_mxfp4_weight &w)
{
    MxGeometry g;
    return w.packed && w.c_in % 512 == 0 && w.c_out % 16 == 0 && mx_geometry(w.c_in, w.c_out, 1, g) &&
           (size_t)w.c_out * w.c_in / 2 + (size_t)w.c_out * w.c_in / 32 < (1ull << 31);
}

// tokens one pass of the streaming kernel takes for this K (64, 32 or 16)
static int mxfp4_pass_tokens(const paro_mxfp4_weight &w, int T)
{
    MxGeometry g;
    return mx_geometry(w.c_in, w.c_out, T, g) ? 16 * g.tb : 16;
}

template <int SPW, int TB>
static hipError_t launch_mxfp4_decode_cfg(const MxArgs &a, const MxGeometry &g, hipStream_t s)
{
    static std::atomic<uint64_t> attr_done{0};
    if (const int dev = once_pending(attr_done); dev >= 0) {
        hipError_t e = hipFuncSetAttribute((const void *)mxfp4_decode_kernel<SPW, TB>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        once_done(attr_done, dev);
    }
    hipLaunchKernelGGL((mxfp4_decode_kernel<SPW, TB>), dim3(g.blocks), dim3(g.waves * 64), g.lds, s, a);
    return hipGetLastError();
}

// one pass of up to mxfp4_pass_tokens() tokens
static hipError_t launch_mxfp4_decode(const paro_mxfp4_weight &w, const uint32_t *xc, const uint8_t *xs, int T,
                                      paro_half_t *Y, int64_t ldy, hipStream_t s)
{
    MxGeometry g;
    if (!mx_geometry(w.c_in, w.c_out, T, g) || T > 16 * g.tb) return hipErrorInvalidValue;
    MxArgs a;
    a.blob = w.packed;
    a.scales_off = (uint32_t)((size_t)w.c_out * w.c_in / 2);
    a.blob_bytes = a.scales_off + (uint32_t)((size_t)w.c_out * w.c_in / 32);
    a.xc = xc; a.xs = xs; a.Y = (_Float16 *)Y; a.ldy = ldy; a.bias = (const _Float16 *)w.bias;
    a.T = T; a.C = w.c_in; a.N = w.c_out; a.NT = w.c_out / kTileN; a.KS = w.c_in / 512;
    a.tiles_per_block = g.tiles_per_block;
    switch (g.tb * 8 + g.spw) {
    case 1 * 8 + 1: return launch_mxfp4_decode_cfg<1, 1>(a, g, s);
    case 1 * 8 + 2: return launch_mxfp4_decode_cfg<2, 1>(a, g, s);
    case 1 * 8 + 3: return launch_mxfp4_decode_cfg<3, 1>(a, g, s);
    case 1 * 8 + 4: return launch_mxfp4_decode_cfg<4, 1>(a, g, s);
    case 1 * 8 + 5: return launch_mxfp4_decode_cfg<5, 1>(a, g, s);
    case 2 * 8 + 1: return launch_mxfp4_decode_cfg<1, 2>(a, g, s);
    case 2 * 8 + 2: return launch_mxfp4_decode_cfg<2, 2>(a, g, s);
    case 2 * 8 + 3: return launch_mxfp4_decode_cfg<3, 2>(a, g, s);
    case 2 * 8 + 4: return launch_mxfp4_decode_cfg<4, 2>(a, g, s);
    case 4 * 8 + 1: return launch_mxfp4_decode_cfg<1, 4>(a, g, s);
    case 4 * 8 + 2: return launch_mxfp4_decode_cfg<2, 4>(a, g, s);
    default: return hipErrorInvalidValue;
    }
}

// ------------------------------------------------------------------------------------------
// More than 16 tokens: tiled GEMM.  Block tile 256 (or 128, see the launcher) tokens x 256 outputs x 128 channels (one K-step of
// the matrix instruction: 64 bytes per row of either operand), 8 waves side by side along the outputs:
// wave tile 256 tokens x 32 outputs = 16 x 2 MFMA tiles of 16 x 16 (128 accumulator registers).
//   - Weights never touch LDS: the repacked blob IS the operand order, every 16-row tile of a K-step
//     is needed by exactly one wave, which fetches it straight into registers, 3 K-steps ahead.
//   - Activations (16 KB of codes + 1 KB of scale bytes per K-step) are shared by all 8 waves: fetched
//     into registers five K-steps ahead (2 x 16 B + 4 B per thread and stage), written two K-steps ahead
//     into a ring of three LDS tiles; one barrier per K-step.  LDS rows are 64
//     bytes; the 16-byte chunk index is XOR-ed with bits 1..2 of the row so that the 16-byte fragment
//     reads of 8 consecutive rows fall into 8 different bank groups.
// What bounds the loop is the data in flight per compute unit (measured: with a single K-step in
// flight a K-step takes 3 us, 7 x the time of its 32 MFMAs per wave), hence the deep register queues.
// Blocks are numbered in XCD patches as in the fp16 GEMM.
// ------------------------------------------------------------------------------------------
struct MxGemmArgs {
    const void *blob; uint32_t blob_bytes, scales_off;
    const uint32_t *xc; const uint8_t *xs;
    _Float16 *Y; int64_t ldy;
    const _Float16 *bias;
    int T, C, N, K128, KS;
    int m_tiles, n_tiles, n_tile0, patch_m, patch_n;     // the launch covers output tiles [n_tile0, n_tile0 + n_tiles)
};

constexpr int kMxBM = 256, kMxBN = 256;
constexpr int kMxRowBytes = 64;                          // one K-step of one row
constexpr int mx_stage_bytes(int bm) { return bm * kMxRowBytes + bm * 4; }   // codes | scale dwords (4 blocks per row)
constexpr int kMxChunk = 12;                             // K-steps written out in the loop body (24: no faster)

__device__ __forceinline__ int mx_lds_off(int row, int chunk) { return row * kMxRowBytes + ((chunk ^ ((row >> 1) & 3)) << 4); }

// BM: tokens per block tile, 256, or 128 where 256-token tiles would leave half of the compute units idle
template <int BM>
__global__ __launch_bounds__(512) void mxfp4_gemm_kernel(MxGemmArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char smem_mx[];          // [3][kStage]
    constexpr int kStage = mx_stage_bytes(BM);
    constexpr int MI = BM / 16;                                             // 16-row MFMA tiles of a wave
    const int bid = blockIdx.x;
    const int xcd = bid & 7, j = bid >> 3;
    const int pb = a.patch_m * a.patch_n;
    const int patch = j / pb, q = j % pb;
    const int m_patches = (a.m_tiles + a.patch_m - 1) / a.patch_m;
    const int gp = patch * 8 + xcd;
    const int pm = gp % m_patches, pn = gp / m_patches;
    const int mt = pm * a.patch_m + q % a.patch_m, ntile = pn * a.patch_n + q / a.patch_m;
    if (mt >= a.m_tiles || ntile >= a.n_tiles) return;
    const int m0 = mt * BM, n0 = (a.n_tile0 + ntile) * kMxBN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const __amdgpu_buffer_rsrc_t xr = mx_rsrc(a.xc, (uint32_t)((size_t)a.T * a.C / 2));
    const __amdgpu_buffer_rsrc_t sr = mx_rsrc(a.xs, (uint32_t)((size_t)a.T * a.C / 32));
    const __amdgpu_buffer_rsrc_t br = mx_rsrc(a.blob, a.blob_bytes);
    const int n_ks = a.K128;

    // ---- activations: thread -> chunks (row tid / 4 [+ 128], chunk tid % 4); threads 0..255 also the scale
    // dword of row tid.  Rows beyond T start beyond the end of their buffers: they read as zero. ----
    const uint32_t ga = (uint32_t)((size_t)(m0 + (tid >> 2)) * (a.C / 2) + (tid & 3) * 16);
    const uint32_t ga_step = (uint32_t)(128 * (a.C / 2));
    const int la0 = mx_lds_off(tid >> 2, tid & 3), la1 = mx_lds_off((tid >> 2) + 128, tid & 3);
    const uint32_t gs = tid < BM ? (uint32_t)((size_t)(m0 + tid) * (a.C / 32)) : kOobM;
    const int ls = BM * kMxRowBytes + (tid & (BM - 1)) * 4;
    struct AStage { u32x4 c0, c1; uint32_t sc; };
    auto load_a = [&](int ks, AStage &st) {
        const bool ok = ks < n_ks;
        st.c0 = __builtin_amdgcn_raw_buffer_load_b128(xr, ok ? (int)ga : (int)kOobM, ks * kMxRowBytes, 0);
        if constexpr (BM == 256) st.c1 = __builtin_amdgcn_raw_buffer_load_b128(xr, ok ? (int)(ga + ga_step) : (int)kOobM, ks * kMxRowBytes, 0);
        st.sc = __builtin_amdgcn_raw_buffer_load_b32(sr, ok ? (int)gs : (int)kOobM, ks * 4, 0);
    };
    auto store_a = [&](char *buf, const AStage &st) {
        *(u32x4 *)(buf + la0) = st.c0;
        if constexpr (BM == 256) *(u32x4 *)(buf + la1) = st.c1;
        if (tid < BM) *(uint32_t *)(buf + ls) = st.sc;
    };
    // ---- weights: the wave's two 16-row tiles, as they lie in the blob ----
    const int nt16 = n0 / 16 + wave * 2;
    const bool n_ok0 = nt16 * 16 < a.N, n_ok1 = (nt16 + 1) * 16 < a.N;
    const uint32_t gb0 = ((uint32_t)nt16 * a.K128 * 64u + lane) * 16u;
    const uint32_t gb_step = (uint32_t)a.K128 * 1024u;
    const uint32_t gw0 = a.scales_off + ((uint32_t)nt16 * a.KS * 64u + lane) * 4u;
    const uint32_t gw_step = (uint32_t)a.KS * 256u;
    struct BStage { u32x4 t0, t1; };
    auto load_b = [&](int ks, BStage &st) {
        const bool ok = ks < n_ks;
        st.t0 = __builtin_amdgcn_raw_buffer_load_b128(br, ok && n_ok0 ? (int)gb0 : (int)kOobM, ks * 1024, 0);
        st.t1 = __builtin_amdgcn_raw_buffer_load_b128(br, ok && n_ok1 ? (int)(gb0 + gb_step) : (int)kOobM, ks * 1024, 0);
    };
    uint32_t wq0 = 0, wq1 = 0, wq0_n, wq1_n;                 // scale dwords of the current / the next 512-channel slice
    auto load_wscales = [&](int slice, uint32_t &d0, uint32_t &d1) {
        const bool ok = slice < a.KS;
        d0 = __builtin_amdgcn_raw_buffer_load_b32(br, ok && n_ok0 ? (int)gw0 : (int)kOobM, slice * 256, 0);
        d1 = __builtin_amdgcn_raw_buffer_load_b32(br, ok && n_ok1 ? (int)(gw0 + gw_step) : (int)kOobM, slice * 256, 0);
    };

    float4v acc[MI][2];
#pragma unroll
    for (int i = 0; i < MI; ++i) { acc[i][0] = float4v{0.f, 0.f, 0.f, 0.f}; acc[i][1] = float4v{0.f, 0.f, 0.f, 0.f}; }

    // ---- prologue ----
    // LDS holds three K-steps of activations: step k is multiplied from buffer k % 3 while step k + 2 is written
    // into buffer (k + 2) % 3 (last read during step k - 1, i.e. before the previous barrier), so the first
    // fragments of step k + 1 (written during step k - 1) can be requested BEFORE the barrier that ends step k and
    // the matrix pipe does not wait for an LDS round trip after every barrier.
    // Register queues are rings indexed by the K-step (A: 3 deep, holding steps k + 2 .. k + 4; B: 3 deep,
    // k .. k + 2); a ring must be indexed at compile time and a value still in flight must never be copied (a copy
    // waits for it), hence the loop body is written out for kMxChunk consecutive K-steps (a multiple of the
    // rings' periods and of the 4 K-steps of a scale dword) with one early exit.
    AStage ar[3];
    BStage bq[3];
    load_a(0, ar[0]);
    load_a(1, ar[1]);
    load_b(0, bq[0]);
    load_wscales(0, wq0, wq1);
    load_wscales(1, wq0_n, wq1_n);
    store_a(smem_mx, ar[0]);
    store_a(smem_mx + kStage, ar[1]);
    load_a(2, ar[2]);
    load_a(3, ar[0]);
    load_a(4, ar[1]);
    load_b(1, bq[1]);
    load_b(2, bq[2]);
    __syncthreads();

    const int fr = lane & 15, fkb = lane >> 4;
    const int fa_off = mx_lds_off(fr, fkb);                                          // + 1024 per MFMA tile (16 rows)
    const int fs_off = BM * kMxRowBytes + fr * 4 + fkb;                           // + 64 per MFMA tile
    // fragments are requested kFragAhead tiles before their MFMAs (an LDS read takes several times as long as the
    // two MFMAs of a tile), across the end of a K-step as well
    constexpr int kFragAhead = 3;
    u32x4 fa[kFragAhead + 1];
    uint32_t xsb[kFragAhead + 1];
#pragma unroll
    for (int i = 0; i < kFragAhead; ++i) {
        fa[i] = *(const u32x4 *)(smem_mx + fa_off + i * 1024);
        xsb[i] = *(const uint8_t *)(smem_mx + fs_off + i * 64);
    }

    for (int ks0 = 0; ks0 < n_ks; ks0 += kMxChunk) {
        mx_static_while<kMxChunk>([&](auto I) {
            constexpr int u = I;
            const int ks = ks0 + u;
            if (ks >= n_ks) return false;
            const char *cur = smem_mx + (u % 3) * kStage;
            const char *nxt = smem_mx + ((u + 1) % 3) * kStage;
            char *fill = smem_mx + ((u + 2) % 3) * kStage;
            AStage &an = ar[(u + 2) % 3];                                           // holds K-step ks + 2
            BStage &bc = bq[u % 3];
            const uint32_t ws0 = wq0 >> (8 * (u & 3)), ws1 = wq1 >> (8 * (u & 3));
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                constexpr int kRing = kFragAhead + 1;
                const int ip = i + kFragAhead;
                if (ip < MI) {
                    fa[ip % kRing] = *(const u32x4 *)(cur + fa_off + ip * 1024);
                    xsb[ip % kRing] = *(const uint8_t *)(cur + fs_off + ip * 64);
                } else {
                    fa[ip % kRing] = *(const u32x4 *)(nxt + fa_off + (ip - MI) * 1024);
                    xsb[ip % kRing] = *(const uint8_t *)(nxt + fs_off + (ip - MI) * 64);
                }
                if (i == MI / 4) {                                                  // requested three K-steps ago
                    store_a(fill, an);
                    load_a(ks + 5, an);
                }
                const u32x4 fa_cur = fa[i % kRing];
                const uint32_t xs_cur = xsb[i % kRing];
                acc[i][0] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(as_operand(fa_cur), as_operand(bc.t0), acc[i][0], 4, 4, 0, (int)xs_cur, 0, (int)ws0);
                acc[i][1] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(as_operand(fa_cur), as_operand(bc.t1), acc[i][1], 4, 4, 0, (int)xs_cur, 0, (int)ws1);
                __builtin_amdgcn_sched_barrier(0);                                  // keep the reads this far ahead of their use
            }
            load_b(ks + 3, bc);
            if constexpr ((u & 3) == 3) {
                wq0 = wq0_n; wq1 = wq1_n;                                          // requested 4 K-steps ago
                load_wscales((ks >> 2) + 2, wq0_n, wq1_n);
            }
            __syncthreads();
            return true;
        });
    }

    // ---- epilogue.  Lane holds column fr, tokens 4 fkb + r of every 16 x 16 tile; a 16 x 32 strip of the wave's
    // tile goes through a wave-private 1 KB of LDS (the K loop's buffers are free now) and leaves as one 16-byte
    // store per lane: 64 contiguous bytes per token row instead of 2-byte stores. ----
    __syncthreads();
    _Float16 *strip = (_Float16 *)(smem_mx + wave * 1024);                          // [16 tokens][32 outputs]
    const __amdgpu_buffer_rsrc_t yr = mx_rsrc(a.Y, (uint32_t)(((size_t)(a.T - 1) * a.ldy + a.N) * 2));
    const int nw0 = n0 + wave * 32;
    float bv[2];
#pragma unroll
    for (int jn = 0; jn < 2; ++jn) {
        const int n = nw0 + jn * 16 + fr;
        bv[jn] = (a.bias && n < a.N) ? (float)a.bias[n] : 0.f;
    }
    const int orow = lane >> 2, ocol = (lane & 3) * 8;                               // this lane's 8 outputs of the strip
    const bool row_wide = a.ldy % 8 == 0 && ((uintptr_t)a.Y % 16) == 0 && nw0 + 32 <= a.N;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
        for (int jn = 0; jn < 2; ++jn)
#pragma unroll
            for (int r = 0; r < 4; ++r) strip[(fkb * 4 + r) * 32 + jn * 16 + fr] = (_Float16)(acc[i][jn][r] + bv[jn]);
        __builtin_amdgcn_wave_barrier();
        const int m = m0 + i * 16 + orow;
        if (row_wide) {
            const u32x4 v = *(const u32x4 *)(strip + orow * 32 + ocol);
            const uint32_t off = m < a.T ? (uint32_t)(((size_t)m * a.ldy + nw0 + ocol) * 2) : kOobM;
            __builtin_amdgcn_raw_buffer_store_b128(v, yr, (int)off, 0, 0);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                union { _Float16 h; uint16_t u; } o; o.h = strip[orow * 32 + ocol + e];
                const int n = nw0 + ocol + e;
                const uint32_t off = (m < a.T && n < a.N) ? (uint32_t)(((size_t)m * a.ldy + n) * 2) : kOobM;
                __builtin_amdgcn_raw_buffer_store_b16(o.u, yr, (int)off, 0, 0);
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

template <int BM>
static hipError_t launch_mxfp4_gemm_bm(MxGemmArgs &a, int n_tile0, int n_count, hipStream_t s)
{
    a.m_tiles = (a.T + BM - 1) / BM; a.n_tiles = n_count; a.n_tile0 = n_tile0;
    int blocks;
    gemm_patches(a.m_tiles, a.n_tiles, a.patch_m, a.patch_n, blocks);
    constexpr int lds = 3 * mx_stage_bytes(BM);
    static std::atomic<uint64_t> attr_done{0};
    if (const int dev = once_pending(attr_done); dev >= 0) {
        hipError_t e = hipFuncSetAttribute((const void *)mxfp4_gemm_kernel<BM>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        once_done(attr_done, dev);
    }
    hipLaunchKernelGGL(mxfp4_gemm_kernel<BM>, dim3(blocks), dim3(512), lds, s, a);
    return hipGetLastError();
}

// 256-token tiles fill at most half a round of blocks: 128-token tiles, twice as many
static bool mxfp4_gemm_small_tiles(const paro_mxfp4_weight &w, int T)
{
    return (long)((T + kMxBM - 1) / kMxBM) * ((w.c_out + kMxBN - 1) / kMxBN) <= 128;
}

static hipError_t launch_mxfp4_gemm(const paro_mxfp4_weight &w, const uint32_t *xc, const uint8_t *xs, int T, paro_half_t *Y,
                                    int64_t ldy, hipStream_t s)
{
    MxGemmArgs a;
    a.blob = w.packed;
    a.scales_off = (uint32_t)((size_t)w.c_out * w.c_in / 2);
    a.blob_bytes = a.scales_off + (uint32_t)((size_t)w.c_out * w.c_in / 32);
    a.xc = xc; a.xs = xs; a.Y = (_Float16 *)Y; a.ldy = ldy; a.bias = (const _Float16 *)w.bias;
    a.T = T; a.C = w.c_in; a.N = w.c_out; a.K128 = w.c_in / 128; a.KS = w.c_in / 512;
    const int m_big = (T + kMxBM - 1) / kMxBM, n_all = (w.c_out + kMxBN - 1) / kMxBN;
    if (mxfp4_gemm_small_tiles(w, T)) return launch_mxfp4_gemm_bm<128>(a, 0, n_all, s);
    // A last round of 256-token tiles that would be at most half full runs as a launch of its own with 128-token
    // tiles (896 tiles = 3 rounds + one round of 256 half-size tiles instead of 4 rounds).
    const long tiles = (long)m_big * n_all, full = tiles / 256, rem = tiles - full * 256;
    const int n_main = (int)(full * 256 / m_big);
    if (rem > 0 && rem <= 128 && n_main > 0 && n_main < n_all) {
        hipError_t e = launch_mxfp4_gemm_bm<256>(a, 0, n_main, s);
        return e != hipSuccess ? e : launch_mxfp4_gemm_bm<128>(a, n_main, n_all - n_main, s);
    }
    return launch_mxfp4_gemm_bm<256>(a, 0, n_all, s);
}

// Which kernel: the streaming kernel reads the whole weight once per 64 tokens (32 or 16 where K is deep), the
// GEMM once per 256 (or 128) but works on whole tiles whatever T is, one round of them per 256 compute units.
// Measured: a pass of TB blocks of 16 tokens takes ~3 us + the blob at 5.5 TB/s + TB x (0.8 us + the blob at
// 30 TB/s); a round of GEMM tiles ~0.9 us per K-step (0.8 us with 128-token tiles) + 3 us.
hipError_t launch_mxfp4_linear(const paro_mxfp4_weight &w, const uint32_t *x_codes, const uint8_t *x_scales, int T,
                               paro_half_t *Y, int64_t ldy, hipStream_t s)
{
    const int pass = mxfp4_pass_tokens(w, T);
    // the GEMM addresses the activations with 32-bit offsets
    if (T > pass && (size_t)T * w.c_in / 2 < (1ull << 31) && ((size_t)(T - 1) * ldy + w.c_out) * 2 < (1ull << 31)) {
        const double mb = ((double)w.c_out * w.c_in / 2 + (double)w.c_out * w.c_in / 32) / 1.0e6;
        const double pass_us = 3.0 + mb / 5.5 + (pass / 16) * (0.8 + mb / 30.0);
        const double stream_us = (double)((T + pass - 1) / pass) * pass_us;
        const bool small = mxfp4_gemm_small_tiles(w, T);
        const int bm = small ? 128 : kMxBM;
        const long tiles = (long)((T + bm - 1) / bm) * ((w.c_out + kMxBN - 1) / kMxBN);
        const double gemm_us = (double)((tiles + 255) / 256) * ((w.c_in / 128) * (small ? 0.8 : 0.9) + 3.0);
        if (gemm_us < stream_us) return launch_mxfp4_gemm(w, x_codes, x_scales, T, Y, ldy, s);
    }
    for (int t0 = 0; t0 < T;) {
        const int pass = mxfp4_pass_tokens(w, T - t0);
        const int tp = T - t0 < pass ? T - t0 : pass;
        hipError_t e = launch_mxfp4_decode(w, x_codes + (size_t)t0 * (w.c_in / 8), x_scales + (size_t)t0 * (w.c_in / 32), tp,
                                           Y + (size_t)t0 * ldy, ldy, s);
        if (e != hipSuccess) return e;
        t0 += tp;
    }
    return hipSuccess;
}

}  // namespace paro
