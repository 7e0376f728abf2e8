// Prefill-side W4A16 linear: Y[T x N] = X'[T x C] . W^[N x C]^T for many tokens (Eq. 2), the one
// dense contraction of the path, on fp16 MFMA with fp32 accumulation.
//
// Block tile BM (tokens: 256 or 128) x 256 (outputs) x 64 (channels), 4 wavefronts as 2 x 2,
// each wave a (BM/2) x 128 sub-tile of v_mfma_f32_32x32x16_f16 tiles (up to 256 accumulator
// registers).  Per K-step a block fetches BM x 128 B of activations and 8 KB of packed INT4
// codes; the codes are dequantised ONCE per block into an fp16 LDS tile
//      w^ = fp16( (q - z) * s )        ((q - z) exact in fp16, one rounding in the multiply:
//                                        the same value paro_w4_dequant produces)
// so the VALU cost per weight is amortised over the block's token rows.
//
// Software pipeline.  There is one wave per SIMD, so nothing hides a stall: every K-step is
// written as 4 phases (one per 16-channel MFMA step) of explicitly ordered slots
//      slot = 1 MFMA + at most one LDS fragment read + at most one piece of staging work,
// pinned with scheduling barriers so that the matrix pipe always has the next MFMA queued
// while the vector/LDS/memory instructions of the slot issue in its shadow:
//   - fragments of MFMA step kk+1 are read from LDS during the MFMAs of step kk (two register
//     sets);
//   - the global data of K-step s+1 sits in registers during K-step s, is dequantised /
//     copied into the other LDS buffer piece by piece in phases 0..2, and each register is
//     refilled at once with the load for K-step s+2 (a full K-step of latency allowance);
//   - one barrier per K-step, after phase 2: by then every wave has finished reading the
//     current buffer into registers and writing the next one, so phase 3 already reads the
//     next K-step's first fragments.
// LDS rows are padded by 16 bytes so that the 16-byte fragment reads of 32 consecutive rows
// spread over all banks.
//
// Blocks are numbered so that the 32 blocks resident on one XCD (block id mod 8) form an
// 8 (token tiles) x 4 (output tiles) patch that walks K in step: they share activation and
// weight panels through that XCD's L2.  With fewer than 8 token tiles the patch is narrower
// in tokens and wider in outputs, so that no block id of a patch is left without work, and
// with fewer than 256 tiles the patches shrink so that all 8 XCDs still get one.
#include "paro_internal.h"
#include <type_traits>

namespace paro {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBN = 256, kBK = 64;
constexpr int kLdsRow = kBK + 8;                    // halfs per padded LDS row
constexpr int kPatchBlocks = 32;                    // most blocks of one XCD patch (8 x 4 token x output tiles)

constexpr uint32_t kOobG = 0x80000000u;
__device__ inline __amdgpu_buffer_rsrc_t make_rsrc_g(const void *p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}
__device__ inline half2v g_as_h2(uint32_t u) { union { uint32_t u; half2v h; } c; c.u = u; return c.h; }
__device__ inline uint32_t g_as_u32(half2v h) { union { uint32_t u; half2v h; } c; c.h = h; return c.u; }

template <int N, class F, int I = 0>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<N, F, I + 1>(static_cast<F &&>(f));
    }
}

struct GemmArgs {
    const void *blob; uint32_t blob_bytes, scales_off, zeros_off;
    const _Float16 *X; int64_t ldx;
    _Float16 *Y; int64_t ldy;
    const _Float16 *bias;
    int T, C, N, G, S;          // S = G / 4 K-slices of the scales/zeros tiling
    int m_tiles, n_tiles;       // tiles of this launch
    int n_tile0;                // first 256-output tile of this launch
    int patch_m, patch_n;       // token tiles x output tiles of the patch of blocks one XCD works on
    uint32_t m_lo, m_hi, k_lo, k_hi;   // 0x000F000F, 0x00F000F0, 0x64006400, 0x54005400: passed as arguments and
                                       // moved to VGPRs so that (u & mask) | magic becomes one v_and_or_b32
};

// Staging work of one K-step, cut into items that are spread over the MFMA slots:
//   0..15   dequantise half of one 8-code word pair: code = p * 8 + w4 * 2 + h   (p: which of the
//           thread's 16-byte code loads, w4: word, h: low / high byte pair)
//   16..23  copy activation register r = code - 16 to LDS and refill it from global memory
//   24, 25  refill the code / scale / zero registers of load p = code - 24
// ALP activation registers per code load; the order interleaves LDS writes and global loads.
template <int ALP, int PB>
__host__ __device__ constexpr int staging_item(int k)
{
    // per p: 8 dequant halves with the A copies spread between them, then the refill of p
    constexpr int per_p = 8 + ALP + 1;
    if (k < 0 || k >= PB * per_p) return -1;
    const int p = k / per_p, r = k % per_p;
    if (r == per_p - 1) return 24 + p;
    constexpr int stride = 8 / ALP + 1;               // ALP = 4: 2 halves + 1 copy; ALP = 2: 4 halves + 1 copy
    const int grp = r / stride, in = r % stride;
    if (in == stride - 1) return 16 + p * ALP + grp;
    const int hidx = grp * (stride - 1) + in;          // 0..7 = w4 * 2 + h
    return p * 8 + hidx;
}

// MI x NI: 32x32 MFMA tiles per wave (tokens x outputs); WM x WN: waves per block.
// Block tile = (WM MI 32) tokens x (WN NI 32 = 256) outputs.
template <int MI, int NI, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64) void gemm_w4a16_kernel(GemmArgs a)
{
    constexpr int THREADS = WM * WN * 64;
    constexpr int BM = WM * MI * 32;
    static_assert(WN * NI * 32 == kBN, "256 outputs per block");
    constexpr int AL = BM * 8 / THREADS;                   // 16-byte activation loads per thread and K-step
    constexpr int PB = 512 / THREADS;                      // 16-byte code loads per thread and K-step
    constexpr int ALP = AL / PB;
    static_assert(ALP == 2 || ALP == 4, "staging schedule");
    constexpr int kSlots = MI * NI;                        // MFMAs per phase
    constexpr int kItems = PB * (8 + ALP + 1);
    // staging is packed into the first phases: the refill loads then have the rest of the K-step
    // (plus a whole further K-step) before their data is needed
    constexpr int kStagePhases = (2 * kSlots >= kItems && THREADS > 256) ? 2 : 3;
    static_assert(kStagePhases * kSlots >= kItems, "one staging item per slot at most");
    static_assert(MI + NI <= kSlots, "one fragment read per slot at most");
    extern __shared__ __attribute__((aligned(16))) _Float16 smem[];
    _Float16 *As = smem;                                   // [2][BM][kLdsRow]
    _Float16 *Bs = smem + 2 * BM * kLdsRow;                // [2][kBN][kLdsRow]

    // ---- block -> (m tile, n tile), XCD-aware --------------------------------------------------
    const int bid = blockIdx.x;
    const int xcd = bid & 7, j = bid >> 3;
    const int pb = a.patch_m * a.patch_n;
    const int patch = j / pb, q = j % pb;
    const int m_patches = (a.m_tiles + a.patch_m - 1) / a.patch_m;
    const int gp = patch * 8 + xcd;                        // global patch index
    const int pm = gp % m_patches, pn = gp / m_patches;
    const int mt = pm * a.patch_m + q % a.patch_m, ntile = pn * a.patch_n + q / a.patch_m;
    if (mt >= a.m_tiles || ntile >= a.n_tiles) return;
    const int m0 = mt * BM, n0 = (a.n_tile0 + ntile) * kBN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    const __amdgpu_buffer_rsrc_t xr = make_rsrc_g(a.X, (uint32_t)(((size_t)(a.T - 1) * a.ldx + a.C) * 2));
    const __amdgpu_buffer_rsrc_t br = make_rsrc_g(a.blob, a.blob_bytes);

    // per-thread load coordinates; the K-step enters every address as a wave-uniform byte offset
    // A: AL x 16 B per thread: row tid/8 + (THREADS/8) r, 16-byte column tid%8
    // B: PB x 16 B per thread: 16-row tile tid/32 + (THREADS/32) p, lane-in-half tid%32
    constexpr int kARows = THREADS / 8, kBTiles = THREADS / 32;
    const int a_c16 = tid & 7, a_row = tid >> 3;
    const int b_l32 = tid & 31, b_rt = tid >> 5;
    const int b_n = b_l32 & 15, b_kq = b_l32 >> 4;         // row in tile, 32-channel quarter within the half
    uint32_t a_voff[AL], bw_voff[PB], bs_voff[PB], bz_voff[PB];
#pragma unroll
    for (int r = 0; r < AL; ++r) {
        const int row = m0 + a_row + kARows * r;
        a_voff[r] = row < a.T ? (uint32_t)(((size_t)row * a.ldx + a_c16 * 8) * 2) : kOobG;
    }
#pragma unroll
    for (int p = 0; p < PB; ++p) {
        const int nt = n0 / kTileN + b_rt + kBTiles * p;
        const bool ok = nt * kTileN < a.N;
        bw_voff[p] = ok ? ((uint32_t)nt * a.G * 64u + b_kq * 16 + b_n) * 16u : kOobG;
        const uint32_t sidx = (uint32_t)nt * a.S * kTileN + b_n;
        bs_voff[p] = ok ? a.scales_off + sidx * 8u : kOobG;
        bz_voff[p] = ok ? a.zeros_off + sidx * 2u : kOobG;
    }
    const int a_lds = a_row * kLdsRow + a_c16 * 8;                          // + kARows r rows
    int b_lds[PB];
#pragma unroll
    for (int p = 0; p < PB; ++p) b_lds[p] = ((b_rt + kBTiles * p) * kTileN + b_n) * kLdsRow + b_kq * 32;

    u32x4 areg[AL];
    u32x4 bw[PB];
    uint16_t bsc[PB], bzq[PB];      // widened where they are used: no ALU op (hence no wait) at the load
    const int n_ks = a.C / kBK;
    auto load_a = [&](int r, int ks) {
        areg[r] = __builtin_amdgcn_raw_buffer_load_b128(xr, (int)a_voff[r], ks * (kBK * 2), 0);
    };
    auto load_b = [&](int p, int ks) {
        const int g = ks >> 1, half = ks & 1;
        bw[p] = __builtin_amdgcn_raw_buffer_load_b128(br, (int)bw_voff[p], g * 1024 + half * 512, 0);
        bsc[p] = __builtin_amdgcn_raw_buffer_load_b16(br, (int)bs_voff[p], (g >> 2) * (kTileN * 8) + (g & 3) * 2, 0);
        bzq[p] = __builtin_amdgcn_raw_buffer_load_b16(br, (int)bz_voff[p], (g >> 2) * (kTileN * 2), 0);
    };
    half2v nlo[PB], nhi[PB], s2[PB];
    auto deq_consts = [&](int p, int ks) {
        const int g = ks >> 1;
        const uint32_t z = ((uint32_t)bzq[p] >> (4 * (g & 3))) & 15u;
        nlo[p] = g_as_h2((0xE400u + z) * 0x00010001u);          // -(1024 + z), twice
        nhi[p] = g_as_h2((0xD400u + (z << 4)) * 0x00010001u);   // -(64 + z), twice
        s2[p] = g_as_h2((uint32_t)bsc[p] * 0x00010001u);
    };
    // half h of word w4 of load p -> 4 fp16 weights; the second half stores the word's 8 weights
    auto to_vgpr = [&](uint32_t v) { return (uint32_t)__builtin_amdgcn_ds_bpermute(lane << 2, (int)v); };
    const uint32_t c_mlo = to_vgpr(a.m_lo), c_mhi = to_vgpr(a.m_hi), c_klo = to_vgpr(a.k_lo), c_khi = to_vgpr(a.k_hi);
    uint32_t dq_keep[2];
    auto deq_half = [&](_Float16 *Bn, int p, int w4, int h) {
        const uint32_t u = bw[p][w4] >> (8 * h);
        const uint32_t o0 = g_as_u32((g_as_h2((u & c_mlo) | c_klo) + nlo[p]) * s2[p]);
        const uint32_t o1 = g_as_u32((g_as_h2((u & c_mhi) | c_khi) + nhi[p]) * s2[p]);
        if (h == 0) { dq_keep[0] = o0; dq_keep[1] = o1; }
        else {
            const u32x4 o = {dq_keep[0], dq_keep[1], o0, o1};
            *(u32x4 *)&Bn[b_lds[p] + w4 * 8] = o;
        }
    };

    float16v acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int jn = 0; jn < NI; ++jn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jn][v] = 0.f;

    // ---- prologue: K-step 0 into LDS buffer 0, K-step 1 into the registers -------------------
#pragma unroll
    for (int r = 0; r < AL; ++r) load_a(r, 0);
#pragma unroll
    for (int p = 0; p < PB; ++p) load_b(p, 0);
#pragma unroll
    for (int r = 0; r < AL; ++r) *(u32x4 *)&As[a_lds + kARows * r * kLdsRow] = areg[r];
#pragma unroll
    for (int p = 0; p < PB; ++p) {
        deq_consts(p, 0);
#pragma unroll
        for (int w4 = 0; w4 < 4; ++w4) { deq_half(Bs, p, w4, 0); deq_half(Bs, p, w4, 1); }
    }
    {
        // same order as in the steady state, so that the loop's load counting is exact from the start
        const int k1 = n_ks > 1 ? 1 : 0;
        static_for<kItems>([&](auto KI) {
            constexpr int code = staging_item<ALP, PB>(KI);
            if constexpr (code >= 16 && code < 24) load_a(code - 16, k1);
            else if constexpr (code >= 24) load_b(code - 24, k1);
        });
    }
    __syncthreads();

    const int fr = lane & 31, fh = lane >> 5;
    const int fa_off = (wm * MI * 32 + fr) * kLdsRow + fh * 8;
    const int fb_off = (wn * NI * 32 + fr) * kLdsRow + fh * 8;
    half8 fa[2][MI], fb[2][NI];
    // fragment `f` (0..MI-1: token tiles, MI..MI+NI-1: output tiles) of MFMA step kk
    auto read_frag = [&](const _Float16 *Ab, const _Float16 *Bb, int f, int kk, int set) {
        if (f < MI) fa[set][f] = *(const half8 *)&Ab[fa_off + f * 32 * kLdsRow + kk * 16];
        else fb[set][f - MI] = *(const half8 *)&Bb[fb_off + (f - MI) * 32 * kLdsRow + kk * 16];
    };
#pragma unroll
    for (int f = 0; f < MI + NI; ++f) read_frag(As, Bs, f, 0, 0);

    for (int ks = 0; ks < n_ks; ++ks) {
        const int buf = ks & 1;
        const _Float16 *Ac = As + buf * BM * kLdsRow, *Bc = Bs + buf * kBN * kLdsRow;
        _Float16 *An = As + (buf ^ 1) * BM * kLdsRow, *Bn = Bs + (buf ^ 1) * kBN * kLdsRow;
        const int ks_store = ks + 1;                                      // K-step held in the registers
        const int ks_load = ks + 2 < n_ks ? ks + 2 : n_ks - 1;            // clamped: the surplus data is never used
        static_for<4>([&](auto PH) {
            constexpr int ph = PH;
            static_for<kSlots>([&](auto SL) {
                constexpr int slot = SL;
                constexpr int i = slot / NI, jn = slot % NI;
                acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[ph & 1][i], fb[ph & 1][jn], acc[i][jn], 0, 0, 0);
                if constexpr (slot < MI + NI) {
                    if constexpr (ph < 3) read_frag(Ac, Bc, slot, ph + 1, (ph + 1) & 1);
                    else read_frag(An, Bn, slot, 0, 0);
                }
                if constexpr (ph < kStagePhases) {
                    // item k is placed at slot floor(k * total_slots / kItems) of the staging phases
                    constexpr int gs = ph * kSlots + slot, total = kStagePhases * kSlots;
                    constexpr int k = (gs * kItems + total - 1) / total;
                    constexpr int code = (k < kItems && k * total / kItems == gs) ? staging_item<ALP, PB>(k) : -1;
                    if constexpr (code >= 0 && code < 16) {
                        constexpr int p = code / 8, w4 = (code % 8) / 2, h = code % 2;
                        if constexpr (w4 == 0 && h == 0) deq_consts(p, ks_store);
                        deq_half(Bn, p, w4, h);
                    } else if constexpr (code >= 16 && code < 24) {
                        constexpr int r = code - 16;
                        *(u32x4 *)&An[a_lds + kARows * r * kLdsRow] = areg[r];
                        load_a(r, ks_load);
                    } else if constexpr (code >= 24) {
                        load_b(code - 24, ks_load);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            });
            if constexpr (ph == 2) __syncthreads();
        });
    }

    // ---- epilogue: + bias, fp16 store.  Lane (column fr, half fh) holds rows 8b + 4 fh + r. ------
    const __amdgpu_buffer_rsrc_t yr = make_rsrc_g(a.Y, (uint32_t)(((size_t)(a.T - 1) * a.ldy + a.N) * 2));
#pragma unroll
    for (int jn = 0; jn < NI; ++jn) {
        const int n = n0 + wn * NI * 32 + jn * 32 + fr;
        const float bv = (a.bias && n < a.N) ? (float)a.bias[n] : 0.f;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * MI * 32 + i * 32 + (v >> 2) * 8 + fh * 4 + (v & 3);
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

// Rough duration of the GEMM in microseconds, for the choice between it and repeated passes of the
// streaming decode kernel at moderate token counts.  A block walks c_in / 64 K-steps; measured
// per K-step and round of blocks: ~0.95 us with 128-token tiles, ~1.9 us with 256-token tiles.
double gemm_estimate_us(const paro_w4_weight &w, int T)
{
    const long n_tiles = (w.c_out + kBN - 1) / kBN;
    const long big_tiles = (long)((T + 255) / 256) * n_tiles;
    const bool big = big_tiles >= 256;
    const long blocks = big ? big_tiles : (long)((T + 127) / 128) * n_tiles;
    const long rounds = (blocks + 255) / 256;
    return (double)(w.c_in / kBK) * (double)rounds * (big ? 1.9 : 0.95);
}

// output tiles [n_tile0, n_tile0 + n_count) x all token tiles
template <int MI, int NI, int WM, int WN>
static hipError_t launch_gemm_cfg(GemmArgs &a, int n_tile0, int n_count, hipStream_t s)
{
    constexpr int BM = WM * MI * 32;
    a.m_tiles = (a.T + BM - 1) / BM; a.n_tiles = n_count; a.n_tile0 = n_tile0;
    // 32 blocks per patch when there is work for all 8 XCDs at that size; smaller patches
    // otherwise, so that a small grid is still spread over every XCD's L2 and memory channels
    int pb = kPatchBlocks;
    while (pb > 1 && (long)a.m_tiles * a.n_tiles < 8L * pb) pb >>= 1;
    a.patch_m = 1;
    while (a.patch_m * 2 <= pb && a.patch_m * 2 <= 8 && a.patch_m * 2 <= a.m_tiles) a.patch_m <<= 1;
    a.patch_n = pb / a.patch_m;
    const int m_patches = (a.m_tiles + a.patch_m - 1) / a.patch_m, n_patches = (a.n_tiles + a.patch_n - 1) / a.patch_n;
    const int patches = m_patches * n_patches;
    const int rounds = (patches + 7) / 8;                 // patches per XCD
    const int blocks = rounds * 8 * pb;
    const size_t lds = (size_t)2 * (BM + kBN) * kLdsRow * sizeof(_Float16);
    static std::atomic<uint64_t> attr_done{0};
    if (const int dev = once_pending(attr_done); dev >= 0) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_w4a16_kernel<MI, NI, WM, WN>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        once_done(attr_done, dev);
    }
    hipLaunchKernelGGL((gemm_w4a16_kernel<MI, NI, WM, WN>), dim3(blocks), dim3(WM * WN * 64), lds, s, a);
    return hipGetLastError();
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
    a.m_lo = 0x000F000Fu; a.m_hi = 0x00F000F0u; a.k_lo = 0x64006400u; a.k_hi = 0x54005400u;
    // 256-token tiles unless they leave compute units idle.  Fewer than one full round of 256
    // blocks: 128-token tiles throughout.  Otherwise, when the last round would be at most half
    // full, that remainder (a range of output tiles) is launched separately with 128-token tiles:
    // e.g. 896 tiles = 3 rounds of 256-token tiles + one round of 256 half-size tiles instead of 4.
    const int n_all = (w.c_out + kBN - 1) / kBN, m_big = (T + 255) / 256;
    const long big_tiles = (long)m_big * n_all;
#ifdef PARO_GEMM_4WAVES
    auto big = [&](int n0, int n) { return launch_gemm_cfg<4, 4, 2, 2>(a, n0, n, s); };
    auto small = [&](int n0, int n) { return launch_gemm_cfg<2, 4, 2, 2>(a, n0, n, s); };
#else
    auto big = [&](int n0, int n) { return launch_gemm_cfg<4, 2, 2, 4>(a, n0, n, s); };
    auto small = [&](int n0, int n) { return launch_gemm_cfg<2, 2, 2, 4>(a, n0, n, s); };
#endif
    if (big_tiles < 256) return small(0, n_all);
    const long full = big_tiles / 256, rem = big_tiles - full * 256;
#ifndef PARO_GEMM_NO_TAIL_SPLIT
    if (rem > 0 && rem <= 128) {
        const int n_main = (int)(full * 256 / m_big);
        if (n_main > 0 && n_main < n_all) {
            hipError_t e = big(0, n_main);
            if (e != hipSuccess) return e;
            return small(n_main, n_all - n_main);
        }
    }
#endif
    return big(0, n_all);
}

}  // namespace paro
