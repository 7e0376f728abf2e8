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
//
// Split K.  Some tens to hundreds of tokens give only a handful of tiles, each walking all of K on
// one compute unit.  Then K is cut into slices (blockIdx.y), as many as fit one round of blocks;
// every slice stores its fp32 tile to scratch memory and a second kernel sums the slices in index
// order, adds the bias and rounds once (deterministic; no atomics).
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
    int k_split, k_steps;       // blockIdx.y walks K-steps [y k_steps, (y+1) k_steps); k_split > 1: fp32 partial tiles
    float *partial;             //   [k_split][T][part_w] instead of Y (outputs part_n0 .. part_n0 + part_w), summed
    int part_n0, part_w;        //   by gemm_splitk_reduce_kernel
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
// Block tile = (WM MI 32) tokens x (WN NI 32 = 256 or 192) outputs.
// SPLITK: blockIdx.y selects a slice of K and the block stores fp32 partial tiles.
template <int MI, int NI, int WM, int WN, bool SPLITK = false>
__global__ __launch_bounds__(WM * WN * 64) void gemm_w4a16_kernel(GemmArgs a)
{
    constexpr int THREADS = WM * WN * 64;
    constexpr int BM = WM * MI * 32;
    constexpr int BN = WN * NI * 32;                       // outputs per block: 256, or 192 (the B tile is still staged as 256 rows)
    static_assert(BN <= kBN && BN % 32 == 0, "at most 256 outputs per block");
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
    const int m0 = mt * BM, n0 = (a.n_tile0 + ntile) * BN;

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
        const bool ok = nt * kTileN < a.N && (b_rt + kBTiles * p) * kTileN < BN;    // rows beyond a 192-wide tile: not fetched
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
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    u32x2 bsc[PB];                  // the 4 fp16 group scales of the thread's row in the current 512-channel slice
    uint16_t bzq[PB];               // its 4 zero points; widened where it is used: no ALU op (hence no wait) at the load
    const int k_begin = SPLITK ? blockIdx.y * a.k_steps : 0;             // this block's K-steps (split K: a slice)
    const int k_end = SPLITK ? min(a.C / kBK, k_begin + a.k_steps) : a.C / kBK;
    auto load_a = [&](int r, int ks) {
        areg[r] = __builtin_amdgcn_raw_buffer_load_b128(xr, (int)a_voff[r], ks * (kBK * 2), 0);
    };
    // Codes of K-step ks; scales and zero points only where a new 512-channel slice (8 K-steps)
    // begins - they are laid out 4 groups together, and a thread keeps its row for the whole loop.
    // The branch is uniform; the registers of the old slice are free by then (the refill of a load
    // comes after the last dequantisation that uses it).
    auto load_b = [&](int p, int ks, bool first = false) {
        const int g = ks >> 1, half = ks & 1;
        bw[p] = __builtin_amdgcn_raw_buffer_load_b128(br, (int)bw_voff[p], g * 1024 + half * 512, 0);
        if (first || (ks & 7) == 0) {
            bsc[p] = __builtin_amdgcn_raw_buffer_load_b64(br, (int)bs_voff[p], (g >> 2) * (kTileN * 8), 0);
            bzq[p] = __builtin_amdgcn_raw_buffer_load_b16(br, (int)bz_voff[p], (g >> 2) * (kTileN * 2), 0);
        }
    };
    half2v nlo[PB], nhi[PB], s2[PB];
    auto deq_consts = [&](int p, int ks) {
        const int g = ks >> 1;
        const uint32_t z = ((uint32_t)bzq[p] >> (4 * (g & 3))) & 15u;
        nlo[p] = g_as_h2((0xE400u + z) * 0x00010001u);          // -(1024 + z), twice
        nhi[p] = g_as_h2((0xD400u + (z << 4)) * 0x00010001u);   // -(64 + z), twice
        const uint32_t sc = ((g & 2) ? bsc[p][1] : bsc[p][0]) >> (16 * (g & 1));
        s2[p] = g_as_h2((sc & 0xffffu) * 0x00010001u);
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
    for (int r = 0; r < AL; ++r) load_a(r, k_begin);
#pragma unroll
    for (int p = 0; p < PB; ++p) load_b(p, k_begin, true);
#pragma unroll
    for (int r = 0; r < AL; ++r) *(u32x4 *)&As[a_lds + kARows * r * kLdsRow] = areg[r];
#pragma unroll
    for (int p = 0; p < PB; ++p) {
        deq_consts(p, k_begin);
#pragma unroll
        for (int w4 = 0; w4 < 4; ++w4) { deq_half(Bs, p, w4, 0); deq_half(Bs, p, w4, 1); }
    }
    {
        // same order as in the steady state, so that the loop's load counting is exact from the start
        const int k1 = k_begin + 1 < k_end ? k_begin + 1 : k_begin;
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

    for (int ks = k_begin; ks < k_end; ++ks) {
        const int buf = (ks - k_begin) & 1;
        const _Float16 *Ac = As + buf * BM * kLdsRow, *Bc = Bs + buf * kBN * kLdsRow;
        _Float16 *An = As + (buf ^ 1) * BM * kLdsRow, *Bn = Bs + (buf ^ 1) * kBN * kLdsRow;
        const int ks_store = ks + 1;                                      // K-step held in the registers
        const int ks_load = ks + 2 < k_end ? ks + 2 : k_end - 1;          // clamped: the surplus data is never used
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

    // ---- epilogue.  Lane (column fr, half fh) holds rows 8b + 4 fh + r. --------------------------
    if constexpr (SPLITK) {
        // split K: this slice's fp32 sums; bias and rounding happen once, in the reduction
        const __amdgpu_buffer_rsrc_t pr =
            make_rsrc_g(a.partial + (size_t)blockIdx.y * a.T * a.part_w, (uint32_t)((size_t)a.T * a.part_w * 4));
#pragma unroll
        for (int jn = 0; jn < NI; ++jn) {
            const int n = n0 + wn * NI * 32 + jn * 32 + fr;
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + wm * MI * 32 + i * 32 + (v >> 2) * 8 + fh * 4 + (v & 3);
                    const uint32_t off =
                        (m < a.T && n < a.N) ? (uint32_t)(((size_t)m * a.part_w + (n - a.part_n0)) * 4) : kOobG;
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[i][jn][v]), pr, (int)off, 0, 0);
                }
        }
        return;
    }
    // + bias, fp16 store
    const __amdgpu_buffer_rsrc_t yr = make_rsrc_g(a.Y, SPLITK ? 0u : (uint32_t)(((size_t)(a.T - 1) * a.ldy + a.N) * 2));
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

// Split K, second step: Y[t][n0 + n] = fp16( sum_k partial[k][t][n] + bias[n0 + n] ) for n < width,
// slices added in index order (deterministic).  One thread per 4 consecutive outputs of a token.
__global__ __launch_bounds__(256) void gemm_splitk_reduce_kernel(const float *__restrict__ partial, int k_split, int T,
                                                                 int n0, int width, const _Float16 *__restrict__ bias,
                                                                 _Float16 *__restrict__ Y, int64_t ldy)
{
    const int n4 = width / 4;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)T * n4) return;
    const int t = (int)(idx / n4), n = (int)(idx % n4) * 4;
    const size_t slice = (size_t)T * width;
    const float *p = partial + (size_t)t * width + n;
    float4 sum = *(const float4 *)p;
    for (int k = 1; k < k_split; ++k) {
        const float4 v = *(const float4 *)(p + k * slice);
        sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
    }
    if (bias) {
        const _Float16 *b = bias + n0 + n;
        sum.x += (float)b[0]; sum.y += (float)b[1]; sum.z += (float)b[2]; sum.w += (float)b[3];
    }
    union { _Float16 h[4]; uint2 u; } o;
    o.h[0] = (_Float16)sum.x; o.h[1] = (_Float16)sum.y; o.h[2] = (_Float16)sum.z; o.h[3] = (_Float16)sum.w;
    *(uint2 *)(Y + (size_t)t * ldy + n0 + n) = o.u;
}

// Block slots of a launch over m_tiles x n_tiles tiles: the XCD patches are rounded up to whole
// rounds of 8 (see the kernel's block numbering); slots without a tile exit at once.
void gemm_patches(int m_tiles, int n_tiles, int &patch_m, int &patch_n, int &blocks)
{
    int pb = kPatchBlocks;
    while (pb > 1 && (long)m_tiles * n_tiles < 8L * pb) pb >>= 1;
    patch_m = 1;
    while (patch_m * 2 <= pb && patch_m * 2 <= 8 && patch_m * 2 <= m_tiles) patch_m <<= 1;
    patch_n = pb / patch_m;
    const int m_patches = (m_tiles + patch_m - 1) / patch_m, n_patches = (n_tiles + patch_n - 1) / patch_n;
    blocks = (m_patches * n_patches + 7) / 8 * 8 * pb;
}

// How a (weight, T) pair is launched.
//   Tiles: 256 tokens x 256 outputs unless they leave compute units idle.  Up to half a round of
//   256 blocks: 128-token tiles throughout (twice the blocks, still one round).  More than half a
//   round but less than a full one: 256-token tiles all the same - two rounds of half-size tiles
//   take as long on paper and longer in practice (2048 x 4096 -> 6144, 192 tiles: 120 us against
//   136 us).  Otherwise, when the last round would be at most half full, that remainder (a range
//   of output tiles, the "tail") is launched separately with 128-token tiles: e.g. 896 tiles =
//   3 rounds of 256-token tiles + one round of 256 half-size tiles instead of 4.
//   Split K: a launch of 128-token tiles that fills at most half of the block slots (the whole
//   call at some tens to hundreds of tokens, or the tail) cuts K into slices over blockIdx.y, as
//   many as fit one round of slots with at least 4 K-steps each; the slices' fp32 tiles go to
//   scratch memory and are summed by a second kernel.  The number of slices minimises a measured
//   cost model: ~0.95 us per K-step of a block in a long launch, ~5 us + 1.2 us per K-step for the
//   short blocks of a whole-call split, partial tiles written and read at ~4.5 TB/s, ~2 us for the
//   reduction launch.  (More than one round of slots was measured slower.)
struct GemmPlan {
    int n_all, m_big;
    int n_192;               // > 0: the whole call as 256-token x 192-output tiles, this many across (see plan_gemm)
    int n_main;              // output tiles [0, n_main) with 256-token tiles (0: none)
    int n_small;             // output tiles [n_main, n_main + n_small) with 128-token tiles (0: none)
    int k_split, k_steps;    // of the 128-token-tile launch
    int big_split, big_steps;// of the 256-token-tile launch (only without a 128-token-tile launch; 1: not split)
    size_t scratch;          // bytes of partial tiles
    double est_us;
};

static void plan_split(GemmPlan &p, int T, int n_ks, int width, double base_us, double fixed_us, double step_us)
{
    p.k_split = 1; p.k_steps = n_ks; p.scratch = 0;
    const int m_tiles = (T + 127) / 128;
    if ((long)m_tiles * p.n_small > 128 || n_ks < 8 || (size_t)T * width * 4 >= (1ull << 31)) return;
    int pm, pn, slots;
    gemm_patches(m_tiles, p.n_small, pm, pn, slots);
    double best = base_us;
    for (int ks = 2; ks <= n_ks / 4 && (long)slots * ks <= 256; ++ks) {
        const int steps = (n_ks + ks - 1) / ks, split = (n_ks + steps - 1) / steps;
        if (split != ks) continue;
        const double us = fixed_us + steps * step_us + 2.0 + (double)ks * T * width * 8.0 / 4.5e6;
        if (us < best) { best = us; p.k_split = ks; p.k_steps = steps; }
    }
    if (p.k_split > 1) { p.scratch = (size_t)p.k_split * T * width * sizeof(float); p.est_us += best - base_us; }
}

static GemmPlan plan_gemm(const paro_w4_weight &w, int T)
{
    GemmPlan p{};
    p.big_split = 1;
    const int n_ks = w.c_in / kBK;
    p.n_all = (w.c_out + kBN - 1) / kBN; p.m_big = (T + 255) / 256;
    const long big_tiles = (long)p.m_big * p.n_all;
    if (big_tiles <= 128) {                                  // 128-token tiles throughout
        p.n_main = 0; p.n_small = p.n_all;
        const long tiles = (long)((T + 127) / 128) * p.n_all;
        p.est_us = (double)n_ks * 0.95 * (double)((tiles + 255) / 256);
        if (T <= 512) plan_split(p, T, n_ks, w.c_out, p.est_us, 5.0, 1.2);
        else { p.k_split = 1; p.k_steps = n_ks; }
        // Long K on few tiles (2048 x 14336 -> 4096): 256-token tiles with K cut so that they fill the
        // round do more MFMA work per staged byte than one round of 128-token tiles.  Measured per
        // K-step: ~1.1 us for the half-size tile in such launches, ~1.95 us for the full one; the
        // partial tiles cost about their bytes at 9 TB/s (they overlap the tail of the main kernel).
        // 254 -> 236 us on that shape; not worth it for K = 4096.
        if (p.k_split == 1 && T > 512 && (size_t)T * w.c_out * 4 < (1ull << 31)) {
            int pm, pn, slots;
            gemm_patches(p.m_big, p.n_all, pm, pn, slots);
            double best = (double)n_ks * 1.1 * (double)((tiles + 255) / 256);
            for (int ks = 2; ks <= 4 && (long)slots * ks <= 256 && n_ks / ks >= 32; ++ks) {
                const int steps = (n_ks + ks - 1) / ks;
                if ((n_ks + steps - 1) / steps != ks) continue;
                const double us = steps * 1.95 + 2.0 + (double)ks * T * w.c_out * 8.0 / 9.0e6;
                if (us < best) { best = us; p.big_split = ks; p.big_steps = steps; }
            }
            if (p.big_split > 1) {
                p.n_main = p.n_all; p.n_small = 0; p.est_us = best;
                p.scratch = (size_t)p.big_split * T * w.c_out * sizeof(float);
            }
        }
        return p;
    }
    const long full = big_tiles / 256, rem = big_tiles - full * 256;
    p.n_main = p.n_all; p.n_small = 0; p.k_split = 1; p.k_steps = n_ks;
    p.est_us = (double)n_ks * 1.9 * (double)((big_tiles + 255) / 256);
    // Less than one round of 256 x 256 tiles, but one round of 256 x 192 tiles: narrower tiles, every
    // compute unit busy (2048 x 4096 -> 6144: 192 tiles become 256; measured 125 -> 100 us).
    const int n_192 = (w.c_out + 191) / 192;
    if (full == 0 && (long)p.m_big * n_192 <= 256 && (long)p.m_big * n_192 > big_tiles) {
        p.n_192 = n_192; p.est_us = (double)n_ks * 1.9 * 0.8;
        return p;
    }
    if (rem > 0 && rem <= 128) {
        const int n_main = (int)(full * 256 / p.m_big);
        if (n_main > 0 && n_main < p.n_all) {
            p.n_main = n_main; p.n_small = p.n_all - n_main;
            const double tail_us = (double)n_ks * 0.95;      // one (partly filled) round of 128-token tiles
            p.est_us = (double)n_ks * 1.9 * (double)full + tail_us;
            const int width = w.c_out - n_main * kBN;
            plan_split(p, T, n_ks, width, tail_us, 0.0, 0.95);
        }
    }
    return p;
}

size_t gemm_scratch_bytes(const paro_w4_weight &w, int T) { return plan_gemm(w, T).scratch; }

bool gemm_supported(const paro_w4_weight &w, int64_t ldx, int64_t ldy, int T)
{
    size_t blob = packed_tiles_bytes(w.c_in, w.c_out) + packed_scales_bytes(w.c_in, w.c_out) +
                  packed_zeros_bytes(w.c_in, w.c_out);
    return blob < (1ull << 31) && ((size_t)T * ldx) * 2 < (1ull << 31) && ((size_t)T * ldy) * 2 < (1ull << 31) &&
           w.c_in % kBK == 0;
}

// Rough duration of the GEMM in microseconds, for the choice between it and repeated passes of the
// streaming decode kernel at moderate token counts (see plan_gemm for the model).
double gemm_estimate_us(const paro_w4_weight &w, int T) { return plan_gemm(w, T).est_us; }

// output tiles [n_tile0, n_tile0 + n_count) x all token tiles
template <int MI, int NI, int WM, int WN, bool SPLITK = false>
static hipError_t launch_gemm_cfg(GemmArgs &a, int n_tile0, int n_count, hipStream_t s)
{
    constexpr int BM = WM * MI * 32;
    a.m_tiles = (a.T + BM - 1) / BM; a.n_tiles = n_count; a.n_tile0 = n_tile0;
    // 32 blocks per patch when there is work for all 8 XCDs at that size; smaller patches
    // otherwise, so that a small grid is still spread over every XCD's L2 and memory channels
    int blocks;
    gemm_patches(a.m_tiles, a.n_tiles, a.patch_m, a.patch_n, blocks);
    const size_t lds = (size_t)2 * (BM + kBN) * kLdsRow * sizeof(_Float16);
    static std::atomic<uint64_t> attr_done{0};
    if (const int dev = once_pending(attr_done); dev >= 0) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_w4a16_kernel<MI, NI, WM, WN, SPLITK>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        once_done(attr_done, dev);
    }
    hipLaunchKernelGGL((gemm_w4a16_kernel<MI, NI, WM, WN, SPLITK>), dim3(blocks, SPLITK ? a.k_split : 1),
                       dim3(WM * WN * 64), lds, s, a);
    return hipGetLastError();
}

hipError_t launch_gemm(const paro_w4_weight &w, const paro_half_t *X, int64_t ldx, paro_half_t *Y, int64_t ldy, int T,
                       void *scratch, size_t scratch_bytes, hipStream_t s)
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
    a.k_split = 1; a.k_steps = w.c_in / kBK; a.partial = nullptr; a.part_n0 = 0; a.part_w = 0;
    const GemmPlan p = plan_gemm(w, T);
    if (p.n_192 > 0) return launch_gemm_cfg<2, 3, 4, 2>(a, 0, p.n_192, s);
    auto reduce = [&](int k_split) {
        const long quads = (long)T * (a.part_w / 4);
        hipLaunchKernelGGL(gemm_splitk_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s,
                           (const float *)scratch, k_split, T, a.part_n0, a.part_w, (const _Float16 *)w.bias, (_Float16 *)Y, ldy);
        return hipGetLastError();
    };
    const bool have_scratch = scratch && scratch_bytes >= p.scratch && ((uintptr_t)scratch % 16) == 0;
    if (p.big_split > 1) {
        if (have_scratch) {
            a.k_split = p.big_split; a.k_steps = p.big_steps; a.partial = (float *)scratch; a.part_n0 = 0; a.part_w = w.c_out;
            hipError_t e = launch_gemm_cfg<4, 2, 2, 4, true>(a, 0, p.n_all, s);
            return e != hipSuccess ? e : reduce(p.big_split);
        }
        return launch_gemm_cfg<2, 2, 2, 4>(a, 0, p.n_all, s);      // no room for partial tiles: the unsplit choice
    }
    if (p.n_main > 0) {
        hipError_t e = launch_gemm_cfg<4, 2, 2, 4>(a, 0, p.n_main, s);
        if (e != hipSuccess || p.n_small == 0) return e;
    }
    if (!(p.k_split > 1 && have_scratch)) return launch_gemm_cfg<2, 2, 2, 4>(a, p.n_main, p.n_small, s);
    a.k_split = p.k_split; a.k_steps = p.k_steps; a.partial = (float *)scratch;
    a.part_n0 = p.n_main * kBN; a.part_w = w.c_out - a.part_n0;
    hipError_t e = launch_gemm_cfg<2, 2, 2, 4, true>(a, p.n_main, p.n_small, s);
    return e != hipSuccess ? e : reduce(p.k_split);
}

}  // namespace paro
