// Decode-side W4A16 linear (1..16 tokens per pass), bare or with the scaled pairwise rotation
// fused in front (Eq. 2 with T of Eq. 8).  HBM-bound: the packed INT4 weights are streamed
// exactly once, as 1 KB tiles, and everything else is arranged around that stream.
//
// The input channels are cut into K-slices of 4 groups (512 channels).  A wave needs the
// activations of one slice only and keeps them as MFMA A-fragments in registers for its whole
// stream (tokens padded to 16).  Two kernels share the stream code:
//
//  - decode_kernel (rotation fused, up to 4 tokens): a block owns ONE K-slice and a range of
//    16-row output tiles; its 4 waves share the slice and take different tiles.  Each wave
//    rotates one of the slice's 4 groups (one wavefront per (token, group), see rotate.hip) -
//    the prologue costs one group-rotation per wave however wide the layer is, and runs while
//    the first weight tiles are in flight.  The K-slices' partial sums are exchanged between
//    blocks at the end.
//  - decode_wide_kernel (bare, up to 16 tokens): a block takes ALL K-slices of its tile range,
//    one per wave, and sums them through LDS; no exchange between blocks up to 6144 channels.
//
// Inner loop per 16x128 tile and lane: one 16-byte load (32 codes), v_and_or_b32 with the fp16
// magic numbers 1024 / 64 (the code lands in the mantissa: 5 VALU ops per 8 weights), four
// v_mfma_f32_16x16x32_f16 whose accumulator starts at the bias / zero-point correction (see
// tile_dot), then the group's scale is applied once to the fp32 sum:  y += s * sum_k (q - z) x'.
//
// Split-K exchange: blocks store fp32 partial tiles to the workspace, then each sums its share
// of the output range over the partials in a fixed order (deterministic), adds the bias and
// rounds to fp16.  Agent-scope release/acquire fences would cost an L2 write-back and
// invalidate per wave on this multi-XCD part (measured: +40..85 us per launch), so none are
// used: each partial word is its own full/empty flag (see splitk_reduce).
#include "decode_common.h"

namespace paro {

// K: rotation layers fused in front.  SPLIT: more than one K-slice.  T1: exactly one token.
template <int K, bool SPLIT, bool T1, int W = kDecWaves>
__device__ __forceinline__ void decode_body(const DecodeArgs &a, const int ks, const int nb,
                                            _Float16 (*s_x)[kSliceCh + kXPad], float *s_red)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tile_lo = nb * a.tiles_per_block;
    const int tile_hi = min(a.NT, tile_lo + a.tiles_per_block);
    const int n_iter = (tile_hi - tile_lo + W - 1) / W;      // same for all waves of the block
    auto tile_of = [&](int i) {                                              // -1: nothing to do
        int t = tile_lo + wave + i * W;
        return (i < n_iter && t < tile_hi) ? t : -1;
    };
    const __amdgpu_buffer_rsrc_t blob = make_rsrc(a.blob, a.blob_bytes);

    Stage st0, st1, st2;

    // ---- activations of this K-slice -> MFMA A fragments ---------------------------------
    half8 xf[kSliceGroups][4];
    const int ft = lane & 15, fkb = lane >> 4;
    const size_t c0 = (size_t)ks * kSliceCh;
    {
        // wave w < 4 rotates group w of the slice for all T tokens; further waves only stream
        const int gi = wave & (kSliceGroups - 1);
        const bool rw = W == kSliceGroups || wave < kSliceGroups;
        const uint32_t *gplan = a.plan + ((size_t)ks * kSliceGroups + gi) * plan_group_dwords(K);
        // natural-order load first (independent of the plan), staged through LDS
        if (rw)
            for (int t = 0; t < a.T; ++t)
                *(uint32_t *)&s_x[t][gi * kGroup + 2 * lane] =
                    *(const uint32_t *)(a.X + (size_t)t * a.ldx + c0 + gi * kGroup + 2 * lane);
        uint32_t io = gplan[lane];
        float sia = __uint_as_float(gplan[64 + lane]), sib = __uint_as_float(gplan[128 + lane]);
        float soa = __uint_as_float(gplan[192 + lane]), sob = __uint_as_float(gplan[256 + lane]);
        float pc[K > 0 ? K : 1], ps[K > 0 ? K : 1];
        uint32_t pm[K > 0 ? K : 1];
#pragma unroll
        for (int l = 0; l < K; ++l) {
            const uint32_t *row = gplan + (size_t)(kPlanHeadRows + kPlanRowsPerLayer * l) * 64;
            pc[l] = __uint_as_float(row[lane]); ps[l] = __uint_as_float(row[64 + lane]); pm[l] = row[128 + lane];
        }
        // The weight stream starts here, behind the (older, L2-resident) plan and X loads: vector
        // memory returns in order, so waiting for the plan must not mean waiting for HBM tiles.
        load_stage(blob, a, tile_of(0), ks, lane, st0);
        load_stage(blob, a, tile_of(1), ks, lane, st1);
        const int in_a = io & 0xff, in_b = (io >> 8) & 0xff, out_a = (io >> 16) & 0xff, out_b = io >> 24;
        // up to 4 tokens side by side: the chains of a layer (4 multiply-adds, then a permute that takes far longer)
        // are independent between tokens, so a batch costs little more than one token
        constexpr int TB = T1 ? 1 : 4;
        for (int t0 = 0; t0 < (rw ? a.T : 0); t0 += TB) {
            float va[TB], vb[TB];
#pragma unroll
            for (int u = 0; u < TB; ++u) {
                const int t = min(t0 + u, a.T - 1);                          // surplus slots repeat the last token
                va[u] = (float)s_x[t][gi * kGroup + in_a] * sia;
                vb[u] = (float)s_x[t][gi * kGroup + in_b] * sib;
            }
#pragma unroll
            for (int l = 0; l < K; ++l) {
                const bool ai = pm[l] & kMetaAIsI, ki = pm[l] & kMetaKeepI;
                const float c = pc[l], s = ps[l];
                const float ni_a = ai ? c : -s, ni_b = ai ? -s : c, nj_a = ai ? s : c, nj_b = ai ? c : s;
                const float m00 = ki ? ni_a : nj_a, m01 = ki ? ni_b : nj_b, m10 = ki ? nj_a : ni_a, m11 = ki ? nj_b : ni_b;
#pragma unroll
                for (int u = 0; u < TB; ++u) {
                    const float na = m00 * va[u] + m01 * vb[u], nb2 = m10 * va[u] + m11 * vb[u];
                    va[u] = na;
                    vb[u] = (l + 1 < K) ? __int_as_float(__builtin_amdgcn_ds_bpermute((int)(pm[l] & 0xff), __float_as_int(nb2)))
                                        : nb2;
                }
            }
            // all lanes have read their inputs of these tokens (the permutes above are wave-wide), so the staging
            // rows can be overwritten with the results
#pragma unroll
            for (int u = 0; u < TB; ++u)
                if (t0 + u < a.T) {
                    s_x[t0 + u][gi * kGroup + out_a] = (_Float16)(va[u] * soa);
                    s_x[t0 + u][gi * kGroup + out_b] = (_Float16)(vb[u] * sob);
                }
        }
        __syncthreads();
#pragma unroll
        for (int g2 = 0; g2 < kSliceGroups; ++g2)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
                if (ft < a.T) v = *(const half8 *)&s_x[ft][g2 * kGroup + fkb * 32 + j * 8];
                xf[g2][j] = v;
            }
    }

    // per token and group: nb1 = -sum_k b_k x'_k, nb2 = -sum_k x'_k, as MFMAs against constant
    // operands whose 16 columns are equal - every lane gets the sums of its own 4 token rows
    float4v nb1[kSliceGroups], nb2[kSliceGroups];
    {
        const half8 cb1 = {-1024, -1024, -64, -64, -1024, -1024, -64, -64};
        const half8 cb2 = {-1, -1, -1, -1, -1, -1, -1, -1};
#pragma unroll
        for (int g2 = 0; g2 < kSliceGroups; ++g2) {
            float4v s1 = {0.f, 0.f, 0.f, 0.f}, s2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                s1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf[g2][j], cb1, s1, 0, 0, 0);
                s2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf[g2][j], cb2, s2, 0, 0, 0);
            }
            nb1[g2] = s1; nb2[g2] = s2;
        }
    }
    // the four constants must live in VGPRs for v_and_or_b32 to be selected: route them through a
    // lane permute (identity), whose result the compiler treats as a per-lane value
    auto to_vgpr = [&](uint32_t v) { return (uint32_t)__builtin_amdgcn_ds_bpermute(lane << 2, (int)v); };
    const DequantConsts dq = {to_vgpr(a.m_lo), to_vgpr(a.m_hi), to_vgpr(a.k_lo), to_vgpr(a.k_hi)};

    // ---- stream the tiles: three register stages, two tiles in flight while one is used -----
    const int n_in_tile = lane & 15, tq = lane >> 4;
    const __amdgpu_buffer_rsrc_t yr = make_rsrc(a.Y, (uint32_t)(((size_t)(a.T - 1) * a.ldy + a.N) * 2));
    const __amdgpu_buffer_rsrc_t pr = make_rsrc(a.partial, SPLIT ? (uint32_t)((size_t)a.KS * a.T * a.N * 4) : 0u);
    const __amdgpu_buffer_rsrc_t br = make_rsrc(a.bias, a.bias ? (uint32_t)a.N * 2u : 0u);      // no bias: reads 0
    auto emit = [&](const Stage &stg, int tile) {
        float4v tot = tile_dot<T1>(stg, xf, nb1, nb2, dq);
        const uint32_t n = (uint32_t)tile * kTileN + n_in_tile;
        if constexpr (!SPLIT) {
            union { uint16_t u; _Float16 h; } bb;
            bb.u = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(br, tile >= 0 ? (int)(n * 2u) : (int)kOob, 0, 0);
            const float bv = (float)bb.h;
#pragma unroll
            for (int r = 0; r < (T1 ? 1 : 4); ++r) {
                int t = tq * 4 + r;
                union { _Float16 h; uint16_t u; } o; o.h = (_Float16)(tot[r] + bv);
                uint32_t off = (tile >= 0 && t < a.T) ? (uint32_t)(((size_t)t * a.ldy + n) * 2) : kOob;
                __builtin_amdgcn_raw_buffer_store_b16(o.u, yr, (int)off, 0, 0);
            }
        } else {
#pragma unroll
            for (int r = 0; r < (T1 ? 1 : 4); ++r) {
                int t = tq * 4 + r;
                uint32_t bits = __float_as_uint(tot[r]);
                if ((bits << 1) == 0u) bits = 0x80000000u;      // +-0 is stored as -0: 0 means "empty"
                uint32_t off = (tile >= 0 && t < a.T) ? (uint32_t)((((size_t)ks * a.T + t) * a.N + n) * 4) : kOob;
                __builtin_amdgcn_raw_buffer_store_b32(bits, pr, (int)off, 0, kAuxSc1);
            }
        }
    };
    // Fully unrolled (n_iter <= decode_max_iter(W), guaranteed by the host): straight-line code with uniform
    // early exits and no back edge, so the waits inserted by the compiler are exact - a stage is
    // awaited while the two younger ones stay in flight.
#pragma unroll
    for (int i = 0; i < decode_max_iter(W); i += 3) {
        load_stage(blob, a, tile_of(i + 2), ks, lane, st2);
        emit(st0, tile_of(i));
        if (i + 1 >= n_iter) break;
        load_stage(blob, a, tile_of(i + 3), ks, lane, st0);
        emit(st1, tile_of(i + 1));
        if (i + 2 >= n_iter) break;
        load_stage(blob, a, tile_of(i + 4), ks, lane, st1);
        emit(st2, tile_of(i + 2));
        if (i + 3 >= n_iter) break;
    }

    // ---- split-K: exchange with the other K-slices of this output range ----------------------
    if constexpr (SPLIT) splitk_reduce(a, a.KS, ks, tile_lo, tile_hi, s_red);
}

template <int K, bool SPLIT, bool T1, int W = kDecWaves>
__global__ __launch_bounds__(W * 64) void decode_kernel(DecodeArgs a)
{
    __shared__ _Float16 s_x[16][kSliceCh + kXPad];
    __shared__ float s_red[kReduceWords];
    decode_body<K, SPLIT, T1, W>(a, blockIdx.x, blockIdx.y, s_x, s_red);
}

// Several linears that read the same activations, each with its own transform (every linear of
// the method has its own pairs, angles and scales - q / k / v or gate / up of a decoder layer),
// in one launch: the block rows (blockIdx.y) are divided among the parts, and a block runs the
// single-linear body on its part's arguments.
constexpr int kMaxParts = 4;
struct MultiArgs {
    DecodeArgs part[kMaxParts];
    int nb_end[kMaxParts];      // block rows [nb_end[p-1], nb_end[p]) belong to part p
    int n_parts;
};

template <int K, bool SPLIT, bool T1>
__global__ __launch_bounds__(kDecThreads) void decode_multi_kernel(MultiArgs m)
{
    __shared__ _Float16 s_x[16][kSliceCh + kXPad];
    __shared__ float s_red[kReduceWords];
    const int by = blockIdx.y;
    int p = 0, lo = 0;
#pragma unroll
    for (int q = 0; q + 1 < kMaxParts; ++q)
        if (q + 1 < m.n_parts && by >= m.nb_end[q]) { p = q + 1; lo = m.nb_end[q]; }
    decode_body<K, SPLIT, T1>(m.part[p], blockIdx.x, by - lo, s_x, s_red);
}

// target_blocks > 0: block budget given by the caller (one part of a multi-linear launch)
DecodeGeometry decode_geometry(int c_in, int c_out, int T, int target_blocks)
{
    DecodeGeometry d;
    int G = c_in / kGroup, NT = c_out / kTileN;
    d.ks = G / kSliceGroups;
    // measured: with many K-slices (few tiles per slice and block) one 8-wave block per CU beats
    // two 4-wave blocks (14336 -> 4096, one token: 10.4 against 11.2 us); single launches only
    // ... and so does, by a little, a long stream whose 8-wave blocks still fit one round
    // (4096 -> 28672: 14.65 against 14.9 us); the small linears are faster with 4 waves
    const bool many_slices = d.ks >= 16, big = packed_tiles_bytes(c_in, c_out) >= (24u << 20);
    // (the 8-wave kernel exists in its split-K form only: never with a single K-slice)
    d.waves = (T == 1 && d.ks > 1 && (many_slices || big) && target_blocks == 0) ? 2 * kDecWaves : kDecWaves;
    // measured on MI355X: one 4-wave block per CU for the small linears (the prologue is repeated
    // less often), two per CU once the weight stream exceeds ~24 MB
    int target = target_blocks;
    if (target <= 0) target = packed_tiles_bytes(c_in, c_out) >= (24u << 20) ? 512 : 256;
    if (d.waves > kDecWaves) target = 256;
    int nb = target / d.ks;
    if (nb < 1) nb = 1;
    int tpb = (NT + nb - 1) / nb;
    tpb = (tpb + d.waves - 1) / d.waves * d.waves;           // whole rounds of the block's waves
    if (tpb > decode_max_iter(d.waves) * d.waves) tpb = decode_max_iter(d.waves) * d.waves;
    d.tiles_per_block = tpb;
    d.nb = (NT + tpb - 1) / tpb;
    if (d.waves > kDecWaves && d.ks * d.nb > 256) {           // would not fit one round of 8-wave blocks
        d.waves = kDecWaves;
        target = packed_tiles_bytes(c_in, c_out) >= (24u << 20) ? 512 : 256;
        nb = target / d.ks;
        if (nb < 1) nb = 1;
        tpb = (NT + nb - 1) / nb;
        tpb = (tpb + d.waves - 1) / d.waves * d.waves;
        if (tpb > decode_max_iter(d.waves) * d.waves) tpb = decode_max_iter(d.waves) * d.waves;
        d.tiles_per_block = tpb;
        d.nb = (NT + tpb - 1) / tpb;
    }
    int t16 = T < 16 ? T : 16;
    d.partial_bytes = d.ks > 1 ? (size_t)d.ks * t16 * c_out * sizeof(float) : 0;
    return d;
}

template <int K>
static hipError_t launch_decode_k(const DecodeArgs &a, const DecodeGeometry &d, hipStream_t s)
{
    const dim3 grid(d.ks, d.nb), block(d.waves * 64);
    if (d.waves == 2 * kDecWaves) {      // only chosen for one token and more than one K-slice (decode_geometry)
        hipLaunchKernelGGL((decode_kernel<K, true, true, 2 * kDecWaves>), grid, block, 0, s, a);
        return hipGetLastError();
    }
    if (a.T == 1) {
        if (d.ks > 1) hipLaunchKernelGGL((decode_kernel<K, true, true>), grid, block, 0, s, a);
        else          hipLaunchKernelGGL((decode_kernel<K, false, true>), grid, block, 0, s, a);
    } else {
        if (d.ks > 1) hipLaunchKernelGGL((decode_kernel<K, true, false>), grid, block, 0, s, a);
        else          hipLaunchKernelGGL((decode_kernel<K, false, false>), grid, block, 0, s, a);
    }
    return hipGetLastError();
}

static hipError_t fill_decode_args(DecodeArgs &a, DecodeGeometry &d, const paro_rotation *rot, const paro_w4_weight &w,
                                   const paro_half_t *X, int64_t ldx, paro_half_t *Y, int64_t ldy, int T, void *ws,
                                   size_t partial_off, int target_blocks = 0)
{
    if (!rot || !rot->plan) return hipErrorInvalidValue;
    d = decode_geometry(w.c_in, w.c_out, T, target_blocks);
    if (d.ks > kReduceWords) return hipErrorInvalidValue;
    if (packed_blob_bytes(w.c_in, w.c_out) >= (1ull << 31)) return hipErrorInvalidValue;   // 32-bit buffer offsets (checked by the caller)
    a.blob = w.packed;
    a.scales_off = (uint32_t)packed_tiles_bytes(w.c_in, w.c_out);
    a.zeros_off = a.scales_off + (uint32_t)packed_scales_bytes(w.c_in, w.c_out);
    a.blob_bytes = a.zeros_off + (uint32_t)packed_zeros_bytes(w.c_in, w.c_out);
    a.X = (const _Float16 *)X; a.ldx = ldx; a.Y = (_Float16 *)Y; a.ldy = ldy;
    a.bias = (const _Float16 *)w.bias;
    a.plan = (const uint32_t *)rot->plan;
    a.partial = (float *)((char *)ws + kWsPartialOff + partial_off);
    a.err = (uint32_t *)ws + kWsErrorWord;
    a.T = T; a.C = w.c_in; a.N = w.c_out; a.G = w.c_in / kGroup; a.NT = w.c_out / kTileN; a.KS = d.ks;
    a.tiles_per_block = d.tiles_per_block;
    a.m_lo = 0x000F000Fu; a.m_hi = 0x00F000F0u; a.k_lo = 0x64006400u; a.k_hi = 0x54005400u;
    return hipSuccess;
}

hipError_t launch_decode(const paro_rotation *rot, const paro_w4_weight &w, const paro_half_t *X, int64_t ldx,
                         paro_half_t *Y, int64_t ldy, int T, void *ws, hipStream_t s)
{
    DecodeArgs a;
    DecodeGeometry d;
    hipError_t e = fill_decode_args(a, d, rot, w, X, ldx, Y, ldy, T, ws, 0);
    if (e != hipSuccess) return e;
    switch (rot->n_layers) {
    case 0: return launch_decode_k<0>(a, d, s);
    case 1: return launch_decode_k<1>(a, d, s);
    case 2: return launch_decode_k<2>(a, d, s);
    case 3: return launch_decode_k<3>(a, d, s);
    case 4: return launch_decode_k<4>(a, d, s);
    case 5: return launch_decode_k<5>(a, d, s);
    case 6: return launch_decode_k<6>(a, d, s);
    case 7: return launch_decode_k<7>(a, d, s);
    default: return launch_decode_k<8>(a, d, s);
    }
}

template <int K>
static hipError_t launch_multi_k(const MultiArgs &m, int ks, int nb_total, int T, hipStream_t s)
{
    const dim3 grid(ks, nb_total), block(kDecThreads);
    if (T == 1) {
        if (ks > 1) hipLaunchKernelGGL((decode_multi_kernel<K, true, true>), grid, block, 0, s, m);
        else        hipLaunchKernelGGL((decode_multi_kernel<K, false, true>), grid, block, 0, s, m);
    } else {
        if (ks > 1) hipLaunchKernelGGL((decode_multi_kernel<K, true, false>), grid, block, 0, s, m);
        else        hipLaunchKernelGGL((decode_multi_kernel<K, false, false>), grid, block, 0, s, m);
    }
    return hipGetLastError();
}

// The parts of one launch share the block budget of a single linear of their combined size, in
// proportion to their outputs.
static int multi_part_target(int n_parts, const paro_w4_weight *const *w, int p)
{
    size_t n_all = 0;
    for (int q = 0; q < n_parts; ++q) n_all += (size_t)w[q]->c_out;
    const int target = packed_tiles_bytes(w[0]->c_in, (int)n_all) >= (24u << 20) ? 512 : 256;
    const int ks = w[p]->c_in / kGroup / kSliceGroups;
    int mine = (int)(((size_t)target * w[p]->c_out + n_all / 2) / n_all);
    return mine < ks ? ks : mine;
}

// workspace of the one-launch path: the parts' split-K partials one after the other
size_t decode_multi_bytes(int n_parts, const paro_w4_weight *const *w, int T)
{
    size_t total = 0;
    for (int p = 0; p < n_parts; ++p)
        total += (decode_geometry(w[p]->c_in, w[p]->c_out, T, multi_part_target(n_parts, w, p)).partial_bytes + 255) / 256 * 256;
    return total;
}

// All parts: same c_in and layer count, plan and repacked weight present, T <= 4.
hipError_t launch_decode_multi(int n_parts, const paro_rotation *const *rot, const paro_w4_weight *const *w,
                               const paro_half_t *X, int64_t ldx, paro_half_t *const *Y, const int64_t *ldy, int T,
                               void *ws, hipStream_t s)
{
    if (n_parts < 1 || n_parts > kMaxParts) return hipErrorInvalidValue;
    MultiArgs m;
    m.n_parts = n_parts;
    int nb_total = 0, ks = 0;
    size_t off = 0;
    for (int p = 0; p < n_parts; ++p) {
        DecodeGeometry d;
        hipError_t e = fill_decode_args(m.part[p], d, rot[p], *w[p], X, ldx, Y[p], ldy[p], T, ws, off,
                                        multi_part_target(n_parts, w, p));
        if (e != hipSuccess) return e;
        if (p && (d.ks != ks || rot[p]->n_layers != rot[0]->n_layers)) return hipErrorInvalidValue;
        ks = d.ks;
        nb_total += d.nb;
        m.nb_end[p] = nb_total;
        off += (d.partial_bytes + 255) / 256 * 256;
    }
    for (int p = n_parts; p < kMaxParts; ++p) { m.part[p] = m.part[0]; m.nb_end[p] = nb_total; }
    switch (rot[0]->n_layers) {
    case 0: return launch_multi_k<0>(m, ks, nb_total, T, s);
    case 1: return launch_multi_k<1>(m, ks, nb_total, T, s);
    case 2: return launch_multi_k<2>(m, ks, nb_total, T, s);
    case 3: return launch_multi_k<3>(m, ks, nb_total, T, s);
    case 4: return launch_multi_k<4>(m, ks, nb_total, T, s);
    case 5: return launch_multi_k<5>(m, ks, nb_total, T, s);
    case 6: return launch_multi_k<6>(m, ks, nb_total, T, s);
    case 7: return launch_multi_k<7>(m, ks, nb_total, T, s);
    default: return launch_multi_k<8>(m, ks, nb_total, T, s);
    }
}

// ------------------------------------------------------------------------------------------
// Generic linear on the interchange layout: one wave per output row, plain fp32 FMAs.
// Slow; used when no repacked blob was supplied.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void linear_generic_kernel(const uint32_t *__restrict__ qweight,
                                                             const _Float16 *__restrict__ scales,
                                                             const uint32_t *__restrict__ qzeros,
                                                             const _Float16 *__restrict__ bias, int C, int N,
                                                             const _Float16 *__restrict__ X, int64_t ldx,
                                                             _Float16 *__restrict__ Y, int64_t ldy, int T)
{
    const int lane = threadIdx.x & 63;
    const size_t n = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= (size_t)N) return;
    const int words = C / 8;
    for (int t0 = 0; t0 < T; t0 += 4) {
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int wi = lane; wi < words; wi += 64) {
            uint32_t w = qweight[n * words + wi];
            int g = wi / 16;
            float s = (float)scales[(size_t)g * N + n];
            int z = (int)((qzeros[(size_t)g * (N / 8) + n / 8] >> (4 * (n % 8))) & 15u);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float wv = (float)((int)((w >> (4 * e)) & 15u) - z) * s;
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (t0 + u < T) acc[u] += wv * (float)X[(size_t)(t0 + u) * ldx + (size_t)wi * 8 + e];
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float v = acc[u];
            for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
            if (lane == 0 && t0 + u < T) Y[(size_t)(t0 + u) * ldy + n] = (_Float16)(v + (bias ? (float)bias[n] : 0.f));
        }
    }
}

hipError_t launch_linear_generic(const paro_w4_weight &w, const paro_half_t *X, int64_t ldx, paro_half_t *Y,
                                 int64_t ldy, int T, hipStream_t s)
{
    hipLaunchKernelGGL(linear_generic_kernel, dim3((w.c_out + 3) / 4), dim3(256), 0, s, w.qweight,
                       (const _Float16 *)w.scales, w.qzeros, (const _Float16 *)w.bias, w.c_in, w.c_out,
                       (const _Float16 *)X, ldx, (_Float16 *)Y, ldy, T);
    return hipGetLastError();
}

}  // namespace paro
