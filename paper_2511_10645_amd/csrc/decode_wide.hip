// Decode-side bare W4A16 linear, 1..16 tokens per pass (17..32 in decode_wide2_kernel below): a block takes ALL K-slices of its tile
// range, one 512-channel slice per wave (up to 12 waves = 6144 channels; beyond that the slices
// are spread evenly over several blocks of at most 8 waves and only those few partial sums are
// exchanged between blocks); the waves' partial tiles are summed through LDS, so layers up to
// 6144 channels need no exchange between blocks at all.
//
// Stream.  Every wave keeps NS = 3 weight stages (one 16 x 512 tile slice each: 4 KB of codes plus
// scales and zero points) in registers: two are in flight while the third is multiplied, and the
// request for the next tile is issued before the multiplication of the current one starts.
// Deeper staging was measured and is slower on this part (gate/up 4096 -> 28672, one token:
// 12.6 us with 3 stages, 13.0 with 4, 14.4 with 6): what bounds the stream is not the number of
// bytes a wave has requested.  Nor is it the order of the tiles: a walk in which the blocks of the
// grid read one contiguous window of the blob at any moment (tiles nb, nb + grid, ...) is no faster.  One block per compute unit; for one token the partial sums of a
// tile take 64 bytes of LDS per wave, so a block can run up to 16 tiles per wave and every shape
// of the benchmark fits one round of blocks.
//
// The transform.  Several tokens: it cannot be hosted here at a profit.  Measured: the rotation units dealt out to
// the first waves of the grid, results published through agent-scope stores and fetched by every wave with
// agent-scope loads (self-flagging words, no fences) costs +5 us per launch at one token and +6..8 us at 16, more
// than a separate rotation launch (+3 us): vector memory returns in order for the whole compute unit, so a poll
// waits behind every weight tile the unit has requested, and throttling the requests until the activations have
// arrived delays the stream by the same time.  Hence 2..4 tokens the K-major kernel (decode.hip), whose blocks rotate
// only their own slice; 5..16 tokens a rotation pass, then this kernel.  One token: a wave needs the transformed
// activations of its own K-slice only, and produces them itself (ROTK below) - used where the weight stream is long
// enough to hide that prologue, the K-major kernel elsewhere.
#include "decode_common.h"
#include <algorithm>
#include <type_traits>

namespace paro {

// most tiles per wave (the stream loop is unrolled): one token keeps 64 B of partial sums per tile
// and wave in LDS, several tokens 1 KB (the launcher also keeps the block's total within the LDS)
__host__ __device__ constexpr int wide_max_tiles(bool one_token) { return one_token ? 16 : 14; }
constexpr size_t kWideLdsBytes = 160 * 1024;
constexpr int kWideStages = 3;
constexpr int kWideWaves = 12;                  // most K-slices (waves) of one block
constexpr int kWideMaxTokens = 32;              // tokens of one pass: 16 per token block, one or two blocks per wave

// f(0), f(1), ... while f returns true, at most N times; nested, so that stopping is ONE forward jump
// past all remaining steps (instruction fetch matters at these kernel durations)
template <int N, class F, int I = 0>
__device__ __forceinline__ void static_while(F &&f)
{
    if constexpr (I < N) {
        if (f(std::integral_constant<int, I>{})) static_while<N, F, I + 1>(static_cast<F &&>(f));
    }
}

// Activation fragments of several tokens.  An MFMA A fragment wants, per lane, 16 bytes of token lane % 16 at
// channel offset 32 (lane / 16) + 8 j: loaded straight from X, one instruction touches 32 cache lines (16 rows x 2)
// and uses 32 bytes of each, and the compute unit's vector-memory path, which takes a cache line per cycle, spends
// 2 us per launch on a 16-token input of 4096 channels (128 KB per block) before the first weight tile can be
// multiplied.  Instead every instruction reads 4 token rows x 256 contiguous bytes (8 full lines), the wave parks
// the 16 x 128 sub-block in a private LDS area (rows padded to 272 bytes: the 16-byte accesses of both directions
// are conflict-free) and reads its fragments from there.  Measured, bare linear at 16 tokens: 4096 -> 6144
// 8.0 -> 6.3 us, 4096 -> 4096 7.4 -> 5.3 us.  No block barrier: the area is private to the wave and LDS operations
// of one wave execute in issue order.
constexpr int kXsRowBytes = kGroup * 2 + 16;
constexpr int kXsWords = 16 * kXsRowBytes / 4;      // 1088 floats per wave
template <int TB>
__device__ __forceinline__ void load_x_fragments(const DecodeArgs &a, int ks, bool slice_ok, int lane, char *xs,
                                                 half8 (&xf)[TB][kSliceGroups][4])
{
    const __amdgpu_buffer_rsrc_t xr = make_rsrc(a.X, (uint32_t)(((size_t)(a.T - 1) * a.ldx + a.C) * 2));
    const int lr = lane >> 4, lc = lane & 15;
    u32x4 raw[TB][kSliceGroups][4];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int t = tb * 16 + q * 4 + lr;
            const uint32_t off = (t < a.T && slice_ok) ? (uint32_t)(((size_t)t * a.ldx + (size_t)ks * kSliceCh) * 2 + lc * 16) : kOob;
#pragma unroll
            for (int g2 = 0; g2 < kSliceGroups; ++g2)
                raw[tb][g2][q] = __builtin_amdgcn_raw_buffer_load_b128(xr, (int)(off + g2 * kGroup * 2), 0, 0);
        }
    const int ft = lane & 15, fkb = lane >> 4;
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int g2 = 0; g2 < kSliceGroups; ++g2) {
#pragma unroll
            for (int q = 0; q < 4; ++q) *(u32x4 *)(xs + (q * 4 + lr) * kXsRowBytes + lc * 16) = raw[tb][g2][q];
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int j = 0; j < 4; ++j) xf[tb][g2][j] = *(const half8 *)(xs + ft * kXsRowBytes + fkb * 64 + j * 16);
            __builtin_amdgcn_wave_barrier();
        }
}

// ROTK > 0 (one token only): the transform of Eq. 8 with ROTK rotation layers is hosted.  A wave owns one K-slice,
// so it needs the transformed activations of that slice only - its 4 groups - and produces them itself: no
// hand-over between waves, no block barrier, and nothing is exchanged between blocks that the bare kernel would
// not exchange.  The 4 groups are rotated side by side (their chains of 4 multiply-adds and a permute are
// independent) from the compact copy of the plan (4 bytes per lane and layer: 44 registers hold all of it, so
// every plan row is requested before the first weight stage and none waits behind a weight tile - vector memory
// returns in order; sine and cosine come from the hardware functions, which fill the permutes' latency), and the
// first weight stages are in flight the whole time: what the launch pays for the transform is one 4-wide rotation
// (~0.7 us) where the stream is too short to hide it, and next to nothing in front of a long stream.  Every block
// repeats the work of its column of K-slices (the compact plan, 22 bytes per channel, comes out of L2 for all but
// the first), which is what makes this form unsuitable for more than one token.
// MAXW: most waves per block (8: two waves per SIMD and 256 registers; otherwise kWideWaves).
constexpr int kRotStageWords = kSliceCh / 2;     // the slice's 512 fp16 activations of one token, in floats

template <bool SPLIT, bool T1, int ROTK = 0, int MAXW = kWideWaves>
__global__ __launch_bounds__(MAXW * 64) void decode_wide_kernel(DecodeArgs a)
{
    static_assert(ROTK == 0 || T1, "the hosted transform is for one token");
    constexpr int NS = kWideStages;
    // [waves][tiles per block] partial tiles | kReduceWords reduce scratch
    extern __shared__ __attribute__((aligned(16))) float s_wide[];
    const int kb = blockIdx.x, nb = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw = blockDim.x >> 6;                                        // K-slices (waves) per block
    const int ks = kb * nw + wave;
    const bool slice_ok = ks < a.KS;
    const int tile_lo = nb * a.tiles_per_block;
    const int tile_hi = min(a.NT, tile_lo + a.tiles_per_block);
    const int n_iter = tile_hi - tile_lo;
    auto tile_of = [&](int i) { return (i < n_iter && slice_ok) ? tile_lo + i : -1; };
    const __amdgpu_buffer_rsrc_t blob = make_rsrc(a.blob, a.blob_bytes);
    constexpr int kTileWords = T1 ? kTileN : 256;
    // a wave's partial tiles are contiguous; several tokens: the same area first parks its activations
    const int wstride = ROTK > 0 ? max(a.tiles_per_block * kTileWords, kRotStageWords)
                        : T1     ? a.tiles_per_block * kTileWords
                                 : max(a.tiles_per_block * kTileWords, kXsWords);
    float *s_mine = s_wide + (size_t)wave * wstride;
    float *s_red = s_wide + (size_t)nw * wstride;

    Stage st[NS];
    half8 xf[kSliceGroups][4];
    const int ft = lane & 15, fkb = lane >> 4;
    if constexpr (ROTK > 0) {
        constexpr int K = ROTK;
        const int ksp = slice_ok ? ks : 0;                                   // a surplus wave repeats slice 0 (its tiles are empty)
        _Float16 *sx = (_Float16 *)s_mine;                                   // the slice of the token, 512 fp16
        const __amdgpu_buffer_rsrc_t xr = make_rsrc(a.X, (uint32_t)a.C * 2u);
        uint32_t xin[kSliceGroups];
#pragma unroll
        for (int g2 = 0; g2 < kSliceGroups; ++g2)
            xin[g2] = __builtin_amdgcn_raw_buffer_load_b32(xr, (int)(((size_t)ksp * kSliceCh + g2 * kGroup + 2 * lane) * 2), 0, 0);
        // the compact plan of the slice's 4 groups: 3 + K dwords per lane and group, all requested at once
        const uint32_t *cplan = a.plan + (size_t)ksp * kSliceGroups * plan_compact_group_dwords(K) + lane;
        uint32_t io[kSliceGroups], sci[kSliceGroups], sco[kSliceGroups], pm[kSliceGroups][K];
#pragma unroll
        for (int g2 = 0; g2 < kSliceGroups; ++g2) {
            const uint32_t *gp = cplan + (size_t)g2 * plan_compact_group_dwords(K);
            io[g2] = gp[0]; sci[g2] = gp[64]; sco[g2] = gp[128];
#pragma unroll
            for (int l = 0; l < K; ++l) pm[g2][l] = gp[(kPlanCompactHeadRows + l) * 64];
        }
        // the weight stream starts here, behind the plan and the activations (vector memory returns in order)
#pragma unroll
        for (int s = 0; s + 1 < NS; ++s) load_stage(blob, a, tile_of(s), ks, lane, st[s]);
#pragma unroll
        for (int g2 = 0; g2 < kSliceGroups; ++g2) *(uint32_t *)&sx[g2 * kGroup + 2 * lane] = xin[g2];
        __builtin_amdgcn_wave_barrier();
        // the 4 groups side by side: their chains (4 multiply-adds, then a permute that takes far longer) are independent
        float va[kSliceGroups], vb[kSliceGroups];
#pragma unroll
        for (int g2 = 0; g2 < kSliceGroups; ++g2) {
            va[g2] = (float)sx[g2 * kGroup + (io[g2] & 0xff)] * (float)as_h2(sci[g2])[0];
            vb[g2] = (float)sx[g2 * kGroup + ((io[g2] >> 8) & 0xff)] * (float)as_h2(sci[g2])[1];
        }
#pragma unroll
        for (int l = 0; l < K; ++l) {
#pragma unroll
            for (int g2 = 0; g2 < kSliceGroups; ++g2) {
                const uint32_t m = pm[g2][l];
                const float rev = (float)(m >> 8) * (1.0f / 16777216.0f);      // exact: 24 bits
                const float c = __builtin_amdgcn_cosf(rev), sn = __builtin_amdgcn_sinf(rev);
                const float na = c * va[g2] - sn * vb[g2], nb2 = c * vb[g2] + sn * va[g2];
                va[g2] = na;
                vb[g2] = (l + 1 < K) ? __int_as_float(__builtin_amdgcn_ds_bpermute((int)(m & 0xffu), __float_as_int(nb2))) : nb2;
            }
        }
        // every lane has read its inputs: the staging rows take the results
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int g2 = 0; g2 < kSliceGroups; ++g2) {
            sx[g2 * kGroup + ((io[g2] >> 16) & 0xff)] = (_Float16)(va[g2] * (float)as_h2(sco[g2])[0]);
            sx[g2 * kGroup + (io[g2] >> 24)] = (_Float16)(vb[g2] * (float)as_h2(sco[g2])[1]);
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int g2 = 0; g2 < kSliceGroups; ++g2)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
                if (ft == 0) v = *(const half8 *)&sx[g2 * kGroup + fkb * 32 + j * 8];
                xf[g2][j] = v;
            }
        __builtin_amdgcn_wave_barrier();                                      // the area holds partial sums from here on
    } else if constexpr (!T1) {
        half8 xt[1][kSliceGroups][4];
        load_x_fragments<1>(a, ks, slice_ok, lane, (char *)s_mine, xt);
#pragma unroll
        for (int g2 = 0; g2 < kSliceGroups; ++g2)
#pragma unroll
            for (int j = 0; j < 4; ++j) xf[g2][j] = xt[0][g2][j];
#pragma unroll
        for (int s = 0; s + 1 < NS; ++s) load_stage(blob, a, tile_of(s), ks, lane, st[s]);
    } else {
        const __amdgpu_buffer_rsrc_t xr = make_rsrc(a.X, (uint32_t)(((size_t)(a.T - 1) * a.ldx + a.C) * 2));
        const uint32_t xoff = (ft < a.T && slice_ok) ? (uint32_t)(((size_t)ft * a.ldx + (size_t)ks * kSliceCh + fkb * 32) * 2) : kOob;
#pragma unroll
        for (int g2 = 0; g2 < kSliceGroups; ++g2)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                union { u32x4 u; half8 h; } v;
                v.u = __builtin_amdgcn_raw_buffer_load_b128(xr, (int)(xoff + (g2 * kGroup + j * 8) * 2), 0, 0);
                xf[g2][j] = v.h;
            }
#pragma unroll
        for (int s = 0; s + 1 < NS; ++s) load_stage(blob, a, tile_of(s), ks, lane, st[s]);
    }
    // per token and group: nb1 = -sum_k b_k x'_k, nb2 = -sum_k x'_k (see tile_dot)
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
    auto to_vgpr = [&](uint32_t v) { return (uint32_t)__builtin_amdgcn_ds_bpermute(lane << 2, (int)v); };
    const DequantConsts dq = {to_vgpr(a.m_lo), to_vgpr(a.m_hi), to_vgpr(a.k_lo), to_vgpr(a.k_hi)};

    // partial tile of (tile i of the block, this wave).  More than one token: element lane*4 + r <-> token
    // 4*(lane/16)+r, row lane%16 (1 KB per tile and wave); one token: the 16 rows only (64 B)
    auto emit = [&](const Stage &stg, int i) {
        float4v tot = tile_dot<T1>(stg, xf, nb1, nb2, dq);
        float *dst = s_mine + i * kTileWords;
        if constexpr (T1) { if (lane < 16) dst[lane] = tot[0]; }
        else *(float4v *)(dst + lane * 4) = tot;
    };
    // Fully unrolled (n_iter <= MAXI, guaranteed by the launcher): straight-line code with one uniform
    // early exit and no back edge, so every wait inserted by the compiler names exactly the stage it
    // needs and the younger ones stay in flight.  (A rolled loop makes the compiler wait for all but
    // the newest load at the back edge; skipping the unused steps one by one instead of with one jump
    // costs 0.3-0.7 us per launch in instruction fetches.)
    constexpr int MAXI = wide_max_tiles(T1);
    static_while<MAXI>([&](auto I) {
        constexpr int i = I;
        if (i >= n_iter) return false;
        // the request for tile i + NS - 1 goes out before tile i is multiplied: NS - 1 stages in flight
        load_stage(blob, a, tile_of(i + NS - 1), ks, lane, st[(i + NS - 1) % NS]);
        emit(st[i % NS], i);
        return true;
    });
    __syncthreads();
    // ---- sum the K-slices; outputs indexed (i, t, n) with n fastest for coalesced stores -----
    const int per_tile = a.T * kTileN;
    for (int idx = threadIdx.x; idx < n_iter * per_tile; idx += blockDim.x) {
        const int i = idx / per_tile, rem = idx % per_tile;
        const int t = rem / kTileN, nn = rem % kTileN;
        const int e = T1 ? nn : ((t >> 2) * 16 + nn) * 4 + (t & 3);
        float sum = 0.f;
        for (int w = 0; w < nw; ++w) sum += s_wide[(size_t)w * wstride + i * kTileWords + e];
        const size_t n = (size_t)(tile_lo + i) * kTileN + nn;
        if constexpr (!SPLIT) {
            if (a.bias) sum += (float)a.bias[n];
            a.Y[(size_t)t * a.ldy + n] = (_Float16)sum;
        } else {
            uint32_t bits = __float_as_uint(sum);
            if ((bits << 1) == 0u) bits = 0x80000000u;
            __hip_atomic_store((uint32_t *)(a.partial + ((size_t)kb * a.T + t) * a.N + n), bits, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if constexpr (SPLIT) splitk_reduce(a, gridDim.x, kb, tile_lo, tile_hi, s_red);
}

// ------------------------------------------------------------------------------------------
// 17..32 tokens in ONE pass over the weights: the same block / wave / stream structure with two blocks of 16
// tokens per wave.  Two sets of activation fragments fill half the register file, so the zero-point trick of
// tile_dot (two more sums per token block and group) does not fit; the zero point is subtracted from the codes
// instead ( q - z, exact in fp16: 9 vector instructions per 8 weights instead of 5 ), once per tile for both token
// blocks, and the scale of a group multiplies its fp32 sums as in tile_dot.
// ------------------------------------------------------------------------------------------
constexpr int kWide2MaxTiles = 9;
constexpr int kWide2Waves = 8;                   // 2 waves per SIMD: the two sets of activation fragments need 256 registers

template <bool SPLIT>
__global__ __launch_bounds__(kWide2Waves * 64) void decode_wide2_kernel(DecodeArgs a)
{
    constexpr int NS = kWideStages;
    extern __shared__ __attribute__((aligned(16))) float s_wide[];       // [waves][tiles per block][2][256] | reduce scratch
    const int kb = blockIdx.x, nb = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw = blockDim.x >> 6;
    const int ks = kb * nw + wave;
    const bool slice_ok = ks < a.KS;
    const int tile_lo = nb * a.tiles_per_block;
    const int tile_hi = min(a.NT, tile_lo + a.tiles_per_block);
    const int n_iter = tile_hi - tile_lo;
    auto tile_of = [&](int i) { return (i < n_iter && slice_ok) ? tile_lo + i : -1; };
    const __amdgpu_buffer_rsrc_t blob = make_rsrc(a.blob, a.blob_bytes);
    const int wstride = max(a.tiles_per_block * 512, kXsWords);
    float *s_mine = s_wide + (size_t)wave * wstride;
    float *s_red = s_wide + (size_t)nw * wstride;

    Stage st[NS];
    half8 xf[2][kSliceGroups][4];
    load_x_fragments<2>(a, ks, slice_ok, lane, (char *)s_mine, xf);
#pragma unroll
    for (int s = 0; s + 1 < NS; ++s) load_stage(blob, a, tile_of(s), ks, lane, st[s]);
    auto to_vgpr = [&](uint32_t v) { return (uint32_t)__builtin_amdgcn_ds_bpermute(lane << 2, (int)v); };
    const DequantConsts dq = {to_vgpr(a.m_lo), to_vgpr(a.m_hi), to_vgpr(a.k_lo), to_vgpr(a.k_hi)};
    // B holds q - z exactly (the code or-ed into the mantissa of 1024 or 64, minus 1024 + z or 64 + z: 9 vector
    // instructions per 8 weights); the group's scale multiplies the fp32 sums of the group, once per tile.
    auto emit = [&](const Stage &stg, int i) {
        float4v tot[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
        union { uint2 v; _Float16 h[4]; } sc; sc.v = stg.sc;
#pragma unroll
        for (int gi = 0; gi < kSliceGroups; ++gi) {
            const uint32_t z = (stg.zq >> (4 * gi)) & 15u;
            const half2v nlo = as_h2((0xE400u + z) * 0x00010001u);          // -(1024 + z), twice
            const half2v nhi = as_h2((0xD400u + (z << 4)) * 0x00010001u);   // -(64 + z), twice
            float4v acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t u = stg.w[gi][j], t = u >> 8;
                union { uint32_t d[4]; half8 h; } b;
                b.d[0] = as_u32(as_h2(and_or(u, dq.m_lo, dq.k_lo)) + nlo);
                b.d[1] = as_u32(as_h2(and_or(u, dq.m_hi, dq.k_hi)) + nhi);
                b.d[2] = as_u32(as_h2(and_or(t, dq.m_lo, dq.k_lo)) + nlo);
                b.d[3] = as_u32(as_h2(and_or(t, dq.m_hi, dq.k_hi)) + nhi);
                acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf[0][gi][j], b.h, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf[1][gi][j], b.h, acc[1], 0, 0, 0);
            }
            const float sg = (float)sc.h[gi];
            tot[0] += sg * acc[0];
            tot[1] += sg * acc[1];
        }
        float *dst = s_mine + i * 512;
        *(float4v *)(dst + lane * 4) = tot[0];
        *(float4v *)(dst + 256 + lane * 4) = tot[1];
    };
    static_while<kWide2MaxTiles>([&](auto I) {
        constexpr int i = I;
        if (i >= n_iter) return false;
        load_stage(blob, a, tile_of(i + NS - 1), ks, lane, st[(i + NS - 1) % NS]);
        emit(st[i % NS], i);
        return true;
    });
    __syncthreads();
    const int per_tile = a.T * kTileN;
    for (int idx = threadIdx.x; idx < n_iter * per_tile; idx += blockDim.x) {
        const int i = idx / per_tile, rem = idx % per_tile;
        const int t = rem / kTileN, nn = rem % kTileN;
        const int e = (t >> 4) * 256 + (((t & 15) >> 2) * 16 + nn) * 4 + (t & 3);
        float sum = 0.f;
        for (int w = 0; w < nw; ++w) sum += s_wide[(size_t)w * wstride + i * 512 + e];
        const size_t n = (size_t)(tile_lo + i) * kTileN + nn;
        if constexpr (!SPLIT) {
            if (a.bias) sum += (float)a.bias[n];
            a.Y[(size_t)t * a.ldy + n] = (_Float16)sum;
        } else {
            uint32_t bits = __float_as_uint(sum);
            if ((bits << 1) == 0u) bits = 0x80000000u;
            __hip_atomic_store((uint32_t *)(a.partial + ((size_t)kb * a.T + t) * a.N + n), bits, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if constexpr (SPLIT) splitk_reduce(a, gridDim.x, kb, tile_lo, tile_hi, s_red);
}

struct WideGeometry { int kb, nb, waves, tiles_per_block; size_t lds; };
static WideGeometry wide_geometry(int c_in, int c_out, int T, bool hosted = false)
{
    const bool two = T > 16;                                 // two blocks of 16 tokens per wave (decode_wide2_kernel)
    WideGeometry g;
    const int KS = c_in / kGroup / kSliceGroups, NT = c_out / kTileN;
    // up to 12 slices fit one block (3 waves per SIMD): no exchange between blocks at all.  Beyond
    // that the slices are spread evenly over blocks of at most 8 waves.
    g.kb = KS <= (two ? kWide2Waves : kWideWaves) ? 1 : (KS + 7) / 8;
    g.waves = (KS + g.kb - 1) / g.kb;
    int nb = 256 / g.kb;                                     // one block per compute unit
    if (nb < 1) nb = 1;
    int tpb = (NT + nb - 1) / nb;
    const int max_tiles = two ? kWide2MaxTiles : wide_max_tiles(T == 1);
    if (tpb > max_tiles) tpb = max_tiles;
    if (two && tpb * g.waves > 76) tpb = 76 / g.waves;         // 2 KB of LDS per (tile, wave)
    if (!two && T > 1) {                                     // 1 KB of LDS per (tile, wave), next to the reduce scratch
        const int fit = (int)((kWideLdsBytes - kReduceWords * sizeof(float)) / ((size_t)g.waves * 1024));
        if (tpb > fit) tpb = fit;
    }
    g.tiles_per_block = tpb;
    g.nb = (NT + tpb - 1) / tpb;
    const int tile_words = two ? 512 : T == 1 ? kTileN : 256;
    const int wstride = hosted ? std::max(tpb * tile_words, kRotStageWords)                // as in the kernels
                        : T == 1 ? tpb * tile_words : std::max(tpb * tile_words, kXsWords);
    g.lds = ((size_t)g.waves * wstride + kReduceWords) * sizeof(float);
    return g;
}

size_t decode_wide_partial_bytes(int c_in, int c_out, int T)
{
    WideGeometry g = wide_geometry(c_in, c_out, T);
    int tp = T < kWideMaxTokens ? T : kWideMaxTokens;
    return g.kb > 1 ? (size_t)g.kb * tp * c_out * sizeof(float) : 0;
}

// Whether the one-token kernel can host this transform (instantiated for the paper's 8 layers)
bool decode_wide_hosts(const paro_rotation &rot, int T) { return T == 1 && rot.plan && rot.n_layers == 8; }

// Whether it pays: every wave spends ~1.5 us on its 4 groups before it consumes its first tile, which its weight
// stream hides from about 4 tiles per wave on (6 where a block has more than 8 waves, three per SIMD).  Measured on
// MI355X, this kernel against the K-major kernel (or rotation pass + bare kernel where that is faster), us:
// 4096 -> 12288 (3 tiles per wave) 8.7 / 8.9, 4096 -> 16384 (4) 9.7 / 10.3, 4096 -> 28672 (7) 12.8 / 14.8,
// 2048 -> 28672 (7) 8.3 / 10.2, 14336 -> 4096 (4) 10.3 / 10.5, 14336 -> 8192 (8) 14.1 / 17.4, 8192 -> 8192 (4)
// 11.0 / 10.9, 27648 -> 5120 (9) 15.5 / 18.9, 5120 -> 55296 (14, 10 waves) 26.1 / 28.8; but 4096 -> 6144 (2)
// 7.5 / 6.8, 5120 -> 7168 (2) 9.1 / 7.9, 6144 -> 12288 (3, 12 waves) 11.9 / 11.5.
bool decode_wide_hosting_pays(int c_in, int c_out)
{
    const WideGeometry g = wide_geometry(c_in, c_out, 1, true);
    return g.tiles_per_block >= (g.waves <= 8 ? 4 : 6);
}

// ws: the exchange part of the workspace (may be NULL where no partial sums are exchanged).
// rot: NULL for the bare linear; otherwise a transform decode_wide_hosts() accepts, applied to X by the kernel itself.
hipError_t launch_decode_wide(const paro_w4_weight &w, const paro_half_t *X, int64_t ldx, paro_half_t *Y, int64_t ldy,
                              int T, void *ws, hipStream_t s, const paro_rotation *rot)
{
    if (packed_blob_bytes(w.c_in, w.c_out) >= (1ull << 31)) return hipErrorInvalidValue;   // 32-bit buffer offsets (checked by the caller)
    if (rot && (!decode_wide_hosts(*rot, T) || rot->c_in != w.c_in)) return hipErrorInvalidValue;
    const WideGeometry g = wide_geometry(w.c_in, w.c_out, T, rot != nullptr);
    if (g.kb > 64 || g.lds > kWideLdsBytes || (g.kb > 1 && !ws)) return hipErrorInvalidValue;
    DecodeArgs a;
    a.blob = w.packed;
    a.scales_off = (uint32_t)packed_tiles_bytes(w.c_in, w.c_out);
    a.zeros_off = a.scales_off + (uint32_t)packed_scales_bytes(w.c_in, w.c_out);
    a.blob_bytes = a.zeros_off + (uint32_t)packed_zeros_bytes(w.c_in, w.c_out);
    a.X = (const _Float16 *)X; a.ldx = ldx; a.Y = (_Float16 *)Y; a.ldy = ldy;
    a.bias = (const _Float16 *)w.bias;
    a.plan = rot ? (const uint32_t *)rot->plan + plan_compact_offset_dwords(rot->c_in / kGroup, rot->n_layers) : nullptr;
    a.err = ws ? (uint32_t *)ws + kWsErrorWord : nullptr;
    a.partial = ws ? (float *)((char *)ws + kWsPartialOff) : nullptr;
    a.T = T; a.C = w.c_in; a.N = w.c_out; a.G = w.c_in / kGroup; a.NT = w.c_out / kTileN;
    a.KS = a.G / kSliceGroups;
    a.tiles_per_block = g.tiles_per_block;
    a.m_lo = 0x000F000Fu; a.m_hi = 0x00F000F0u; a.k_lo = 0x64006400u; a.k_hi = 0x54005400u;
    static std::atomic<uint64_t> attr_done{0};
    if (const int dev = once_pending(attr_done); dev >= 0) {
        const void *fns[] = {(const void *)decode_wide_kernel<false, false>, (const void *)decode_wide_kernel<false, true>,
                             (const void *)decode_wide_kernel<true, false>, (const void *)decode_wide_kernel<true, true>,
                             (const void *)decode_wide2_kernel<false>, (const void *)decode_wide2_kernel<true>,
                             (const void *)decode_wide_kernel<false, true, 8, 8>, (const void *)decode_wide_kernel<true, true, 8, 8>,
                             (const void *)decode_wide_kernel<false, true, 8>};
        for (const void *f : fns) {
            hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return e;
        }
        once_done(attr_done, dev);
    }
    const dim3 grid(g.kb, g.nb), block(g.waves * 64);
    if (rot) {
        // blocks of more than 8 waves hold all K-slices of their rows (wide_geometry): only the 8-wave form is split
        if (g.kb > 1 && g.waves > 8) return hipErrorInvalidValue;
        if (g.kb > 1)          hipLaunchKernelGGL((decode_wide_kernel<true, true, 8, 8>), grid, block, g.lds, s, a);
        else if (g.waves <= 8) hipLaunchKernelGGL((decode_wide_kernel<false, true, 8, 8>), grid, block, g.lds, s, a);
        else                   hipLaunchKernelGGL((decode_wide_kernel<false, true, 8>), grid, block, g.lds, s, a);
    } else if (T > 16) {
        if (g.kb > 1) hipLaunchKernelGGL((decode_wide2_kernel<true>), grid, block, g.lds, s, a);
        else          hipLaunchKernelGGL((decode_wide2_kernel<false>), grid, block, g.lds, s, a);
    } else if (T == 1) {
        if (g.kb > 1) hipLaunchKernelGGL((decode_wide_kernel<true, true>), grid, block, g.lds, s, a);
        else          hipLaunchKernelGGL((decode_wide_kernel<false, true>), grid, block, g.lds, s, a);
    } else {
        if (g.kb > 1) hipLaunchKernelGGL((decode_wide_kernel<true, false>), grid, block, g.lds, s, a);
        else          hipLaunchKernelGGL((decode_wide_kernel<false, false>), grid, block, g.lds, s, a);
    }
    return hipGetLastError();
}

}  // namespace paro
