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
#include "paro_internal.h"

namespace paro {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kDecWaves = 4;
constexpr int kDecThreads = kDecWaves * 64;
constexpr int kSliceCh = kSliceGroups * kGroup;      // 512
constexpr int kXPad = 8;                             // halfs of padding per LDS row
constexpr int kReducePerThread = 4;                   // partial words requested per thread and round
constexpr int kReduceWords = kReducePerThread * 256;  // partial words gathered per reduction round (LDS floats)
constexpr int kMaxIter = 9;                          // tiles per wave (unrolled stream), multiple of 3
constexpr int kSpinLimit = 1 << 22;                  // bounded wait for a partial word to fill

static int g_decode_target_blocks = 0;      // 0: choose by size (see decode_geometry)

struct DecodeArgs {
    const void *blob;            // repacked weight: tiles | scales | zeros
    uint32_t blob_bytes, scales_off, zeros_off;
    const _Float16 *X; int64_t ldx;
    _Float16 *Y; int64_t ldy;
    const _Float16 *bias;
    const uint32_t *plan;
    float *partial;
    int T, C, N, G, NT, KS, tiles_per_block;
    uint32_t m_lo, m_hi, k_lo, k_hi;     // dequant constants, see DequantConsts
};

// Raw buffer resources (stride 0): an access whose byte offset lies beyond num_records returns 0
// (loads) or is dropped (stores).  Predication by offset keeps every memory instruction of the
// stream loop unconditional, so the outstanding-load count is static and the compiler can wait
// for exactly the stage it needs while later stages stay in flight.
constexpr uint32_t kOob = 0x80000000u;
constexpr int kRsrcFlags = 0x00020000;        // 32-bit data format field of a gfx9-family raw buffer
#ifndef PARO_TILE_AUX
#define PARO_TILE_AUX 2
#endif
constexpr int kTileAux = PARO_TILE_AUX;       // weight tiles are read once: non-temporal (bit 1); measured 6 % faster than default
constexpr int kAuxSc1 = 16;                   // agent-scope (write-through / cache-bypassing) access
__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, kRsrcFlags);
}

struct Stage {
    u32x4 w[kSliceGroups];
    uint2 sc;
    uint32_t zq;
};

// tile < 0 loads nothing (all zeros)
__device__ inline void load_stage(__amdgpu_buffer_rsrc_t blob, const DecodeArgs &a, int tile, int ks, int lane,
                                  Stage &st)
{
    const bool ok = tile >= 0;
    const uint32_t toff = ok ? (((uint32_t)tile * a.G + (uint32_t)ks * kSliceGroups) * 64u + lane) * 16u : kOob;
#pragma unroll
    for (int gi = 0; gi < kSliceGroups; ++gi)
        st.w[gi] = __builtin_amdgcn_raw_buffer_load_b128(blob, (int)(toff + gi * 1024u), 0, kTileAux);
    const uint32_t sidx = ((uint32_t)tile * a.KS + ks) * kTileN + (lane & 15);
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    u32x2 sc = __builtin_amdgcn_raw_buffer_load_b64(blob, ok ? (int)(a.scales_off + sidx * 8u) : (int)kOob, 0, 0);
    st.sc = make_uint2(sc[0], sc[1]);
    st.zq = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(blob, ok ? (int)(a.zeros_off + sidx * 2u) : (int)kOob, 0, 0);
}

__device__ inline half2v as_h2(uint32_t u) { union { uint32_t u; half2v h; } c; c.u = u; return c.h; }
__device__ inline uint32_t as_u32(half2v h) { union { uint32_t u; half2v h; } c; c.h = h; return c.u; }

// (a & mask) | magic is one VALU op (v_and_or_b32) when mask and magic sit in registers.  GFX9-family
// VOP3 encodings take no literals, so with compile-time constants the compiler emits two VOP2
// ops with literals instead; the four constants therefore travel as kernel arguments and are
// moved into VGPRs once per wave.  (Inline
// asm is not an option: instructions hidden from the compiler's hazard handling next to MFMAs
// produced wrong results.)
__device__ inline uint32_t and_or(uint32_t a, uint32_t mask, uint32_t magic) { return (a & mask) | magic; }

struct DequantConsts {
    uint32_t m_lo, m_hi, k_lo, k_hi;     // 0x000F000F, 0x00F000F0, 0x64006400 (1024.0 x2), 0x54005400 (64.0 x2)
};

// Sum over the slice's 4 groups of s_g * sum_k (q - z_g) x' for one 16-row tile.
//
// The codes are turned into fp16 by or-ing them into the mantissa of 1024.0 (low nibble of a
// byte) or 64.0 (high nibble): B holds b_k + q with b_k in {1024, 64}.  Instead of subtracting
// b_k + z from every weight, the MFMA accumulator starts at
//      -(sum_k b_k x'_k) - z * (sum_k x'_k)  =  nb1 + z * nb2
// (two per-token, per-group sums computed once per block), so that after the four MFMAs it
// holds sum_k (q - z) x'.  fp32 accumulation: the bias inflates partial sums by <= 1039x, which
// costs ~2^-24 * 1039 relative to the group's |x'| mass - far inside the output tolerance.
// T1: one token, only accumulator row 0 is live.
template <bool T1>
__device__ inline float4v tile_dot(const Stage &st, const half8 (&xf)[kSliceGroups][4],
                                   const float4v (&nb1)[kSliceGroups], const float4v (&nb2)[kSliceGroups],
                                   const DequantConsts &k)
{
    float4v tot = {0.f, 0.f, 0.f, 0.f};
    union { uint2 v; _Float16 h[4]; } sc; sc.v = st.sc;
#pragma unroll
    for (int gi = 0; gi < kSliceGroups; ++gi) {
        const float zf = (float)((st.zq >> (4 * gi)) & 15u);
        float4v acc;
        if constexpr (T1) { acc[0] = zf * nb2[gi][0] + nb1[gi][0]; acc[1] = acc[2] = acc[3] = 0.f; }
        else acc = zf * nb2[gi] + nb1[gi];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t u = st.w[gi][j], t = u >> 8;
            union { uint32_t d[4]; half8 h; } b;
            b.d[0] = and_or(u, k.m_lo, k.k_lo);
            b.d[1] = and_or(u, k.m_hi, k.k_hi);
            b.d[2] = and_or(t, k.m_lo, k.k_lo);
            b.d[3] = and_or(t, k.m_hi, k.k_hi);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf[gi][j], b.h, acc, 0, 0, 0);
        }
        const float s = (float)sc.h[gi];
        if constexpr (T1) tot[0] += s * acc[0];
        else tot += s * acc;
    }
    return tot;
}

// Split-K reduction, spread over the `parts` blocks of one output range.  The T*width outputs of
// the range are cut into `parts` contiguous shares; block `part` sums the partials of its share
// in a fixed order (deterministic), adds the bias and stores fp16.  No fences and no counters:
// every partial word is its own full/empty flag (0 = empty; a value is never stored as +0),
// written with agent-scope stores and taken by its reader with an agent-scope atomic exchange
// against 0, which reads the word and leaves it empty in one operation (an exchange that finds
// 0 changes nothing and is repeated).  Measured: the returning atomic comes back faster than an
// agent-scope load (the fused launches lose 0.3-0.7 us), while atomics on the writer side would
// serialise.  The writers are the blocks dispatched next to the reader, which never wait on
// anything before writing.  The poll is bounded; a word that never fills is reported as NaN.
__device__ inline void splitk_reduce(const DecodeArgs &a, int parts, int part, int tile_lo, int tile_hi, float *s_red)
{
    const int THREADS = blockDim.x;                 // >= 256: kReducePerThread requests per thread cover a round
    const int n_lo = tile_lo * kTileN, width = (tile_hi - tile_lo) * kTileN;
    const int outputs = a.T * width;
    const int share = (outputs + parts - 1) / parts;
    const int o_lo = part * share, o_hi = min(outputs, o_lo + share);
    const int round_outputs = kReduceWords / parts;
    for (int base = o_lo; base < o_hi; base += round_outputs) {
        const int n_out = min(round_outputs, o_hi - base);
        __syncthreads();
        // all of a thread's words are requested before any is examined: one round trip
        constexpr int PER = kReducePerThread;
        uint32_t bits[PER];
        uint32_t *ptr[PER];
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int j = threadIdx.x + u * THREADS;
            const bool on = j < n_out * parts;
            // consecutive threads take consecutive outputs of one K-part: coalesced requests
            const int o = base + (on ? j % n_out : 0), k2 = on ? j / n_out : 0;
            const int t = o / width, n = n_lo + o % width;
            ptr[u] = (uint32_t *)(a.partial + ((size_t)k2 * a.T + t) * a.N + n);
            bits[u] = on ? __hip_atomic_exchange(ptr[u], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0x80000000u;
        }
        // words still empty are requested again, all of a thread's in one round trip
        for (int spin = 0; spin < kSpinLimit; ++spin) {
            bool empty = false;
#pragma unroll
            for (int u = 0; u < PER; ++u) empty |= bits[u] == 0u;
            if (!empty) break;
#pragma unroll
            for (int u = 0; u < PER; ++u)
                if (bits[u] == 0u)
                    bits[u] = __hip_atomic_exchange(ptr[u], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int j = threadIdx.x + u * THREADS;
            if (j < n_out * parts) s_red[j] = bits[u] == 0u ? __builtin_nanf("") : __uint_as_float(bits[u]);
        }
        __syncthreads();
        for (int i = threadIdx.x; i < n_out; i += THREADS) {
            const int o = base + i;
            const int t = o / width, n = n_lo + o % width;
            float sum = 0.f;
            for (int k2 = 0; k2 < parts; ++k2) sum += s_red[k2 * n_out + i];
            if (a.bias) sum += (float)a.bias[n];
            a.Y[(size_t)t * a.ldy + n] = (_Float16)sum;
        }
    }
}

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
        for (int t = 0; t < (rw ? a.T : 0); ++t) {
            float va = (float)s_x[t][gi * kGroup + in_a] * sia;
            float vb = (float)s_x[t][gi * kGroup + in_b] * sib;
#pragma unroll
            for (int l = 0; l < K; ++l) {
                float m00, m01, m10, m11;
                bool ai = pm[l] & kMetaAIsI, ki = pm[l] & kMetaKeepI;
                float c = pc[l], s = ps[l];
                float ni_a = ai ? c : -s, ni_b = ai ? -s : c, nj_a = ai ? s : c, nj_b = ai ? c : s;
                m00 = ki ? ni_a : nj_a; m01 = ki ? ni_b : nj_b; m10 = ki ? nj_a : ni_a; m11 = ki ? nj_b : ni_b;
                float na = m00 * va + m01 * vb, nb2 = m10 * va + m11 * vb;
                va = na;
                vb = (l + 1 < K) ? __int_as_float(__builtin_amdgcn_ds_bpermute((int)(pm[l] & 0xff), __float_as_int(nb2)))
                                 : nb2;
            }
            // all lanes have read their inputs of token t (the bpermutes above are wave-wide),
            // so the staging row can be overwritten with the result
            s_x[t][gi * kGroup + out_a] = (_Float16)(va * soa);
            s_x[t][gi * kGroup + out_b] = (_Float16)(vb * sob);
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
    // Fully unrolled (n_iter <= kMaxIter, guaranteed by the host): straight-line code with uniform
    // early exits and no back edge, so the waits inserted by the compiler are exact - a stage is
    // awaited while the two younger ones stay in flight.
#pragma unroll
    for (int i = 0; i < kMaxIter; i += 3) {
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
    d.waves = (T == 1 && (many_slices || big) && target_blocks == 0 && g_decode_target_blocks == 0) ? 2 * kDecWaves : kDecWaves;
    // measured on MI355X: one 4-wave block per CU for the small linears (the prologue is repeated
    // less often), two per CU once the weight stream exceeds ~24 MB
    int target = target_blocks > 0 ? target_blocks : g_decode_target_blocks;
    if (target <= 0) target = packed_tiles_bytes(c_in, c_out) >= (24u << 20) ? 512 : 256;
    if (d.waves > kDecWaves) target = 256;
    int nb = target / d.ks;
    if (nb < 1) nb = 1;
    int tpb = (NT + nb - 1) / nb;
    tpb = (tpb + d.waves - 1) / d.waves * d.waves;           // whole rounds of the block's waves
    if (tpb > kMaxIter * d.waves) tpb = kMaxIter * d.waves;
    d.tiles_per_block = tpb;
    d.nb = (NT + tpb - 1) / tpb;
    if (d.waves > kDecWaves && d.ks * d.nb > 256) {           // would not fit one round of 8-wave blocks
        d.waves = kDecWaves;
        target = packed_tiles_bytes(c_in, c_out) >= (24u << 20) ? 512 : 256;
        nb = target / d.ks;
        if (nb < 1) nb = 1;
        tpb = (NT + nb - 1) / nb;
        tpb = (tpb + d.waves - 1) / d.waves * d.waves;
        if (tpb > kMaxIter * d.waves) tpb = kMaxIter * d.waves;
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
    if (d.waves == 2 * kDecWaves) {      // only chosen for one token and many K-slices
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
                                   const paro_half_t *X, int64_t ldx, paro_half_t *Y, int64_t ldy, int T, void *partial,
                                   int target_blocks = 0)
{
    if (!rot || !rot->plan) return hipErrorInvalidValue;
    d = decode_geometry(w.c_in, w.c_out, T, target_blocks);
    if (d.ks > kReduceWords) return hipErrorInvalidValue;
    if (packed_tiles_bytes(w.c_in, w.c_out) + packed_scales_bytes(w.c_in, w.c_out) + packed_zeros_bytes(w.c_in, w.c_out) >= (1ull << 31))
        return hipErrorInvalidValue;   // 32-bit buffer offsets
    a.blob = w.packed;
    a.scales_off = (uint32_t)packed_tiles_bytes(w.c_in, w.c_out);
    a.zeros_off = a.scales_off + (uint32_t)packed_scales_bytes(w.c_in, w.c_out);
    a.blob_bytes = a.zeros_off + (uint32_t)packed_zeros_bytes(w.c_in, w.c_out);
    a.X = (const _Float16 *)X; a.ldx = ldx; a.Y = (_Float16 *)Y; a.ldy = ldy;
    a.bias = (const _Float16 *)w.bias;
    a.plan = (const uint32_t *)rot->plan;
    a.partial = (float *)partial;
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
    hipError_t e = fill_decode_args(a, d, rot, w, X, ldx, Y, ldy, T, ws);
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
    int target = g_decode_target_blocks;
    if (target <= 0) target = packed_tiles_bytes(w[0]->c_in, (int)n_all) >= (24u << 20) ? 512 : 256;
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
        hipError_t e = fill_decode_args(m.part[p], d, rot[p], *w[p], X, ldx, Y[p], ldy[p], T, (char *)ws + off,
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
// Wide variant: the waves of a block cover different K-slices (one each, up to 12 = 6144
// channels) of the SAME tiles; their partial tiles are summed through LDS, so such layers need no
// exchange between blocks at all, and wider ones (slices spread evenly over blocks of at most 8
// waves) exchange correspondingly fewer partial sums.  Used for the bare linear and for 5..16
// tokens, where partial sums (T x N fp32 per K-part) would otherwise rival the weight stream.
// The transform, if any, has run as a separate pass.
// ------------------------------------------------------------------------------------------
#ifndef PARO_WIDE_WAVES
#define PARO_WIDE_WAVES 12
#endif
constexpr int kWideWaves = PARO_WIDE_WAVES;     // most K-slices (waves) of one block
constexpr int kWideThreads = kWideWaves * 64;

template <bool SPLIT, bool T1>
__global__ __launch_bounds__(kWideThreads) void decode_wide_kernel(DecodeArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float s_wide[];      // [n_iter][8 waves][256] + reduce scratch
    const int kb = blockIdx.x, nb = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nw = blockDim.x >> 6;                                        // K-slices (waves) per block, <= 8
    const int ks = kb * nw + wave;
    const bool slice_ok = ks < a.KS;
    const int tile_lo = nb * a.tiles_per_block;
    const int tile_hi = min(a.NT, tile_lo + a.tiles_per_block);
    const int n_iter = tile_hi - tile_lo;                                  // <= kMaxIter
    auto tile_of = [&](int i) { return (i < n_iter && slice_ok) ? tile_lo + i : -1; };
    const __amdgpu_buffer_rsrc_t blob = make_rsrc(a.blob, a.blob_bytes);

    Stage st0, st1, st2;
    half8 xf[kSliceGroups][4];
    const int ft = lane & 15, fkb = lane >> 4;
    {
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
        load_stage(blob, a, tile_of(0), ks, lane, st0);
        load_stage(blob, a, tile_of(1), ks, lane, st1);
    }
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

    // partial tile of (iteration i, this wave): element lane*4 + r <-> token 4*(lane/16)+r, row lane%16
    auto emit = [&](const Stage &stg, int i) {
        float4v tot = tile_dot<T1>(stg, xf, nb1, nb2, dq);
        float *dst = s_wide + ((size_t)i * nw + wave) * 256 + lane * 4;
        if constexpr (T1) { if (lane < 16) dst[0] = tot[0]; }
        else *(float4v *)dst = tot;
    };
#pragma unroll
    for (int i = 0; i < kMaxIter; i += 3) {
        load_stage(blob, a, tile_of(i + 2), ks, lane, st2);
        emit(st0, i);
        if (i + 1 >= n_iter) break;
        load_stage(blob, a, tile_of(i + 3), ks, lane, st0);
        emit(st1, i + 1);
        if (i + 2 >= n_iter) break;
        load_stage(blob, a, tile_of(i + 4), ks, lane, st1);
        emit(st2, i + 2);
        if (i + 3 >= n_iter) break;
    }
    __syncthreads();

    // ---- sum the 8 K-slices; outputs indexed (i, t, n) with n fastest for coalesced stores -----
    const int per_tile = a.T * kTileN;
    for (int idx = threadIdx.x; idx < n_iter * per_tile; idx += blockDim.x) {
        const int i = idx / per_tile, rem = idx % per_tile;
        const int t = rem / kTileN, nn = rem % kTileN;
        const int e = ((t >> 2) * 16 + nn) * 4 + (t & 3);
        float sum = 0.f;
        for (int w = 0; w < nw; ++w) sum += s_wide[((size_t)i * nw + w) * 256 + e];
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
    if constexpr (SPLIT)
        splitk_reduce(a, gridDim.x, kb, tile_lo, tile_hi, s_wide + (size_t)kMaxIter * nw * 256);
}

struct WideGeometry { int kb, nb, waves, tiles_per_block; size_t lds; };
static WideGeometry wide_geometry(int c_in, int c_out)
{
    WideGeometry g;
    const int KS = c_in / kGroup / kSliceGroups, NT = c_out / kTileN;
    // up to 12 slices fit one block (3 waves per SIMD): no exchange between blocks at all.  Beyond
    // that the slices are spread evenly over blocks of at most 8 waves.
    g.kb = KS <= kWideWaves ? 1 : (KS + 7) / 8;
    g.waves = (KS + g.kb - 1) / g.kb;
    int nb = (g.waves > 8 ? 256 : 2048 / g.waves) / g.kb;   // about 8 waves per CU; one block per CU beyond 8 waves
    if (nb < 1) nb = 1;
    int tpb = (NT + nb - 1) / nb;
    if (tpb > kMaxIter) tpb = kMaxIter;
    g.tiles_per_block = tpb;
    g.nb = (NT + tpb - 1) / tpb;
    g.lds = ((size_t)kMaxIter * g.waves * 256 + kReduceWords) * sizeof(float);
    return g;
}

size_t decode_wide_partial_bytes(int c_in, int c_out, int T)
{
    WideGeometry g = wide_geometry(c_in, c_out);
    int t16 = T < 16 ? T : 16;
    return g.kb > 1 ? (size_t)g.kb * t16 * c_out * sizeof(float) : 0;
}

hipError_t launch_decode_wide(const paro_w4_weight &w, const paro_half_t *X, int64_t ldx, paro_half_t *Y, int64_t ldy,
                              int T, void *ws, hipStream_t s)
{
    if (packed_tiles_bytes(w.c_in, w.c_out) + packed_scales_bytes(w.c_in, w.c_out) + packed_zeros_bytes(w.c_in, w.c_out) >= (1ull << 31))
        return hipErrorInvalidValue;   // 32-bit buffer offsets
    WideGeometry g = wide_geometry(w.c_in, w.c_out);
    if (g.kb > 64) return hipErrorInvalidValue;
    DecodeArgs a;
    a.blob = w.packed;
    a.scales_off = (uint32_t)packed_tiles_bytes(w.c_in, w.c_out);
    a.zeros_off = a.scales_off + (uint32_t)packed_scales_bytes(w.c_in, w.c_out);
    a.blob_bytes = a.zeros_off + (uint32_t)packed_zeros_bytes(w.c_in, w.c_out);
    a.X = (const _Float16 *)X; a.ldx = ldx; a.Y = (_Float16 *)Y; a.ldy = ldy;
    a.bias = (const _Float16 *)w.bias;
    a.plan = nullptr;
    a.partial = (float *)ws;
    a.T = T; a.C = w.c_in; a.N = w.c_out; a.G = w.c_in / kGroup; a.NT = w.c_out / kTileN;
    a.KS = a.G / kSliceGroups;
    a.tiles_per_block = g.tiles_per_block;
    a.m_lo = 0x000F000Fu; a.m_hi = 0x00F000F0u; a.k_lo = 0x64006400u; a.k_hi = 0x54005400u;
    static std::atomic<uint64_t> attr_done{0};
    if (const int dev = once_pending(attr_done); dev >= 0) {
        const void *fns[4] = {(const void *)decode_wide_kernel<false, false>, (const void *)decode_wide_kernel<false, true>,
                              (const void *)decode_wide_kernel<true, false>, (const void *)decode_wide_kernel<true, true>};
        for (const void *f : fns) {
            hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize,
                                               (int)(((size_t)kMaxIter * kWideWaves * 256 + kReduceWords) * sizeof(float)));
            if (e != hipSuccess) return e;
        }
        once_done(attr_done, dev);
    }
    const dim3 grid(g.kb, g.nb), block(g.waves * 64);
    if (T == 1) {
        if (g.kb > 1) hipLaunchKernelGGL((decode_wide_kernel<true, true>), grid, block, g.lds, s, a);
        else          hipLaunchKernelGGL((decode_wide_kernel<false, true>), grid, block, g.lds, s, a);
    } else {
        if (g.kb > 1) hipLaunchKernelGGL((decode_wide_kernel<true, false>), grid, block, g.lds, s, a);
        else          hipLaunchKernelGGL((decode_wide_kernel<false, false>), grid, block, g.lds, s, a);
    }
    return hipGetLastError();
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

void set_decode_target_waves(int waves) { g_decode_target_blocks = waves > 0 ? (waves + kDecWaves - 1) / kDecWaves : 0; }

}  // namespace paro
