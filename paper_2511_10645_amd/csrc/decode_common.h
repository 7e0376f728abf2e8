// Device code shared by the decode-side kernels (decode.hip: K-major kernel with the rotation
// fused per K-slice; decode_wide.hip: all K-slices in one block): the weight-tile stream
// (load_stage, tile_dot) and the fence-free split-K exchange (splitk_reduce).
#pragma once
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
// tiles per wave of the K-major kernel (unrolled stream, multiple of 3).  Longer streams in 8-wave blocks, so that
// 5120 -> 55296 fits one round of blocks, were measured and are slower (32.0 against 31.1 us; 27648 -> 5120: 21.8
// against 18.2 us).
__host__ __device__ constexpr int decode_max_iter(int) { return 9; }
constexpr int kSpinLimit = 1 << 22;                  // bounded wait for a partial word to fill

struct DecodeArgs {
    const void *blob;            // repacked weight: tiles | scales | zeros
    uint32_t blob_bytes, scales_off, zeros_off;
    const _Float16 *X; int64_t ldx;
    _Float16 *Y; int64_t ldy;
    const _Float16 *bias;
    const uint32_t *plan;
    float *partial;
    uint32_t *err;               // error word of the workspace header (set when a bounded wait runs out)
    int T, C, N, G, NT, KS, tiles_per_block;
    uint32_t m_lo, m_hi, k_lo, k_hi;     // dequant constants, see DequantConsts
};

// Raw buffer resources (stride 0): an access whose byte offset lies beyond num_records returns 0
// (loads) or is dropped (stores).  Predication by offset keeps every memory instruction of the
// stream loop unconditional, so the outstanding-load count is static and the compiler can wait
// for exactly the stage it needs while later stages stay in flight.
constexpr uint32_t kOob = 0x80000000u;
constexpr int kRsrcFlags = 0x00020000;        // 32-bit data format field of a gfx9-family raw buffer
constexpr int kTileAux = 2;                   // weight tiles are read once: non-temporal (bit 1); measured 6 % faster than default
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
            if (j < n_out * parts) {
                s_red[j] = bits[u] == 0u ? __builtin_nanf("") : __uint_as_float(bits[u]);
                if (bits[u] == 0u) __hip_atomic_store(a.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
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

}  // namespace paro
