// Weight side of the method, offline: the equivalent transform of Eq. 8 applied to every output
// row of a dense fp16 weight, then the round-to-nearest INT4 quantiser of Eq. 1 with one
// (scale, zero) per 128 input channels (Section 2.1), written in the interchange layout that
// paro_w4_repack and the linear kernels consume.
//
//      w'_n = R_K ... R_1 . diag(1 / ch_scale) . w_n          (scale_order 0; Eq. 8, weight side)
//      s = (max - min) / 15,  z = -round(min / s),  q = clamp(round(w' / s) + z, 0, 15)
//
// so that  sum_c (q - z) s . x'_c  ~  w_n . x  for the activations x' = R_K ... R_1 . S . x that
// paro_rotate_scale produces (Eq. 2).  One wavefront per (row, group), exactly as the
// activation kernel: the lane's two fp32 registers hold the pair being rotated; the group's
// minimum and maximum are wave reductions.  The integer decisions are taken in fp32 with the
// fp16-rounded scale that is stored (IEEE division, round-half-to-even); the scale has the
// floor 2^-14; the zero point is clamped to 0..15.  A block handles 8 consecutive rows of one
// group, so that their 8 zero points fill one output word.
#include "paro_internal.h"
#include "rotate_lane.h"

namespace paro {

constexpr int kQuantRows = 8;      // rows (waves) per block = zero points per packed word

// K >= 0: rotation with K layers from the plan; K < 0: no transform (plain RTN).
template <int K>
__global__ __launch_bounds__(kQuantRows * 64) void quantize_rows_kernel(const uint32_t *__restrict__ plan,
                                                                         const _Float16 *__restrict__ W, int64_t ldw,
                                                                         int N, int C, uint32_t *__restrict__ qweight,
                                                                         _Float16 *__restrict__ scales,
                                                                         uint32_t *__restrict__ qzeros)
{
    __shared__ _Float16 s_stage[kQuantRows][kGroup];
    __shared__ uint8_t s_codes[kQuantRows][kGroup];
    __shared__ uint32_t s_z[kQuantRows];
    __shared__ _Float16 s_s[kQuantRows];
    const int g = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = blockIdx.y * kQuantRows + wave;      // N is a multiple of 8

    // the row's 128 channels of this group, two per lane in channel order
    const uint32_t raw = *((const uint32_t *)(W + (size_t)n * ldw + (size_t)g * kGroup) + lane);
    float va, vb;
    int ch_a, ch_b;
    if constexpr (K >= 0) {
        LanePlan<K> P;
        load_lane_plan<K>(plan + (size_t)g * plan_group_dwords(K), lane, P);
        *(uint32_t *)&s_stage[wave][2 * lane] = raw;
        __builtin_amdgcn_wave_barrier();
        // the plan carries the activation-side multipliers; the weights take their reciprocals
        float a[1] = {(float)s_stage[wave][P.in_a] * (1.0f / P.sia)};
        float b[1] = {(float)s_stage[wave][P.in_b] * (1.0f / P.sib)};
        rotate_layers<K, 1>(P, a, b);
        va = a[0] * (1.0f / P.soa); vb = b[0] * (1.0f / P.sob);
        ch_a = P.out_a; ch_b = P.out_b;
    } else {
        union { uint32_t u; _Float16 h[2]; } c; c.u = raw;
        va = (float)c.h[0]; vb = (float)c.h[1];
        ch_a = 2 * lane; ch_b = 2 * lane + 1;
    }

    // Eq. 1 on the group
    float mn = fminf(va, vb), mx = fmaxf(va, vb);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        mn = fminf(mn, __shfl_xor(mn, off, 64));
        mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    }
    float s32 = (mx - mn) / 15.0f;
    if (!(s32 >= 6.103515625e-05f)) s32 = 6.103515625e-05f;
    const _Float16 s16 = (_Float16)s32;
    const float s = (float)s16;
    float zf = -rintf(mn / s);
    zf = fminf(fmaxf(zf, 0.0f), 15.0f);
    const float qa = fminf(fmaxf(rintf(va / s) + zf, 0.0f), 15.0f);
    const float qb = fminf(fmaxf(rintf(vb / s) + zf, 0.0f), 15.0f);
    s_codes[wave][ch_a] = (uint8_t)qa;
    s_codes[wave][ch_b] = (uint8_t)qb;
    if (lane == 0) { s_z[wave] = (uint32_t)zf; s_s[wave] = s16; }
    __syncthreads();

    if (lane < kGroup / 8) {        // 16 words of 8 codes, code k of a word in bits 4k..4k+3
        uint32_t word = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) word |= (uint32_t)s_codes[wave][lane * 8 + k] << (4 * k);
        qweight[(size_t)n * (C / 8) + (size_t)g * (kGroup / 8) + lane] = word;
    }
    if (threadIdx.x < kQuantRows) scales[(size_t)g * N + (size_t)blockIdx.y * kQuantRows + threadIdx.x] = s_s[threadIdx.x];
    if (threadIdx.x == 0) {
        uint32_t word = 0;
#pragma unroll
        for (int k = 0; k < kQuantRows; ++k) word |= s_z[k] << (4 * k);
        qzeros[(size_t)g * (N / 8) + blockIdx.y] = word;
    }
}

template <int K>
static hipError_t launch_quantize_k(const uint32_t *plan, const paro_half_t *W, int64_t ldw, int N, int C,
                                    uint32_t *qweight, paro_half_t *scales, uint32_t *qzeros, hipStream_t s)
{
    hipLaunchKernelGGL(quantize_rows_kernel<K>, dim3(C / kGroup, N / kQuantRows), dim3(kQuantRows * 64), 0, s, plan,
                       (const _Float16 *)W, ldw, N, C, qweight, (_Float16 *)scales, qzeros);
    return hipGetLastError();
}

hipError_t launch_quantize(const paro_rotation *rot, const paro_half_t *W, int64_t ldw, int N, int C, uint32_t *qweight,
                           paro_half_t *scales, uint32_t *qzeros, hipStream_t s)
{
    if (!rot) return launch_quantize_k<-1>(nullptr, W, ldw, N, C, qweight, scales, qzeros, s);
    const uint32_t *plan = (const uint32_t *)rot->plan;
    switch (rot->n_layers) {
    case 0: return launch_quantize_k<0>(plan, W, ldw, N, C, qweight, scales, qzeros, s);
    case 1: return launch_quantize_k<1>(plan, W, ldw, N, C, qweight, scales, qzeros, s);
    case 2: return launch_quantize_k<2>(plan, W, ldw, N, C, qweight, scales, qzeros, s);
    case 3: return launch_quantize_k<3>(plan, W, ldw, N, C, qweight, scales, qzeros, s);
    case 4: return launch_quantize_k<4>(plan, W, ldw, N, C, qweight, scales, qzeros, s);
    case 5: return launch_quantize_k<5>(plan, W, ldw, N, C, qweight, scales, qzeros, s);
    case 6: return launch_quantize_k<6>(plan, W, ldw, N, C, qweight, scales, qzeros, s);
    case 7: return launch_quantize_k<7>(plan, W, ldw, N, C, qweight, scales, qzeros, s);
    default: return launch_quantize_k<8>(plan, W, ldw, N, C, qweight, scales, qzeros, s);
    }
}

// ------------------------------------------------------------------------------------------
// Activation side of the W4A4 extension (App. A.3: Y' = Q(X T^-1) . Q(T W) + b): the transformed
// activations are quantised to INT4 right after the rotation, while they are still in the
// wave's registers.  The paper names no activation quantiser of its own, so Eq. 1 (b = 4) is
// applied per token and 128-channel group, with the same decisions as on the weight side.
// One wavefront per (token, group); outputs per token: codes [c_in/8] words, scale and zero
// point per group.
// ------------------------------------------------------------------------------------------
constexpr int kActWaves = 4;

template <int K>
__global__ __launch_bounds__(kActWaves * 64) void quantize_act_kernel(const uint32_t *__restrict__ plan,
                                                                       const _Float16 *__restrict__ X, int64_t ldx, int T,
                                                                       int C, int rows_per_wave, uint32_t *__restrict__ codes,
                                                                       _Float16 *__restrict__ scales,
                                                                       uint8_t *__restrict__ zeros)
{
    __shared__ _Float16 s_stage[kActWaves][kGroup];
    __shared__ uint8_t s_codes[kActWaves][kGroup];
    const int g = blockIdx.x, G = C / kGroup;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t0 = (blockIdx.y * kActWaves + wave) * rows_per_wave;
    if (t0 >= T) return;
    const int t1 = min(T, t0 + rows_per_wave);

    // the group's plan once per wave, then a run of tokens
    LanePlan<K> P;
    load_lane_plan<K>(plan + (size_t)g * plan_group_dwords(K), lane, P);
    uint32_t raw = *((const uint32_t *)(X + (size_t)t0 * ldx + (size_t)g * kGroup) + lane);
    for (int t = t0; t < t1; ++t) {
        *(uint32_t *)&s_stage[wave][2 * lane] = raw;
        if (t + 1 < t1) raw = *((const uint32_t *)(X + (size_t)(t + 1) * ldx + (size_t)g * kGroup) + lane);
        __builtin_amdgcn_wave_barrier();
        float a[1] = {(float)s_stage[wave][P.in_a] * P.sia};
        float b[1] = {(float)s_stage[wave][P.in_b] * P.sib};
        rotate_layers<K, 1>(P, a, b);
        const float va = a[0] * P.soa, vb = b[0] * P.sob;

        float mn = fminf(va, vb), mx = fmaxf(va, vb);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            mn = fminf(mn, __shfl_xor(mn, off, 64));
            mx = fmaxf(mx, __shfl_xor(mx, off, 64));
        }
        float s32 = (mx - mn) / 15.0f;
        if (!(s32 >= 6.103515625e-05f)) s32 = 6.103515625e-05f;
        const _Float16 s16 = (_Float16)s32;
        const float s = (float)s16;
        float zf = -rintf(mn / s);
        zf = fminf(fmaxf(zf, 0.0f), 15.0f);
        s_codes[wave][P.out_a] = (uint8_t)fminf(fmaxf(rintf(va / s) + zf, 0.0f), 15.0f);
        s_codes[wave][P.out_b] = (uint8_t)fminf(fmaxf(rintf(vb / s) + zf, 0.0f), 15.0f);
        __builtin_amdgcn_wave_barrier();
        if (lane < kGroup / 8) {
            uint32_t word = 0;
#pragma unroll
            for (int k = 0; k < 8; ++k) word |= (uint32_t)s_codes[wave][lane * 8 + k] << (4 * k);
            codes[(size_t)t * (C / 8) + (size_t)g * (kGroup / 8) + lane] = word;
        }
        if (lane == 0) { scales[(size_t)t * G + g] = s16; zeros[(size_t)t * G + g] = (uint8_t)zf; }
        __builtin_amdgcn_wave_barrier();
    }
}

template <int K>
static hipError_t launch_quantize_act_k(const paro_rotation &rot, const paro_half_t *X, int64_t ldx, int T,
                                        uint32_t *codes, paro_half_t *scales, uint8_t *zeros, hipStream_t s)
{
    // runs of up to 32 tokens per wave, shorter while that leaves fewer than ~4096 waves
    const int G = rot.c_in / kGroup;
    int rpw = 32;
    while (rpw > 1 && (int64_t)G * ((T + rpw - 1) / rpw) < 4096) rpw >>= 1;
    const int waves_t = (T + rpw - 1) / rpw;
    hipLaunchKernelGGL(quantize_act_kernel<K>, dim3(G, (waves_t + kActWaves - 1) / kActWaves), dim3(kActWaves * 64), 0, s,
                       (const uint32_t *)rot.plan, (const _Float16 *)X, ldx, T, rot.c_in, rpw, codes, (_Float16 *)scales, zeros);
    return hipGetLastError();
}

hipError_t launch_quantize_act(const paro_rotation &rot, const paro_half_t *X, int64_t ldx, int T, uint32_t *codes,
                               paro_half_t *scales, uint8_t *zeros, hipStream_t s)
{
    switch (rot.n_layers) {
    case 0: return launch_quantize_act_k<0>(rot, X, ldx, T, codes, scales, zeros, s);
    case 1: return launch_quantize_act_k<1>(rot, X, ldx, T, codes, scales, zeros, s);
    case 2: return launch_quantize_act_k<2>(rot, X, ldx, T, codes, scales, zeros, s);
    case 3: return launch_quantize_act_k<3>(rot, X, ldx, T, codes, scales, zeros, s);
    case 4: return launch_quantize_act_k<4>(rot, X, ldx, T, codes, scales, zeros, s);
    case 5: return launch_quantize_act_k<5>(rot, X, ldx, T, codes, scales, zeros, s);
    case 6: return launch_quantize_act_k<6>(rot, X, ldx, T, codes, scales, zeros, s);
    case 7: return launch_quantize_act_k<7>(rot, X, ldx, T, codes, scales, zeros, s);
    default: return launch_quantize_act_k<8>(rot, X, ldx, T, codes, scales, zeros, s);
    }
}

// ------------------------------------------------------------------------------------------
// The same activation side with a microscaling FP4 quantiser (MXFP4 of the OCP Microscaling
// Formats specification, the 4-bit type the matrix cores of this chip take directly): 32
// consecutive channels share a power-of-two scale 2^e, e = floor(log2(max|v|)) - 2 (>= -127),
// stored as the byte e + 127; each value becomes the E2M1 code of v / 2^e, rounded to nearest
// with ties to the even code and saturated at 6.  Everything after the rotation is exact.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t e2m1_code(float r)
{
    const float a = fabsf(r);
    uint32_t c = a <= 0.25f ? 0u : a < 0.75f ? 1u : a <= 1.25f ? 2u : a < 1.75f ? 3u
               : a <= 2.5f ? 4u : a < 3.5f ? 5u : a <= 5.0f ? 6u : 7u;
    return c | ((__float_as_uint(r) >> 28) & 8u);
}

// WSIDE: the rows are output rows of a dense weight and take the weight side of the transform
// (the reciprocals of the activation-side multipliers, as in quantize_rows_kernel): Q(T W) of
// App. A.3.  K < 0: no transform at all (rows quantised as they are).
template <int K, bool WSIDE>
__global__ __launch_bounds__(kActWaves * 64) void quantize_act_mxfp4_kernel(const uint32_t *__restrict__ plan,
                                                                             const _Float16 *__restrict__ X, int64_t ldx,
                                                                             int T, int C, int rows_per_wave,
                                                                             uint32_t *__restrict__ codes,
                                                                             uint8_t *__restrict__ scales)
{
    __shared__ _Float16 s_stage[kActWaves][kGroup];
    __shared__ float s_val[kActWaves][kGroup];
    __shared__ __attribute__((aligned(4))) uint8_t s_codes[kActWaves][kLanes];
    const int g = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t0 = (blockIdx.y * kActWaves + wave) * rows_per_wave;
    if (t0 >= T) return;
    const int t1 = min(T, t0 + rows_per_wave);

    // The group's plan once per wave, then a run of rows: the plan is 7.4 KB at K = 8, re-reading it per row would
    // outweigh the row itself 30 times.  (Rotating four rows at a time as the activation kernel does was measured
    // and is no faster here: the conversion, not the permute latency, is what a row costs.)
    LanePlan<K> P;
    float ia = 1.f, ib = 1.f, oa = 1.f, ob = 1.f;
    if constexpr (K >= 0) {
        load_lane_plan<K>(plan + (size_t)g * plan_group_dwords(K), lane, P);
        ia = WSIDE ? 1.0f / P.sia : P.sia; ib = WSIDE ? 1.0f / P.sib : P.sib;
        oa = WSIDE ? 1.0f / P.soa : P.soa; ob = WSIDE ? 1.0f / P.sob : P.sob;
    }
    uint32_t raw = *((const uint32_t *)(X + (size_t)t0 * ldx + (size_t)g * kGroup) + lane);
    for (int t = t0; t < t1; ++t) {
        const uint32_t cur = raw;
        if (t + 1 < t1) raw = *((const uint32_t *)(X + (size_t)(t + 1) * ldx + (size_t)g * kGroup) + lane);
        float2 v;
        if constexpr (K >= 0) {
            *(uint32_t *)&s_stage[wave][2 * lane] = cur;
            __builtin_amdgcn_wave_barrier();
            float a[1] = {(float)s_stage[wave][P.in_a] * ia};
            float b[1] = {(float)s_stage[wave][P.in_b] * ib};
            rotate_layers<K, 1>(P, a, b);
            s_val[wave][P.out_a] = a[0] * oa;
            s_val[wave][P.out_b] = b[0] * ob;
            __builtin_amdgcn_wave_barrier();
            // channel order from here: lane l holds channels 2l, 2l+1; 16 lanes = one 32-channel block
            v = *(const float2 *)&s_val[wave][2 * lane];
        } else {
            union { uint32_t u; _Float16 h[2]; } c; c.u = cur;
            v = make_float2((float)c.h[0], (float)c.h[1]);
        }
        float amax = fmaxf(fabsf(v.x), fabsf(v.y));
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
        int e = (int)(__float_as_uint(amax) >> 23) - 127 - 2;
        if (e < -127) e = -127;
        const uint32_t byte = e2m1_code(ldexpf(v.x, -e)) | (e2m1_code(ldexpf(v.y, -e)) << 4);
        s_codes[wave][lane] = (uint8_t)byte;
        __builtin_amdgcn_wave_barrier();
        if (lane < kGroup / 8) codes[(size_t)t * (C / 8) + (size_t)g * (kGroup / 8) + lane] = *(const uint32_t *)&s_codes[wave][4 * lane];
        if ((lane & 15) == 0) scales[(size_t)t * (C / 32) + (size_t)g * (kGroup / 32) + (lane >> 4)] = (uint8_t)(e + 127);
        __builtin_amdgcn_wave_barrier();
    }
}

template <int K, bool WSIDE>
static hipError_t launch_quantize_mxfp4_k(const uint32_t *plan, int C, const paro_half_t *X, int64_t ldx, int T,
                                          uint32_t *codes, uint8_t *scales, hipStream_t s)
{
    // runs of up to 32 rows per wave, shorter while that leaves fewer than ~4096 waves
    const int G = C / kGroup;
    int rpw = 32;
    while (rpw > 1 && (int64_t)G * ((T + rpw - 1) / rpw) < 4096) rpw >>= 1;
    const int waves_t = (T + rpw - 1) / rpw;
    hipLaunchKernelGGL((quantize_act_mxfp4_kernel<K, WSIDE>), dim3(G, (waves_t + kActWaves - 1) / kActWaves),
                       dim3(kActWaves * 64), 0, s, plan, (const _Float16 *)X, ldx, T, C, rpw, codes, scales);
    return hipGetLastError();
}

template <bool WSIDE>
static hipError_t launch_quantize_mxfp4_side(const paro_rotation *rot, int C, const paro_half_t *X, int64_t ldx, int T,
                                             uint32_t *codes, uint8_t *scales, hipStream_t s)
{
    if (!rot) return launch_quantize_mxfp4_k<-1, WSIDE>(nullptr, C, X, ldx, T, codes, scales, s);
    const uint32_t *plan = (const uint32_t *)rot->plan;
    switch (rot->n_layers) {
    case 0: return launch_quantize_mxfp4_k<0, WSIDE>(plan, C, X, ldx, T, codes, scales, s);
    case 1: return launch_quantize_mxfp4_k<1, WSIDE>(plan, C, X, ldx, T, codes, scales, s);
    case 2: return launch_quantize_mxfp4_k<2, WSIDE>(plan, C, X, ldx, T, codes, scales, s);
    case 3: return launch_quantize_mxfp4_k<3, WSIDE>(plan, C, X, ldx, T, codes, scales, s);
    case 4: return launch_quantize_mxfp4_k<4, WSIDE>(plan, C, X, ldx, T, codes, scales, s);
    case 5: return launch_quantize_mxfp4_k<5, WSIDE>(plan, C, X, ldx, T, codes, scales, s);
    case 6: return launch_quantize_mxfp4_k<6, WSIDE>(plan, C, X, ldx, T, codes, scales, s);
    case 7: return launch_quantize_mxfp4_k<7, WSIDE>(plan, C, X, ldx, T, codes, scales, s);
    default: return launch_quantize_mxfp4_k<8, WSIDE>(plan, C, X, ldx, T, codes, scales, s);
    }
}

hipError_t launch_quantize_act_mxfp4(const paro_rotation &rot, const paro_half_t *X, int64_t ldx, int T, uint32_t *codes,
                                     uint8_t *scales, hipStream_t s)
{
    return launch_quantize_mxfp4_side<false>(&rot, rot.c_in, X, ldx, T, codes, scales, s);
}

// rows of a dense weight [N][ldw]; rot == nullptr: no transform
hipError_t launch_quantize_weight_mxfp4(const paro_rotation *rot, const paro_half_t *W, int64_t ldw, int N, int C,
                                        uint32_t *codes, uint8_t *scales, hipStream_t s)
{
    return launch_quantize_mxfp4_side<true>(rot, C, W, ldw, N, codes, scales, s);
}

}  // namespace paro
