// Scaled pairwise rotation of activations (Section 4.1, Eq. 4/5/8; kernel idea of Section 4.3
// re-designed for CDNA4 wave64):
//
//   one wavefront owns one (token, channel group); lane p owns the pair it is currently
//   rotating, as two fp32 registers (a, b).  Because the pairs of a layer are disjoint
//   (Def. 1) the 64 lanes never need to synchronise inside a layer.  Between layer l and
//   l+1 the union of the two perfect matchings is a set of alternating cycles, so the pair
//   of layer l+1 can be placed in a lane that already holds one of its two channels: every
//   lane keeps one value and receives exactly one from another lane - a single
//   ds_bpermute_b32 per layer, no LDS allocation, no barrier.  The routing, cos/sin (fp64
//   evaluation rounded to fp32) and the folded channel scales are precomputed once per
//   weight into a "plan" (paro_rotation_plan_build).
#include "paro_internal.h"
#include "rotate_lane.h"
#include <type_traits>

namespace paro {

// ------------------------------------------------------------------------------------------
// Plan build: one 64-thread block per channel group.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void plan_build_kernel(const int16_t *__restrict__ pairs,
                                                        const float *__restrict__ theta,
                                                        const paro_half_t *__restrict__ ch_scale, int n_layers,
                                                        int ppl, int scale_order, uint32_t *__restrict__ plan)
{
    __shared__ uint8_t s_pi[kMaxLayers][64], s_pj[kMaxLayers][64];   // completed matching per layer
    __shared__ int16_t s_slot[kMaxLayers][64];                        // source slot of pair, -1 = filler
    __shared__ float s_c[kMaxLayers][64], s_s[kMaxLayers][64];
    __shared__ uint32_t s_rev[kMaxLayers][64];                        // angle of the pair in units of 2^-24 of a revolution
    __shared__ uint8_t s_cha[kMaxLayers][64], s_chb[kMaxLayers][64];  // channels in slots a, b before layer l
    __shared__ uint8_t s_pair[kMaxLayers][64];                        // which completed pair lane p processes
    __shared__ uint8_t s_src[kMaxLayers][64];                         // lane to pull from after layer l
    __shared__ uint8_t s_keep[kMaxLayers][64], s_send[kMaxLayers][64];
    __shared__ uint8_t s_tmp[3][128];
    __shared__ int s_bad;                                             // the table violates Def. 1 (or an index is out of range)

    const int g = blockIdx.x;
    const int lane = threadIdx.x;
    const int16_t *gp = pairs + (size_t)g * n_layers * ppl * 2;
    const float *gt = theta + (size_t)g * n_layers * ppl;

    // Phase A: complete every layer to a perfect matching of the 128 channels.  Channels that
    // no pair of the layer names are paired among themselves with the identity rotation.
    if (lane == 0) {
        uint8_t *used = s_tmp[0];
        s_bad = 0;
        for (int l = 0; l < n_layers; ++l) {
            for (int c = 0; c < kGroup; ++c) used[c] = 0;
            int cnt = 0;
            for (int p = 0; p < ppl && cnt < 64; ++p) {
                int i = gp[((size_t)l * ppl + p) * 2], j = gp[((size_t)l * ppl + p) * 2 + 1];
                if (i == j) continue;                                   // empty slot
                if (i < 0 || j < 0 || i >= kGroup || j >= kGroup || used[i] || used[j]) { s_bad = 1; continue; }
                used[i] = used[j] = 1;
                s_pi[l][cnt] = (uint8_t)i; s_pj[l][cnt] = (uint8_t)j; s_slot[l][cnt] = (int16_t)p;
                ++cnt;
            }
            int first = -1;
            for (int c = 0; c < kGroup && cnt < 64; ++c) {
                if (used[c]) continue;
                if (first < 0) { first = c; continue; }
                s_pi[l][cnt] = (uint8_t)first; s_pj[l][cnt] = (uint8_t)c; s_slot[l][cnt] = -1;
                ++cnt; first = -1;
            }
        }
    }
    __syncthreads();
    for (int l = 0; l < n_layers; ++l) {
        int slot = s_slot[l][lane];
        float c = 1.0f, s = 0.0f;
        uint32_t rev = 0;
        if (slot >= 0) {
            double sd, cd;
            const double th = (double)gt[(size_t)l * ppl + slot];
            sincos(th, &sd, &cd);
            c = (float)cd; s = (float)sd;
            double turns = th * 0.15915494309189535;                  // 1 / (2 pi)
            turns -= floor(turns);
            rev = (uint32_t)llrint(turns * 16777216.0) & 0xFFFFFFu;
        }
        s_c[l][lane] = c; s_s[l][lane] = s; s_rev[l][lane] = rev;
    }
    __syncthreads();

    // Phase B: lane assignment.  Layer 0: lane p takes completed pair p with a = i, b = j.
    // For each following layer walk the alternating cycles of (layer l) U (layer l+1).
    if (lane == 0) {
        for (int p = 0; p < 64; ++p) {
            if (n_layers > 0) { s_cha[0][p] = s_pi[0][p]; s_chb[0][p] = s_pj[0][p]; s_pair[0][p] = (uint8_t)p; }
        }
        uint8_t *lane_of = s_tmp[0], *partner = s_tmp[1], *pair_of = s_tmp[2];
        for (int l = 0; l + 1 < n_layers; ++l) {
            for (int p = 0; p < 64; ++p) {
                lane_of[s_cha[l][p]] = (uint8_t)p; lane_of[s_chb[l][p]] = (uint8_t)p;
                partner[s_pi[l + 1][p]] = s_pj[l + 1][p]; partner[s_pj[l + 1][p]] = s_pi[l + 1][p];
                pair_of[s_pi[l + 1][p]] = (uint8_t)p; pair_of[s_pj[l + 1][p]] = (uint8_t)p;
            }
            uint64_t visited = 0;
            for (int p0 = 0; p0 < 64; ++p0) {
                if ((visited >> p0) & 1) continue;
                int p = p0;
                int x = s_cha[l][p0];                     // channel this lane hands on
                for (int guard = 0; guard < 64; ++guard) {
                    visited |= 1ull << p;
                    int y = (s_cha[l][p] == x) ? s_chb[l][p] : s_cha[l][p];   // channel that stays
                    s_send[l][p] = (uint8_t)x; s_keep[l][p] = (uint8_t)y;
                    int xn = partner[y];
                    int pn = lane_of[xn];
                    s_src[l][p] = (uint8_t)pn;
                    s_cha[l + 1][p] = (uint8_t)y; s_chb[l + 1][p] = (uint8_t)xn; s_pair[l + 1][p] = pair_of[y];
                    p = pn; x = xn;
                    if (p == p0) break;
                }
            }
        }
        if (n_layers > 0) {
            int l = n_layers - 1;
            for (int p = 0; p < 64; ++p) {
                s_keep[l][p] = s_pi[l][s_pair[l][p]]; s_send[l][p] = s_pj[l][s_pair[l][p]]; s_src[l][p] = (uint8_t)p;
            }
        }
    }
    __syncthreads();

    // Phase C: write the rows.
    uint32_t *out = plan + (size_t)g * plan_group_dwords(n_layers);
    int in_a, in_b, out_a, out_b;
    if (n_layers > 0) {
        in_a = s_cha[0][lane]; in_b = s_chb[0][lane];
        out_a = s_keep[n_layers - 1][lane]; out_b = s_send[n_layers - 1][lane];
    } else {
        in_a = out_a = 2 * lane; in_b = out_b = 2 * lane + 1;
    }
    out[0 * 64 + lane] = (uint32_t)in_a | ((uint32_t)in_b << 8) | ((uint32_t)out_a << 16) | ((uint32_t)out_b << 24);
    const _Float16 *cs = (const _Float16 *)ch_scale;
    float one = 1.0f;
    float sia = one, sib = one, soa = one, sob = one;
    if (cs) {
        if (scale_order == 0) { sia = (float)cs[(size_t)g * kGroup + in_a]; sib = (float)cs[(size_t)g * kGroup + in_b]; }
        else                  { soa = (float)cs[(size_t)g * kGroup + out_a]; sob = (float)cs[(size_t)g * kGroup + out_b]; }
    }
    // A pair table that is not an independent rotation (Def. 1) has no defined result: the group's outputs
    // become NaN on every path that uses this plan, as they do on the planless path.
    if (s_bad) sia = sib = soa = sob = __builtin_nanf("");
    out[1 * 64 + lane] = __float_as_uint(sia); out[2 * 64 + lane] = __float_as_uint(sib);
    out[3 * 64 + lane] = __float_as_uint(soa); out[4 * 64 + lane] = __float_as_uint(sob);
    for (int l = 0; l < n_layers; ++l) {
        int pr = s_pair[l][lane];
        uint32_t meta = (uint32_t)s_src[l][lane] << 2;
        if (s_cha[l][lane] == s_pi[l][pr]) meta |= kMetaAIsI;
        if (s_keep[l][lane] == s_pi[l][pr]) meta |= kMetaKeepI;
        uint32_t *row = out + (size_t)(kPlanHeadRows + kPlanRowsPerLayer * l) * 64;
        row[0 * 64 + lane] = __float_as_uint(s_c[l][pr]);
        row[1 * 64 + lane] = __float_as_uint(s_s[l][pr]);
        row[2 * 64 + lane] = meta;
    }
    // The compact copy (see plan_compact_group_dwords).  Per lane and layer ONE angle phi and the lane to pull from:
    //     keep = cos(phi) A - sin(phi) B,   send = cos(phi) B + sin(phi) A
    // with no case distinction at run time.  The 2 x 2 block that maps the lane's (A, B) to (keep, send) is
    // [k0 k1; s (-k1) s k0] with (k0, k1) one of (c, -s), (s, c), (-s, c), (c, s) and s = +1 where "A holds i" and
    // "i is kept" agree, -1 otherwise; the formula above yields s * send, so the sent value may carry a sign that
    // is known here: eps of the value a lane receives multiplies its k1 (which turns phi into another multiple of
    // the pair's angle and a quarter turn), the kept value is always true, and the sign of the last layer's
    // second output goes into its output scale.
    __shared__ int8_t s_eps[64];
    uint32_t *cout = plan + plan_compact_offset_dwords(gridDim.x, n_layers) + (size_t)g * plan_compact_group_dwords(n_layers);
    auto h16 = [](float f) { union { _Float16 h; uint16_t u; } v; v.h = (_Float16)f; return (uint32_t)v.u; };
    int eps_b = 1, eps_out = 1;
    for (int l = 0; l < n_layers; ++l) {
        const int pr = s_pair[l][lane];
        const bool ai = s_cha[l][lane] == s_pi[l][pr], ki = s_keep[l][lane] == s_pi[l][pr];
        const uint32_t th = s_rev[l][pr], q4 = 1u << 22;
        uint32_t phi;
        if (ai && ki)        phi = eps_b > 0 ? th : 0u - th;
        else if (ai && !ki)  phi = eps_b > 0 ? th - q4 : q4 - th;
        else if (!ai && ki)  phi = eps_b > 0 ? 0u - th - q4 : th + q4;
        else                 phi = eps_b > 0 ? 0u - th : th;
        cout[(size_t)(kPlanCompactHeadRows + l) * 64 + lane] = ((uint32_t)s_src[l][lane] << 2) | ((phi & 0xFFFFFFu) << 8);
        const int eps_send = (ai == ki) ? eps_b : -eps_b;
        __syncthreads();
        s_eps[lane] = (int8_t)eps_send;
        __syncthreads();
        if (l + 1 < n_layers) eps_b = s_eps[s_src[l][lane]];
        else eps_out = eps_send;
    }
    cout[0 * 64 + lane] = out[0 * 64 + lane];
    cout[1 * 64 + lane] = h16(sia) | (h16(sib) << 16);
    cout[2 * 64 + lane] = h16(soa) | (h16(eps_out > 0 ? sob : -sob) << 16);
}

hipError_t launch_plan_build(const paro_rotation &rot, void *plan_out, hipStream_t s)
{
    int G = rot.c_in / rot.group;
    hipLaunchKernelGGL(plan_build_kernel, dim3(G), dim3(64), 0, s, rot.pairs, rot.theta, rot.ch_scale, rot.n_layers,
                       rot.pairs_per_layer, rot.scale_order, (uint32_t *)plan_out);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Planned rotation kernel.
// ------------------------------------------------------------------------------------------
constexpr int kRotWaves = 4;   // waves per block
constexpr int kRotTU = 4;      // tokens in flight per wave
constexpr int kRotMaxBatches = 8;   // batches of kRotTU tokens per wave (the batch loop is unrolled)

// f(0), f(1), ... while f returns true, at most N times; nested, so that stopping is one forward jump
template <int N, class F, int I = 0>
__device__ __forceinline__ void static_while_rot(F &&f)
{
    if constexpr (I < N) {
        if (f(std::integral_constant<int, I>{})) static_while_rot<N, F, I + 1>(static_cast<F &&>(f));
    }
}

// A wave owns one group and a run of tokens.  Global traffic is one coalesced 4-byte access per
// lane, token and direction (a group row is 256 contiguous bytes); the permutation between
// channel order and the plan's lane order goes through a wave-private LDS buffer (no block
// barrier: LDS operations of one wave execute in issue order).  The loads of the next batch of
// tokens are issued before the current batch is rotated.  Rows are read completely before any of
// them is written, so X and Xr may be the same buffer.
template <int K>
__global__ __launch_bounds__(kRotWaves * 64) void rotate_planned_kernel(const uint32_t *__restrict__ plan,
                                                                         const _Float16 *X, int64_t ldx,
                                                                         _Float16 *Xr, int64_t ldxr, int T,
                                                                         int tokens_per_wave)
{
    __shared__ _Float16 s_stage[kRotWaves][kRotTU][kGroup];
    const int g = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int t0 = (blockIdx.y * kRotWaves + wave) * tokens_per_wave;
    if (t0 >= T) return;
    const int n_tok = min(T, t0 + tokens_per_wave) - t0;

    // The wave's rows through raw buffer resources based at its first row: offsets are 32-bit
    // (a scalar row offset plus the lane's 4 bytes, in the range-checked vector offset), and rows
    // beyond the run read as zero and are not written - no 64-bit address arithmetic, no clamps,
    // no predication.
    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<_Float16 *>(X + (size_t)t0 * ldx + (size_t)g * kGroup), 0, (int)((size_t)(n_tok - 1) * ldx * 2 + kGroup * 2),
        0x00020000);
    const __amdgpu_buffer_rsrc_t yr = __builtin_amdgcn_make_buffer_rsrc(
        Xr + (size_t)t0 * ldxr + (size_t)g * kGroup, 0, (int)((size_t)(n_tok - 1) * ldxr * 2 + kGroup * 2), 0x00020000);
    const int row_x = (int)(ldx * 2), row_y = (int)(ldxr * 2);         // bytes per token row
    const int v4 = lane * 4;
    uint32_t cur[kRotTU], nxt[kRotTU];
#pragma unroll
    for (int u = 0; u < kRotTU; ++u) cur[u] = __builtin_amdgcn_raw_buffer_load_b32(xr, v4 + u * row_x, 0, 0);

    LanePlan<K> P;
    load_lane_plan<K>(plan + (size_t)g * plan_group_dwords(K), lane, P);
    // Staging layout: [channel][token of the batch], 4 fp16 = 8 bytes per channel, so that the
    // gather of a lane's two channels and the scatter of its two results take one 8-byte LDS access
    // each for all 4 tokens (the LDS pipe, shared by the CU's four SIMDs, is as loaded as the vector
    // pipes in this kernel).  A lane's loads hold channels 2 lane and 2 lane + 1 of each token:
    // transposed in registers to (4 tokens of channel 2 lane, 4 tokens of channel 2 lane + 1) =
    // 16 contiguous bytes, and back on the way out.
    static_assert(kRotTU == 4, "8 bytes per channel");
    typedef _Float16 half4v __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
    char *sp = (char *)s_stage[wave];                      // 128 channels x 8 bytes
    auto lo_pair = [](uint32_t x, uint32_t y) { return (x & 0xffffu) | (y << 16); };
    auto hi_pair = [](uint32_t x, uint32_t y) { return (x >> 16) | (y & 0xffff0000u); };

    // Unrolled over the wave's batches (at most kRotMaxBatches, guaranteed by the launcher) with one early exit:
    // with a back edge the compiler waits for ALL outstanding memory operations at the loop head, i.e. for the
    // previous batch's stores to be acknowledged before the next batch may be touched; straight-line code waits
    // for the loads only.
    static_while_rot<kRotMaxBatches>([&](auto I) {
        constexpr int t = I * kRotTU;
        if (t >= n_tok) return false;
#pragma unroll
        for (int u = 0; u < kRotTU; ++u) nxt[u] = __builtin_amdgcn_raw_buffer_load_b32(xr, v4 + (t + kRotTU + u) * row_x, 0, 0);
        const u32x4v in = {lo_pair(cur[0], cur[1]), lo_pair(cur[2], cur[3]), hi_pair(cur[0], cur[1]), hi_pair(cur[2], cur[3])};
        *(u32x4v *)(sp + lane * 16) = in;
        __builtin_amdgcn_wave_barrier();
        const half4v ha = *(const half4v *)(sp + P.in_a * 8), hb = *(const half4v *)(sp + P.in_b * 8);
        float a[kRotTU], b[kRotTU];
#pragma unroll
        for (int u = 0; u < kRotTU; ++u) {
            a[u] = (float)ha[u] * P.sia;
            b[u] = (float)hb[u] * P.sib;
        }
        rotate_layers<K, kRotTU>(P, a, b);
        __builtin_amdgcn_wave_barrier();
        half4v oa, ob;
#pragma unroll
        for (int u = 0; u < kRotTU; ++u) {
            oa[u] = (_Float16)(a[u] * P.soa);
            ob[u] = (_Float16)(b[u] * P.sob);
        }
        *(half4v *)(sp + P.out_a * 8) = oa;
        *(half4v *)(sp + P.out_b * 8) = ob;
        __builtin_amdgcn_wave_barrier();
        const u32x4v out = *(const u32x4v *)(sp + lane * 16);
        const uint32_t o[kRotTU] = {lo_pair(out[0], out[2]), hi_pair(out[0], out[2]), lo_pair(out[1], out[3]), hi_pair(out[1], out[3])};
#pragma unroll
        for (int u = 0; u < kRotTU; ++u) __builtin_amdgcn_raw_buffer_store_b32(o[u], yr, v4 + (t + u) * row_y, 0, 0);
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < kRotTU; ++u) cur[u] = nxt[u];
        return true;
    });
}

template <int K>
static hipError_t launch_rotate_k(const paro_rotation &rot, const paro_half_t *X, int64_t ldx, paro_half_t *Xr,
                                  int64_t ldxr, int T, hipStream_t s)
{
    int G = rot.c_in / kGroup;
    // the plan (7.4 KB per wave at K = 8) is re-read by every wave: long token runs per wave, as
    // long as there are still enough waves to fill 256 CUs several times over
    int tpw = kRotMaxBatches * kRotTU;
    while (tpw > kRotTU && (int64_t)G * ((T + tpw - 1) / tpw) < 4096) tpw >>= 1;
    int waves_t = (T + tpw - 1) / tpw;
    dim3 grid(G, (waves_t + kRotWaves - 1) / kRotWaves);
    hipLaunchKernelGGL(rotate_planned_kernel<K>, grid, dim3(kRotWaves * 64), 0, s, (const uint32_t *)rot.plan,
                       (const _Float16 *)X, ldx, (_Float16 *)Xr, ldxr, T, tpw);
    return hipGetLastError();
}

hipError_t launch_rotate_planned(const paro_rotation &rot, const paro_half_t *X, int64_t ldx, paro_half_t *Xr,
                                 int64_t ldxr, int T, hipStream_t s)
{
    switch (rot.n_layers) {
    case 0: return launch_rotate_k<0>(rot, X, ldx, Xr, ldxr, T, s);
    case 1: return launch_rotate_k<1>(rot, X, ldx, Xr, ldxr, T, s);
    case 2: return launch_rotate_k<2>(rot, X, ldx, Xr, ldxr, T, s);
    case 3: return launch_rotate_k<3>(rot, X, ldx, Xr, ldxr, T, s);
    case 4: return launch_rotate_k<4>(rot, X, ldx, Xr, ldxr, T, s);
    case 5: return launch_rotate_k<5>(rot, X, ldx, Xr, ldxr, T, s);
    case 6: return launch_rotate_k<6>(rot, X, ldx, Xr, ldxr, T, s);
    case 7: return launch_rotate_k<7>(rot, X, ldx, Xr, ldxr, T, s);
    default: return launch_rotate_k<8>(rot, X, ldx, Xr, ldxr, T, s);
    }
}

// ------------------------------------------------------------------------------------------
// Generic rotation kernel: reads pairs/theta directly (no plan).  One wave per block; the
// group's 128 channels of one token live in LDS as fp32, each lane updates the pair of its
// slot (Eq. 4), layers in array order (Eq. 5).  Slower; used when no plan was built.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void rotate_generic_kernel(const int16_t *__restrict__ pairs,
                                                            const float *__restrict__ theta,
                                                            const _Float16 *__restrict__ ch_scale, int n_layers,
                                                            int ppl, int scale_order, const _Float16 *X, int64_t ldx,
                                                            _Float16 *Xr, int64_t ldxr, int T, int tokens_per_block)
{
    __shared__ float s_c[kMaxLayers][64], s_s[kMaxLayers][64];
    __shared__ int16_t s_i[kMaxLayers][64], s_j[kMaxLayers][64];
    __shared__ float s_u[kGroup];
    __shared__ int s_claims[kGroup];                                  // slots of the current layer that name a channel
    __shared__ int s_bad;                                             // Def. 1 violated / index out of range: outputs NaN
    const int g = blockIdx.x, lane = threadIdx.x;
    if (lane == 0) s_bad = 0;
    for (int l = 0; l < n_layers; ++l) {
        s_claims[lane] = 0; s_claims[64 + lane] = 0;
        __syncthreads();
        int i = 0, j = 0;
        float c = 1.0f, s = 0.0f;
        if (lane < ppl) {
            size_t k = ((size_t)g * n_layers + l) * ppl + lane;
            i = pairs[2 * k]; j = pairs[2 * k + 1];
            if (i < 0 || j < 0 || i >= kGroup || j >= kGroup) { i = 0; j = 0; s_bad = 1; }
            if (i != j && (atomicAdd(&s_claims[i], 1) > 0 || atomicAdd(&s_claims[j], 1) > 0)) { s_bad = 1; i = j = 0; }
            if (i != j) {
                double sd, cd;
                sincos((double)theta[k], &sd, &cd);
                c = (float)cd; s = (float)sd;
            }
        }
        s_i[l][lane] = (int16_t)i; s_j[l][lane] = (int16_t)j; s_c[l][lane] = c; s_s[l][lane] = s;
    }
    float sc0 = 1.0f, sc1 = 1.0f;
    if (ch_scale) { sc0 = (float)ch_scale[(size_t)g * kGroup + lane]; sc1 = (float)ch_scale[(size_t)g * kGroup + 64 + lane]; }
    __syncthreads();
    const bool bad = s_bad != 0;
    const int t0 = blockIdx.y * tokens_per_block, t1 = min(T, t0 + tokens_per_block);
    for (int t = t0; t < t1; ++t) {
        float v0 = (float)X[(size_t)t * ldx + (size_t)g * kGroup + lane];
        float v1 = (float)X[(size_t)t * ldx + (size_t)g * kGroup + 64 + lane];
        if (scale_order == 0) { v0 *= sc0; v1 *= sc1; }
        s_u[lane] = v0; s_u[64 + lane] = v1;
        __syncthreads();
        for (int l = 0; l < n_layers; ++l) {
            int i = s_i[l][lane], j = s_j[l][lane];
            float ui = s_u[i], uj = s_u[j];
            __syncthreads();
            if (i != j) {
                float c = s_c[l][lane], s = s_s[l][lane];
                s_u[i] = c * ui - s * uj;
                s_u[j] = s * ui + c * uj;
            }
            __syncthreads();
        }
        v0 = s_u[lane]; v1 = s_u[64 + lane];
        if (scale_order == 1) { v0 *= sc0; v1 *= sc1; }
        Xr[(size_t)t * ldxr + (size_t)g * kGroup + lane] = (_Float16)(bad ? __builtin_nanf("") : v0);
        Xr[(size_t)t * ldxr + (size_t)g * kGroup + 64 + lane] = (_Float16)(bad ? __builtin_nanf("") : v1);
        __syncthreads();
    }
}

hipError_t launch_rotate_generic(const paro_rotation &rot, const paro_half_t *X, int64_t ldx, paro_half_t *Xr,
                                 int64_t ldxr, int T, hipStream_t s)
{
    int G = rot.c_in / kGroup;
    int tpb = 16;
    dim3 grid(G, (T + tpb - 1) / tpb);
    hipLaunchKernelGGL(rotate_generic_kernel, grid, dim3(64), 0, s, rot.pairs, rot.theta,
                       (const _Float16 *)rot.ch_scale, rot.n_layers, rot.pairs_per_layer, rot.scale_order,
                       (const _Float16 *)X, ldx, (_Float16 *)Xr, ldxr, T, tpb);
    return hipGetLastError();
}

}  // namespace paro
