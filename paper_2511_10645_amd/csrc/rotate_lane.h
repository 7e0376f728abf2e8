// Per-lane view of a rotation plan and the layer loop shared by the kernels that rotate one
// (row, group) per wavefront (Eq. 4, 5): the activation transform and the weight-side quantiser.
#pragma once
#include "paro_internal.h"

namespace paro {

template <int K>
struct LanePlan {
    float m00[K > 0 ? K : 1], m01[K > 0 ? K : 1], m10[K > 0 ? K : 1], m11[K > 0 ? K : 1];
    int src[K > 0 ? K : 1];
    int in_a, in_b, out_a, out_b;
    float sia, sib, soa, sob;
};

// Expand (cos, sin, meta) into the 2x2 block that maps the lane's (a, b) to (keep, send).
__device__ inline void expand_coeffs(float c, float s, uint32_t meta, float &m00, float &m01, float &m10, float &m11)
{
    bool ai = meta & kMetaAIsI, ki = meta & kMetaKeepI;
    // updated channel i and j as combinations of (a, b)   (Eq. 4)
    float ni_a = ai ? c : -s, ni_b = ai ? -s : c;
    float nj_a = ai ? s : c,  nj_b = ai ? c : s;
    m00 = ki ? ni_a : nj_a; m01 = ki ? ni_b : nj_b;
    m10 = ki ? nj_a : ni_a; m11 = ki ? nj_b : ni_b;
}

template <int K>
__device__ inline void load_lane_plan(const uint32_t *__restrict__ gplan, int lane, LanePlan<K> &P)
{
    uint32_t io = gplan[lane];
    P.in_a = io & 0xff; P.in_b = (io >> 8) & 0xff; P.out_a = (io >> 16) & 0xff; P.out_b = io >> 24;
    P.sia = __uint_as_float(gplan[1 * 64 + lane]); P.sib = __uint_as_float(gplan[2 * 64 + lane]);
    P.soa = __uint_as_float(gplan[3 * 64 + lane]); P.sob = __uint_as_float(gplan[4 * 64 + lane]);
#pragma unroll
    for (int l = 0; l < K; ++l) {
        const uint32_t *row = gplan + (size_t)(kPlanHeadRows + kPlanRowsPerLayer * l) * 64;
        float c = __uint_as_float(row[lane]), s = __uint_as_float(row[64 + lane]);
        uint32_t meta = row[128 + lane];
        expand_coeffs(c, s, meta, P.m00[l], P.m01[l], P.m10[l], P.m11[l]);
        P.src[l] = (int)(meta & 0xff);
    }
}

// Run the K layers on TU independent tokens held as (a[u], b[u]); results: a = kept, b = sent slot.
template <int K, int TU>
__device__ inline void rotate_layers(const LanePlan<K> &P, float (&a)[TU], float (&b)[TU])
{
#pragma unroll
    for (int l = 0; l < K; ++l) {
#pragma unroll
        for (int u = 0; u < TU; ++u) {
            float na = P.m00[l] * a[u] + P.m01[l] * b[u];
            float nb = P.m10[l] * a[u] + P.m11[l] * b[u];
            a[u] = na;
            b[u] = (l + 1 < K) ? __int_as_float(__builtin_amdgcn_ds_bpermute(P.src[l], __float_as_int(nb))) : nb;
        }
    }
}

}  // namespace paro
