// Internal declarations shared by the HIP translation units of libparo.
// Nothing here is part of the C ABI (see include/paro.h for that).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <atomic>

#include "paro.h"

namespace paro {

constexpr int kGroup = 128;        // channel-group size g (Section 5, "Implementation")
constexpr int kMaxLayers = 8;      // K
constexpr int kLanes = 64;         // one wavefront owns one (token, group): lane p <-> pair slot p
constexpr int kTileN = 16;         // output rows per weight tile (MFMA 16x16x32 B operand)
constexpr int kSliceGroups = 4;    // groups per K-slice: unit of the scales/zeros tiling

// ---------------------------------------------------------------------------------------
// Rotation plan (blob of paro_rotation_plan_build).  One block per channel group, made of
// rows of 64 dwords (one per lane), so every row is one coalesced 256-byte load:
//   row 0            io word: in_a | in_b<<8 | out_a<<16 | out_b<<24   (local channel ids)
//   row 1, 2         fp32 multipliers applied to the two loaded values (ch_scale or 1)
//   row 3, 4         fp32 multipliers applied to the two stored values (1 or ch_scale)
//   row 5+3l .. 7+3l layer l: cos(theta), sin(theta), meta
// meta bits: [7:0] byte address (lane*4) this lane pulls its next "b" value from,
//            bit 8  A_IS_I  : slot a holds channel i of the pair (else channel j)
//            bit 9  KEEP_I  : the updated channel i stays in this lane (else channel j stays)
// A lane holds two values (a, b).  After a layer it keeps one result in `a` and hands the
// other to exactly one other lane, receiving one in return: one ds_bpermute per layer.
// ---------------------------------------------------------------------------------------
constexpr int kPlanHeadRows = 5;
constexpr int kPlanRowsPerLayer = 3;
constexpr uint32_t kMetaAIsI = 1u << 8;
constexpr uint32_t kMetaKeepI = 1u << 9;

__host__ __device__ inline int plan_rows(int n_layers) { return kPlanHeadRows + kPlanRowsPerLayer * n_layers; }
__host__ __device__ inline size_t plan_group_dwords(int n_layers) { return (size_t)plan_rows(n_layers) * kLanes; }
// Second part of the plan blob, behind the rows of all groups: the same plan in 4 bytes per lane and layer, for the
// one-token linear whose waves each transform their own K-slice (every block reads the whole plan, so its size
// counts, and every (group, layer) is used once per wave, so nothing can be expanded ahead).  Per group 3 + n_layers
// rows of 64 dwords: [in_a | in_b << 8 | out_a << 16 | out_b << 24], [fp16 scale of in_a | fp16 scale of in_b << 16],
// [the same for out_a, out_b], then per layer [4 x lane to pull from | phi << 8]: keep = cos(phi) A - sin(phi) B,
// send = cos(phi) B + sin(phi) A, phi in units of 2^-24 of a revolution (the hardware sine and cosine take
// revolutions and are accurate to 1.3e-7 on these arguments, measured); see plan_build_kernel for how one angle
// per lane covers the four ways a pair can sit in a lane.
constexpr int kPlanCompactHeadRows = 3;
__host__ __device__ inline size_t plan_compact_group_dwords(int n_layers) { return (size_t)(kPlanCompactHeadRows + n_layers) * kLanes; }
__host__ __device__ inline size_t plan_compact_offset_dwords(int n_groups, int n_layers) { return (size_t)n_groups * plan_group_dwords(n_layers); }
__host__ __device__ inline size_t plan_total_dwords(int n_groups, int n_layers)
{
    return (size_t)n_groups * (plan_group_dwords(n_layers) + plan_compact_group_dwords(n_layers));
}

// ---------------------------------------------------------------------------------------
// Repacked weight blob (paro_w4_repack).  NT = c_out/16 row tiles, G = c_in/128 groups,
// S = G/4 K-slices.
//   tiles  [NT][G][64 lanes][4 dwords]   lane = kb*16 + n; dword j holds the 8 codes of row
//          16*nt+n, channels 128*g + 32*kb + 8*j + (0..7); code e sits in nibble
//          (e>>1) + 4*(e&1), so that (w & 0x000F000F), ((w>>4) & 0x000F000F), ... give
//          channel pairs (0,1), (2,3), (4,5), (6,7) as packed 16-bit lanes
//   scales [NT][S][16 n][4 groups] fp16
//   zeros  [NT][S][16 n] uint16: nibble gi = zero point of group 4*s+gi, row 16*nt+n
// ---------------------------------------------------------------------------------------
struct PackedView {
    const uint4 *tiles;
    const uint2 *scales;     // 4 fp16 per (nt, s, n)
    const uint16_t *zeros;   // 4 nibbles per (nt, s, n)
};

__host__ __device__ inline size_t packed_tiles_bytes(int c_in, int c_out) {
    return (size_t)(c_out / kTileN) * (size_t)(c_in / kGroup) * 1024u;
}
__host__ __device__ inline size_t packed_scales_bytes(int c_in, int c_out) {
    return (size_t)(c_out / kTileN) * (size_t)(c_in / kGroup / kSliceGroups) * (kTileN * kSliceGroups * 2u);
}
__host__ __device__ inline size_t packed_zeros_bytes(int c_in, int c_out) {
    return (size_t)(c_out / kTileN) * (size_t)(c_in / kGroup / kSliceGroups) * (kTileN * 2u);
}
__host__ __device__ inline PackedView packed_view(const void *blob, int c_in, int c_out) {
    const char *p = (const char *)blob;
    PackedView v;
    v.tiles = (const uint4 *)p;
    v.scales = (const uint2 *)(p + packed_tiles_bytes(c_in, c_out));
    v.zeros = (const uint16_t *)(p + packed_tiles_bytes(c_in, c_out) + packed_scales_bytes(c_in, c_out));
    return v;
}

__host__ __device__ inline size_t packed_blob_bytes(int c_in, int c_out) {
    return packed_tiles_bytes(c_in, c_out) + packed_scales_bytes(c_in, c_out) + packed_zeros_bytes(c_in, c_out);
}

// ---------------------------------------------------------------------------------------
// Exchange part of the caller's workspace (zero-filled once by the caller):
//   [0, 256)               header: word kWsErrorWord = error flags (non-zero: a bounded wait between
//                          blocks of a launch ran out)
//   [kWsPartialOff, ...)   fp32 split-K partial sums, every word reset by its reader
// ---------------------------------------------------------------------------------------
constexpr size_t kWsHeaderBytes = 256;
constexpr size_t kWsPartialOff = kWsHeaderBytes;
constexpr size_t kWsErrorWord = 2;          // index of the error word in the header

// nibble position of logical element e (0..7) inside a repacked dword
__host__ __device__ inline int packed_nibble_pos(int e) { return (e >> 1) + 4 * (e & 1); }

// Kernel attributes (dynamic LDS limit) are per device: a launcher sets them the first time it
// runs on each device.  once_pending() returns the current device if the caller still has to do
// that there (two threads may both do it: the call is idempotent), -1 if it is done.
inline int once_pending(std::atomic<uint64_t> &done)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 64;      // not tracked: set every time
    return ((done.load(std::memory_order_acquire) >> dev) & 1) ? -1 : dev;
}
inline void once_done(std::atomic<uint64_t> &done, int dev)
{
    if (dev < 64) done.fetch_or(1ull << dev, std::memory_order_release);
}

// ---------------------------------------------------------------------------------------
// Launchers (defined next to their kernels).  All return the hipError_t of the launch.
// ---------------------------------------------------------------------------------------
hipError_t launch_plan_build(const paro_rotation &rot, void *plan_out, hipStream_t s);
hipError_t launch_rotate_planned(const paro_rotation &rot, const paro_half_t *X, int64_t ldx,
                                 paro_half_t *Xr, int64_t ldxr, int T, hipStream_t s);
hipError_t launch_rotate_generic(const paro_rotation &rot, const paro_half_t *X, int64_t ldx,
                                 paro_half_t *Xr, int64_t ldxr, int T, hipStream_t s);

hipError_t launch_repack(const paro_w4_weight &w, void *packed_out, hipStream_t s);
hipError_t launch_unpack_codes(const paro_w4_weight &w, uint8_t *codes, hipStream_t s);
hipError_t launch_unpack_zeros(const paro_w4_weight &w, uint8_t *zeros, hipStream_t s);
hipError_t launch_dequant(const paro_w4_weight &w, paro_half_t *W, hipStream_t s);

// Decode-side linear with the rotation fused (K-major kernel, T <= 4 at the call sites; the
// kernel itself takes up to 16 tokens).
struct DecodeGeometry {
    int ks;           // K-slices (grid.x)
    int nb;           // N-blocks per slice (grid.y)
    int waves;        // waves per block (4, or 8 for one token and many K-slices)
    int tiles_per_block;
    size_t partial_bytes;   // fp32 partial sums [ks][T][c_out] (0 when ks == 1)
};
DecodeGeometry decode_geometry(int c_in, int c_out, int T, int target_blocks = 0);
hipError_t launch_decode(const paro_rotation *rot, const paro_w4_weight &w, const paro_half_t *X, int64_t ldx,
                         paro_half_t *Y, int64_t ldy, int T, void *ws, hipStream_t s);
// Several linears on the same activations, each with its own transform, in one launch (T <= 4;
// every part planned and repacked, same c_in and layer count).  Workspace: decode_multi_bytes.
size_t decode_multi_bytes(int n_parts, const paro_w4_weight *const *w, int T);
hipError_t launch_decode_multi(int n_parts, const paro_rotation *const *rot, const paro_w4_weight *const *w,
                               const paro_half_t *X, int64_t ldx, paro_half_t *const *Y, const int64_t *ldy, int T,
                               void *ws, hipStream_t s);
// Wide decode kernel (bare linear, T <= 16): all K-slices of a tile range in one block (up to 12),
// reduced through LDS; wider layers spread the slices over several blocks and exchange partials.
// ws: the exchange part of the workspace.
size_t decode_wide_partial_bytes(int c_in, int c_out, int T);
bool decode_wide_hosts(const paro_rotation &rot, int T);
bool decode_wide_hosting_pays(int c_in, int c_out);
hipError_t launch_decode_wide(const paro_w4_weight &w, const paro_half_t *X, int64_t ldx, paro_half_t *Y, int64_t ldy,
                              int T, void *ws, hipStream_t s, const paro_rotation *rot = nullptr);
hipError_t launch_linear_generic(const paro_w4_weight &w, const paro_half_t *X, int64_t ldx,
                                 paro_half_t *Y, int64_t ldy, int T, hipStream_t s);

// Weight-side transform + RTN quantiser (rot == nullptr: no transform; otherwise rot->plan is set).
hipError_t launch_quantize(const paro_rotation *rot, const paro_half_t *W, int64_t ldw, int N, int C, uint32_t *qweight,
                           paro_half_t *scales, uint32_t *qzeros, hipStream_t s);

// Transformed activations quantised to INT4 per (token, group) right after the rotation (rot.plan set).
hipError_t launch_quantize_act(const paro_rotation &rot, const paro_half_t *X, int64_t ldx, int T, uint32_t *codes,
                               paro_half_t *scales, uint8_t *zeros, hipStream_t s);

// The same with the MXFP4 quantiser: E2M1 codes, one E8M0 scale byte per 32 channels.
hipError_t launch_quantize_weight_mxfp4(const paro_rotation *rot, const paro_half_t *W, int64_t ldw, int N, int C,
                                        uint32_t *codes, uint8_t *scales, hipStream_t s);
// XCD patches of a tiled launch (gemm.hip): tiles of one patch share panels through one XCD's L2
void gemm_patches(int m_tiles, int n_tiles, int &patch_m, int &patch_n, int &blocks);
// MXFP4 x MXFP4 linear (App. A.3) on the block-scaled FP4 matrix instruction
hipError_t launch_mxfp4_repack(const paro_mxfp4_weight &w, void *packed_out, hipStream_t s);
hipError_t launch_mxfp4_unpack(const paro_mxfp4_weight &w, uint8_t *codes, uint8_t *scales, hipStream_t s);
bool mxfp4_linear_supported(const paro_mxfp4_weight &w);
hipError_t launch_mxfp4_linear(const paro_mxfp4_weight &w, const uint32_t *x_codes, const uint8_t *x_scales, int T,
                               paro_half_t *Y, int64_t ldy, hipStream_t s);
hipError_t launch_quantize_act_mxfp4(const paro_rotation &rot, const paro_half_t *X, int64_t ldx, int T, uint32_t *codes,
                                     uint8_t *scales, hipStream_t s);

// Prefill-side linear (MFMA GEMM on the repacked weight), any T.
bool gemm_supported(const paro_w4_weight &w, int64_t ldx, int64_t ldy, int T);
double gemm_estimate_us(const paro_w4_weight &w, int T);
// scratch: room for split-K partial tiles (gemm_scratch_bytes; any contents before and after);
// without it the call runs unsplit.
size_t gemm_scratch_bytes(const paro_w4_weight &w, int T);
hipError_t launch_gemm(const paro_w4_weight &w, const paro_half_t *X, int64_t ldx, paro_half_t *Y, int64_t ldy,
                       int T, void *scratch, size_t scratch_bytes, hipStream_t s);

}  // namespace paro
