// C ABI of libparo (include/paro.h): argument validation on the host, then dispatch to the
// kernels.  No device memory is allocated or retained here.
#include "paro_internal.h"
#include <algorithm>
#include <vector>

using namespace paro;

namespace {

constexpr int kFuseMaxTokens = 4;            // the K-major decode kernel hosts the rotation up to this many tokens
constexpr int64_t kMaxRowStride = 1 << 22;   // elements; the kernels address a run of up to 256 rows with 31-bit byte offsets
constexpr int kDecodeMaxTokens = 16;         // above this the MFMA GEMM competes with passes of the streaming decode kernel
constexpr int kStreamPassTokens = 32;        // tokens of one pass of the streaming kernel (two blocks of 16)

inline bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

paro_status check_rotation(const paro_rotation *r)
{
    if (!r) return PARO_ERR_NULL;
    if (r->group != kGroup) return PARO_ERR_UNSUPPORTED;
    if (r->n_layers < 0 || r->n_layers > kMaxLayers) return PARO_ERR_UNSUPPORTED;
    if (r->pairs_per_layer < 1 || r->pairs_per_layer > kGroup / 2) return PARO_ERR_UNSUPPORTED;
    if (r->scale_order != 0 && r->scale_order != 1) return PARO_ERR_UNSUPPORTED;
    if (r->c_in <= 0 || r->c_in % r->group) return PARO_ERR_SHAPE;
    if (r->n_layers > 0 && (!r->pairs || !r->theta)) return PARO_ERR_NULL;
    if (!aligned(r->pairs, 4) || !aligned(r->theta, 4) || !aligned(r->ch_scale, 2) || !aligned(r->plan, 256))
        return PARO_ERR_ALIGN;
    return PARO_OK;
}

paro_status check_weight(const paro_w4_weight *w, bool need_interchange)
{
    if (!w) return PARO_ERR_NULL;
    if (w->group != kGroup) return PARO_ERR_UNSUPPORTED;
    if (w->c_in <= 0 || w->c_out <= 0 || w->c_in % w->group || w->c_out % kTileN) return PARO_ERR_SHAPE;
    bool have_ic = w->qweight && w->scales && w->qzeros;
    if (need_interchange ? !have_ic : (!have_ic && !w->packed)) return PARO_ERR_NULL;
    if (!aligned(w->qweight, 16) || !aligned(w->scales, 2) || !aligned(w->qzeros, 4) || !aligned(w->bias, 2) ||
        !aligned(w->packed, 256))
        return PARO_ERR_ALIGN;
    return PARO_OK;
}

// the tiled kernels address the repacked blob with 32-bit byte offsets
inline bool fast_weight(const paro_w4_weight *w)
{
    return w->packed && (w->c_in / kGroup) % kSliceGroups == 0 && packed_blob_bytes(w->c_in, w->c_out) < (1ull << 31);
}

// The K-major decode kernel can host the rotation: planned rotation, repacked weight, few tokens.
inline bool can_fuse_decode(const paro_rotation *rot, const paro_w4_weight *w, int T)
{
    return rot && rot->plan && fast_weight(w) && T <= kFuseMaxTokens;
}

// Whether it does.  Its blocks exchange KS x T x c_out fp32 partial sums at the end, which costs a
// device-scope round trip plus the volume; a rotation pass followed by the bare kernel (all K-slices
// in one block, no exchange up to 6144 channels) costs one more launch, 2.6 us on the small
// linears and well under 1 us in front of a long weight stream.  Measured break-even on MI355X
// (4096 / 5120 / 14336 / 27648 input channels, 4096 .. 55296 outputs): 1 - 2 MB of partial sums
// for one token, 0.75 MB for 2..4 tokens.  `always`: for callers without a scratch part.
constexpr size_t kFusePartialOne = 3u << 19, kFusePartialFew = 3u << 18;
// One token, the paper's 8 layers, a weight stream of some length per wave: the kernel in which every wave transforms
// its own K-slice (decode_wide.hip) - nothing is exchanged between blocks that the bare linear would not exchange, and
// the stream hides the transform (decode_wide_hosting_pays has the measurements behind the rule).
inline bool fused_wide(const paro_rotation *rot, const paro_w4_weight *w, int T)
{
    return can_fuse_decode(rot, w, T) && decode_wide_hosts(*rot, T) && decode_wide_hosting_pays(w->c_in, w->c_out);
}
inline bool fused_decode(const paro_rotation *rot, const paro_w4_weight *w, int T, bool always = false)
{
    if (!can_fuse_decode(rot, w, T)) return false;
    if (always || fused_wide(rot, w, T)) return true;
    return decode_geometry(w->c_in, w->c_out, T).partial_bytes <= (T == 1 ? kFusePartialOne : kFusePartialFew);
}

paro_status check_io(const void *X, int64_t ldx, int width_x, const void *Y, int64_t ldy, int width_y, int T,
                     int64_t ld_mult)
{
    if (!X || !Y) return PARO_ERR_NULL;
    if (T <= 0 || ldx < width_x || ldy < width_y) return PARO_ERR_SHAPE;
    if (ldx >= kMaxRowStride || ldy >= kMaxRowStride) return PARO_ERR_UNSUPPORTED;   // 32-bit offsets inside a run of rows
    if (ldx % ld_mult || ldy % ld_mult || !aligned(X, 2 * ld_mult) || !aligned(Y, 2 * ld_mult)) return PARO_ERR_ALIGN;
    return PARO_OK;
}

// The exchange part (split-K partial sums; zero-filled between calls, every kernel that uses it
// leaves it zero-filled) sits at the start of the caller's buffer, the scratch part (rotated
// activations when the rotation is a separate pass; left in any state) at its END: a buffer that
// holds the largest exchange part plus the largest scratch part of all calls that share it keeps
// every call's scratch out of every other call's exchange part.
struct WsLayout {
    size_t exchange_bytes;
    size_t xr_bytes;        // scratch, first piece: rotated activations of a separate rotation pass
    size_t gemm_bytes;      // scratch, second piece: split-K partial tiles of the GEMM at moderate token counts
    size_t scratch_bytes;
    size_t total;
};

WsLayout ws_layout(const paro_rotation *rot, const paro_w4_weight *w, int T, bool always_fuse = false)
{
    WsLayout L{0, 0, 0, 0, 0};
    const bool fused = fused_decode(rot, w, T, always_fuse);
    if (fast_weight(w)) {
        // partial sums of the kernel this call launches: the K-major one (one part per K-slice) or the bare one
        // (parts only beyond 6144 channels)
        const size_t part = fused && !fused_wide(rot, w, T) ? decode_geometry(w->c_in, w->c_out, T).partial_bytes
                                                            : decode_wide_partial_bytes(w->c_in, w->c_out, T);
        // the bare linear without partial sums to exchange needs no workspace at all
        L.exchange_bytes = (rot || part) ? kWsPartialOff + round_up(part, 256) : 0;
        if (T > kDecodeMaxTokens) L.gemm_bytes = round_up(gemm_scratch_bytes(*w, T), 256);
    }
    L.xr_bytes = (rot && !fused) ? round_up((size_t)T * w->c_in * 2, 256) : 0;
    L.scratch_bytes = L.xr_bytes + L.gemm_bytes;
    L.total = L.exchange_bytes + L.scratch_bytes;
    return L;
}

inline char *ws_scratch(void *ws, size_t ws_bytes, const WsLayout &L)
{
    return (char *)ws + (ws_bytes - L.scratch_bytes) / 256 * 256;
}

paro_status from_hip(hipError_t e) { return e == hipSuccess ? PARO_OK : PARO_ERR_HIP; }

// Exchange part for callers that cannot allocate (paro_rotated_linear_noalloc): one array per GPU,
// part of the loaded code object, zero-initialised when the library is loaded on that GPU and
// kept consistent by the calls themselves like any caller-owned exchange part.  In host code the
// array's name is only a handle; its device address is looked up once per device and kept.
constexpr size_t kStaticScratchBytes = PARO_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::atomic<void *> g_scratch_ptr[64];

paro_status static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return PARO_ERR_HIP;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PARO_ERR_HIP;
        g_scratch_ptr[dev].store(p, std::memory_order_release);      // same address from every thread: idempotent
    }
    *out = p;
    return PARO_OK;
}

// bare linear on (already transformed) activations, any T
paro_status run_linear(const paro_w4_weight *w, const paro_half_t *X, int64_t ldx, paro_half_t *Y, int64_t ldy, int T,
                       void *ws, void *gemm_scratch, size_t gemm_bytes, hipStream_t s)
{
    if (!fast_weight(w)) {
        if (!(w->qweight && w->scales && w->qzeros)) return PARO_ERR_UNSUPPORTED;
        return from_hip(launch_linear_generic(*w, X, ldx, Y, ldy, T, s));
    }
    if (T >= 512 && !gemm_supported(*w, ldx, ldy, T) && gemm_supported(*w, ldx, ldy, 256)) {
        // The GEMM addresses X and Y through 31-bit byte offsets: walk longer inputs in runs of
        // whole 256-token tiles that fit.
        const int64_t ld = ldx > ldy ? ldx : ldy;
        const int64_t chunk = (((int64_t)1 << 30) - 1) / ld / 256 * 256;
        for (int64_t t0 = 0; t0 < T; t0 += chunk) {
            const int tc = (int)(T - t0 < chunk ? T - t0 : chunk);
            paro_status st = run_linear(w, X + t0 * ldx, ldx, Y + t0 * ldy, ldy, tc, ws, gemm_scratch, gemm_bytes, s);
            if (st != PARO_OK) return st;
        }
        return PARO_OK;
    }
    if (T > kDecodeMaxTokens && gemm_supported(*w, ldx, ldy, T)) {
        // Moderate token counts leave most of the chip idle in the GEMM (few token tiles), while the
        // streaming kernel re-reads the weights once per 32 tokens: take the cheaper.  Measured per pass:
        // 17..32 tokens ~5 us plus the tile bytes at ~3.75 TB/s, up to 16 tokens ~3.5 us plus the bytes at
        // ~5.2 TB/s, and ~2.5 us (4 us at 17..32 tokens) more where the K-slices of a row are spread over several blocks.
        const double mb = (double)packed_tiles_bytes(w->c_in, w->c_out) / 1.0e6;
        const int rem = T % kStreamPassTokens;
        const double ex32 = decode_wide_partial_bytes(w->c_in, w->c_out, kStreamPassTokens) ? 4.0 : 0.0;
        const double ex16 = decode_wide_partial_bytes(w->c_in, w->c_out, 16) ? 2.5 : 0.0;
        const double pass32 = 5.0 + mb / 3.75 + ex32;
        const double stream_us = (double)(T / kStreamPassTokens) * pass32 +
                                 (rem == 0 ? 0.0 : rem <= 16 ? 3.5 + mb / 5.2 + ex16 : pass32);
        if (T >= 512 || gemm_estimate_us(*w, T) <= stream_us)
            return from_hip(launch_gemm(*w, X, ldx, Y, ldy, T, gemm_scratch, gemm_bytes, s));
    }
    for (int t0 = 0; t0 < T; t0 += kStreamPassTokens) {
        int tc = T - t0 < kStreamPassTokens ? T - t0 : kStreamPassTokens;
        hipError_t e = launch_decode_wide(*w, X + (size_t)t0 * ldx, ldx, Y + (size_t)t0 * ldy, ldy, tc, ws, s);
        if (e != hipSuccess) return PARO_ERR_HIP;
    }
    return PARO_OK;
}

}  // namespace

extern "C" {

int paro_version(void) { return 110; }

const char *paro_status_string(paro_status s)
{
    switch (s) {
    case PARO_OK: return "ok";
    case PARO_ERR_NULL: return "a required pointer is NULL";
    case PARO_ERR_SHAPE: return "inconsistent sizes";
    case PARO_ERR_ALIGN: return "misaligned pointer or row stride";
    case PARO_ERR_PAIRS: return "pairs of a layer are not independent (Def. 1) or an index is out of range";
    case PARO_ERR_UNSUPPORTED: return "unsupported configuration";
    case PARO_ERR_WORKSPACE: return "workspace missing or too small";
    case PARO_ERR_HIP: return "HIP runtime error at launch";
    }
    return "unknown status";
}

paro_status paro_validate_pairs_host(const int16_t *pairs_host, int32_t n_groups, int32_t n_layers,
                                     int32_t pairs_per_layer, int32_t group)
{
    if (!pairs_host) return PARO_ERR_NULL;
    if (n_groups < 0 || n_layers < 0 || pairs_per_layer < 0 || group <= 0 || group > 32767) return PARO_ERR_SHAPE;
    uint8_t used[32768 / 8];
    for (int64_t gl = 0; gl < (int64_t)n_groups * n_layers; ++gl) {
        for (int c = 0; c < (group + 7) / 8; ++c) used[c] = 0;
        const int16_t *p = pairs_host + gl * pairs_per_layer * 2;
        for (int k = 0; k < pairs_per_layer; ++k) {
            int i = p[2 * k], j = p[2 * k + 1];
            if (i < 0 || j < 0 || i >= group || j >= group) return PARO_ERR_PAIRS;
            if (i == j) continue;   // empty slot: names no channel
            if ((used[i >> 3] >> (i & 7)) & 1 || (used[j >> 3] >> (j & 7)) & 1) return PARO_ERR_PAIRS;
            used[i >> 3] |= (uint8_t)(1u << (i & 7));
            used[j >> 3] |= (uint8_t)(1u << (j & 7));
        }
    }
    return PARO_OK;
}

paro_status paro_select_pairs_host(const int32_t *order_host, int32_t group, int32_t n_rotations,
                                   int32_t pairs_per_rotation, int16_t *pairs_out_host, int32_t *counts_out_host)
{
    if (!order_host || !pairs_out_host) return PARO_ERR_NULL;
    if (group < 2 || group > 1024 || n_rotations < 0 || pairs_per_rotation < 0 || pairs_per_rotation > group / 2)
        return PARO_ERR_SHAPE;
    const int32_t n_pairs = group * (group - 1) / 2;
    // pair number -> (i, j): row i of the upper triangle starts at i*g - i(i+1)/2
    std::vector<int16_t> pi((size_t)n_pairs), pj((size_t)n_pairs);
    for (int32_t i = 0, k = 0; i < group; ++i)
        for (int32_t j = i + 1; j < group; ++j, ++k) { pi[(size_t)k] = (int16_t)i; pj[(size_t)k] = (int16_t)j; }
    std::vector<uint8_t> seen((size_t)n_pairs, 0);
    for (int32_t k = 0; k < n_pairs; ++k) {
        const int32_t e = order_host[k];
        if (e < 0 || e >= n_pairs || seen[(size_t)e]) return PARO_ERR_PAIRS;
        seen[(size_t)e] = 1;
    }
    std::vector<uint8_t> taken((size_t)n_pairs, 0);      // pair used by an earlier rotation
    std::vector<uint8_t> busy((size_t)group);            // channel used in the current rotation
    for (int32_t r = 0; r < n_rotations; ++r) {
        std::fill(busy.begin(), busy.end(), (uint8_t)0);
        int16_t *out = pairs_out_host + (size_t)r * pairs_per_rotation * 2;
        int32_t cnt = 0;
        for (int32_t k = 0; k < n_pairs && cnt < pairs_per_rotation; ++k) {
            const int32_t e = order_host[k];
            const int i = pi[(size_t)e], j = pj[(size_t)e];
            if (taken[(size_t)e] || busy[(size_t)i] || busy[(size_t)j]) continue;
            out[2 * cnt] = (int16_t)i; out[2 * cnt + 1] = (int16_t)j;
            ++cnt;
            busy[(size_t)i] = busy[(size_t)j] = 1;
            taken[(size_t)e] = 1;
        }
        if (counts_out_host) counts_out_host[r] = cnt;
        for (int32_t k = cnt; k < pairs_per_rotation; ++k) { out[2 * k] = 0; out[2 * k + 1] = 0; }
    }
    return PARO_OK;
}

size_t paro_workspace_error_offset(void) { return kWsErrorWord * sizeof(uint32_t); }
size_t paro_workspace_partials_offset(void) { return kWsPartialOff; }

size_t paro_rotation_plan_bytes(const paro_rotation *rot)
{
    if (check_rotation(rot) != PARO_OK) return 0;
    return round_up(plan_total_dwords(rot->c_in / kGroup, rot->n_layers) * 4, 256);
}

paro_status paro_rotation_plan_build(const paro_rotation *rot, void *plan_out, void *stream)
{
    paro_status st = check_rotation(rot);
    if (st != PARO_OK) return st;
    if (!plan_out) return PARO_ERR_NULL;
    if (!aligned(plan_out, 256)) return PARO_ERR_ALIGN;
    return from_hip(launch_plan_build(*rot, plan_out, (hipStream_t)stream));
}

size_t paro_w4_repack_bytes(const paro_w4_weight *w)
{
    if (check_weight(w, false) != PARO_OK) return 0;
    if ((w->c_in / kGroup) % kSliceGroups) return 0;   // the tiled layout needs whole 512-channel slices
    return round_up(packed_tiles_bytes(w->c_in, w->c_out) + packed_scales_bytes(w->c_in, w->c_out) +
                        packed_zeros_bytes(w->c_in, w->c_out),
                    256);
}

paro_status paro_w4_repack(const paro_w4_weight *w, void *packed_out, void *stream)
{
    paro_status st = check_weight(w, true);
    if (st != PARO_OK) return st;
    if (!packed_out) return PARO_ERR_NULL;
    if (!aligned(packed_out, 256)) return PARO_ERR_ALIGN;
    if ((w->c_in / kGroup) % kSliceGroups) return PARO_ERR_UNSUPPORTED;
    return from_hip(launch_repack(*w, packed_out, (hipStream_t)stream));
}

size_t paro_workspace_bytes(const paro_rotation *rot, const paro_w4_weight *w, int32_t T)
{
    if (check_weight(w, false) != PARO_OK || T <= 0) return 0;
    if (rot && (check_rotation(rot) != PARO_OK || rot->c_in != w->c_in)) return 0;
    return ws_layout(rot, w, T).total;
}

size_t paro_workspace_exchange_bytes(const paro_rotation *rot, const paro_w4_weight *w, int32_t T)
{
    if (check_weight(w, false) != PARO_OK || T <= 0) return 0;
    if (rot && (check_rotation(rot) != PARO_OK || rot->c_in != w->c_in)) return 0;
    return ws_layout(rot, w, T).exchange_bytes;
}

paro_status paro_rotate_scale(const paro_rotation *rot, const paro_half_t *X, int64_t ldx, paro_half_t *Xr,
                              int64_t ldxr, int32_t T, void *stream)
{
    paro_status st = check_rotation(rot);
    if (st != PARO_OK) return st;
    st = check_io(X, ldx, rot->c_in, Xr, ldxr, rot->c_in, T, 2);
    if (st != PARO_OK) return st;
    if (X == Xr && ldx != ldxr) return PARO_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    if (rot->plan) return from_hip(launch_rotate_planned(*rot, X, ldx, Xr, ldxr, T, s));
    return from_hip(launch_rotate_generic(*rot, X, ldx, Xr, ldxr, T, s));
}

paro_status paro_w4a16_linear(const paro_w4_weight *w, const paro_half_t *X, int64_t ldx, paro_half_t *Y, int64_t ldy,
                              int32_t T, void *ws, size_t ws_bytes, void *stream)
{
    paro_status st = check_weight(w, false);
    if (st != PARO_OK) return st;
    st = check_io(X, ldx, w->c_in, Y, ldy, w->c_out, T, 8);
    if (st != PARO_OK) return st;
    WsLayout L = ws_layout(nullptr, w, T);
    if (L.total && (!ws || ws_bytes < L.total)) return PARO_ERR_WORKSPACE;
    if (L.total && !aligned(ws, 256)) return PARO_ERR_ALIGN;
    return run_linear(w, X, ldx, Y, ldy, T, ws, L.gemm_bytes ? ws_scratch(ws, ws_bytes, L) + L.xr_bytes : nullptr,
                      L.gemm_bytes, (hipStream_t)stream);
}

static paro_status rotated_linear(const paro_rotation *rot, const paro_w4_weight *w, const paro_half_t *X, int64_t ldx,
                                  paro_half_t *Y, int64_t ldy, int32_t T, void *ws, size_t ws_bytes, void *stream,
                                  bool always_fuse)
{
    paro_status st = check_rotation(rot);
    if (st != PARO_OK) return st;
    st = check_weight(w, false);
    if (st != PARO_OK) return st;
    if (rot->c_in != w->c_in) return PARO_ERR_SHAPE;
    st = check_io(X, ldx, w->c_in, Y, ldy, w->c_out, T, 8);
    if (st != PARO_OK) return st;
    WsLayout L = ws_layout(rot, w, T, always_fuse);
    if (L.total && (!ws || ws_bytes < L.total)) return PARO_ERR_WORKSPACE;
    if (L.total && !aligned(ws, 256)) return PARO_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;

    if (fused_wide(rot, w, T)) return from_hip(launch_decode_wide(*w, X, ldx, Y, ldy, T, ws, s, rot));
    if (fused_decode(rot, w, T, always_fuse)) return from_hip(launch_decode(rot, *w, X, ldx, Y, ldy, T, ws, s));

    // two passes: transform into the workspace, then the bare linear
    paro_half_t *xr = (paro_half_t *)ws_scratch(ws, ws_bytes, L);
    hipError_t e = rot->plan ? launch_rotate_planned(*rot, X, ldx, xr, w->c_in, T, s)
                             : launch_rotate_generic(*rot, X, ldx, xr, w->c_in, T, s);
    if (e != hipSuccess) return PARO_ERR_HIP;
    return run_linear(w, xr, w->c_in, Y, ldy, T, ws, L.gemm_bytes ? ws_scratch(ws, ws_bytes, L) + L.xr_bytes : nullptr,
                      L.gemm_bytes, s);
}

paro_status paro_rotated_linear(const paro_rotation *rot, const paro_w4_weight *w, const paro_half_t *X, int64_t ldx,
                                paro_half_t *Y, int64_t ldy, int32_t T, void *ws, size_t ws_bytes, void *stream)
{
    return rotated_linear(rot, w, X, ldx, Y, ldy, T, ws, ws_bytes, stream, false);
}

// Always the kernel that hosts the rotation where it can (it needs no scratch part), also for the
// shapes on which paro_rotated_linear prefers the two-pass route.
paro_status paro_rotated_linear_noalloc(const paro_rotation *rot, const paro_w4_weight *w, const paro_half_t *X,
                                        int64_t ldx, paro_half_t *Y, int64_t ldy, int32_t T, void *stream)
{
    paro_status st = check_rotation(rot);
    if (st != PARO_OK) return st;
    st = check_weight(w, false);
    if (st != PARO_OK) return st;
    if (rot->c_in != w->c_in) return PARO_ERR_SHAPE;
    st = check_io(X, ldx, w->c_in, Y, ldy, w->c_out, T, 8);
    if (st != PARO_OK) return st;
    const WsLayout L = ws_layout(rot, w, T, true);
    if (L.scratch_bytes) return PARO_ERR_UNSUPPORTED;                 // needs a scratch part: only the allocating call serves it
    if (L.exchange_bytes > kStaticScratchBytes) return PARO_ERR_WORKSPACE;
    void *ws = nullptr;
    st = static_scratch(&ws);
    if (st != PARO_OK) return st;
    return rotated_linear(rot, w, X, ldx, Y, ldy, T, ws, kStaticScratchBytes, stream, true);
}

paro_status paro_w4_unpack_codes(const paro_w4_weight *w, uint8_t *codes, void *stream)
{
    paro_status st = check_weight(w, false);
    if (st != PARO_OK) return st;
    if (!codes) return PARO_ERR_NULL;
    if (!aligned(codes, 8)) return PARO_ERR_ALIGN;
    if (w->packed && (w->c_in / kGroup) % kSliceGroups) return PARO_ERR_UNSUPPORTED;
    return from_hip(launch_unpack_codes(*w, codes, (hipStream_t)stream));
}

paro_status paro_w4_unpack_zeros(const paro_w4_weight *w, uint8_t *zeros, void *stream)
{
    paro_status st = check_weight(w, false);
    if (st != PARO_OK) return st;
    if (!zeros) return PARO_ERR_NULL;
    if (w->packed && (w->c_in / kGroup) % kSliceGroups) return PARO_ERR_UNSUPPORTED;
    return from_hip(launch_unpack_zeros(*w, zeros, (hipStream_t)stream));
}

paro_status paro_w4_dequant(const paro_w4_weight *w, paro_half_t *W, void *stream)
{
    paro_status st = check_weight(w, false);
    if (st != PARO_OK) return st;
    if (!W) return PARO_ERR_NULL;
    if (!aligned(W, 16)) return PARO_ERR_ALIGN;
    if (w->packed && (w->c_in / kGroup) % kSliceGroups) return PARO_ERR_UNSUPPORTED;
    return from_hip(launch_dequant(*w, W, (hipStream_t)stream));
}

static bool multi_one_launch(int32_t n, const paro_rotation *const *rots, const paro_w4_weight *const *ws_, int32_t T)
{
    if (T > kFuseMaxTokens) return false;
    for (int p = 0; p < n; ++p)
        if (!fast_weight(ws_[p]) || !rots[p]->plan || rots[p]->n_layers != rots[0]->n_layers) return false;
    return true;
}

static paro_status check_multi(int32_t n, const paro_rotation *const *rots, const paro_w4_weight *const *ws_)
{
    if (!rots || !ws_) return PARO_ERR_NULL;
    if (n < 1 || n > 4) return PARO_ERR_SHAPE;
    for (int p = 0; p < n; ++p) {
        paro_status st = check_rotation(rots[p]);
        if (st != PARO_OK) return st;
        st = check_weight(ws_[p], false);
        if (st != PARO_OK) return st;
        if (rots[p]->c_in != ws_[p]->c_in || ws_[p]->c_in != ws_[0]->c_in) return PARO_ERR_SHAPE;
    }
    return PARO_OK;
}

static WsLayout ws_layout_multi(int32_t n_parts, const paro_rotation *const *rots, const paro_w4_weight *const *weights,
                                int32_t T)
{
    WsLayout M{0, 0, 0};
    for (int p = 0; p < n_parts; ++p) {
        WsLayout one = ws_layout(rots[p], weights[p], T);
        if (one.exchange_bytes > M.exchange_bytes) M.exchange_bytes = one.exchange_bytes;
        if (one.scratch_bytes > M.scratch_bytes) M.scratch_bytes = one.scratch_bytes;
    }
    if (multi_one_launch(n_parts, rots, weights, T)) {
        size_t m = kWsPartialOff + round_up(paro::decode_multi_bytes(n_parts, weights, T), 256);
        if (m > M.exchange_bytes) M.exchange_bytes = m;
        M.scratch_bytes = 0;
    }
    M.total = M.exchange_bytes + M.scratch_bytes;
    return M;
}

size_t paro_workspace_bytes_multi(int32_t n_parts, const paro_rotation *const *rots,
                                  const paro_w4_weight *const *weights, int32_t T)
{
    if (check_multi(n_parts, rots, weights) != PARO_OK || T <= 0) return 0;
    return ws_layout_multi(n_parts, rots, weights, T).total;
}

size_t paro_workspace_exchange_bytes_multi(int32_t n_parts, const paro_rotation *const *rots,
                                           const paro_w4_weight *const *weights, int32_t T)
{
    if (check_multi(n_parts, rots, weights) != PARO_OK || T <= 0) return 0;
    return ws_layout_multi(n_parts, rots, weights, T).exchange_bytes;
}

paro_status paro_rotated_linear_multi(int32_t n_parts, const paro_rotation *const *rots,
                                      const paro_w4_weight *const *weights, const paro_half_t *X, int64_t ldx,
                                      paro_half_t *const *Y, const int64_t *ldy, int32_t T, void *ws, size_t ws_bytes,
                                      void *stream)
{
    paro_status st = check_multi(n_parts, rots, weights);
    if (st != PARO_OK) return st;
    if (!Y || !ldy) return PARO_ERR_NULL;
    for (int p = 0; p < n_parts; ++p) {
        st = check_io(X, ldx, weights[p]->c_in, Y[p], ldy[p], weights[p]->c_out, T, 8);
        if (st != PARO_OK) return st;
    }
    const size_t need = paro_workspace_bytes_multi(n_parts, rots, weights, T);
    if (need && (!ws || ws_bytes < need)) return PARO_ERR_WORKSPACE;
    if (need && !aligned(ws, 256)) return PARO_ERR_ALIGN;
    if (multi_one_launch(n_parts, rots, weights, T))
        return from_hip(paro::launch_decode_multi(n_parts, rots, weights, X, ldx, Y, ldy, T, ws, (hipStream_t)stream));
    for (int p = 0; p < n_parts; ++p) {
        st = paro_rotated_linear(rots[p], weights[p], X, ldx, Y[p], ldy[p], T, ws, ws_bytes, stream);
        if (st != PARO_OK) return st;
    }
    return PARO_OK;
}

paro_status paro_w4_quantize(const paro_rotation *rot, const paro_half_t *W, int64_t ldw, int32_t c_in, int32_t c_out,
                             uint32_t *qweight, paro_half_t *scales, uint32_t *qzeros, void *stream)
{
    if (!W || !qweight || !scales || !qzeros) return PARO_ERR_NULL;
    if (c_in <= 0 || c_out <= 0 || c_in % paro::kGroup || c_out % 8 || ldw < c_in) return PARO_ERR_SHAPE;
    if (ldw % 2 || !aligned(W, 4) || !aligned(qweight, 4) || !aligned(scales, 2) || !aligned(qzeros, 4))
        return PARO_ERR_ALIGN;
    if (rot) {
        paro_status st = check_rotation(rot);
        if (st != PARO_OK) return st;
        if (rot->c_in != c_in) return PARO_ERR_SHAPE;
        if (!rot->plan) return PARO_ERR_UNSUPPORTED;
    }
    return from_hip(paro::launch_quantize(rot, W, ldw, c_out, c_in, qweight, scales, qzeros, (hipStream_t)stream));
}

paro_status paro_rotate_scale_quantize_int4(const paro_rotation *rot, const paro_half_t *X, int64_t ldx, int32_t T,
                                            uint32_t *codes, paro_half_t *scales, uint8_t *zeros, void *stream)
{
    paro_status st = check_rotation(rot);
    if (st != PARO_OK) return st;
    if (!X || !codes || !scales || !zeros) return PARO_ERR_NULL;
    if (T <= 0 || ldx < rot->c_in) return PARO_ERR_SHAPE;
    if (ldx >= kMaxRowStride) return PARO_ERR_UNSUPPORTED;
    if (ldx % 2 || !aligned(X, 4) || !aligned(codes, 4) || !aligned(scales, 2)) return PARO_ERR_ALIGN;
    if (!rot->plan) return PARO_ERR_UNSUPPORTED;
    return from_hip(paro::launch_quantize_act(*rot, X, ldx, T, codes, scales, zeros, (hipStream_t)stream));
}

paro_status paro_rotate_scale_quantize_mxfp4(const paro_rotation *rot, const paro_half_t *X, int64_t ldx, int32_t T,
                                             uint32_t *codes, uint8_t *scales, void *stream)
{
    paro_status st = check_rotation(rot);
    if (st != PARO_OK) return st;
    if (!X || !codes || !scales) return PARO_ERR_NULL;
    if (T <= 0 || ldx < rot->c_in) return PARO_ERR_SHAPE;
    if (ldx >= kMaxRowStride) return PARO_ERR_UNSUPPORTED;
    if (ldx % 2 || !aligned(X, 4) || !aligned(codes, 4)) return PARO_ERR_ALIGN;
    if (!rot->plan) return PARO_ERR_UNSUPPORTED;
    return from_hip(paro::launch_quantize_act_mxfp4(*rot, X, ldx, T, codes, scales, (hipStream_t)stream));
}

static paro_status check_mxfp4_weight(const paro_mxfp4_weight *w, bool for_linear)
{
    if (!w) return PARO_ERR_NULL;
    if (w->c_in <= 0 || w->c_out <= 0 || w->c_in % paro::kGroup) return PARO_ERR_SHAPE;
    if (for_linear && (w->c_in % 512 || w->c_out % 16)) return PARO_ERR_SHAPE;
    if (!w->packed && (!w->codes || !w->scales)) return PARO_ERR_NULL;
    if ((w->codes && !aligned(w->codes, 16)) || (w->packed && !aligned(w->packed, 256)) || (w->bias && !aligned(w->bias, 2)))
        return PARO_ERR_ALIGN;
    return PARO_OK;
}

paro_status paro_mxfp4_quantize_weight(const paro_rotation *rot, const paro_half_t *W, int64_t ldw, int32_t c_in,
                                       int32_t c_out, uint32_t *codes, uint8_t *scales, void *stream)
{
    if (!W || !codes || !scales) return PARO_ERR_NULL;
    if (c_in <= 0 || c_out <= 0 || c_in % paro::kGroup || ldw < c_in) return PARO_ERR_SHAPE;
    if (ldw % 2 || !aligned(W, 4) || !aligned(codes, 4)) return PARO_ERR_ALIGN;
    if (rot) {
        paro_status st = check_rotation(rot);
        if (st != PARO_OK) return st;
        if (rot->c_in != c_in) return PARO_ERR_SHAPE;
        if (!rot->plan) return PARO_ERR_UNSUPPORTED;
    }
    return from_hip(paro::launch_quantize_weight_mxfp4(rot, W, ldw, c_out, c_in, codes, scales, (hipStream_t)stream));
}

size_t paro_mxfp4_packed_bytes(const paro_mxfp4_weight *w)
{
    if (!w || w->c_in <= 0 || w->c_out <= 0 || w->c_in % 512 || w->c_out % 16) return 0;
    return (size_t)w->c_out * w->c_in / 2 + (size_t)w->c_out * w->c_in / 32;
}

paro_status paro_mxfp4_repack(const paro_mxfp4_weight *w, void *packed_out, void *stream)
{
    paro_status st = check_mxfp4_weight(w, true);
    if (st != PARO_OK) return st;
    if (!w->codes || !w->scales || !packed_out) return PARO_ERR_NULL;
    if (!aligned(packed_out, 256)) return PARO_ERR_ALIGN;
    return from_hip(paro::launch_mxfp4_repack(*w, packed_out, (hipStream_t)stream));
}

paro_status paro_mxfp4_unpack(const paro_mxfp4_weight *w, uint8_t *codes, uint8_t *scales, void *stream)
{
    paro_status st = check_mxfp4_weight(w, w && w->packed);
    if (st != PARO_OK) return st;
    if (!codes || !scales) return PARO_ERR_NULL;
    return from_hip(paro::launch_mxfp4_unpack(*w, codes, scales, (hipStream_t)stream));
}

paro_status paro_mxfp4_linear(const paro_mxfp4_weight *w, const uint32_t *x_codes, const uint8_t *x_scales, int32_t T,
                              paro_half_t *Y, int64_t ldy, void *stream)
{
    paro_status st = check_mxfp4_weight(w, true);
    if (st != PARO_OK) return st;
    if (!x_codes || !x_scales || !Y) return PARO_ERR_NULL;
    if (T <= 0 || ldy < w->c_out) return PARO_ERR_SHAPE;
    if (ldy >= kMaxRowStride) return PARO_ERR_UNSUPPORTED;
    if (!aligned(x_codes, 16) || !aligned(x_scales, 16) || !aligned(Y, 2)) return PARO_ERR_ALIGN;
    if (!paro::mxfp4_linear_supported(*w)) return PARO_ERR_UNSUPPORTED;
    return from_hip(paro::launch_mxfp4_linear(*w, x_codes, x_scales, T, Y, ldy, (hipStream_t)stream));
}

size_t paro_workspace_bytes_mxfp4(int32_t c_in, int32_t T)
{
    if (c_in <= 0 || T <= 0 || c_in % 512) return 0;
    return round_up((size_t)T * c_in / 2, 256) + round_up((size_t)T * c_in / 32, 256);
}

paro_status paro_rotated_linear_mxfp4(const paro_rotation *rot, const paro_mxfp4_weight *w, const paro_half_t *X,
                                      int64_t ldx, paro_half_t *Y, int64_t ldy, int32_t T, void *ws, size_t ws_bytes,
                                      void *stream)
{
    paro_status st = check_rotation(rot);
    if (st != PARO_OK) return st;
    st = check_mxfp4_weight(w, true);
    if (st != PARO_OK) return st;
    if (rot->c_in != w->c_in) return PARO_ERR_SHAPE;
    if (!X || !Y) return PARO_ERR_NULL;
    if (T <= 0 || ldx < w->c_in || ldy < w->c_out) return PARO_ERR_SHAPE;
    if (ldx >= kMaxRowStride || ldy >= kMaxRowStride) return PARO_ERR_UNSUPPORTED;
    if (ldx % 2 || !aligned(X, 4) || !aligned(Y, 2)) return PARO_ERR_ALIGN;
    if (!rot->plan || !paro::mxfp4_linear_supported(*w)) return PARO_ERR_UNSUPPORTED;
    const size_t need = paro_workspace_bytes_mxfp4(w->c_in, T);
    if (!ws || ws_bytes < need) return PARO_ERR_WORKSPACE;
    if (!aligned(ws, 256)) return PARO_ERR_ALIGN;
    uint32_t *xc = (uint32_t *)ws;
    uint8_t *xs = (uint8_t *)ws + round_up((size_t)T * w->c_in / 2, 256);
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = paro::launch_quantize_act_mxfp4(*rot, X, ldx, T, xc, xs, s);
    if (e != hipSuccess) return PARO_ERR_HIP;
    return from_hip(paro::launch_mxfp4_linear(*w, xc, xs, T, Y, ldy, s));
}

}  // extern "C"
