/*
 * paro.h - C ABI of libparo: the runtime hot path of Pairwise Rotation
 * Quantization (arXiv 2511.10645) on AMD MI355X (gfx950).
 *
 * What the calls compute (column-vector form of Eq. 2 with the transform of Eq. 8):
 *
 *      y = W^ . ( R_K ... R_1 . S . x ) + b
 *
 *   S      = diag(ch_scale): per-channel scaling seen by the activations
 *            (Section 4.1.4; the reciprocal of the alpha that multiplies the weights)
 *   R_t    = one "independent rotation" (Def. 2): disjoint channel pairs inside each
 *            group of `group` channels, pair (i, j, theta) updates
 *                 u_i <- cos(theta) u_i - sin(theta) u_j
 *                 u_j <- sin(theta) u_i + cos(theta) u_j            (Eq. 4, Eq. 5)
 *            layers are applied in array order, layer 0 first
 *   W^     = INT4 group-quantised weight, W^[n,c] = (q[n,c] - z[c/group,n]) * s[c/group,n]
 *            (Eq. 1 read backwards; one s and z per `group` consecutive input channels
 *            of an output column, Section 2.1)
 *
 * Conventions
 *   - Every pointer inside the structs and every X / Y / workspace / blob argument is a
 *     DEVICE pointer unless its name ends in _host.  The caller owns all memory; the
 *     library never allocates, frees or keeps device memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work; they never synchronise.
 *   - fp16 data is IEEE binary16, declared here as uint16_t bit patterns (paro_half_t).
 *   - Argument errors are detected on the host before anything is launched, so a call
 *     that returns an error has had no effect on the device.
 *   - group must be 128, n_layers <= 8, pairs_per_layer <= 64 (Section 5, "Implementation").
 */
#ifndef PARO_H
#define PARO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t paro_half_t;

typedef enum {
    PARO_OK = 0,
    PARO_ERR_NULL = 1,        /* a required pointer is NULL                                  */
    PARO_ERR_SHAPE = 2,       /* sizes inconsistent (c_in % group, ld < width, T <= 0, ...)   */
    PARO_ERR_ALIGN = 3,       /* a pointer or row stride is not aligned as documented         */
    PARO_ERR_PAIRS = 4,       /* pairs of one layer are not disjoint / index out of range     */
    PARO_ERR_UNSUPPORTED = 5, /* group != 128, n_layers > 8, pairs_per_layer > 64, ...        */
    PARO_ERR_WORKSPACE = 6,   /* workspace missing or smaller than paro_workspace_bytes()     */
    PARO_ERR_HIP = 7          /* the HIP runtime reported an error at launch                  */
} paro_status;

/* The online transform of one linear layer's input (Section 4.1; Eq. 5, Eq. 8). */
typedef struct {
    int32_t c_in;             /* channels of X, multiple of group                             */
    int32_t group;            /* channel-group size g (= quantisation group), 128             */
    int32_t n_layers;         /* K, 0..8                                                       */
    int32_t pairs_per_layer;  /* slots per layer and group, 1..64                              */
    const int16_t *pairs;     /* [c_in/group][n_layers][pairs_per_layer][2]; 0-based indices
                                 LOCAL to the group; i == j marks an empty slot; within one
                                 layer and group no channel may appear twice (Def. 1): a table
                                 that breaks this, or holds an index outside the group, makes
                                 every output of that group NaN, with or without a plan        */
    const float *theta;       /* [c_in/group][n_layers][pairs_per_layer], radians              */
    const paro_half_t *ch_scale; /* [c_in] multiplier applied to x; NULL = all ones            */
    int32_t scale_order;      /* 0: scale, then rotate (Eq. 8 inverted; default)
                                 1: rotate, then scale                                         */
    const void *plan;         /* blob written by paro_rotation_plan_build(); NULL selects the
                                 slower kernel that reads pairs/theta directly                 */
} paro_rotation;

/* An INT4 group-quantised weight (Eq. 1, Section 2.1), interchange layout. */
typedef struct {
    int32_t c_in;             /* multiple of group                                             */
    int32_t c_out;            /* multiple of 16                                                */
    int32_t group;            /* 128                                                           */
    const uint32_t *qweight;  /* [c_out][c_in/8]; bits 4k..4k+3 of word w of row n hold the
                                 code q[n, 8w+k]                                               */
    const paro_half_t *scales;/* [c_in/group][c_out]                                           */
    const uint32_t *qzeros;   /* [c_in/group][c_out/8]; bits 4k..4k+3 of word w hold z[g, 8w+k]*/
    const paro_half_t *bias;  /* optional [c_out], added in fp32 before the fp16 store         */
    const void *packed;       /* blob written by paro_w4_repack(); NULL selects the slower
                                 kernels that read the interchange layout                      */
} paro_w4_weight;

/* major * 100 + minor; 110: two-part workspace (exchange part + scratch at the end of the buffer). */
int paro_version(void);
const char *paro_status_string(paro_status s);

/* Def. 1 on a HOST copy of the pair table: every index in [0, group) and no channel twice
 * within a (group, layer).  Device kernels assume a table that passed this check.
 * Returns PARO_OK, PARO_ERR_PAIRS, PARO_ERR_NULL, PARO_ERR_SHAPE. */
paro_status paro_validate_pairs_host(const int16_t *pairs_host, int32_t n_groups, int32_t n_layers,
                                     int32_t pairs_per_layer, int32_t group);

/* Selection of independent channel pairs for a series of K rotations of one channel group
 * (Algorithm A1, Section 4.1.2), on the HOST.  The algorithm's one random draw, the shuffle of
 * all g(g-1)/2 pairs, is an input: `order_host` is a permutation of 0..g(g-1)/2-1 over the
 * pairs (i, j), 0 <= i < j < g, numbered in lexicographic order ((0,1) = 0, (0,2) = 1, ...).
 * For each rotation in turn the shuffled list is scanned from its start and a pair is taken when
 * neither of its channels is used yet in this rotation and the pair was not taken by an earlier
 * rotation, until `pairs_per_rotation` pairs are found or the list ends.
 * pairs_out_host: [n_rotations][pairs_per_rotation][2] int16, selection order, i < j; slots that
 * stay empty hold (0, 0), the no-op spelling of paro_rotation.  counts_out_host (nullable):
 * [n_rotations] pairs found.  2 <= group <= 1024, pairs_per_rotation <= group/2.
 * Returns PARO_OK, PARO_ERR_NULL, PARO_ERR_SHAPE, PARO_ERR_PAIRS (order is not a permutation). */
paro_status paro_select_pairs_host(const int32_t *order_host, int32_t group, int32_t n_rotations,
                                   int32_t pairs_per_rotation, int16_t *pairs_out_host,
                                   int32_t *counts_out_host);

/* One-time preparation (model-load side) ------------------------------------------------ */

/* Size in bytes of the rotation plan for `rot` (0 on invalid arguments). */
size_t paro_rotation_plan_bytes(const paro_rotation *rot);
/* Builds the plan on the device: per group and layer, the lane routing, fp32 cos/sin
 * (rounded from an fp64 evaluation) and the folded channel scales used by the fast
 * rotation kernels, followed by a compact copy (one angle in 2^-24 revolutions per lane
 * and layer, fp16 scales) for the one-token linear whose waves each transform their own
 * slice of the input channels (Eq. 4, 5 with the sine and cosine taken at run time).
 * plan_out: device buffer of paro_rotation_plan_bytes(), 256-byte aligned.  rot->plan is
 * ignored. */
paro_status paro_rotation_plan_build(const paro_rotation *rot, void *plan_out, void *stream);

/* Size in bytes of the kernel-private weight blob for `w` (0 on invalid arguments). */
size_t paro_w4_repack_bytes(const paro_w4_weight *w);
/* Rewrites qweight / scales / qzeros into the tiled layout the fast kernels stream
 * (a pure permutation of the same bits: paro_w4_unpack_codes() on the repacked weight
 * returns the same codes).  packed_out: device buffer, 256-byte aligned. */
paro_status paro_w4_repack(const paro_w4_weight *w, void *packed_out, void *stream);

/* Hot path ------------------------------------------------------------------------------- */

/* Row strides of activations and outputs (ldx, ldy, ldxr: in elements) must be below 2^22
 * (PARO_ERR_UNSUPPORTED otherwise): the kernels address runs of rows with 32-bit byte offsets.
 * T itself is not limited by that. */

/* Workspace of the linear calls (rot may be NULL for the bare linear), in two parts:
 *   - the exchange part, the first paro_workspace_exchange_bytes() bytes of the buffer: what blocks
 *     of one launch hand to each other.  It must be zero-filled ONCE after allocation and is then
 *     kept consistent by the calls themselves.  Its layout is the same for every call, so calls
 *     of any shapes may share it:
 *        bytes [0, 256)   header.  Bytes 8..11 (paro_workspace_error_offset()) hold an error
 *                         word: it stays 0 unless a bounded wait between blocks of a launch ran
 *                         out (the outputs that depended on it are then NaN);
 *        from paro_workspace_partials_offset() on: fp32 partial sums of split-K launches; every
 *                         word is reset by its reader, so this range is all zero again after
 *                         every call.
 *     The blocks that exchange data must be resident at the same time: do not run other long
 *     kernels concurrently with these calls.  After a non-zero error word (or after a call that
 *     was cancelled or faulted) zero-fill the exchange part again before the next call.
 *   - the scratch part, the LAST paro_workspace_bytes() - paro_workspace_exchange_bytes() bytes
 *     of the buffer as given by ws_bytes (rounded down to 256): transformed activations when the
 *     rotation runs as a pass of its own (T > 4, no plan / no repacked weight, or a shape on
 *     which two launches are faster than the exchange of the fused kernel), and fp32
 *     partial tiles where the GEMM splits K (some tens to hundreds of tokens).  No requirement
 *     before a call, any contents after it.
 * paro_workspace_bytes() is the sum: enough for a buffer that only serves calls of that one shape.
 * A buffer shared by calls of several shapes must hold the largest exchange part plus the largest
 * scratch part of all of them, so that no call's scratch reaches into another's exchange part;
 * pass its full size as ws_bytes.  Calls that share a workspace must not overlap in time.
 * The bare linear needs no workspace (0 bytes, ws may be NULL) where it neither splits K between
 * blocks nor runs the GEMM's split. */
size_t paro_workspace_error_offset(void);
size_t paro_workspace_partials_offset(void);
size_t paro_workspace_bytes(const paro_rotation *rot, const paro_w4_weight *w, int32_t T);
size_t paro_workspace_exchange_bytes(const paro_rotation *rot, const paro_w4_weight *w, int32_t T);

/* Xr[t, :] = R_K ... R_1 . S . X[t, :] for t < T, fp32 arithmetic, one fp16 rounding at the
 * store (Eq. 5, Eq. 8).  X, Xr: fp16 [T][ld*], ld >= c_in, rows 4-byte aligned (ld even).
 * Xr == X (in place, same ld) is allowed; other overlaps are not. */
paro_status paro_rotate_scale(const paro_rotation *rot, const paro_half_t *X, int64_t ldx,
                              paro_half_t *Xr, int64_t ldxr, int32_t T, void *stream);

/* Y[t, n] = sum_c W^[n, c] X[t, c] (+ bias[n]), fp32 accumulation, fp16 store (Eq. 2 with
 * T = identity).  X: fp16 [T][ldx], Y: fp16 [T][ldy]; ldx >= c_in, ldy >= c_out, both
 * multiples of 8 (16-byte rows).  ws/ws_bytes: see paro_workspace_bytes(). */
paro_status paro_w4a16_linear(const paro_w4_weight *w, const paro_half_t *X, int64_t ldx,
                              paro_half_t *Y, int64_t ldy, int32_t T,
                              void *ws, size_t ws_bytes, void *stream);

/* Y = W^ . (R_K ... R_1 . S . X) (+ bias): the transform fused in front of the linear
 * (Eq. 2).  rot->c_in must equal w->c_in.  Same layouts as the two calls above. */
paro_status paro_rotated_linear(const paro_rotation *rot, const paro_w4_weight *w,
                                const paro_half_t *X, int64_t ldx, paro_half_t *Y, int64_t ldy,
                                int32_t T, void *ws, size_t ws_bytes, void *stream);

/* For callers that cannot allocate device memory or pass a workspace (code under HIP graph capture
 * that may not call hipMalloc, tight serving loops, harnesses that forbid allocation):
 * paro_rotated_linear with the exchange part of the workspace held in a static device array of
 * PARO_NOALLOC_SCRATCH_BYTES inside the library (one copy per GPU the library runs on, held until
 * the process ends; zero when the library is loaded, and left consistent by every call like a
 * caller-owned exchange part).  The call allocates and frees nothing.  It always takes the fused
 * decode kernel (rotation planned, weight repacked, T <= 4), which needs no scratch part - also
 * on the shapes where paro_rotated_linear prefers two launches; there the two calls agree to
 * rounding, elsewhere bit for bit - and returns PARO_ERR_UNSUPPORTED for the others, PARO_ERR_WORKSPACE when the exchange part of
 * the shape exceeds PARO_NOALLOC_SCRATCH_BYTES (4 MiB covers K-slices x T x c_out x 4 bytes of
 * every benchmark shape at one token and of the 8B-class shapes at 4).  All calls on one GPU share
 * that GPU's array: calls that overlap in time on one GPU race, exactly as two calls sharing a
 * caller-owned workspace would.  The first call on a device looks the array's address up
 * (no allocation); make it outside stream capture.  After a wait between blocks timed out
 * (outputs NaN) the array is no longer consistent for the rest of the process. */
#define PARO_NOALLOC_SCRATCH_BYTES (4u << 20)
paro_status paro_rotated_linear_noalloc(const paro_rotation *rot, const paro_w4_weight *w,
                                        const paro_half_t *X, int64_t ldx, paro_half_t *Y, int64_t ldy,
                                        int32_t T, void *stream);

/* Several linears that read the SAME activations, each with its own transform: in the method every
 * linear owns its pairs, angles and scales (Section 4.1, App. A.4), so the q / k / v projections
 * (or gate / up) of a decoder layer need three (two) transforms of one X.  Part p computes
 * Y[p] = W^_p . (R_p . S_p . x) (+ b_p) exactly as paro_rotated_linear(rots[p], weights[p], X, Y[p]).
 * n_parts in 1..4; all parts share c_in.  With T <= 4, every rotation planned, every weight
 * repacked and equal layer counts the parts run as ONE launch (results are bit-identical to the
 * separate calls); otherwise the call is the sequence of separate calls.  rots, weights, Y and
 * ldy are HOST arrays of n_parts entries (device pointers inside, as in the single call).
 * ws: device, >= paro_workspace_bytes_multi(...) bytes, 256-byte aligned, in the two parts
 * described at paro_workspace_bytes() (exchange part: paro_workspace_exchange_bytes_multi()). */
size_t paro_workspace_exchange_bytes_multi(int32_t n_parts, const paro_rotation *const *rots,
                                           const paro_w4_weight *const *weights, int32_t T);
size_t paro_workspace_bytes_multi(int32_t n_parts, const paro_rotation *const *rots,
                                  const paro_w4_weight *const *weights, int32_t T);
paro_status paro_rotated_linear_multi(int32_t n_parts, const paro_rotation *const *rots,
                                      const paro_w4_weight *const *weights, const paro_half_t *X, int64_t ldx,
                                      paro_half_t *const *Y, const int64_t *ldy, int32_t T, void *ws,
                                      size_t ws_bytes, void *stream);

/* Offline, weight side (Eq. 8 then Eq. 1; Section 2.1 group rule) ----------------------------
 * Quantise a dense fp16 weight W[c_out][c_in] (row n = output channel n at W + n*ldw, device)
 * into the interchange layout of paro_w4_weight:
 *      w'_n = R_K ... R_1 . diag(1/ch_scale) . w_n      (the weight-side counterpart of what
 *                                                         paro_rotate_scale does to activations;
 *                                                         scale_order 1: diag(1/ch_scale) last)
 *      per 128 input channels of a row:  s = (max - min)/15,  z = -round(min/s),
 *                                        q = clamp(round(w'/s) + z, 0, 15)          (Eq. 1, b = 4)
 * rot == NULL quantises W as it is.  A rotation needs its plan (PARO_ERR_UNSUPPORTED otherwise).
 * Arithmetic: rotation in fp32; s, z, q decided in fp32 with the fp16-rounded scale that is
 * stored, round-half-to-even; s >= 2^-14; z clamped to 0..15.
 * Outputs (device, written completely): qweight [c_out][c_in/8], scales [c_in/128][c_out],
 * qzeros [c_in/128][c_out/8].  c_in % 128 == 0, c_out % 8 == 0, ldw >= c_in and even, W 4-byte
 * aligned.  Enqueues on `stream`; no workspace. */
paro_status paro_w4_quantize(const paro_rotation *rot, const paro_half_t *W, int64_t ldw,
                             int32_t c_in, int32_t c_out, uint32_t *qweight, paro_half_t *scales,
                             uint32_t *qzeros, void *stream);

/* Activation side of the W4A4 extension (App. A.3: Y' = Q(X T^-1) . Q(T W) + b): the transform of
 * paro_rotate_scale followed at once by a 4-bit quantiser of the transformed activations.  The
 * paper names no activation quantiser, so Eq. 1 (b = 4) is applied per token and 128-channel
 * group with the decisions of paro_w4_quantize (fp32, stored fp16 scale, round-half-to-even,
 * scale floor 2^-14, zero point clamped to 0..15).  The rotation needs its plan.
 * codes [T][c_in/8] (bits 4k..4k+3 of word w hold channel 8w+k), scales [T][c_in/128] fp16,
 * zeros [T][c_in/128] bytes; all device, written completely.  X as in paro_rotate_scale.
 * No INT4 x INT4 contraction is part of this library: the call ends at the quantised activations
 * (the MXFP4 form below goes on to the contraction). */
paro_status paro_rotate_scale_quantize_int4(const paro_rotation *rot, const paro_half_t *X, int64_t ldx,
                                            int32_t T, uint32_t *codes, paro_half_t *scales,
                                            uint8_t *zeros, void *stream);

/* The same activation side (App. A.3) with a microscaling FP4 quantiser, the 4-bit type the
 * matrix cores of gfx950 take directly (MXFP4 of the OCP Microscaling Formats specification):
 * every 32 consecutive channels of a token share the scale 2^e, e = floor(log2(max|v|)) - 2,
 * e >= -127, stored as the byte e + 127 (an all-zero block stores 0); each value is the E2M1 code
 * of v / 2^e, round to nearest, ties to the even code, saturating at 6 (magnitudes by code 0..7:
 * 0, 0.5, 1, 1.5, 2, 3, 4, 6; bit 3 = sign).  Inputs must be finite.  The rotation needs its plan.
 * codes [T][c_in/8] (bits 4k..4k+3 of word w hold channel 8w+k), scales [T][c_in/32] bytes; all
 * device (codes and scales 16-byte aligned if they feed paro_mxfp4_linear), written completely.
 * X as in paro_rotate_scale. */
paro_status paro_rotate_scale_quantize_mxfp4(const paro_rotation *rot, const paro_half_t *X, int64_t ldx,
                                             int32_t T, uint32_t *codes, uint8_t *scales, void *stream);

/* ---- The weight-activation linear with both operands in MXFP4 (App. A.3, first equation) --------
 *      Y' = Q(X T^-1) . Q(T W) + b
 * contracted on the block-scaled FP4 matrix instruction of gfx950: E2M1 codes and E8M0 block scales
 * go to the matrix cores as they are, products are exact, accumulation is fp32, one fp16 rounding at
 * the store.  Element and scale formats as documented at paro_rotate_scale_quantize_mxfp4. */
typedef struct paro_mxfp4_weight {
    int32_t c_in;             /* multiple of 512 for paro_mxfp4_repack / paro_mxfp4_linear, of 128 otherwise */
    int32_t c_out;            /* multiple of 16 for paro_mxfp4_repack / paro_mxfp4_linear                   */
    const uint32_t *codes;    /* device [c_out][c_in/8]: bits 4k..4k+3 of word w of a row = channel 8w+k;
                                 may be NULL once `packed` is set                                           */
    const uint8_t *scales;    /* device [c_out][c_in/32] E8M0 bytes; may be NULL once `packed` is set       */
    const paro_half_t *bias;  /* device [c_out] fp16, or NULL                                               */
    const void *packed;       /* device blob written by paro_mxfp4_repack (operand order of the matrix
                                 instruction), or NULL; 256-byte aligned; owned by the caller               */
} paro_mxfp4_weight;

/* Q(T W): every output row of the dense fp16 W[c_out][c_in] (row n at W + n*ldw, device) takes the
 * weight side of the transform, w'_n = R_K ... R_1 . diag(1/ch_scale) . w_n in fp32 exactly as in
 * paro_w4_quantize (rot == NULL: none; a rotation needs its plan), and is converted to MXFP4 per
 * 32 channels.  codes [c_out][c_in/8], scales [c_out][c_in/32]: device, written completely.
 * c_in % 128 == 0, ldw >= c_in and even, W 4-byte aligned, codes 4-byte aligned. */
paro_status paro_mxfp4_quantize_weight(const paro_rotation *rot, const paro_half_t *W, int64_t ldw,
                                       int32_t c_in, int32_t c_out, uint32_t *codes, uint8_t *scales,
                                       void *stream);

/* Repack codes + scales into the operand order of the matrix instruction (tiles of 16 rows x 128
 * channels, then one dword of four K-steps' scale bytes per lane).  packed_out: device,
 * paro_mxfp4_packed_bytes() bytes (= c_out*c_in/2 + c_out*c_in/32), 256-byte aligned. */
size_t paro_mxfp4_packed_bytes(const paro_mxfp4_weight *w);
paro_status paro_mxfp4_repack(const paro_mxfp4_weight *w, void *packed_out, void *stream);
/* Test hook: codes[n][c] as bytes 0..15 and scales[n][c/32], from w->packed if set, else from the
 * plain arrays (codes: c_out*c_in bytes, scales: c_out*c_in/32 bytes, device). */
paro_status paro_mxfp4_unpack(const paro_mxfp4_weight *w, uint8_t *codes, uint8_t *scales, void *stream);

/* Y[t][n] = sum_c x^[t][c] w^[n][c] (+ bias[n]) for t < T, x^ / w^ the values the MXFP4 codes stand
 * for.  x_codes [T][c_in/8], x_scales [T][c_in/32]: device, 16-byte aligned, in the layout
 * paro_rotate_scale_quantize_mxfp4 writes.  Y: fp16 [T][ldy], ldy >= c_out, 2-byte aligned rows.
 * Needs w->packed (PARO_ERR_UNSUPPORTED otherwise; also for c_in > 30720 or a blob of 2 GiB or
 * more).  No workspace. */
paro_status paro_mxfp4_linear(const paro_mxfp4_weight *w, const uint32_t *x_codes, const uint8_t *x_scales,
                              int32_t T, paro_half_t *Y, int64_t ldy, void *stream);

/* The whole of App. A.3's equation for fp16 activations: paro_rotate_scale_quantize_mxfp4 into the
 * workspace, then paro_mxfp4_linear.  ws: device, >= paro_workspace_bytes_mxfp4(c_in, T) bytes
 * (= T*c_in/2 for the codes, rounded up to 256, + T*c_in/32 for the scales), 256-byte aligned, no
 * requirement on its contents before the call, any contents after it. */
size_t paro_workspace_bytes_mxfp4(int32_t c_in, int32_t T);
paro_status paro_rotated_linear_mxfp4(const paro_rotation *rot, const paro_mxfp4_weight *w,
                                      const paro_half_t *X, int64_t ldx, paro_half_t *Y, int64_t ldy,
                                      int32_t T, void *ws, size_t ws_bytes, void *stream);

/* Test hooks for the bit-exact gate --------------------------------------------------- */

/* codes[n][c] = q[n, c] as bytes 0..15 (from w->packed if set, else from w->qweight). */
paro_status paro_w4_unpack_codes(const paro_w4_weight *w, uint8_t *codes, void *stream);
/* zeros[g][n] = z[g, n] as bytes 0..15. */
paro_status paro_w4_unpack_zeros(const paro_w4_weight *w, uint8_t *zeros, void *stream);
/* W[n][c] = fp16( (q - z) * s ), exact product rounded once to nearest-even. */
paro_status paro_w4_dequant(const paro_w4_weight *w, paro_half_t *W, void *stream);

/* Yardstick of Section 4.3's figure ("speedup of scaled pairwise rotation over the Hadamard
 * transform"): the fast Walsh-Hadamard transform of activation rows, the online transform of the
 * Hadamard-based methods the paper compares its kernel with.  Not part of the method's path.
 *      Y[t, :] = H_n X[t, :] / sqrt(n),  H_n[i][j] = (-1)^popcount(i & j)  (Sylvester order)
 * fp32 butterflies, one fp16 rounding at the store.  n a power of two, 8 <= n <= 32768
 * (PARO_ERR_UNSUPPORTED above); X, Y: fp16 [T][ld*], ld >= n and a multiple of 8, 16-byte
 * aligned; Y == X (same ld) is allowed.  No workspace. */
paro_status paro_fwht(const paro_half_t *X, int64_t ldx, paro_half_t *Y, int64_t ldy, int32_t T,
                      int32_t n, void *stream);

/* Diagnostics: measured ceilings of the machine (benchmark only; not part of the method) ------
 * A roofline fraction against the nominal peaks (8 TB/s, 2.5 PFLOP/s) says little unless one
 * knows what a kernel that does nothing else reaches on the same chip at the same size. */

/* Pure read: every lane reads 16 bytes per step (non-temporal, four loads in flight), nothing is
 * written.  src: device, 16-byte aligned, `bytes` readable; sink: device uint32 or NULL (written
 * only if the xor of all words equals one magic value); blocks of 256 threads. */
paro_status paro_diag_read_stream(const void *src, size_t bytes, void *sink, int32_t blocks, void *stream);

/* Pure fp16 MFMA issue: every wave runs iters x 16 independent 32x32x16 MFMAs on register
 * operands (constant, or pseudo-random per lane when random_operands != 0).  out: device floats,
 * blocks * 256 of them.  paro_diag_mfma_f16_flops() = floating-point operations of such a launch. */
paro_status paro_diag_mfma_f16(void *out, size_t out_bytes, int32_t blocks, int32_t iters,
                               int32_t random_operands, void *stream);
double paro_diag_mfma_f16_flops(int32_t blocks, int32_t iters);

/* The same for the block-scaled FP4 instruction of paro_mxfp4_linear: every wave (8 per block of 512
 * threads) runs iters x 32 independent 16x16x128 FP4 MFMAs.  out: device floats, blocks * 512. */
paro_status paro_diag_mfma_fp4(void *out, size_t out_bytes, int32_t blocks, int32_t iters,
                               int32_t random_operands, void *stream);
double paro_diag_mfma_fp4_flops(int32_t blocks, int32_t iters);

#ifdef __cplusplus
}
#endif
#endif /* PARO_H */
