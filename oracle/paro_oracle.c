/*
 * CPU oracle for the rotated-W4A16 linear path of Pairwise Rotation Quantization
 * (arXiv 2511.10645).  TEST INFRASTRUCTURE ONLY: it exists to check the GPU
 * library and to be timed beside it.  Nothing in the product path may call it.
 *
 * Plain C, fp64 arithmetic, no blocking, no fusion: every function is the
 * definition written out, so it can be checked against the paper by eye.
 * It shares no code, header, table or constant with the GPU library.
 *
 * Column-vector form of the whole path (equivalent to the row-vector Eq. 2):
 *      y = W^ . ( R_K ... R_1 . S . x ),
 *      W^[n,c] = (q[n,c] - z[c/g,n]) * s[c/g,n],      S = diag(ch_scale)
 *
 * Passages followed
 *   Eq. 1 + the group rule of Section 2.1 : linear quantiser; dequantisation is
 *                                           its inverse map  w^ = (q - z) * s,
 *                                           one (s, z) per g consecutive input
 *                                           channels of one output column
 *   Eq. 2                                  : Y = (X T^-1)(T W) + b
 *   Eq. 4                                  : the pair update and its signs
 *   Eq. 5                                  : activation side, layers in index order
 *   Eq. 8, Fig. 2 caption, App. A.4        : weights get scaling first, then the
 *                                           K rotations => activations get the
 *                                           inverse scale first, then the
 *                                           rotations, layer 1 first
 *   Def. 1                                 : pairs of one layer are disjoint
 *   Eq. 1, Eq. 8 (weight side)             : W' = R_K ... R_1 . diag(alpha) . W per
 *                                           output row, then RTN per group
 *   Section 4.3, speed-up figure           : the Hadamard transform it is compared with
 *                                           (Sylvester order, orthonormal)
 *   App. A.3, first equation               : Y' = Q(X T^-1) . Q(T W) + b with both
 *                                           operands in MXFP4 (element and scale
 *                                           formats of the OCP Microscaling
 *                                           Formats specification)
 *
 * Readings where the paper leaves a choice
 *   - theta on the activation side.  Eq. 5 right-multiplies a row vector by
 *     G(i,j,-theta).  With G(i,j,theta) as in Eq. 4 (G_ii = G_jj = cos,
 *     G_ij = -sin, G_ji = +sin), (x G(-theta))_i = cos x_i - sin x_j and
 *     (x G(-theta))_j = sin x_i + cos x_j: the same formula as Eq. 4 with
 *     +theta.  The caller passes the learned theta unchanged.
 *   - ch_scale is the multiplier seen by the activations (1/alpha of Eq. 8).
 *   - a pair (i, i) is a no-op slot (layers may hold fewer than g/2 pairs).
 *   - pair indices are 0-based and local to the group; (j, i, theta) is the
 *     same rotation as (i, j, -theta).
 *   - cos/sin: libm in fp64 on the fp32 angle widened to fp64.
 *   - packing: 8 codes per uint32, code k in bits 4k..4k+3, along the input
 *     dimension for weights and along the output dimension for zero points.
 *
 * Pins (tests/test_oracle_*.py): hand-computed one- and two-layer cases fix the
 * sign and the layer order; per-layer norm preservation; inverse round trip;
 * explicit dense-matrix formulation multiplied by a library matmul; theta = 0,
 * scale = 1 reduces to numpy's X @ W^T; brute-force Eq. 2 on tiny unquantised
 * inputs; exhaustive unpack; exhaustive fp64->fp16 rounding against numpy.
 * Weight side: hand-computed RTN groups, the s/2 error bound of Eq. 1, and
 * transformed weights times transformed activations reproducing W.x (Eq. 2).
 * Hadamard yardstick: n = 2 and n = 4 by hand, scipy's Hadamard matrix, involution and norm.
 * The paper's accuracy tables are not on this path: parity unpinned for them.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- fp16 <-> fp64, written out by hand (IEEE 754 binary16) -------------- */

double oracle_fp16_to_f64(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0) {
        v = ldexp((double)m, -24);                 /* subnormal: m * 2^-24 */
    } else if (e == 31) {
        v = m ? NAN : INFINITY;
    } else {
        v = ldexp((double)(m | 0x400), e - 25);    /* (1024+m) * 2^(e-15-10) */
    }
    return sign ? -v : v;
}

/* round-to-nearest-even of a double to binary16, returned as bits */
uint16_t oracle_f64_to_fp16(double v)
{
    uint16_t sign = 0;
    if (v != v) return 0x7e00;
    if (signbit(v)) { sign = 0x8000; v = -v; }
    if (v == 0.0) return sign;
    if (isinf(v)) return sign | 0x7c00;
    int ex;
    (void)frexp(v, &ex);            /* v = fr * 2^ex, fr in [0.5,1) */
    int e = ex - 1;                 /* v = (2 fr) * 2^e, 2fr in [1,2) */
    /* quantum of the target binade: 2^(e-10) for normals, 2^-24 below 2^-14 */
    int qexp = (e < -14) ? -24 : e - 10;
    double scaled = ldexp(v, -qexp);            /* exact: power-of-two scaling */
    double fl = floor(scaled);
    double rem = scaled - fl;                   /* exact in fp64 (53 > 11 bits kept) */
    uint64_t n = (uint64_t)fl;
    if (rem > 0.5 || (rem == 0.5 && (n & 1))) n += 1;
    /* n counts quanta; rebuild the encoding */
    if (e < -14) {
        /* subnormal range: n in [0, 1024]; n == 1024 is the smallest normal */
        return sign | (uint16_t)n;              /* 1024 -> exponent field 1, mantissa 0 */
    }
    if (n == 2048) { n = 1024; e += 1; }        /* mantissa overflowed into next binade */
    if (e > 15) return sign | 0x7c00;           /* overflow -> inf */
    return sign | (uint16_t)(((e + 15) << 10) | (n & 0x3ff));
}

void oracle_round_fp16(const double *v, int64_t n, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = oracle_f64_to_fp16(v[i]);
}

void oracle_widen_fp16(const uint16_t *h, int64_t n, double *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = oracle_fp16_to_f64(h[i]);
}

/* ---- scaled pairwise rotation on activations (Eq. 4, 5, 8) --------------- */

/*
 * The K rotation layers alone, in place on fp64 rows (Eq. 4 applied pair by
 * pair, layers in array order as in Eq. 5).  pairs: [G][n_layers][ppl][2]
 * local indices; theta: [G][n_layers][ppl].  Returns 0, or -1 if an index is
 * out of range.
 */
int oracle_rotate_inplace(double *u, int64_t ldu, int32_t T, int32_t C,
                          int32_t group, int32_t n_layers, int32_t ppl,
                          const int16_t *pairs, const float *theta)
{
    int32_t G = C / group;
    for (int64_t k = 0; k < (int64_t)G * n_layers * ppl * 2; ++k)
        if (pairs[k] < 0 || pairs[k] >= group) return -1;
#pragma omp parallel for schedule(static)
    for (int32_t t = 0; t < T; ++t) {
        for (int32_t g = 0; g < G; ++g) {
            double *ug = u + (int64_t)t * ldu + (int64_t)g * group;
            for (int32_t l = 0; l < n_layers; ++l) {           /* layer 1 first */
                for (int32_t p = 0; p < ppl; ++p) {
                    int64_t k = (((int64_t)g * n_layers + l) * ppl + p);
                    int i = pairs[2 * k], j = pairs[2 * k + 1];
                    if (i == j) continue;                       /* empty slot */
                    double th = (double)theta[k];
                    double cs = cos(th), sn = sin(th);
                    double ui = ug[i], uj = ug[j];
                    ug[i] = cs * ui - sn * uj;                  /* Eq. 4, first row  */
                    ug[j] = sn * ui + cs * uj;                  /* Eq. 4, second row */
                }
            }
        }
    }
    return 0;
}

/*
 * u[t][c] on exit = ( R_K ... R_1 . S . x_t )[c]      (scale_order == 0, the paper)
 *                 = ( S . R_K ... R_1 . x_t )[c]      (scale_order == 1)
 * x16: fp16 bits, row t at x16 + t*ldx; ch_scale16: [C] fp16 bits or NULL (ones).
 */
int oracle_rotate_scale(const uint16_t *x16, int64_t ldx, int32_t T, int32_t C,
                        int32_t group, int32_t n_layers, int32_t ppl,
                        const int16_t *pairs, const float *theta,
                        const uint16_t *ch_scale16, int32_t scale_order,
                        double *u, int64_t ldu)
{
    for (int32_t t = 0; t < T; ++t)
        for (int32_t c = 0; c < C; ++c) {
            double v = oracle_fp16_to_f64(x16[(int64_t)t * ldx + c]);
            if (scale_order == 0 && ch_scale16) v *= oracle_fp16_to_f64(ch_scale16[c]);
            u[(int64_t)t * ldu + c] = v;
        }
    int rc = oracle_rotate_inplace(u, ldu, T, C, group, n_layers, ppl, pairs, theta);
    if (rc) return rc;
    if (scale_order == 1 && ch_scale16)
        for (int32_t t = 0; t < T; ++t)
            for (int32_t c = 0; c < C; ++c) u[(int64_t)t * ldu + c] *= oracle_fp16_to_f64(ch_scale16[c]);
    return 0;
}

/* ---- weight side: equivalent transform (Eq. 8) and RTN quantiser (Eq. 1) -- */

/*
 * wt[n][c] = ( R_K ... R_1 . diag(alpha) . w_n )[c]      (scale_order == 0, the paper: Eq. 8)
 *          = ( diag(alpha) . R_K ... R_1 . w_n )[c]      (scale_order == 1)
 * with alpha = 1 / ch_scale: the weight-side counterpart of oracle_rotate_scale, so that
 * wt_n . u = w_n . x when u is the transformed activation vector (Eq. 2).  w16: fp16 bits,
 * row n (one output channel, C input channels) at w16 + n*ldw.
 */
int oracle_weight_transform(const uint16_t *w16, int64_t ldw, int32_t N, int32_t C,
                            int32_t group, int32_t n_layers, int32_t ppl,
                            const int16_t *pairs, const float *theta,
                            const uint16_t *ch_scale16, int32_t scale_order,
                            double *wt, int64_t ldwt)
{
    for (int32_t n = 0; n < N; ++n)
        for (int32_t c = 0; c < C; ++c) {
            double v = oracle_fp16_to_f64(w16[(int64_t)n * ldw + c]);
            if (scale_order == 0 && ch_scale16) v /= oracle_fp16_to_f64(ch_scale16[c]);
            wt[(int64_t)n * ldwt + c] = v;
        }
    if (n_layers > 0) {
        int rc = oracle_rotate_inplace(wt, ldwt, N, C, group, n_layers, ppl, pairs, theta);
        if (rc) return rc;
    }
    if (scale_order == 1 && ch_scale16)
        for (int32_t n = 0; n < N; ++n)
            for (int32_t c = 0; c < C; ++c) wt[(int64_t)n * ldwt + c] /= oracle_fp16_to_f64(ch_scale16[c]);
    return 0;
}

/*
 * Eq. 1 with b = 4, one (s, z) per `group` consecutive input channels of one output row:
 *      s = (max - min) / 15,   z = -round(min / s),   q = clamp(round(w / s) + z, 0, 15),
 * written out in fp64 exactly as printed.  The one step that is not fp64 is marked below: the
 * scale is STORED as fp16 (the weight format of Section 2.1 as used here keeps one fp16 scale
 * per group), and z and q are computed with the stored value, so that (q - z) * s reproduces w
 * to within s/2 wherever nothing was clamped.
 * Readings (the paper gives the formula only):
 *   - round() is round-half-to-even (rint);
 *   - s has the floor 2^-14 (smallest normal fp16), which also covers constant groups;
 *   - z is an INT4 value: clamped to 0..15.
 * codes: [N][C] bytes; scales16: [G][N] fp16 bits; zeros: [G][N] bytes.
 */
void oracle_rtn_quantize(const double *wt, int64_t ldwt, int32_t N, int32_t C, int32_t group,
                         uint8_t *codes, uint16_t *scales16, uint8_t *zeros)
{
    int32_t G = C / group;
#pragma omp parallel for schedule(static)
    for (int32_t n = 0; n < N; ++n)
        for (int32_t g = 0; g < G; ++g) {
            const double *wg = wt + (int64_t)n * ldwt + (int64_t)g * group;
            double mn = wg[0], mx = wg[0];
            for (int32_t c = 1; c < group; ++c) {
                if (wg[c] < mn) mn = wg[c];
                if (wg[c] > mx) mx = wg[c];
            }
            double s_exact = (mx - mn) / 15.0;
            if (!(s_exact >= 6.103515625e-05)) s_exact = 6.103515625e-05;
            uint16_t sb = oracle_f64_to_fp16(s_exact);      /* <- the single rounding: the stored fp16 scale */
            double s = oracle_fp16_to_f64(sb);
            double z = -rint(mn / s);
            if (z < 0.0) z = 0.0;
            if (z > 15.0) z = 15.0;
            scales16[(int64_t)g * N + n] = sb;
            zeros[(int64_t)g * N + n] = (uint8_t)z;
            for (int32_t c = 0; c < group; ++c) {
                double q = rint(wg[c] / s) + z;
                if (q < 0.0) q = 0.0;
                if (q > 15.0) q = 15.0;
                codes[(int64_t)n * C + (int64_t)g * group + c] = (uint8_t)q;
            }
        }
}

/*
 * Microscaling FP4 (MXFP4: 32 consecutive values share one power-of-two scale stored as an
 * E8M0 byte, each value is an FP4 E2M1 code), the conversion the OCP Microscaling Formats
 * specification gives for a block V:
 *      shared_exp = floor(log2(max |V_i|)) - 2          (2 = largest E2M1 exponent), >= -127
 *      code_i     = E2M1( V_i / 2^shared_exp ), round to nearest, ties to even, saturating at 6
 * E2M1 magnitudes by code 0..7: 0, 0.5, 1, 1.5, 2, 3, 4, 6; bit 3 is the sign.  An all-zero
 * block gets the smallest scale (byte 0) and zero codes.  Input rows are fp64; scaling by a power of
 * two and the comparisons against the eight magnitudes are exact in fp64, so nothing is rounded
 * before the code is chosen.
 * codes: [T][C] bytes (0..15); scales: [T][C/32] bytes (shared_exp + 127).
 */
void oracle_mxfp4_quantize(const double *u, int64_t ldu, int32_t T, int32_t C, uint8_t *codes, uint8_t *scales)
{
    static const double grid[8] = {0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0};
#pragma omp parallel for schedule(static)
    for (int32_t t = 0; t < T; ++t)
        for (int32_t b = 0; b < C / 32; ++b) {
            const double *v = u + (int64_t)t * ldu + (int64_t)b * 32;
            double amax = 0.0;
            for (int i = 0; i < 32; ++i) {
                double a = fabs(v[i]);
                if (a > amax) amax = a;
            }
            int shared = -127;
            if (amax > 0.0) {
                int e;
                (void)frexp(amax, &e);               /* amax = m * 2^e, 0.5 <= m < 1  =>  floor(log2) = e - 1 */
                shared = (e - 1) - 2;
                if (shared < -127) shared = -127;
            }
            scales[(int64_t)t * (C / 32) + b] = (uint8_t)(shared + 127);
            for (int i = 0; i < 32; ++i) {
                double r = ldexp(v[i], -shared);
                double a = fabs(r);
                int code = 7;                        /* saturate */
                if (a <= 6.0) {
                    /* nearest grid point, ties to the code with an even mantissa bit (even code) */
                    double best = 1e300;
                    code = 0;
                    for (int k = 0; k < 8; ++k) {
                        double d = fabs(a - grid[k]);
                        if (d < best || (d == best && (k & 1) == 0)) { best = d; code = k; }
                    }
                }
                if (r < 0.0 || (r == 0.0 && signbit(r))) code |= 8;
                codes[(int64_t)t * C + (int64_t)b * 32 + i] = (uint8_t)code;
            }
        }
}

/*
 * The value an MXFP4 element stands for (OCP Microscaling Formats specification):
 *      v = (-1)^sign * M[code & 7] * 2^(scale_byte - 127),   M = 0, 0.5, 1, 1.5, 2, 3, 4, 6
 * (E2M1: exponent bias 1, subnormal 0.5; E8M0 scale: bias 127).  Exact in fp64.
 * codes: [T][C] bytes, scales: [T][C/32] bytes, out: [T][C] fp64.
 */
void oracle_mxfp4_dequant(const uint8_t *codes, const uint8_t *scales, int32_t T, int32_t C, double *out)
{
    for (int64_t t = 0; t < T; ++t)
        for (int32_t c = 0; c < C; ++c) {
            int code = codes[t * C + c];
            int e = (code >> 1) & 3, m = code & 1;
            double mag = e == 0 ? 0.5 * m : ldexp(1.0 + 0.5 * m, e - 1);
            double v = ldexp(mag, (int)scales[t * (C / 32) + c / 32] - 127);
            out[t * C + c] = (code & 8) ? -v : v;
        }
}

/*
 * The weight-activation form of the linear layer (App. A.3, first equation):
 *      Y' = Q(X T^-1) . Q(T W) + b
 * for operands that are already quantised to MXFP4: y[t][n] = sum_c x^[t][c] w^[n][c] (+ bias[n]),
 * x^ and w^ the values the codes stand for.  fp64; every product is exact and the sum is exact as
 * long as the block exponents of a row span fewer than ~40 binades.
 * xc: [T][C], xs: [T][C/32], wc: [N][C], ws: [N][C/32], bias16: [N] fp16 bits or NULL, y: [T][N].
 */
void oracle_mxfp4_linear(const uint8_t *xc, const uint8_t *xs, int32_t T, const uint8_t *wc, const uint8_t *ws,
                         int32_t N, int32_t C, const uint16_t *bias16, double *y)
{
    double *xv = (double *)malloc((size_t)T * C * sizeof(double));
    double *wv = (double *)malloc((size_t)N * C * sizeof(double));
    oracle_mxfp4_dequant(xc, xs, T, C, xv);
    oracle_mxfp4_dequant(wc, ws, N, C, wv);
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t t = 0; t < T; ++t) {
            double acc = 0.0;
            for (int32_t c = 0; c < C; ++c) acc += xv[t * C + c] * wv[n * C + c];
            if (bias16) acc += oracle_fp16_to_f64(bias16[n]);
            y[t * N + n] = acc;
        }
    free(xv);
    free(wv);
}

/* ---- INT4 unpack and dequantisation (Eq. 1 inverted, group rule) --------- */

void oracle_unpack_codes(const uint32_t *qweight, int32_t N, int32_t C, uint8_t *codes)
{
    for (int64_t n = 0; n < N; ++n)
        for (int32_t c = 0; c < C; ++c)
            codes[n * C + c] = (uint8_t)((qweight[n * (C / 8) + c / 8] >> (4 * (c % 8))) & 15u);
}

void oracle_unpack_zeros(const uint32_t *qzeros, int32_t G, int32_t N, uint8_t *zeros)
{
    for (int64_t g = 0; g < G; ++g)
        for (int32_t n = 0; n < N; ++n)
            zeros[g * N + n] = (uint8_t)((qzeros[g * (N / 8) + n / 8] >> (4 * (n % 8))) & 15u);
}

static inline double deq_one(const uint32_t *qweight, const uint16_t *scales16, const uint32_t *qzeros,
                             int32_t N, int32_t C, int32_t group, int64_t n, int32_t c)
{
    int q = (int)((qweight[n * (C / 8) + c / 8] >> (4 * (c % 8))) & 15u);
    int64_t g = c / group;
    int z = (int)((qzeros[g * (N / 8) + n / 8] >> (4 * (n % 8))) & 15u);
    return (double)(q - z) * oracle_fp16_to_f64(scales16[g * N + n]);
}

/* W[n][c] = (q - z) * s, fp64 (exact: a 5-bit integer times an 11-bit significand) */
void oracle_dequant(const uint32_t *qweight, const uint16_t *scales16, const uint32_t *qzeros,
                    int32_t N, int32_t C, int32_t group, double *W)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int32_t c = 0; c < C; ++c)
            W[n * C + c] = deq_one(qweight, scales16, qzeros, N, C, group, n, c);
}

/* squared L2 norm of each dequantised row (used by the linear tolerance) */
void oracle_row_sqnorms(const uint32_t *qweight, const uint16_t *scales16, const uint32_t *qzeros,
                        int32_t N, int32_t C, int32_t group, double *sq)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double a = 0.0;
        for (int32_t c = 0; c < C; ++c) {
            double w = deq_one(qweight, scales16, qzeros, N, C, group, n, c);
            a += w * w;
        }
        sq[n] = a;
    }
}

/* ---- the contraction (Eq. 2) --------------------------------------------- */

/* y[t][n] = sum_c W^[n][c] * u[t][c] (+ bias[n]),  all fp64, c ascending */
void oracle_linear(const double *u, int64_t ldu, int32_t T,
                   const uint32_t *qweight, const uint16_t *scales16, const uint32_t *qzeros,
                   const uint16_t *bias16, int32_t N, int32_t C, int32_t group,
                   double *y, int64_t ldy)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double *w = (double *)malloc(sizeof(double) * (size_t)C);
        for (int32_t c = 0; c < C; ++c) w[c] = deq_one(qweight, scales16, qzeros, N, C, group, n, c);
        double b = bias16 ? oracle_fp16_to_f64(bias16[n]) : 0.0;
        for (int32_t t = 0; t < T; ++t) {
            const double *ut = u + (int64_t)t * ldu;
            double a = 0.0;
            for (int32_t c = 0; c < C; ++c) a += w[c] * ut[c];
            y[(int64_t)t * ldy + n] = a + b;
        }
        free(w);
    }
}

/* the same sum for a list of (t, n) samples, one by one */
void oracle_linear_samples(const double *u, int64_t ldu,
                           const uint32_t *qweight, const uint16_t *scales16, const uint32_t *qzeros,
                           const uint16_t *bias16, int32_t N, int32_t C, int32_t group,
                           const int32_t *t_idx, const int32_t *n_idx, int64_t n_samples,
                           double *y, double *w_sqnorm)
{
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < n_samples; ++s) {
        int64_t n = n_idx[s];
        const double *ut = u + (int64_t)t_idx[s] * ldu;
        double a = 0.0, ww = 0.0;
        for (int32_t c = 0; c < C; ++c) {
            double w = deq_one(qweight, scales16, qzeros, N, C, group, n, c);
            a += w * ut[c];
            ww += w * w;
        }
        y[s] = a + (bias16 ? oracle_fp16_to_f64(bias16[n]) : 0.0);
        if (w_sqnorm) w_sqnorm[s] = ww;
    }
}

/*
 * Walsh-Hadamard transform of each row, Sylvester (natural) order, orthonormal scaling - the
 * yardstick the transform kernel is compared with in Section 4.3 (figure "speedup of scaled
 * pairwise rotation over the Hadamard transform"):
 *      y = H_n x / sqrt(n),   H_1 = [1],  H_2m = [[H_m, H_m], [H_m, -H_m]],
 * i.e. H_n[i][j] = (-1)^popcount(i & j).  Written as that definition, one dot product per output
 * (O(n^2) per row): no butterfly, so that it can be read against the definition by eye.
 * x16: [T][ldx] fp16 bits, y: [T][ldy] fp64, n a power of two.  Returns -1 if n is not.
 */
int oracle_fwht(const uint16_t *x16, int64_t ldx, int32_t T, int32_t n, double *y, int64_t ldy)
{
    if (n < 1 || (n & (n - 1))) return -1;
    const double inv = 1.0 / sqrt((double)n);
#pragma omp parallel for schedule(static) collapse(2)
    for (int32_t t = 0; t < T; ++t)
        for (int32_t i = 0; i < n; ++i) {
            double acc = 0.0;
            for (int32_t j = 0; j < n; ++j) {
                double v = oracle_fp16_to_f64(x16[(int64_t)t * ldx + j]);
                acc += (__builtin_popcount((unsigned)(i & j)) & 1) ? -v : v;
            }
            y[(int64_t)t * ldy + i] = acc * inv;
        }
    return 0;
}
