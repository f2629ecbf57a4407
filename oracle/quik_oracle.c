/*
 * CPU oracle for the QUIK hybrid-quantized linear layer (arXiv 2310.09259).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, step-by-step CPU
 * implementation of "QUIK Matmul" (Algorithm 1 of the paper) used to check the
 * GPU library.  It shares no code, header, table or helper with the HIP path and
 * must never be called from the product path: only tests, the smoke check and
 * the benchmark's cpu_baseline leg may load it.
 *
 * Every function takes HOST pointers.  Arithmetic follows the paper's steps in
 * the paper's order; there is no blocking, fusion or reordering.  Floating point
 * in the quantizer is IEEE binary32 (round-to-nearest-even, no FMA contraction:
 * build with -ffp-contract=off and without -ffast-math), because the quantized
 * integers must be reproduced bit for bit.  The dequantized output is formed in
 * binary64 and rounded once to binary32.
 *
 * Readings taken where the paper leaves a choice (Section 3.3, Algorithm 1):
 *   - findZeroScale: zero = row minimum, scale = (max - min) / (2^bits - 1),
 *     both over the NON-outlier columns only; a constant row gets scale = 1.
 *   - halfRange = 2^(bits-1).
 *   - "(elem - zero) / scale" is evaluated as (elem - zero) * (1 / scale) with
 *     one correctly rounded reciprocal per token; rounding to integer is
 *     round-half-to-even followed by a clamp to [0, 2^bits - 1].
 *   - wReduced[n] = scaleWeight[n] * sum_k wInt[n,k]   (scale folded in).
 *   - packed INT4: two's-complement nibbles.  The paper only says "packed format"; the
 *     nibble order is a free choice per operand.  Weights: element 2p in the low nibble of
 *     byte p.  Activations: element 2p in the HIGH nibble (so that on the target GPU every
 *     operand register is produced from a packed word with one AND; the GEMM pairs an
 *     activation's high nibble with a weight's low nibble of the same k and vice versa).
 *   - base (non-outlier) columns keep ascending original order; outlier column
 *     j of xFP / wFP corresponds to FPindices[j].
 *
 * Parity pins (tests/test_oracle_*.py, all CPU): closed forms for scale/zero,
 * range and round-trip invariants, brute-force integer dot products, Eq. (1)
 * re-evaluated by an independent float64 GEMM of the dequantized operands, and
 * special cases that reduce to a textbook matmul.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define QO_OK 0
#define QO_EINVAL (-1)
#define QO_EOVERFLOW (-2)
#define QO_ENOMEM (-3)

/* ---- binary16 -> binary32, exact (own conversion; no compiler half type) ---- */
static float half_bits_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    uint32_t expo = (uint32_t)(h >> 10) & 0x1Fu;
    uint32_t mant = (uint32_t)h & 0x3FFu;
    double v;
    if (expo == 0) {
        v = ldexp((double)mant, -24);                /* zero or subnormal */
    } else if (expo == 31) {
        v = mant ? NAN : INFINITY;
    } else {
        v = ldexp((double)(mant | 0x400u), (int)expo - 25);
    }
    return (float)(sign ? -v : v);                   /* exact: 11-bit significand */
}

int quik_oracle_version(void) { return 1; }

void quik_oracle_half_to_float(const uint16_t *h, int64_t n, float *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = half_bits_to_float(h[i]);
}

/*
 * Algorithm 1, "split": list of base columns = all columns not in FPindices,
 * ascending.  Returns the number of base columns, or a negative error if an
 * index is out of range or repeated.
 */
int quik_oracle_base_columns(int K, const int32_t *idx, int n_out, int32_t *base)
{
    if (K <= 0 || n_out < 0 || n_out >= K) return QO_EINVAL;
    unsigned char *is_out = (unsigned char *)calloc((size_t)K, 1);
    if (!is_out) return QO_ENOMEM;
    for (int j = 0; j < n_out; ++j) {
        if (idx[j] < 0 || idx[j] >= K || is_out[idx[j]]) { free(is_out); return QO_EINVAL; }
        is_out[idx[j]] = 1;
    }
    int nb = 0;
    for (int k = 0; k < K; ++k)
        if (!is_out[k]) base[nb++] = k;
    free(is_out);
    return nb;
}

/*
 * Packed storage of quantized values (Section 3.3, "packed format").
 * bits = 4, two's complement nibbles: byte p holds elements 2p and 2p+1;
 *   even_high = 0 (weights):     element 2p in bits 0..3, element 2p+1 in bits 4..7;
 *   even_high = 1 (activations): element 2p in bits 4..7, element 2p+1 in bits 0..3.
 * bits = 8: one signed byte per element (even_high ignored).
 */
int quik_oracle_pack(const int8_t *q, int64_t rows, int K_b, int bits, int even_high, uint8_t *packed)
{
    if (bits == 8) {
        memcpy(packed, q, (size_t)rows * (size_t)K_b);
        return QO_OK;
    }
    if (bits != 4 || (K_b & 1)) return QO_EINVAL;
    for (int64_t r = 0; r < rows; ++r)
        for (int p = 0; p < K_b / 2; ++p) {
            int e0 = q[r * K_b + 2 * p], e1 = q[r * K_b + 2 * p + 1];
            int lo = even_high ? e1 : e0, hi = even_high ? e0 : e1;
            packed[r * (K_b / 2) + p] = (uint8_t)((lo & 0xF) | ((hi & 0xF) << 4));
        }
    return QO_OK;
}

int quik_oracle_unpack(const uint8_t *packed, int64_t rows, int K_b, int bits, int even_high, int8_t *q)
{
    if (bits == 8) {
        memcpy(q, packed, (size_t)rows * (size_t)K_b);
        return QO_OK;
    }
    if (bits != 4 || (K_b & 1)) return QO_EINVAL;
    for (int64_t r = 0; r < rows; ++r)
        for (int p = 0; p < K_b / 2; ++p) {
            int b = packed[r * (K_b / 2) + p];
            int lo = b & 0xF, hi = (b >> 4) & 0xF;
            int e0 = even_high ? hi : lo, e1 = even_high ? lo : hi;
            q[r * K_b + 2 * p] = (int8_t)(e0 >= 8 ? e0 - 16 : e0);
            q[r * K_b + 2 * p + 1] = (int8_t)(e1 >= 8 ? e1 - 16 : e1);
        }
    return QO_OK;
}

/*
 * Algorithm 1, "split" + "Quantization" (lines 3-4 and the Quantization
 * function).  x: fp16 bits [T, K] row-major.  Outputs:
 *   q      int8  [T, K_b]   signed quantized values in [-halfRange, halfRange-1]
 *   scale  f32   [T]        scaleAct
 *   zero   f32   [T]        zeroAct (the row minimum, a float offset)
 *   x_out  fp16  [T, n_out] outlier columns, bit copies, column j <- idx[j]
 *   n_tie_mismatch (optional): number of elements whose code differs from
 *       clamp(rint((x - zero) / scale)) evaluated in binary64 -- an audit of the
 *       reciprocal-multiply reading; such elements are all near .5 ties.
 */
int quik_oracle_quantize(const uint16_t *x, int T, int K, const int32_t *idx, int n_out, int bits,
                         int8_t *q, float *scale, float *zero, uint16_t *x_out,
                         int64_t *n_tie_mismatch)
{
    if (T < 0 || (bits != 4 && bits != 8)) return QO_EINVAL;
    int32_t *base = (int32_t *)malloc(sizeof(int32_t) * (size_t)(K > 0 ? K : 1));
    if (!base) return QO_ENOMEM;
    int K_b = quik_oracle_base_columns(K, idx, n_out, base);
    if (K_b < 0) { free(base); return K_b; }
    const int levels = (1 << bits) - 1;        /* 2^bits - 1 */
    const int half_range = 1 << (bits - 1);
    int64_t mismatches = 0;

#pragma omp parallel for schedule(static) reduction(+ : mismatches)
    for (int t = 0; t < T; ++t) {
        const uint16_t *row = x + (int64_t)t * K;
        /* split: outlier part, untouched */
        for (int j = 0; j < n_out; ++j) x_out[(int64_t)t * n_out + j] = row[idx[j]];
        /* findZeroScale over the base part */
        float mn = half_bits_to_float(row[base[0]]), mx = mn;
        for (int k = 1; k < K_b; ++k) {
            float v = half_bits_to_float(row[base[k]]);
            if (v < mn) mn = v;
            if (v > mx) mx = v;
        }
        if (mn == 0.0f) mn = 0.0f;             /* drop a possible minus sign of zero */
        float range = mx - mn;
        float s = (range == 0.0f) ? 1.0f : range / (float)levels;
        float inv = 1.0f / s;
        scale[t] = s;
        zero[t] = mn;
        /* quantize: (elem - zero) / scale, round, clamp, - halfRange */
        for (int k = 0; k < K_b; ++k) {
            float v = half_bits_to_float(row[base[k]]);
            float d = v - mn;
            float u = d * inv;
            int qu = (int)rintf(u);
            if (qu < 0) qu = 0;
            if (qu > levels) qu = levels;
            q[(int64_t)t * K_b + k] = (int8_t)(qu - half_range);
            if (n_tie_mismatch) {
                double ud = ((double)v - (double)mn) / (double)s;
                long qd = lrint(ud);
                if (qd < 0) qd = 0;
                if (qd > levels) qd = levels;
                if (qd != qu) ++mismatches;
            }
        }
    }
    if (n_tie_mismatch) *n_tie_mismatch = mismatches;
    free(base);
    return QO_OK;
}

/*
 * Algorithm 1, "INTmatmul": acc[t,n] = sum_k q[t,k] * wq[n,k], exact integers.
 * The entry check proves every partial sum fits in int32 for the given bit
 * width, so the int32 accumulator below is exact.
 */
int quik_oracle_int_gemm(const int8_t *q, const int8_t *wq, int T, int N, int K_b, int bits,
                         int32_t *acc)
{
    if (T < 0 || N < 0 || K_b <= 0 || (bits != 4 && bits != 8)) return QO_EINVAL;
    int64_t max_prod = (int64_t)1 << (2 * (bits - 1));       /* halfRange^2 */
    if ((int64_t)K_b * max_prod >= ((int64_t)1 << 31)) return QO_EOVERFLOW;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const int8_t *a = q + (int64_t)t * K_b;
        for (int n = 0; n < N; ++n) {
            const int8_t *b = wq + (int64_t)n * K_b;
            int32_t s = 0;
            for (int k = 0; k < K_b; ++k) s += (int32_t)a[k] * (int32_t)b[k];
            acc[(int64_t)t * N + n] = s;
        }
    }
    return QO_OK;
}

/*
 * wReduced (Section 3.3, text after Eq. (1)): the static per-output-row sum of
 * the quantized base weights, with the weight scale folded in:
 *   wReduced[n] = float(scaleWeight[n]) * float(sum_k wq[n,k]).
 * The integer sum is exact and below 2^24 in magnitude, so its float is exact.
 */
int quik_oracle_weight_reduce(const int8_t *wq, const uint16_t *w_scale, int N, int K_b,
                              float *w_reduced)
{
    if (N < 0 || K_b <= 0) return QO_EINVAL;
    for (int n = 0; n < N; ++n) {
        int64_t s = 0;
        for (int k = 0; k < K_b; ++k) s += wq[(int64_t)n * K_b + k];
        w_reduced[n] = half_bits_to_float(w_scale[n]) * (float)s;
    }
    return QO_OK;
}

/* Algorithm 1, "FPmatmul": resultFP[t,n] = sum_j xFP[t,j] * wFP[n,j], binary64. */
int quik_oracle_fp_matmul(const uint16_t *x_out, const uint16_t *w_out, int T, int N, int n_out,
                          double *result_fp)
{
    if (T < 0 || N < 0 || n_out < 0) return QO_EINVAL;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int n = 0; n < N; ++n) {
            double s = 0.0;
            for (int j = 0; j < n_out; ++j)
                s += (double)half_bits_to_float(x_out[(int64_t)t * n_out + j]) *
                     (double)half_bits_to_float(w_out[(int64_t)n * n_out + j]);
            result_fp[(int64_t)t * N + n] = s;
        }
    return QO_OK;
}

/*
 * Algorithm 1, "Dequantization" followed by the final add (line 8):
 *   x     = elem * scaleAct * scaleWeight
 *   shift = (zeroAct + halfRange * scaleAct) * wReduced
 *   y     = x + shift + resultFP (+ bias)
 * evaluated in binary64 and rounded once to binary32.
 * result_fp may be NULL (no outliers); bias (fp16 [N]) may be NULL.
 */
int quik_oracle_dequant_add(const int32_t *acc, const float *scale, const float *zero,
                            const uint16_t *w_scale, const float *w_reduced,
                            const double *result_fp, const uint16_t *bias, int T, int N, int bits,
                            float *y)
{
    if (T < 0 || N < 0 || (bits != 4 && bits != 8)) return QO_EINVAL;
    const double half_range = (double)(1 << (bits - 1));
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int n = 0; n < N; ++n) {
            int64_t i = (int64_t)t * N + n;
            double xv = (double)acc[i] * (double)scale[t] * (double)half_bits_to_float(w_scale[n]);
            double shift = (double)zero[t] + half_range * (double)scale[t];
            shift = shift * (double)w_reduced[n];
            double out = xv + shift;
            if (result_fp) out += result_fp[i];
            if (bias) out += (double)half_bits_to_float(bias[n]);
            y[i] = (float)out;
        }
    return QO_OK;
}

/*
 * "QUIK Matmul" end to end (Algorithm 1, lines 1-9), from the layer's inputs:
 * x fp16 [T,K], FPindices, packed wInt [N, K_b*bits/8], scaleWeight fp16 [N],
 * wFP fp16 [N, n_out], optional bias.  Any of the optional outputs may be NULL.
 */
int quik_oracle_linear(const uint16_t *x, int T, int K, const int32_t *idx, int n_out, int bits,
                       const uint8_t *w_packed, const uint16_t *w_scale, const uint16_t *w_out,
                       const uint16_t *bias, int N,
                       float *y, int8_t *q_opt, float *scale_opt, float *zero_opt,
                       uint16_t *x_out_opt, int32_t *acc_opt, float *w_reduced_opt)
{
    if (T <= 0 || N <= 0 || K <= 0 || n_out < 0 || n_out >= K) return QO_EINVAL;
    const int K_b = K - n_out;
    if ((K_b * bits) % 8) return QO_EINVAL;
    int rc = QO_ENOMEM;
    int8_t *q = (int8_t *)malloc((size_t)T * K_b);
    int8_t *wq = (int8_t *)malloc((size_t)N * K_b);
    float *scale = (float *)malloc(sizeof(float) * T), *zero = (float *)malloc(sizeof(float) * T);
    uint16_t *xo = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)T * (n_out ? n_out : 1));
    int32_t *acc = (int32_t *)malloc(sizeof(int32_t) * (size_t)T * N);
    float *wred = (float *)malloc(sizeof(float) * N);
    double *rfp = (double *)malloc(sizeof(double) * (size_t)T * N);
    if (!q || !wq || !scale || !zero || !xo || !acc || !wred || !rfp) goto done;

    if ((rc = quik_oracle_unpack(w_packed, N, K_b, bits, 0, wq))) goto done;
    if ((rc = quik_oracle_weight_reduce(wq, w_scale, N, K_b, wred))) goto done;
    if ((rc = quik_oracle_quantize(x, T, K, idx, n_out, bits, q, scale, zero, xo, NULL))) goto done;
    if ((rc = quik_oracle_fp_matmul(xo, w_out, T, N, n_out, rfp))) goto done;
    if ((rc = quik_oracle_int_gemm(q, wq, T, N, K_b, bits, acc))) goto done;
    if ((rc = quik_oracle_dequant_add(acc, scale, zero, w_scale, wred, rfp, bias, T, N, bits, y)))
        goto done;

    if (q_opt) memcpy(q_opt, q, (size_t)T * K_b);
    if (scale_opt) memcpy(scale_opt, scale, sizeof(float) * T);
    if (zero_opt) memcpy(zero_opt, zero, sizeof(float) * T);
    if (x_out_opt) memcpy(x_out_opt, xo, sizeof(uint16_t) * (size_t)T * n_out);
    if (acc_opt) memcpy(acc_opt, acc, sizeof(int32_t) * (size_t)T * N);
    if (w_reduced_opt) memcpy(w_reduced_opt, wred, sizeof(float) * N);
done:
    free(q); free(wq); free(scale); free(zero); free(xo); free(acc); free(wred); free(rfp);
    return rc;
}
