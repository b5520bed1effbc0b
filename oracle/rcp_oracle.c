/*
 * rcp_oracle.c - plain CPU oracle for the RCP W2A4 GEMV path.
 *
 * TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only tests, the smoke check and the
 * benchmark's cpu_baseline leg may call this file.  It shares no code with the
 * HIP library: it is written from the paper ("Rotate, Clip, and Partition",
 * arXiv 2502.15779) and from the written data layouts alone, takes HOST
 * pointers, and is deliberately slow and literal: every function is the plain
 * definition of what it computes, in IEEE double unless a precision is fixed.
 * Compile with -ffp-contract=off so that no multiply-add is fused.
 *
 * What pins each function (see tests/test_oracle_*.py): the Hadamard functions
 * against scipy's Sylvester matrix and the orthogonality the paper states; the
 * LDP grid against the closed forms and the paper's uniform initial point (where
 * it must reduce to the 2-bit asymmetric integer quantizer of Eqn. 1); the
 * fp16 conversions against numpy's; pack/unpack against each other; the
 * quantiser against its error bound; the GEMV against brute force and numpy
 * integer matmuls; the 3-bit variant against nearest-level brute force, the
 * integer-grid case of its printed rounding rule and the 2-bit GEMV; the 4-bit
 * KV cache against exact reproduction of integer grids, nearest-point brute
 * force and the half-step error bound, and attention over it against scipy's
 * softmax and its closed-form special cases.  No function here is "parity
 * unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define RCP_REF_OK 0
#define RCP_REF_ERR_SHAPE -2
#define RCP_REF_ERR_OVERFLOW -7

int rcp_ref_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void rcp_ref_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ------------------------------------------------------------------------
 * IEEE binary16 <-> double.  One rounding, to nearest, ties to even;
 * subnormals kept; overflow goes to infinity.
 * ---------------------------------------------------------------------- */
uint16_t rcp_ref_f64_to_f16_bits(double v)
{
    uint16_t sign = signbit(v) ? 0x8000u : 0u;
    if (isnan(v)) return (uint16_t)(sign | 0x7e00u);
    double a = fabs(v);
    if (isinf(a)) return (uint16_t)(sign | 0x7c00u);
    if (a == 0.0) return sign;
    /* Spacing of binary16 numbers near a: 2^(e-10) for a normal a in
       [2^e, 2^(e+1)), and 2^-24 below 2^-14 (the subnormal range). */
    int e;
    (void)frexp(a, &e); /* a = f * 2^e, f in [0.5, 1)  ->  a in [2^(e-1), 2^e) */
    int exp2 = e - 1;
    if (exp2 < -14) exp2 = -14;
    double ulp = ldexp(1.0, exp2 - 10);
    /* a / ulp is exact (power-of-two scaling); nearbyint rounds half to even
       in the default rounding mode. */
    double steps = nearbyint(a / ulp);
    double r = steps * ulp; /* exact */
    if (r >= 65520.0) return (uint16_t)(sign | 0x7c00u);
    /* re-read exponent: rounding may have carried into the next binade */
    if (r < ldexp(1.0, -14)) {
        return (uint16_t)(sign | (uint16_t)(r / ldexp(1.0, -24)));
    }
    (void)frexp(r, &e);
    int be = (e - 1) + 15;
    double mant = r / ldexp(1.0, e - 1) - 1.0; /* in [0,1), multiple of 2^-10 */
    return (uint16_t)(sign | (uint16_t)(be << 10) | (uint16_t)(mant * 1024.0));
}

double rcp_ref_f16_bits_to_f64(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int be = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (be == 0)
        v = ldexp((double)frac, -24);
    else if (be == 31)
        v = frac ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)frac / 1024.0, be - 15);
    return sign ? -v : v;
}

/* ------------------------------------------------------------------------
 * Hadamard matrix (Appendix, definition of the normalised Hadamard matrix):
 *   H'_1 = [1],  H'_{2n} = [[H'_n, H'_n], [H'_n, -H'_n]],  H_n = H'_n / sqrt(n).
 * ---------------------------------------------------------------------- */

/* Fill `out` (n*n int8, row-major) with H'_n by the recursion itself. */
int rcp_ref_hadamard_matrix(int n, int8_t* out)
{
    if (n < 1 || (n & (n - 1)) != 0) return RCP_REF_ERR_SHAPE;
    out[0] = 1;
    for (int s = 1; s < n; s *= 2) {
        /* the top-left s x s block holds H'_s (row stride n); extend to 2s */
        for (int i = 0; i < s; ++i)
            for (int j = 0; j < s; ++j) {
                int8_t v = out[(size_t)i * n + j];
                out[(size_t)i * n + (j + s)] = v;
                out[(size_t)(i + s) * n + j] = v;
                out[(size_t)(i + s) * n + (j + s)] = (int8_t)(-v);
            }
    }
    return RCP_REF_OK;
}

/*
 * y = R x for M tokens, fp64, dense, straight from the definition.
 *   kind 0: R = I.
 *   kind 1: R = H_K                         (K = n_wht, a power of two)
 *   kind 2: R = H_{n_wht} (x) Q, K = n_wht*m: with k = i*m + j,
 *           R[(i',j'),(i,j)] = H[i'][i] * Q[j'][j]   (Kronecker product)
 *   kind 3: R = H_{n_wht} (x) I_m, K = n_wht*m: the Hadamard matrix across n_wht heads of m
 *           channels (Section 2.1: the online factor of R_2 applied to the self-attention output)
 * Q: m x m row-major doubles (kind 2 only).
 */
int rcp_ref_rotate(const double* x, int M, int K, int kind, int n_wht, int m,
                   const double* Q, double* y)
{
    if (M < 1 || K < 1) return RCP_REF_ERR_SHAPE;
    if (kind == 0) {
        memcpy(y, x, (size_t)M * K * sizeof(double));
        return RCP_REF_OK;
    }
    if (kind == 1) {
        if (n_wht != K) return RCP_REF_ERR_SHAPE;
        m = 1;
    } else if (kind == 2) {
        if (m < 1 || (long long)n_wht * m != K || Q == NULL) return RCP_REF_ERR_SHAPE;
    } else if (kind == 3) {
        if (m < 1 || (long long)n_wht * m != K) return RCP_REF_ERR_SHAPE;
    } else
        return RCP_REF_ERR_SHAPE;
    if (n_wht < 1 || (n_wht & (n_wht - 1)) != 0) return RCP_REF_ERR_SHAPE;

    int n = n_wht;
    int8_t* Hp = (int8_t*)malloc((size_t)n * n);
    if (!Hp) return RCP_REF_ERR_SHAPE;
    rcp_ref_hadamard_matrix(n, Hp);
    const double one = 1.0;
    const double norm = 1.0 / sqrt((double)n);

    for (int t = 0; t < M; ++t) {
        const double* xt = x + (size_t)t * K;
        double* yt = y + (size_t)t * K;
#pragma omp parallel for schedule(static)
        for (int ko = 0; ko < K; ++ko) {
            int io = ko / m, jo = ko % m;
            const double* qrow = (kind == 2) ? Q + (size_t)jo * m : &one;
            double acc = 0.0;
            for (int i = 0; i < n; ++i) {
                double hij = (double)Hp[(size_t)io * n + i];
                if (kind == 3) {
                    acc += hij * xt[(size_t)i * m + jo];
                } else {
                    for (int j = 0; j < m; ++j)
                        acc += hij * qrow[j] * xt[(size_t)i * m + j];
                }
            }
            yt[ko] = acc * norm;
        }
    }
    free(Hp);
    return RCP_REF_OK;
}

/*
 * Fast Walsh-Hadamard transform in binary32, the precision the GPU kernel works
 * in.  Stage s = 1, 2, 4, ... n/2 replaces every pair (v[i], v[i+s]) whose index
 * has bit s clear by (v[i] + v[i+s], v[i] - v[i+s]); each stage is the factor
 * I (x) H'_2 (x) I of the Sylvester recursion, so the product of all stages is
 * H'_n.  Every output of a stage is one IEEE operation on two stage inputs, so
 * the result does not depend on how the work is spread over threads.  The final
 * scaling multiplies by (float)(1/sqrt(n)).
 */
int rcp_ref_fwht_f32(float* v, int n)
{
    if (n < 1 || (n & (n - 1)) != 0) return RCP_REF_ERR_SHAPE;
    for (int s = 1; s < n; s *= 2)
        for (int i = 0; i < n; ++i)
            if ((i & s) == 0) {
                float a = v[i], b = v[i + s];
                v[i] = a + b;
                v[i + s] = a - b;
            }
    float norm = (float)(1.0 / sqrt((double)n));
    for (int i = 0; i < n; ++i) v[i] = v[i] * norm;
    return RCP_REF_OK;
}

/* ------------------------------------------------------------------------
 * LDP quantisation grid and LUT for one quantisation unit (Section 4.3,
 * "Partition"; LUT equation of Section 4.4).  Inputs are binary32 values.
 *   t1 = p1/2, t_i = t_{i-1} + (p_{i-1} + p_i)/2           (quantisation grid)
 *   w0 = 0, w1 = (t1+t2)/2, w2 = (t2+t3)/2, w3 = 1        (dequantisation grid)
 *   T_i = lo + range*t_i  -> binary32
 *   L_i = lo + range*w_i  -> binary16;  L_0 = lo and L_3 = hi exactly (the
 *   paper's footnote: lo + range is the upper clip value)
 * ---------------------------------------------------------------------- */
void rcp_ref_ldp_grid(float clip_lo, float clip_hi, float p1f, float p2f, float p3f,
                      float thresholds[3], uint16_t levels[4])
{
    double lo = (double)clip_lo, hi = (double)clip_hi;
    double p1 = (double)p1f, p2 = (double)p2f, p3 = (double)p3f;
    double range = hi - lo;
    double t1 = p1 / 2.0;
    double t2 = t1 + (p1 + p2) / 2.0;
    double t3 = t2 + (p2 + p3) / 2.0;
    double w1 = (t1 + t2) / 2.0;
    double w2 = (t2 + t3) / 2.0;
    thresholds[0] = (float)(lo + range * t1);
    thresholds[1] = (float)(lo + range * t2);
    thresholds[2] = (float)(lo + range * t3);
    levels[0] = rcp_ref_f64_to_f16_bits(lo);
    levels[1] = rcp_ref_f64_to_f16_bits(lo + range * w1);
    levels[2] = rcp_ref_f64_to_f16_bits(lo + range * w2);
    levels[3] = rcp_ref_f64_to_f16_bits(hi);
}

/* Q_LDP: the number of grid points at or below w (step function u(0) = 1). */
static inline int ldp_index(float w, const float T[3])
{
    return (w >= T[0]) + (w >= T[1]) + (w >= T[2]);
}

/* Position of idx[h][k] in the packed buffer (layout in include/rcp.h, restated
 * from its text): cell (h/4, k/8) of 8 bytes; word 0 carries bit 0 of the index
 * and word 1 bit 1; inside a word the bit number is 4*(k%8) + (h%4). */
static inline void packed_position(int h, int k, int K, size_t* cell_byte, int* bit)
{
    size_t g = (size_t)(h / 4), o = (size_t)(k / 8);
    *cell_byte = 8u * (g * (size_t)(K / 8) + o);
    *bit = 4 * (k % 8) + (h % 4);
}

static inline int packed_get(const uint8_t* packed, int h, int k, int K)
{
    size_t cb;
    int bit;
    packed_position(h, k, K, &cb, &bit);
    /* little-endian words: bit b of a word is bit b%8 of its byte b/8 */
    int b0 = (packed[cb + (size_t)(bit / 8)] >> (bit % 8)) & 1;
    int b1 = (packed[cb + 4 + (size_t)(bit / 8)] >> (bit % 8)) & 1;
    return b0 + 2 * b1;
}

static inline void packed_set(uint8_t* packed, int h, int k, int K, int idx)
{
    size_t cb;
    int bit;
    packed_position(h, k, K, &cb, &bit);
    if (idx & 1) packed[cb + (size_t)(bit / 8)] |= (uint8_t)(1u << (bit % 8));
    if (idx & 2) packed[cb + 4 + (size_t)(bit / 8)] |= (uint8_t)(1u << (bit % 8));
}

/*
 * Offline export.  W: N x K binary32 (a 16-bit input is widened exactly by the
 * caller).  Writes packed (N*K/4 bytes), codebook (N*4 binary16 bit patterns)
 * and, when idx_or_null is given, the plain N x K index matrix.
 */
int rcp_ref_pack_weights(const float* W, int N, int K, const float* clip_lo,
                         const float* clip_hi, const float* part, uint8_t* packed,
                         uint16_t* codebook, uint8_t* idx_or_null)
{
    if (N < 4 || N % 4 || K < 32 || K % 32) return RCP_REF_ERR_SHAPE;
    memset(packed, 0, (size_t)N * K / 4);
#pragma omp parallel for schedule(static)
    for (int g = 0; g < N / 4; ++g) { /* a thread owns whole cells: no byte is shared */
        for (int r = 0; r < 4; ++r) {
            int h = 4 * g + r;
            float T[3];
            rcp_ref_ldp_grid(clip_lo[h], clip_hi[h], part[3 * h], part[3 * h + 1],
                             part[3 * h + 2], T, codebook + 4 * (size_t)h);
            for (int k = 0; k < K; ++k) {
                int idx = ldp_index(W[(size_t)h * K + k], T);
                packed_set(packed, h, k, K, idx);
                if (idx_or_null) idx_or_null[(size_t)h * K + k] = (uint8_t)idx;
            }
        }
    }
    return RCP_REF_OK;
}

int rcp_ref_unpack_indices(const uint8_t* packed, int N, int K, uint8_t* idx)
{
    if (N < 4 || N % 4 || K < 32 || K % 32) return RCP_REF_ERR_SHAPE;
#pragma omp parallel for schedule(static)
    for (int h = 0; h < N; ++h)
        for (int k = 0; k < K; ++k)
            idx[(size_t)h * K + k] = (uint8_t)packed_get(packed, h, k, K);
    return RCP_REF_OK;
}

/* Pack a plain index matrix (values 0..3) into the layout; used by tests that
 * start from chosen indices rather than from weights. */
int rcp_ref_pack_indices(const uint8_t* idx, int N, int K, uint8_t* packed)
{
    if (N < 4 || N % 4 || K < 32 || K % 32) return RCP_REF_ERR_SHAPE;
    memset(packed, 0, (size_t)N * K / 4);
    for (int h = 0; h < N; ++h)
        for (int k = 0; k < K; ++k) packed_set(packed, h, k, K, idx[(size_t)h * K + k] & 3);
    return RCP_REF_OK;
}

/* ------------------------------------------------------------------------
 * Per-token symmetric int4 quantiser (Appendix table "Quantization
 * configurations": activation, symmetric, per token, clipping ratio; Section
 * 4.4: X_q is 1 x C/2 int8 holding two int4, S an fp16 scalar).
 * The rounding decision is taken in binary32, the precision of the GPU kernel:
 *     a = max|y|,  S = fp16((ratio * a) / 7)   [S = 1 if that is 0; capped at 65504]
 *     q = clamp(rint(y / S), -8, 7)            [rint = round half to even]
 * ---------------------------------------------------------------------- */
static inline int8_t decode_low_nibble(uint8_t byte)
{
    /* shift the nibble's sign bit to the top, then arithmetic shift back
       (Appendix, "Online Dequantization and Vectorization") */
    return (int8_t)((int8_t)(byte << 4) >> 4);
}
static inline int8_t decode_high_nibble(uint8_t byte) { return (int8_t)((int8_t)byte >> 4); }

int rcp_ref_quantize_act(const float* y, int M, int K, float clip_ratio, uint8_t* xq,
                         uint16_t* scale_bits, int8_t* q_or_null)
{
    if (M < 1 || K < 2 || K % 2) return RCP_REF_ERR_SHAPE;
    for (int t = 0; t < M; ++t) {
        const float* yt = y + (size_t)t * K;
        float a = 0.0f;
        for (int k = 0; k < K; ++k) {
            float v = fabsf(yt[k]);
            if (v > a) a = v;
        }
        float raw = (clip_ratio * a) / 7.0f;
        uint16_t sb = rcp_ref_f64_to_f16_bits((double)raw);
        if ((sb & 0x7fffu) == 0) sb = 0x3c00u;      /* 1.0 */
        if ((sb & 0x7fffu) >= 0x7c00u) sb = 0x7bffu; /* 65504 */
        scale_bits[t] = sb;
        float s = (float)rcp_ref_f16_bits_to_f64(sb);
        for (int k = 0; k < K; k += 2) {
            int q[2];
            for (int e = 0; e < 2; ++e) {
                float r = rintf(yt[k + e] / s);
                if (r > 7.0f) r = 7.0f;
                if (r < -8.0f) r = -8.0f;
                q[e] = (int)r;
                if (q_or_null) q_or_null[(size_t)t * K + k + e] = (int8_t)q[e];
            }
            xq[(size_t)t * (K / 2) + k / 2] = (uint8_t)((q[0] & 0xF) | ((q[1] & 0xF) << 4));
        }
    }
    return RCP_REF_OK;
}

int rcp_ref_unpack_act(const uint8_t* xq, int M, int K, int8_t* q)
{
    if (M < 1 || K < 2 || K % 2) return RCP_REF_ERR_SHAPE;
    for (size_t b = 0; b < (size_t)M * (K / 2); ++b) {
        q[2 * b] = decode_low_nibble(xq[b]);
        q[2 * b + 1] = decode_high_nibble(xq[b]);
    }
    return RCP_REF_OK;
}

/* ------------------------------------------------------------------------
 * W2A4 GEMV (Section 4.4).
 *   P[t][h][l] = sum_{k: idx[h][k]=l} q[t][k]
 *   O[t][h]    = S[t] * sum_l LUT[h][l] * P[t][h][l]          (binary64)
 * out: M x N doubles.  P_or_null: int32 [M][N][4].
 * ---------------------------------------------------------------------- */
int rcp_ref_w2a4_gemv(const uint8_t* packed, const uint16_t* codebook, int N, int K,
                      const uint8_t* xq, const uint16_t* scale_bits, int M, double* out,
                      int32_t* P_or_null)
{
    if (N < 4 || N % 4 || K < 32 || K % 32 || M < 1) return RCP_REF_ERR_SHAPE;
    int8_t* q = (int8_t*)malloc((size_t)M * K);
    if (!q) return RCP_REF_ERR_SHAPE;
    rcp_ref_unpack_act(xq, M, K, q);
    int overflow = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow)
    for (int h = 0; h < N; ++h) {
        double lut[4];
        for (int l = 0; l < 4; ++l) lut[l] = rcp_ref_f16_bits_to_f64(codebook[4 * (size_t)h + l]);
        for (int t = 0; t < M; ++t) {
            int64_t P[4] = {0, 0, 0, 0};
            for (int k = 0; k < K; ++k) P[packed_get(packed, h, k, K)] += q[(size_t)t * K + k];
            double acc = 0.0;
            for (int l = 0; l < 4; ++l) {
                if (P[l] > INT32_MAX || P[l] < INT32_MIN) overflow |= 1;
                if (P_or_null) P_or_null[((size_t)t * N + h) * 4 + l] = (int32_t)P[l];
                acc += lut[l] * (double)P[l];
            }
            out[(size_t)t * N + h] = rcp_ref_f16_bits_to_f64(scale_bits[t]) * acc;
        }
    }
    free(q);
    return overflow ? RCP_REF_ERR_OVERFLOW : RCP_REF_OK;
}

/* The paper's own statement of the same product: dequantise every weight through
 * the LUT, dequantise every activation as S*q, and take the dot product. */
int rcp_ref_dequant_dot(const uint8_t* packed, const uint16_t* codebook, int N, int K,
                        const uint8_t* xq, const uint16_t* scale_bits, int M, double* out)
{
    if (N < 4 || N % 4 || K < 32 || K % 32 || M < 1) return RCP_REF_ERR_SHAPE;
    int8_t* q = (int8_t*)malloc((size_t)M * K);
    if (!q) return RCP_REF_ERR_SHAPE;
    rcp_ref_unpack_act(xq, M, K, q);
#pragma omp parallel for schedule(static)
    for (int h = 0; h < N; ++h)
        for (int t = 0; t < M; ++t) {
            double s = rcp_ref_f16_bits_to_f64(scale_bits[t]);
            double acc = 0.0;
            for (int k = 0; k < K; ++k) {
                double w = rcp_ref_f16_bits_to_f64(codebook[4 * (size_t)h + packed_get(packed, h, k, K)]);
                acc += w * (s * (double)q[(size_t)t * K + k]);
            }
            out[(size_t)t * N + h] = acc;
        }
    free(q);
    return RCP_REF_OK;
}

/* ------------------------------------------------------------------------
 * Weight-only variant (the W2-only decode measurement of the paper's inference-latency
 * section: non-uniform dequantisation of the weights merged with a 16-bit linear layer):
 *   O[t][h] = sum_k LUT[h][idx[h][k]] * x[t][k]                   (binary64)
 * x: M x K doubles holding the exact values of the 16-bit (or 32-bit) activations.
 * ---------------------------------------------------------------------- */
int rcp_ref_w2a16_gemv(const uint8_t* packed, const uint16_t* codebook, int N, int K, const double* x, int M,
                       double* out)
{
    if (N < 4 || N % 4 || K < 32 || K % 32 || M < 1) return RCP_REF_ERR_SHAPE;
#pragma omp parallel for schedule(static)
    for (int h = 0; h < N; ++h) {
        double lut[4];
        for (int l = 0; l < 4; ++l) lut[l] = rcp_ref_f16_bits_to_f64(codebook[4 * (size_t)h + l]);
        for (int t = 0; t < M; ++t) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k) acc += lut[packed_get(packed, h, k, K)] * x[(size_t)t * K + k];
            out[(size_t)t * N + h] = acc;
        }
    }
    return RCP_REF_OK;
}

/* ------------------------------------------------------------------------
 * Group-wise quantisation units (Appendix table "Quantization configurations": weights are
 * quantised in groups of 128 input channels; Section 4.4: the LUT is H x N*4 with N groups
 * per channel).  Every (row, group) has its own clip range, partition and 4-entry LUT.
 *
 * Grouped packed layout (restated from include/rcp.h): the same 8-byte cells as above, but
 * inside a group of four rows the 16-byte units (two cells = 16 columns) are stored in
 * "lane-major" order.  With NG = K/128 groups, group g belongs to round g/32 and lane g%32;
 * a round holds R = min(32, NG - 32*(g/32)) groups; unit i (0..7) of group g, i.e. columns
 * 128g + 16i .. 128g + 16i + 15, sits at unit position 256*(g/32) + i*R + g%32.
 * Grouped LUT layout: fp16 [N/4][NG][4 rows][4 levels].
 * ---------------------------------------------------------------------- */
#define RCP_REF_GROUP 128

static inline size_t grouped_cell_byte(int h, int k, int K)
{
    int NG = K / RCP_REF_GROUP;
    int u = k / 16, g = u / 8, i = u % 8;
    int round = g / 32, lane = g % 32;
    int R = NG - 32 * round;
    if (R > 32) R = 32;
    size_t pos = (size_t)256 * round + (size_t)i * R + lane;
    size_t rowgroup_base = (size_t)(h / 4) * (size_t)(K / 16) * 16u;
    return rowgroup_base + pos * 16u + (size_t)((k % 16) / 8) * 8u;
}

static inline int grouped_get(const uint8_t* packed, int h, int k, int K)
{
    size_t cb = grouped_cell_byte(h, k, K);
    int bit = 4 * (k % 8) + (h % 4);
    int b0 = (packed[cb + (size_t)(bit / 8)] >> (bit % 8)) & 1;
    int b1 = (packed[cb + 4 + (size_t)(bit / 8)] >> (bit % 8)) & 1;
    return b0 + 2 * b1;
}

static inline void grouped_set(uint8_t* packed, int h, int k, int K, int idx)
{
    size_t cb = grouped_cell_byte(h, k, K);
    int bit = 4 * (k % 8) + (h % 4);
    if (idx & 1) packed[cb + (size_t)(bit / 8)] |= (uint8_t)(1u << (bit % 8));
    if (idx & 2) packed[cb + 4 + (size_t)(bit / 8)] |= (uint8_t)(1u << (bit % 8));
}

static inline size_t grouped_lut_index(int h, int g, int NG) /* half-word index of level 0 */
{
    return (((size_t)(h / 4) * NG + g) * 4u + (size_t)(h % 4)) * 4u;
}

static int grouped_shape_ok(int N, int K, int group)
{
    return group == RCP_REF_GROUP && N >= 4 && N % 4 == 0 && K >= group && K % group == 0;
}

/* clip_lo, clip_hi: [N][NG]; part: [N][NG][3]; codebook: N*NG*4 half-words in the grouped
 * LUT layout; idx_or_null: plain N x K indices. */
int rcp_ref_pack_weights_grouped(const float* W, int N, int K, int group, const float* clip_lo,
                                 const float* clip_hi, const float* part, uint8_t* packed,
                                 uint16_t* codebook, uint8_t* idx_or_null)
{
    if (!grouped_shape_ok(N, K, group)) return RCP_REF_ERR_SHAPE;
    int NG = K / group;
    memset(packed, 0, (size_t)N * K / 4);
#pragma omp parallel for schedule(static)
    for (int g4 = 0; g4 < N / 4; ++g4)
        for (int r = 0; r < 4; ++r) {
            int h = 4 * g4 + r;
            for (int g = 0; g < NG; ++g) {
                float T[3];
                size_t q = (size_t)h * NG + g;
                rcp_ref_ldp_grid(clip_lo[q], clip_hi[q], part[3 * q], part[3 * q + 1], part[3 * q + 2], T,
                                 codebook + grouped_lut_index(h, g, NG));
                for (int k = g * group; k < (g + 1) * group; ++k) {
                    int idx = ldp_index(W[(size_t)h * K + k], T);
                    grouped_set(packed, h, k, K, idx);
                    if (idx_or_null) idx_or_null[(size_t)h * K + k] = (uint8_t)idx;
                }
            }
        }
    return RCP_REF_OK;
}

int rcp_ref_pack_indices_grouped(const uint8_t* idx, int N, int K, int group, uint8_t* packed)
{
    if (!grouped_shape_ok(N, K, group)) return RCP_REF_ERR_SHAPE;
    memset(packed, 0, (size_t)N * K / 4);
    for (int h = 0; h < N; ++h)
        for (int k = 0; k < K; ++k) grouped_set(packed, h, k, K, idx[(size_t)h * K + k] & 3);
    return RCP_REF_OK;
}

int rcp_ref_unpack_indices_grouped(const uint8_t* packed, int N, int K, int group, uint8_t* idx)
{
    if (!grouped_shape_ok(N, K, group)) return RCP_REF_ERR_SHAPE;
#pragma omp parallel for schedule(static)
    for (int h = 0; h < N; ++h)
        for (int k = 0; k < K; ++k) idx[(size_t)h * K + k] = (uint8_t)grouped_get(packed, h, k, K);
    return RCP_REF_OK;
}

/* O[t][h] = S[t] * sum_g sum_l LUT[h][g][l] * P[t][h][g][l],  P[t][h][g][l] = sum of q[t] over the
 * columns of group g whose index is l.  M tokens.  out: M x N; P_or_null: int32 [M][N][NG][4]. */
int rcp_ref_w2a4_gemv_grouped(const uint8_t* packed, const uint16_t* codebook, int N, int K, int group,
                              const uint8_t* xq, const uint16_t* scale_bits, int M, double* out,
                              int32_t* P_or_null)
{
    if (!grouped_shape_ok(N, K, group) || M < 1) return RCP_REF_ERR_SHAPE;
    int NG = K / group;
    int8_t* q = (int8_t*)malloc((size_t)M * K);
    if (!q) return RCP_REF_ERR_SHAPE;
    rcp_ref_unpack_act(xq, M, K, q);
#pragma omp parallel for schedule(static)
    for (int h = 0; h < N; ++h)
        for (int t = 0; t < M; ++t) {
            double acc = 0.0;
            for (int g = 0; g < NG; ++g) {
                int64_t P[4] = {0, 0, 0, 0};
                for (int k = g * group; k < (g + 1) * group; ++k)
                    P[grouped_get(packed, h, k, K)] += q[(size_t)t * K + k];
                const uint16_t* lut = codebook + grouped_lut_index(h, g, NG);
                for (int l = 0; l < 4; ++l) {
                    if (P_or_null) P_or_null[(((size_t)t * N + h) * NG + g) * 4 + l] = (int32_t)P[l];
                    acc += rcp_ref_f16_bits_to_f64(lut[l]) * (double)P[l];
                }
            }
            out[(size_t)t * N + h] = rcp_ref_f16_bits_to_f64(scale_bits[t]) * acc;
        }
    free(q);
    return RCP_REF_OK;
}

/* ------------------------------------------------------------------------
 * 3-bit variant: LDP applied to the asymmetric normal-float format (Section
 * 4.3, paragraph "Application of LDP on NF3 format").  The clip values lo, hi
 * (the learnt sigma(beta)*min(W), sigma(gamma)*max(W)) and one partition
 * fraction p = sigma(s_1) give per quantisation unit
 *     c = lo + (hi - lo) * p,   s_neg = |c - lo|,   s_pos = |hi - c|;
 * a weight above c is divided by s_pos, any other by s_neg, and the result is
 * rounded to the format's grid; dequantisation multiplies the scale back and
 * adds c.  The paper does not print the grid (it is the cited format's): here
 * it is an INPUT, eight ascending binary32 values.  With that,
 *     L_j = c + (g_j < 0 ? s_neg : s_pos) * g_j            (the eight levels, binary16)
 *     T_j = (L_{j-1} + L_j) / 2,  j = 1..7                  (binary32)
 *     idx = number of T_j at or below w                      (u(0) = 1, as for 2 bits)
 * When the grid holds 0 the level there is c itself, and counting thresholds is
 * the same as rounding (w - c)/s to the nearest grid value on w's own side.
 * ---------------------------------------------------------------------- */
void rcp_ref_w3_grid(float clip_lo, float clip_hi, float p, const float grid[8], float thresholds[7],
                     uint16_t levels[8])
{
    double lo = (double)clip_lo, hi = (double)clip_hi;
    double c = lo + (hi - lo) * (double)p;
    double s_neg = fabs(c - lo), s_pos = fabs(hi - c);
    double L[8];
    for (int j = 0; j < 8; ++j) {
        double g = (double)grid[j];
        L[j] = c + (g < 0.0 ? s_neg : s_pos) * g;
        levels[j] = rcp_ref_f64_to_f16_bits(L[j]);
    }
    for (int j = 1; j < 8; ++j) thresholds[j - 1] = (float)((L[j - 1] + L[j]) / 2.0);
}

static inline int w3_index(float w, const float T[7])
{
    int idx = 0;
    for (int j = 0; j < 7; ++j) idx += (w >= T[j]);
    return idx;
}

/* Position of bit p of idx[h][k] in the 3-bit packed buffer (layout in include/rcp.h,
 * restated from its text).  A row group (4 rows) is K/32 units of 4 rows x 32 columns;
 * units go in blocks of 64; a block of R = min(64, units left) units stores plane 0 of
 * all its units, then plane 1, then plane 2, 16 bytes per unit and plane: four
 * little-endian words, word k%32/8, bit 4*(k%8) + h%4. */
static inline void w3_position(int h, int k, int p, int K, size_t* byte, int* bit)
{
    int U = K / 32, u = k / 32, j = u / 64;
    int R = U - 64 * j < 64 ? U - 64 * j : 64;
    size_t group_base = (size_t)(h / 4) * (size_t)U * 48u;
    size_t unit16 = group_base + 3072u * (size_t)j + 16u * (size_t)R * (size_t)p + 16u * (size_t)(u % 64);
    int word = (k % 32) / 8, b = 4 * (k % 8) + (h % 4);
    *byte = unit16 + 4u * (size_t)word + (size_t)(b / 8);
    *bit = b % 8;
}

static inline int w3_get(const uint8_t* packed, int h, int k, int K)
{
    int idx = 0;
    for (int p = 0; p < 3; ++p) {
        size_t by;
        int bit;
        w3_position(h, k, p, K, &by, &bit);
        idx |= ((packed[by] >> bit) & 1) << p;
    }
    return idx;
}

static inline void w3_set(uint8_t* packed, int h, int k, int K, int idx)
{
    for (int p = 0; p < 3; ++p) {
        size_t by;
        int bit;
        w3_position(h, k, p, K, &by, &bit);
        if ((idx >> p) & 1) packed[by] |= (uint8_t)(1u << bit);
    }
}

/* W: N x K binary32; clip_lo, clip_hi, frac: N each; grid: 8.  Writes packed (3*N*K/8
 * bytes), codebook (N*8 binary16 bit patterns) and optionally the plain indices. */
int rcp_ref_pack_weights_w3(const float* W, int N, int K, const float* clip_lo, const float* clip_hi,
                            const float* frac, const float* grid, uint8_t* packed,
                            uint16_t* codebook, uint8_t* idx_or_null)
{
    if (N < 4 || N % 4 || K < 32 || K % 32) return RCP_REF_ERR_SHAPE;
    memset(packed, 0, (size_t)N * K / 8 * 3);
#pragma omp parallel for schedule(static)
    for (int g = 0; g < N / 4; ++g) {
        for (int r = 0; r < 4; ++r) {
            int h = 4 * g + r;
            float T[7];
            rcp_ref_w3_grid(clip_lo[h], clip_hi[h], frac[h], grid, T, codebook + 8 * (size_t)h);
            for (int k = 0; k < K; ++k) {
                int idx = w3_index(W[(size_t)h * K + k], T);
                w3_set(packed, h, k, K, idx);
                if (idx_or_null) idx_or_null[(size_t)h * K + k] = (uint8_t)idx;
            }
        }
    }
    return RCP_REF_OK;
}

int rcp_ref_unpack_indices_w3(const uint8_t* packed, int N, int K, uint8_t* idx)
{
    if (N < 4 || N % 4 || K < 32 || K % 32) return RCP_REF_ERR_SHAPE;
#pragma omp parallel for schedule(static)
    for (int h = 0; h < N; ++h)
        for (int k = 0; k < K; ++k) idx[(size_t)h * K + k] = (uint8_t)w3_get(packed, h, k, K);
    return RCP_REF_OK;
}

int rcp_ref_pack_indices_w3(const uint8_t* idx, int N, int K, uint8_t* packed)
{
    if (N < 4 || N % 4 || K < 32 || K % 32) return RCP_REF_ERR_SHAPE;
    memset(packed, 0, (size_t)N * K / 8 * 3);
    for (int h = 0; h < N; ++h)
        for (int k = 0; k < K; ++k) w3_set(packed, h, k, K, idx[(size_t)h * K + k] & 7);
    return RCP_REF_OK;
}

/* The GEMV of Section 4.4 with an eight-entry LUT per output channel:
 *   P[h][l] = sum over k with idx[h][k] = l of q[k]   (exact integers)
 *   O[h]    = S * sum_l LUT[h][l] * P[h][l]           (binary64)
 * P_or_null: int32 [N][8]. */
int rcp_ref_w3a4_gemv(const uint8_t* packed, const uint16_t* codebook, int N, int K, const uint8_t* xq,
                      const uint16_t* scale_bits, double* out, int32_t* P_or_null)
{
    if (N < 4 || N % 4 || K < 32 || K % 32) return RCP_REF_ERR_SHAPE;
    int8_t* q = (int8_t*)malloc((size_t)K);
    if (!q) return RCP_REF_ERR_SHAPE;
    rcp_ref_unpack_act(xq, 1, K, q);
    double S = rcp_ref_f16_bits_to_f64(scale_bits[0]);
#pragma omp parallel for schedule(static)
    for (int h = 0; h < N; ++h) {
        int64_t P[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int k = 0; k < K; ++k) P[w3_get(packed, h, k, K)] += q[k];
        double acc = 0.0;
        for (int l = 0; l < 8; ++l) {
            if (P_or_null) P_or_null[(size_t)h * 8 + l] = (int32_t)P[l];
            acc += rcp_ref_f16_bits_to_f64(codebook[8 * (size_t)h + l]) * (double)P[l];
        }
        out[h] = S * acc;
    }
    free(q);
    return RCP_REF_OK;
}

/* ------------------------------------------------------------------------
 * 4-bit KV cache (Appendix table of quantisation configurations: asymmetric,
 * groups of 128 = one head vector, clipping ratio 0.95; quantiser of Eqn. 1
 * with N = 4) and one-token attention over it (Section 2.1: R3 rotates Q and
 * K so that the cache can be compressed without changing attention outputs).
 *
 * Cache of one tensor (K or V) of one layer, HEAD_DIM = 128:
 *   codes  uint8 [H][S_max][64]   element j of a head vector in byte j / 2,
 *                                 bits 4 * (j % 2) .. 4 * (j % 2) + 3
 *   params       [H][S_max][4 B]  bytes 0..1 the binary16 step size s,
 *                                 bytes 2..3 the int16 zero point z
 * The rounding decisions are taken in binary32, the precision of the GPU
 * kernel:
 *   lo = ratio * min(x), hi = ratio * max(x), s = fp16((hi - lo) / 15)
 *       [s = 1 if that is 0; capped at 65504]
 *   z = -rint(lo / s)                       [clamped to the int16 range]
 *   code = clamp(rint(x / s) + z, 0, 15)    [rint = round half to even]
 * and a code stands for the value s * (code - z).  The zero point is taken
 * from min / s (the printed equation divides the minimum by the range h, which
 * would make z one of -1, 0, 1 whatever the data; s is what makes the codes of
 * the minimum and the maximum land on 0 and 15).
 * ---------------------------------------------------------------------- */
#define KV_D 128

static inline size_t kv_code_byte(int h, int t, int j, int S_max)
{
    return ((size_t)h * S_max + t) * (KV_D / 2) + (size_t)(j / 2);
}
static inline size_t kv_param_byte(int h, int t, int S_max) { return ((size_t)h * S_max + t) * 4; }

/* x: [n_tokens][H][128] binary32; writes tokens pos .. pos + n_tokens - 1.  rotate != 0: every head
 * vector first goes through the normalised order-128 Hadamard transform in binary32 (R3 of Section
 * 2.1 on the keys; the butterflies of rcp_ref_fwht_f32). */
int rcp_ref_kv4_append(const float* x, int n_tokens, int H, int S_max, int pos, int rotate, float clip_ratio,
                       uint8_t* codes, uint8_t* params)
{
    if (n_tokens < 0 || H < 1 || S_max < 1 || pos < 0 || pos + n_tokens > S_max) return RCP_REF_ERR_SHAPE;
    for (int i = 0; i < n_tokens; ++i)
        for (int h = 0; h < H; ++h) {
            float v[KV_D];
            memcpy(v, x + ((size_t)i * H + h) * KV_D, sizeof(v));
            if (rotate) rcp_ref_fwht_f32(v, KV_D);
            float lo = v[0], hi = v[0];
            for (int j = 1; j < KV_D; ++j) {
                if (v[j] < lo) lo = v[j];
                if (v[j] > hi) hi = v[j];
            }
            float lo_c = clip_ratio * lo, hi_c = clip_ratio * hi;
            float range = hi_c - lo_c;
            float raw = range / 15.0f;
            uint16_t sb = rcp_ref_f64_to_f16_bits((double)raw);
            if ((sb & 0x7fffu) == 0) sb = 0x3c00u;       /* 1.0 */
            if ((sb & 0x7fffu) >= 0x7c00u) sb = 0x7bffu; /* 65504 */
            float s = (float)rcp_ref_f16_bits_to_f64(sb);
            float zf = -rintf(lo_c / s);
            if (zf > 32767.0f) zf = 32767.0f;
            if (zf < -32768.0f) zf = -32768.0f;
            int16_t z = (int16_t)zf;
            zf = (float)z; /* drops the sign of a negative zero */
            const int t = pos + i;
            uint8_t* pp = params + kv_param_byte(h, t, S_max);
            pp[0] = (uint8_t)(sb & 0xff);
            pp[1] = (uint8_t)(sb >> 8);
            pp[2] = (uint8_t)((uint16_t)z & 0xff);
            pp[3] = (uint8_t)((uint16_t)z >> 8);
            for (int j = 0; j < KV_D; ++j) {
                float r = rintf(v[j] / s) + zf;
                if (r > 15.0f) r = 15.0f;
                if (r < 0.0f) r = 0.0f;
                uint8_t c = (uint8_t)r;
                uint8_t* b = codes + kv_code_byte(h, t, j, S_max);
                if (j % 2 == 0) *b = (uint8_t)((*b & 0xf0u) | c);
                else *b = (uint8_t)((*b & 0x0fu) | (c << 4));
            }
        }
    return RCP_REF_OK;
}

static inline double kv_value(const uint8_t* codes, const uint8_t* params, int h, int t, int j, int S_max)
{
    const uint8_t* pp = params + kv_param_byte(h, t, S_max);
    double s = rcp_ref_f16_bits_to_f64((uint16_t)(pp[0] | (pp[1] << 8)));
    int z = (int16_t)(uint16_t)(pp[2] | (pp[3] << 8));
    uint8_t b = codes[kv_code_byte(h, t, j, S_max)];
    int c = (j % 2 == 0) ? (b & 0xf) : (b >> 4);
    return s * (double)(c - z);
}

/* out: [n_tokens][H][128] double, the values the codes stand for */
int rcp_ref_kv4_dequant(const uint8_t* codes, const uint8_t* params, int H, int S_max, int pos, int n_tokens,
                        double* out)
{
    if (n_tokens < 0 || H < 1 || S_max < 1 || pos < 0 || pos + n_tokens > S_max) return RCP_REF_ERR_SHAPE;
    for (int i = 0; i < n_tokens; ++i)
        for (int h = 0; h < H; ++h)
            for (int j = 0; j < KV_D; ++j)
                out[((size_t)i * H + h) * KV_D + j] = kv_value(codes, params, h, pos + i, j, S_max);
    return RCP_REF_OK;
}

/* One query token against the first S cached tokens.  q, out: [H_q][128] double.  Query head
 * h reads cache head h / (H_q / H_kv).  out_h = sum_t softmax_t(scale * q_h . K_t) * V_t. */
int rcp_ref_kv4_attn_decode(const double* q, int H_q, int H_kv, int S_max, int S, const uint8_t* k_codes,
                            const uint8_t* k_params, const uint8_t* v_codes, const uint8_t* v_params,
                            double softmax_scale, double* out)
{
    if (H_q < 1 || H_kv < 1 || H_q % H_kv != 0 || S < 1 || S > S_max) return RCP_REF_ERR_SHAPE;
    const int rep = H_q / H_kv;
    int rc = RCP_REF_OK;
#pragma omp parallel for schedule(static)
    for (int h = 0; h < H_q; ++h) {
        const int hk = h / rep;
        double* score = (double*)malloc((size_t)S * sizeof(double));
        if (!score) {
            rc = RCP_REF_ERR_OVERFLOW;
            continue;
        }
        double top = -INFINITY;
        for (int t = 0; t < S; ++t) {
            double acc = 0.0;
            for (int j = 0; j < KV_D; ++j) acc += q[(size_t)h * KV_D + j] * kv_value(k_codes, k_params, hk, t, j, S_max);
            score[t] = softmax_scale * acc;
            if (score[t] > top) top = score[t];
        }
        double denom = 0.0;
        for (int t = 0; t < S; ++t) {
            score[t] = exp(score[t] - top);
            denom += score[t];
        }
        for (int j = 0; j < KV_D; ++j) {
            double acc = 0.0;
            for (int t = 0; t < S; ++t) acc += score[t] * kv_value(v_codes, v_params, hk, t, j, S_max);
            out[(size_t)h * KV_D + j] = acc / denom;
        }
        free(score);
    }
    return rc;
}
