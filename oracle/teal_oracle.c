/*
 * CPU oracle for the TEAL decode path: magnitude thresholding of a hidden
 * state followed by the matrix-vector product over the thresholded state.
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists to check the GPU library and to be
 * timed as a CPU baseline.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the product never does.  It shares no code,
 * header, table or helper with the GPU library.
 *
 * The method computes exactly (up to rounding order) a result with a plain
 * definition, so the oracle is that definition written out in fp64:
 *
 *   Definition 1 (Section 4.2):  s_t(x)_i = 0 if |x_i| <= t, else x_i.
 *   Layer forward (Section 4.2): Y = s_t(x) W^T, W in R^{n x m}, x in R^m
 *                                (orientation as in Section 3).
 *   Kernel contract (Section 4.4): mask s = [|x| > t]; result (x . s) W^T.
 *
 * The product loop is dense: it multiplies by the explicit zeros and knows
 * nothing about skipping channels, compaction, tiling or split-K.
 *
 * Storage formats are decoded from their bit patterns here (IEEE 754
 * binary16 for x and the scales; bfloat16 = the upper 16 bits of a binary32
 * for W), so that no rounding happens anywhere before the fp64 arithmetic.
 *
 * Pins (tests/test_oracle_*.py): decoders against numpy/torch on all 65536
 * patterns; mask against brute-force enumeration incl. ties; t = 0 against
 * a dense numpy fp64 product; general t against the dense product on an
 * explicitly zeroed x; exact rational arithmetic on tiny shapes; measured
 * sparsity against the order statistic that chose t; the closed-form
 * relative error of Theorem A.1; the batched criterion of Section 5.4.4
 * against exact rational arithmetic, its reduction to Definition 1 at batch
 * size 1 and on a batch of identical rows, and a dense numpy product; the
 * binary32 arithmetic of the MLP intermediate against the fp64 formula and
 * the binary16 rounding against numpy on every boundary case.  The int4 nibble order and the scale
 * indexing of the quantised variants are conventions of this build, not of
 * the paper (Section 5.3 only names the bit widths): for those two layout
 * conventions parity is unpinned by the paper and pinned only by hand-built
 * single-entry matrices.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- storage formats ---------------------------------------------------- */

/* IEEE 754 binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
double oracle_f16_bits_to_f64(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int f = h & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);               /* subnormal: f * 2^-10 * 2^-14 */
    else if (e == 0x1F)
        v = f ? (double)NAN : (double)INFINITY;
    else
        v = ldexp((double)(0x400 + f), e - 25);  /* (1 + f/1024) * 2^(e-15) */
    return sign ? -v : v;
}

/* bfloat16: 1 sign, 8 exponent (bias 127), 7 fraction bits. */
double oracle_bf16_bits_to_f64(uint16_t b)
{
    int sign = (b >> 15) & 1;
    int e = (b >> 7) & 0xFF;
    int f = b & 0x7F;
    double v;
    if (e == 0)
        v = ldexp((double)f, -133);              /* subnormal: f * 2^-7 * 2^-126 */
    else if (e == 0xFF)
        v = f ? (double)NAN : (double)INFINITY;
    else
        v = ldexp((double)(0x80 + f), e - 134);  /* (1 + f/128) * 2^(e-127) */
    return sign ? -v : v;
}

/* ---- Definition 1 ------------------------------------------------------- */

/*
 * xs[i] = s_t(x)_i in fp64; mask[i] = 1 where the entry is kept (|x_i| > t,
 * strictly: an entry equal to the threshold is zeroed); idx = ascending list
 * of kept positions; returns their number.  NaN compares false and is
 * dropped.  Any of xs / mask / idx may be NULL.
 */
int32_t oracle_sparsify(const uint16_t *x_f16, int32_t m, float t,
                        double *xs, uint8_t *mask, int32_t *idx)
{
    const double td = (double)t;
    int32_t count = 0;
    for (int32_t i = 0; i < m; ++i) {
        double xd = oracle_f16_bits_to_f64(x_f16[i]);
        int keep = fabs(xd) > td;
        if (xs) xs[i] = keep ? xd : 0.0;
        if (mask) mask[i] = (uint8_t)keep;
        if (keep) {
            if (idx) idx[count] = i;
            ++count;
        }
    }
    return count;
}

/* ---- Y = s_t(x) W^T ----------------------------------------------------- */

/*
 * W is canonical: n rows (output channels) of m bf16 values (input channels),
 * row-major.  xs is the already thresholded state in fp64.  y[j] = sum_i
 * xs[i] * W[j][i], summed in index order.
 */
static void dense_rows_bf16(const uint16_t *W_bf16, const double *xs,
                            double *y, int32_t m, int32_t n)
{
#pragma omp parallel for schedule(static)
    for (int32_t j = 0; j < n; ++j) {
        const uint16_t *row = W_bf16 + (size_t)j * (size_t)m;
        double acc = 0.0;
        for (int32_t i = 0; i < m; ++i)
            acc += xs[i] * oracle_bf16_bits_to_f64(row[i]);
        y[j] = acc;
    }
}

/* scratch_xs: caller-provided m doubles. Returns the number of kept entries. */
int32_t oracle_sparse_gemv_bf16(const uint16_t *W_bf16, const uint16_t *x_f16,
                                float t, double *y, int32_t m, int32_t n,
                                double *scratch_xs)
{
    int32_t count = oracle_sparsify(x_f16, m, t, scratch_xs, NULL, NULL);
    dense_rows_bf16(W_bf16, scratch_xs, y, m, n);
    return count;
}

/* Selected output channels only: y[r] = sum_i xs[i] * W[rows[r]][i]. */
int32_t oracle_sparse_gemv_bf16_rows(const uint16_t *W_bf16,
                                     const uint16_t *x_f16, float t,
                                     const int32_t *rows, int32_t nrows,
                                     double *y, int32_t m, int32_t n,
                                     double *scratch_xs)
{
    int32_t count = oracle_sparsify(x_f16, m, t, scratch_xs, NULL, NULL);
    for (int32_t r = 0; r < nrows; ++r) {
        int32_t j = rows[r];
        if (j < 0 || j >= n) { y[r] = (double)NAN; continue; }
        const uint16_t *row = W_bf16 + (size_t)j * (size_t)m;
        double acc = 0.0;
        for (int32_t i = 0; i < m; ++i)
            acc += scratch_xs[i] * oracle_bf16_bits_to_f64(row[i]);
        y[r] = acc;
    }
    return count;
}

/*
 * 8-bit weights (Section 5.3, channel-wise): the stored arrays are
 * q[m][n] (input-channel-major int8) and scale[n] (fp16, one per output
 * channel); they DEFINE W[j][i] = q[i][j] * scale[j].
 */
int32_t oracle_sparse_gemv_w8(const int8_t *q, const uint16_t *scale_f16,
                              const uint16_t *x_f16, float t, double *y,
                              int32_t m, int32_t n, double *scratch_xs)
{
    int32_t count = oracle_sparsify(x_f16, m, t, scratch_xs, NULL, NULL);
#pragma omp parallel for schedule(static)
    for (int32_t j = 0; j < n; ++j) {
        double s = oracle_f16_bits_to_f64(scale_f16[j]);
        double acc = 0.0;
        for (int32_t i = 0; i < m; ++i) {
            double w = (double)q[(size_t)i * (size_t)n + (size_t)j] * s;
            acc += scratch_xs[i] * w;
        }
        y[j] = acc;
    }
    return count;
}

/*
 * 4-bit weights with group scales: q is [m][n/2] bytes, two two's-complement
 * nibbles per byte along the output axis (low nibble = even j); scale is
 * fp16 [m/group][n].  They DEFINE W[j][i] = nibble(i, j) * scale[i/group][j].
 */
static int nibble_value(const uint8_t *q, int32_t n, int32_t i, int32_t j)
{
    uint8_t byte = q[(size_t)i * (size_t)(n / 2) + (size_t)(j / 2)];
    int v = (j & 1) ? (byte >> 4) : (byte & 0x0F);
    return v >= 8 ? v - 16 : v;
}

int32_t oracle_sparse_gemv_w4(const uint8_t *q, const uint16_t *scale_f16,
                              int32_t group, const uint16_t *x_f16, float t,
                              double *y, int32_t m, int32_t n,
                              double *scratch_xs)
{
    int32_t count = oracle_sparsify(x_f16, m, t, scratch_xs, NULL, NULL);
#pragma omp parallel for schedule(static)
    for (int32_t j = 0; j < n; ++j) {
        double acc = 0.0;
        for (int32_t i = 0; i < m; ++i) {
            double s = oracle_f16_bits_to_f64(
                scale_f16[(size_t)(i / group) * (size_t)n + (size_t)j]);
            double w = (double)nibble_value(q, n, i, j) * s;
            acc += scratch_xs[i] * w;
        }
        y[j] = acc;
    }
    return count;
}

/* ---- batched sparsification (Section 5.4.4) ------------------------------ */

/*
 * Section 5.4.4 extends the method to a small batch: one set of channels is
 * dropped for the whole batch, chosen by the magnitude of the activations
 * averaged over the batch dimension, and the criterion is still a single
 * threshold.  X is [batch][m] fp16 (one hidden state per row).  Channel i is
 * kept iff
 *
 *     (1 / batch) * sum_b |X[b][i]|  >  t .
 *
 * The inequality is evaluated as  sum_b |X[b][i]| > batch * t : fp16
 * magnitudes are multiples of 2^-24 below 2^16, so the sum of a few thousand
 * of them is exact in fp64, and batch * t is exact as well; no division, no
 * rounding, the same decision whatever the order of the batch.  A NaN anywhere
 * in a channel makes the sum NaN, which compares false: the channel is dropped
 * for every row.  mean_abs (may be NULL) receives sum / batch for inspection.
 * mask / idx as in oracle_sparsify; returns the number of kept channels.
 */
int32_t oracle_sparsify_batch(const uint16_t *X_f16, int32_t batch, int32_t m,
                              float t, double *mean_abs, uint8_t *mask,
                              int32_t *idx)
{
    const double bound = (double)batch * (double)t;
    int32_t count = 0;
    for (int32_t i = 0; i < m; ++i) {
        double sum = 0.0;
        for (int32_t b = 0; b < batch; ++b)
            sum += fabs(oracle_f16_bits_to_f64(X_f16[(size_t)b * (size_t)m + (size_t)i]));
        int keep = sum > bound;
        if (mean_abs) mean_abs[i] = sum / (double)batch;
        if (mask) mask[i] = (uint8_t)keep;
        if (keep) {
            if (idx) idx[count] = i;
            ++count;
        }
    }
    return count;
}

/*
 * Y[b][j] = sum_i s_i * X[b][i] * W[j][i] with the batch-wide mask s above:
 * every row of the batch is multiplied with the same thresholded set of
 * channels.  Dense loop in index order on canonical W[n][m], fp64.
 * scratch_mask: m bytes; scratch_xs: m doubles.  Returns the kept count.
 */
int32_t oracle_sparse_gemv_bf16_batch(const uint16_t *W_bf16,
                                      const uint16_t *X_f16, int32_t batch,
                                      float t, double *Y, int32_t m, int32_t n,
                                      uint8_t *scratch_mask, double *scratch_xs)
{
    int32_t count = oracle_sparsify_batch(X_f16, batch, m, t, NULL, scratch_mask, NULL);
    for (int32_t b = 0; b < batch; ++b) {
        for (int32_t i = 0; i < m; ++i)
            scratch_xs[i] = scratch_mask[i]
                ? oracle_f16_bits_to_f64(X_f16[(size_t)b * (size_t)m + (size_t)i]) : 0.0;
        dense_rows_bf16(W_bf16, scratch_xs, Y + (size_t)b * (size_t)n, m, n);
    }
    return count;
}

/* ---- the MLP intermediate as the input of W_down (Appendix A.3) ----------- */

/*
 * Appendix A.3: MLP(x) = (SiLU(x W_gate^T) . x W_up^T) W_down^T with
 * SiLU(v) = v * sigma(v).  Under the method the input of W_down, the
 * intermediate h = SiLU(g) . u, is thresholded like any other hidden state
 * (Section 4.2).  A kernel that forms h itself from g = x W_gate^T and
 * u = x W_up^T (both fp32, as the products leave the previous calls) has to
 * fix h's arithmetic, because h decides the mask: which side of t an entry
 * falls on must not depend on who evaluates exp.  So this part of the oracle
 * is NOT fp64: it states, operation by operation in IEEE binary32 with
 * round-to-nearest-even, the arithmetic that defines h (the kernel's
 * precision), and the tests pin it against the fp64 formula to a few units in
 * the last place.  Everything after h (Definition 1, the product) is the fp64
 * oracle above.
 *
 *   z  = clamp(-g, -80, 80)               (exp(+-80) is far inside binary32;
 *                                          beyond it sigma is 1 or 0 to rounding)
 *   k  = rint(z * log2(e))
 *   r  = fma(k, -ln2_hi, z); r = fma(k, -ln2_lo, r)       (|r| <= ln2 / 2)
 *   p  = 1 + r + r^2/2! + ... + r^7/7!   by Horner's rule with fma
 *   e  = p * 2^k                          (exact scaling)
 *   sg = 1 / (1 + e);  SiLU = g * sg;  h32 = SiLU * u;  h = binary16(h32)
 * A NaN in g or u gives h = NaN (dropped by Definition 1's comparison).
 */
static float exp_neg_f32(float g)
{
    float z = -g;
    if (z > 80.0f) z = 80.0f;
    if (z < -80.0f) z = -80.0f;
    const float k = rintf(z * 1.44269502f);             /* log2(e) in binary32 */
    float r = fmaf(k, -0.693145752f, z);                /* ln 2, high part (0x3f317200) */
    r = fmaf(k, -1.42860677e-06f, r);                   /* ln 2, low part */
    float p = 1.0f / 5040.0f;
    p = fmaf(p, r, 1.0f / 720.0f);
    p = fmaf(p, r, 1.0f / 120.0f);
    p = fmaf(p, r, 1.0f / 24.0f);
    p = fmaf(p, r, 1.0f / 6.0f);
    p = fmaf(p, r, 0.5f);
    p = fmaf(p, r, 1.0f);
    p = fmaf(p, r, 1.0f);
    return ldexpf(p, (int)k);
}

float oracle_silu_f32(float g)
{
    if (g != g) return g;
    const float e = exp_neg_f32(g);
    const float sg = 1.0f / (1.0f + e);
    return g * sg;
}

/* binary32 -> binary16 bit pattern, round to nearest even (overflow -> Inf). */
uint16_t oracle_f32_to_f16_bits(float v)
{
    uint32_t u;
    memcpy(&u, &v, sizeof u);
    const uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    const uint32_t mag = u & 0x7FFFFFFFu;
    if (mag > 0x7F800000u) return (uint16_t)(sign | 0x7E00u);          /* NaN */
    if (mag >= 0x47800000u) return (uint16_t)(sign | 0x7C00u);          /* >= 65536: Inf (also Inf) */
    if (mag < 0x33000000u) return sign;                                 /* < 2^-25: rounds to zero */
    const int e = (int)(mag >> 23) - 127;                               /* unbiased exponent */
    uint32_t frac = (mag & 0x7FFFFFu) | 0x800000u;                      /* 24-bit significand */
    /* number of low bits to drop: 13 for normal halves, more for subnormal ones */
    int drop = e >= -14 ? 13 : 13 + (-14 - e);
    uint32_t kept = frac >> drop;
    const uint32_t rem = frac & ((1u << drop) - 1u);
    const uint32_t half = 1u << (drop - 1);
    if (rem > half || (rem == half && (kept & 1u))) ++kept;
    uint32_t out;
    if (e >= -14)
        out = ((uint32_t)(e + 15) << 10) + (kept - 0x400u);            /* a carry bumps the exponent */
    else
        out = kept;                                                     /* subnormal (0x400 = smallest normal) */
    return (uint16_t)(sign | (uint16_t)out);                            /* 65520..65535.99 round to 0x7C00 = Inf */
}

/* h[i] = binary16(SiLU(gate[i]) * up[i]) as defined above. */
void oracle_swiglu_f16(const float *gate, const float *up, int32_t m, uint16_t *h_f16)
{
    for (int32_t i = 0; i < m; ++i) {
        const float h32 = oracle_silu_f32(gate[i]) * up[i];
        h_f16[i] = oracle_f32_to_f16_bits(h32);
    }
}

/*
 * y = s_t(h) W_down^T with h formed from gate and up as above; W is canonical
 * [n][m].  scratch_h: m uint16; scratch_xs: m doubles.  Returns the kept count.
 */
int32_t oracle_sparse_gemv_bf16_swiglu(const uint16_t *W_bf16, const float *gate,
                                       const float *up, float t, double *y,
                                       int32_t m, int32_t n, uint16_t *scratch_h,
                                       double *scratch_xs)
{
    oracle_swiglu_f16(gate, up, m, scratch_h);
    return oracle_sparse_gemv_bf16(W_bf16, scratch_h, t, y, m, n, scratch_xs);
}

/* ---- the normalised hidden state as the input of W_q, W_k, W_v / W_gate, W_up ---- */

/*
 * The inputs of the attention and MLP projections (Appendix A.3) are the
 * block's hidden state after the normalisation layer (Section 4.1 attributes
 * their zero-mean shape to it).  The paper does not print the layer's formula;
 * the reading taken here is the root-mean-square normalisation of the model
 * family it evaluates (Section 5):
 *     x_i = gamma_i * h_i / sqrt(mean_j(h_j^2) + eps).
 * A kernel that forms x itself from h has to fix x's arithmetic, because x
 * decides the mask (as for the MLP intermediate above), including the order
 * of the sum of squares.  Stated here operation by operation, h and gamma
 * binary32:
 *   ss = sum of the squares h_j^2 in binary64 (each square is exact there),
 *        added by pairwise summation: the index range [0, P), P the smallest
 *        power of two >= m and entries past m zero, is halved recursively and
 *        the two halves' sums are added (each addition rounded to binary64)
 *   v  = ss / m + eps                       (binary64: division, then addition)
 *   r  = binary32(1 / sqrt(v))              (binary64 square root and division)
 *   a  = h_i * r;  b = a * gamma_i          (binary32, each rounded)
 *   x_i = binary16(b)
 * Everything after x (Definition 1, the product) is the fp64 oracle above.
 */
static double tree_sum_of_squares(const float *h, size_t lo, size_t size, size_t m)
{
    if (lo >= m) return 0.0;
    if (size == 1) return (double)h[lo] * (double)h[lo];
    const size_t half = size / 2;
    return tree_sum_of_squares(h, lo, half, m) + tree_sum_of_squares(h, lo + half, half, m);
}

/* ss as defined above (0 for m < 1). */
double oracle_sum_of_squares(const float *h, int32_t m)
{
    if (m < 1) return 0.0;
    size_t P = 1;
    while (P < (size_t)m) P *= 2;
    return tree_sum_of_squares(h, 0, P, (size_t)m);
}

/* r = binary32(1 / sqrt(mean(h^2) + eps)) as defined above (m >= 1). */
float oracle_rms_scale(const float *h, int32_t m, float eps)
{
    const double ss = oracle_sum_of_squares(h, m);
    const double v = ss / (double)m + (double)eps;
    return (float)(1.0 / sqrt(v));
}

/* x[i] = binary16((h[i] * r) * gamma[i]) as defined above. */
void oracle_rmsnorm_f16(const float *h, const float *gamma, float eps, int32_t m, uint16_t *x_f16)
{
    if (m < 1) return;
    const float r = oracle_rms_scale(h, m, eps);
    for (int32_t i = 0; i < m; ++i) {
        const float a = h[i] * r;
        const float b = a * gamma[i];
        x_f16[i] = oracle_f32_to_f16_bits(b);
    }
}

/*
 * y = s_t(x) W^T with x formed from h and gamma as above; W is canonical
 * [n][m].  scratch_x: m uint16; scratch_xs: m doubles.  Returns the kept count.
 */
int32_t oracle_sparse_gemv_bf16_rmsnorm(const uint16_t *W_bf16, const float *h,
                                        const float *gamma, float eps, float t, double *y,
                                        int32_t m, int32_t n, uint16_t *scratch_x,
                                        double *scratch_xs)
{
    oracle_rmsnorm_f16(h, gamma, eps, m, scratch_x);
    return oracle_sparse_gemv_bf16(W_bf16, scratch_x, t, y, m, n, scratch_xs);
}

/* Threads the parallel loops above use (1 when built without OpenMP). */
int32_t oracle_num_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int32_t k)
{
#ifdef _OPENMP
    if (k > 0) omp_set_num_threads(k);
#else
    (void)k;
#endif
}

/* ---- threshold calibration (Section 4.2) -------------------------------- */

/*
 * Section 4.2 estimates t_p from an empirical distribution of activations
 * collected offline.  The plain definition used here: over a sample of N
 * values (NaNs left out), t_p is the smallest sample magnitude t with
 * #{|x| <= t} >= p N, i.e. the k-th smallest |x| with k = ceil(p N); p = 0
 * gives t = 0.  Found by sorting the magnitudes.
 */
#include <stdlib.h>
#include <string.h>

static int cmp_u16(const void *a, const void *b)
{
    uint16_t x = *(const uint16_t *)a, y = *(const uint16_t *)b;
    return (x > y) - (x < y);
}

/* Rank of the order statistic for level p among n_valid values (0 = "t is 0").
 * The subtraction guards binary round-off in p*n (0.3 * 10 is slightly above 3). */
uint64_t oracle_quantile_rank(uint64_t n_valid, double p)
{
    double prod = p * (double)n_valid;
    double k = ceil(prod - 1e-9);
    if (k < 0.0) k = 0.0;
    if (k > (double)n_valid) k = (double)n_valid;
    return (uint64_t)k;
}

/* Returns t_p as a float (an fp16 value, exactly). scratch: count uint16. */
float oracle_quantile_threshold(const uint16_t *x_f16, uint64_t count, double p,
                                uint16_t *scratch)
{
    uint64_t n_valid = 0;
    for (uint64_t i = 0; i < count; ++i) {
        uint16_t mag = x_f16[i] & 0x7FFF;            /* |x|: clear the sign bit */
        if (mag > 0x7C00) continue;                   /* NaN */
        scratch[n_valid++] = mag;
    }
    uint64_t k = oracle_quantile_rank(n_valid, p);
    if (k == 0) return 0.0f;
    /* non-negative fp16 values order like their bit patterns */
    qsort(scratch, (size_t)n_valid, sizeof(uint16_t), cmp_u16);
    return (float)oracle_f16_bits_to_f64(scratch[k - 1]);
}

/* hist[b] += number of non-NaN samples whose magnitude has bit pattern b (b < 32768). */
void oracle_abs_histogram(const uint16_t *x_f16, uint64_t count, uint64_t *hist)
{
    for (uint64_t i = 0; i < count; ++i) {
        uint16_t mag = x_f16[i] & 0x7FFF;
        if (mag > 0x7C00) continue;
        hist[mag] += 1;
    }
}
