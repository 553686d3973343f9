/*
 * rsparse_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * Plain, slow, fp64 CPU implementation of the R-Sparse linear layer
 * (R-Sparse, Sec. 3.4) used to check the HIP library.  Only the test-suite,
 * the smoke check and the benchmark's "cpu_baseline" leg may call it.  It
 * shares no code with the HIP path and takes the algorithm's steps in the
 * paper's order and notation:
 *
 *   1. sparsification function  sigma_t(X)_j = X_j if |X_j| >= t else 0   (Sec. 3.4, "Sparsifying Input Activation")
 *   2. sparse part              Y_s = sigma_t(X) W^T, only the columns of W whose channel survived
 *   3. low-rank part            Y_r = (X - sigma_t(X)) (A_r B_r)^T       (Sec. 3.4, "R-Sparse Inference")
 *   4. sum                      Y   = Y_s + Y_r
 *
 * with A_r B_r stored as the two factors U_r [d_out][r] and S_r V_r^T [r][d_in]
 * (same product as the paper's U_r S^1/2 and S^1/2 V_r^T).  Operands are the
 * *stored* values (fp16 / bf16 bit patterns, widened exactly to double, or
 * doubles); nothing is rounded on the way and the result stays in double.
 *
 * Pins (tests/test_oracle_pins.py): tau = -inf or r = rank(W) gives the dense
 * product; r = 0 and tau = +inf give the "Sparse" and "Low-Rank" ablations of
 * Sec. 4.4; the (singular component, channel) double sum of Sec. 3.3 restricted
 * to the kept block, brute-forced over all masks of 8x8 layers; closed-form
 * factors; the Eckart-Young bound; numpy's matvec.  Variants (fixed-count
 * activation, signed threshold, output bias, the multi-phase activation and
 * residual biases of Sec. 3.2) are pinned in tests/test_oracle_variants.py:
 * numpy's stable sort, literal loops, a hand-worked example, the identity
 * Y_s + Y_r = sigma_T(H) W^T.  No function here is "parity unpinned".
 *
 * W is [d_out][d_in] row-major (nn.Linear orientation, Y = X W^T); "columns of
 * W" are input channels.  X is [B][d_in], Y is [B][d_out].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F16 = 0, ORC_BF16 = 1, ORC_F64 = 2 };

/* ---- exact widening of the 16-bit storage formats ---------------------- */

double orc_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1F;
    int frac = h & 0x3FF;
    double v;
    if (expo == 0)
        v = ldexp((double)frac, -24);                 /* zero and subnormals: frac * 2^-10 * 2^-14 */
    else if (expo == 31)
        v = frac ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)frac / 1024.0, expo - 15);
    return sign ? -v : v;
}

double orc_bf16_to_double(uint16_t h)
{
    /* bf16 is the upper half of an IEEE binary32 */
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static inline double ld(const void *p, size_t i, int kind)
{
    switch (kind) {
    case ORC_F16:  return orc_half_to_double(((const uint16_t *)p)[i]);
    case ORC_BF16: return orc_bf16_to_double(((const uint16_t *)p)[i]);
    default:       return ((const double *)p)[i];
    }
}

void orc_decode16(const uint16_t *in, size_t n, int dtype, double *out)
{
    for (size_t i = 0; i < n; ++i) out[i] = ld(in, i, dtype);
}

/* ---- step 1: the sparsification mask ----------------------------------- */

/* Keep-predicate of sigma_t: |x| >= t (the paper's definition, cmp_mode 0) or the
 * strict variant |x| > t (cmp_mode 1).  A NaN compares false: it is not kept. */
/* cmp_mode 0: |x| >= t (the printed sigma_t of Sec. 3.4); 1: |x| > t; 2: x >= t, signed -- the sparse components of
 * the multi-phase activation of Sec. 3.2 are the values at or above T_0, whatever their magnitude. */
static inline int keep(double x, float tau, int cmp_mode)
{
    if (cmp_mode == 2) return x >= (double)tau;
    double a = fabs(x);
    return cmp_mode == 0 ? (a >= (double)tau) : (a > (double)tau);
}

/* mask[c] = 1 if channel c of token x is kept.  Returns the number kept. */
int orc_mask(const void *x, int x_kind, int d_in, float tau, int cmp_mode, uint8_t *mask)
{
    int k = 0;
    for (int c = 0; c < d_in; ++c) {
        mask[c] = (uint8_t)keep(ld(x, (size_t)c, x_kind), tau, cmp_mode);
        k += mask[c];
    }
    return k;
}

/* ascending list of the channels with mask[c] == want */
static int list_of(const uint8_t *mask, int d_in, int want, int32_t *out)
{
    int n = 0;
    for (int c = 0; c < d_in; ++c)
        if (mask[c] == want) out[n++] = c;
    return n;
}

/* ---- the R-Sparse linear layer ------------------------------------------ */

/* Steps 2-4 for given masks: mask [B][d_in], 1 = the channel is kept (sigma(X) != 0 there).  bias: NULL, or [d_out]
 * added to every token's output (the static form of the residual biases of Sec. 3.2). */
int orc_rsparse_linear_masked(const void *W, const void *U, const void *SV, int kind_w,
                              const void *X, int kind_x,
                              int B, int d_in, int d_out, int r,
                              const uint8_t *mask, const double *bias, double *Y, int nthreads)
{
    if (B < 1 || d_in < 1 || d_out < 1 || r < 0 || !mask) return -1;
    if (nthreads < 1) nthreads = 1;
    int32_t *a_list = malloc(sizeof(int32_t) * (size_t)d_in);
    int32_t *i_list = malloc(sizeof(int32_t) * (size_t)d_in);
    double *xs = malloc(sizeof(double) * (size_t)d_in);
    double *t = malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
    if (!a_list || !i_list || !xs || !t) {
        free(a_list); free(i_list); free(xs); free(t);
        return -1;
    }
    for (int b = 0; b < B; ++b) {
        const uint8_t *mb = mask + (size_t)b * d_in;
        int k = list_of(mb, d_in, 1, a_list);         /* kept channels:  sigma_t(X) != 0      */
        int z = list_of(mb, d_in, 0, i_list);         /* the rest:       X - sigma_t(X) != 0  */
        for (int c = 0; c < d_in; ++c) xs[c] = ld(X, (size_t)b * d_in + c, kind_x);

        /* step 3a: t = (S_r V_r^T) (x - sigma_t(x)), only the channels that were zeroed */
#pragma omp parallel for num_threads(nthreads) schedule(static)
        for (int i = 0; i < r; ++i) {
            double s = 0.0;
            for (int j = 0; j < z; ++j) {
                int c = i_list[j];
                s += ld(SV, (size_t)i * d_in + c, kind_w) * xs[c];
            }
            t[i] = s;
        }

#pragma omp parallel for num_threads(nthreads) schedule(static)
        for (int o = 0; o < d_out; ++o) {
            /* step 2: sparse part, skipping the columns of W whose channel is zero */
            double ys = 0.0;
            for (int j = 0; j < k; ++j) {
                int c = a_list[j];
                ys += ld(W, (size_t)o * d_in + c, kind_w) * xs[c];
            }
            /* step 3b: y_r = U_r t */
            double yr = 0.0;
            for (int i = 0; i < r; ++i)
                yr += ld(U, (size_t)o * r + i, kind_w) * t[i];
            /* step 4 */
            Y[(size_t)b * d_out + o] = bias ? ys + yr + bias[o] : ys + yr;
        }
    }
    free(a_list); free(i_list); free(xs); free(t);
    return 0;
}

/* Fixed-count activation: keep the k channels of largest magnitude of one token (a variant of the thresholding of
 * Sec. 3.4 in which the sparsity is exact per token instead of in expectation).  Among equal magnitudes the lower
 * channel index is kept first; NaN is never kept (as under a threshold, where it compares false); with fewer than k
 * non-NaN channels all of them are kept.  Returns the number kept. */
typedef struct { double a; int c; } orc_mag;
static int cmp_mag(const void *p, const void *q)
{
    const orc_mag *x = p, *y = q;
    if (x->a != y->a) return x->a > y->a ? -1 : 1;     /* larger magnitude first */
    return x->c < y->c ? -1 : (x->c > y->c ? 1 : 0);   /* then lower channel */
}
int orc_topk_mask(const void *x, int x_kind, int d_in, int k, uint8_t *mask)
{
    if (d_in < 1 || k < 0) return -1;
    orc_mag *m = malloc(sizeof(orc_mag) * (size_t)d_in);
    if (!m) return -1;
    int n = 0;
    for (int c = 0; c < d_in; ++c) {
        double v = ld(x, (size_t)c, x_kind);
        mask[c] = 0;
        if (v == v) { m[n].a = fabs(v); m[n].c = c; ++n; }
    }
    qsort(m, (size_t)n, sizeof(orc_mag), cmp_mag);
    int kept = k < n ? k : n;
    for (int i = 0; i < kept; ++i) mask[m[i].c] = 1;
    free(m);
    return kept;
}

/*
 * kind_w / kind_x: ORC_F16, ORC_BF16 (W, U, SV, X are uint16 bit patterns) or ORC_F64.
 * topk 0: masks from the threshold tau under cmp_mode; topk > 0: fixed-count masks (tau, cmp_mode unused).
 * batch_mask_mode 0: every token uses its own mask (the paper's elementwise sigma_t).
 * batch_mask_mode 1: every token uses the union of the batch's masks.
 * bias: NULL or [d_out].
 * Optional outputs (may be NULL): act [B][d_in] ascending kept channels per token (first
 * cnt[b] entries valid), cnt [B], uni [d_in] ascending union of kept channels, ucnt [1].
 * Returns 0, or -1 on allocation failure / bad arguments.
 */
int orc_rsparse_linear_ex(const void *W, const void *U, const void *SV, int kind_w,
                          const void *X, int kind_x,
                          int B, int d_in, int d_out, int r,
                          float tau, int cmp_mode, int topk, int batch_mask_mode, const double *bias,
                          double *Y, int32_t *act, int32_t *cnt, int32_t *uni, int32_t *ucnt,
                          int nthreads)
{
    if (B < 1 || d_in < 1 || d_out < 1 || r < 0 || tau != tau || topk < 0) return -1;
    size_t esz = (kind_x == ORC_F64) ? 8 : 2;
    uint8_t *mask = malloc((size_t)B * d_in);
    uint8_t *umask = calloc((size_t)d_in, 1);
    if (!mask || !umask) { free(mask); free(umask); return -1; }

    /* step 1 for every token, and the union over the batch */
    for (int b = 0; b < B; ++b) {
        const void *xb = (const char *)X + (size_t)b * d_in * esz;
        if (topk > 0) orc_topk_mask(xb, kind_x, d_in, topk, mask + (size_t)b * d_in);
        else orc_mask(xb, kind_x, d_in, tau, cmp_mode, mask + (size_t)b * d_in);
        for (int c = 0; c < d_in; ++c) umask[c] |= mask[(size_t)b * d_in + c];
    }
    if (uni && ucnt) *ucnt = list_of(umask, d_in, 1, uni);
    if (batch_mask_mode == 1)
        for (int b = 0; b < B; ++b) memcpy(mask + (size_t)b * d_in, umask, (size_t)d_in);
    for (int b = 0; b < B; ++b) {
        int k = 0;
        for (int c = 0; c < d_in; ++c)
            if (mask[(size_t)b * d_in + c]) { if (act) act[(size_t)b * d_in + k] = c; ++k; }
        if (cnt) cnt[b] = k;
    }
    int rc = orc_rsparse_linear_masked(W, U, SV, kind_w, X, kind_x, B, d_in, d_out, r, mask, bias, Y, nthreads);
    free(mask); free(umask);
    return rc;
}

int orc_rsparse_linear(const void *W, const void *U, const void *SV, int kind_w,
                       const void *X, int kind_x,
                       int B, int d_in, int d_out, int r,
                       float tau, int cmp_mode, int batch_mask_mode,
                       double *Y, int32_t *act, int32_t *cnt, int32_t *uni, int32_t *ucnt,
                       int nthreads)
{
    return orc_rsparse_linear_ex(W, U, SV, kind_w, X, kind_x, B, d_in, d_out, r, tau, cmp_mode, 0, batch_mask_mode, NULL,
                                 Y, act, cnt, uni, ucnt, nthreads);
}

/* ---- Sec. 3.2: the multi-phase activation and its residual biases ----------------------------------------------
 *
 * sigma_T(x) = x                      if x >= T_0
 *            = (T_i + T_{i+1}) / 2    if T_{i+1} <= x < T_i,   i = 0 .. l-2,     T_0 > T_1 > ... > T_{l-1}.
 * The paper takes T_{l-1} as the minimum of the input, so nothing lies below it; for thresholds fixed in advance a
 * value below T_{l-1} is put into the last interval (reading).  l = 1: everything below T_0 becomes 0 (with T_0 = 0
 * this is ReLU, as Sec. 3.2 notes).
 */
static int phase_of(double x, const double *T, int l)   /* x < T_0, l >= 2: the i with T_{i+1} <= x < T_i */
{
    for (int i = 0; i + 1 < l; ++i)
        if (x >= T[i + 1]) return i;
    return l - 2;                                        /* below T_{l-1}: the last interval */
}
double orc_multiphase(double x, const double *T, int l)
{
    if (x != x) return x;
    if (x >= T[0]) return x;
    if (l < 2) return 0.0;
    int i = phase_of(x, T, l);
    return 0.5 * (T[i] + T[i + 1]);
}

/* The data-dependent residual of one token h (Sec. 3.2):
 *   Y_r = sum_{j=0}^{l-2} (T_j + T_{j+1})/2 * ( sum_{k in U_j} W^T[:, k] ),   U_j = { k : T_{j+1} <= h_k < T_j }.
 * Yr [d_out].  Each inner sum is the bias B_j of the paper; Bj (optional, [l-1][d_out]) receives them. */
int orc_multiphase_residual(const void *W, int kind_w, const void *h, int kind_h, int d_in, int d_out,
                            const double *T, int l, double *Yr, double *Bj)
{
    if (d_in < 1 || d_out < 1 || l < 1) return -1;
    for (int i = 0; i + 1 < l; ++i) if (!(T[i] > T[i + 1])) return -1;
    for (int o = 0; o < d_out; ++o) Yr[o] = 0.0;
    for (int j = 0; j + 1 < l; ++j) {
        for (int o = 0; o < d_out; ++o) {
            double bsum = 0.0;                                   /* B_j[o] = sum over the channels of U_j of W[o][k] */
            for (int k = 0; k < d_in; ++k) {
                double v = ld(h, (size_t)k, kind_h);
                if (v < T[0] && phase_of(v, T, l) == j) bsum += ld(W, (size_t)o * d_in + k, kind_w);
            }
            if (Bj) Bj[(size_t)j * d_out + o] = bsum;
            Yr[o] += 0.5 * (T[j] + T[j + 1]) * bsum;
        }
    }
    return 0;
}

/* Static bias: the data-dependent residual averaged over N calibration tokens (reading: Sec. 3.2 says the biases can
 * be made static and pre-computed but not how; the mean over calibration data is the least-squares constant). */
int orc_static_bias(const void *W, int kind_w, const void *H, int kind_h, int N, int d_in, int d_out,
                    const double *T, int l, double *bias)
{
    if (N < 1) return -1;
    size_t esz = (kind_h == ORC_F64) ? 8 : 2;
    double *yr = malloc(sizeof(double) * (size_t)d_out);
    if (!yr) return -1;
    for (int o = 0; o < d_out; ++o) bias[o] = 0.0;
    for (int n = 0; n < N; ++n) {
        if (orc_multiphase_residual(W, kind_w, (const char *)H + (size_t)n * d_in * esz, kind_h, d_in, d_out, T, l, yr, NULL)) {
            free(yr);
            return -1;
        }
        for (int o = 0; o < d_out; ++o) bias[o] += yr[o];
    }
    for (int o = 0; o < d_out; ++o) bias[o] /= (double)N;
    free(yr);
    return 0;
}

/* The full linear layer Y = X W^T (Sec. 3.1), the thing R-Sparse approximates. */
int orc_dense_linear(const void *W, int kind_w, const void *X, int kind_x,
                     int B, int d_in, int d_out, double *Y, int nthreads)
{
    if (B < 1 || d_in < 1 || d_out < 1) return -1;
    if (nthreads < 1) nthreads = 1;
    double *xs = malloc(sizeof(double) * (size_t)d_in);
    if (!xs) return -1;
    for (int b = 0; b < B; ++b) {
        for (int c = 0; c < d_in; ++c) xs[c] = ld(X, (size_t)b * d_in + c, kind_x);
#pragma omp parallel for num_threads(nthreads) schedule(static)
        for (int o = 0; o < d_out; ++o) {
            double s = 0.0;
            for (int c = 0; c < d_in; ++c)
                s += ld(W, (size_t)o * d_in + c, kind_w) * xs[c];
            Y[(size_t)b * d_out + o] = s;
        }
    }
    free(xs);
    return 0;
}

/* ---- threshold estimation ----------------------------------------------- */

static int cmp_double(const void *a, const void *b)
{
    double x = *(const double *)a, y = *(const double *)b;
    return (x > y) - (x < y);
}

/*
 * t(s): the s-quantile of |X| over the pooled calibration activations
 * (Sec. 3.4: P(|X| < t(s)) = s), taken as the order statistic a_(floor(s N)) of the
 * ascending magnitudes (0-based, clamped to N-1, no interpolation), so that
 * #{|x| < t} <= floor(s N) <= #{|x| <= t}.  `x` holds n values of kind x_kind.
 * Returns NaN on failure.
 */
double orc_quantile_tau(const void *x, int x_kind, size_t n, double s)
{
    if (n == 0 || !(s >= 0.0) || s > 1.0) return NAN;
    double *a = malloc(sizeof(double) * n);
    if (!a) return NAN;
    for (size_t i = 0; i < n; ++i) a[i] = fabs(ld(x, i, x_kind));
    qsort(a, n, sizeof(double), cmp_double);
    size_t idx = (size_t)floor(s * (double)n);
    if (idx > n - 1) idx = n - 1;
    double tau = a[idx];
    free(a);
    return tau;
}

/* ---- gated MLP input (Sec. 3.1: H = X W_up^T (.) sigma(X W_gate^T), sigma = SiLU) --------------
 *
 * The down projection's input is h = silu(g) * u, rounded once to the 16-bit storage type, and the
 * sparsification function then compares |h| with t.  That compare decides an index set, so both
 * sides must produce the same 16-bit h: the activation is DEFINED as the following fp32 recipe
 * (every operation a single correctly rounded IEEE fp32 operation, no contraction), which this
 * function writes out step by step:
 *
 *   NaN -> NaN;  g < -87 -> -0
 *   x = max(-g, -86);  n = rint(x * log2(e));  r = x - n ln2, with ln2 = hi + lo and two fused
 *   multiply-adds (hi has few enough bits that n * hi is exact)            (|r| <= ln2 / 2)
 *   p = exp(r) by the degree-7 Taylor polynomial (Horner, fused multiply-adds)
 *   e = p * 2^n (exponent-field addition);  silu = g / (1 + e);  h = round16(silu * u)
 *
 * Pins: silu32 against the fp64 value g / (1 + exp(-g)): within 3 ulp (measured 2.4); the rounding step
 * against torch's fp16 / bf16 conversions; the whole recipe against orc_gated_input_plain below (the plain
 * fp64 definition): equal bits except next to a rounding flip point.
 */
static inline uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static inline float f32_from(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

float orc_silu32(float g)
{
    if (g != g) return g;
    if (!(g >= -87.0f)) return -0.0f;
    float x = -g;
    if (x < -86.0f) x = -86.0f;
    const float n = rintf(x * 1.44269504f);
    float r = fmaf(-n, 0.693145752f, x);
    r = fmaf(-n, 1.42860677e-6f, r);
    float p = 1.98412698e-4f;
    p = fmaf(p, r, 1.38888889e-3f);
    p = fmaf(p, r, 8.33333333e-3f);
    p = fmaf(p, r, 4.16666667e-2f);
    p = fmaf(p, r, 1.66666667e-1f);
    p = fmaf(p, r, 0.5f);
    p = fmaf(p, r, 1.0f);
    p = fmaf(p, r, 1.0f);
    const float e = f32_from(f32_bits(p) + ((uint32_t)(int32_t)n << 23));
    const float d = 1.0f + e;
    return g / d;
}

static uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = f32_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

static uint16_t f32_to_f16_rne(float f)
{
    const uint32_t x = f32_bits(f);
    const uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    const uint32_t a = x & 0x7fffffffu;
    if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);              /* NaN */
    if (a >= 0x47800000u) return (uint16_t)(sign | 0x7c00u);             /* >= 65536, inf */
    if (a < 0x38800000u) {                                               /* below 2^-14: fp16 subnormal or zero */
        const float m = rintf(fabsf(f) * 16777216.0f);                   /* units of 2^-24, ties to even */
        return (uint16_t)(sign | (uint16_t)m);                           /* m = 1024 is the smallest normal */
    }
    uint32_t h = (((a >> 23) - 112u) << 10) | ((a & 0x7fffffu) >> 13);
    const uint32_t rem = a & 0x1fffu;
    if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) ++h;              /* may carry into the exponent, up to inf */
    return (uint16_t)(sign | h);
}

/* out16[i] = round16( silu32(g16[i]) * u16[i] ); kind = ORC_F16 or ORC_BF16. */
int orc_gated_input(const uint16_t *g16, const uint16_t *u16, int kind, size_t n, uint16_t *out16)
{
    if (kind != ORC_F16 && kind != ORC_BF16) return 1;
    for (size_t i = 0; i < n; ++i) {
        const float g = (float)(kind == ORC_F16 ? orc_half_to_double(g16[i]) : orc_bf16_to_double(g16[i]));
        const float u = (float)(kind == ORC_F16 ? orc_half_to_double(u16[i]) : orc_bf16_to_double(u16[i]));
        const float h = orc_silu32(g) * u;
        out16[i] = kind == ORC_F16 ? f32_to_f16_rne(h) : f32_to_bf16_rne(h);
    }
    return 0;
}

void orc_silu32_array(const float *g, size_t n, float *out)
{
    for (size_t i = 0; i < n; ++i) out[i] = orc_silu32(g[i]);
}

/* The two fp32 -> 16-bit roundings above, exposed so that the tests can pin them against an independent
 * implementation (torch's CPU conversions). */
void orc_round16_array(const float *f, size_t n, int kind, uint16_t *out16)
{
    for (size_t i = 0; i < n; ++i) out16[i] = kind == ORC_F16 ? f32_to_f16_rne(f[i]) : f32_to_bf16_rne(f[i]);
}

/* ---- the gated input by its plain definition (Sec. 3.1) -----------------------------------------
 *
 * h = u * g / (1 + exp(-g)) evaluated in fp64 with the C library's exp, then ONE rounding (nearest, ties to
 * even) of that double to the 16-bit storage type.  No recipe, no fp32 intermediate: this is the definition
 * the fp32 recipe above approximates, and the cross-check of that recipe and of the device's copy of it.
 *
 * The rounding is written from the formats' definitions (p significand bits, smallest normal exponent
 * emin, largest finite value), not from bit manipulation: scale the magnitude so that one unit in the
 * last place becomes 1.0, round with rint (the default rounding mode is nearest-even), scale back.
 *   fp16:  p = 11, emin = -14, max = 65504         bf16:  p = 8, emin = -126, max = (2 - 2^-7) 2^127
 * out16[i]: the rounded bits.  margin[i] (may be NULL): how far the fp64 value is from the nearest point
 * where the rounding flips (a midpoint between two neighbouring 16-bit values), as a fraction of the
 * spacing of the 16-bit values there -- 0 = exactly on a midpoint, 0.5 = exactly representable.  A result
 * whose margin exceeds the error of an approximate evaluation cannot differ from that evaluation's.
 */
static uint16_t round_double_to16(double v, int kind, double *margin)
{
    const int p = kind == ORC_F16 ? 11 : 8, emin = kind == ORC_F16 ? -14 : -126;
    const int emax = kind == ORC_F16 ? 15 : 127, ebits = kind == ORC_F16 ? 5 : 8, bias = emax;
    const uint16_t sign = signbit(v) ? 0x8000u : 0u;
    const uint16_t inf = (uint16_t)(((1u << ebits) - 1u) << (p - 1));
    if (margin) *margin = 0.5;
    if (isnan(v)) return (uint16_t)(inf | (1u << (p - 2)));          /* quiet NaN, sign dropped */
    double a = fabs(v);
    if (isinf(a)) return (uint16_t)(sign | inf);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                    /* a = m 2^e, 0.5 <= m < 1, i.e. 2^(e-1) <= a < 2^e */
    int ex = e - 1;                        /* exponent of the leading bit */
    if (ex < emin) ex = emin;              /* subnormal range: fixed spacing 2^(emin - p + 1) */
    const double q = ldexp(a, -(ex - (p - 1)));      /* a in units of the spacing: exact (power of two) */
    const double n = rint(q);                         /* nearest, ties to even */
    if (margin) {
        const double f = q - floor(q);                /* position between two neighbours */
        *margin = fabs(f - 0.5);
    }
    double r = ldexp(n, ex - (p - 1));
    /* the largest finite value is (2 - 2^(1-p)) 2^emax; rounding reached 2^(emax+1) -> infinity */
    if (r >= ldexp(1.0, emax + 1)) return (uint16_t)(sign | inf);
    if (r == 0.0) return sign;
    int e2;
    const double m2 = frexp(r, &e2);       /* r = m2 2^e2 */
    int ex2 = e2 - 1;
    uint32_t bits;
    if (ex2 < emin) {
        bits = (uint32_t)ldexp(r, -(emin - (p - 1)));                  /* subnormal: the count of spacings */
    } else {
        const uint32_t frac = (uint32_t)(ldexp(m2, p) - ldexp(1.0, p - 1));   /* significand without the leading bit */
        bits = ((uint32_t)(ex2 + bias) << (p - 1)) | frac;
    }
    return (uint16_t)(sign | bits);
}

int orc_gated_input_plain(const uint16_t *g16, const uint16_t *u16, int kind, size_t n, uint16_t *out16,
                          double *margin)
{
    if (kind != ORC_F16 && kind != ORC_BF16) return 1;
    for (size_t i = 0; i < n; ++i) {
        const double g = kind == ORC_F16 ? orc_half_to_double(g16[i]) : orc_bf16_to_double(g16[i]);
        const double u = kind == ORC_F16 ? orc_half_to_double(u16[i]) : orc_bf16_to_double(u16[i]);
        /* g = -inf: the quotient reads inf / inf; the function's limit there is 0 from below */
        const double silu = (isinf(g) && g < 0) ? -0.0 : g / (1.0 + exp(-g));
        out16[i] = round_double_to16(silu * u, kind, margin ? margin + i : NULL);
    }
    return 0;
}

/* One rounding of doubles to the 16-bit type, by the definition above (test hook). */
void orc_round16_from_double(const double *v, size_t n, int kind, uint16_t *out16)
{
    for (size_t i = 0; i < n; ++i) out16[i] = round_double_to16(v[i], kind, NULL);
}

/* ---- 4-bit weights ------------------------------------------------------- */

/* The combination with weight quantisation (Sec. 4.4, the answer on quantisation and Table 2:
 * 4-bit GPTQ weights, groups of 128).  GPTQ's storage format: every output row o is cut into groups
 * of `group` consecutive input channels, each with a 16-bit scale s and a 4-bit zero point z; the
 * weight the layer multiplies by is the real number
 *
 *     W~[o][c] = s[o][c / group] * (q[o][c] - z[o][c / group]),      q, z in 0..15
 *
 * which a double holds exactly.  The R-Sparse layer on 4-bit weights is orc_rsparse_linear with this
 * W~ as its (double) W; the low-rank factors stay 16-bit inputs of their own.
 * q: [d_out][d_in] one code per byte;  s16: [d_out][d_in / group];  z: [d_out][d_in / group]. */
int orc_dequant_q4(const uint8_t *q, const void *s16, int s_kind, const uint8_t *z, int d_out, int d_in,
                   int group, double *W)
{
    if (!q || !s16 || !z || !W || d_out < 1 || d_in < 1 || group < 1 || d_in % group) return 1;
    if (s_kind != ORC_F16 && s_kind != ORC_BF16) return 1;
    const size_t G = (size_t)d_in / group;
    for (size_t o = 0; o < (size_t)d_out; ++o)
        for (size_t c = 0; c < (size_t)d_in; ++c) {
            const size_t g = c / group;
            if (q[o * d_in + c] > 15 || z[o * G + g] > 15) return 1;
            W[o * d_in + c] = ld(s16, o * G + g, s_kind) * ((double)q[o * d_in + c] - (double)z[o * G + g]);
        }
    return 0;
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
