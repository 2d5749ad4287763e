/*
 * CrossQuant CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, single-translation-unit statement of what the CrossQuant activation
 * quantization path computes, written from the paper (arxiv 2410.07505) alone.  It shares no
 * code, header, table or helper with the HIP library; only tests, the smoke check and the
 * benchmark's cpu_baseline leg may load it.  Every function below is pinned by CPU tests
 * against closed forms, brute force and a float64 restatement (no function is "parity unpinned").
 *
 * Arithmetic (fixed so that a GPU can reproduce it bit for bit):
 *   - X, W are IEEE binary16 bit patterns (uint16_t); they are widened exactly to binary32.
 *   - the T+I scale factors use binary64 pow(), rounded once to binary32;
 *   - every per-element operation is one binary32 multiply or divide, rounded to nearest even,
 *     with no fused multiply-add (build with -ffp-contract=off, no fast-math);
 *   - round() is round-half-to-even (rintf in the default rounding mode);
 *   - integer work (counts, accumulators) is exact.
 *
 * Loops over rows carry an OpenMP pragma so the timed baseline can use the host's cores; the
 * pragma changes no arithmetic and no order of any floating-point operation.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------- binary16 <-> binary32, written out bit by bit ---------- */

/* Exact widening of a binary16 bit pattern (every binary16 value is a binary32 value). */
float cq_oracle_half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    uint32_t e = (uint32_t)(h >> 10) & 0x1Fu;
    uint32_t m = (uint32_t)h & 0x3FFu;
    float v;
    if (e == 0) {
        v = ldexpf((float)m, -24);                 /* zero and subnormals: m * 2^-24 */
    } else if (e == 31) {
        v = (m == 0) ? INFINITY : NAN;
    } else {
        v = ldexpf((float)(m | 0x400u), (int)e - 25); /* (1024+m) * 2^(e-15-10) */
    }
    return sign ? -v : v;
}

/* binary32 -> binary16, round to nearest even, overflow to infinity, gradual underflow. */
uint16_t cq_oracle_float_to_half(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t au = u & 0x7FFFFFFFu;
    if (au > 0x7F800000u) return (uint16_t)(sign | 0x7E00u);          /* NaN */
    if (au == 0x7F800000u) return (uint16_t)(sign | 0x7C00u);         /* Inf */
    float a = fabsf(f);
    if (a >= 65520.0f) return (uint16_t)(sign | 0x7C00u);             /* rounds past max finite */
    if (a == 0.0f) return sign;
    int ex;
    (void)frexpf(a, &ex);                     /* a = frac * 2^ex, frac in [0.5,1) */
    int e = ex - 1;                           /* a = 1.xxx * 2^e */
    if (e < -14) e = -14;                     /* subnormal range uses the fixed quantum 2^-24 */
    /* quantum of binary16 at this exponent is 2^(e-10); a / quantum is exact in binary32
       (power-of-two scaling, result well inside the normal range) */
    float scaled = ldexpf(a, 10 - e);
    float r = rintf(scaled);                  /* round half to even; r in [0, 2048] */
    uint32_t q = (uint32_t)r;
    uint32_t bits;
    if (e == -14 && q < 1024u) {
        bits = q;                             /* subnormal (or zero) */
    } else {
        if (q == 2048u) { q = 1024u; e += 1; } /* mantissa carried into the next binade */
        bits = ((uint32_t)(e + 15) << 10) | (q - 1024u);
    }
    return (uint16_t)(sign | bits);
}

static int qmax_of_bits(int bits) { return (1 << (bits - 1)) - 1; } /* 2^(N-1)-1, Eq. 1 */

int cq_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of threads the row loops may use from now on (timing only: no result depends on it). */
void cq_oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---------- row and column absolute maxima (Eq. 1: t_i ; CrossQuant equation: c_j) ---------- */
/* X: T x I binary16, row-major with leading dimension ldx (elements). */
void cq_oracle_absmax(const uint16_t *X, int64_t T, int64_t I, int64_t ldx, float *t, float *c)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < T; ++i) {
        float m = 0.0f;
        for (int64_t j = 0; j < I; ++j) {
            float v = fabsf(cq_oracle_half_to_float(X[i * ldx + j]));
            if (v > m) m = v;
        }
        t[i] = m;
    }
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < I; ++j) {
        float m = 0.0f;
        for (int64_t i = 0; i < T; ++i) {
            float v = fabsf(cq_oracle_half_to_float(X[i * ldx + j]));
            if (v > m) m = v;
        }
        c[j] = m;
    }
}

/* ---------- scale factors: the CrossQuant step split into a row and a column factor ----------
 * Delta~_ij = t_i^alpha * c_j^(1-alpha) / (2^(N-1)-1)  =  a_i * b_j  with
 *   a_i = t_i^alpha / q_max   (the appendix listing's row scale, carrying 1/q_max)
 *   b_j = c_j^(1-alpha)       (the appendix listing's column scale)
 * pow in binary64, one rounding to binary32.  pow(x, 0) = 1 for every x (C semantics), so
 * alpha = 1 gives b = 1 exactly (per-token quantization) and alpha = 0 gives a = fl32(1/q_max). */
void cq_oracle_scales(const float *t, const float *c, int64_t T, int64_t I, float alpha, int bits,
                      float *a, float *b)
{
    double al = (double)alpha;
    double qm = (double)qmax_of_bits(bits);
    for (int64_t i = 0; i < T; ++i) a[i] = (float)(pow((double)t[i], al) / qm);
    for (int64_t j = 0; j < I; ++j) b[j] = (float)pow((double)c[j], 1.0 - al);
}

/* one element of the CrossQuant equation, given its step D = fl32(a_i * b_j) */
static int quantize_one(float x, float D, int qmax)
{
    if (D == 0.0f) return 0;            /* all-zero row or column: x is 0 as well */
    float r = rintf(x / D);             /* round(X_ij / Delta~_ij), half to even */
    if (r > (float)qmax) r = (float)qmax;      /* guard; never fires for exact t, c */
    if (r < (float)-qmax) r = (float)-qmax;
    return (int)r;
}

/* ---------- CrossQuant quantize + dequantize + kernel count ----------
 * codes: bits==8 -> int8 [T][I]; bits==4 -> packed two's-complement nibbles [T][I/2], even
 *        column in the low nibble.  xhat (nullable): binary16 [T][I] = fl16(fl32(q * D)).
 * a[T], b[I] are outputs (the scale factors).  Z (nullable) = #{codes == 0}: the size of the
 * quantization kernel K(CQ) of Definition 1 (first line: the elements with Q(X_ij) = 0).
 * clamp_hits (nullable) counts how often the +-q_max guard changed a value. */
void cq_oracle_quantize(const uint16_t *X, int64_t T, int64_t I, int64_t ldx, const float *t,
                        const float *c, float alpha, int bits, void *codes, uint16_t *xhat,
                        float *a, float *b, uint64_t *Z, uint64_t *clamp_hits)
{
    int qmax = qmax_of_bits(bits);
    cq_oracle_scales(t, c, T, I, alpha, bits, a, b);
    uint64_t zeros = 0, clamps = 0;
#pragma omp parallel for schedule(static) reduction(+ : zeros, clamps)
    for (int64_t i = 0; i < T; ++i) {
        for (int64_t j = 0; j < I; ++j) {
            float x = cq_oracle_half_to_float(X[i * ldx + j]);
            float D = a[i] * b[j];
            int q = quantize_one(x, D, qmax);
            if (D != 0.0f && fabsf(rintf(x / D)) > (float)qmax) ++clamps;
            if (q == 0) ++zeros;
            if (bits == 8) {
                ((int8_t *)codes)[i * I + j] = (int8_t)q;
            } else {
                uint8_t *p = (uint8_t *)codes + i * (I / 2) + j / 2;
                uint8_t nib = (uint8_t)(q & 0xF);
                if ((j & 1) == 0) *p = nib;                        /* even column: low nibble */
                else              *p = (uint8_t)(*p | (uint8_t)(nib << 4)); /* odd: high nibble */
            }
            if (xhat) xhat[i * I + j] = cq_oracle_float_to_half((float)q * D);
        }
    }
    if (Z) *Z = zeros;
    if (clamp_hits) *clamp_hits = clamps;
}

/* ---------- kernel count only (Definition 1; the proportion is Z / (T*I)) ---------- */
void cq_oracle_kernel_count(const uint16_t *X, int64_t T, int64_t I, int64_t ldx, const float *t,
                            const float *c, float alpha, int bits, float *a_work, float *b_work,
                            uint64_t *Z)
{
    int qmax = qmax_of_bits(bits);
    cq_oracle_scales(t, c, T, I, alpha, bits, a_work, b_work);
    uint64_t zeros = 0;
#pragma omp parallel for schedule(static) reduction(+ : zeros)
    for (int64_t i = 0; i < T; ++i)
        for (int64_t j = 0; j < I; ++j) {
            float x = cq_oracle_half_to_float(X[i * ldx + j]);
            if (quantize_one(x, a_work[i] * b_work[j], qmax) == 0) ++zeros;
        }
    *Z = zeros;
}

/* ---------- per-channel weight quantization (Eq. 2), one step per OUTPUT channel ----------
 * W: I x O binary16 row-major (the paper's layout, Y = X W).  fold (nullable, [I]) multiplies
 * row j of W first: W'_jk = fl32(f_j * W_jk); this is how the column factor b_j of the
 * element-wise CrossQuant step is carried into an integer GEMM.  s_k = fl32(max_j|W'_jk| / q_max),
 * qw_kj = round(W'_jk / s_k), stored transposed as [O][I] (contraction axis contiguous). */
void cq_oracle_weight_quantize(const uint16_t *W, int64_t I, int64_t O, const float *fold, int bits,
                               int8_t *qw, float *s)
{
    int qmax = qmax_of_bits(bits);
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < O; ++k) {
        float m = 0.0f;
        for (int64_t j = 0; j < I; ++j) {
            float w = cq_oracle_half_to_float(W[j * O + k]);
            if (fold) w = fold[j] * w;
            if (fabsf(w) > m) m = fabsf(w);
        }
        float sk = m / (float)qmax;
        s[k] = sk;
        for (int64_t j = 0; j < I; ++j) {
            float w = cq_oracle_half_to_float(W[j * O + k]);
            if (fold) w = fold[j] * w;
            qw[k * I + j] = (int8_t)quantize_one(w, sk, qmax);
        }
    }
}

/* ---------- W8A8 linear: Y = X W on integer codes (Background section, Y = X . W) ----------
 * acc_ik = sum_j qx_ij * qw_kj (exact int32); Y_ik = fl16(fl32(fl32(float(acc_ik) * a_i) * s_k)).
 * qx: [T][I] int8; qw: [O][I] int8; acc (nullable): [T][O] int32; Y (nullable): binary16, ld ldy. */
void cq_oracle_w8a8_linear(const int8_t *qx, const float *a, const int8_t *qw, const float *s,
                           int64_t T, int64_t I, int64_t O, uint16_t *Y, int64_t ldy, int32_t *acc)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < T; ++i)
        for (int64_t k = 0; k < O; ++k) {
            int32_t sum = 0;
            for (int64_t j = 0; j < I; ++j) sum += (int32_t)qx[i * I + j] * (int32_t)qw[k * I + j];
            if (acc) acc[i * O + k] = sum;
            if (Y) {
                float y = (float)sum * a[i];
                y = y * s[k];
                Y[i * ldy + k] = cq_oracle_float_to_half(y);
            }
        }
}

/* ---------- quantization-kernel analysis: "Remove Kernel" and the Table 1 indicators ----------
 * "Remove Kernel" (captions of the zero-shot accuracy figures): the elements of the quantization
 * kernel K(Q) are set to zero and every other element is left untouched in FP16:
 *     xrk_ij = (q_ij == 0) ? 0 : X_ij        with q_ij the code of the chosen quantizer (alpha, bits).
 * Table 1's two indicators over all (i, j) of the matrix, for the kernel-size analysis' cases I/II:
 *     n_col_ge_row    = #{ c_j >= t_i }                      (case II)
 *     n_bound_smaller = #{ B~_ij < B_ij }, B~_ij = 0.5 * fl32(a_i * b_j)  (zero bound of CrossQuant),
 *                                          B_ij  = 0.5 * fl32(t_i / q_max) (zero bound of per-token, Eq. 1)
 * counters[0] = Z (kernel size), counters[1] = n_col_ge_row, counters[2] = n_bound_smaller.
 * xrk (nullable): binary16 [T][I]. a, b are outputs as in cq_oracle_quantize. */
void cq_oracle_kernel_analysis(const uint16_t *X, int64_t T, int64_t I, int64_t ldx, const float *t,
                               const float *c, float alpha, int bits, uint16_t *xrk, float *a, float *b,
                               uint64_t *counters)
{
    int qmax = qmax_of_bits(bits);
    cq_oracle_scales(t, c, T, I, alpha, bits, a, b);
    uint64_t zeros = 0, col_ge = 0, smaller = 0;
#pragma omp parallel for schedule(static) reduction(+ : zeros, col_ge, smaller)
    for (int64_t i = 0; i < T; ++i) {
        float step_pt = (float)((double)t[i] / (double)qmax);   /* per-token step of Eq. 1 */
        for (int64_t j = 0; j < I; ++j) {
            uint16_t h = X[i * ldx + j];
            float x = cq_oracle_half_to_float(h);
            float D = a[i] * b[j];
            int q = quantize_one(x, D, qmax);
            if (q == 0) ++zeros;
            if (c[j] >= t[i]) ++col_ge;
            if (0.5f * D < 0.5f * step_pt) ++smaller;
            if (xrk) xrk[i * I + j] = (q == 0) ? (uint16_t)0 : h;
        }
    }
    counters[0] = zeros;
    counters[1] = col_ge;
    counters[2] = smaller;
}

/* ---------- group-wise weight quantization (Background section: W reshaped to (I*O/g) x g) ----------
 * Each output channel k is cut into groups of g consecutive input channels (the contraction axis,
 * as in the weight-only code bases the paper builds on); every group has its own step:
 *   s_{k,G} = fl32(max_{j in G} |W'_jk| / q_max),  qw_kj = clamp(rne(fl32(W'_jk / s_{k, j/g})))
 * with W'_jk = fl32(f_j * W_jk) as in the per-channel case (g = I reduces to it exactly).
 * W: I x O binary16 row-major; qw: [O][I]; s: [O][I/g]; wdq (nullable): binary16 [I][O],
 * the dequantized (fake-quantized) weights fl16(fl32(q * s)).  I must be a multiple of g. */
void cq_oracle_weight_quantize_grouped(const uint16_t *W, int64_t I, int64_t O, const float *fold,
                                       int64_t g, int bits, int8_t *qw, float *s, uint16_t *wdq)
{
    int qmax = qmax_of_bits(bits);
    int64_t ng = I / g;
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < O; ++k)
        for (int64_t G = 0; G < ng; ++G) {
            float m = 0.0f;
            for (int64_t j = G * g; j < (G + 1) * g; ++j) {
                float w = cq_oracle_half_to_float(W[j * O + k]);
                if (fold) w = fold[j] * w;
                if (fabsf(w) > m) m = fabsf(w);
            }
            float sk = m / (float)qmax;
            s[k * ng + G] = sk;
            for (int64_t j = G * g; j < (G + 1) * g; ++j) {
                float w = cq_oracle_half_to_float(W[j * O + k]);
                if (fold) w = fold[j] * w;
                int q = quantize_one(w, sk, qmax);
                qw[k * I + j] = (int8_t)q;
                if (wdq) wdq[j * O + k] = cq_oracle_float_to_half((float)q * sk);
            }
        }
}
