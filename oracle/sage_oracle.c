/*
 * CPU oracle for the SageAttention2++ "8+8" attention forward pass
 * (INT8 Q.K^T, FP8-E4M3 P.V).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, double-precision
 * statement of what the method computes, written from the paper so that a
 * reader can check it against the text by eye.  It shares no code with the
 * GPU library, is never linked into it and must never be reached from the
 * product path: only the test-suite, the smoke check and the benchmark's
 * "cpu_baseline" leg may call it.
 *
 * What each routine follows (all references are to the paper):
 *   - tiling of Q, K, P~, V into blocks and the online softmax: Section 2.1;
 *   - per-block INT8 scales  delta_Q = max|Q|/127, delta_K = max|K|/127,
 *     per-channel FP8 scale  delta_V = colmax|V| / V_r,  the rounding
 *     X^ = round(X / delta)  and the de-quantisation
 *     PV = P^ V^ * delta_P * delta_V: Section 2.1 and Section 3.1, Eq. (2);
 *   - narrowed FP8 ranges P_r, V_r (defaults 224 and 4.5): Section 3.1-3.2;
 *   - smoothing of K (subtracting the per-channel mean over tokens):
 *     Section 3, first paragraph (the paper names the step, gives no formula;
 *     the per-(batch, head, channel) mean over all N tokens is the reading
 *     taken here);
 *   - the "4+8" variant (INT4 Q.K^T, Section 2.1 "INT4/INT8", Section 3 "smoothing of Q and K",
 *     Section 4.1 "SageAttn2++(4+8)"): the routines marked 4+8 below; the paper names its ingredients and
 *     prints no formula for them, the readings taken are stated at each routine;
 *   - accuracy metrics are NOT here (they are measurement, not method).
 *
 * Readings taken where the paper is silent (listed again in the design notes):
 *   round(.) is round-to-nearest-even everywhere; max(|.|) is used for every
 *   scale; delta_P is the constant 1/P_r (P~ <= 1 by construction); the softmax
 *   denominator l accumulates the UNQUANTISED P~; exponentials are base 2 with
 *   sm_scale*log2(e) folded into the de-quantisation constant; causal means key
 *   n is visible to query r iff n <= r; partial blocks take their scale over the
 *   valid rows only; an all-zero block or channel gets scale 0 and codes 0; the
 *   output is rounded (RNE) to the 16-bit input type.
 *
 * Steps that are *defined* as IEEE binary32 operations (so that "bit-exact
 * codes and scales" is a meaningful requirement) are evaluated in `float`
 * with contraction disabled (compile with -ffp-contract=off): the channel
 * mean's final rounding, K - mean, scale = a/range, r = range/a, x*r.
 * Everything else is double.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define SAGE_ORACLE_LOG2E 1.4426950408889634073599246810019

/* --------------------------------------------------------------------- */
/* number formats                                                        */
/* --------------------------------------------------------------------- */

/* FP8 E4M3 in the OCP "FN" flavour (Section 3.1 quotes its range, +-448):
 * 1 sign, 4 exponent (bias 7), 3 mantissa bits; no infinities; exponent 15
 * with mantissa 7 is NaN; exponent 0 is subnormal with step 2^-9.            */
double sage_oracle_e4m3_decode(uint8_t code)
{
    int sign = code >> 7;
    int e = (code >> 3) & 15;
    int m = code & 7;
    double mag;
    if (e == 15 && m == 7)
        return NAN;
    if (e == 0)
        mag = ldexp((double)m, -9);          /* m/8 * 2^-6 */
    else
        mag = ldexp((double)(8 + m), e - 10); /* (1 + m/8) * 2^(e-7) */
    return sign ? -mag : mag;
}

/* Round-to-nearest-even encoder from a real number; magnitudes that would
 * round beyond 448 saturate to 448 (never reached with the default ranges,
 * Section 3.1).                                                              */
uint8_t sage_oracle_e4m3_encode(double x)
{
    uint8_t sign = signbit(x) ? 0x80 : 0x00;
    double a = fabs(x);
    if (isnan(x))
        return 0x7f;
    if (a >= 464.0) /* 464 is the midpoint between 448 and the next (absent) step */
        return sign | 0x7e;
    if (a < ldexp(1.0, -6)) {
        /* subnormal range, step 2^-9; a result of 8 steps is the smallest normal */
        int r = (int)nearbyint(ldexp(a, 9));
        return sign | (uint8_t)r;
    }
    int ex;
    (void)frexp(a, &ex);            /* a = f * 2^ex, f in [0.5, 1) */
    int E = ex - 1;                 /* a in [2^E, 2^(E+1)) */
    int r = (int)nearbyint(ldexp(a, 3 - E)); /* in [8, 16] */
    if (r == 16) {
        r = 8;
        E += 1;
    }
    int biased = E + 7;
    if (biased > 15 || (biased == 15 && r - 8 > 6))
        return sign | 0x7e;
    return sign | (uint8_t)((biased << 3) | (r - 8));
}

/* Round a double to a 16-bit floating type and return the rounded value as a
 * double.  dtype 0 = IEEE binary16 (fp16), 1 = bfloat16.  RNE, gradual
 * underflow, overflow to infinity.                                           */
double sage_oracle_round16(double x, int dtype)
{
    int p = dtype == 0 ? 11 : 8;          /* significand bits incl. the hidden one */
    int emin = dtype == 0 ? -14 : -126;
    double maxv = dtype == 0 ? 65504.0 : ldexp(255.0, 120); /* (2 - 2^-7) * 2^127 */
    if (x == 0.0 || isnan(x) || isinf(x))
        return x;
    int ex;
    (void)frexp(fabs(x), &ex);
    int E = ex - 1;
    if (E < emin)
        E = emin;
    double q = ldexp(1.0, E - (p - 1));
    double r = nearbyint(x / q) * q;
    if (fabs(r) > maxv)
        return x > 0 ? INFINITY : -INFINITY;
    return r;
}

/* --------------------------------------------------------------------- */
/* quantisation stage                                                    */
/* --------------------------------------------------------------------- */

/* Smoothing statistic (Section 3): mu[c] = mean over the N tokens of K[n][c].
 * The sum is taken in double, the quotient is rounded once to binary32.      */
void sage_oracle_k_mean(const float *K, int N, int d, float *mu)
{
    for (int c = 0; c < d; ++c) {
        double s = 0.0;
        for (int n = 0; n < N; ++n)
            s += (double)K[(size_t)n * d + c];
        mu[c] = (float)(s / (double)N);
    }
}

/* Per-block INT8 quantisation (Section 2.1): rows are grouped into blocks of
 * `block` consecutive tokens (the last may be partial); for each block
 *   a = max|X'|,  delta = a/127,  X^ = round(X' * (127/a)),   X' = X - mu
 * (mu == NULL means no smoothing, i.e. X' = X).  binary32 operations.        */
void sage_oracle_quant_int8(const float *X, const float *mu, int N, int d, int block,
                            int8_t *codes, float *delta)
{
    int nb = (N + block - 1) / block;
    for (int j = 0; j < nb; ++j) {
        int n0 = j * block;
        int n1 = n0 + block < N ? n0 + block : N;
        float a = 0.0f;
        for (int n = n0; n < n1; ++n)
            for (int c = 0; c < d; ++c) {
                float x = X[(size_t)n * d + c];
                if (mu)
                    x = x - mu[c];
                float ax = fabsf(x);
                if (ax > a)
                    a = ax;
            }
        if (a == 0.0f) {
            delta[j] = 0.0f;
            for (int n = n0; n < n1; ++n)
                memset(codes + (size_t)n * d, 0, (size_t)d);
            continue;
        }
        delta[j] = a / 127.0f;
        float r = 127.0f / a;
        for (int n = n0; n < n1; ++n)
            for (int c = 0; c < d; ++c) {
                float x = X[(size_t)n * d + c];
                if (mu)
                    x = x - mu[c];
                float y = x * r;
                codes[(size_t)n * d + c] = (int8_t)nearbyintf(y);
            }
    }
}

/* ---- 4+8 variant: smoothing of Q and INT4 codes ----------------------------------------------------- */

/* Smoothing statistic of Q (Section 3 names "smoothing of Q and K"; reading: what is subtracted from Q is
 * the mean of each Q block, per channel, over the block's valid tokens):
 *   qbar[i][c] = mean over rows r of block i of Q[r][c];  double sum, one rounding to binary32.            */
void sage_oracle_block_mean(const float *Q, int N, int d, int block, float *qbar)
{
    int nb = (N + block - 1) / block;
    for (int i = 0; i < nb; ++i) {
        int r0 = i * block;
        int r1 = r0 + block < N ? r0 + block : N;
        for (int c = 0; c < d; ++c) {
            double s = 0.0;
            for (int r = r0; r < r1; ++r)
                s += (double)Q[(size_t)r * d + c];
            qbar[(size_t)i * d + c] = (float)(s / (double)(r1 - r0));
        }
    }
}

/* X' = X - mu as binary32 values (one correctly rounded subtraction per element).  mu_per_block = 0: one
 * vector mu[d] for all rows (K smoothing); otherwise mu[i][d] for the rows of block i of `block` rows
 * (Q smoothing).                                                                                          */
void sage_oracle_smooth(const float *X, const float *mu, int mu_per_block, int N, int d, int block, float *out)
{
    for (int n = 0; n < N; ++n) {
        const float *m = mu + (mu_per_block ? (size_t)(n / block) * d : 0);
        for (int c = 0; c < d; ++c)
            out[(size_t)n * d + c] = X[(size_t)n * d + c] - m[c];
    }
}

/* Per-block integer quantisation with a symmetric range [-qmax, qmax] (Section 2.1: "INT4/INT8 with
 * per-block granularity", delta = max|X| / qmax with qmax = 127 printed for INT8; reading for INT4:
 * qmax = 7).  Same binary32 steps as sage_oracle_quant_int8: a = max|X'|, delta = a/qmax, r = qmax/a,
 * code = round(X' * r); X' = X - mu with mu as in sage_oracle_smooth (NULL: no smoothing).  The codes are
 * returned one per byte whatever qmax is.                                                                 */
void sage_oracle_quant_int(const float *X, const float *mu, int mu_per_block, int N, int d, int block,
                           int qmax, int8_t *codes, float *delta)
{
    int nb = (N + block - 1) / block;
    float fq = (float)qmax;
    for (int j = 0; j < nb; ++j) {
        int n0 = j * block;
        int n1 = n0 + block < N ? n0 + block : N;
        const float *m = mu ? mu + (mu_per_block ? (size_t)j * d : 0) : NULL;
        float a = 0.0f;
        for (int n = n0; n < n1; ++n)
            for (int c = 0; c < d; ++c) {
                float x = X[(size_t)n * d + c];
                if (m)
                    x = x - m[c];
                float ax = fabsf(x);
                if (ax > a)
                    a = ax;
            }
        if (a == 0.0f) {
            delta[j] = 0.0f;
            for (int n = n0; n < n1; ++n)
                memset(codes + (size_t)n * d, 0, (size_t)d);
            continue;
        }
        delta[j] = a / fq;
        float r = fq / a;
        for (int n = n0; n < n1; ++n)
            for (int c = 0; c < d; ++c) {
                float x = X[(size_t)n * d + c];
                if (m)
                    x = x - m[c];
                float y = x * r;
                codes[(size_t)n * d + c] = (int8_t)nearbyintf(y);
            }
    }
}

/* What smoothing of Q removes from the scores has to be put back (Section 3 keeps the smoothing of
 * SageAttention2; reading): with Q' = Q - qbar_i on block i,
 *     Q K'^T = Q' K'^T + qbar_i K'^T,
 * the first product is the quantised one and the second,
 *     dS[i][n] = sum_c qbar[i][c] * K'[n][c],        K' = K - mu_K (the smoothed, UNquantised keys),
 * is evaluated in full precision (double here) and added to the de-quantised scores.                      */
void sage_oracle_delta_s(const float *qbar, const float *Kp, int nQ, int N, int d, double *dS)
{
    for (int i = 0; i < nQ; ++i)
        for (int n = 0; n < N; ++n) {
            double s = 0.0;
            for (int c = 0; c < d; ++c)
                s += (double)qbar[(size_t)i * d + c] * (double)Kp[(size_t)n * d + c];
            dS[(size_t)i * N + n] = s;
        }
}

/* Per-channel FP8 quantisation of V (Section 2.1 and Eq. (2)):
 *   a_c = max_n |V[n][c]|,  delta_V[c] = a_c / V_r,  V^ = e4m3(V * (V_r/a_c)).
 * Codes are returned token-major, codes[n][c].                               */
void sage_oracle_quant_v(const float *V, int N, int d, float v_r, uint8_t *codes, float *delta)
{
    for (int c = 0; c < d; ++c) {
        float a = 0.0f;
        for (int n = 0; n < N; ++n) {
            float ax = fabsf(V[(size_t)n * d + c]);
            if (ax > a)
                a = ax;
        }
        if (a == 0.0f) {
            delta[c] = 0.0f;
            for (int n = 0; n < N; ++n)
                codes[(size_t)n * d + c] = 0;
            continue;
        }
        delta[c] = a / v_r;
        float r = v_r / a;
        for (int n = 0; n < N; ++n) {
            float y = V[(size_t)n * d + c] * r;
            codes[(size_t)n * d + c] = sage_oracle_e4m3_encode((double)y);
        }
    }
}

/* --------------------------------------------------------------------- */
/* attention stage                                                       */
/* --------------------------------------------------------------------- */

/* Quantised attention for the query rows [row0, row1) of ONE head
 * (Sections 2.1 and 3.1).  For every row r, key steps of W keys are taken in
 * ascending order; per step
 *     x_n   = S_int[r][n] * (delta_Q[r/BQ] * delta_K[n/BK] * sm_scale * log2 e)
 *     m'    = max(m, max_n x_n)            masked keys count as -inf
 *     alpha = 2^(m - m')
 *     P~_n  = 2^(x_n - m')                 masked keys give exactly 0
 *     l     = alpha*l + sum_n P~_n         (unquantised)
 *     P^_n  = e4m3(P~_n * P_r)
 *     acc   = alpha*acc + sum_n P^_n * V^[n][:]
 * and finally O[r][c] = acc[c] * delta_V[c] / (P_r * l), rounded to `out_dtype`
 * (0 fp16, 1 bf16, -1 no rounding).  For a causal row the loop stops after
 * the step that holds its last visible key: later steps are fully masked and
 * change nothing.
 *
 * Q has Nq rows, K and V have Nk rows (Nq = Nk for self-attention).  With a
 * causal mask and Nq != Nk the mask is aligned to the END of both sequences:
 * key n is visible to query r iff n <= r + (Nk - Nq), which needs Nk >= Nq.
 * Grouped-query attention is the caller's loop: several query heads use the
 * same quantised K, V head.
 *
 * P_out, if not NULL, receives the normalised probabilities 2^(x - m_final)/l
 * as (row1-row0) x Nk doubles (test use only: rows must sum to one).
 *
 * dS, if not NULL, is the score correction of the 4+8 variant (see sage_oracle_delta_s), [ceil(Nq/BQ)][Nk]
 * doubles in the units of Q K^T: the de-quantised score of (r, n) becomes
 *     S_int * delta_Q * delta_K + dS[r/BQ][n]      before the factor sm_scale * log2 e.
 * The integer codes may come from either quantiser (INT8 or INT4 range); nothing else differs.              */
void sage_oracle_attn_rows(const int8_t *Qc, const int8_t *Kc, const uint8_t *Vc,
                           const float *dq, const float *dk, const float *dv,
                           int Nq, int Nk, int d, int causal, double sm_scale, double p_r,
                           int BQ, int BK, int W, int row0, int row1, int out_dtype,
                           double *out, double *P_out, const double *dS)
{
    const int N = Nk;
    const int shift = Nk - Nq; /* causal alignment */
    (void)Nq;
    double *Vd = (double *)malloc((size_t)N * d * sizeof(double));
    for (size_t i = 0; i < (size_t)N * d; ++i)
        Vd[i] = sage_oracle_e4m3_decode(Vc[i]);

#pragma omp parallel
    {
        double *x = (double *)malloc((size_t)W * sizeof(double));
        double *acc = (double *)malloc((size_t)d * sizeof(double));
        double *xs = P_out ? (double *)malloc((size_t)N * sizeof(double)) : NULL;
#pragma omp for schedule(dynamic, 1)
        for (int r = row0; r < row1; ++r) {
            const int8_t *qr = Qc + (size_t)r * d;
            double m = -INFINITY, l = 0.0;
            for (int c = 0; c < d; ++c)
                acc[c] = 0.0;
            int last = causal ? r + shift : N - 1;
            for (int t0 = 0; t0 <= last; t0 += W) {
                int t1 = t0 + W < N ? t0 + W : N;
                double mx = -INFINITY;
                for (int n = t0; n < t1; ++n) {
                    if (causal && n > r + shift) {
                        x[n - t0] = -INFINITY;
                        continue;
                    }
                    const int8_t *kn = Kc + (size_t)n * d;
                    int32_t s = 0;
                    for (int c = 0; c < d; ++c)
                        s += (int32_t)qr[c] * (int32_t)kn[c];
                    double cst = (double)dq[r / BQ] * (double)dk[n / BK] * sm_scale * SAGE_ORACLE_LOG2E;
                    x[n - t0] = (double)s * cst;
                    if (dS)
                        x[n - t0] += dS[(size_t)(r / BQ) * N + n] * (sm_scale * SAGE_ORACLE_LOG2E);
                    if (x[n - t0] > mx)
                        mx = x[n - t0];
                }
                double m_new = m > mx ? m : mx;
                double alpha = exp2(m - m_new); /* m = -inf on the first step gives 0 */
                l *= alpha;
                for (int c = 0; c < d; ++c)
                    acc[c] *= alpha;
                for (int n = t0; n < t1; ++n) {
                    double p = isinf(x[n - t0]) ? 0.0 : exp2(x[n - t0] - m_new);
                    l += p;
                    double ph = sage_oracle_e4m3_decode(sage_oracle_e4m3_encode(p * p_r));
                    if (ph != 0.0) {
                        const double *vn = Vd + (size_t)n * d;
                        for (int c = 0; c < d; ++c)
                            acc[c] += ph * vn[c];
                    }
                    if (xs)
                        xs[n] = x[n - t0];
                }
                m = m_new;
            }
            for (int c = 0; c < d; ++c) {
                double o = acc[c] * (double)dv[c] / (p_r * l);
                out[(size_t)(r - row0) * d + c] = out_dtype < 0 ? o : sage_oracle_round16(o, out_dtype);
            }
            if (P_out) {
                double *pr = P_out + (size_t)(r - row0) * N;
                for (int n = 0; n < N; ++n)
                    pr[n] = (n <= last && !isinf(xs[n])) ? exp2(xs[n] - m) / l : 0.0;
            }
        }
        free(x);
        free(acc);
        free(xs);
    }
    free(Vd);
}

/* Key-split evaluation of the same attention (not in the paper; the decode-shaped path of the library).
 * The keys are cut into ranges of `split_keys` keys (a multiple of W).  For every row and every range the
 * recurrence of sage_oracle_attn_rows is run on the keys of that range alone, from m = -inf, l = 0,
 * acc = 0 -- so P~ is taken against the running maximum of the RANGE before its FP8 rounding, which is what
 * makes this a mode of its own and not a reordering -- and gives (m_s, l_s, acc_s).  The ranges are then
 * combined the way two partial softmax sums always combine:
 *     m = max_s m_s,   l = sum_s 2^(m_s - m) l_s,   acc = sum_s 2^(m_s - m) acc_s,
 *     O[r][c] = acc[c] * delta_V[c] / (P_r * l),
 * a range in which the row sees no key (causal mask) contributing nothing.  With split_keys >= Nk this is
 * sage_oracle_attn_rows.  Arguments as there (no P_out, no dS).                                           */
void sage_oracle_attn_rows_split(const int8_t *Qc, const int8_t *Kc, const uint8_t *Vc,
                                 const float *dq, const float *dk, const float *dv,
                                 int Nq, int Nk, int d, int causal, double sm_scale, double p_r,
                                 int BQ, int BK, int W, int split_keys, int row0, int row1, int out_dtype,
                                 double *out)
{
    const int N = Nk;
    const int shift = Nk - Nq;
    (void)Nq;
    double *Vd = (double *)malloc((size_t)N * d * sizeof(double));
    for (size_t i = 0; i < (size_t)N * d; ++i)
        Vd[i] = sage_oracle_e4m3_decode(Vc[i]);

#pragma omp parallel
    {
        double *x = (double *)malloc((size_t)W * sizeof(double));
        double *acc = (double *)malloc((size_t)d * sizeof(double));   /* of the current range */
        double *tot = (double *)malloc((size_t)d * sizeof(double));   /* combined so far */
#pragma omp for schedule(dynamic, 1)
        for (int r = row0; r < row1; ++r) {
            const int8_t *qr = Qc + (size_t)r * d;
            int last = causal ? r + shift : N - 1;
            double M = -INFINITY, L = 0.0;
            for (int c = 0; c < d; ++c)
                tot[c] = 0.0;
            for (int k0 = 0; k0 <= last; k0 += split_keys) {
                int k1 = k0 + split_keys < N ? k0 + split_keys : N;
                double m = -INFINITY, l = 0.0;
                for (int c = 0; c < d; ++c)
                    acc[c] = 0.0;
                for (int t0 = k0; t0 < k1 && t0 <= last; t0 += W) {
                    int t1 = t0 + W < k1 ? t0 + W : k1;
                    double mx = -INFINITY;
                    for (int n = t0; n < t1; ++n) {
                        if (n > last) {
                            x[n - t0] = -INFINITY;
                            continue;
                        }
                        const int8_t *kn = Kc + (size_t)n * d;
                        int32_t s = 0;
                        for (int c = 0; c < d; ++c)
                            s += (int32_t)qr[c] * (int32_t)kn[c];
                        x[n - t0] = (double)s * ((double)dq[r / BQ] * (double)dk[n / BK] * sm_scale * SAGE_ORACLE_LOG2E);
                        if (x[n - t0] > mx)
                            mx = x[n - t0];
                    }
                    double m_new = m > mx ? m : mx;   /* finite: key t0 <= last is visible */
                    double alpha = exp2(m - m_new);
                    l *= alpha;
                    for (int c = 0; c < d; ++c)
                        acc[c] *= alpha;
                    for (int n = t0; n < t1; ++n) {
                        double p = isinf(x[n - t0]) ? 0.0 : exp2(x[n - t0] - m_new);
                        l += p;
                        double ph = sage_oracle_e4m3_decode(sage_oracle_e4m3_encode(p * p_r));
                        if (ph != 0.0) {
                            const double *vn = Vd + (size_t)n * d;
                            for (int c = 0; c < d; ++c)
                                acc[c] += ph * vn[c];
                        }
                    }
                    m = m_new;
                }
                /* combine the range with what came before */
                double Mn = M > m ? M : m;
                double a = exp2(M - Mn), b = exp2(m - Mn);   /* M = -inf for the first range gives a = 0 */
                L = a * L + b * l;
                for (int c = 0; c < d; ++c)
                    tot[c] = a * tot[c] + b * acc[c];
                M = Mn;
            }
            for (int c = 0; c < d; ++c) {
                double o = tot[c] * (double)dv[c] / (p_r * L);
                out[(size_t)(r - row0) * d + c] = out_dtype < 0 ? o : sage_oracle_round16(o, out_dtype);
            }
        }
        free(x);
        free(acc);
        free(tot);
    }
    free(Vd);
}

/* Study variant of sage_oracle_attn_rows: Section 3.1, Eq. (2) read literally.  There the scale of P~ is
 * taken per block, delta_P = max(P~) / P_r, a block of P~ being one Q block (BQ rows) times one key step
 * (W keys); the routine above uses the constant delta_P = 1 / P_r instead (P~ <= 1 by construction, and a
 * block's maximum IS 1 whenever one of its rows finds its running maximum in that step).  Here, per
 * Q block and key step,
 *     b     = max over the block's rows and visible keys of P~      (0 < b <= 1; b = 0: nothing visible)
 *     P^_n  = e4m3(P~_n * P_r / b)                                  i.e. P~ / delta_P with delta_P = b / P_r
 *     acc   = alpha*acc + b * sum_n P^_n * V^[n][:]                 i.e. P^ V^ * delta_P, P_r divided out at the end
 * everything else as above (m, alpha, l per row; l from the unquantised P~).  The block maximum couples the
 * rows of a Q block, so whole Q blocks are evaluated even if only rows [row0, row1) are returned.
 * This mode exists to measure what the static scale costs or gains; the GPU library does not implement it. */
void sage_oracle_attn_rows_blockmax(const int8_t *Qc, const int8_t *Kc, const uint8_t *Vc,
                                    const float *dq, const float *dk, const float *dv,
                                    int Nq, int Nk, int d, int causal, double sm_scale, double p_r,
                                    int BQ, int BK, int W, int row0, int row1, int out_dtype, double *out)
{
    const int N = Nk;
    const int shift = Nk - Nq;
    double *Vd = (double *)malloc((size_t)N * d * sizeof(double));
    for (size_t i = 0; i < (size_t)N * d; ++i)
        Vd[i] = sage_oracle_e4m3_decode(Vc[i]);
    int blk0 = row0 / BQ, blk1 = (row1 + BQ - 1) / BQ;

#pragma omp parallel
    {
        double *x = (double *)malloc((size_t)BQ * W * sizeof(double));   /* scores, then P~, of one block */
        double *acc = (double *)malloc((size_t)BQ * d * sizeof(double));
        double *m = (double *)malloc((size_t)BQ * sizeof(double));
        double *l = (double *)malloc((size_t)BQ * sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int i = blk0; i < blk1; ++i) {
            int r0 = i * BQ;
            int r1 = r0 + BQ < Nq ? r0 + BQ : Nq;
            int rows = r1 - r0;
            for (int a = 0; a < rows; ++a) {
                m[a] = -INFINITY;
                l[a] = 0.0;
                for (int c = 0; c < d; ++c)
                    acc[(size_t)a * d + c] = 0.0;
            }
            int last = causal ? (r1 - 1) + shift : N - 1;  /* last key any row of the block sees */
            for (int t0 = 0; t0 <= last; t0 += W) {
                int t1 = t0 + W < N ? t0 + W : N;
                double b = 0.0;
                for (int a = 0; a < rows; ++a) {
                    int r = r0 + a;
                    const int8_t *qr = Qc + (size_t)r * d;
                    double *xa = x + (size_t)a * W;
                    double mx = -INFINITY;
                    for (int n = t0; n < t1; ++n) {
                        if (causal && n > r + shift) {
                            xa[n - t0] = -INFINITY;
                            continue;
                        }
                        const int8_t *kn = Kc + (size_t)n * d;
                        int32_t s = 0;
                        for (int c = 0; c < d; ++c)
                            s += (int32_t)qr[c] * (int32_t)kn[c];
                        double cst = (double)dq[r / BQ] * (double)dk[n / BK] * sm_scale * SAGE_ORACLE_LOG2E;
                        xa[n - t0] = (double)s * cst;
                        if (xa[n - t0] > mx)
                            mx = xa[n - t0];
                    }
                    double m_new = m[a] > mx ? m[a] : mx;
                    /* a row with nothing visible yet keeps m = -inf: alpha is irrelevant (l = acc = 0) */
                    double alpha = isinf(m_new) ? 1.0 : exp2(m[a] - m_new);
                    l[a] *= alpha;
                    for (int c = 0; c < d; ++c)
                        acc[(size_t)a * d + c] *= alpha;
                    for (int n = t0; n < t1; ++n) {
                        double p = isinf(xa[n - t0]) ? 0.0 : exp2(xa[n - t0] - m_new);
                        xa[n - t0] = p;       /* the block of P~ */
                        l[a] += p;
                        if (p > b)
                            b = p;
                    }
                    m[a] = m_new;
                }
                if (b == 0.0)
                    continue;
                for (int a = 0; a < rows; ++a) {
                    const double *xa = x + (size_t)a * W;
                    for (int n = t0; n < t1; ++n) {
                        double ph = sage_oracle_e4m3_decode(sage_oracle_e4m3_encode(xa[n - t0] * p_r / b));
                        if (ph != 0.0) {
                            const double *vn = Vd + (size_t)n * d;
                            for (int c = 0; c < d; ++c)
                                acc[(size_t)a * d + c] += b * ph * vn[c];
                        }
                    }
                }
            }
            for (int a = 0; a < rows; ++a) {
                int r = r0 + a;
                if (r < row0 || r >= row1)
                    continue;
                for (int c = 0; c < d; ++c) {
                    double o = acc[(size_t)a * d + c] * (double)dv[c] / (p_r * l[a]);
                    out[(size_t)(r - row0) * d + c] = out_dtype < 0 ? o : sage_oracle_round16(o, out_dtype);
                }
            }
        }
        free(x);
        free(acc);
        free(m);
        free(l);
    }
    free(Vd);
}

/* The same block-wise online softmax on UNQUANTISED double operands
 * (Section 2.1 without any quantiser: P^ := P~, all scales 1).  It exists so
 * that the tiling / online-softmax skeleton can be pinned against the plain
 * definition softmax(Q K^T * sm_scale) V.                                     */
void sage_oracle_attn_rows_fp(const double *Q, const double *K, const double *V,
                              int Nq, int Nk, int d, int causal, double sm_scale, int W,
                              int row0, int row1, double *out, double *P_out)
{
    const int N = Nk;
    const int shift = Nk - Nq; /* causal alignment, as above */
    (void)Nq;
#pragma omp parallel
    {
        double *x = (double *)malloc((size_t)W * sizeof(double));
        double *acc = (double *)malloc((size_t)d * sizeof(double));
        double *xs = P_out ? (double *)malloc((size_t)N * sizeof(double)) : NULL;
#pragma omp for schedule(dynamic, 1)
        for (int r = row0; r < row1; ++r) {
            const double *qr = Q + (size_t)r * d;
            double m = -INFINITY, l = 0.0;
            for (int c = 0; c < d; ++c)
                acc[c] = 0.0;
            int last = causal ? r + shift : N - 1;
            for (int t0 = 0; t0 <= last; t0 += W) {
                int t1 = t0 + W < N ? t0 + W : N;
                double mx = -INFINITY;
                for (int n = t0; n < t1; ++n) {
                    if (causal && n > r + shift) {
                        x[n - t0] = -INFINITY;
                        continue;
                    }
                    const double *kn = K + (size_t)n * d;
                    double s = 0.0;
                    for (int c = 0; c < d; ++c)
                        s += qr[c] * kn[c];
                    x[n - t0] = s * sm_scale * SAGE_ORACLE_LOG2E;
                    if (x[n - t0] > mx)
                        mx = x[n - t0];
                }
                double m_new = m > mx ? m : mx;
                double alpha = exp2(m - m_new);
                l *= alpha;
                for (int c = 0; c < d; ++c)
                    acc[c] *= alpha;
                for (int n = t0; n < t1; ++n) {
                    double p = isinf(x[n - t0]) ? 0.0 : exp2(x[n - t0] - m_new);
                    l += p;
                    const double *vn = V + (size_t)n * d;
                    for (int c = 0; c < d; ++c)
                        acc[c] += p * vn[c];
                    if (xs)
                        xs[n] = x[n - t0];
                }
                m = m_new;
            }
            for (int c = 0; c < d; ++c)
                out[(size_t)(r - row0) * d + c] = acc[c] / l;
            if (P_out) {
                double *pr = P_out + (size_t)(r - row0) * N;
                for (int n = 0; n < N; ++n)
                    pr[n] = (n <= last && !isinf(xs[n])) ? exp2(xs[n] - m) / l : 0.0;
            }
        }
        free(x);
        free(acc);
        free(xs);
    }
}

int sage_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
