/*
 * swaa_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain fp64 CPU definition of sliding-window attention with "keep first k"
 * sink tokens (paper Sec. 1: each token attends to a fixed-size local window;
 * Sec. 3.2.1 and Fig. 1b: every later token attends to its local window AND
 * the initial k tokens; Sec. 4.1.2: a window at least as long as the context
 * is full causal attention).  It exists only so that tests, the smoke check
 * and the benchmark's cpu_baseline leg have an independent answer to compare
 * the GPU library with.  It shares no code with the GPU path and is never
 * called by it.
 *
 * For batch b, query head h, KV head g = h / (Hq/Hkv), query row i:
 *
 *   Vis(i) = { j : 0 <= j <= i  and  ( j > i - W  or  j < S ) }   (a set)
 *   s_j    = scale * sum_d q[b,h,i,d] * k[b,g,j,d]
 *   m      = max_{j in Vis(i)} s_j
 *   lse    = m + ln sum_{j in Vis(i)} exp(s_j - m)                (natural log)
 *   o[d]   = sum_{j in Vis(i)} exp(s_j - lse) * v[b,g,j,d]
 *
 * Inputs are bf16 bit patterns (uint16; binary16 after swaa_oracle_set_format(1)),
 * widened exactly to double; all
 * arithmetic is double; outputs are double and are not rounded.  There is no
 * tiling, no running maximum and no reordering: three passes over the
 * explicit visible set, exactly as written above.  Rows are independent, so
 * the only parallelism is an OpenMP loop over (b, h, row).
 *
 * FA Decode (paper Sec. 3.1.1, Fig. 1a): the window applies to prompt tokens
 * only; a generated token attends to every earlier token.  With P = n_prompt,
 * rows i >= P therefore have Vis(i) = { j : 0 <= j <= i }.  P = N is the pure
 * prefill mask above, P = 0 is full causal attention.
 *
 * Readings where the paper is silent: the window (i-W, i] holds W keys and
 * includes the query itself; a key that is both a sink and in the window is
 * counted once; sinks are causal (row i < S sees only [0, i]); the
 * logsumexp is natural-log of the scaled scores.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/*
 * Input element format: 0 = bfloat16 (the library's main path), 1 = IEEE binary16
 * (the precision the paper serves its models in, Sec. 4.1.1).  A process-wide
 * setting of this test helper; set it before a call, not during one.
 */
static int g_format = 0;

int swaa_oracle_set_format(int format)
{
    if (format != 0 && format != 1)
        return -1;
    g_format = format;
    return 0;
}

/* binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits, written out from the format. */
static double f16_to_double(uint16_t bits)
{
    const int sign = bits >> 15, e = (bits >> 10) & 0x1f, frac = bits & 0x3ff;
    double x;
    if (e == 0)
        x = ldexp((double)frac, -24); /* zero and subnormals: frac * 2^-10 * 2^-14 */
    else if (e == 31)
        x = frac ? NAN : INFINITY;
    else
        x = ldexp(1.0 + (double)frac / 1024.0, e - 15);
    return sign ? -x : x;
}

static double bf16_to_double(uint16_t bits)
{
    if (g_format == 1)
        return f16_to_double(bits);
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* The decoder on its own (for the tests that pin it). */
void swaa_oracle_decode_elems(const uint16_t *bits, long n, double *out)
{
    for (long i = 0; i < n; i++)
        out[i] = bf16_to_double(bits[i]);
}

/* 1 if key j is visible from query i under (window W, sinks S), when the
 * first P rows are prompt tokens and the rest are generated tokens. */
static int visible(long i, long j, long W, long S, long P)
{
    if (j < 0 || j > i)
        return 0; /* causal */
    if (i >= P)
        return 1; /* a generated token sees everything before it */
    return (j > i - W) || (j < S);
}

int swaa_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Evaluate rows `rows[0..n_rows)` (NULL: every row 0..N-1, n_rows ignored) of
 * every (b, h).  out: [B, Hq, R, D] doubles, lse: [B, Hq, R] doubles, with
 * R = n_rows (or N).  P = n_prompt: rows >= P are generated tokens (any P >= N
 * means there are none).  n_threads <= 0 keeps the OpenMP default.
 * Returns 0, or -1 on a bad argument, -2 when out of memory.
 */
int swaa_oracle_rows_mixed(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                           int B, int Hq, int Hkv, int N, int D, long W, long S,
                           long P, double scale, const int *rows, int n_rows,
                           double *out, double *lse, int n_threads)
{
    if (!q || !k || !v || !out || !lse)
        return -1;
    if (B < 1 || Hq < 1 || Hkv < 1 || N < 1 || D < 1 || Hq % Hkv || W < 1 || S < 0 || P < 0)
        return -1;
    const long R = rows ? n_rows : N;
    if (R < 0)
        return -1;
    for (long r = 0; rows && r < R; r++)
        if (rows[r] < 0 || rows[r] >= N)
            return -1;
    const int G = Hq / Hkv;
    const long total = (long)B * Hq * R;
    int failed = 0;
#ifdef _OPENMP
    if (n_threads > 0)
        omp_set_num_threads(n_threads);
#else
    (void)n_threads;
#endif

#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)N);
        double *qi = (double *)malloc(sizeof(double) * (size_t)D);
        if (!s || !qi) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (long t = 0; t < total; t++) {
            if (!s || !qi)
                continue;
            const long r = t % R;
            const long h = (t / R) % Hq;
            const long b = t / (R * Hq);
            const long g = h / G;
            const long i = rows ? rows[r] : r;
            const uint16_t *qrow = q + (((size_t)b * Hq + h) * N + i) * D;
            const uint16_t *kb = k + ((size_t)b * Hkv + g) * (size_t)N * D;
            const uint16_t *vb = v + ((size_t)b * Hkv + g) * (size_t)N * D;
            double *o = out + (size_t)t * D;
            for (int d = 0; d < D; d++)
                qi[d] = bf16_to_double(qrow[d]);

            /* scores and their maximum over the visible set */
            double m = -INFINITY;
            for (long j = 0; j <= i; j++) {
                if (!visible(i, j, W, S, P))
                    continue;
                const uint16_t *kr = kb + (size_t)j * D;
                double acc = 0.0;
                for (int d = 0; d < D; d++)
                    acc += qi[d] * bf16_to_double(kr[d]);
                s[j] = scale * acc;
                if (s[j] > m)
                    m = s[j];
            }
            /* normaliser */
            double l = 0.0;
            for (long j = 0; j <= i; j++)
                if (visible(i, j, W, S, P))
                    l += exp(s[j] - m);
            const double lse_i = m + log(l);
            lse[t] = lse_i;
            /* weighted sum of value rows */
            for (int d = 0; d < D; d++)
                o[d] = 0.0;
            for (long j = 0; j <= i; j++) {
                if (!visible(i, j, W, S, P))
                    continue;
                const double p = exp(s[j] - lse_i);
                const uint16_t *vr = vb + (size_t)j * D;
                for (int d = 0; d < D; d++)
                    o[d] += p * bf16_to_double(vr[d]);
            }
        }
        free(s);
        free(qi);
    }
    return failed ? -2 : 0;
}

/* The pure prefill mask: every row is a prompt token. */
int swaa_oracle_rows(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                     int B, int Hq, int Hkv, int N, int D, long W, long S,
                     double scale, const int *rows, int n_rows, double *out,
                     double *lse, int n_threads)
{
    return swaa_oracle_rows_mixed(q, k, v, B, Hq, Hkv, N, D, W, S, (long)N, scale,
                                  rows, n_rows, out, lse, n_threads);
}

/*
 * Decode shape (paper Sec. 3.1.1: during auto-regressive generation a token
 * attends to the cached keys and values of the tokens before it -- all of them
 * under FA Decode, i.e. W >= Nk, or its window plus the sinks when decoding
 * stays on sliding-window attention).  The Nq query rows are the newest
 * tokens of a sequence of Nk: row r sits at position Nk - Nq + r, and the
 * cache k, v [B, Hkv, Nk, D] already holds their own keys and values.
 *
 *   Vis(r) = { j : 0 <= j <= pos and ( j > pos - W or j < S ) },  pos = Nk - Nq + r
 *
 * The same shape is a chunk of a longer prefill (the Nq rows are the next
 * chunk of the prompt, the cache holds the chunks before it); P is the prompt
 * length as in swaa_oracle_rows_mixed: a row whose position is >= P is a
 * generated token and sees every key up to its own (P > Nk: there is none).
 *
 * q: [B, Hq, Nq, D] bf16 bits; out: [B, Hq, Nq, D] doubles; lse: [B, Hq, Nq].
 * Returns 0, or -1 on a bad argument, -2 when out of memory.
 */
int swaa_oracle_decode(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                       int B, int Hq, int Hkv, int Nq, int Nk, int D, long W, long S,
                       long P, double scale, double *out, double *lse, int n_threads)
{
    if (!q || !k || !v || !out || !lse)
        return -1;
    if (B < 1 || Hq < 1 || Hkv < 1 || Nq < 1 || Nk < Nq || D < 1 || Hq % Hkv || W < 1 || S < 0 || P < 0)
        return -1;
    const int G = Hq / Hkv;
    const long total = (long)B * Hq * Nq;
    const long never_generated = P;
    int failed = 0;
#ifdef _OPENMP
    if (n_threads > 0)
        omp_set_num_threads(n_threads);
#else
    (void)n_threads;
#endif

#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)Nk);
        if (!s) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (long t = 0; t < total; t++) {
            if (!s)
                continue;
            const long r = t % Nq;
            const long h = (t / Nq) % Hq;
            const long b = t / ((long)Nq * Hq);
            const long g = h / G;
            const long pos = (long)Nk - Nq + r;
            const uint16_t *qrow = q + (size_t)t * D;
            const uint16_t *kb = k + ((size_t)b * Hkv + g) * (size_t)Nk * D;
            const uint16_t *vb = v + ((size_t)b * Hkv + g) * (size_t)Nk * D;
            double *o = out + (size_t)t * D;

            double m = -INFINITY;
            for (long j = 0; j < Nk; j++) {
                if (!visible(pos, j, W, S, never_generated))
                    continue;
                double acc = 0.0;
                for (int d = 0; d < D; d++)
                    acc += bf16_to_double(qrow[d]) * bf16_to_double(kb[(size_t)j * D + d]);
                s[j] = scale * acc;
                if (s[j] > m)
                    m = s[j];
            }
            double l = 0.0;
            for (long j = 0; j < Nk; j++)
                if (visible(pos, j, W, S, never_generated))
                    l += exp(s[j] - m);
            const double lse_r = m + log(l);
            lse[t] = lse_r;
            for (int d = 0; d < D; d++)
                o[d] = 0.0;
            for (long j = 0; j < Nk; j++) {
                if (!visible(pos, j, W, S, never_generated))
                    continue;
                const double p = exp(s[j] - lse_r);
                for (int d = 0; d < D; d++)
                    o[d] += p * bf16_to_double(vb[(size_t)j * D + d]);
            }
        }
        free(s);
    }
    return failed ? -2 : 0;
}

/*
 * Backward pass of the one-pass forward above (SWA-aware fine-tuning, paper
 * Sec. 3.2.2, trains through this mask).  With p_ij = exp(s_ij - lse_i) on
 * Vis(i) (0 elsewhere) and the upstream gradient dO:
 *
 *   dV_j = sum_i p_ij dO_i
 *   dP_ij = <dO_i, v_j>,   delta_i = sum_j p_ij dP_ij
 *   dS_ij = p_ij (dP_ij - delta_i)
 *   dQ_i = scale * sum_j dS_ij k_j,     dK_j = scale * sum_i dS_ij q_i
 *
 * (the derivative of softmax followed by the two products, written out; dK and
 * dV of a KV head sum over the Hq/Hkv query heads that read it).  Two passes,
 * each a plain loop: rows i for lse, delta and dQ; then key rows j for dK and
 * dV, recomputing p_ij from the stored lse_i.  All arithmetic in double.
 *
 * dout: [B, Hq, N, D] bf16 bits.  dq: [B, Hq, N, D], dk, dv: [B, Hkv, N, D]
 * doubles.  Returns 0, -1 on a bad argument, -2 when out of memory.
 */
int swaa_oracle_bwd(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                    const uint16_t *dout, int B, int Hq, int Hkv, int N, int D,
                    long W, long S, long P, double scale, double *dq, double *dk,
                    double *dv, int n_threads)
{
    if (!q || !k || !v || !dout || !dq || !dk || !dv)
        return -1;
    if (B < 1 || Hq < 1 || Hkv < 1 || N < 1 || D < 1 || Hq % Hkv || W < 1 || S < 0 || P < 0)
        return -1;
    const int G = Hq / Hkv;
    const long rows = (long)B * Hq * N;
    double *lse = (double *)malloc(sizeof(double) * (size_t)rows);
    double *delta = (double *)malloc(sizeof(double) * (size_t)rows);
    if (!lse || !delta) {
        free(lse);
        free(delta);
        return -2;
    }
    int failed = 0;
#ifdef _OPENMP
    if (n_threads > 0)
        omp_set_num_threads(n_threads);
#else
    (void)n_threads;
#endif

    /* pass 1: per query row */
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)N);
        double *dp = (double *)malloc(sizeof(double) * (size_t)N);
        if (!s || !dp) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (long t = 0; t < rows; t++) {
            if (!s || !dp)
                continue;
            const long i = t % N;
            const long h = (t / N) % Hq;
            const long b = t / ((long)N * Hq);
            const long g = h / G;
            const uint16_t *qi = q + (size_t)t * D;
            const uint16_t *doi = dout + (size_t)t * D;
            const uint16_t *kb = k + ((size_t)b * Hkv + g) * (size_t)N * D;
            const uint16_t *vb = v + ((size_t)b * Hkv + g) * (size_t)N * D;
            double m = -INFINITY;
            for (long j = 0; j <= i; j++) {
                if (!visible(i, j, W, S, P))
                    continue;
                double a = 0.0, c = 0.0;
                for (int d = 0; d < D; d++) {
                    a += bf16_to_double(qi[d]) * bf16_to_double(kb[(size_t)j * D + d]);
                    c += bf16_to_double(doi[d]) * bf16_to_double(vb[(size_t)j * D + d]);
                }
                s[j] = scale * a;
                dp[j] = c;
                if (s[j] > m)
                    m = s[j];
            }
            double l = 0.0;
            for (long j = 0; j <= i; j++)
                if (visible(i, j, W, S, P))
                    l += exp(s[j] - m);
            const double lse_i = m + log(l);
            double del = 0.0;
            for (long j = 0; j <= i; j++)
                if (visible(i, j, W, S, P))
                    del += exp(s[j] - lse_i) * dp[j];
            lse[t] = lse_i;
            delta[t] = del;
            double *dqi = dq + (size_t)t * D;
            for (int d = 0; d < D; d++)
                dqi[d] = 0.0;
            for (long j = 0; j <= i; j++) {
                if (!visible(i, j, W, S, P))
                    continue;
                const double ds = exp(s[j] - lse_i) * (dp[j] - del);
                for (int d = 0; d < D; d++)
                    dqi[d] += scale * ds * bf16_to_double(kb[(size_t)j * D + d]);
            }
        }
        free(s);
        free(dp);
    }

    /* pass 2: per key row */
    const long krows = (long)B * Hkv * N;
#pragma omp parallel for schedule(dynamic, 1)
    for (long t = 0; t < krows; t++) {
        const long j = t % N;
        const long g = (t / N) % Hkv;
        const long b = t / ((long)N * Hkv);
        const uint16_t *kj = k + (size_t)t * D;
        const uint16_t *vj = v + (size_t)t * D;
        double *dkj = dk + (size_t)t * D;
        double *dvj = dv + (size_t)t * D;
        for (int d = 0; d < D; d++) {
            dkj[d] = 0.0;
            dvj[d] = 0.0;
        }
        for (long h = g * G; h < (g + 1) * G; h++) {
            for (long i = j; i < N; i++) {
                if (!visible(i, j, W, S, P))
                    continue;
                const size_t r = ((size_t)b * Hq + h) * (size_t)N + i;
                const uint16_t *qi = q + r * D;
                const uint16_t *doi = dout + r * D;
                double a = 0.0, c = 0.0;
                for (int d = 0; d < D; d++) {
                    a += bf16_to_double(qi[d]) * bf16_to_double(kj[d]);
                    c += bf16_to_double(doi[d]) * bf16_to_double(vj[d]);
                }
                const double p = exp(scale * a - lse[r]);
                const double ds = p * (c - delta[r]);
                for (int d = 0; d < D; d++) {
                    dvj[d] += p * bf16_to_double(doi[d]);
                    dkj[d] += scale * ds * bf16_to_double(qi[d]);
                }
            }
        }
    }
    free(lse);
    free(delta);
    return failed ? -2 : 0;
}
