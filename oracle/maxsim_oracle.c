/*
 * MaxSim CPU oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, obviously-correct fp64 loop implementation of what the GPU
 * library computes.  Only the test-suite, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the GPU path shares no code with this file
 * and never falls back to it.
 *
 * What it follows in the paper ("Flash-MaxSim"):
 *   - forward score      : Eq. 1  (score = sum_i max_j <Q_i, D_j>) and the
 *                          naive definition of Listing 1 / Alg. 3;
 *                          Prop. 1 says the fused kernel reaches exactly this
 *                          value up to floating-point evaluation order, so
 *                          the oracle is the definition itself.
 *   - tie rule           : "Tied maxima" paragraph (first occurrence wins).
 *   - backward           : Eqs. 2-3 and Alg. 2 (routing through the stored
 *                          argmax), dQ gather and dD scatter.
 *   - int8 scoring       : Sec. "Quantised Scoring" and Alg. 4 (integer dot
 *                          product, per-token scales applied per output cell
 *                          before the row max).
 *   - quantiser          : Sec. "Quantised Scoring" (per-token symmetric
 *                          absmax).  The paper does not state rounding or
 *                          clamping; this file fixes: scale = absmax/127,
 *                          round-half-to-even, clamp to [-127,127], an
 *                          all-zero row gets scale 0 and codes 0.
 *   - contrastive loss   : in-batch negatives (Sec. 2.1 / training step
 *                          experiment); the paper leaves the loss open, this
 *                          file fixes softmax cross-entropy with temperature
 *                          tau, label of query i = document i, mean over
 *                          queries.
 *
 * Pins (tests/test_oracle_*.py, run without a GPU): brute force over a
 * materialised similarity tensor, the closed form at L_d = 1, permutation
 * invariance over document tokens, D containing Q with unit-norm rows,
 * chunk additivity over query tokens, finite differences and the Euler
 * identity for the backward, exact integer cases for int8, the dequantised
 * float identity of App. "INT8 Kernel", and exhaustive comparison of the
 * hand-written fp16/bf16 decoders against numpy/torch conversions.
 * Nothing in this file is "parity unpinned".
 *
 * Arithmetic: every input element is decoded exactly to double; dot products
 * are accumulated in double with k ascending; compile with
 * -ffp-contract=off so no fused multiply-add changes the rounding.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_F16 = 1, ORACLE_BF16 = 2 };

/* ---------- exact decoders (written out by hand; IEEE 754 binary16 and
 * bfloat16 = upper 16 bits of binary32) ---------- */

double oracle_decode_f16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24); /* subnormal: m * 2^-10 * 2^-14 */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)m / 1024.0, e - 15);
    return sign ? -v : v;
}

double oracle_decode_bf16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 7) & 0xff;
    int m = h & 0x7f;
    double v;
    if (e == 0)
        v = ldexp((double)m, -133); /* subnormal: m * 2^-7 * 2^-126 */
    else if (e == 255)
        v = m ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)m / 128.0, e - 127);
    return sign ? -v : v;
}

static double load_elem(const void *p, int dtype, int64_t idx)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)p)[idx];
    if (dtype == ORACLE_F16)
        return oracle_decode_f16(((const uint16_t *)p)[idx]);
    return oracle_decode_bf16(((const uint16_t *)p)[idx]);
}

static double *decode_block(const void *p, int dtype, int64_t first, int64_t count)
{
    double *out = (double *)malloc(sizeof(double) * (size_t)(count > 0 ? count : 1));
    if (!out)
        return NULL;
    for (int64_t i = 0; i < count; ++i)
        out[i] = load_elem(p, dtype, first + i);
    return out;
}

/* ---------- forward: Eq. 1, one (query, document) pair at a time ---------- */

typedef struct {
    const double *Q; /* [n_q, l_q, d] decoded */
    const void *D;
    const int32_t *offsets; /* NULL => uniform */
    int n_q, l_q, l_d, d, dtype;
    int64_t b;
    double *scores;  /* [n_q, b] */
    int32_t *argmax; /* [n_q, b, l_q] or NULL */
    double *margin;  /* [n_q, b, l_q] or NULL */
    int tid, n_threads;
    int failed;
} fwd_job;

static void *fwd_worker(void *arg)
{
    fwd_job *J = (fwd_job *)arg;
    const int d = J->d, l_q = J->l_q;
    for (int64_t doc = J->tid; doc < J->b; doc += J->n_threads) {
        int64_t first_tok, n_tok;
        if (J->offsets) {
            first_tok = J->offsets[doc];
            n_tok = (int64_t)J->offsets[doc + 1] - first_tok;
        } else {
            first_tok = doc * (int64_t)J->l_d;
            n_tok = J->l_d;
        }
        double *Dd = decode_block(J->D, J->dtype, first_tok * d, n_tok * d);
        if (!Dd) {
            J->failed = 1;
            return NULL;
        }
        for (int q = 0; q < J->n_q; ++q) {
            double score = 0.0;
            for (int i = 0; i < l_q; ++i) {
                const double *qi = J->Q + ((int64_t)q * l_q + i) * d;
                double best = -INFINITY, second = -INFINITY;
                int32_t arg = -1;
                for (int64_t j = 0; j < n_tok; ++j) {
                    const double *dj = Dd + j * d;
                    double s = 0.0;
                    for (int k = 0; k < d; ++k)
                        s += qi[k] * dj[k];
                    if (s > best) { /* strict: the first occurrence keeps a tie */
                        second = best;
                        best = s;
                        arg = (int32_t)j;
                    } else if (s > second) {
                        second = s;
                    }
                }
                score += best;
                int64_t o = ((int64_t)q * J->b + doc) * l_q + i;
                if (J->argmax)
                    J->argmax[o] = arg;
                if (J->margin)
                    J->margin[o] = best - second;
            }
            J->scores[(int64_t)q * J->b + doc] = score;
        }
        free(Dd);
    }
    return NULL;
}

/*
 * Q: [n_q, l_q, d]; D: uniform [b, l_d, d] when offsets == NULL, else packed
 * [offsets[b], d] with int32 offsets[b+1].  scores [n_q, b] (double),
 * argmax [n_q, b, l_q] (document-local token index, -1 for an empty
 * document), margin = best - second best (inf when the document has a single
 * token).  argmax and margin may be NULL.  Returns 0, or -1 on bad arguments
 * or allocation failure.
 */
int oracle_forward(const void *Q, int n_q, int l_q, const void *D, int64_t b, int l_d,
                   const int32_t *offsets, int d, int dtype, double *scores, int32_t *argmax,
                   double *margin, int n_threads)
{
    if (!Q || !D || !scores || n_q < 1 || l_q < 1 || b < 1 || d < 1 || dtype < 0 || dtype > 2)
        return -1;
    if (!offsets && l_d < 1)
        return -1;
    if (n_threads < 1)
        n_threads = 1;
    if (n_threads > 256)
        n_threads = 256;
    double *Qd = decode_block(Q, dtype, 0, (int64_t)n_q * l_q * d);
    if (!Qd)
        return -1;
    fwd_job *jobs = (fwd_job *)calloc((size_t)n_threads, sizeof(fwd_job));
    pthread_t *th = (pthread_t *)calloc((size_t)n_threads, sizeof(pthread_t));
    if (!jobs || !th) {
        free(Qd);
        free(jobs);
        free(th);
        return -1;
    }
    for (int t = 0; t < n_threads; ++t) {
        fwd_job j = {Qd, D, offsets, n_q, l_q, l_d, d, dtype, b, scores, argmax, margin, t, n_threads, 0};
        jobs[t] = j;
    }
    int started = 0;
    for (int t = 1; t < n_threads; ++t) {
        if (pthread_create(&th[t], NULL, fwd_worker, &jobs[t]) != 0)
            break;
        started = t;
    }
    fwd_worker(&jobs[0]);
    /* any thread that failed to start: run its share here */
    for (int t = started + 1; t < n_threads; ++t)
        fwd_worker(&jobs[t]);
    int failed = jobs[0].failed;
    for (int t = 1; t <= started; ++t) {
        pthread_join(th[t], NULL);
        failed |= jobs[t].failed;
    }
    for (int t = started + 1; t < n_threads; ++t)
        failed |= jobs[t].failed;
    free(Qd);
    free(jobs);
    free(th);
    return failed ? -1 : 0;
}

/* ---------- backward: Eqs. 2-3 (uniform corpus), routed through argmax ---------- */

/*
 * dQ[q,i,:] = sum_b g[q,b] * D[b, A[q,b,i], :]
 * dD[b,t,:] = sum_{(q,i): A[q,b,i]=t} g[q,b] * Q[q,i,:]
 * Entries of A that are negative are skipped.  Outputs are double and fully
 * overwritten.  Returns -1 on bad arguments or an index outside [0, l_d).
 */
int oracle_backward(const void *Q, int n_q, int l_q, const void *D, int64_t b, int l_d, int d,
                    int dtype, const int32_t *A, const double *g, double *dQ, double *dD)
{
    if (!Q || !D || !A || !g || !dQ || !dD || n_q < 1 || l_q < 1 || b < 1 || l_d < 1 || d < 1 ||
        dtype < 0 || dtype > 2)
        return -1;
    memset(dQ, 0, sizeof(double) * (size_t)n_q * l_q * d);
    memset(dD, 0, sizeof(double) * (size_t)b * l_d * d);
    for (int q = 0; q < n_q; ++q)
        for (int64_t doc = 0; doc < b; ++doc)
            for (int i = 0; i < l_q; ++i) {
                int32_t t = A[((int64_t)q * b + doc) * l_q + i];
                if (t < 0)
                    continue;
                if (t >= l_d)
                    return -1;
                double gg = g[(int64_t)q * b + doc];
                int64_t qrow = ((int64_t)q * l_q + i) * d;
                int64_t drow = (doc * (int64_t)l_d + t) * d;
                for (int k = 0; k < d; ++k) {
                    dQ[qrow + k] += gg * load_elem(D, dtype, drow + k);
                    dD[drow + k] += gg * load_elem(Q, dtype, qrow + k);
                }
            }
    return 0;
}

/* ---------- int8 scoring: Alg. 4 with the order
 *   cell:  v_ij = fl32(n_ij * d_s[j])      (n_ij exact integer dot product)
 *   row :  m_i  = max_j v_ij ;  r_i = fl32(q_s[i] * m_i)
 *   pair:  score = fl32(sum_i r_i)          (sum carried in double)
 * Both products are formed exactly in double (24 x 24 significant bits) and
 * rounded once to float, i.e. they equal an IEEE fp32 multiply. ---------- */

typedef struct {
    const int8_t *Q;
    const float *qs;
    const int8_t *D;
    const float *ds;
    int n_q, l_q, l_d, d;
    int64_t b;
    float *scores;
    int tid, n_threads;
} i8_job;

static void *i8_worker(void *arg)
{
    i8_job *J = (i8_job *)arg;
    const int d = J->d;
    for (int64_t doc = J->tid; doc < J->b; doc += J->n_threads) {
        const int8_t *Dd = J->D + doc * (int64_t)J->l_d * d;
        const float *dsd = J->ds + doc * (int64_t)J->l_d;
        for (int q = 0; q < J->n_q; ++q) {
            double total = 0.0;
            for (int i = 0; i < J->l_q; ++i) {
                const int8_t *qi = J->Q + ((int64_t)q * J->l_q + i) * d;
                float m = -INFINITY;
                for (int j = 0; j < J->l_d; ++j) {
                    const int8_t *dj = Dd + (int64_t)j * d;
                    int64_t n = 0;
                    for (int k = 0; k < d; ++k)
                        n += (int64_t)qi[k] * (int64_t)dj[k];
                    float v = (float)((double)n * (double)dsd[j]);
                    if (v > m)
                        m = v;
                }
                float r = (float)((double)J->qs[(int64_t)q * J->l_q + i] * (double)m);
                total += (double)r;
            }
            J->scores[(int64_t)q * J->b + doc] = (float)total;
        }
    }
    return NULL;
}

int oracle_forward_i8(const int8_t *Q, const float *q_scale, int n_q, int l_q, const int8_t *D,
                      const float *d_scale, int64_t b, int l_d, int d, float *scores, int n_threads)
{
    if (!Q || !q_scale || !D || !d_scale || !scores || n_q < 1 || l_q < 1 || b < 1 || l_d < 1 || d < 1)
        return -1;
    if (n_threads < 1)
        n_threads = 1;
    if (n_threads > 256)
        n_threads = 256;
    i8_job jobs[256];
    pthread_t th[256];
    for (int t = 0; t < n_threads; ++t) {
        i8_job j = {Q, q_scale, D, d_scale, n_q, l_q, l_d, d, b, scores, t, n_threads};
        jobs[t] = j;
    }
    int started = 0;
    for (int t = 1; t < n_threads; ++t) {
        if (pthread_create(&th[t], NULL, i8_worker, &jobs[t]) != 0)
            break;
        started = t;
    }
    i8_worker(&jobs[0]);
    for (int t = started + 1; t < n_threads; ++t)
        i8_worker(&jobs[t]);
    for (int t = 1; t <= started; ++t)
        pthread_join(th[t], NULL);
    return 0;
}

/* Exact integer dot products n[i,j] for one (query, doc) pair; used by pins. */
int oracle_dot_i8(const int8_t *Q, int l_q, const int8_t *D, int l_d, int d, int64_t *n)
{
    if (!Q || !D || !n || l_q < 1 || l_d < 1 || d < 1)
        return -1;
    for (int i = 0; i < l_q; ++i)
        for (int j = 0; j < l_d; ++j) {
            int64_t s = 0;
            for (int k = 0; k < d; ++k)
                s += (int64_t)Q[(int64_t)i * d + k] * (int64_t)D[(int64_t)j * d + k];
            n[(int64_t)i * l_d + j] = s;
        }
    return 0;
}

/* ---------- per-token symmetric absmax quantiser ---------- */

int oracle_quantize_rows_i8(const void *X, int64_t rows, int d, int dtype, int8_t *X_i8, float *scale)
{
    if (!X || !X_i8 || !scale || rows < 1 || d < 1 || dtype < 0 || dtype > 2)
        return -1;
    for (int64_t r = 0; r < rows; ++r) {
        double a = 0.0;
        for (int k = 0; k < d; ++k) {
            double v = fabs(load_elem(X, dtype, r * d + k));
            if (v > a)
                a = v;
        }
        float s = (float)(a / 127.0);
        scale[r] = s;
        for (int k = 0; k < d; ++k) {
            int8_t code = 0;
            if (s != 0.0f) {
                float t = (float)(load_elem(X, dtype, r * d + k) / (double)s);
                float rr = rintf(t); /* default rounding mode: half to even */
                if (rr > 127.0f)
                    rr = 127.0f;
                if (rr < -127.0f)
                    rr = -127.0f;
                code = (int8_t)rr;
            }
            X_i8[r * d + k] = code;
        }
    }
    return 0;
}

/* ---------- in-batch-negatives cross-entropy on a score matrix ---------- */

/*
 * s: [n, b] scores (double), label of row i is column i (requires b >= n).
 * loss = (1/n) sum_i [ log sum_j exp(s_ij/tau) - s_ii/tau ]
 * g_ij = (softmax_j(s_i./tau) - [i==j]) / (tau * n)
 */
int oracle_ce_grad(const double *s, int n, int b, double tau, double *loss, double *g)
{
    if (!s || !g || n < 1 || b < n || !(tau > 0.0))
        return -1;
    double L = 0.0;
    for (int i = 0; i < n; ++i) {
        const double *row = s + (int64_t)i * b;
        double mx = -INFINITY;
        for (int j = 0; j < b; ++j)
            if (row[j] / tau > mx)
                mx = row[j] / tau;
        double z = 0.0;
        for (int j = 0; j < b; ++j)
            z += exp(row[j] / tau - mx);
        L += log(z) + mx - row[i] / tau;
        for (int j = 0; j < b; ++j) {
            double p = exp(row[j] / tau - mx) / z;
            g[(int64_t)i * b + j] = (p - (i == j ? 1.0 : 0.0)) / (tau * n);
        }
    }
    if (loss)
        *loss = L / n;
    return 0;
}
