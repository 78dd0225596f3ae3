/*
 * CPU oracle for the HashEvict pre-attention eviction path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, obviously-correct
 * statement of what the path computes, written from the paper.  It shares no
 * code with the HIP library, and nothing in the product path may call it: only
 * the tests, the smoke check and the benchmark's CPU-baseline leg do.
 *
 * All inputs are float (for bf16 workloads the caller passes values that are
 * already bf16-representable); every sum -- projections, logits, softmax, key
 * norms -- is accumulated in double.
 *
 * Where each function comes from:
 *   lsheo_hash          Section 2, eq. (2): h(x) = sgn(Rx), sgn = Heaviside step
 *                       with sgn(0) = 1.
 *   lsheo_score         Section 3, eq. (5): F_score = -d_H(h(q), H); this returns
 *                       the Hamming distance itself (so larger = evict first),
 *                       summed over the query heads that share the KV head.
 *   lsheo_select        Section 3, eq. (6) and Algorithm 1 step 1: the slot most
 *                       distant from the current query; ties go to the lowest
 *                       slot.  Optional always-kept first / most-recent tokens
 *                       follow the experimental set-up of Section 4.
 *   lsheo_apply         Algorithm 1 steps 2-5: drop the victim and add the new
 *                       key, value and code (done as an in-place slot overwrite).
 *   lsheo_attend        Section 2, eq. (1) and Algorithm 1 step 6: softmax
 *                       attention of each query over the updated cache.
 *   lsheo_decode_step   Algorithm 1, one time step ("Decoding Stage").
 *   lsheo_prefill       "Prompt Encoding Stage": the first C tokens fill the
 *                       cache, then Algorithm 1 runs token by token.
 *   lsheo_evicted_mass  Section 4.8's attention loss, per step: the attention
 *                       probability that falls on the token being evicted.
 *   lsheo_l2_*          the L2-norm comparator the paper measures against
 *                       (Sections 1, 2.1, 4): same slots, victim = the key with
 *                       the largest L2 norm (squared norms in double).
 *
 * Pins (tests/test_oracle_*.py): NumPy packbits special case, the LSH collision
 * law of eq. (3), hand-worked tiny caches, brute-force bit loops, closed-form
 * attention cases and trajectory invariants.  No printed worked example exists
 * in the paper, so a full eviction trajectory has no external pin: for whole
 * trajectories this oracle is "parity unpinned" beyond those checks.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- eq. (2): sign random projection ------------------------------------ */

/* X [n][d], R [d][r] (column j is hyperplane j), codes [n][W], W = ceil(r/32).
 * Bit j of a code sits at bit (j mod 32) of word (j div 32); other bits are 0.
 * margin (nullable) [n][r] = |p_j| / (||x|| * ||R[:,j]||), 0 if a norm is 0. */
void lsheo_hash(const float *X, int64_t n, int d, const float *R, int r,
                uint32_t *codes, double *margin)
{
    int W = (r + 31) / 32;
    double *rn = (double *)malloc(sizeof(double) * (size_t)r);
    for (int j = 0; j < r; ++j) {
        double s = 0.0;
        for (int i = 0; i < d; ++i) {
            double v = (double)R[(size_t)i * r + j];
            s += v * v;
        }
        rn[j] = sqrt(s);
    }
    for (int64_t t = 0; t < n; ++t) {
        const float *x = X + (size_t)t * d;
        uint32_t *c = codes + (size_t)t * W;
        double xn = 0.0;
        for (int i = 0; i < d; ++i)
            xn += (double)x[i] * (double)x[i];
        xn = sqrt(xn);
        for (int w = 0; w < W; ++w)
            c[w] = 0u;
        for (int j = 0; j < r; ++j) {
            double p = 0.0;
            for (int i = 0; i < d; ++i)
                p += (double)x[i] * (double)R[(size_t)i * r + j];
            if (p >= 0.0)
                c[j / 32] |= (uint32_t)1u << (j % 32);
            if (margin) {
                double den = xn * rn[j];
                margin[(size_t)t * r + j] = den > 0.0 ? fabs(p) / den : 0.0;
            }
        }
    }
    free(rn);
}

/* ---- eq. (5): Hamming distance of the query codes to every cached code --- */

static int hamming_word(uint32_t a, uint32_t b)
{
    uint32_t x = a ^ b;
    int c = 0;
    for (int k = 0; k < 32; ++k)
        c += (int)((x >> k) & 1u);
    return c;
}

/* codes [C][W], cq [G][W]  ->  score [n_slots] */
void lsheo_score(const uint32_t *codes, int n_slots, int W, const uint32_t *cq, int G,
                 int32_t *score)
{
    for (int s = 0; s < n_slots; ++s) {
        int acc = 0;
        for (int g = 0; g < G; ++g)
            for (int w = 0; w < W; ++w)
                acc += hamming_word(codes[(size_t)s * W + w], cq[(size_t)g * W + w]);
        score[s] = acc;
    }
}

/* ---- eq. (6) / Algorithm 1 step 1 ---------------------------------------- */

/* While the cache is not full the new token is appended (no eviction).
 * Once full: the lowest slot whose score is maximal among evictable slots.
 * A slot is evictable when the token it holds is neither one of the first
 * n_sink tokens nor one of the n_recent tokens before t. */
int lsheo_select(const int32_t *score, const int32_t *slot_pos, int C, int n_valid, int t,
                 int n_sink, int n_recent)
{
    if (n_valid < C)
        return n_valid;
    int best = -1, best_score = -1;
    for (int s = 0; s < C; ++s) {
        int p = slot_pos[s];
        if (p < n_sink || p > t - 1 - n_recent)
            continue;
        if (score[s] > best_score) {
            best_score = score[s];
            best = s;
        }
    }
    return best;
}

/* ---- Algorithm 1 steps 2-5 ----------------------------------------------- */

/* Returns 0, or -1 without touching anything when e is no slot of the cache
 * (lsheo_select found nothing evictable: a budget no larger than the number of
 * always-kept tokens, which no valid configuration has).  codes may be NULL
 * with W = 0 (the L2-norm comparator keeps no hash codes). */
int lsheo_apply(float *K, float *V, uint32_t *codes, int32_t *slot_pos, int32_t *n_valid,
                int C, int d, int W, int e, const float *k_new, const float *v_new,
                const uint32_t *c_new, int t)
{
    if (e < 0 || e >= C || e > *n_valid)
        return -1;
    memcpy(K + (size_t)e * d, k_new, sizeof(float) * (size_t)d);
    memcpy(V + (size_t)e * d, v_new, sizeof(float) * (size_t)d);
    if (W > 0)
        memcpy(codes + (size_t)e * W, c_new, sizeof(uint32_t) * (size_t)W);
    slot_pos[e] = t;
    if (*n_valid < C && e == *n_valid)
        *n_valid += 1;
    return 0;
}

/* ---- eq. (1): softmax(q K^T / sqrt(d)) V over the occupied slots ---------- */

/* q [G][d], K, V [n_valid][d]  ->  out [G][d] (double).  Optional prob [G][n_valid]. */
void lsheo_attend(const float *q, const float *K, const float *V, int n_valid, int d, int G,
                  double *out, double *prob)
{
    double *a = (double *)malloc(sizeof(double) * (size_t)(n_valid > 0 ? n_valid : 1));
    double inv = 1.0 / sqrt((double)d);
    for (int g = 0; g < G; ++g) {
        const float *qg = q + (size_t)g * d;
        double *o = out + (size_t)g * d;
        for (int i = 0; i < d; ++i)
            o[i] = 0.0;
        if (n_valid <= 0)
            continue;
        double mx = -INFINITY;
        for (int s = 0; s < n_valid; ++s) {
            double dot = 0.0;
            for (int i = 0; i < d; ++i)
                dot += (double)qg[i] * (double)K[(size_t)s * d + i];
            a[s] = dot * inv;
            if (a[s] > mx)
                mx = a[s];
        }
        double den = 0.0;
        for (int s = 0; s < n_valid; ++s) {
            a[s] = exp(a[s] - mx);
            den += a[s];
        }
        for (int s = 0; s < n_valid; ++s) {
            double p = a[s] / den;
            if (prob)
                prob[(size_t)g * n_valid + s] = p;
            for (int i = 0; i < d; ++i)
                o[i] += p * (double)V[(size_t)s * d + i];
        }
    }
    free(a);
}

/* ---- attention mass of the evicted token (Section 4.8's attention loss, per step) --- */

/* Section 4.8 measures an eviction policy by the attention probability of the tokens
 * it evicted.  Per step that is: among the keys the query could have attended to at
 * this step -- the C cached keys BEFORE the eviction plus the new key -- the softmax
 * probability (eq. 1 scaling) that falls on the victim.  q [G][d], K [C][d] (the cache
 * before the overwrite), k_new [d], e = victim slot -> mass [G]. */
void lsheo_evicted_mass(const float *q, const float *K, int C, int d, int G, const float *k_new,
                        int e, double *mass)
{
    double inv = 1.0 / sqrt((double)d);
    double *a = (double *)malloc(sizeof(double) * (size_t)(C + 1));
    for (int g = 0; g < G; ++g) {
        const float *qg = q + (size_t)g * d;
        double mx = -INFINITY;
        for (int s = 0; s <= C; ++s) {
            const float *k = s < C ? K + (size_t)s * d : k_new;
            double dot = 0.0;
            for (int i = 0; i < d; ++i)
                dot += (double)qg[i] * (double)k[i];
            a[s] = dot * inv;
            if (a[s] > mx)
                mx = a[s];
        }
        double den = 0.0;
        for (int s = 0; s <= C; ++s)
            den += exp(a[s] - mx);
        mass[g] = exp(a[e] - mx) / den;
    }
    free(a);
}

/* ---- Algorithm 1: one time step for one unit ------------------------------ */

/* State of one unit (one KV head of one layer of one sequence):
 *   K, V [C][d]; codes [C][W]; slot_pos [C] (token index per slot, -1 empty);
 *   n_valid.  q [G][d], k_new, v_new [d]; t = index of the new token.
 * codes_in (nullable) [G+1][W]: query codes then the key code to use instead of
 *   hashing here (the lock-step parity harness passes the device's codes after
 *   checking that they differ from this oracle's only in near-zero projections).
 * Outputs (each nullable): out [G][d], evicted, scores [C] (-1 for empty
 *   slots), codes_out [G+1][W], mass [G] (lsheo_evicted_mass of the victim).
 * Returns 0, or -1 (cache untouched, no attention) when no slot is evictable. */
int lsheo_decode_step(float *K, float *V, uint32_t *codes, int32_t *slot_pos, int32_t *n_valid,
                       int C, int d, int r, int G, int n_sink, int n_recent,
                       const float *R, const float *q, const float *k_new, const float *v_new,
                       int t, const uint32_t *codes_in, int do_attend,
                       double *out, int32_t *evicted, int32_t *scores, uint32_t *codes_out,
                       double *mass)
{
    int W = (r + 31) / 32;
    uint32_t cbuf[(64 + 1) * 2];
    uint32_t *c = cbuf;
    if (G + 1 > 65) {
        c = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(G + 1) * W);
    }
    if (codes_in) {
        memcpy(c, codes_in, sizeof(uint32_t) * (size_t)(G + 1) * W);
    } else {
        lsheo_hash(q, G, d, R, r, c, NULL);
        lsheo_hash(k_new, 1, d, R, r, c + (size_t)G * W, NULL);
    }
    if (codes_out)
        memcpy(codes_out, c, sizeof(uint32_t) * (size_t)(G + 1) * W);

    int32_t *sc = (int32_t *)malloc(sizeof(int32_t) * (size_t)C);
    for (int s = 0; s < C; ++s)
        sc[s] = -1;
    lsheo_score(codes, *n_valid, W, c, G, sc);
    int e = lsheo_select(sc, slot_pos, C, *n_valid, t, n_sink, n_recent);
    if (scores)
        memcpy(scores, sc, sizeof(int32_t) * (size_t)C);
    free(sc);
    if (evicted)
        *evicted = e;
    if (mass) {   /* nothing is evicted while the cache is filling */
        if (*n_valid == C && e >= 0)
            lsheo_evicted_mass(q, K, C, d, G, k_new, e, mass);
        else
            for (int g = 0; g < G; ++g)
                mass[g] = 0.0;
    }
    int rc = lsheo_apply(K, V, codes, slot_pos, n_valid, C, d, W, e, k_new, v_new, c + (size_t)G * W, t);
    if (rc == 0 && do_attend && out)
        lsheo_attend(q, K, V, *n_valid, d, G, out, NULL);
    if (c != cbuf)
        free(c);
    return rc;
}

/* ---- Prompt Encoding Stage for one unit ----------------------------------- */

/* Kp, Vp [N][d]; Qp [G][N][d].  Cache arrays as in lsheo_decode_step, any
 * contents on entry.  codes_k_in [N][W] / codes_q_in [G][N][W] (both nullable,
 * given together): codes to use instead of hashing here.
 * evict_log (nullable) [max(N-C,0)]: victim slot of each token t >= C. */
void lsheo_prefill(const float *Kp, const float *Vp, const float *Qp, int N,
                   float *K, float *V, uint32_t *codes, int32_t *slot_pos, int32_t *n_valid,
                   int C, int d, int r, int G, int n_sink, int n_recent, const float *R,
                   const uint32_t *codes_k_in, const uint32_t *codes_q_in, int32_t *evict_log)
{
    int W = (r + 31) / 32;
    for (int s = 0; s < C; ++s) {
        slot_pos[s] = -1;
        for (int w = 0; w < W; ++w)
            codes[(size_t)s * W + w] = 0u;
        for (int i = 0; i < d; ++i) {
            K[(size_t)s * d + i] = 0.0f;
            V[(size_t)s * d + i] = 0.0f;
        }
    }
    *n_valid = 0;
    float *q = (float *)malloc(sizeof(float) * (size_t)G * d);
    uint32_t *cin = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(G + 1) * W);
    for (int t = 0; t < N; ++t) {
        for (int g = 0; g < G; ++g)
            memcpy(q + (size_t)g * d, Qp + ((size_t)g * N + t) * d, sizeof(float) * (size_t)d);
        const uint32_t *ci = NULL;
        if (codes_k_in && codes_q_in) {
            for (int g = 0; g < G; ++g)
                memcpy(cin + (size_t)g * W, codes_q_in + ((size_t)g * N + t) * W,
                       sizeof(uint32_t) * (size_t)W);
            memcpy(cin + (size_t)G * W, codes_k_in + (size_t)t * W, sizeof(uint32_t) * (size_t)W);
            ci = cin;
        }
        int32_t e;
        lsheo_decode_step(K, V, codes, slot_pos, n_valid, C, d, r, G, n_sink, n_recent, R,
                          q, Kp + (size_t)t * d, Vp + (size_t)t * d, t, ci, 0,
                          NULL, &e, NULL, NULL, NULL);
        if (evict_log && t >= C)
            evict_log[t - C] = e;
    }
    free(q);
    free(cin);
}

/* ---- L2-norm comparator (the attention-free baseline of Sections 1, 2.1, 4) -- */

/* The comparator keeps low-norm keys: the victim is the evictable slot whose key
 * has the LARGEST L2 norm (lowest slot on ties); nothing else changes -- same
 * slots, same protection of first / recent tokens, same attention.  Per slot the
 * oracle keeps the squared norm (same order as the norm) in double. */
double lsheo_norm2(const float *x, int d)
{
    double s = 0.0;
    for (int i = 0; i < d; ++i)
        s += (double)x[i] * (double)x[i];
    return s;
}

/* norm2 [C]: squared norms of the cached keys.  Append while filling, else the
 * lowest evictable slot whose squared norm is maximal; -1 if none is evictable. */
int lsheo_l2_select(const double *norm2, const int32_t *slot_pos, int C, int n_valid, int t,
                    int n_sink, int n_recent)
{
    if (n_valid < C)
        return n_valid;
    int best = -1;
    double best_norm = -1.0;
    for (int s = 0; s < C; ++s) {
        int p = slot_pos[s];
        if (p < n_sink || p > t - 1 - n_recent)
            continue;
        if (norm2[s] > best_norm) {
            best_norm = norm2[s];
            best = s;
        }
    }
    return best;
}

/* One step of the comparator for one unit.  victim_in: -1, or the slot to write
 * instead of this oracle's own choice (the lock-step parity harness passes the
 * device's victim after checking that it is evictable and that its squared norm
 * is within fp32 summation error of the oracle's choice, so that one tolerated
 * near tie cannot fork the trajectories).  Returns 0, or -1 when no slot is
 * evictable (cache untouched). */
int lsheo_l2_decode_step(float *K, float *V, double *norm2, int32_t *slot_pos,
                         int32_t *n_valid, int C, int d, int G, int n_sink, int n_recent,
                         const float *q, const float *k_new, const float *v_new, int t,
                         int victim_in, int do_attend, double *out, int32_t *evicted,
                         double *mass)
{
    int e = victim_in >= 0 ? victim_in
                           : lsheo_l2_select(norm2, slot_pos, C, *n_valid, t, n_sink, n_recent);
    if (evicted)
        *evicted = e;
    if (mass) {
        if (*n_valid == C && e >= 0)
            lsheo_evicted_mass(q, K, C, d, G, k_new, e, mass);
        else
            for (int g = 0; g < G; ++g)
                mass[g] = 0.0;
    }
    int rc = lsheo_apply(K, V, NULL, slot_pos, n_valid, C, d, 0, e, k_new, v_new, NULL, t);
    if (rc != 0)
        return rc;
    norm2[e] = lsheo_norm2(k_new, d);
    if (do_attend && out)
        lsheo_attend(q, K, V, *n_valid, d, G, out, NULL);
    return 0;
}

void lsheo_l2_prefill(const float *Kp, const float *Vp, int N, float *K, float *V,
                      double *norm2, int32_t *slot_pos, int32_t *n_valid, int C, int d,
                      int n_sink, int n_recent, int32_t *evict_log)
{
    for (int s = 0; s < C; ++s) {
        slot_pos[s] = -1;
        norm2[s] = 0.0;
        for (int i = 0; i < d; ++i) {
            K[(size_t)s * d + i] = 0.0f;
            V[(size_t)s * d + i] = 0.0f;
        }
    }
    *n_valid = 0;
    for (int t = 0; t < N; ++t) {
        int32_t e;
        lsheo_l2_decode_step(K, V, norm2, slot_pos, n_valid, C, d, 1, n_sink, n_recent, NULL,
                             Kp + (size_t)t * d, Vp + (size_t)t * d, t, -1, 0, NULL, &e, NULL);
        if (evict_log && t >= C)
            evict_log[t - C] = e;
    }
}

/* ---- many independent units (timed CPU baseline; optional OpenMP) --------- */

/* Arrays are the single-unit ones with a leading [n_units] dimension; t [n_units]. */
void lsheo_decode_step_units(int n_units, float *K, float *V, uint32_t *codes, int32_t *slot_pos,
                             int32_t *n_valid, int C, int d, int r, int G, int n_sink,
                             int n_recent, const float *R, const float *q, const float *k_new,
                             const float *v_new, const int32_t *t, double *out, int32_t *evicted,
                             int n_threads)
{
    int W = (r + 31) / 32;
    (void)n_threads;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(n_threads > 0 ? n_threads : 1)
#endif
    for (int u = 0; u < n_units; ++u) {
        lsheo_decode_step(K + (size_t)u * C * d, V + (size_t)u * C * d, codes + (size_t)u * C * W,
                          slot_pos + (size_t)u * C, n_valid + u, C, d, r, G, n_sink, n_recent, R,
                          q + (size_t)u * G * d, k_new + (size_t)u * d, v_new + (size_t)u * d,
                          t[u], NULL, 1, out + (size_t)u * G * d,
                          evicted ? evicted + u : NULL, NULL, NULL, NULL);
    }
}

int lsheo_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
