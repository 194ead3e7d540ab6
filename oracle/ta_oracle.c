/*
 * ta_oracle.c -- plain fp64 CPU oracle for single-query (decode) attention.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only tests, the smoke check
 * and the benchmark's reported CPU baseline may call it.  It shares no code,
 * header, table or helper with the HIP library and never includes or links it.
 *
 * Every function here is the paper's definition (or the algorithm's steps in
 * the paper's order) written out with sequential loops in double precision.
 * There is no blocking, no fusion and no reordering beyond what the cited
 * passage states.  Inputs stored as bf16 or fp32 are widened exactly.
 *
 * Readings adopted where the paper is silent (Tree Attention, arXiv 2408.04093):
 *   - score s_a = scale * (q . k_a); scale = 1 gives the paper's softmax
 *     (Section 3, attention definition).  In the energy function the scale
 *     multiplies only the q.k term, never the zeta.v term.
 *   - grouped queries: query head h reads key/value head floor(h / g),
 *     g = Hq / Hkv.  Heads are independent (Appendix C.1, multi-head energy).
 *   - keys at positions >= valid_len[b] do not exist.  With no keys at all the
 *     output is 0 and lse is -infinity.
 *   - lse is the natural-log logsumexp of the scaled scores = F(0)
 *     (Observation 1).
 *
 * Every function is pinned by tests/test_oracle_pins.py against closed forms,
 * library routines, finite differences of the energy and brute force.
 *
 * Build: gcc -O2 -std=c11 -fopenmp -shared -fPIC ta_oracle.c -o libta_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { TAO_BF16 = 0, TAO_F32 = 1, TAO_F64 = 2 };

/* Exact widening of one stored element to double. */
static double widen(const void *base, int dtype, int64_t idx)
{
    if (dtype == TAO_BF16) {
        /* bfloat16 is the upper 16 bits of an IEEE binary32. */
        uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    if (dtype == TAO_F32)
        return (double)((const float *)base)[idx];
    return ((const double *)base)[idx];
}

/* s_a = scale * sum_c q_c k_{a,c}  (Section 3: the argument of the softmax). */
static double score(const void *q, int64_t q_off, const void *K, int64_t k_off,
                    int dtype, int d, double scale)
{
    double acc = 0.0;
    for (int c = 0; c < d; ++c)
        acc += widen(q, dtype, q_off + c) * widen(K, dtype, k_off + c);
    return scale * acc;
}

/*
 * One (b, hq) problem, straight from the definition
 *     z = sum_a P_a v_a,  P_a = exp(s_a) / Z,  Z = sum_a exp(s_a)
 * (Section 3 and Appendix C.1), evaluated with every exponent shifted by
 * M = max_a s_a, which leaves z unchanged (Appendix F), and
 *     lse = F(0) = log Z = M + log sum_a exp(s_a - M)   (Observation 1).
 */
static void decode_one(const void *q, int64_t q_off, const void *K, const void *V,
                       int64_t kv_off, int dtype, int d, int64_t L, double scale,
                       double *out, double *lse, double *s_buf)
{
    if (L <= 0) {
        for (int c = 0; c < d; ++c) out[c] = 0.0;
        *lse = -INFINITY;
        return;
    }
    double M = -INFINITY;
    for (int64_t a = 0; a < L; ++a) {
        s_buf[a] = score(q, q_off, K, kv_off + a * d, dtype, d, scale);
        if (s_buf[a] > M) M = s_buf[a];
    }
    double Z = 0.0;
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    for (int64_t a = 0; a < L; ++a) {
        double e = exp(s_buf[a] - M);
        Z += e;
        for (int c = 0; c < d; ++c)
            out[c] += e * widen(V, dtype, kv_off + a * d + c);
    }
    for (int c = 0; c < d; ++c) out[c] /= Z;
    *lse = M + log(Z);
}

/*
 * Batched decode attention.
 *   q [B,Hq,d], K,V [B,Hkv,N,d] contiguous, element type `dtype`.
 *   valid_len: host int32 [B] or NULL (= N for every b).
 *   out [B,Hq,d], lse [B,Hq] in double.
 * Threads split the independent (b,hq) problems only; each problem is the
 * sequential loop above, so the result does not depend on nthreads.
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int ta_oracle_decode(int B, int Hq, int Hkv, int d, int64_t N,
                     const void *q, const void *K, const void *V, int dtype,
                     double scale, const int32_t *valid_len,
                     double *out, double *lse, int nthreads)
{
    if (B < 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || N < 0 || Hq % Hkv != 0) return -1;
    if (dtype < TAO_BF16 || dtype > TAO_F64) return -1;
    const int g = Hq / Hkv;
    const int nprob = B * Hq;
    int fail = 0;
#ifdef _OPENMP
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
#endif
    for (int pidx = 0; pidx < nprob; ++pidx) {
        const int b = pidx / Hq, hq = pidx % Hq, hk = hq / g;
        int64_t L = valid_len ? (int64_t)valid_len[b] : N;
        if (L > N) L = N;
        if (L < 0) L = 0;
        double *s_buf = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
        if (!s_buf) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            fail = 1;
            continue;
        }
        decode_one(q, ((int64_t)b * Hq + hq) * d, K, V,
                   ((int64_t)b * Hkv + hk) * N * d, dtype, d, L, scale,
                   out + (int64_t)pidx * d, lse + pidx, s_buf);
        free(s_buf);
    }
    return fail ? -1 : 0;
}

/*
 * Several query tokens at once with causal masking among them (Appendix C.1,
 * causal energy F_tot = sum_i log sum_{a <= i} exp(q_i.k_a + zeta_i.v_a)):
 * the cache of sequence b holds L = valid_len[b] keys, the last Sq of which
 * belong to the Sq query tokens themselves; query token t (0-based) sees keys
 * 0 .. L - Sq + t, i.e. L - Sq + t + 1 of them (none if that is <= 0).
 *   q [B,Sq,Hq,d], K,V [B,Hkv,N,d];  out [B,Sq,Hq,d], lse [B,Sq,Hq] in double.
 * Each (b, t, h) is the single-query definition above on its own prefix.
 */
int ta_oracle_decode_causal(int B, int Sq, int Hq, int Hkv, int d, int64_t N,
                            const void *q, const void *K, const void *V, int dtype,
                            double scale, const int32_t *valid_len,
                            double *out, double *lse, int nthreads)
{
    if (B < 0 || Sq <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || N < 0 || Hq % Hkv != 0) return -1;
    if (dtype < TAO_BF16 || dtype > TAO_F64) return -1;
    const int g = Hq / Hkv;
    const int nprob = B * Sq * Hq;
    int fail = 0;
#ifdef _OPENMP
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
#endif
    for (int pidx = 0; pidx < nprob; ++pidx) {
        const int b = pidx / (Sq * Hq), t = (pidx / Hq) % Sq, hq = pidx % Hq, hk = hq / g;
        int64_t L = valid_len ? (int64_t)valid_len[b] : N;
        if (L > N) L = N;
        if (L < 0) L = 0;
        int64_t Lt = L - Sq + t + 1;          /* keys visible to token t */
        if (Lt < 0) Lt = 0;
        double *s_buf = (double *)malloc(sizeof(double) * (size_t)(Lt > 0 ? Lt : 1));
        if (!s_buf) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            fail = 1;
            continue;
        }
        decode_one(q, (((int64_t)b * Sq + t) * Hq + hq) * d, K, V,
                   ((int64_t)b * Hkv + hk) * N * d, dtype, d, Lt, scale,
                   out + (int64_t)pidx * d, lse + pidx, s_buf);
        free(s_buf);
    }
    return fail ? -1 : 0;
}

/*
 * Causal total energy of Appendix C.1 for one head and Sq query tokens:
 *     F_tot(zeta) = sum_t log sum_{a < L - Sq + t + 1} exp(scale q_t.k_a + zeta_t.v_a).
 * q [Sq,d], K,V [L,d], zeta [Sq,d] (double).  Every token must see >= 1 key.
 */
double ta_oracle_energy_causal(int d, int64_t L, int Sq, const void *q, const void *K,
                               const void *V, int dtype, double scale, const double *zeta)
{
    double total = 0.0;
    for (int t = 0; t < Sq; ++t) {
        const int64_t Lt = L - Sq + t + 1;
        if (Lt <= 0) return NAN;
        double m = -INFINITY, acc = 0.0;
        double *r = (double *)malloc(sizeof(double) * (size_t)Lt);
        if (!r) return NAN;
        for (int64_t a = 0; a < Lt; ++a) {
            double zv = 0.0;
            for (int c = 0; c < d; ++c) zv += zeta[(size_t)t * d + c] * widen(V, dtype, a * d + c);
            r[a] = score(q, (int64_t)t * d, K, a * d, dtype, d, scale) + zv;
            if (r[a] > m) m = r[a];
        }
        for (int64_t a = 0; a < Lt; ++a) acc += exp(r[a] - m);
        free(r);
        total += m + log(acc);
    }
    return total;
}

int ta_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Partial statistics of one chunk [lo, hi) of one head's keys:
 *     m = max_a s_a,  l = sum_a exp(s_a - m),  o = sum_a exp(s_a - m) v_a.
 * This is the per-device quantity of Algorithm 3 step 2 kept unnormalised:
 * the paper's (o_norm, lse) of a chunk are o / l and m + log l.
 * q [d], K,V [N,d] for that head.  An empty chunk gives the identity
 * (m, l, o) = (-inf, 0, 0).
 */
int ta_oracle_partial(int d, const void *q, const void *K, const void *V, int dtype,
                      double scale, int64_t lo, int64_t hi,
                      double *m, double *l, double *o)
{
    if (d <= 0 || dtype < TAO_BF16 || dtype > TAO_F64) return -1;
    *m = -INFINITY;
    *l = 0.0;
    for (int c = 0; c < d; ++c) o[c] = 0.0;
    if (hi <= lo) return 0;
    for (int64_t a = lo; a < hi; ++a) {
        double s = score(q, 0, K, a * d, dtype, d, scale);
        if (s > *m) *m = s;
    }
    for (int64_t a = lo; a < hi; ++a) {
        double e = exp(score(q, 0, K, a * d, dtype, d, scale) - *m);
        *l += e;
        for (int c = 0; c < d; ++c) o[c] += e * widen(V, dtype, a * d + c);
    }
    return 0;
}

/*
 * The associative merge of two partials (Section 5.1: max and logsumexp are
 * associative; Algorithm 3 steps 3-5 are its p-ary form):
 *     m = max(m1, m2)
 *     l = l1 exp(m1 - m) + l2 exp(m2 - m)
 *     o = o1 exp(m1 - m) + o2 exp(m2 - m)
 * A partial with l = 0 is the identity and is skipped, so (-inf) - (-inf) is
 * never evaluated.  Result overwrites (m1, l1, o1).
 */
static void merge_into(int d, double *m1, double *l1, double *o1,
                       const double *m2, const double *l2, const double *o2)
{
    if (*l2 == 0.0) return;
    if (*l1 == 0.0) {
        *m1 = *m2;
        *l1 = *l2;
        for (int c = 0; c < d; ++c) o1[c] = o2[c];
        return;
    }
    double m = *m1 > *m2 ? *m1 : *m2;
    double w1 = exp(*m1 - m), w2 = exp(*m2 - m);
    *l1 = *l1 * w1 + *l2 * w2;
    for (int c = 0; c < d; ++c) o1[c] = o1[c] * w1 + o2[c] * w2;
    *m1 = m;
}

/*
 * Reduce P partials with an arbitrary tree.  `merges` lists n_merges pairs
 * (dst, src): node[dst] = node[dst] (+) node[src], applied in order; after all
 * of them node[root] holds the total.  Any binary, k-ary or flat shape and any
 * leaf order can be written this way (Appendix B).
 * Then  out = o / l  (Algorithm 3 step 6) and  lse = m + log l.
 * m [P], l [P], o [P,d] are not modified.
 */
int ta_oracle_combine(int P, int d, const double *m, const double *l, const double *o,
                      int n_merges, const int32_t *merges, int root,
                      double *out, double *lse)
{
    if (P <= 0 || d <= 0 || root < 0 || root >= P) return -1;
    double *mm = (double *)malloc(sizeof(double) * (size_t)P);
    double *ll = (double *)malloc(sizeof(double) * (size_t)P);
    double *oo = (double *)malloc(sizeof(double) * (size_t)P * (size_t)d);
    if (!mm || !ll || !oo) { free(mm); free(ll); free(oo); return -1; }
    memcpy(mm, m, sizeof(double) * (size_t)P);
    memcpy(ll, l, sizeof(double) * (size_t)P);
    memcpy(oo, o, sizeof(double) * (size_t)P * (size_t)d);
    int rc = 0;
    for (int t = 0; t < n_merges; ++t) {
        int dst = merges[2 * t], src = merges[2 * t + 1];
        if (dst < 0 || dst >= P || src < 0 || src >= P || dst == src) { rc = -1; break; }
        merge_into(d, &mm[dst], &ll[dst], oo + (size_t)dst * d,
                   &mm[src], &ll[src], oo + (size_t)src * d);
    }
    if (rc == 0) {
        if (ll[root] == 0.0) {
            for (int c = 0; c < d; ++c) out[c] = 0.0;
            *lse = -INFINITY;
        } else {
            for (int c = 0; c < d; ++c) out[c] = oo[(size_t)root * d + c] / ll[root];
            *lse = mm[root] + log(ll[root]);
        }
    }
    free(mm); free(ll); free(oo);
    return rc;
}

/*
 * Algorithm 3 steps 3-6 exactly as printed, from per-chunk normalised outputs
 * o_j [P,d] and true per-chunk logsumexps lse_j [P]:
 *     m   = max_j lse_j
 *     n_j = o_j exp(lse_j - m),  d_j = exp(lse_j - m)
 *     n_g = sum_j n_j,           d_g = sum_j d_j
 *     z   = n_g / d_g
 * and the total logsumexp  m + log d_g.  Chunks with lse_j = -inf hold no keys
 * and contribute nothing.
 */
int ta_oracle_combine_alg3(int P, int d, const double *o_norm, const double *lse_j,
                           double *out, double *lse)
{
    if (P <= 0 || d <= 0) return -1;
    double m = -INFINITY;
    for (int j = 0; j < P; ++j)
        if (lse_j[j] > m) m = lse_j[j];
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    if (m == -INFINITY) { *lse = -INFINITY; return 0; }
    double dg = 0.0;
    for (int j = 0; j < P; ++j) {
        if (lse_j[j] == -INFINITY) continue;
        double dj = exp(lse_j[j] - m);
        dg += dj;
        for (int c = 0; c < d; ++c) out[c] += o_norm[(size_t)j * d + c] * dj;
    }
    for (int c = 0; c < d; ++c) out[c] /= dg;
    *lse = m + log(dg);
    return 0;
}

/*
 * The energy function of Observation 1 for one head,
 *     F(zeta) = log sum_a exp(scale q.k_a + zeta.v_a),
 * evaluated as  max_a r_a + log sum_a exp(r_a - max)  (Algorithm 1 steps 3-6).
 * zeta is double [d].  q [d], K,V [L,d].  L must be >= 1.
 */
double ta_oracle_energy(int d, int64_t L, const void *q, const void *K, const void *V,
                        int dtype, double scale, const double *zeta)
{
    if (L <= 0) return -INFINITY;
    double *r = (double *)malloc(sizeof(double) * (size_t)L);
    if (!r) return NAN;
    double m = -INFINITY;
    for (int64_t a = 0; a < L; ++a) {
        double zv = 0.0;
        for (int c = 0; c < d; ++c) zv += zeta[c] * widen(V, dtype, a * d + c);
        r[a] = score(q, 0, K, a * d, dtype, d, scale) + zv;
        if (r[a] > m) m = r[a];
    }
    double acc = 0.0;
    for (int64_t a = 0; a < L; ++a) acc += exp(r[a] - m);
    free(r);
    return m + log(acc);
}

/*
 * The memory-efficient recurrence of Section 3 with no max shift:
 *     s_i = exp(q.k_i),  n_i = n_{i-1} + v_i s_i,  d_i = d_{i-1} + s_i,  z = n / d.
 * Only safe while exp(s) neither overflows nor underflows; used as a second
 * route to the definition on small scores.
 */
int ta_oracle_recurrence(int d, int64_t L, const void *q, const void *K, const void *V,
                         int dtype, double scale, double *out)
{
    if (d <= 0 || L <= 0) return -1;
    double den = 0.0;
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    for (int64_t i = 0; i < L; ++i) {
        double s = exp(score(q, 0, K, i * d, dtype, d, scale));
        for (int c = 0; c < d; ++c) out[c] += widen(V, dtype, i * d + c) * s;
        den += s;
    }
    for (int c = 0; c < d; ++c) out[c] /= den;
    return 0;
}

/*
 * Algorithm 1 followed by Algorithm 2 over p contiguous chunks given by
 * bounds [p+1]:
 *   Alg. 1: r_a = s_a (zeta = 0); m = max over chunks of the chunk max;
 *           lse' = logsumexp over chunks of the chunk logsumexp of (r - m).
 *   Alg. 2: R_a = exp(r_a - m - lse') v_a;  z = sum over chunks of the chunk sums.
 * Returns z in out and the true logsumexp m + lse' in lse.  The per-chunk
 * reductions are left folds in chunk order.
 */
int ta_oracle_two_pass(int d, const void *q, const void *K, const void *V, int dtype,
                       double scale, int p, const int64_t *bounds,
                       double *out, double *lse)
{
    if (d <= 0 || p <= 0) return -1;
    double m = -INFINITY;
    for (int j = 0; j < p; ++j) {
        double mj = -INFINITY;
        for (int64_t a = bounds[j]; a < bounds[j + 1]; ++a) {
            double r = score(q, 0, K, a * d, dtype, d, scale);
            if (r > mj) mj = r;
        }
        if (mj > m) m = mj;
    }
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    if (m == -INFINITY) { *lse = -INFINITY; return 0; }
    /* logsumexp across chunks of the per-chunk logsumexp of shifted scores */
    double lse_sh = -INFINITY;
    for (int j = 0; j < p; ++j) {
        double acc = 0.0;
        for (int64_t a = bounds[j]; a < bounds[j + 1]; ++a)
            acc += exp(score(q, 0, K, a * d, dtype, d, scale) - m);
        if (acc == 0.0) continue;
        double lj = log(acc);
        if (lse_sh == -INFINITY) lse_sh = lj;
        else {
            double hi = lse_sh > lj ? lse_sh : lj;
            lse_sh = hi + log(exp(lse_sh - hi) + exp(lj - hi));
        }
    }
    for (int j = 0; j < p; ++j) {
        for (int64_t a = bounds[j]; a < bounds[j + 1]; ++a) {
            double w = exp(score(q, 0, K, a * d, dtype, d, scale) - m - lse_sh);
            for (int c = 0; c < d; ++c) out[c] += w * widen(V, dtype, a * d + c);
        }
    }
    *lse = m + lse_sh;
    return 0;
}
