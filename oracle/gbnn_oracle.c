/*
 * gbnn_oracle.c -- plain CPU oracle for retrieval in the Gripon-Berrou clustered
 * associative memory (GBNN).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It exists so that the GPU library can be
 * checked bit for bit against something slow and obviously right.  Only the tests, the
 * smoke check and the benchmark's "cpu_baseline" leg may call it; the product path never
 * does, and this file shares no code, header, table or helper with the GPU sources.
 *
 * Everything is written out from the paper's equations in the paper's notation:
 *   C clusters of L neurons, n = C*L neurons, neuron (c,l) has flat index i = c*L + l
 *   (Section IV-B "Vectorization"; 0-based here, 1-based in the paper);
 *   W is a full n x n byte matrix, W[j*n + i] = w_{ji} in {0,1}, with no self loops and no
 *   edges inside a cluster (Section II-A); the reinforcement gamma is a separate term
 *   gamma*v_i exactly as in Eq. (3) and Eq. (6), not folded into the diagonal;
 *   v is one byte (0/1) per neuron, s is one int32 per neuron.
 *
 * Conventions where the paper leaves a choice (all integer, so results are exact):
 *   - max_iters is the number of passes v^t -> v^{t+1}; the returned vector is the last one
 *     computed.  The return value is +p if pass p reproduced its input (v^p == v^{p-1},
 *     the confirming pass counts) and -max_iters if the cap was reached first.
 *   - convergence is decided per probe (a fixed point is absorbing, so this gives the same
 *     vectors as the batch-wide test of Algorithm 1).
 *   - sum-of-sum ties: every neuron reaching its cluster's maximum turns on (Eq. 4-5 read
 *     literally), including the case where that maximum is 0.  The latter sub-case is not
 *     covered by any value printed in the paper: PARITY UNPINNED for it.
 *   - sum-of-max runs with gamma = 1 (Theorem 1: any gamma > 0 behaves like gamma = 1);
 *     clusters that are all-zero in the probe are set to all-one first (Section III-C).
 *   - bail-out-early: the own-cluster contribution is gamma*v_i as in Eq. (6), so a
 *     neuron that is off stays off (Lemma 1).
 *   - hybrid (Algorithm 2): e is the number of all-zero clusters of that probe; pass 1
 *     keeps, inside erased clusters, exactly the neurons whose sum-of-sum score equals
 *     C - e; the following passes are bail-out-early on erased clusters only, known
 *     clusters are never touched; the cap counts pass 1 too; the stop test is made only
 *     after a bail-out-early pass.
 *
 * Pins (tests/test_oracle_pins.py): the printed code of message (9,4,3,10); the printed
 * 9x9 W, scores and activity vectors of the oscillation example of Section V-A; Lemmas
 * 1-3 and Theorems 1-4 as properties; brute-force clique enumeration on tiny networks;
 * edge density against 1-(1-1/L^2)^M.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_SUM_OF_SUM = 0, ORACLE_SUM_OF_MAX = 1, ORACLE_HYBRID = 2, ORACLE_SUM_OF_MAX_EQ = 3 };

/* ---- storing (Section II-A): each message adds the clique on its C active neurons ---- */
/* msgs: int32[M][C], symbols in [0,L).  Returns the number of messages skipped because a
 * symbol was out of range.  W is OR-ed into (zero it first for an empty network). */
int64_t gbnn_oracle_store(uint8_t *W, int C, int L, const int32_t *msgs, int64_t M)
{
    const int64_t n = (int64_t)C * L;
    int64_t skipped = 0;
    for (int64_t m = 0; m < M; ++m) {
        const int32_t *sym = msgs + m * C;
        int ok = 1;
        for (int c = 0; c < C; ++c)
            if (sym[c] < 0 || sym[c] >= L) ok = 0;
        if (!ok) { ++skipped; continue; }
        for (int c = 0; c < C; ++c)
            for (int c2 = 0; c2 < C; ++c2) {
                if (c2 == c) continue;              /* edges only between different clusters */
                int64_t a = (int64_t)c * L + sym[c];
                int64_t b = (int64_t)c2 * L + sym[c2];
                W[a * n + b] = 1;
            }
    }
    return skipped;
}

/* ---- sum-of-sum (Section III-A) ---- */

/* Eq. (3): s_i = gamma*v_i + sum over all neurons j of v_j * w_{ji}.  Terms with v_j = 0
 * are zero and are skipped. */
void gbnn_oracle_sos_scores(const uint8_t *W, int C, int L, const uint8_t *v, int gamma, int32_t *s)
{
    const int64_t n = (int64_t)C * L;
    for (int64_t i = 0; i < n; ++i) s[i] = gamma * (int32_t)v[i];
    for (int64_t j = 0; j < n; ++j) {
        if (!v[j]) continue;
        const uint8_t *row = W + j * n;
        for (int64_t i = 0; i < n; ++i) s[i] += row[i];
    }
}

/* Eq. (4)-(5): per cluster, the maximum score, then every neuron that reaches it. */
void gbnn_oracle_sos_select(const int32_t *s, int C, int L, uint8_t *v_next)
{
    for (int c = 0; c < C; ++c) {
        const int32_t *sc = s + (int64_t)c * L;
        int32_t smax = sc[0];
        for (int l = 1; l < L; ++l)
            if (sc[l] > smax) smax = sc[l];
        for (int l = 0; l < L; ++l)
            v_next[(int64_t)c * L + l] = (uint8_t)(sc[l] == smax);
    }
}

static int same_bytes(const uint8_t *a, const uint8_t *b, int64_t n) { return memcmp(a, b, (size_t)n) == 0; }

/* Algorithm 1 for one probe.  v0 has the erased clusters all-zero. */
int gbnn_oracle_sos(const uint8_t *W, int C, int L, const uint8_t *v0, uint8_t *v_out, int gamma, int max_iters)
{
    const int64_t n = (int64_t)C * L;
    uint8_t *v = (uint8_t *)malloc((size_t)n), *vn = (uint8_t *)malloc((size_t)n);
    int32_t *s = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    memcpy(v, v0, (size_t)n);
    int p = 0, ret = 0;
    for (;;) {
        gbnn_oracle_sos_scores(W, C, L, v, gamma, s);
        gbnn_oracle_sos_select(s, C, L, vn);
        ++p;
        int same = same_bytes(v, vn, n);
        memcpy(v, vn, (size_t)n);
        if (same) { ret = p; break; }
        if (p == max_iters) { ret = -p; break; }
    }
    memcpy(v_out, v, (size_t)n);
    free(v); free(vn); free(s);
    return ret;
}

/* ---- sum-of-max (Section III-C) ---- */

/* Initialisation for sum-of-max: every cluster with no active neuron becomes all active. */
void gbnn_oracle_som_init(int C, int L, uint8_t *v)
{
    for (int c = 0; c < C; ++c) {
        int any = 0;
        for (int l = 0; l < L; ++l) any |= v[(int64_t)c * L + l];
        if (!any)
            for (int l = 0; l < L; ++l) v[(int64_t)c * L + l] = 1;
    }
}

/* Eq. (6): s_i = gamma*v_i + sum over clusters c' of max over l' of v_{c'l'} * w_{(c'l') i}. */
void gbnn_oracle_som_scores_eq(const uint8_t *W, int C, int L, const uint8_t *v, int gamma, int32_t *s)
{
    const int64_t n = (int64_t)C * L;
    for (int64_t i = 0; i < n; ++i) {
        int32_t acc = gamma * (int32_t)v[i];
        for (int c2 = 0; c2 < C; ++c2) {
            int32_t mx = 0;
            for (int l2 = 0; l2 < L; ++l2) {
                int64_t j = (int64_t)c2 * L + l2;
                int32_t t = (int32_t)v[j] * (int32_t)W[j * n + i];
                if (t > mx) mx = t;
            }
            acc += mx;
        }
        s[i] = acc;
    }
}

/* Eq. (6)-(7), one pass: v_i <- [s_i == gamma + C - 1]. */
void gbnn_oracle_som_pass_eq(const uint8_t *W, int C, int L, const uint8_t *v, int gamma, uint8_t *v_next)
{
    const int64_t n = (int64_t)C * L;
    int32_t *s = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    gbnn_oracle_som_scores_eq(W, C, L, v, gamma, s);
    for (int64_t i = 0; i < n; ++i) v_next[i] = (uint8_t)(s[i] == gamma + C - 1);
    free(s);
}

/* Bail-out-early pass (Section IV-D) with gamma = 1.  Neuron i walks the clusters in order;
 * its own cluster contributes v_i; another cluster contributes 1 at the first j in it with
 * v_j > 0 and w_{ji} > 0; the walk stops at the first cluster that contributes nothing.
 * The scan of a cluster visits only its currently active neurons, in index order (the
 * "candidate pool" of Section VI): these are the only j that can pass the v_j > 0 test.
 * update_cluster (may be NULL = all): clusters whose neurons are updated; the others are
 * copied (Algorithm 2 updates erased clusters only). */
void gbnn_oracle_som_pass_boe(const uint8_t *W, int C, int L, const uint8_t *v, uint8_t *v_next,
                              const uint8_t *update_cluster)
{
    const int64_t n = (int64_t)C * L;
    int32_t *act = (int32_t *)malloc(sizeof(int32_t) * (size_t)n); /* active neurons, cluster by cluster */
    int32_t *beg = (int32_t *)malloc(sizeof(int32_t) * (size_t)(C + 1));
    int32_t cnt = 0;
    for (int c = 0; c < C; ++c) {
        beg[c] = cnt;
        for (int l = 0; l < L; ++l)
            if (v[(int64_t)c * L + l]) act[cnt++] = c * L + l;
    }
    beg[C] = cnt;
    for (int ci = 0; ci < C; ++ci) {
        for (int l = 0; l < L; ++l) {
            const int64_t i = (int64_t)ci * L + l;
            if (update_cluster && !update_cluster[ci]) { v_next[i] = v[i]; continue; }
            int32_t score = 0;
            for (int c = 0; c < C; ++c) {
                int32_t before = score;
                if (c == ci) {
                    score += (int32_t)v[i];          /* gamma*v_i with gamma = 1 */
                } else {
                    for (int32_t a = beg[c]; a < beg[c + 1]; ++a)
                        if (W[(int64_t)act[a] * n + i]) { score += 1; break; }
                }
                if (score == before) break;          /* this cluster gave nothing: bail out */
            }
            v_next[i] = (uint8_t)(score == C);       /* gamma + C - 1 with gamma = 1 */
        }
    }
    free(act); free(beg);
}

/* Sum-of-max retrieval of one probe.  form 0: Eq. (6)-(7) literally with the given gamma > 0;
 * form 1: bail-out-early (gamma = 1). */
int gbnn_oracle_som(const uint8_t *W, int C, int L, const uint8_t *v0, uint8_t *v_out, int form, int gamma,
                    int max_iters)
{
    const int64_t n = (int64_t)C * L;
    uint8_t *v = (uint8_t *)malloc((size_t)n), *vn = (uint8_t *)malloc((size_t)n);
    memcpy(v, v0, (size_t)n);
    gbnn_oracle_som_init(C, L, v);
    int p = 0, ret = 0;
    for (;;) {
        if (form == 0) gbnn_oracle_som_pass_eq(W, C, L, v, gamma, vn);
        else gbnn_oracle_som_pass_boe(W, C, L, v, vn, NULL);
        ++p;
        int same = same_bytes(v, vn, n);
        memcpy(v, vn, (size_t)n);
        if (same) { ret = p; break; }
        if (p == max_iters) { ret = -p; break; }
    }
    memcpy(v_out, v, (size_t)n);
    free(v); free(vn);
    return ret;
}

/* ---- hybrid / joint scheme (Algorithm 2) ---- */
int gbnn_oracle_hybrid(const uint8_t *W, int C, int L, const uint8_t *v0, uint8_t *v_out, int max_iters)
{
    const int64_t n = (int64_t)C * L;
    uint8_t *v = (uint8_t *)malloc((size_t)n), *vn = (uint8_t *)malloc((size_t)n);
    uint8_t *erased = (uint8_t *)malloc((size_t)C);
    int32_t *s = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    int e = 0;
    for (int c = 0; c < C; ++c) {
        int any = 0;
        for (int l = 0; l < L; ++l) any |= v0[(int64_t)c * L + l];
        erased[c] = (uint8_t)!any;
        e += !any;
    }
    /* lines 1-5: erased clusters stay off, S^0 = W V^0 (no reinforcement term is needed:
     * erased neurons are off), keep the neurons of erased clusters that got exactly C - e
     * signals; known clusters are kept as they are. */
    gbnn_oracle_sos_scores(W, C, L, v0, 0, s);
    for (int c = 0; c < C; ++c)
        for (int l = 0; l < L; ++l) {
            int64_t i = (int64_t)c * L + l;
            v[i] = erased[c] ? (uint8_t)(s[i] == C - e) : v0[i];
        }
    int p = 1, ret = 0;
    if (p == max_iters) {
        ret = -p;
    } else {
        for (;;) {                                    /* lines 8-13 */
            gbnn_oracle_som_pass_boe(W, C, L, v, vn, erased);
            ++p;
            int same = same_bytes(v, vn, n);          /* known clusters are copies: this compares erased ones */
            memcpy(v, vn, (size_t)n);
            if (same) { ret = p; break; }
            if (p == max_iters) { ret = -p; break; }
        }
    }
    memcpy(v_out, v, (size_t)n);
    free(v); free(vn); free(erased); free(s);
    return ret;
}

/* ---- batch driver: K independent probes, V0 / V_out are uint8[K][n] ---- */
/* Returns the number of threads used.  iters_out may be NULL. */
int gbnn_oracle_retrieve(const uint8_t *W, int C, int L, const uint8_t *V0, uint8_t *V_out, int64_t K, int rule,
                         int gamma, int max_iters, int32_t *iters_out, int nthreads)
{
    const int64_t n = (int64_t)C * L;
    int used = 1;
#ifdef _OPENMP
    if (nthreads < 1) nthreads = omp_get_max_threads();
    used = nthreads;
#pragma omp parallel for schedule(dynamic, 16) num_threads(nthreads)
#endif
    for (int64_t k = 0; k < K; ++k) {
        const uint8_t *v0 = V0 + k * n;
        uint8_t *vo = V_out + k * n;
        int it;
        switch (rule) {
        case ORACLE_SUM_OF_SUM:    it = gbnn_oracle_sos(W, C, L, v0, vo, gamma, max_iters); break;
        case ORACLE_SUM_OF_MAX:    it = gbnn_oracle_som(W, C, L, v0, vo, 1, 1, max_iters); break;
        case ORACLE_SUM_OF_MAX_EQ: it = gbnn_oracle_som(W, C, L, v0, vo, 0, gamma, max_iters); break;
        default:                   it = gbnn_oracle_hybrid(W, C, L, v0, vo, max_iters); break;
        }
        if (iters_out) iters_out[k] = it;
    }
    return used;
}
