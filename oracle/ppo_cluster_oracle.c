/*
 * CPU oracle for the cluster form of the exact partition-and-placement search.  TEST INFRASTRUCTURE
 * ONLY: nothing in the product path may call into this file.  It shares no code with the HIP library.
 *
 * Problem.  In the paper's setting the cluster is larger than the set of nodes that end up hosting a
 * partition: the partitioner decides how many partitions there are (Sec. III-B1, the path found by
 * Alg. 1 fixes |S|), and the placement picks that many nodes out of the communication graph as a
 * simple path (Sec. III-B2, "N ... with length |S|"; Sec. IV tests clusters of 5 to 50 nodes).  The
 * exact counterpart therefore minimises over the number of segments as well:
 *   a chain of L layers (m[i] weight size, t[i] size of the tensor leaving layer i);
 *   a cluster of n nodes with capacities M[j] and a symmetric bandwidth matrix B;
 *   a solution is a number p, 1 <= p <= min(pmax, L), a sequence of p DISTINCT nodes j_0..j_{p-1}
 *   and cuts 0 = c_0 < c_1 < ... < c_p = L; segment s = layers [c_s, c_{s+1}) runs on node j_s;
 *   gamma_s = t[c_s - 1] / B[j_{s-1}][j_s] (Eq. 3), beta = max over s >= 1 of gamma_s (Eq. 2; 0 if
 *   p = 1), feasible iff every segment's weight sum is within its node's capacity;
 *   beta* = min over all feasible solutions; +inf if there is none.
 * Precision as in the fixed-k oracle: binary64 sequential prefix sums of m, "fits" is <=, gamma is
 * one IEEE binary32 division, min and max exact.
 * Tie rules that make the answer unique:
 *   C1: among node sequences reaching beta*, the lexicographically smallest, a sequence sorting
 *       before every sequence it is a proper prefix of;
 *   C2: among the feasible cut vectors of that sequence with bottleneck beta*, the one that
 *       minimises c_{p-1}, then c_{p-2}, ..., then c_1 (rule T2 of the fixed-k problem).
 *
 * Three routes:
 *   ppo_cluster_oracle_bruteforce  every (sequence, cut vector) pair from the definition (tiny inputs);
 *   ppo_cluster_oracle_exhaustive  every sequence in lexicographic order, a plain windowed min-max
 *                                  chain DP for each;
 *   ppo_cluster_oracle_subset_dp   dynamic programme over sets of still-unused nodes (n <= 20).
 * The first two take clusters of up to 64 nodes: with few segments allowed (pmax) the sequences to walk are few.
 * Pins (tests/test_cluster_oracle_pins.py): agreement with the fixed-k oracle's definition route on
 * every node subset of every size (assembled in Python), closed forms (whole model on one node;
 * two nodes), monotonicity in pmax and in the cluster, a useless node changes nothing, relabelling,
 * the paper's 10.2 Mbit / 6 Mbps example placed in a larger cluster, agreement of the three routes.
 * Parity unpinned: nothing in this file.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_ETOOBIG (-2)
#define ORC_EDATA (-3)
#define ORC_ENOMEM (-4)

#define ORC_MAX_N 64        /* routes that walk node sequences */
#define ORC_MAX_N_SUBSETS 20 /* the route over sets of unused nodes keeps n 2^n rows */
#define ORC_MAX_L 4096

typedef struct {
    const float *t, *m, *M, *B;
    int L, n, pmax;
    double *P; /* L+1 prefix sums */
} cl_t;

static int cl_fits(const cl_t *I, int i, int e, int node) { return (I->P[e] - I->P[i]) <= (double)I->M[node]; }

static float cl_gamma(const cl_t *I, int cut, int a, int b) {
    volatile float q = I->t[cut - 1] / I->B[a * I->n + b];
    if (q == 0.0f) return 0.0f; /* nothing to send takes no time: +0, also when t carries a sign bit */
    return q;
}

static int cl_check(const float *t, const float *m, int L, const float *M, const float *B, int n, int pmax) {
    if (L < 1 || n < 1 || pmax < 1 || pmax > n) return ORC_EINVAL;
    if (n > ORC_MAX_N || L > ORC_MAX_L) return ORC_ETOOBIG;
    if (!t || !m || !M || !B) return ORC_EINVAL;
    for (int i = 0; i < L; ++i)
        if (!isfinite(t[i]) || !isfinite(m[i]) || t[i] < 0.0f || m[i] < 0.0f) return ORC_EDATA;
    for (int j = 0; j < n; ++j)
        if (!isfinite(M[j]) || M[j] < 0.0f) return ORC_EDATA;
    for (int a = 0; a < n; ++a)
        for (int b = 0; b < n; ++b) {
            if (a == b) continue;
            float x = B[a * n + b], y = B[b * n + a];
            if (!isfinite(x) || !(x > 0.0f) || memcmp(&x, &y, sizeof x) != 0) return ORC_EDATA;
        }
    return ORC_OK;
}

static int cl_open(cl_t *I, const float *t, const float *m, int L, const float *M, const float *B, int n, int pmax) {
    int rc = cl_check(t, m, L, M, B, n, pmax);
    if (rc) return rc;
    I->t = t; I->m = m; I->M = M; I->B = B; I->L = L; I->n = n; I->pmax = pmax < L ? pmax : L;
    I->P = (double *)malloc(sizeof(double) * (L + 1));
    if (!I->P) return ORC_ENOMEM;
    I->P[0] = 0.0;
    for (int i = 0; i < L; ++i) I->P[i + 1] = I->P[i] + (double)m[i];
    return ORC_OK;
}

static void cl_none(const cl_t *I, float *beta, int32_t *segs, int32_t *cuts, int32_t *order) {
    *beta = INFINITY;
    *segs = 0;
    for (int s = 0; s < I->n; ++s) order[s] = -1;
    for (int s = 0; s + 1 < I->n; ++s) cuts[s] = -1;
}

static void cl_emit(const cl_t *I, float b, int p, const int *seq, const int *cut, float *beta, int32_t *segs,
                    int32_t *cuts, int32_t *order) {
    cl_none(I, beta, segs, cuts, order);
    *beta = b;
    *segs = p;
    for (int s = 0; s < p; ++s) order[s] = seq[s];
    for (int s = 0; s + 1 < p; ++s) cuts[s] = cut[s];
}

/* ------------------------------------------------------------------ route 1: the definition */

typedef struct {
    const cl_t *I;
    int seq[ORC_MAX_N], used[ORC_MAX_N];
    int found, bp, bseq[ORC_MAX_N], bcut[ORC_MAX_N];
    float bbeta;
} bf_t;

/* best cut vector (rule C2) of the sequence seq[0..p-1]; returns 0 if none is feasible */
static int bf_best_cuts(const cl_t *I, const int *seq, int p, float *beta, int *cut) {
    const int L = I->L;
    int c[ORC_MAX_N + 1], found = 0;
    float bb = INFINITY;
    c[0] = 0; c[p] = L;
    for (int s = 1; s < p; ++s) c[s] = s;
    for (;;) {
        int ok = 1;
        float b = 0.0f;
        for (int s = 0; s < p && ok; ++s) {
            if (!cl_fits(I, c[s], c[s + 1], seq[s])) ok = 0;
            else if (s > 0) {
                float g = cl_gamma(I, c[s], seq[s - 1], seq[s]);
                if (g > b) b = g;
            }
        }
        if (ok) {
            int better = !found || b < bb;
            if (!better && b == bb) {
                /* compare c_{p-1} first, then c_{p-2}, ... */
                for (int s = p - 1; s >= 1; --s)
                    if (c[s] != cut[s - 1]) { better = c[s] < cut[s - 1]; break; }
            }
            if (better) {
                found = 1; bb = b;
                for (int s = 1; s < p; ++s) cut[s - 1] = c[s];
            }
        }
        int s = p - 1;
        while (s >= 1 && c[s] == L - (p - s)) --s;
        if (s < 1) break;
        ++c[s];
        for (int u = s + 1; u < p; ++u) c[u] = c[u - 1] + 1;
    }
    *beta = bb;
    return found;
}

/* sequences in lexicographic order, each before its extensions; strict < keeps the first optimum */
static void bf_walk(bf_t *W, int p) {
    const cl_t *I = W->I;
    if (p >= 1) {
        float b;
        int cut[ORC_MAX_N];
        if (bf_best_cuts(I, W->seq, p, &b, cut) && (!W->found || b < W->bbeta)) {
            W->found = 1; W->bbeta = b; W->bp = p;
            memcpy(W->bseq, W->seq, sizeof(int) * p);
            memcpy(W->bcut, cut, sizeof(int) * (p > 1 ? p - 1 : 0));
        }
    }
    if (p == I->pmax) return;
    for (int j = 0; j < I->n; ++j) {
        if (W->used[j]) continue;
        W->used[j] = 1; W->seq[p] = j;
        bf_walk(W, p + 1);
        W->used[j] = 0;
    }
}

int ppo_cluster_oracle_bruteforce(const float *t, const float *m, int L, const float *M, const float *B, int n,
                                  int pmax, float *beta, int32_t *segs, int32_t *cuts, int32_t *order) {
    cl_t I;
    int rc = cl_open(&I, t, m, L, M, B, n, pmax);
    if (rc) return rc;
    bf_t *W = (bf_t *)calloc(1, sizeof(bf_t));
    if (!W) { free(I.P); return ORC_ENOMEM; }
    W->I = &I;
    bf_walk(W, 0);
    if (W->found) cl_emit(&I, W->bbeta, W->bp, W->bseq, W->bcut, beta, segs, cuts, order);
    else cl_none(&I, beta, segs, cuts, order);
    free(W); free(I.P);
    return ORC_OK;
}

/* ------------------------------------------------------------------ route 2: a chain DP per sequence */

/* D_s[e] = least bottleneck of layers [0,e) on seq[0..s], one non-empty segment each; rows of L+1 */
static float seq_dp(const cl_t *I, const int *seq, int p, float *rows) {
    const int L = I->L, W = L + 1;
    for (int x = 0; x < p * W; ++x) rows[x] = INFINITY;
    for (int e = 1; e <= L - (p - 1); ++e)
        if (cl_fits(I, 0, e, seq[0])) rows[e] = 0.0f;
    for (int s = 1; s < p; ++s) {
        const float *prev = rows + (s - 1) * W;
        float *cur = rows + s * W;
        for (int e = s + 1; e <= L - (p - 1 - s); ++e) {
            float best = INFINITY;
            for (int i = e - 1; i >= s; --i) {
                if (!cl_fits(I, i, e, seq[s])) break; /* the sum only grows as i falls */
                float g = cl_gamma(I, i, seq[s - 1], seq[s]);
                float c = prev[i] > g ? prev[i] : g;
                if (c < best) best = c;
            }
            cur[e] = best;
        }
    }
    return rows[(p - 1) * W + L];
}

static void seq_cuts(const cl_t *I, const int *seq, int p, const float *rows, float beta, int *cut) {
    const int W = I->L + 1;
    int e = I->L;
    for (int s = p - 1; s >= 1; --s) {
        const float *prev = rows + (s - 1) * W;
        int chosen = -1;
        for (int i = s; i <= e - 1 && chosen < 0; ++i) {
            if (!cl_fits(I, i, e, seq[s])) continue;
            float g = cl_gamma(I, i, seq[s - 1], seq[s]);
            float c = prev[i] > g ? prev[i] : g;
            if (c <= beta) chosen = i;
        }
        cut[s - 1] = chosen;
        e = chosen;
    }
}

typedef struct {
    const cl_t *I;
    float *rows;
    int seq[ORC_MAX_N], used[ORC_MAX_N];
    int found, bp, bseq[ORC_MAX_N];
    float bbeta;
    uint64_t visited;
} ex_t;

static void ex_walk(ex_t *W, int p) {
    const cl_t *I = W->I;
    if (p >= 1) {
        float b = seq_dp(I, W->seq, p, W->rows);
        ++W->visited;
        if (!isinf(b) && (!W->found || b < W->bbeta)) {
            W->found = 1; W->bbeta = b; W->bp = p;
            memcpy(W->bseq, W->seq, sizeof(int) * p);
        }
    }
    if (p == I->pmax) return;
    for (int j = 0; j < I->n; ++j) {
        if (W->used[j]) continue;
        W->used[j] = 1; W->seq[p] = j;
        ex_walk(W, p + 1);
        W->used[j] = 0;
    }
}

int ppo_cluster_oracle_exhaustive(const float *t, const float *m, int L, const float *M, const float *B, int n,
                                  int pmax, float *beta, int32_t *segs, int32_t *cuts, int32_t *order,
                                  uint64_t *sequences_out) {
    cl_t I;
    int rc = cl_open(&I, t, m, L, M, B, n, pmax);
    if (rc) return rc;
    ex_t *W = (ex_t *)calloc(1, sizeof(ex_t));
    float *rows = (float *)malloc(sizeof(float) * (size_t)n * (L + 1));
    if (!W || !rows) { free(W); free(rows); free(I.P); return ORC_ENOMEM; }
    W->I = &I; W->rows = rows;
    ex_walk(W, 0);
    if (W->found) {
        int cut[ORC_MAX_N];
        seq_dp(&I, W->bseq, W->bp, rows);
        seq_cuts(&I, W->bseq, W->bp, rows, W->bbeta, cut);
        cl_emit(&I, W->bbeta, W->bp, W->bseq, cut, beta, segs, cuts, order);
    } else {
        cl_none(&I, beta, segs, cuts, order);
    }
    if (sequences_out) *sequences_out = W->visited;
    free(W); free(rows); free(I.P);
    return ORC_OK;
}

/* beta of ONE given sequence (least over its cut vectors), +inf if none is feasible */
int ppo_cluster_oracle_sequence(const float *t, const float *m, int L, const float *M, const float *B, int n,
                                const int32_t *seq, int p, float *beta) {
    cl_t I;
    if (p < 1 || p > n || p > L) return ORC_EINVAL;
    int rc = cl_open(&I, t, m, L, M, B, n, n);
    if (rc) return rc;
    int s32[ORC_MAX_N], seen[ORC_MAX_N] = {0};
    for (int s = 0; s < p; ++s) {
        if (seq[s] < 0 || seq[s] >= n || seen[seq[s]]) { free(I.P); return ORC_EINVAL; }
        seen[seq[s]] = 1; s32[s] = seq[s];
    }
    float *rows = (float *)malloc(sizeof(float) * (size_t)p * (L + 1));
    if (!rows) { free(I.P); return ORC_ENOMEM; }
    *beta = seq_dp(&I, s32, p, rows);
    free(rows); free(I.P);
    return ORC_OK;
}

/* ------------------------------------------------------------------ route 3: subsets of unused nodes */

/* G[S][j][i], S the set of nodes not used before layer i, j in S: least bottleneck of layers [i,L) if
 * node j hosts the segment that starts at i and the segments after it go to distinct nodes of S \ {j}.
 * The number of segments before this one is n - |S|, so one more segment may follow only while
 * n - |S| + 1 < pmax. */
int ppo_cluster_oracle_subset_dp(const float *t, const float *m, int L, const float *M, const float *B, int n,
                                 int pmax, float *beta, int32_t *segs, int32_t *cuts, int32_t *order) {
    if (n > ORC_MAX_N_SUBSETS) return ORC_ETOOBIG;
    cl_t I;
    int rc = cl_open(&I, t, m, L, M, B, n, pmax);
    if (rc) return rc;
    pmax = I.pmax;
    const int W = L + 1;
    const size_t nS = (size_t)1 << n;
    float *G = (float *)malloc(sizeof(float) * nS * n * W);
    unsigned char *reach = (unsigned char *)calloc((size_t)n * W, 1);
    if (!G || !reach) { free(G); free(reach); free(I.P); return ORC_ENOMEM; }
#define GX(S, j, i) G[((size_t)(S) * n + (j)) * W + (i)]
    for (size_t x = 0; x < nS * n * W; ++x) G[x] = INFINITY;
    /* increasing numeric order: S \ {j} always comes before S */
    for (size_t S = 1; S < nS; ++S) {
        const int before = n - __builtin_popcountll(S);
        if (before + 1 > pmax) continue;
        const int more = before + 1 < pmax;
        for (int j = 0; j < n; ++j) {
            if (!(S >> j & 1)) continue;
            const size_t rest = S & ~((size_t)1 << j);
            for (int i = 0; i < L; ++i) {
                float best = INFINITY;
                for (int e = i + 1; e <= L; ++e) {
                    if (!cl_fits(&I, i, e, j)) break;
                    if (e == L) { best = 0.0f < best ? 0.0f : best; break; }
                    if (!more) continue;
                    for (int j2 = 0; j2 < n; ++j2) {
                        if (!(rest >> j2 & 1)) continue;
                        float g = cl_gamma(&I, e, j, j2);
                        float tail = GX(rest, j2, e);
                        float c = tail > g ? tail : g;
                        if (c < best) best = c;
                    }
                }
                GX(S, j, i) = best;
            }
        }
    }
    const size_t all = nS - 1;
    float b = INFINITY;
    for (int j = 0; j < n; ++j)
        if (GX(all, j, 0) < b) b = GX(all, j, 0);
    if (isinf(b)) {
        cl_none(&I, beta, segs, cuts, order);
    } else {
        /* Rule C1, position by position.  reach[s][e] = 1 iff layers [0,e) can go on seq[0..s] with every
         * segment fitting and every gamma <= b.  The sequence ends as soon as reach[s][L] holds. */
        int seq[ORC_MAX_N], p = 0;
        size_t remaining = all;
        for (int s = 0; s < pmax; ++s) {
            int pick = -1;
            for (int j = 0; j < n && pick < 0; ++j) {
                if (!(remaining >> j & 1)) continue;
                if (s == 0) {
                    if (GX(remaining, j, 0) <= b) pick = j;
                } else {
                    for (int e = s; e < L && pick < 0; ++e)
                        if (reach[(s - 1) * W + e] && cl_gamma(&I, e, seq[s - 1], j) <= b && GX(remaining, j, e) <= b)
                            pick = j;
                }
            }
            seq[s] = pick;
            remaining &= ~((size_t)1 << pick);
            for (int e = s + 1; e <= L; ++e) {
                int r = 0;
                if (s == 0) r = cl_fits(&I, 0, e, pick);
                else
                    for (int i = s; i < e && !r; ++i)
                        r = reach[(s - 1) * W + i] && cl_fits(&I, i, e, pick) && cl_gamma(&I, i, seq[s - 1], pick) <= b;
                reach[s * W + e] = (unsigned char)r;
            }
            p = s + 1;
            if (reach[s * W + L]) break;
        }
        /* Rule C2 from the reachability table */
        int cut[ORC_MAX_N], e = L;
        for (int s = p - 1; s >= 1; --s) {
            int chosen = -1;
            for (int i = s; i < e && chosen < 0; ++i)
                if (reach[(s - 1) * W + i] && cl_fits(&I, i, e, seq[s]) && cl_gamma(&I, i, seq[s - 1], seq[s]) <= b)
                    chosen = i;
            cut[s - 1] = chosen;
            e = chosen;
        }
        cl_emit(&I, b, p, seq, cut, beta, segs, cuts, order);
    }
#undef GX
    free(G); free(reach); free(I.P);
    return ORC_OK;
}
