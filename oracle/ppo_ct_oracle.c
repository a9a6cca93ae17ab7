/*
 * CPU oracle for the search with the compute-time term.  TEST INFRASTRUCTURE ONLY: nothing in the
 * product path may call into this file; it shares no code with the HIP library.
 *
 * Sec. I, Eq. 1 of the paper defines the bottleneck latency over BOTH kinds of stage of the inference
 * pipeline: the compute time c_k of the operations on node k and the communication time gamma_k
 * between node k-1 and node k; beta is the largest of all of them.  The paper then drops the compute
 * times (Eq. 2).  This file keeps them:
 *   a chain of L layers with weight sizes m[i], transfer sizes t[i] and compute work w[i];
 *   k nodes with capacities M[j], speeds v[j] and a symmetric bandwidth matrix B;
 *   a solution is a permutation pi of the nodes and cuts 0=c_0<c_1<...<c_{k-1}<c_k=L;
 *   comp_s  = (work of layers [c_s, c_{s+1})) / v[pi[s]]                      s = 0..k-1
 *   gamma_s = t[c_s - 1] / B[pi[s-1]][pi[s]]                                   s = 1..k-1   (Eq. 3)
 *   beta    = max over all comp_s and gamma_s                                               (Eq. 1)
 *   feasible iff every segment's weight sum is within its node's capacity (memory rule of Sec. III-B).
 * The paper gives no per-layer compute data and no unit; the reading taken here: work in any unit, speed
 * in that unit per second, so that comp is in seconds like gamma.
 *
 * Precision, fixed for both sides of every comparison:
 *   P[i+1] = P[i] + (double)m[i] and Q[i+1] = Q[i] + (double)w[i], sequentially in binary64;
 *   a segment fits iff (P[e]-P[i]) <= (double)M[j];
 *   comp = (float)((Q[e]-Q[i]) / (double)v[j]): binary64 difference and division, rounded once to binary32;
 *   gamma is one binary32 division (a zero of either sign gives +0); min and max are exact.
 * Tie rules as in the search without the term: lowest lexicographic rank among the optimal orderings, then
 * the cut vector that minimises c_{k-1}, then c_{k-2}, ...
 *
 * Three routes: bruteforce (every cut vector x permutation, the definition), exhaustive (one chain DP per
 * permutation, in lexicographic order), subset_dp (over node subsets, boolean reachability for the tie rules).
 * Pins: tests/test_ct_oracle_pins.py (w = 0 gives the answers of the oracle without the term, bit for bit;
 * closed forms for k = 1, for t = 0 with equal work, and a hand-worked slow node; the three routes agree;
 * monotonicity; exact scaling by two).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define CT_OK 0
#define CT_EINVAL (-1)
#define CT_ETOOBIG (-2)
#define CT_EDATA (-3)
#define CT_ENOMEM (-4)
#define CT_MAX_K 12
#define CT_MAX_L 1024

typedef struct {
    const float *t, *m, *w, *M, *v, *B;
    int L, k;
    double *P, *Q;
} ct_t;

static int ct_check(const float *t, const float *m, const float *w, int L, const float *M, const float *v,
                    const float *B, int k) {
    if (L < 1 || k < 1 || k > L) return CT_EINVAL;
    if (k > CT_MAX_K || L > CT_MAX_L) return CT_ETOOBIG;
    if (!t || !m || !w || !M || !v || !B) return CT_EINVAL;
    for (int i = 0; i < L; ++i)
        if (!isfinite(t[i]) || !isfinite(m[i]) || !isfinite(w[i]) || t[i] < 0.0f || m[i] < 0.0f || w[i] < 0.0f)
            return CT_EDATA;
    for (int j = 0; j < k; ++j)
        if (!isfinite(M[j]) || M[j] < 0.0f || !isfinite(v[j]) || !(v[j] > 0.0f)) return CT_EDATA;
    for (int a = 0; a < k; ++a)
        for (int b = 0; b < k; ++b) {
            if (a == b) continue;
            float x = B[a * k + b], y = B[b * k + a];
            if (!isfinite(x) || !(x > 0.0f) || memcmp(&x, &y, sizeof x) != 0) return CT_EDATA;
        }
    return CT_OK;
}

static int ct_open(ct_t *I, const float *t, const float *m, const float *w, int L, const float *M, const float *v,
                   const float *B, int k) {
    int rc = ct_check(t, m, w, L, M, v, B, k);
    if (rc) return rc;
    I->t = t; I->m = m; I->w = w; I->M = M; I->v = v; I->B = B; I->L = L; I->k = k;
    I->P = (double *)malloc(sizeof(double) * 2 * (L + 1));
    if (!I->P) return CT_ENOMEM;
    I->Q = I->P + (L + 1);
    I->P[0] = 0.0; I->Q[0] = 0.0;
    for (int i = 0; i < L; ++i) {
        I->P[i + 1] = I->P[i] + (double)m[i];
        I->Q[i + 1] = I->Q[i] + (double)w[i];
    }
    return CT_OK;
}

static int ct_fits(const ct_t *I, int i, int e, int node) { return (I->P[e] - I->P[i]) <= (double)I->M[node]; }

/* compute time of layers [i, e) on a node: the c_k of Eq. 1 */
static float ct_comp(const ct_t *I, int i, int e, int node) {
    volatile double d = (I->Q[e] - I->Q[i]) / (double)I->v[node];
    volatile float f = (float)d;
    return f;
}

/* communication time over a cut: Eq. 3 */
static float ct_gamma(const ct_t *I, int cut, int a, int b) {
    volatile float q = I->t[cut - 1] / I->B[a * I->k + b];
    if (q == 0.0f) return 0.0f;
    return q;
}

static float fmax2(float a, float b) { return a > b ? a : b; }

static uint64_t ct_factorial(int n) {
    uint64_t f = 1;
    for (int i = 2; i <= n; ++i) f *= (uint64_t)i;
    return f;
}

static void ct_unrank(uint64_t rank, int k, int *perm) {
    int avail[CT_MAX_K + 1], n = k;
    for (int j = 0; j < k; ++j) avail[j] = j;
    for (int p = 0; p < k; ++p) {
        uint64_t f = ct_factorial(k - 1 - p);
        int d = (int)(rank / f);
        rank -= (uint64_t)d * f;
        perm[p] = avail[d];
        for (int j = d; j + 1 < n; ++j) avail[j] = avail[j + 1];
        --n;
    }
}

static int ct_next_perm(int *a, int n) {
    int i = n - 2;
    while (i >= 0 && a[i] > a[i + 1]) --i;
    if (i < 0) return 0;
    int j = n - 1;
    while (a[j] < a[i]) --j;
    int tmp = a[i]; a[i] = a[j]; a[j] = tmp;
    for (int l = i + 1, r = n - 1; l < r; ++l, --r) { tmp = a[l]; a[l] = a[r]; a[r] = tmp; }
    return 1;
}

/* beta of one explicit solution, from the definition; +inf and feasible = 0 if a segment does not fit */
int ppo_ct_oracle_evaluate(const float *t, const float *m, const float *w, int L, const float *M, const float *v,
                           const float *B, int k, const int32_t *order, const int32_t *cuts, float *beta,
                           int32_t *feasible) {
    ct_t I;
    int rc = ct_open(&I, t, m, w, L, M, v, B, k);
    if (rc) return rc;
    int ok = 1, prev = 0;
    float b = 0.0f;
    for (int s = 0; ok && s < k; ++s) {
        int end = s == k - 1 ? L : cuts[s];
        if (end <= prev || end > L || order[s] < 0 || order[s] >= k) { ok = 0; break; }
        if (!ct_fits(&I, prev, end, order[s])) ok = 0;
        b = fmax2(b, ct_comp(&I, prev, end, order[s]));
        if (s > 0) b = fmax2(b, ct_gamma(&I, prev, order[s - 1], order[s]));
        prev = end;
    }
    *feasible = ok;
    *beta = ok ? b : INFINITY;
    free(I.P);
    return CT_OK;
}

static void ct_report(int k, int found, float beta, uint64_t rank, const int *cuts, float *beta_out, int32_t *cuts_out,
                      int32_t *order_out) {
    if (found) {
        int p[CT_MAX_K];
        ct_unrank(rank, k, p);
        *beta_out = beta;
        for (int s = 0; s < k; ++s) order_out[s] = p[s];
        for (int s = 0; s + 1 < k; ++s) cuts_out[s] = cuts[s];
    } else {
        *beta_out = INFINITY;
        for (int s = 0; s < k; ++s) order_out[s] = -1;
        for (int s = 0; s + 1 < k; ++s) cuts_out[s] = -1;
    }
}

/* ---------------------------------------------------------------- the definition, pair by pair */
int ppo_ct_oracle_bruteforce(const float *t, const float *m, const float *w, int L, const float *M, const float *v,
                             const float *B, int k, float *beta_out, int32_t *cuts_out, int32_t *order_out) {
    ct_t I;
    int rc = ct_open(&I, t, m, w, L, M, v, B, k);
    if (rc) return rc;
    int perm[CT_MAX_K], c[CT_MAX_K + 1], best_cuts[CT_MAX_K], found = 0;
    float best = INFINITY;
    uint64_t best_rank = 0, rank = 0;
    for (int j = 0; j < k; ++j) perm[j] = j;
    do {
        for (int s = 1; s < k; ++s) c[s] = s;
        c[0] = 0; c[k] = L;
        for (;;) {
            int ok = 1;
            float b = 0.0f;
            for (int s = 0; s < k && ok; ++s) {
                if (!ct_fits(&I, c[s], c[s + 1], perm[s])) { ok = 0; break; }
                b = fmax2(b, ct_comp(&I, c[s], c[s + 1], perm[s]));
                if (s > 0) b = fmax2(b, ct_gamma(&I, c[s], perm[s - 1], perm[s]));
            }
            if (ok) {
                int better = !found || b < best;
                if (!better && b == best) {
                    if (rank < best_rank) better = 1;
                    else if (rank == best_rank) {
                        /* rule for the cuts: compare c_{k-1} first, then c_{k-2}, ... */
                        for (int s = k - 1; s >= 1; --s)
                            if (c[s] != best_cuts[s - 1]) { better = c[s] < best_cuts[s - 1]; break; }
                    }
                }
                if (better) {
                    found = 1; best = b; best_rank = rank;
                    for (int s = 1; s < k; ++s) best_cuts[s - 1] = c[s];
                }
            }
            int s = k - 1;
            while (s >= 1 && c[s] == L - (k - s)) --s;
            if (s < 1) break;
            ++c[s];
            for (int u = s + 1; u < k; ++u) c[u] = c[u - 1] + 1;
        }
        ++rank;
    } while (ct_next_perm(perm, k));
    ct_report(k, found, best, best_rank, best_cuts, beta_out, cuts_out, order_out);
    free(I.P);
    return CT_OK;
}

/* ---------------------------------------------------------------- one chain DP per ordering */
/* D_s[e] = least bottleneck of layers [0,e) on nodes perm[0..s], one non-empty segment each:
 *   D_0[e] = comp(0, e, perm[0]) if it fits,
 *   D_s[e] = min over fitting starts i of max(D_{s-1}[i], gamma(i), comp(i, e, perm[s])). */
static float ct_chain_dp(const ct_t *I, const int *perm, float *rows) {
    const int L = I->L, k = I->k, W = L + 1;
    for (int i = 0; i < k * W; ++i) rows[i] = INFINITY;
    for (int e = 1; e <= L - (k - 1); ++e)
        if (ct_fits(I, 0, e, perm[0])) rows[e] = ct_comp(I, 0, e, perm[0]);
    for (int s = 1; s < k; ++s) {
        const float *prev = rows + (s - 1) * W;
        float *cur = rows + s * W;
        for (int e = s + 1; e <= L - (k - 1 - s); ++e) {
            float best = INFINITY;
            for (int i = e - 1; i >= s; --i) {
                if (!ct_fits(I, i, e, perm[s])) break;   /* the weight of [i, e) only grows as i falls */
                float c = fmax2(fmax2(prev[i], ct_gamma(I, i, perm[s - 1], perm[s])), ct_comp(I, i, e, perm[s]));
                if (c < best) best = c;
            }
            cur[e] = best;
        }
    }
    return rows[(k - 1) * W + L];
}

static void ct_traceback(const ct_t *I, const int *perm, const float *rows, float beta, int *cuts) {
    const int L = I->L, k = I->k, W = L + 1;
    int e = L;
    for (int s = k - 1; s >= 1; --s) {
        const float *prev = rows + (s - 1) * W;
        int chosen = -1;
        for (int i = s; i <= e - 1; ++i) {
            if (!ct_fits(I, i, e, perm[s])) continue;
            float c = fmax2(fmax2(prev[i], ct_gamma(I, i, perm[s - 1], perm[s])), ct_comp(I, i, e, perm[s]));
            if (c <= beta) { chosen = i; break; }
        }
        cuts[s - 1] = chosen;
        e = chosen;
    }
}

/* orderings with rank in [rank_begin, rank_end); per_ordering (may be NULL) receives beta of each */
int ppo_ct_oracle_exhaustive(const float *t, const float *m, const float *w, int L, const float *M, const float *v,
                             const float *B, int k, uint64_t rank_begin, uint64_t rank_end, float *per_ordering,
                             float *beta_out, int32_t *cuts_out, int32_t *order_out) {
    ct_t I;
    int rc = ct_open(&I, t, m, w, L, M, v, B, k);
    if (rc) return rc;
    if (rank_begin > rank_end || rank_end > ct_factorial(k)) { free(I.P); return CT_EINVAL; }
    float *rows = (float *)malloc(sizeof(float) * (size_t)k * (L + 1));
    if (!rows) { free(I.P); return CT_ENOMEM; }
    int perm[CT_MAX_K], found = 0, cuts[CT_MAX_K];
    float best = INFINITY;
    uint64_t best_rank = 0;
    ct_unrank(rank_begin, k, perm);
    for (uint64_t r = rank_begin; r < rank_end; ++r) {
        float b = ct_chain_dp(&I, perm, rows);
        if (per_ordering) per_ordering[r - rank_begin] = b;
        if (b < best) { best = b; best_rank = r; found = 1; }   /* strict: the first optimum has the lowest rank */
        ct_next_perm(perm, k);
    }
    if (found) {
        ct_unrank(best_rank, k, perm);
        ct_chain_dp(&I, perm, rows);
        ct_traceback(&I, perm, rows, best, cuts);
    }
    if (beta_out) ct_report(k, found, best, best_rank, cuts, beta_out, cuts_out, order_out);
    free(rows);
    free(I.P);
    return CT_OK;
}

/* ---------------------------------------------------------------- dynamic programme over node subsets */
/* G[S][j][i] = least bottleneck of layers [i, L) on the nodes of S, all used, j first:
 *   G[{j}][j][i] = comp(i, L, j) if it fits,
 *   G[S][j][i]   = min over fitting ends e and j2 in S \ j of max(comp(i, e, j), gamma(e; j, j2), G[S\j][j2][e]).
 * beta* = min_j G[all][j][0].  The optimal ordering of lowest rank, position by position: the smallest unused
 * node that, from some cut the prefix reaches within beta*, completes within beta*; then the cut rule from
 * the reach sets, last cut first. */
int ppo_ct_oracle_subset_dp(const float *t, const float *m, const float *w, int L, const float *M, const float *v,
                            const float *B, int k, float *beta_out, int32_t *cuts_out, int32_t *order_out) {
    ct_t I;
    int rc = ct_open(&I, t, m, w, L, M, v, B, k);
    if (rc) return rc;
    const int W = L + 1, full = (1 << k) - 1;
    float *G = (float *)malloc(sizeof(float) * ((size_t)1 << k) * k * W);
    unsigned char *reach = (unsigned char *)calloc((size_t)k * W, 1);
    if (!G || !reach) { free(G); free(reach); free(I.P); return CT_ENOMEM; }
#define GX(S, j, i) G[((size_t)(S) * k + (j)) * W + (i)]
    for (size_t x = 0; x < ((size_t)1 << k) * k * W; ++x) G[x] = INFINITY;
    for (int S = 1; S <= full; ++S) {
        int size = 0;
        for (int j = 0; j < k; ++j) size += (S >> j) & 1;
        for (int j = 0; j < k; ++j) {
            if (!((S >> j) & 1)) continue;
            for (int i = 0; i < L; ++i) {
                float best = INFINITY;
                if (size == 1) {
                    if (ct_fits(&I, i, L, j)) best = ct_comp(&I, i, L, j);
                } else {
                    for (int e = i + 1; e < L && ct_fits(&I, i, e, j); ++e) {
                        float own = ct_comp(&I, i, e, j);
                        for (int j2 = 0; j2 < k; ++j2) {
                            if (j2 == j || !((S >> j2) & 1)) continue;
                            float c = fmax2(fmax2(own, ct_gamma(&I, e, j, j2)), GX(S & ~(1 << j), j2, e));
                            if (c < best) best = c;
                        }
                    }
                }
                GX(S, j, i) = best;
            }
        }
    }
    float beta = INFINITY;
    for (int j = 0; j < k; ++j)
        if (GX(full, j, 0) < beta) beta = GX(full, j, 0);
    int seq[CT_MAX_K], cuts[CT_MAX_K], found = isfinite(beta);
    if (found) {
        /* reach[s][e]: layers [0, e) can be placed on seq[0..s-1]... with every stage <= beta (s segments) */
        int remaining = full;
        unsigned char *cur = reach;   /* reach[0]: before the first segment only e = 0 */
        cur[0] = 1;
        for (int s = 0; s < k; ++s) {
            int chosen = -1;
            for (int j = 0; j < k && chosen < 0; ++j) {
                if (!((remaining >> j) & 1)) continue;
                for (int e = 0; e < L && chosen < 0; ++e) {
                    if (!cur[e]) continue;
                    if (s > 0 && !(ct_gamma(&I, e, seq[s - 1], j) <= beta)) continue;
                    if (GX(remaining, j, e) <= beta) chosen = j;
                }
            }
            seq[s] = chosen;
            if (s + 1 < k) {
                unsigned char *nxt = reach + (size_t)(s + 1) * W;
                for (int e = 0; e < L; ++e) {
                    if (!cur[e]) continue;
                    if (s > 0 && !(ct_gamma(&I, e, seq[s - 1], chosen) <= beta)) continue;
                    for (int e2 = e + 1; e2 < L && ct_fits(&I, e, e2, chosen); ++e2)
                        if (ct_comp(&I, e, e2, chosen) <= beta) nxt[e2] = 1;
                }
                cur = nxt;
            }
            remaining &= ~(1 << chosen);
        }
        /* cuts, last first: the smallest start i of segment s reachable after s segments whose stages
         * (link into seq[s], compute of [i, e)) stay within beta */
        int e = L;
        for (int s = k - 1; s >= 1; --s) {
            const unsigned char *r = reach + (size_t)s * W;
            int chosen = -1;
            for (int i = s; i < e && chosen < 0; ++i) {
                if (!r[i] || !ct_fits(&I, i, e, seq[s])) continue;
                if (ct_gamma(&I, i, seq[s - 1], seq[s]) <= beta && ct_comp(&I, i, e, seq[s]) <= beta) chosen = i;
            }
            cuts[s - 1] = chosen;
            e = chosen;
        }
    }
    uint64_t rank = 0;
    if (found)
        for (int p = 0; p < k; ++p) {
            int smaller = 0;
            for (int q = p + 1; q < k; ++q) smaller += seq[q] < seq[p];
            rank += (uint64_t)smaller * ct_factorial(k - 1 - p);
        }
    ct_report(k, found, beta, rank, cuts, beta_out, cuts_out, order_out);
#undef GX
    free(G); free(reach); free(I.P);
    return CT_OK;
}
