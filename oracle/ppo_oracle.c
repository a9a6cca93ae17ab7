/*
 * CPU oracle for the exact partition-and-placement search.  TEST INFRASTRUCTURE ONLY:
 * nothing in the product path may call into this file; it exists so that the GPU
 * results can be compared, bit for bit, against a plain implementation written
 * from the paper's problem statement.  It shares no code with the HIP library.
 *
 * Problem (Sec. I Eq. 2, Sec. III-B Eq. 3 and the memory rule that defines the
 * vertices of the partition graph, Eq. 6 with its explanatory text):
 *   a chain of L layers, weight sizes m[i], size t[i] of the tensor leaving layer i;
 *   k nodes with capacities M[j] and a symmetric bandwidth matrix B.
 *   A solution is a permutation pi of the nodes and cuts 0=c_0<c_1<...<c_{k-1}<c_k=L;
 *   segment s = layers [c_s, c_{s+1}) runs on node pi[s].
 *   gamma_s = t[c_s-1] / B[pi[s-1]][pi[s]]  (Eq. 3),  beta = max_s gamma_s  (Eq. 2),
 *   feasible iff every segment's weight sum is within its node's capacity.
 *   beta* = min over all feasible (pi, c);  +inf if none.
 *
 * Precision, fixed for both sides of every comparison:
 *   P[0]=0, P[i+1]=P[i]+(double)m[i] sequentially in binary64;
 *   segment [i,e) fits node j iff (P[e]-P[i]) <= (double)M[j]   ("within capacity": <=);
 *   gamma is one IEEE binary32 division, round to nearest even;
 *   min and max of floats are exact.
 * Tie rules that make the answer unique:
 *   T1: among orderings reaching beta*, the one of lowest lexicographic rank;
 *   T2: among feasible cut vectors of that ordering with bottleneck beta*, the one that
 *       minimises c_{k-1}, then c_{k-2}, ..., then c_1.
 *
 * Three independent routes to the same answer live here:
 *   ppo_oracle_bruteforce   every (cut vector, permutation) pair, straight from the definition;
 *   ppo_oracle_exhaustive   for every permutation in lexicographic order, a plain windowed
 *                           min-max chain-partition DP (division and memory test inside the loop);
 *   ppo_oracle_subset_dp    a dynamic programme over node subsets (exponential, not factorial),
 *                           with boolean reachability for the tie rules.
 * Pins (tests/test_oracle_*.py): the paper's worked example 10.2 Mbit / 6 Mbps (Sec. I),
 * closed forms for k=1, k=2 and the unconstrained constant-bandwidth case, Theorem 1 as a
 * lower bound on the output, monotonicity, exact power-of-two scaling, relabelling of nodes,
 * and agreement of the three routes on thousands of small instances with forced ties.
 * Parity unpinned: nothing in this file (the paper's own heuristic results, Sec. IV-V, are
 * outside its scope).
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_ETOOBIG (-2)
#define ORC_EDATA (-3)   /* precondition on the data violated */
#define ORC_ENOMEM (-4)

#define ORC_MAX_K 12
#define ORC_MAX_L 4096

typedef struct {
    const float *t, *m, *M, *B;
    int L, k;
    double *P; /* L+1 prefix sums */
} inst_t;

static int check_scalars(int L, int k) {
    if (L < 1 || k < 1 || k > L) return ORC_EINVAL;
    if (k > ORC_MAX_K || L > ORC_MAX_L) return ORC_ETOOBIG;
    return ORC_OK;
}

/* Data preconditions: finite, t >= 0 (a zero of either sign is a size of zero), m,M >= 0, off-diagonal
 * B > 0 and bit-symmetric. */
int ppo_oracle_check_inputs(const float *t, const float *m, int L, const float *M, const float *B, int k,
                            int n_inst) {
    int rc = check_scalars(L, k);
    if (rc) return rc;
    if (n_inst < 0 || (n_inst > 0 && (!t || !m || !M || !B))) return ORC_EINVAL;
    for (int n = 0; n < n_inst; ++n) {
        for (int i = 0; i < L; ++i) {
            float a = t[(size_t)n * L + i], b = m[(size_t)n * L + i];
            if (!isfinite(a) || !isfinite(b) || a < 0.0f || b < 0.0f) return ORC_EDATA;
        }
        for (int j = 0; j < k; ++j) {
            float c = M[(size_t)n * k + j];
            if (!isfinite(c) || c < 0.0f) return ORC_EDATA;
        }
        const float *Bn = B + (size_t)n * k * k;
        for (int a = 0; a < k; ++a)
            for (int b = 0; b < k; ++b) {
                if (a == b) continue;
                float x = Bn[a * k + b], y = Bn[b * k + a];
                if (!isfinite(x) || !(x > 0.0f)) return ORC_EDATA;
                if (memcmp(&x, &y, sizeof x) != 0) return ORC_EDATA;
            }
    }
    return ORC_OK;
}

static void prefix_sums(const float *m, int L, double *P) {
    P[0] = 0.0;
    for (int i = 0; i < L; ++i) P[i + 1] = P[i] + (double)m[i];
}

static int fits(const inst_t *I, int i, int e, int node) { return (I->P[e] - I->P[i]) <= (double)I->M[node]; }

static float gamma_of(const inst_t *I, int cut, int a, int b) {
    /* Eq. 3: the tensor leaving the last layer before the cut, over the link between the two hosts */
    volatile float q = I->t[cut - 1] / I->B[a * I->k + b];
    if (q == 0.0f) return 0.0f; /* nothing to send takes no time: +0, also when t carries a sign bit */
    return q;
}

static uint64_t factorial(int n) {
    uint64_t f = 1;
    for (int i = 2; i <= n; ++i) f *= (uint64_t)i;
    return f;
}

/* Lexicographic rank of a permutation of 0..k-1: the number of permutations that sort before it. */
uint64_t ppo_oracle_rank(const int32_t *perm, int k) {
    uint64_t r = 0;
    for (int p = 0; p < k; ++p) {
        int smaller = 0;
        for (int q = p + 1; q < k; ++q)
            if (perm[q] < perm[p]) ++smaller;
        r += (uint64_t)smaller * factorial(k - 1 - p);
    }
    return r;
}

/* The permutation with the given lexicographic rank. */
void ppo_oracle_unrank(uint64_t rank, int k, int32_t *perm) {
    int avail[ORC_MAX_K + 4];
    for (int j = 0; j < k; ++j) avail[j] = j;
    int n = k;
    for (int p = 0; p < k; ++p) {
        uint64_t f = factorial(k - 1 - p);
        int d = (int)(rank / f);
        rank -= (uint64_t)d * f;
        perm[p] = avail[d];
        for (int j = d; j + 1 < n; ++j) avail[j] = avail[j + 1];
        --n;
    }
}

/* Step to the next permutation in lexicographic order; returns 0 after the last one. */
static int next_perm(int *a, int n) {
    int i = n - 2;
    while (i >= 0 && a[i] > a[i + 1]) --i;
    if (i < 0) return 0;
    int j = n - 1;
    while (a[j] < a[i]) --j;
    int tmp = a[i]; a[i] = a[j]; a[j] = tmp;
    for (int l = i + 1, r = n - 1; l < r; ++l, --r) { tmp = a[l]; a[l] = a[r]; a[r] = tmp; }
    return 1;
}

/* Definition of beta for one explicit solution (Eq. 2, Eq. 3, memory rule). cuts has k-1 entries. */
int ppo_oracle_evaluate(const float *t, const float *m, int L, const float *M, const float *B, int k,
                        const int32_t *order, const int32_t *cuts, float *beta, int32_t *feasible) {
    int rc = ppo_oracle_check_inputs(t, m, L, M, B, k, 1);
    if (rc) return rc;
    double *P = (double *)malloc(sizeof(double) * (L + 1));
    if (!P) return ORC_ENOMEM;
    prefix_sums(m, L, P);
    inst_t I = {t, m, M, B, L, k, P};
    int ok = 1, seen[ORC_MAX_K] = {0};
    for (int s = 0; s < k; ++s) {
        if (order[s] < 0 || order[s] >= k || seen[order[s]]) ok = 0; else seen[order[s]] = 1;
    }
    float b = 0.0f;
    int prev = 0;
    for (int s = 0; ok && s < k; ++s) {
        int end = (s == k - 1) ? L : cuts[s];
        if (end <= prev || end > L) { ok = 0; break; }
        if (!fits(&I, prev, end, order[s])) ok = 0;
        if (s > 0) {
            float g = gamma_of(&I, prev, order[s - 1], order[s]);
            if (g > b) b = g;
        }
        prev = end;
    }
    *feasible = ok;
    *beta = ok ? b : INFINITY;
    free(P);
    return ORC_OK;
}

/* ---------------------------------------------------------------- brute force (tiny inputs) */

typedef struct {
    float beta;
    uint64_t rank;
    int cuts[ORC_MAX_K];
    int found;
} best_t;

/* is cut vector a (k-1 entries) before b when compared c_{k-1} first, then c_{k-2}, ... (rule T2) */
static int cuts_rev_less(const int *a, const int *b, int k) {
    for (int s = k - 2; s >= 0; --s) {
        if (a[s] != b[s]) return a[s] < b[s];
    }
    return 0;
}

int ppo_oracle_bruteforce(const float *t, const float *m, int L, const float *M, const float *B, int k,
                          float *beta_out, int32_t *cuts_out, int32_t *order_out) {
    int rc = ppo_oracle_check_inputs(t, m, L, M, B, k, 1);
    if (rc) return rc;
    double *P = (double *)malloc(sizeof(double) * (L + 1));
    if (!P) return ORC_ENOMEM;
    prefix_sums(m, L, P);
    inst_t I = {t, m, M, B, L, k, P};
    best_t best; best.beta = INFINITY; best.rank = 0; best.found = 0;
    int perm[ORC_MAX_K], c[ORC_MAX_K + 1];
    for (int j = 0; j < k; ++j) perm[j] = j;
    uint64_t rank = 0;
    do {
        /* all strictly increasing cut vectors c_1..c_{k-1} in 1..L-1 */
        for (int s = 1; s < k; ++s) c[s] = s;
        c[0] = 0; c[k] = L;
        for (;;) {
            int ok = 1;
            float b = 0.0f;
            for (int s = 0; s < k; ++s) {
                if (!fits(&I, c[s], c[s + 1], perm[s])) { ok = 0; break; }
                if (s > 0) {
                    float g = gamma_of(&I, c[s], perm[s - 1], perm[s]);
                    if (g > b) b = g;
                }
            }
            if (ok) {
                int better = 0;
                if (!best.found || b < best.beta) better = 1;
                else if (b == best.beta) {
                    if (rank < best.rank) better = 1;
                    else if (rank == best.rank && cuts_rev_less(c + 1, best.cuts, k)) better = 1;
                }
                if (better) {
                    best.found = 1; best.beta = b; best.rank = rank;
                    for (int s = 1; s < k; ++s) best.cuts[s - 1] = c[s];
                }
            }
            /* next combination */
            int s = k - 1;
            while (s >= 1 && c[s] == L - (k - s)) --s;
            if (s < 1) break;
            ++c[s];
            for (int u = s + 1; u < k; ++u) c[u] = c[u - 1] + 1;
        }
        ++rank;
    } while (next_perm(perm, k));
    if (best.found) {
        *beta_out = best.beta;
        int32_t p[ORC_MAX_K];
        ppo_oracle_unrank(best.rank, k, p);
        for (int s = 0; s < k; ++s) order_out[s] = p[s];
        for (int s = 0; s + 1 < k; ++s) cuts_out[s] = best.cuts[s];
    } else {
        *beta_out = INFINITY;
        for (int s = 0; s < k; ++s) order_out[s] = -1;
        for (int s = 0; s + 1 < k; ++s) cuts_out[s] = -1;
    }
    free(P);
    return ORC_OK;
}

/* ---------------------------------------------------------------- per-ordering chain DP */

/* D_s[e] = least bottleneck of putting layers [0,e) on nodes perm[0..s], one non-empty segment each.
 * rows: k*(L+1) floats (row s at rows + s*(L+1)); entries outside s+1 <= e <= L-(k-1-s) are +inf.
 * cand, if given, is increased by the number of (i -> e) candidates examined in rows 1..k-1. */
static float chain_dp(const inst_t *I, const int *perm, float *rows, uint64_t *cand) {
    const int L = I->L, k = I->k, W = L + 1;
    for (int s = 0; s < k; ++s)
        for (int e = 0; e <= L; ++e) rows[s * W + e] = INFINITY;
    for (int e = 1; e <= L - (k - 1); ++e)
        if (fits(I, 0, e, perm[0])) rows[e] = 0.0f;
    uint64_t n = 0;
    for (int s = 1; s < k; ++s) {
        const float *prev = rows + (s - 1) * W;
        float *cur = rows + s * W;
        for (int e = s + 1; e <= L - (k - 1 - s); ++e) {
            float best = INFINITY;
            for (int i = e - 1; i >= s; --i) {
                /* P[e]-P[i] grows as i falls, so the legal starts form one run ending at e-1 */
                if (!fits(I, i, e, perm[s])) break;
                ++n;
                float g = gamma_of(I, i, perm[s - 1], perm[s]);
                float c = prev[i] > g ? prev[i] : g;
                if (c < best) best = c;
            }
            cur[e] = best;
        }
    }
    if (cand) *cand += n;
    return rows[(k - 1) * W + L];
}

/* Rule T2 on the stored rows of the winning ordering. */
static void traceback(const inst_t *I, const int *perm, const float *rows, float beta, int32_t *cuts) {
    const int L = I->L, k = I->k, W = L + 1;
    int e = L;
    for (int s = k - 1; s >= 1; --s) {
        const float *prev = rows + (s - 1) * W;
        int chosen = -1;
        for (int i = s; i <= e - 1; ++i) {
            if (!fits(I, i, e, perm[s])) continue;
            float g = gamma_of(I, i, perm[s - 1], perm[s]);
            float c = prev[i] > g ? prev[i] : g;
            if (c <= beta) { chosen = i; break; }
        }
        cuts[s - 1] = chosen;
        e = chosen;
    }
}

typedef struct {
    /* inputs */
    const float *t, *m, *M, *B;
    int L, k, n_inst;
    int mode;             /* 0: exhaustive solve, 1: per-ordering export, 2: subset DP */
    uint64_t rank_begin, rank_end, chunk;
    float *per_ordering;  /* mode 1 */
    /* shared work counter */
    pthread_mutex_t mu;
    uint64_t next_task, n_tasks, tasks_per_inst;
    /* results */
    float *best_beta;     /* [n_inst] */
    uint64_t *best_rank;  /* [n_inst] */
    uint64_t cand_total;
    int error;
    float *beta_out; int32_t *cuts_out, *order_out; /* mode 2 */
} job_t;

static int subset_dp_one(const inst_t *I, float *beta_out, int32_t *cuts_out, int32_t *order_out);

static void *worker(void *arg) {
    job_t *J = (job_t *)arg;
    const int L = J->L, k = J->k;
    double *P = (double *)malloc(sizeof(double) * (L + 1));
    float *rows = (float *)malloc(sizeof(float) * (size_t)k * (L + 1));
    if (!P || !rows) { J->error = ORC_ENOMEM; free(P); free(rows); return NULL; }
    for (;;) {
        pthread_mutex_lock(&J->mu);
        uint64_t task = J->next_task++;
        pthread_mutex_unlock(&J->mu);
        if (task >= J->n_tasks) break;
        int inst = (int)(task / J->tasks_per_inst);
        inst_t I = {J->t + (size_t)inst * L, J->m + (size_t)inst * L, J->M + (size_t)inst * k,
                    J->B + (size_t)inst * k * k, L, k, P};
        prefix_sums(I.m, L, P);
        if (J->mode == 2) {
            int rc = subset_dp_one(&I, J->beta_out + inst, J->cuts_out + (size_t)inst * (k > 1 ? k - 1 : 0),
                                   J->order_out + (size_t)inst * k);
            if (rc) J->error = rc;
            continue;
        }
        uint64_t r0 = J->rank_begin + (task % J->tasks_per_inst) * J->chunk;
        uint64_t r1 = r0 + J->chunk < J->rank_end ? r0 + J->chunk : J->rank_end;
        int32_t p32[ORC_MAX_K];
        int perm[ORC_MAX_K];
        ppo_oracle_unrank(r0, k, p32);
        for (int j = 0; j < k; ++j) perm[j] = p32[j];
        float lb = INFINITY; uint64_t lr = 0; int have = 0;
        uint64_t cand = 0;
        for (uint64_t r = r0; r < r1; ++r) {
            float b = chain_dp(&I, perm, rows, &cand);
            if (J->mode == 1) J->per_ordering[r - J->rank_begin] = b;
            if (!have || b < lb) { lb = b; lr = r; have = 1; }   /* strict <: the first optimum stays */
            next_perm(perm, k);
        }
        pthread_mutex_lock(&J->mu);
        J->cand_total += cand;
        if (have && J->best_beta) {
            if (lb < J->best_beta[inst] || (lb == J->best_beta[inst] && lr < J->best_rank[inst])) {
                J->best_beta[inst] = lb; J->best_rank[inst] = lr;
            }
        }
        pthread_mutex_unlock(&J->mu);
    }
    free(P); free(rows);
    return NULL;
}

static int run_job(job_t *J, int n_threads) {
    if (n_threads < 1) n_threads = 1;
    if (n_threads > 256) n_threads = 256;
    pthread_mutex_init(&J->mu, NULL);
    J->next_task = 0; J->cand_total = 0; J->error = 0;
    pthread_t th[256];
    int started = 0;
    for (int i = 0; i < n_threads; ++i)
        if (pthread_create(&th[started], NULL, worker, J) == 0) ++started;
    if (started == 0) worker(J);
    for (int i = 0; i < started; ++i) pthread_join(th[i], NULL);
    pthread_mutex_destroy(&J->mu);
    return J->error;
}

/* Exhaustive oracle over the rank range [rank_begin, rank_end) of every instance (whole range:
 * 0, k!).  cand_out (may be NULL) receives the total number of DP candidates examined. */
int ppo_oracle_exhaustive_range(const float *t, const float *m, int L, const float *M, const float *B, int k,
                                int n_inst, uint64_t rank_begin, uint64_t rank_end, float *beta_out,
                                int32_t *cuts_out, int32_t *order_out, int n_threads, uint64_t *cand_out) {
    int rc = ppo_oracle_check_inputs(t, m, L, M, B, k, n_inst);
    if (rc) return rc;
    if (rank_end > factorial(k) || rank_begin > rank_end) return ORC_EINVAL;
    if (n_inst == 0) { if (cand_out) *cand_out = 0; return ORC_OK; }
    job_t J; memset(&J, 0, sizeof J);
    J.t = t; J.m = m; J.M = M; J.B = B; J.L = L; J.k = k; J.n_inst = n_inst; J.mode = 0;
    J.rank_begin = rank_begin; J.rank_end = rank_end;
    uint64_t span = rank_end - rank_begin;
    J.chunk = span / 64 + 1;
    if (J.chunk > 20000) J.chunk = 20000;
    J.tasks_per_inst = span ? (span + J.chunk - 1) / J.chunk : 0;
    J.n_tasks = J.tasks_per_inst * (uint64_t)n_inst;
    J.best_beta = (float *)malloc(sizeof(float) * n_inst);
    J.best_rank = (uint64_t *)malloc(sizeof(uint64_t) * n_inst);
    if (!J.best_beta || !J.best_rank) { free(J.best_beta); free(J.best_rank); return ORC_ENOMEM; }
    for (int n = 0; n < n_inst; ++n) { J.best_beta[n] = INFINITY; J.best_rank[n] = UINT64_MAX; }
    rc = run_job(&J, n_threads);
    if (!rc) {
        double *P = (double *)malloc(sizeof(double) * (L + 1));
        float *rows = (float *)malloc(sizeof(float) * (size_t)k * (L + 1));
        if (!P || !rows) rc = ORC_ENOMEM;
        for (int n = 0; !rc && n < n_inst; ++n) {
            int32_t *ord = order_out + (size_t)n * k, *cu = cuts_out + (size_t)n * (k - 1);
            beta_out[n] = J.best_beta[n];
            if (isinf(J.best_beta[n])) {
                for (int s = 0; s < k; ++s) ord[s] = -1;
                for (int s = 0; s + 1 < k; ++s) cu[s] = -1;
                continue;
            }
            inst_t I = {t + (size_t)n * L, m + (size_t)n * L, M + (size_t)n * k, B + (size_t)n * k * k, L, k, P};
            prefix_sums(I.m, L, P);
            int perm[ORC_MAX_K];
            ppo_oracle_unrank(J.best_rank[n], k, ord);
            for (int s = 0; s < k; ++s) perm[s] = ord[s];
            chain_dp(&I, perm, rows, NULL);
            traceback(&I, perm, rows, J.best_beta[n], cu);
        }
        free(P); free(rows);
    }
    if (cand_out) *cand_out = J.cand_total;
    free(J.best_beta); free(J.best_rank);
    return rc;
}

int ppo_oracle_exhaustive(const float *t, const float *m, int L, const float *M, const float *B, int k,
                          int n_inst, float *beta_out, int32_t *cuts_out, int32_t *order_out, int n_threads,
                          uint64_t *cand_out) {
    int rc = check_scalars(L, k);
    if (rc) return rc;
    return ppo_oracle_exhaustive_range(t, m, L, M, B, k, n_inst, 0, factorial(k), beta_out, cuts_out, order_out,
                                       n_threads, cand_out);
}

/* beta of each ordering with rank in [rank_begin, rank_end) for ONE instance. */
int ppo_oracle_eval_orderings(const float *t, const float *m, int L, const float *M, const float *B, int k,
                              uint64_t rank_begin, uint64_t rank_end, float *beta_per_ordering, int n_threads,
                              uint64_t *cand_out) {
    int rc = ppo_oracle_check_inputs(t, m, L, M, B, k, 1);
    if (rc) return rc;
    if (rank_end > factorial(k) || rank_begin > rank_end) return ORC_EINVAL;
    job_t J; memset(&J, 0, sizeof J);
    J.t = t; J.m = m; J.M = M; J.B = B; J.L = L; J.k = k; J.n_inst = 1; J.mode = 1;
    J.rank_begin = rank_begin; J.rank_end = rank_end;
    uint64_t span = rank_end - rank_begin;
    J.chunk = span / 64 + 1;
    if (J.chunk > 20000) J.chunk = 20000;
    J.tasks_per_inst = span ? (span + J.chunk - 1) / J.chunk : 0;
    J.n_tasks = J.tasks_per_inst;
    J.per_ordering = beta_per_ordering;
    rc = run_job(&J, n_threads);
    if (cand_out) *cand_out = J.cand_total;
    return rc;
}

/* ---------------------------------------------------------------- subset dynamic programme */

/* G[S][j][i]: least bottleneck of running layers [i,L) on exactly the node set S, one non-empty
 * segment per node, with node j (in S) hosting the segment that starts at i. */
static int subset_dp_one(const inst_t *I, float *beta_out, int32_t *cuts_out, int32_t *order_out) {
    const int L = I->L, k = I->k, W = L + 1;
    const size_t nS = (size_t)1 << k;
    float *G = (float *)malloc(sizeof(float) * nS * k * W);
    if (!G) return ORC_ENOMEM;
#define GX(S, j, i) G[((size_t)(S) * k + (j)) * W + (i)]
    for (size_t x = 0; x < nS * k * W; ++x) G[x] = INFINITY;
    /* subsets in increasing numeric order: every proper subset comes before its supersets */
    for (size_t S = 1; S < nS; ++S) {
        int size = __builtin_popcountll(S);
        for (int j = 0; j < k; ++j) {
            if (!(S >> j & 1)) continue;
            size_t rest = S & ~((size_t)1 << j);
            for (int i = 0; i + size <= L; ++i) {
                float best = INFINITY;
                if (size == 1) {
                    if (fits(I, i, L, j)) best = 0.0f;
                } else {
                    for (int e = i + 1; e + (size - 1) <= L; ++e) {
                        if (!fits(I, i, e, j)) break;
                        for (int j2 = 0; j2 < k; ++j2) {
                            if (!(rest >> j2 & 1)) continue;
                            float g = gamma_of(I, e, j, j2);
                            float tail = GX(rest, j2, e);
                            float c = tail > g ? tail : g;
                            if (c < best) best = c;
                        }
                    }
                }
                GX(S, j, i) = best;
            }
        }
    }
    const size_t all = nS - 1;
    float beta = INFINITY;
    for (int j = 0; j < k; ++j)
        if (GX(all, j, 0) < beta) beta = GX(all, j, 0);
    *beta_out = beta;
    if (isinf(beta)) {
        for (int s = 0; s < k; ++s) order_out[s] = -1;
        for (int s = 0; s + 1 < k; ++s) cuts_out[s] = -1;
        free(G);
        return ORC_OK;
    }
    /* Rule T1: fix positions left to right, always the smallest node that still admits a completion
     * with bottleneck <= beta.  reach[s][e] = 1 iff layers [0,e) can be put on order[0..s] with every
     * segment fitting and every gamma <= beta. */
    unsigned char *reach = (unsigned char *)calloc((size_t)k * W, 1);
    if (!reach) { free(G); return ORC_ENOMEM; }
    size_t remaining = all;
    for (int s = 0; s < k; ++s) {
        int pick = -1;
        for (int j = 0; j < k && pick < 0; ++j) {
            if (!(remaining >> j & 1)) continue;
            if (s == 0) {
                if (GX(remaining, j, 0) <= beta) pick = j;
            } else {
                for (int e = s; e < L && pick < 0; ++e) {
                    if (!reach[(s - 1) * W + e]) continue;
                    if (gamma_of(I, e, order_out[s - 1], j) <= beta && GX(remaining, j, e) <= beta) pick = j;
                }
            }
        }
        order_out[s] = pick;
        remaining &= ~((size_t)1 << pick);
        for (int e = s + 1; e <= L; ++e) {
            int r = 0;
            if (s == 0) r = fits(I, 0, e, pick);
            else
                for (int i = s; i < e && !r; ++i)
                    r = reach[(s - 1) * W + i] && fits(I, i, e, pick) &&
                        gamma_of(I, i, order_out[s - 1], pick) <= beta;
            reach[s * W + e] = (unsigned char)r;
        }
    }
    /* Rule T2 from the reachability table */
    int e = L;
    for (int s = k - 1; s >= 1; --s) {
        int chosen = -1;
        for (int i = s; i < e && chosen < 0; ++i)
            if (reach[(s - 1) * W + i] && fits(I, i, e, order_out[s]) &&
                gamma_of(I, i, order_out[s - 1], order_out[s]) <= beta)
                chosen = i;
        cuts_out[s - 1] = chosen;
        e = chosen;
    }
    free(reach);
    free(G);
#undef GX
    return ORC_OK;
}

int ppo_oracle_subset_dp(const float *t, const float *m, int L, const float *M, const float *B, int k, int n_inst,
                         float *beta_out, int32_t *cuts_out, int32_t *order_out, int n_threads) {
    int rc = ppo_oracle_check_inputs(t, m, L, M, B, k, n_inst);
    if (rc) return rc;
    if (n_inst == 0) return ORC_OK;
    job_t J; memset(&J, 0, sizeof J);
    J.t = t; J.m = m; J.M = M; J.B = B; J.L = L; J.k = k; J.n_inst = n_inst; J.mode = 2;
    J.tasks_per_inst = 1; J.n_tasks = (uint64_t)n_inst;
    J.beta_out = beta_out; J.cuts_out = cuts_out; J.order_out = order_out;
    return run_job(&J, n_threads);
}
