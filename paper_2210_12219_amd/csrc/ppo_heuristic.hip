// The paper's own placement algorithm and its two comparison systems, for scoring against the exact optimum.
//
// Sec. III-B2: the cuts come from the partitioning step (Alg. 1, ppo_partition.hip); their transfer sizes are
// sorted into classes (Eq. 5); classes are matched from the highest down, within a class the runs of consecutive
// cuts from the longest down (Alg. 3); a run of r cuts gets a path of r + 1 nodes of the communication graph
// whose weakest link is as strong as possible: bisection over the descending list of bandwidths for the highest
// threshold at which the graph of links at or above it (Eq. 8) still holds such a path between the ends that
// neighbouring runs have fixed (Alg. 2).  Sec. IV: the random and the greedy joint-optimisation systems.
//
// Readings (the paper leaves them open): classes are bins of equal width between the least and the greatest
// transfer size of the chain's candidate cuts; the path search, colour coding in the paper, is a depth-first
// search in increasing node order that returns the smallest sequence and gives up after kPathBudget nodes put on
// the path; if a run cannot be matched, the matching is tried again with one class fewer.
//
// One wave per instance.  The searches are sequential by nature and run on lane 0, on 64-bit node masks; the
// lanes share the sort of the bandwidth list and the adjacency masks of a threshold.  Not a tuned path.
#include "ppo_common.h"

namespace ppo {

constexpr int kHeurMaxN = PPO_HEURISTIC_MAX_N;
constexpr int kHeurMaxEdges = kHeurMaxN * (kHeurMaxN - 1) / 2;
constexpr uint32_t kPathBudget = 20000u;

struct HeurShared {
    float bw[kHeurMaxEdges];            // bandwidths of all node pairs, descending
    uint16_t pair_ab[kHeurMaxEdges];    // a | b << 8 of the pair at that place
    float thr[kHeurMaxEdges];           // the distinct bandwidths among the nodes of the current search, descending
    unsigned long long adj[kHeurMaxN];  // links at or above the current threshold
    float size[PPO_MAX_L];              // transfer size of every cut
    int cls[PPO_MAX_L];                 // its class
    int node[PPO_MAX_L + 1];            // N: node of every segment, -1 while open
    int run_first[PPO_MAX_L], run_len[PPO_MAX_L];
    int path[kHeurMaxN + 1], nxt[kHeurMaxN + 1], best[kHeurMaxN + 1];
    int n_thr, found;
};

__device__ inline float heur_gamma(float tv, float bw) {
    const float q = __fdiv_rn(tv, bw);
    return q == 0.0f ? 0.0f : q;
}

// Depth-first search for the smallest sequence of k distinct nodes: first `start` and last `end` where given
// (>= 0), every other one from `avail`, consecutive ones linked in adj.  Lane 0 only.  Returns whether found.
__device__ bool heur_k_path(HeurShared& S, int n, unsigned long long avail, int k, int start, int end) {
    uint32_t budget = kPathBudget;
    int len = 0;
    unsigned long long inpath = 0ull;
    S.nxt[0] = 0;
    for (;;) {
        if (len == k) return true;
        unsigned long long cand;
        const bool at_start = len == 0 && start >= 0, at_end = len == k - 1 && end >= 0;
        if (at_start || at_end) {
            cand = ~0ull;
            if (at_start) cand &= 1ull << start;
            if (at_end) cand &= 1ull << end;
        } else {
            cand = avail;
        }
        cand &= ~inpath;
        if (len > 0) cand &= S.adj[S.path[len - 1]];
        const int from = S.nxt[len];
        cand = from >= 64 ? 0ull : cand & (~0ull << from);
        if (n < 64) cand &= (1ull << n) - 1ull;
        if (cand) {
            if (budget == 0u) return false;
            --budget;
            const int v = __ffsll((long long)cand) - 1;
            S.nxt[len] = v + 1;
            S.path[len] = v;
            inpath |= 1ull << v;
            ++len;
            S.nxt[len] = 0;
        } else {
            if (len == 0) return false;
            --len;
            inpath &= ~(1ull << S.path[len]);
        }
    }
}

// Alg. 2 for one run.  All lanes take part (the adjacency masks of a threshold are built by the lanes); the result
// (S.found, S.best[0..k)) is lane 0's.
__device__ void heur_subgraph_k_path(HeurShared& S, const float* __restrict__ B, int n, int n_edges,
                                     unsigned long long avail, int k, int start, int end, int lane) {
    unsigned long long elig = avail;
    if (start >= 0) elig |= 1ull << start;
    if (end >= 0) elig |= 1ull << end;
    if (lane == 0) {
        // the distinct bandwidths among the eligible nodes, in descending order
        int cnt = 0;
        for (int i = 0; i < n_edges; ++i) {
            const int a = S.pair_ab[i] & 0xFF, b = S.pair_ab[i] >> 8;
            if (((elig >> a) & 1ull) && ((elig >> b) & 1ull) && (cnt == 0 || S.thr[cnt - 1] != S.bw[i])) S.thr[cnt++] = S.bw[i];
        }
        S.n_thr = cnt;
        S.found = 0;
    }
    __syncthreads();
    if (k == 1) {
        if (lane == 0) {
            for (int v = 0; v < n; ++v) S.adj[v] = 0ull;
            if (heur_k_path(S, n, avail, 1, start, end)) {
                S.found = 1;
                S.best[0] = S.path[0];
            }
        }
        __syncthreads();
        return;
    }
    int low = 0, high = S.n_thr;
    while (low < high) {
        const int median = (low + high) / 2;
        const float thr = S.thr[median];
        for (int a = lane; a < n; a += 64) {
            unsigned long long mask = 0ull;
            for (int b = 0; b < n; ++b)
                if (b != a && B[a * n + b] >= thr) mask |= 1ull << b;
            S.adj[a] = mask;
        }
        __syncthreads();
        int ok = 0;
        if (lane == 0) {
            ok = heur_k_path(S, n, avail, k, start, end) ? 1 : 0;
            if (ok) {
                S.found = 1;
                for (int i = 0; i < k; ++i) S.best[i] = S.path[i];
            }
        }
        ok = __shfl(ok, 0, 64);
        __syncthreads();
        if (ok) high = median; else low = median + 1;
    }
}

// mode 0: the paper's algorithm (cuts given); 1: joint-optimisation system; 2: random system (draws given)
__global__ __launch_bounds__(64) void heuristic_kernel(const float* __restrict__ t, const float* __restrict__ m, int L,
                                                       const float* __restrict__ kappa, const float* __restrict__ Ball,
                                                       int n, int n_classes, int mode, const float* __restrict__ draws,
                                                       int n_draws, const int32_t* segs_in, const int32_t* cuts_in,
                                                       float* __restrict__ beta_out, int32_t* segs_out, int32_t* cuts_out,
                                                       int32_t* __restrict__ order_out, int32_t* __restrict__ classes_out) {
    // segs_in / cuts_in may be segs_out / cuts_out themselves (the partitioning step wrote them there)
    __shared__ HeurShared S;
    __shared__ double P[PPO_MAX_L + 1];
    __shared__ int cut_s[PPO_MAX_L];
    __shared__ int p_s;
    const int inst = blockIdx.x, lane = threadIdx.x;
    const float* ti = t + (size_t)inst * L;
    const float* B = Ball + (size_t)inst * n * n;
    int32_t* cuts_o = cuts_out + (size_t)inst * (L > 1 ? L - 1 : 0);
    int32_t* order_o = order_out + (size_t)inst * n;
    const float inf = __uint_as_float(kInfBits);
    // the cuts of the partitioning step may arrive in the output arrays themselves: read them before clearing
    if (mode == 0 && lane == 0) {
        p_s = segs_in[inst];
        for (int i = 0; i + 1 < p_s; ++i) cut_s[i] = cuts_in[(size_t)inst * (L - 1) + i];
    }
    __syncthreads();
    for (int i = lane; i < L - 1; i += 64) cuts_o[i] = -1;
    for (int i = lane; i < n; i += 64) order_o[i] = -1;
    __syncthreads();
    auto fail = [&]() {
        if (lane == 0) {
            beta_out[inst] = inf;
            segs_out[inst] = 0;
            if (classes_out) classes_out[inst] = 0;
        }
    };
    // ---- the cuts
    if (mode != 0) {
        if (lane == 0) {
            const float* mi = m + (size_t)inst * L;
            const double cap = (double)kappa[inst];
            double acc = 0.0;
            P[0] = 0.0;
            for (int i = 0; i < L; ++i) {
                acc = acc + (double)mi[i];
                P[i + 1] = acc;
            }
            int p = 0, i = 0, d = 0;
            unsigned long long free_nodes = n < 64 ? (1ull << n) - 1ull : ~0ull;
            bool ok = true;
            while (i < L && ok) {
                int last = i;   // the last end that fits
                while (last < L && (P[last + 1] - P[i]) <= cap) ++last;
                if (last == i) { ok = false; break; }
                int e;
                if (mode == 1) {
                    // the fitting end with the smallest transfer size; the rest of the chain as soon as it fits
                    e = last;
                    if (last < L) {
                        e = i + 1;
                        for (int x = i + 2; x <= last; ++x)
                            if (ti[x - 1] < ti[e - 1]) e = x;
                    }
                } else {
                    // a random free node, then a random fitting end
                    const int nfree = __popcll(free_nodes);
                    if (nfree == 0 || d + 1 >= n_draws) { ok = false; break; }
                    int pick = (int)((double)draws[(size_t)inst * n_draws + d] * (double)nfree);
                    unsigned long long f = free_nodes;
                    for (int s = 0; s < pick; ++s) f &= f - 1ull;
                    const int node = __ffsll((long long)f) - 1;
                    free_nodes &= ~(1ull << node);
                    S.node[p] = node;
                    e = i + 1 + (int)((double)draws[(size_t)inst * n_draws + d + 1] * (double)(last - i));
                    d += 2;
                }
                if (e < L) cut_s[p] = e;
                ++p;
                i = e;
            }
            p_s = ok ? p : 0;
        }
    }
    __syncthreads();
    const int p = p_s;
    if (p == 0 || p > n) { fail(); return; }
    if (mode == 0 || mode == 1) {
        // bandwidths of all pairs in descending order (ties by pair index): rank sort over the lanes
        const int n_edges = n * (n - 1) / 2;
        for (int e = lane; e < n_edges; e += 64) {
            int a = 0, rem = e;
            while (rem >= n - 1 - a) { rem -= n - 1 - a; ++a; }
            const int b = a + 1 + rem;
            const float x = B[a * n + b];
            int rank = 0, e2 = 0;
            for (int a2 = 0; a2 < n; ++a2)
                for (int b2 = a2 + 1; b2 < n; ++b2, ++e2) {
                    const float y = B[a2 * n + b2];
                    rank += (y > x || (y == x && e2 < e)) ? 1 : 0;
                }
            S.bw[rank] = x;
            S.pair_ab[rank] = (uint16_t)(a | (b << 8));
        }
        __syncthreads();
        if (mode == 0) {
            // ---- Eq. 5 classes, then Alg. 3, with fewer classes if a run cannot be matched
            if (lane == 0) {
                float lo = L > 1 ? ti[0] : 0.0f, hi = lo;
                for (int i = 1; i < L - 1; ++i) {
                    lo = ti[i] < lo ? ti[i] : lo;
                    hi = ti[i] > hi ? ti[i] : hi;
                }
                for (int i = 0; i + 1 < p; ++i) S.size[i] = ti[cut_s[i] - 1];
                S.size[PPO_MAX_L - 1] = lo;   // kept for the class loop below
                S.thr[0] = hi;
            }
            __syncthreads();
            const float lo = S.size[PPO_MAX_L - 1], hi = S.thr[0];
            __syncthreads();
            int used = 0;
            for (int nc = n_classes; nc >= 1 && !used; --nc) {
                if (lane == 0) {
                    for (int i = 0; i + 1 < p; ++i) {
                        int c = nc - 1;
                        if (hi != lo) {
                            const double f = floor(((double)S.size[i] - (double)lo) / ((double)hi - (double)lo) * (double)nc);
                            c = f < (double)(nc - 1) ? (int)f : nc - 1;
                        }
                        S.cls[i] = c;
                    }
                    for (int i = 0; i < p; ++i) S.node[i] = -1;
                }
                __syncthreads();
                unsigned long long avail = n < 64 ? (1ull << n) - 1ull : ~0ull;
                bool ok = true;
                if (p == 1) {
                    if (lane == 0) S.node[0] = 0;
                } else {
                    for (int X = nc - 1; X >= 0 && ok; --X) {
                        // runs of class X, longest first, then by position
                        int n_runs = 0;
                        if (lane == 0) {
                            for (int i = 0; i + 1 < p;) {
                                if (S.cls[i] != X) { ++i; continue; }
                                int j = i;
                                while (j + 1 < p && S.cls[j] == X) ++j;
                                S.run_first[n_runs] = i;
                                S.run_len[n_runs] = j - i;
                                ++n_runs;
                                i = j;
                            }
                            for (int a = 1; a < n_runs; ++a) {   // insertion sort, stable
                                const int f = S.run_first[a], l = S.run_len[a];
                                int b = a - 1;
                                while (b >= 0 && S.run_len[b] < l) {
                                    S.run_first[b + 1] = S.run_first[b];
                                    S.run_len[b + 1] = S.run_len[b];
                                    --b;
                                }
                                S.run_first[b + 1] = f;
                                S.run_len[b + 1] = l;
                            }
                            S.n_thr = n_runs;
                        }
                        __syncthreads();
                        n_runs = S.n_thr;
                        __syncthreads();
                        for (int r = 0; r < n_runs && ok; ++r) {
                            const int first = S.run_first[r], len = S.run_len[r];
                            const int start = S.node[first], end = S.node[first + len];
                            if (start >= 0 && end >= 0 && len == 1) continue;
                            heur_subgraph_k_path(S, B, n, n_edges, avail, len + 1, start, end, lane);
                            __syncthreads();
                            if (!S.found) {
                                ok = false;
                            } else {
                                for (int i = 0; i <= len; ++i) avail &= ~(1ull << S.best[i]);
                                if (lane == 0)
                                    for (int i = 0; i <= len; ++i) S.node[first + i] = S.best[i];
                            }
                            __syncthreads();
                        }
                    }
                }
                if (ok) used = nc;
                __syncthreads();
            }
            if (!used) { fail(); return; }
            if (lane == 0 && classes_out) classes_out[inst] = used;
        } else {
            // ---- joint system: from every start node, always on over the best link to a free node; the best start
            if (lane == 0) {
                float best_beta = inf;
                int best_first = -1;
                for (int first = 0; first < n; ++first) {
                    unsigned long long used = 1ull << first;
                    int cur = first;
                    float beta = 0.0f;
                    for (int s = 1; s < p; ++s) {
                        int nxt = -1;
                        for (int v = 0; v < n; ++v)
                            if (!((used >> v) & 1ull) && (nxt < 0 || B[cur * n + v] > B[cur * n + nxt])) nxt = v;
                        const float g = heur_gamma(ti[cut_s[s - 1] - 1], B[cur * n + nxt]);
                        beta = g > beta ? g : beta;
                        used |= 1ull << nxt;
                        cur = nxt;
                    }
                    if (beta < best_beta) { best_beta = beta; best_first = first; }
                }
                unsigned long long used = 1ull << best_first;
                S.node[0] = best_first;
                for (int s = 1; s < p; ++s) {
                    const int cur = S.node[s - 1];
                    int nxt = -1;
                    for (int v = 0; v < n; ++v)
                        if (!((used >> v) & 1ull) && (nxt < 0 || B[cur * n + v] > B[cur * n + nxt])) nxt = v;
                    S.node[s] = nxt;
                    used |= 1ull << nxt;
                }
            }
        }
    }
    __syncthreads();
    // ---- Eq. 2, Eq. 3 of the placement found
    if (lane == 0) {
        float beta = 0.0f;
        for (int s = 1; s < p; ++s) {
            const float g = heur_gamma(ti[cut_s[s - 1] - 1], B[S.node[s - 1] * n + S.node[s]]);
            beta = g > beta ? g : beta;
        }
        beta_out[inst] = beta;
        segs_out[inst] = p;
        for (int s = 0; s < p; ++s) order_o[s] = S.node[s];
        for (int s = 0; s + 1 < p; ++s) cuts_o[s] = cut_s[s];
        if (classes_out && mode != 0) classes_out[inst] = 0;
    }
}

hipError_t launch_heuristic(const float* t, const float* m, int L, const float* kappa, const float* B, int n, int n_inst,
                            int n_classes, int mode, const float* draws, int n_draws, const int32_t* segs_in,
                            const int32_t* cuts_in, float* beta_out, int32_t* segs_out, int32_t* cuts_out,
                            int32_t* order_out, int32_t* classes_out, hipStream_t stream) {
    hipLaunchKernelGGL(heuristic_kernel, dim3(n_inst), dim3(64), 0, stream, t, m, L, kappa, B, n, n_classes, mode, draws,
                       n_draws, segs_in, cuts_in, beta_out, segs_out, cuts_out, order_out, classes_out);
    return hipGetLastError();
}

}  // namespace ppo
