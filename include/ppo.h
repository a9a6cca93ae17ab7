/*
 * ppo — exact joint partition-and-placement search on one AMD MI355X (gfx950).
 *
 * Problem (paper Sec. I, Eq. 2; Sec. III-B, Eq. 3 and the memory rule around Eq. 6):
 * a model is a chain of L layers; layer i has weight size m[i] and emits a tensor of size t[i].
 * The chain is cut into k non-empty contiguous segments, segment s = layers [c_s, c_{s+1}) with
 * 0 = c_0 < c_1 < ... < c_{k-1} < c_k = L, and segment s runs on node order[s]; the k nodes are
 * all distinct.  Node j holds at most M[j]; nodes a and b are joined by a link of bandwidth B[a][b].
 *     gamma_s = t[c_s - 1] / B[order[s-1]][order[s]]      s = 1..k-1          (Eq. 3)
 *     beta    = max_s gamma_s                              (0 when k = 1)      (Eq. 2)
 * The library returns, per instance, the minimum of beta over every feasible (order, cuts) pair —
 * the true optimum that the paper's Theorem 1 bounds from below — by evaluating every one of the
 * k! node orderings with a memory-windowed min-max chain-partition DP.
 *
 * Arithmetic (identical in the CPU oracle used by the tests):
 *     P[0] = 0, P[i+1] = P[i] + (double)m[i], accumulated in index order in binary64;
 *     segment [i,e) fits node j  iff  P[e] - P[i] <= (double)M[j]     ("within the capacity");
 *     gamma is ONE IEEE binary32 division, round to nearest even;  min and max are exact.
 * Uniqueness of the answer:
 *     order = the optimal ordering of lowest lexicographic rank (identity permutation = rank 0);
 *     cuts  = among that ordering's feasible cut vectors with bottleneck beta, the one minimising
 *             c_{k-1}, then c_{k-2}, ..., then c_1.
 *
 * Conventions for every entry point
 *   - All array arguments are DEVICE pointers owned by the caller.  The library reads inputs,
 *     writes outputs, and keeps no pointer after the work enqueued by the call has finished.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is enqueued;
 *     calls do not wait for it.  Outputs are valid once the stream has been synchronised.
 *   - Batches: arrays carry n_inst independent instances, row-major, contiguous:
 *         t, m [n_inst][L]   M [n_inst][k]   B [n_inst][k][k]
 *   - Return value: 0 on success, a negative PPO_E* code otherwise; on error nothing was enqueued
 *     by that call (PPO_EHIP excepted: a launch may have failed half-way).  n_inst = 0 succeeds
 *     and does nothing.
 *   - Data preconditions, not checked on the device: every value finite; t >= 0 (a zero of either sign
 *     counts as +0: sending nothing takes no time), m >= 0, M >= 0; B[a][b] > 0 and bit-identical to
 *     B[b][a] for a != b (the element with the smaller row index is the one read); the diagonal of B and
 *     t[.][L-1] are ignored.
 *   - Limits: 1 <= k <= L, k <= PPO_MAX_K (so that k! fits 32 bits), L <= PPO_MAX_L.
 *   - Concurrent calls are allowed when their outputs and workspaces are distinct.
 */
#ifndef PPO_H
#define PPO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PPO_OK 0
#define PPO_EINVAL (-1)   /* null pointer, L < 1, k < 1, k > L, n_inst < 0, bad rank range, a workspace that is
                             not 256-byte aligned, a key or counter array that is not 8-byte aligned */
#define PPO_ETOOBIG (-2)  /* k > PPO_MAX_K, n > PPO_CLUSTER_MAX_N or L > PPO_MAX_L */
#define PPO_EHIP (-3)     /* a HIP call failed; ppo_strerror gives the runtime's text */
#define PPO_ENOSPC (-4)   /* workspace smaller than ppo_workspace_bytes() */

#define PPO_MAX_K 12
#define PPO_MAX_L 128
#define PPO_CLUSTER_MAX_N 20   /* cluster size of ppo_solve_cluster */

/* Key of an ordering: (IEEE bits of its beta) << 32 | lexicographic rank.  For beta >= +0 the bit
 * pattern orders like the value, so the unsigned minimum of keys is the lowest beta and, among
 * equals, the lowest rank.  An all-ones key means "nothing evaluated yet". */
#define PPO_KEY_NONE 0xFFFFFFFFFFFFFFFFull

int ppo_version(void);

/* Text for a return code (static storage; for PPO_EHIP, the last HIP error seen by this thread). */
const char *ppo_strerror(int code);

/* Which enumeration kernel ppo_solve_range (and everything built on it) launches.  Process-wide,
 * not synchronised with calls in flight on other threads; meant for tests and tuning.
 *   PPO_ENUM_AUTO     paired kernel (two orderings per lane, rows in registers, wave-uniform memory windows)
 *                     when k >= 6 and L-k+2 <= 96, otherwise the generic kernel
 *   PPO_ENUM_GENERIC  always the generic kernel (one ordering per lane, any shape within the limits)
 *   PPO_ENUM_GROUPED  the grouped kernel (one ordering per lane, rows in LDS, wave-uniform windows) where it
 *                     applies (same shapes), otherwise the generic kernel
 * All produce identical results. */
#define PPO_ENUM_AUTO 0
#define PPO_ENUM_GENERIC 1
#define PPO_ENUM_GROUPED 2
int ppo_set_enumeration(int variant);

/* Bytes of device scratch that ppo_solve_ws / ppo_prepare need for this shape (0 on bad shape). */
size_t ppo_workspace_bytes(int L, int k, int n_inst);

/* Whole search: minimum bottleneck latency (Eq. 2 minimised over all orderings and cuts).
 *   beta_out  [n_inst]        seconds if t is in Mbit and B in Mbps; +inf if no feasible solution
 *   cuts_out  [n_inst][k-1]   c_1..c_{k-1} (index of the first layer of segments 1..k-1); -1 if infeasible
 *   order_out [n_inst][k]     node hosting segment s; -1 if infeasible
 * Allocates its scratch with the stream-ordered allocator and releases it on the same stream.
 * Equivalent to ppo_prepare, ppo_init_keys, ppo_solve_range over [0, k!), ppo_finalize. */
int ppo_solve(const float *t, const float *m, int L, const float *M, const float *B, int k, int n_inst,
              float *beta_out, int32_t *cuts_out, int32_t *order_out, void *stream);

/* Same, with caller-supplied device scratch of at least ppo_workspace_bytes(L,k,n_inst) bytes,
 * 256-byte aligned.  The scratch may be reused once the stream has passed this call's work. */
int ppo_solve_ws(const float *t, const float *m, int L, const float *M, const float *B, int k, int n_inst,
                 float *beta_out, int32_t *cuts_out, int32_t *order_out, void *workspace, size_t workspace_bytes,
                 void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid it): ppo_solve with its scratch in an array that is part of the library itself,
 * PPO_STATIC_SCRATCH_BYTES per GPU, held from the library's first use on that GPU until the process ends.
 * Calls no allocator of any kind.  Arguments, results and errors as for ppo_solve; in addition
 * PPO_ENOSPC when ppo_workspace_bytes(L, k, n_inst) exceeds PPO_STATIC_SCRATCH_BYTES (the headline shape,
 * L = 100, k = 10, fits 112 instances).  Every call on one GPU uses that GPU's one array: calls that overlap
 * in time on one GPU (different streams or threads) race and must be serialised by the caller.  The first
 * call on a device looks up the array's address (hipGetSymbolAddress); make it outside a capture. */
#define PPO_STATIC_SCRATCH_BYTES (16u << 20)
int ppo_solve_static(const float *t, const float *m, int L, const float *M, const float *B, int k, int n_inst,
                     float *beta_out, int32_t *cuts_out, int32_t *order_out, void *stream);

/* The same search in separate stages, for callers that split the rank range (over time, streams or
 * devices) or want to time the stages.  All stages of one search share one workspace.
 *
 * Stage 1 — per-instance tables (prefix sums of m and the window of legal segment starts per node
 * and segment end: the memory rule; the quotient t[i]/B[a][b] of Eq. 3 for every link and cut,
 * reduced to order-preserving 16-bit codes).  Must precede stages 2 and 3 on the stream. */
int ppo_prepare(const float *t, const float *m, int L, const float *M, const float *B, int k, int n_inst,
                void *workspace, size_t workspace_bytes, void *stream);

/* Set best_key[0..n_inst) to PPO_KEY_NONE. */
int ppo_init_keys(uint64_t *best_key, int n_inst, void *stream);

/* Stage 2 — evaluate the orderings with rank in [rank_begin, rank_end) (0 <= begin <= end <= k!) of
 * every instance, each with its own full DP, and fold them into best_key [n_inst] by unsigned
 * minimum.  Ranges may be issued in any order, from any number of calls; the result is that of
 * their union.  L, k, n_inst and workspace must be those given to ppo_prepare. */
int ppo_solve_range(int L, int k, int n_inst, const void *workspace, size_t workspace_bytes, uint64_t rank_begin,
                    uint64_t rank_end, uint64_t *best_key, void *stream);

/* Stage 2, the same result with less work (not the unit "full DPs evaluated" that ppo_solve_range stands
 * for).  The orderings are taken in groups that share their first k-6 nodes.  The DP rows of those nodes
 * are the same for the whole group; and since no entry of a DP row is below the least entry of the row
 * before it (D_s[e] is a minimum of maxima over entries of D_{s-1}), a group whose last shared row has no
 * entry at or below the best beta already in best_key cannot hold the optimum or a tie with it, and is left
 * after that row.  What is found is folded into best_key group by group, so that later groups see it.
 * best_key ends up exactly as after ppo_solve_range over the same range.  Shapes neither the paired nor the
 * grouped kernel takes (k < 7, or L-k+2 > 96) are evaluated in full.
 *   skipped_groups  device, [n_inst], may be NULL: incremented by the number of orderings skipped for that
 *                   instance, in units of 360; the caller zeroes it. */
int ppo_solve_range_bounded(int L, int k, int n_inst, const void *workspace, size_t workspace_bytes,
                            uint64_t rank_begin, uint64_t rank_end, uint64_t *best_key, uint64_t *skipped_groups,
                            void *stream);

/* Stage 2 by another route: dynamic programming over node subsets.  The
 * bottleneck of Eq. 2 is a maximum over links, so what is still to be paid after a cut depends only on
 * the node before the cut, the cut and the set of nodes not yet used; k 2^(k-1) rows of L+1 entries
 * replace k! DPs.  Sets best_key [n_inst] to exactly what ppo_solve_range leaves after the whole range
 * [0, k!): the optimum's beta and, among the orderings that reach it, the lowest rank (found position by
 * position as the smallest node that can still reach the optimum).  best_key is overwritten, not folded.
 * Runs the kernels of ppo_solve_cluster (below) with every node required to host a segment.  Allocates
 * k 2^(k-1) rows of L 16-bit entries of scratch per instance (and a small copy of the tables), for at most
 * 1 GiB of instances at a time, with the stream-ordered allocator. */
int ppo_solve_subsets(int L, int k, int n_inst, const void *workspace, size_t workspace_bytes, uint64_t *best_key,
                      void *stream);

/* Stage 3 — turn best_key into (beta, cuts, order): decodes the winning rank, reruns its DP keeping
 * every row, and walks back with the cut rule stated at the top.  A key whose beta is +inf (or
 * PPO_KEY_NONE) gives beta = +inf, cuts = order = -1. */
int ppo_finalize(int L, int k, int n_inst, const void *workspace, size_t workspace_bytes, const uint64_t *best_key,
                 float *beta_out, int32_t *cuts_out, int32_t *order_out, void *stream);

/* Diagnostic export: beta of each ordering of ONE instance (t,m [L]; M [k]; B [k][k]) with rank in
 * [rank_begin, rank_end), written to beta_per_ordering [rank_end - rank_begin].  Same kernels and
 * arithmetic as the search; allocates and releases its scratch on the stream. */
int ppo_eval_orderings(const float *t, const float *m, int L, const float *M, const float *B, int k,
                       uint64_t rank_begin, uint64_t rank_end, float *beta_per_ordering, void *stream);

/* The search with the compute-time term (paper Sec. I, Eq. 1: the bottleneck latency is the largest stage of
 * the pipeline, the compute time c_k of the operations on node k and the communication time gamma_k between
 * nodes k-1 and k alike; the paper then drops the compute times, Eq. 2; this entry point keeps them).
 *   w [n_inst][L]   compute work of layer i (any unit, >= 0)
 *   v [n_inst][k]   speed of node j (that unit per second, > 0)
 *   comp_s = (work of segment s) / v[order[s]]:  Q[i+1] = Q[i] + (double)w[i] in index order in binary64,
 *            comp = (float)((Q[e] - Q[i]) / (double)v[j]), one rounding to binary32
 *   beta   = max over every comp_s (s = 0..k-1) and every gamma_s (s = 1..k-1, Eq. 3)
 * Everything else (memory rule, arithmetic of gamma, uniqueness of order and cuts, outputs, +inf and -1 when
 * nothing is feasible) as for ppo_solve; with w = 0 the results are those of ppo_solve bit for bit.  Every
 * ordering runs its own DP on binary32 values (a compute stage depends on both ends of its segment, so the
 * 16-bit order codes of ppo_solve do not apply); a plain path, not the tuned one.  Allocates its scratch
 * (k (L+1)^2 words per instance, mostly) with the stream-ordered allocator. */
int ppo_solve_ct(const float *t, const float *m, const float *w, int L, const float *M, const float *v,
                 const float *B, int k, int n_inst, float *beta_out, int32_t *cuts_out, int32_t *order_out,
                 void *stream);

/* Diagnostic export for the same: beta (with the compute-time term) of each ordering of ONE instance with
 * rank in [rank_begin, rank_end), written to beta_per_ordering [rank_end - rank_begin]. */
int ppo_eval_orderings_ct(const float *t, const float *m, const float *w, int L, const float *M, const float *v,
                          const float *B, int k, uint64_t rank_begin, uint64_t rank_end, float *beta_per_ordering,
                          void *stream);

/* Cluster form (paper Sec. III-B: the partitioner fixes how many partitions there are and the placement
 * picks that many nodes of the communication graph as a simple path; Sec. IV: clusters of 5 to 50
 * devices).  The exact counterpart: over every number of segments p, 1 <= p <= min(max_segments, L),
 * every sequence of p DISTINCT nodes out of the n of the cluster and every cut vector, the minimum of
 * beta (Eq. 2, Eq. 3; memory rule and arithmetic as stated at the top).  Found by dynamic programming over
 * the sets of nodes not yet used: n 2^(n-1) rows of L 16-bit entries per instance, level by level.
 *   t, m [n_inst][L]   M [n_inst][n]   B [n_inst][n][n]      1 <= n <= PPO_CLUSTER_MAX_N, L <= PPO_MAX_L;
 *                                                            n may exceed L
 *   max_segments       1..n
 *   beta_out  [n_inst]        +inf if no feasible solution
 *   segs_out  [n_inst]        p of the solution returned; 0 if infeasible
 *   order_out [n_inst][n]     the p hosting nodes in chain order, then -1
 *   cuts_out  [n_inst][n-1]   c_1..c_{p-1}, then -1 (may be NULL when n = 1)
 * Uniqueness: among the optimal node sequences the lexicographically smallest, a sequence sorting before
 * every sequence it is a proper prefix of; then the cut rule stated at the top.
 * workspace: device, 256-byte aligned, at least ppo_cluster_workspace_bytes(L, n, 1) bytes; it holds the
 * tables of all instances and the DP rows of as many instances as fit (they are solved that many at a
 * time), so a larger workspace runs more instances per launch.  ppo_cluster_workspace_bytes(L, n, n_inst)
 * is the size at which all n_inst run together, capped at 16 GiB of rows (but never below one instance's:
 * 2.1 GB at n = 20, L = 100).  Returns 0 on a bad shape. */
size_t ppo_cluster_workspace_bytes(int L, int n, int n_inst);
int ppo_solve_cluster(const float *t, const float *m, int L, const float *M, const float *B, int n, int n_inst,
                      int max_segments, float *beta_out, int32_t *segs_out, int32_t *cuts_out, int32_t *order_out,
                      void *workspace, size_t workspace_bytes, void *stream);

/* The same problem for LARGE clusters when FEW segments are allowed (the paper's evaluation, Sec. IV, places a
 * handful of partitions on clusters of 5 to 50 devices): dynamic programming over the sets of nodes still to be
 * used, of at most max_segments members: the sum over c <= max_segments of C(n, c) c rows per instance (11.6
 * million at n = 50, max_segments = 5), in binary32.  Same result as ppo_solve_cluster wherever both apply.
 *   1 <= n <= PPO_CLUSTER_FEW_MAX_N, 1 <= max_segments <= min(n, PPO_CLUSTER_FEW_MAX_SEGMENTS), L <= PPO_MAX_L,
 *   and fewer than 2^31 rows per instance (else PPO_ETOOBIG; ppo_cluster_few_workspace_bytes returns 0)
 *   arguments, outputs and uniqueness as for ppo_solve_cluster
 * workspace: device, 256-byte aligned, at least ppo_cluster_few_workspace_bytes(L, n, max_segments, 1) bytes; it
 * holds the tables of all instances and the rows of as many instances as fit (they are solved that many at a
 * time); ppo_cluster_few_workspace_bytes(L, n, max_segments, n_inst) is the size at which all run together,
 * capped at 16 GiB of rows (but never below one instance's). */
#define PPO_CLUSTER_FEW_MAX_N 64
#define PPO_CLUSTER_FEW_MAX_SEGMENTS 8
size_t ppo_cluster_few_workspace_bytes(int L, int n, int max_segments, int n_inst);
int ppo_solve_cluster_few(const float *t, const float *m, int L, const float *M, const float *B, int n, int n_inst,
                          int max_segments, float *beta_out, int32_t *segs_out, int32_t *cuts_out,
                          int32_t *order_out, void *workspace, size_t workspace_bytes, void *stream);

/* The paper's own partitioning step (Sec. III-B1, Alg. 1), for comparison with the joint optimum: cut the chain
 * into segments that each fit a node of capacity kappa so that the SUM of the transfer sizes at the cuts,
 * t[c_1 - 1] + ... + t[c_{p-1} - 1], is least (the cheapest root-to-leaf path of the partition graph).
 * Memory rule as stated at the top; sums of transfer sizes in binary64, added from the chain's end.
 * Among partitions of equal sum: the fewest segments, then the smallest first cut, second cut, ...
 *   t, m [n_inst][L], kappa [n_inst]      device
 *   segs_out [n_inst]        p; 0 if some layer does not fit
 *   cuts_out [n_inst][L-1]   c_1..c_{p-1}, then -1 (may be NULL when L = 1)
 *   sum_out  [n_inst]        binary64; +inf if infeasible
 * The placement the paper then looks for (Alg. 2, 3) is, for these fixed cuts, what ppo_solve_cluster finds
 * exactly on the chain of the merged segments. */
int ppo_min_sum_partition(const float *t, const float *m, int L, const float *kappa, int n_inst, int32_t *segs_out,
                          int32_t *cuts_out, double *sum_out, void *stream);

/* The paper's own placement algorithm (Sec. III-B2), for scoring against the exact optimum of ppo_solve_cluster:
 * cuts by the partitioning step above (Alg. 1, capacity kappa: the paper's nodes are alike in memory); the
 * transfer sizes at the cuts sorted into n_classes classes (Eq. 5); classes matched from the highest down, within
 * a class the runs of consecutive cuts from the longest down (Alg. 3); a run of r cuts gets the path of r + 1
 * unused nodes whose weakest link is strongest, between the ends that neighbouring runs have fixed: bisection
 * over the descending list of bandwidths for the highest threshold whose graph of links at or above it (Eq. 8)
 * holds such a path (Alg. 2).  Readings where the paper is open: classes are bins of equal width between the
 * least and the greatest of t[0 .. L-2]; the path search (colour coding in the paper) is depth first in
 * increasing node order, returns the smallest node sequence, and gives up after 20,000 nodes put on the path; a
 * run both of whose ends are fixed and adjacent is matched already; if a run cannot be matched, the matching
 * starts again with one class fewer.
 *   t, m [n_inst][L]   kappa [n_inst]   B [n_inst][n][n]      1 <= n <= PPO_HEURISTIC_MAX_N, L <= PPO_MAX_L
 *   beta_out    [n_inst]        Eq. 2 of the placement found; +inf if the chain cannot be partitioned or needs
 *                               more partitions than there are nodes
 *   segs_out    [n_inst]        number of partitions p; 0 if none
 *   cuts_out    [n_inst][L-1]   c_1..c_{p-1}, then -1 (may be NULL when L = 1)
 *   order_out   [n_inst][n]     node of every partition, then -1
 *   classes_out [n_inst]        classes the matching succeeded with; may be NULL
 * Allocates n_inst doubles of scratch with the stream-ordered allocator. */
#define PPO_HEURISTIC_MAX_N 64
int ppo_place_kpath(const float *t, const float *m, int L, const float *kappa, const float *B, int n, int n_inst,
                    int n_classes, float *beta_out, int32_t *segs_out, int32_t *cuts_out, int32_t *order_out,
                    int32_t *classes_out, void *stream);

/* The two systems the paper compares its algorithm with (Sec. IV).
 *   PPO_BASELINE_JOINT   partitions: from the current layer on, the fitting end with the smallest transfer size
 *                        (the rest of the chain as soon as it fits); nodes: from a start node always on over the
 *                        best link to an unused node; the start node with the least bottleneck.  Ties go to the
 *                        smaller index.
 *   PPO_BASELINE_RANDOM  again and again a random unused node and a random number of layers among those that fit
 *                        it.  The random numbers are an input: draws [n_inst][n_draws], values in [0, 1), two per
 *                        partition (value x picks item floor(x * count)); +inf if they or the nodes run out.
 * Outputs as for ppo_place_kpath. */
#define PPO_BASELINE_JOINT 1
#define PPO_BASELINE_RANDOM 2
int ppo_place_baseline(const float *t, const float *m, int L, const float *kappa, const float *B, int n, int n_inst,
                       int kind, const float *draws, int n_draws, float *beta_out, int32_t *segs_out,
                       int32_t *cuts_out, int32_t *order_out, void *stream);

/* From a model's layer graph to the chain (paper Sec. III-A).  HOST routine: every pointer is a host pointer,
 * nothing is enqueued on the GPU.
 *   n_vertices layers, n_edges data dependencies edge_src[e] -> edge_dst[e] (a DAG with exactly one vertex
 *   without predecessors, the source); weight[v] the weight size of layer v, out_size[v] the size of the
 *   tensor it emits (already divided by whatever compression ratio the caller assumes).
 * Topological depth LP(v) = length of the longest path from the source to v.  Candidate partition points:
 * p_0 = the source; going through the vertices in order of depth, u is the next point after p iff no other
 * vertex has u's depth and every path that leaves p reaches u before any vertex deeper than u (a path that
 * ends first does not reach it).  Layer i of the chain = the vertices deeper than point i-1 and not deeper
 * than point i; vertices deeper than the last point form one more layer.
 *   t [max_layers], m [max_layers]   t[i] = out_size of point i (0 for the layer after the last point),
 *                                    m[i] = sum of the weights of layer i (added in binary64, in vertex order)
 *   point [max_layers]               vertex of point i (-1 for the layer after the last point)
 *   n_layers                         L, also set when PPO_ENOSPC says that max_layers is too small
 * PPO_EINVAL: null pointer, vertex index out of range, self loop, no or several sources, a cycle. */
int ppo_chain_from_dag(int n_vertices, int n_edges, const int32_t *edge_src, const int32_t *edge_dst,
                       const float *weight, const float *out_size, int max_layers, float *t, float *m,
                       int32_t *point, int32_t *n_layers);

/* Measurement aid, not part of the search: the rate at which this chip's vector ALUs issue the kind of
 * instruction the enumeration is made of (packed 16-bit minimum / maximum), to quote a measured peak beside
 * the nominal one of one wave instruction per 4 clocks per SIMD.  Enqueues one kernel: 256 workgroups (one per
 * compute unit; each asks for more than half a unit's LDS) of 4 * waves_per_simd waves; every wave runs
 * `iters` rounds of 64 such instructions on eight independent accumulators, without memory traffic, so a SIMD
 * issues 64 * iters * waves_per_simd of them (and 3 scalar instructions of the loop per round).  The caller times the stream.
 *   waves_per_simd  1..4
 *   sink            [256 * 256 * waves_per_simd] device words, written once at the end (so that the work is kept)
 * PPO_EINVAL: waves_per_simd or iters out of range, null sink. */
int ppo_probe_valu(int waves_per_simd, int iters, uint32_t *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PPO_H */
