// Cluster form of the exact search for LARGE clusters and FEW segments: the hosting nodes are a sequence of
// p <= pmax distinct nodes out of n <= 64 (the paper's evaluation, Sec. IV, uses 5 to 50 devices, and its
// partitioner yields a handful of partitions).  The dynamic programme over sets of UNUSED nodes (ppo_cluster.hip)
// keeps n 2^(n-1) rows and stops at n = 20; here the rows are indexed by the set S of nodes still TO BE used:
//     G[S][j][e] = least bottleneck (Eq. 2) of layers [e, L) when node j (in S) takes the segment that starts at
//                  e and every other node of S takes exactly one of the segments after it
//     G[{j}][j][e] = 0 if layers [e, L) fit node j, else +inf
//     G[S][j][e]   = min over e' in (e, hi_j(e)], e' < L, and j'' in S \ j of max(q_{j,j''}[e'-1], G[S \ j][j''][e'])
// (q_{a,b}[i] = t[i] / B[a][b], Eq. 3; hi_j(e) = last end of a segment from e that fits node j), and
// beta* = min over |S| <= pmax, j in S of G[S][j][0]: sum over c <= pmax of C(n, c) c rows (11.6 million at n = 50,
// pmax = 5).  Values are binary32 bit patterns (non-negative, so they order as unsigned integers): with up to
// 2016 links there are more distinct quotients than 16-bit codes.  Level c = |S| is one launch; the unit of a
// wave is a set S' of c - 1 nodes, whose rows it loads once and extends by every node outside it.  Of the last
// level only the entries at e = 0 are kept (all that beta* and the first position of the answer need).
// The lexicographically smallest optimal sequence (a sequence before its extensions) is rebuilt position by
// position as in ppo_cluster.hip: F = cuts the prefix reaches within beta*, G_j = those whose link into
// candidate j is within beta*; j qualifies iff some row G[S][j], S disjoint from the prefix and small enough,
// is within beta* at a cut of G_j (one pass over the rows per position); cuts by the fixed-k cut rule.
#include "ppo_common.h"

namespace ppo {

constexpr int kFewMaxN = PPO_CLUSTER_FEW_MAX_N, kFewMaxP = PPO_CLUSTER_FEW_MAX_SEGMENTS;
constexpr uint32_t kFewNone = 0xFFFFFFFFu;

// binomial coefficients C(i, j), i <= 64, j <= kFewMaxP + 1 (64-bit: C(64, 9) does not fit 32)
struct FewBinomials {
    unsigned long long c[kFewMaxN + 1][kFewMaxP + 2];
    constexpr FewBinomials() : c{} {
        for (int i = 0; i <= kFewMaxN; ++i) {
            c[i][0] = 1;
            for (int j = 1; j <= kFewMaxP + 1; ++j) c[i][j] = i == 0 ? 0 : c[i - 1][j - 1] + c[i - 1][j];
        }
    }
};
constexpr FewBinomials kFewBinomialsHost = FewBinomials();
__constant__ FewBinomials kFewBinomials = FewBinomials();

struct FewState {
    uint32_t best, chosen, done, p, last, pad[3];
    unsigned long long used, F[2];
    unsigned long long cand[kFewMaxN][2];    // G_j of every candidate of the current position
    unsigned long long start[kFewMaxP][2];   // G of the node chosen at every position
    int32_t seq[kFewMaxP];
};

struct FewLayout {
    int L, n, pmax, rs;                    // rs: entries per row (0 .. L-1), rounded up to even
    uint32_t hi_off, qs_off, state_off, stride;   // bytes within one instance's tables
    unsigned long long level_off[kFewMaxP + 1];   // first full row of level c (1 <= c <= full levels)
    unsigned long long full_rows, top_rows;       // rows kept whole; entries of the last level (0 if pmax = 1)
    size_t rows_bytes;                            // of one instance

    __host__ __device__ int full_levels() const { return pmax > 1 ? pmax - 1 : 1; }
    __host__ static FewLayout make(int L, int n, int pmax) {
        FewLayout y{};
        y.L = L;
        y.n = n;
        y.pmax = pmax;
        y.rs = (L + 1) & ~1;
        size_t off = 0;
        y.hi_off = (uint32_t)off;
        off = align_up(off + (size_t)n * (L + 1), 16);
        y.qs_off = (uint32_t)off;
        off = align_up(off + (size_t)n * n * y.rs * 4, 16);
        y.state_off = (uint32_t)off;
        off = align_up(off + sizeof(FewState), 256);
        y.stride = (uint32_t)off;
        unsigned long long rows = 0;
        for (int c = 1; c <= y.full_levels(); ++c) {
            y.level_off[c] = rows;
            rows += kFewBinomialsHost.c[n][c] * (unsigned long long)c;
        }
        y.full_rows = rows;
        y.top_rows = pmax > 1 ? kFewBinomialsHost.c[n][pmax] * (unsigned long long)pmax : 0ull;
        y.rows_bytes = align_up((size_t)(y.full_rows * (unsigned long long)y.rs + y.top_rows) * 4, 256);
        return y;
    }
};

// Shapes this formulation takes: the rows of one instance are counted in 31 bits.
bool cluster_few_supported(int L, int n, int pmax) {
    if (L < 1 || L > PPO_MAX_L || n < 1 || n > kFewMaxN || pmax < 1 || pmax > kFewMaxP || pmax > n) return false;
    unsigned long long rows = 0;
    for (int c = 1; c <= pmax; ++c) rows += kFewBinomialsHost.c[n][c] * (unsigned long long)c;
    return rows < (1ull << 31);
}
size_t cluster_few_tables_bytes(int L, int n, int pmax) { return FewLayout::make(L, n, pmax).stride; }
size_t cluster_few_rows_bytes(int L, int n, int pmax) { return FewLayout::make(L, n, pmax).rows_bytes; }

__device__ __forceinline__ uint32_t few_wave_min(uint32_t v) {
    for (int off = 32; off >= 1; off >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)v, off, 64);
        v = o < v ? o : v;
    }
    return v;
}

// the set of `size` nodes with a given index in numeric order of the sets (combinatorial number system)
__device__ __forceinline__ unsigned long long few_set_at(unsigned long long index, int size, int n) {
    unsigned long long set = 0;
    int b = n;
    for (int i = size; i >= 1; --i) {
        do { --b; } while (kFewBinomials.c[b][i] > index);
        set |= 1ull << b;
        index -= kFewBinomials.c[b][i];
    }
    return set;
}
// the next larger number with as many bits set
__device__ __forceinline__ unsigned long long few_next_set(unsigned long long x) {
    const unsigned long long low = x & (0ull - x), up = x + low;
    return (((up ^ x) >> 2) >> (__ffsll((long long)x) - 1)) | up;
}

// ---------------------------------------------------------------------------------------------
// Tables of one instance (one workgroup): hi, the quotients of every ordered pair shifted by one entry
// (qs[j][j''][e'] = q_{j,j''}[e'-1], +inf at e' = 0 and e' >= L), the state, and the rows of level 1.
// ---------------------------------------------------------------------------------------------
constexpr int kFewTableThreads = 1024;
__global__ __launch_bounds__(kFewTableThreads) void few_tables_kernel(const float* __restrict__ t,
                                                                     const float* __restrict__ m,
                                                                     const float* __restrict__ M,
                                                                     const float* __restrict__ B, FewLayout y,
                                                                     unsigned char* __restrict__ ws,
                                                                     uint32_t* __restrict__ rows) {
    __shared__ double P[PPO_MAX_L + 1];
    __shared__ float t_s[PPO_MAX_L];
    __shared__ unsigned char hi_s[kFewMaxN * (PPO_MAX_L + 1)];
    const int L = y.L, n = y.n, rs = y.rs, inst = blockIdx.x, tid = threadIdx.x;
    const float* ti = t + (size_t)inst * L;
    const float* mi = m + (size_t)inst * L;
    const float* Mi = M + (size_t)inst * n;
    const float* Bi = B + (size_t)inst * n * n;
    unsigned char* base = ws + (size_t)inst * y.stride;
    uint32_t* qs = reinterpret_cast<uint32_t*>(base + y.qs_off);
    FewState* st = reinterpret_cast<FewState*>(base + y.state_off);
    uint32_t* R = rows + (size_t)inst * (y.rows_bytes / 4);
    if (tid == 0) {
        double acc = 0.0;
        P[0] = 0.0;
        for (int i = 0; i < L; ++i) {
            acc = acc + (double)mi[i];
            P[i + 1] = acc;
        }
        st->best = kInfBits;
        st->chosen = kFewNone;
        st->done = 0u;
        st->p = 0u;
        st->last = 0u;
        st->used = 0ull;
    }
    for (int i = tid; i < L; i += kFewTableThreads) t_s[i] = ti[i] == 0.0f ? 0.0f : ti[i];   // -0 is a size of zero: +0
    __syncthreads();
    for (int idx = tid; idx < n * (L + 1); idx += kFewTableThreads) {
        const int j = idx / (L + 1), e = idx - j * (L + 1);
        const double cap = (double)Mi[j];
        int e2 = e;
        while (e2 < L && (P[e2 + 1] - P[e]) <= cap) ++e2;
        hi_s[idx] = (unsigned char)e2;
        base[y.hi_off + idx] = (unsigned char)e2;
    }
    for (int idx = tid; idx < n * n * rs; idx += kFewTableThreads) {
        const int e = idx % rs, pr = idx / rs, a = pr / n, b = pr - a * n;
        uint32_t v = kInfBits;
        if (a != b && e >= 1 && e < L) v = __float_as_uint(__fdiv_rn(t_s[e - 1], Bi[a * n + b]));
        qs[idx] = v;
    }
    __syncthreads();
    // level 1: the rest of the chain on node j alone
    bool whole = false;
    for (int idx = tid; idx < n * rs; idx += kFewTableThreads) {
        const int j = idx / rs, e = idx - j * rs;
        const bool fits = e < L && hi_s[j * (L + 1) + e] >= L;
        R[(size_t)(y.level_off[1] + (unsigned long long)j) * rs + e] = fits ? 0u : kInfBits;
        whole |= fits && e == 0;
    }
    if (whole) atomicMin(&st->best, 0u);
}

// ---------------------------------------------------------------------------------------------
// Level c = C + 1 >= 2.  top: this is the last level, only G[S][j][0] is kept (one word per row).
// ---------------------------------------------------------------------------------------------
constexpr int kFewLevelWaves = 4;
constexpr int kFewRunLevels = 7;     // runs of 2^0 .. 2^6 entries
constexpr int kFewRunRow = 192;      // entries per run-minimum row: 128 computed per row, then +inf

template <int C>
__global__ __launch_bounds__(kFewLevelWaves * 64) void few_level_kernel(FewLayout y, unsigned char* __restrict__ ws,
                                                                       uint32_t* __restrict__ rows, int top) {
    __shared__ unsigned char hi_s[kFewMaxN * (PPO_MAX_L + 1)];
    __shared__ uint32_t run_s[kFewLevelWaves][kFewRunLevels][kFewRunRow];
    constexpr int c = C + 1;
    const int L = y.L, n = y.n, rs = y.rs, rd = rs / 2;
    const int inst = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    unsigned char* base = ws + (size_t)inst * y.stride;
    const uint32_t* __restrict__ qs = reinterpret_cast<const uint32_t*>(base + y.qs_off);
    FewState* st = reinterpret_cast<FewState*>(base + y.state_off);
    uint32_t* R = rows + (size_t)inst * (y.rows_bytes / 4);
    uint32_t* T = R + (size_t)y.full_rows * rs;   // the entries of the last level
    for (int i = tid; i < n * (L + 1); i += kFewLevelWaves * 64) hi_s[i] = base[y.hi_off + i];
    uint32_t (*run)[kFewRunRow] = run_s[wave];
    for (int i = lane; i < kFewRunLevels * (kFewRunRow - 128); i += 64)
        run[i / (kFewRunRow - 128)][128 + i % (kFewRunRow - 128)] = kInfBits;
    __syncthreads();
    const unsigned long long nsets = kFewBinomials.c[n][C];
    const unsigned long long total_waves = (unsigned long long)gridDim.x * kFewLevelWaves;
    const unsigned long long per_wave = (nsets + total_waves - 1ull) / total_waves;
    unsigned long long u = ((unsigned long long)blockIdx.x * kFewLevelWaves + (unsigned long long)wave) * per_wave;
    const unsigned long long u_end = u + per_wave < nsets ? u + per_wave : nsets;
    const unsigned long long all = n == 64 ? ~0ull : (1ull << n) - 1ull;
    const unsigned long long in_off = y.level_off[C];   // rows of level C
    const unsigned long long out_off = top ? 0ull : y.level_off[c];
    uint32_t bestw = kInfBits;
    unsigned long long set = 0;
    if (u < u_end) set = few_set_at(u, C, n);
    for (; u < u_end; ++u) {
        uint32_t a[C][2];
        int b[C];
        {
            unsigned long long bits = set;
            const uint32_t* arow = R + (size_t)(in_off + u * (unsigned long long)C) * rs + 2 * lane;
#pragma unroll
            for (int mm = 0; mm < C; ++mm) {
                b[mm] = __ffsll((long long)bits) - 1;
                bits &= bits - 1ull;
                uint2 v = make_uint2(kInfBits, kInfBits);
                if (lane < rd) v = *reinterpret_cast<const uint2*>(arow + (size_t)mm * rs);
                a[mm][0] = v.x;
                a[mm][1] = v.y;
            }
        }
        // lane j: the row of S' + j in which j stands (index within its level), for every j outside S'
        unsigned long long my_row = 0;
        {
            const int j = lane;
            unsigned long long rank = 0;
            int pos = 0;
#pragma unroll
            for (int mm = 0; mm < C; ++mm) {
                const bool below = b[mm] < j;
                rank += kFewBinomials.c[b[mm]][below ? mm + 1 : mm + 2];
                pos += below ? 1 : 0;
            }
            rank += kFewBinomials.c[j < n ? j : 0][pos + 1];
            my_row = rank * (unsigned long long)c + (unsigned long long)pos;
        }
        for (unsigned long long jb = all & ~set; jb; jb &= jb - 1ull) {
            const int j = __ffsll((long long)jb) - 1;
            const unsigned long long row = (unsigned long long)__shfl((long long)my_row, j, 64);
            uint32_t v0 = kInfBits, v1 = kInfBits;
            if (lane < rd) {
#pragma unroll
                for (int mm = 0; mm < C; ++mm) {
                    const uint2 q = *reinterpret_cast<const uint2*>(qs + (size_t)(j * n + b[mm]) * rs + 2 * lane);
                    const uint32_t x0 = q.x > a[mm][0] ? q.x : a[mm][0], x1 = q.y > a[mm][1] ? q.y : a[mm][1];
                    v0 = x0 < v0 ? x0 : v0;
                    v1 = x1 < v1 ? x1 : v1;
                }
            }
            const int hi0 = hi_s[j * (L + 1)];
            if (top) {
                // G[S][j][0] alone: the least rest[e'] with 1 <= e' <= hi_j(0) (rest is +inf at 0 and from L on)
                uint32_t r = 2 * lane <= hi0 ? v0 : kInfBits;
                const uint32_t r1 = 2 * lane + 1 <= hi0 ? v1 : kInfBits;
                r = few_wave_min(r1 < r ? r1 : r);
                if (lane == 0) T[row] = r;
                bestw = r < bestw ? r : bestw;
                continue;
            }
            // minima over runs of 2^k entries starting at each entry
            run[0][2 * lane] = v0;
            run[0][2 * lane + 1] = v1;
#pragma unroll
            for (int k = 1; k < kFewRunLevels; ++k) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                const int d = 1 << (k - 1);
                const uint32_t p0 = run[k - 1][2 * lane], p1 = run[k - 1][2 * lane + 1];
                const uint32_t f0 = run[k - 1][2 * lane + d], f1 = run[k - 1][2 * lane + 1 + d];
                run[k][2 * lane] = f0 < p0 ? f0 : p0;
                run[k][2 * lane + 1] = f1 < p1 ? f1 : p1;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            uint32_t res[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int e = 2 * lane + h;
                uint32_t r = kInfBits;
                if (e < L) {
                    int hv = hi_s[j * (L + 1) + e];
                    hv = hv < L - 1 ? hv : L - 1;   // the chain cannot end here: other nodes are still to be used
                    const int w = hv - e;
                    if (w >= 1) {
                        const int k = 31 - __clz(w);
                        const uint32_t r1 = run[k][e + 1], r2 = run[k][hv - (1 << k) + 1];
                        r = r1 < r2 ? r1 : r2;
                    }
                }
                res[h] = r;
            }
            if (lane < rd) *reinterpret_cast<uint2*>(R + (size_t)(out_off + row) * rs + 2 * lane) = make_uint2(res[0], res[1]);
            if (lane == 0) bestw = res[0] < bestw ? res[0] : bestw;
            __builtin_amdgcn_wave_barrier();
        }
        if (u + 1ull < u_end) set = few_next_set(set);
    }
    bestw = few_wave_min(bestw);
    if (lane == 0 && bestw < kInfBits) atomicMin(&st->best, bestw);
}

// ---------------------------------------------------------------------------------------------
// One position of the answer.  step(s): takes the node found for position s - 1 (if s > 0), stops if the
// prefix completes the chain, else prepares the masks G_j of position s.  scan(s): the smallest candidate
// with a row within beta* at a cut of its mask.  One wave per instance for the steps.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void few_step_kernel(FewLayout y, unsigned char* __restrict__ ws, int s,
                                                      float* __restrict__ beta_out, int32_t* __restrict__ segs_out,
                                                      int32_t* __restrict__ cuts_out, int32_t* __restrict__ order_out) {
    const int L = y.L, n = y.n, rs = y.rs, inst = blockIdx.x, lane = threadIdx.x;
    unsigned char* base = ws + (size_t)inst * y.stride;
    const unsigned char* __restrict__ hi_t = base + y.hi_off;
    const uint32_t* __restrict__ qs = reinterpret_cast<const uint32_t*>(base + y.qs_off);
    FewState* st = reinterpret_cast<FewState*>(base + y.state_off);
    int32_t* order = order_out + (size_t)inst * n;
    int32_t* cuts = cuts_out ? cuts_out + (size_t)inst * (n - 1) : nullptr;
    auto hi = [&](int j, int e) -> int { return hi_t[j * (L + 1) + e]; };
    // is cut e2 (1 <= e2 <= L) inside the window of node j that starts at the latest cut of (g0, g1) below e2?
    auto covered = [&](unsigned long long g0, unsigned long long g1, int j, int e2) -> bool {
        unsigned long long m0 = g0, m1 = 0;
        if (e2 < 64)
            m0 = g0 & ((1ull << e2) - 1ull);
        else
            m1 = e2 >= 128 ? g1 : g1 & ((1ull << (e2 - 64)) - 1ull);
        const int from = m1 ? 127 - __clzll((long long)m1) : m0 ? 63 - __clzll((long long)m0) : -1;
        return from >= 0 && hi(j, from) >= e2;
    };
    if (s == 0) {
        for (int i = lane; i < n; i += 64) order[i] = -1;
        if (cuts)
            for (int i = lane; i < n - 1; i += 64) cuts[i] = -1;
    }
    if (st->done) return;
    const uint32_t best = st->best;
    unsigned long long F0, F1, used;
    int last = 0, p = 0;
    bool finish = false;
    if (s == 0) {
        F0 = 1ull;   // the first segment starts at 0
        F1 = 0ull;
        used = 0ull;
        if (best >= kInfBits) {
            if (lane == 0) {
                beta_out[inst] = __uint_as_float(kInfBits);
                segs_out[inst] = 0;
                st->done = 1u;
            }
            return;
        }
    } else {
        const uint32_t chosen = st->chosen;
        used = st->used;
        p = (int)st->p;
        if (chosen == kFewNone) {
            finish = true;   // cannot happen: some completion of the prefix reaches beta*
            F0 = F1 = 0ull;
        } else {
            const unsigned long long G0 = st->cand[chosen][0], G1 = st->cand[chosen][1];
            const bool complete = covered(G0, G1, (int)chosen, L);
            F0 = __ballot(lane >= 1 && lane < L && covered(G0, G1, (int)chosen, lane));
            F1 = __ballot(lane + 64 < L && covered(G0, G1, (int)chosen, lane + 64));
            if (lane == 0) {
                st->seq[s - 1] = (int32_t)chosen;
                st->start[s - 1][0] = G0;
                st->start[s - 1][1] = G1;
            }
            used |= 1ull << chosen;
            last = (int)chosen;
            p = s;
            finish = complete || s == y.pmax;
        }
    }
    if (finish) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_wave_barrier();
        // cuts: latest segment first, each time the smallest start (reached by the prefix, link within beta*)
        // whose window covers the end
        int e = L;
        for (int q = p - 1; q >= 1 && cuts; --q) {
            const int jq = q == s - 1 ? last : st->seq[q];
            const unsigned long long g0 = q == s - 1 ? st->cand[last][0] : st->start[q][0];
            const unsigned long long g1 = q == s - 1 ? st->cand[last][1] : st->start[q][1];
            const unsigned long long m0 = __ballot(((g0 >> lane) & 1ull) && lane < e && hi(jq, lane) >= e);
            const unsigned long long m1 = __ballot(((g1 >> lane) & 1ull) && lane + 64 < e && hi(jq, lane + 64 < L ? lane + 64 : L) >= e);
            if (!(m0 | m1)) break;   // cannot happen: e was reached from such a start
            const int first = m0 ? __ffsll((long long)m0) - 1 : 63 + __ffsll((long long)m1);
            if (lane == 0) cuts[q - 1] = (int32_t)first;
            e = first;
        }
        if (lane == 0) {
            beta_out[inst] = __uint_as_float(best);
            segs_out[inst] = p;
            for (int q = 0; q < p; ++q) order[q] = q == s - 1 ? last : st->seq[q];
            st->done = 1u;
        }
        return;
    }
    // the masks of position s
    for (int j = 0; j < n; ++j) {
        unsigned long long g0 = 0ull, g1 = 0ull;
        if (!((used >> j) & 1ull)) {
            const uint32_t* __restrict__ q = qs + (size_t)(last * n + j) * rs;
            const int e0 = lane, e1 = lane + 64;
            g0 = __ballot(((F0 >> lane) & 1ull) && e0 < L && (s == 0 || q[e0] <= best));
            g1 = __ballot(((F1 >> lane) & 1ull) && e1 < L && (s == 0 || q[e1 < rs ? e1 : 0] <= best));
        }
        if (lane == 0) {
            st->cand[j][0] = g0;
            st->cand[j][1] = g1;
        }
    }
    if (lane == 0) {
        st->chosen = kFewNone;
        st->used = used;
        st->p = (uint32_t)p;
        st->last = (uint32_t)last;
        st->F[0] = F0;
        st->F[1] = F1;
    }
}

constexpr int kFewScanWaves = 4;
__global__ __launch_bounds__(kFewScanWaves * 64) void few_scan_kernel(FewLayout y, unsigned char* __restrict__ ws,
                                                                      const uint32_t* __restrict__ rows, int s) {
    const int n = y.n, rs = y.rs, rd = rs / 2;
    const int c = (int)blockIdx.y + 1, inst = blockIdx.z, lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    unsigned char* base = ws + (size_t)inst * y.stride;
    FewState* st = reinterpret_cast<FewState*>(base + y.state_off);
    if (st->done) return;
    const bool top = y.pmax > 1 && c == y.pmax;   // only entries at e = 0 exist; they count at the first position only
    if (top && s != 0) return;
    const uint32_t best = st->best;
    const unsigned long long used = st->used;
    const uint32_t* R = rows + (size_t)inst * (y.rows_bytes / 4);
    const uint32_t* T = R + (size_t)y.full_rows * rs;
    const unsigned long long nsets = kFewBinomials.c[n][c];
    const unsigned long long total_waves = (unsigned long long)gridDim.x * kFewScanWaves;
    const unsigned long long per_wave = (nsets + total_waves - 1ull) / total_waves;
    unsigned long long u = ((unsigned long long)blockIdx.x * kFewScanWaves + (unsigned long long)wave) * per_wave;
    const unsigned long long u_end = u + per_wave < nsets ? u + per_wave : nsets;
    if (u >= u_end) return;
    unsigned long long set = few_set_at(u, c, n);
    uint32_t found = kFewNone;   // the smallest candidate this wave has seen qualify
    for (; u < u_end; ++u) {
        if (!(set & used)) {
            if (top) {
                // lane i < c: the i-th member of the set
                unsigned long long bits = set;
                int j = 0;
                for (int i = 0; i <= lane && i < c; ++i) {
                    j = __ffsll((long long)bits) - 1;
                    bits &= bits - 1ull;
                }
                if (lane < c && T[u * (unsigned long long)c + (unsigned long long)lane] <= best)   // G_j = {0} at the first position
                    found = (uint32_t)j < found ? (uint32_t)j : found;
            } else {
                unsigned long long bits = set;
                for (int i = 0; i < c; ++i) {
                    const int j = __ffsll((long long)bits) - 1;
                    bits &= bits - 1ull;
                    if ((uint32_t)j >= found) continue;   // wave-uniform: `found` is kept the same in all lanes here
                    const unsigned long long g0 = st->cand[j][0], g1 = st->cand[j][1];
                    bool ok = false;
                    if (lane < rd) {
                        const uint2 v = *reinterpret_cast<const uint2*>(R + (size_t)(y.level_off[c] + u * (unsigned long long)c + (unsigned long long)i) * rs + 2 * lane);
                        const int e0 = 2 * lane, e1 = e0 + 1;
                        const bool in0 = ((e0 < 64 ? g0 >> e0 : g1 >> (e0 - 64)) & 1ull) != 0ull;
                        const bool in1 = ((e1 < 64 ? g0 >> e1 : g1 >> (e1 - 64)) & 1ull) != 0ull;
                        ok = (in0 && v.x <= best) || (in1 && v.y <= best);
                    }
                    if (__ballot(ok)) found = (uint32_t)j;
                }
            }
        }
        if (u + 1ull < u_end) set = few_next_set(set);
    }
    found = few_wave_min(found);
    if (lane == 0 && found != kFewNone) atomicMin(&st->chosen, found);
}

// ---------------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------------
hipError_t launch_cluster_few_tables(const float* t, const float* m, const float* M, const float* B, int L, int n,
                                     int pmax, int n_inst, void* ws, void* rows, hipStream_t stream) {
    const FewLayout y = FewLayout::make(L, n, pmax);
    hipLaunchKernelGGL(few_tables_kernel, dim3(n_inst), dim3(kFewTableThreads), 0, stream, t, m, M, B, y,
                       static_cast<unsigned char*>(ws), static_cast<uint32_t*>(rows));
    return hipGetLastError();
}

template <int C>
static hipError_t few_launch_level(dim3 grid, hipStream_t stream, const FewLayout& y, unsigned char* ws, uint32_t* rows, int top) {
    hipLaunchKernelGGL(few_level_kernel<C>, grid, dim3(kFewLevelWaves * 64), 0, stream, y, ws, rows, top);
    return hipGetLastError();
}

static uint32_t few_grid(unsigned long long sets, int waves_per_block) {
    // enough workgroups to fill the chip several times over, never more than there are sets
    unsigned long long blocks = (sets + (unsigned long long)waves_per_block - 1ull) / (unsigned long long)waves_per_block;
    const unsigned long long cap = 256ull * 32ull;
    if (blocks > cap) blocks = cap;
    return (uint32_t)(blocks ? blocks : 1ull);
}

// the tables of the n_inst instances are in ws, the rows of instance i at rows + i * rows_bytes
hipError_t launch_cluster_few_solve(int L, int n, int pmax, int n_inst, void* ws_, void* rows_, float* beta_out,
                                    int32_t* segs_out, int32_t* cuts_out, int32_t* order_out, hipStream_t stream) {
    const FewLayout y = FewLayout::make(L, n, pmax);
    unsigned char* ws = static_cast<unsigned char*>(ws_);
    uint32_t* rows = static_cast<uint32_t*>(rows_);
    for (int c = 2; c <= pmax; ++c) {
        const dim3 grid(few_grid(kFewBinomialsHost.c[n][c - 1], kFewLevelWaves), n_inst);
        const int top = c == pmax ? 1 : 0;
        hipError_t e = hipSuccess;
        switch (c - 1) {
            case 1: e = few_launch_level<1>(grid, stream, y, ws, rows, top); break;
            case 2: e = few_launch_level<2>(grid, stream, y, ws, rows, top); break;
            case 3: e = few_launch_level<3>(grid, stream, y, ws, rows, top); break;
            case 4: e = few_launch_level<4>(grid, stream, y, ws, rows, top); break;
            case 5: e = few_launch_level<5>(grid, stream, y, ws, rows, top); break;
            case 6: e = few_launch_level<6>(grid, stream, y, ws, rows, top); break;
            case 7: e = few_launch_level<7>(grid, stream, y, ws, rows, top); break;
            default: return hipErrorInvalidValue;
        }
        if (e != hipSuccess) return e;
    }
    static_assert(kFewMaxP == 8, "one case per number of members above");
    for (int s = 0; s <= pmax; ++s) {
        hipLaunchKernelGGL(few_step_kernel, dim3(n_inst), dim3(64), 0, stream, y, ws, s, beta_out, segs_out, cuts_out, order_out);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (s == pmax) break;
        unsigned long long most = 0;
        for (int c = 1; c <= pmax - s; ++c) most = kFewBinomialsHost.c[n][c] > most ? kFewBinomialsHost.c[n][c] : most;
        hipLaunchKernelGGL(few_scan_kernel, dim3(few_grid(most, kFewScanWaves), pmax - s, n_inst), dim3(kFewScanWaves * 64), 0,
                           stream, y, ws, rows, s);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace ppo
