// Cluster form of the exact search: the hosting nodes are a sequence of p distinct nodes chosen from a
// cluster of n, and p itself is free (1 <= p <= pmax).  In the paper the partitioner fixes the number of
// partitions and the placement picks that many nodes out of the communication graph as a simple path
// (Sec. III-B1/2); its evaluation uses clusters of 5 to 50 devices (Sec. IV).
//
// The bottleneck of Eq. 2 is a maximum over links, so what is still to be paid from a cut on depends only
// on the node that takes the next segment, the cut, and the set R of nodes not used before it:
//     A[R][j][e]     = min over e' in (e, L] with layers [e, e') fitting node j      of  rest[R \ j][j][e']
//     rest[R'][j][e'] = 0                                                   if e' = L
//                     = min over j'' in R' of max(q_{j,j''}[e'-1], A[R'][j''][e'])   if another segment may
//                                                                            follow (n - |R'| < pmax)
//                     = +inf                                                otherwise
// (q_{a,b}[i] = t[i] / B[a][b], Eq. 3) and beta* = min over j of A[All][j][0].  Rows are computed level by
// level in |R|, one launch per level, one wave per row, on 16-bit order codes of the quotients.  The
// lexicographically smallest optimal sequence (a sequence before its extensions) is rebuilt position by
// position from forward rows of the prefix combined with `rest`, then the cuts by the fixed-k cut rule.
#include "ppo_common.h"

namespace ppo {

constexpr uint32_t kClZero = 0u, kClInf = 0xFFFFu;   // codes: 0 = value 0, 1 + #smaller quotients, 0xFFFF = +inf
constexpr int kClPreThreads = 1024;
constexpr int kClLevelWaves = 4;
constexpr int kClRow = PPO_MAX_L + 2;
static_assert((PPO_CLUSTER_MAX_N * (PPO_CLUSTER_MAX_N - 1) / 2) * (PPO_MAX_L - 1) <= 24 * kClPreThreads,
              "quotients per thread of the tables kernel");
static_assert((PPO_CLUSTER_MAX_N * (PPO_CLUSTER_MAX_N - 1) / 2) * (PPO_MAX_L - 1) + 1 < (int)kClInf, "codes fit 16 bits");

struct ClusterLayout {
    int L, n, npairs, nq, rs;                       // rs: entries per row of A (L+1 rounded up to even)
    uint32_t hi_off, qc_off, dec_off, qv_off, stride;   // bytes within one instance's tables

    __host__ __device__ static ClusterLayout make(int L, int n) {
        ClusterLayout y;
        y.L = L;
        y.n = n;
        y.npairs = n * (n - 1) / 2;
        y.nq = y.npairs * (L - 1);
        y.rs = (L + 2) & ~1;
        size_t off = 0;
        y.hi_off = (uint32_t)off;
        off = align_up(off + (size_t)n * (L + 1), 16);
        y.qc_off = (uint32_t)off;
        off = align_up(off + (size_t)y.npairs * L * 2, 16);
        y.dec_off = (uint32_t)off;
        off = align_up(off + ((size_t)y.nq + 1) * 4, 16);
        y.qv_off = (uint32_t)off;
        off = align_up(off + (size_t)y.nq * 4, 256);
        y.stride = (uint32_t)off;
        return y;
    }
    __host__ __device__ size_t rows_bytes() const { return ((size_t)n << n) * (size_t)rs * sizeof(uint16_t); }
};

size_t cluster_tables_bytes(int L, int n) { return ClusterLayout::make(L, n).stride; }
size_t cluster_rows_bytes(int L, int n) { return ClusterLayout::make(L, n).rows_bytes(); }

// ---------------------------------------------------------------------------------------------
// Tables of one instance: hi[j][e] = last e' such that layers [e, e') fit node j (e if none; the memory
// rule with binary64 prefix sums), the quotients of Eq. 3 and their order codes.
// R = quotients per thread (nq <= R * kClPreThreads).
// ---------------------------------------------------------------------------------------------
template <int R>
__global__ __launch_bounds__(kClPreThreads) void cluster_tables_kernel(const float* __restrict__ t,
                                                                      const float* __restrict__ m,
                                                                      const float* __restrict__ M,
                                                                      const float* __restrict__ B, ClusterLayout y,
                                                                      unsigned char* __restrict__ ws) {
    constexpr int kTile = 4096;
    __shared__ double P[PPO_MAX_L + 1];
    __shared__ float tile[kTile];
    const int L = y.L, n = y.n, inst = blockIdx.x, tid = threadIdx.x;
    const float* ti = t + (size_t)inst * L;
    const float* mi = m + (size_t)inst * L;
    const float* Mi = M + (size_t)inst * n;
    const float* Bi = B + (size_t)inst * n * n;
    unsigned char* base = ws + (size_t)inst * y.stride;
    unsigned char* hi = base + y.hi_off;
    uint16_t* qc = reinterpret_cast<uint16_t*>(base + y.qc_off);
    float* dec = reinterpret_cast<float*>(base + y.dec_off);
    float* qv = reinterpret_cast<float*>(base + y.qv_off);
    if (tid == 0) {
        double acc = 0.0;
        P[0] = 0.0;
        for (int i = 0; i < L; ++i) {
            acc = acc + (double)mi[i];
            P[i + 1] = acc;
        }
    }
    __syncthreads();
    for (int idx = tid; idx < n * (L + 1); idx += kClPreThreads) {
        const int j = idx / (L + 1), e = idx - j * (L + 1);
        const double cap = (double)Mi[j];
        int e2 = e;
        while (e2 < L && (P[e2 + 1] - P[e]) <= cap) ++e2;
        hi[idx] = (unsigned char)e2;
    }
    const int nq = y.nq;
    float x[R];
    int below[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int idx = tid + r * kClPreThreads;
        x[r] = 0.0f;
        below[r] = 0;
        if (idx < nq) {
            const int p = idx / (L - 1), i = idx - p * (L - 1);
            int a = 0, rem = p;
            while (rem >= n - 1 - a) { rem -= n - 1 - a; ++a; }
            const int b = a + 1 + rem;
            x[r] = __fdiv_rn(ti[i], Bi[a * n + b]);
            qv[idx] = x[r];
        }
    }
    __syncthreads();   // qv of the whole instance written (global, one workgroup)
    for (int first = 0; first < nq; first += kTile) {
        const int len = nq - first < kTile ? nq - first : kTile;
        __syncthreads();
        for (int j = tid; j < len; j += kClPreThreads) tile[j] = qv[first + j];
        __syncthreads();
        for (int j = 0; j < len; ++j) {
            const float v = tile[j];
#pragma unroll
            for (int r = 0; r < R; ++r) below[r] += (v < x[r]) ? 1 : 0;
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int idx = tid + r * kClPreThreads;
        if (idx < nq) {
            const int p = idx / (L - 1), i = idx - p * (L - 1);
            qc[p * L + i] = (uint16_t)(1 + below[r]);
            dec[1 + below[r]] = x[r];
        }
    }
    if (tid == 0) dec[0] = 0.0f;
}

// rest[R'][j][e'] for e' = lane, lane + 64, ... <= L into `out` (one wave).  A: rows of the instance.
__device__ __forceinline__ void cluster_rest_row(const ClusterLayout& y, const uint16_t* __restrict__ qc,
                                                 const uint16_t* __restrict__ A, uint32_t rprime, int j, bool more,
                                                 int lane, uint16_t* out) {
    const int L = y.L, n = y.n;
    for (int e = lane; e <= L; e += 64) {
        uint32_t v = kClInf;
        if (e == L) {
            v = kClZero;
        } else if (e >= 1 && more) {
            for (uint32_t b = rprime; b; b &= b - 1u) {
                const int j2 = __ffs(b) - 1;
                const uint32_t q = qc[pair_index(j, j2, n) * L + (e - 1)];
                const uint32_t a = A[((size_t)rprime * n + j2) * y.rs + e];
                const uint32_t c = q > a ? q : a;
                v = c < v ? c : v;
            }
        }
        out[e] = (uint16_t)v;
    }
}

// ---------------------------------------------------------------------------------------------
// One level: every row A[R][j] with |R| = level.  grid.x waves share the masks, grid.y = instance.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kClLevelWaves * 64) void cluster_level_kernel(ClusterLayout y,
                                                                          const unsigned char* __restrict__ ws,
                                                                          uint16_t* __restrict__ rows, int level,
                                                                          int pmax) {
    __shared__ unsigned char hi_s[PPO_CLUSTER_MAX_N * (PPO_MAX_L + 1)];
    __shared__ uint16_t rest_s[kClLevelWaves][kClRow];
    const int L = y.L, n = y.n, inst = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const unsigned char* base = ws + (size_t)inst * y.stride;
    const uint16_t* __restrict__ qc = reinterpret_cast<const uint16_t*>(base + y.qc_off);
    uint16_t* A = rows + (size_t)inst * (((size_t)n << n) * y.rs);
    for (int i = tid; i < n * (L + 1); i += kClLevelWaves * 64) hi_s[i] = base[y.hi_off + i];
    __syncthreads();
    const bool more = n - level + 1 < pmax;   // segments up to and including this row's: n - level + 1
    const uint32_t nmask = 1u << n;
    const uint32_t stride = gridDim.x * kClLevelWaves;
    uint16_t* rest = rest_s[wave];
    uint32_t mask = blockIdx.x * kClLevelWaves + wave;
    if (level == n) mask = mask == 0u ? nmask - 1u : nmask;   // the one set of this level goes to the first wave
    for (; mask < nmask; mask += stride) {
        if (__popc(mask) != level) continue;
        for (uint32_t jb = mask; jb; jb &= jb - 1u) {
            const int j = __ffs(jb) - 1;
            cluster_rest_row(y, qc, A, mask & ~(1u << j), j, more, lane, rest);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            uint16_t* out = A + ((size_t)mask * n + j) * y.rs;
            for (int e = lane; e <= L; e += 64) {
                uint32_t v = kClInf;
                if (e < L) {
                    const int h = hi_s[j * (L + 1) + e];
                    for (int e2 = e + 1; e2 <= h; ++e2) {
                        const uint32_t r = rest[e2];
                        v = r < v ? r : v;
                    }
                }
                out[e] = (uint16_t)v;
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// ---------------------------------------------------------------------------------------------
// The optimum, the smallest optimal sequence and its cuts: one wave per instance.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void cluster_trace_kernel(ClusterLayout y, const unsigned char* __restrict__ ws,
                                                           const uint16_t* __restrict__ rows, int pmax,
                                                           float* __restrict__ beta_out, int32_t* __restrict__ segs_out,
                                                           int32_t* __restrict__ cuts_out,
                                                           int32_t* __restrict__ order_out) {
    __shared__ unsigned char hi_s[PPO_CLUSTER_MAX_N * (PPO_MAX_L + 1)];
    __shared__ uint16_t D[PPO_CLUSTER_MAX_N][kClRow];   // forward rows of the chosen prefix
    __shared__ uint16_t rest[kClRow];
    __shared__ int seq[PPO_CLUSTER_MAX_N];
    const int L = y.L, n = y.n, inst = blockIdx.x, lane = threadIdx.x;
    const unsigned char* base = ws + (size_t)inst * y.stride;
    const uint16_t* __restrict__ qc = reinterpret_cast<const uint16_t*>(base + y.qc_off);
    const float* __restrict__ dec = reinterpret_cast<const float*>(base + y.dec_off);
    const uint16_t* A = rows + (size_t)inst * (((size_t)n << n) * y.rs);
    float* beta = beta_out + inst;
    int32_t* order = order_out + (size_t)inst * n;
    int32_t* cuts = cuts_out ? cuts_out + (size_t)inst * (n - 1) : nullptr;
    for (int i = lane; i < n * (L + 1); i += 64) hi_s[i] = base[y.hi_off + i];
    for (int i = lane; i < n; i += 64) order[i] = -1;
    for (int i = lane; i < n - 1; i += 64) cuts[i] = -1;
    __syncthreads();
    auto wave_min = [&](uint32_t v) -> uint32_t {
        for (int off = 32; off >= 1; off >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)v, off, 64);
            v = o < v ? o : v;
        }
        return v;
    };
    auto hi = [&](int j, int e) -> int { return hi_s[j * (L + 1) + e]; };
    const uint32_t all = (1u << n) - 1u;
    const uint32_t best = wave_min(lane < n ? (uint32_t)A[((size_t)all * n + lane) * y.rs] : kClInf);
    if (best >= kClInf) {
        if (lane == 0) {
            *beta = __uint_as_float(kInfBits);
            segs_out[inst] = 0;
        }
        return;
    }
    uint32_t used = 0;
    int last = -1, p = 0;
    for (int s = 0; s < pmax; ++s) {
        int chosen = -1;
        uint16_t* f2 = D[s];
        for (int j = 0; j < n && chosen < 0; ++j) {
            if ((used >> j) & 1u) continue;
            if (s == 0) {
                for (int e = lane; e <= L; e += 64) f2[e] = (uint16_t)((e >= 1 && e <= hi(j, 0)) ? kClZero : kClInf);
            } else {
                // f2[e2] = min over cuts i in [s, e2) with layers [i, e2) fitting j of max(D[s-1][i], q[i-1])
                const uint16_t* f = D[s - 1];
                const uint16_t* q = qc + pair_index(last, j, n) * L;
                for (int e2 = lane; e2 <= L; e2 += 64) {
                    uint32_t v = kClInf;
                    for (int i = e2 - 1; i >= s && hi(j, i) >= e2; --i) {
                        const uint32_t a = f[i], b = q[i - 1];
                        const uint32_t c = a > b ? a : b;
                        v = c < v ? c : v;
                    }
                    f2[e2] = (uint16_t)v;
                }
            }
            cluster_rest_row(y, qc, A, all & ~used & ~(1u << j), j, s + 1 < pmax, lane, rest);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            uint32_t v = kClInf;
            for (int e = lane; e <= L; e += 64) {
                const uint32_t a = f2[e], b = rest[e];
                const uint32_t c = a > b ? a : b;
                v = (e >= 1 && c < v) ? c : v;
            }
            __builtin_amdgcn_wave_barrier();
            if (wave_min(v) == best) chosen = j;
        }
        if (chosen < 0) break;   // cannot happen: some completion of the prefix reaches `best`
        if (lane == 0) seq[s] = chosen;
        used |= 1u << chosen;
        last = chosen;
        p = s + 1;
        if (f2[L] <= best) break;   // the prefix itself is optimal: it sorts before all its extensions
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    // cuts: latest segment first, each time the smallest cut that keeps the bottleneck at `best`
    int e = L;
    for (int s = p - 1; s >= 1; --s) {
        const int js = seq[s], jl = seq[s - 1];
        const uint16_t* f = D[s - 1];
        const uint16_t* q = qc + pair_index(jl, js, n) * L;
        uint32_t first = 0xFFFFFFFFu;
        for (int i = s + lane; i < e; i += 64) {
            const uint32_t a = f[i], b = q[i - 1];
            const uint32_t c = a > b ? a : b;
            if (hi(js, i) >= e && c <= best && (uint32_t)i < first) first = (uint32_t)i;
        }
        first = wave_min(first);
        if (lane == 0) cuts[s - 1] = (int32_t)first;
        e = (int)first;
    }
    if (lane == 0) {
        *beta = dec[best];
        segs_out[inst] = p;
        for (int s = 0; s < p; ++s) order[s] = seq[s];
    }
}

hipError_t launch_cluster_tables(const float* t, const float* m, const float* M, const float* B, int L, int n,
                                 int n_inst, void* ws, hipStream_t stream) {
    const ClusterLayout y = ClusterLayout::make(L, n);
    unsigned char* w = static_cast<unsigned char*>(ws);
    if (y.nq <= 8 * kClPreThreads)
        hipLaunchKernelGGL(cluster_tables_kernel<8>, dim3(n_inst), dim3(kClPreThreads), 0, stream, t, m, M, B, y, w);
    else
        hipLaunchKernelGGL(cluster_tables_kernel<24>, dim3(n_inst), dim3(kClPreThreads), 0, stream, t, m, M, B, y, w);
    return hipGetLastError();
}

// rows of `n_inst` instances (tables at ws, rows at `rows`), levels n - pmax + 1 .. n, then the trace
hipError_t launch_cluster_solve(int L, int n, int n_inst, int pmax, const void* ws, void* rows, float* beta_out,
                                int32_t* segs_out, int32_t* cuts_out, int32_t* order_out, hipStream_t stream) {
    const ClusterLayout y = ClusterLayout::make(L, n);
    const unsigned char* w = static_cast<const unsigned char*>(ws);
    uint16_t* r = static_cast<uint16_t*>(rows);
    const uint32_t nmask = 1u << n;
    uint32_t blocks = nmask / (kClLevelWaves * 4u);
    if (blocks < 1u) blocks = 1u;
    if (blocks > 2048u) blocks = 2048u;
    for (int level = n - pmax + 1; level <= n; ++level) {
        hipLaunchKernelGGL(cluster_level_kernel, dim3(level == n ? 1u : blocks, n_inst), dim3(kClLevelWaves * 64), 0,
                           stream, y, w, r, level, pmax);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(cluster_trace_kernel, dim3(n_inst), dim3(64), 0, stream, y, w, r, pmax, beta_out, segs_out,
                       cuts_out, order_out);
    return hipGetLastError();
}

}  // namespace ppo
