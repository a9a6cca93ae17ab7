// HIP kernels of the exact partition-and-placement search for gfx950:
//   precompute  per instance: prefix sums, memory windows, latency quotients and their order codes
//   enumerate   per ordering: unrank, memory-windowed min-max chain DP, packed-key argmin
//   traceback   per instance: rerun the winner's DP keeping all rows, recover the cuts
#include "ppo_common.h"

namespace ppo {

// ---------------------------------------------------------------------------------------------
// precompute: one block per instance.
//   P[i+1] = P[i] + (double)m[i] in index order (binary64);
//   lo[j][e] = smallest i with P[e] - P[i] <= (double)M[j]   (memory rule of Sec. III-B, "within
//              the capacity"); legal segment starts for a segment ending before layer e on node j
//              are i in [lo, e-1], one contiguous run because P is non-decreasing;
//   q[p][i]  = t[i] / B[a][b], one binary32 division rounded to nearest (Eq. 3);
//   code     = kCodeZero + 1 + #{quotients of the instance strictly below q}.
// ---------------------------------------------------------------------------------------------
constexpr int kPreThreads = 1024;

__global__ __launch_bounds__(kPreThreads) void precompute_kernel(const float* __restrict__ t,
                                                                 const float* __restrict__ m,
                                                                 const float* __restrict__ M,
                                                                 const float* __restrict__ B, Layout y,
                                                                 unsigned char* __restrict__ ws) {
    __shared__ double P[PPO_MAX_L + 1];
    const int L = y.L, k = y.k, inst = blockIdx.x, tid = threadIdx.x;
    const float* ti = t + (size_t)inst * L;
    const float* mi = m + (size_t)inst * L;
    const float* Mi = M + (size_t)inst * k;
    const float* Bi = B + (size_t)inst * k * k;
    unsigned char* base = ws + (size_t)inst * y.stride;
    unsigned char* lo = base + y.lo_off;
    float* dec = reinterpret_cast<float*>(base + y.dec_off);
    float* qv = reinterpret_cast<float*>(base + y.qv_off);
    uint32_t* low = reinterpret_cast<uint32_t*>(base + y.low_off);

    if (tid == 0) {
        double acc = 0.0;
        P[0] = 0.0;
        for (int i = 0; i < L; ++i) {
            acc = acc + (double)mi[i];
            P[i + 1] = acc;
        }
    }
    __syncthreads();
    for (int idx = tid; idx < k * (L + 1); idx += kPreThreads) {
        int j = idx / (L + 1), e = idx - j * (L + 1);
        double cap = (double)Mi[j];
        int i = 0;
        while (i < e && (P[e] - P[i]) > cap) ++i;
        lo[idx] = (unsigned char)i;
        low[idx] = (uint32_t)i;
    }
    __syncthreads();
    {
        uint32_t* wt = reinterpret_cast<uint32_t*>(base + y.wt_off);
        const int rows = k > 2 ? k - 2 : 0, cols = y.wt_cols;
        const int chunks = cols / kChunkPairs;
        for (int idx = tid; idx < k * rows * chunks; idx += kPreThreads) {
            const int ch = idx % chunks, s = (idx / chunks) % rows + 1, j = idx / (chunks * rows);
            const int emax = L - k + 1 + s;
            uint32_t* row = wt + (size_t)(idx - ch) * (kChunkPairs * WinDesc::kWords);
            uint32_t rare = 0;
            for (int t = 0; t < kChunkPairs; ++t) {
                const int jj = ch * kChunkPairs + t;
                uint32_t w[2];
                for (int h = 0; h < 2; ++h) {
                    const int e = 2 * jj + s + h;
                    int v = 0;
                    if (e >= s + 1 && e <= emax) {
                        const int l = lo[j * (L + 1) + e];
                        v = e - (l > s ? l : s);
                    }
                    w[h] = (uint32_t)v;
                }
                uint32_t& ctrl = row[WinDesc::offset(jj, 0)];
                WinDesc::pack((uint32_t)jj, (jj % kJobPairs) / kChunkPairs, w[0], w[1], ctrl, row[WinDesc::offset(jj, 1)], row[WinDesc::offset(jj, 2)],
                              row[WinDesc::offset(jj, 3)]);
                rare |= ctrl & (WinDesc::kFold | WinDesc::kDeepChain);
            }
            if (rare)
                for (int t = 0; t < kChunkPairs; ++t) row[WinDesc::offset(ch * kChunkPairs + t, 0)] |= WinDesc::kChunkRare;
        }
    }
    {
        uint32_t* d0 = reinterpret_cast<uint32_t*>(base + y.d0_off);
        const int cols = y.wt_cols;
        for (int idx = tid; idx < k * cols; idx += kPreThreads) {
            const int j = idx / cols, col = idx - j * cols;
            uint32_t v[2];
            for (int h = 0; h < 2; ++h) {
                const int i = 2 * col + h;
                v[h] = (i >= 1 && i <= L - k + 1 && lo[j * (L + 1) + i] == 0) ? kCodeZero : kCodeInf;
            }
            d0[idx] = v[0] | (v[1] << 16);
        }
    }
    // The quotients of one link, t[i] / B, are in the order of the t[i] (a correctly rounded division by a
    // positive number is monotone), so each link's row is written sorted: position r holds the quotient of the
    // layer with the r-th smallest t (ties by index).  Ranking a quotient among all of them is then a binary
    // search per link instead of a comparison with every quotient.
    __shared__ float t_s[PPO_MAX_L];
    __shared__ unsigned char ord_s[PPO_MAX_L];
    __syncthreads();
    // a transfer size of zero is +0 whatever its sign bit says: -0 / B would be -0, whose bit pattern does not
    // order like its value in the key
    for (int i = tid; i < L - 1; i += kPreThreads) t_s[i] = ti[i] == 0.0f ? 0.0f : ti[i];
    __syncthreads();
    for (int i = tid; i < L - 1; i += kPreThreads) {
        const float x = t_s[i];
        int pos = 0;
        for (int i2 = 0; i2 < L - 1; ++i2) pos += (t_s[i2] < x || (t_s[i2] == x && i2 < i)) ? 1 : 0;
        ord_s[pos] = (unsigned char)i;
        base[y.ord_off + pos] = (unsigned char)i;
    }
    __syncthreads();
    const int nq = y.npairs * (L - 1);
    for (int idx = tid; idx < nq; idx += kPreThreads) {
        int p = idx / (L - 1), r = idx - p * (L - 1);
        int a = 0, rem = p;
        while (rem >= k - 1 - a) { rem -= k - 1 - a; ++a; }
        int b = a + 1 + rem;
        qv[idx] = __fdiv_rn(t_s[ord_s[r]], Bi[a * k + b]);
    }
    if (tid == 0) dec[0] = 0.0f;
}

// Order codes of the quotients (needs L >= 2): grid.x slices of whole node pairs, grid.y = instance.  All
// sorted rows are staged in LDS; a thread adds up, over the links, how many of a link's quotients are strictly
// below its own (a binary search each, four links at a time); the block then writes the aligned quotient
// rows `qa` of its pairs.
constexpr int kMaxQuot = (PPO_MAX_K * (PPO_MAX_K - 1) / 2) * (PPO_MAX_L - 1);
__global__ __launch_bounds__(kPreThreads) void codes_kernel(Layout y, unsigned char* __restrict__ ws) {
    __shared__ float rows_s[kMaxQuot];           // [npairs][L-1], each row in increasing order
    __shared__ uint16_t code_s[kPreThreads];     // codes of this block's pairs, by layer
    const int L = y.L, len = L - 1, inst = blockIdx.y, tid = threadIdx.x;
    const int ppb = kPreThreads / len;   // pairs per block
    const int nq = y.npairs * len;
    unsigned char* base = ws + (size_t)inst * y.stride;
    uint16_t* qc = reinterpret_cast<uint16_t*>(base + y.qc_off);
    float* dec = reinterpret_cast<float*>(base + y.dec_off);
    const float* __restrict__ qv = reinterpret_cast<const float*>(base + y.qv_off);
    for (int j = tid; j < nq; j += kPreThreads) rows_s[j] = qv[j];
    __syncthreads();
    const int pl = tid / len, r = tid - pl * len, p = blockIdx.x * ppb + pl;
    const bool mine = pl < ppb && p < y.npairs;
    const float x = mine ? rows_s[p * len + r] : 0.0f;
    const int i = mine ? (int)base[y.ord_off + r] : 0;   // the layer whose quotient this is
    int below = 0;
    if (mine) {
        for (int p0 = 0; p0 < y.npairs; p0 += 4) {
            int pos[4] = {0, 0, 0, 0};   // number of entries of each row below x
            const float* row[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) row[u] = rows_s + (p0 + u < y.npairs ? p0 + u : p0) * len;
#pragma unroll
            for (int step = 64; step >= 1; step >>= 1) {
                float v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int np = pos[u] + step;
                    v[u] = row[u][(np <= len ? np : len) - 1];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int np = pos[u] + step;
                    if (np <= len && v[u] < x) pos[u] = np;
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) below += p0 + u < y.npairs ? pos[u] : 0;
        }
    }
    if (mine) {
        const uint16_t code = (uint16_t)(kCodeZero + 1 + below);
        qc[p * L + i] = code;
        code_s[pl * len + i] = code;
        dec[1 + below] = x;
    }
    __syncthreads();
    uint32_t* qa = reinterpret_cast<uint32_t*>(base + y.qa_off);
    const int cols = y.qa_cols, QD = L / 2 + 1;
    const int first_pair = blockIdx.x * ppb;
    const int pairs_here = y.npairs - first_pair < ppb ? y.npairs - first_pair : ppb;
    for (int idx = tid; idx < pairs_here * cols; idx += kPreThreads) {
        const int q = idx / cols, col = idx - q * cols;
        const int i0 = col < QD ? 2 * col : 2 * (col - QD - 1) + 1;
        const uint32_t v0 = (i0 >= 0 && i0 <= L - 2) ? code_s[q * (L - 1) + i0] : kCodeInf;
        const uint32_t v1 = (i0 + 1 >= 0 && i0 + 1 <= L - 2) ? code_s[q * (L - 1) + i0 + 1] : kCodeInf;
        qa[(first_pair + q) * cols + col] = v0 | (v1 << 16);
    }
}

__global__ void init_keys_kernel(unsigned long long* keys, int n) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) keys[i] = PPO_KEY_NONE;
}

// ---------------------------------------------------------------------------------------------
// enumerate (generic variant): one ordering per lane, rank = lexicographic index.
// The lane's DP row lives in LDS as 16-bit codes, laid out [position][thread] so that a wave
// reading one position touches consecutive addresses.  Row s is computed in place:
//   g[i]   = max(D_{s-1}[i], q[{pi_{s-1},pi_s}][i-1])                       i = s .. L-k+s
//   D_s[e] = min_{i in [max(s, lo[pi_s][e]), e-1]} g[i]                      e = L-k+1+s .. s+1 (downwards)
// so that position e is overwritten only after every e' > e has read the g values below it.
// beta(pi) = D_{k-1}[L];  key = bits(beta) << 32 | rank;  wave minimum, then one atomicMin per wave.
// ---------------------------------------------------------------------------------------------
constexpr int kEnumThreads = 256;

__device__ inline uint32_t dp_one_ordering(uint64_t perm, int L, int k, const unsigned char* lo_s,
                                           const uint16_t* qc_s, uint16_t* row /* [L+1][kEnumThreads], + tid */) {
    const int n0 = perm_at(perm, 0);
    const unsigned char* lo0 = lo_s + n0 * (L + 1);
    for (int e = 1; e <= L - (k - 1); ++e) row[e * kEnumThreads] = (lo0[e] == 0) ? (uint16_t)kCodeZero : (uint16_t)kCodeInf;
    int prev = n0;
    for (int s = 1; s < k; ++s) {
        const int node = perm_at(perm, s);
        const uint16_t* q = qc_s + pair_index(prev, node, k) * L;
        const unsigned char* lo = lo_s + node * (L + 1);
        for (int i = s; i <= L - k + s; ++i) {
            uint16_t d = row[i * kEnumThreads], g = q[i - 1];
            row[i * kEnumThreads] = d > g ? d : g;
        }
        for (int e = L - k + 1 + s; e >= s + 1; --e) {
            int first = lo[e];
            first = first > s ? first : s;
            uint32_t acc = kCodeInf;
            for (int i = first; i < e; ++i) {
                uint32_t g = row[i * kEnumThreads];
                acc = g < acc ? g : acc;
            }
            row[e * kEnumThreads] = (uint16_t)acc;
        }
        prev = node;
    }
    return row[L * kEnumThreads];
}

__device__ inline unsigned long long wave_min_u64(unsigned long long v) {
    for (int off = 32; off >= 1; off >>= 1) {
        unsigned long long o = __shfl_xor(v, off, 64);
        v = o < v ? o : v;
    }
    return v;
}

template <bool EXPORT>
__global__ __launch_bounds__(kEnumThreads) void enumerate_kernel(Layout y, const unsigned char* __restrict__ ws,
                                                                 uint32_t rank_begin, uint32_t rank_end,
                                                                 unsigned long long* __restrict__ best_key,
                                                                 float* __restrict__ beta_export) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int L = y.L, k = y.k, inst = blockIdx.y, tid = threadIdx.x;
    const unsigned char* base = ws + (size_t)inst * y.stride;
    const float* dec = reinterpret_cast<const float*>(base + y.dec_off);
    // stage the instance's tables (lo, then qc) into LDS; they are contiguous in the workspace
    const uint32_t table_bytes = y.dec_off;
    for (uint32_t i = tid * 16u; i < table_bytes; i += kEnumThreads * 16u)
        *reinterpret_cast<uint4*>(smem + i) = *reinterpret_cast<const uint4*>(base + i);
    __syncthreads();
    const unsigned char* lo_s = smem + y.lo_off;
    const uint16_t* qc_s = reinterpret_cast<const uint16_t*>(smem + y.qc_off);
    uint16_t* row = reinterpret_cast<uint16_t*>(smem + table_bytes) + tid;

    unsigned long long best = PPO_KEY_NONE;
    const uint32_t span = rank_end - rank_begin;
    for (uint32_t off = blockIdx.x * kEnumThreads + tid; off < span; off += gridDim.x * kEnumThreads) {
        const uint32_t r = rank_begin + off;
        const uint64_t perm = unrank_packed(r, k);
        const uint32_t code = dp_one_ordering(perm, L, k, lo_s, qc_s, row);
        const uint32_t bits = code >= kCodeInf ? kInfBits : __float_as_uint(dec[code - kCodeZero]);
        if (EXPORT) beta_export[off] = __uint_as_float(bits);
        const unsigned long long key = ((unsigned long long)bits << 32) | r;
        best = key < best ? key : best;
    }
    if (!EXPORT) {
        best = wave_min_u64(best);
        if ((tid & 63) == 0 && best != PPO_KEY_NONE) atomicMin(best_key + inst, best);
    }
}

// ---------------------------------------------------------------------------------------------
// traceback: one block per instance, lane 0 works.  Decodes the winning rank, reruns its DP with all
// k rows kept, then walks back from e = L: for s = k-1 .. 1 the cut c_s is the smallest legal start
// i whose candidate max(D_{s-1}[i], q[i-1]) does not exceed beta, and e <- c_s.  Because
// D_{s-1}[i] <= beta exactly when some feasible prefix ends at i within the bottleneck, this yields
// the cut vector that minimises c_{k-1}, then c_{k-2}, ..., then c_1.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void traceback_kernel(Layout y, const unsigned char* __restrict__ ws,
                                                       const unsigned long long* __restrict__ best_key,
                                                       float* __restrict__ beta_out, int32_t* __restrict__ cuts_out,
                                                       int32_t* __restrict__ order_out) {
    __shared__ uint16_t rows[PPO_MAX_K][PPO_MAX_L + 1];
    __shared__ uint16_t q_s[PPO_MAX_K][PPO_MAX_L];              // [s]: link into the node at position s
    __shared__ unsigned char lo_s[PPO_MAX_K][PPO_MAX_L + 1];   // [s]: window starts of the node at position s
    const int L = y.L, k = y.k, inst = blockIdx.x, lane = threadIdx.x;
    const unsigned char* base = ws + (size_t)inst * y.stride;
    const unsigned char* lo_t = base + y.lo_off;
    const uint16_t* qc = reinterpret_cast<const uint16_t*>(base + y.qc_off);
    const float* dec = reinterpret_cast<const float*>(base + y.dec_off);
    int32_t* cuts = cuts_out + (size_t)inst * (k - 1);
    int32_t* order = order_out + (size_t)inst * k;
    const unsigned long long key = best_key[inst];
    const uint32_t bits = (uint32_t)(key >> 32), r = (uint32_t)(key & 0xFFFFFFFFull);
    if (key == PPO_KEY_NONE || bits >= kInfBits || r >= factorial_u32(k)) {
        if (lane == 0) {
            beta_out[inst] = __uint_as_float(kInfBits);
            for (int s = 0; s < k; ++s) order[s] = -1;
            for (int s = 0; s + 1 < k; ++s) cuts[s] = -1;
        }
        return;
    }
    // the rows of the winner's DP: one wave, lanes over the segment end; the quotient codes of its links and
    // the window starts of its nodes are staged first (loads that do not depend on each other)
    const uint64_t perm = unrank_packed(r, k);
    for (int s = 0; s < k; ++s) {
        const unsigned char* lo = lo_t + perm_at(perm, s) * (L + 1);
        for (int e = lane; e <= L; e += 64) lo_s[s][e] = lo[e];
        if (s == 0) continue;
        const uint16_t* q = qc + pair_index(perm_at(perm, s - 1), perm_at(perm, s), k) * L;
        for (int i = lane; i < L; i += 64) q_s[s][i] = q[i];
    }
    __syncthreads();
    for (int e = lane; e <= L; e += 64)
        rows[0][e] = (uint16_t)((e >= 1 && e <= L - (k - 1) && lo_s[0][e] == 0) ? kCodeZero : kCodeInf);
    __syncthreads();
    for (int s = 1; s < k; ++s) {
        const uint16_t* q = q_s[s];
        const unsigned char* lo = lo_s[s];
        for (int e = lane; e <= L; e += 64) {
            uint32_t acc = kCodeInf;
            if (e >= s + 1 && e <= L - (k - 1 - s)) {
                const int first = lo[e] > s ? lo[e] : s;
                for (int i = first; i < e; ++i) {
                    const uint32_t d = rows[s - 1][i], g = q[i - 1];
                    const uint32_t c = d > g ? d : g;
                    acc = c < acc ? c : acc;
                }
            }
            rows[s][e] = (uint16_t)acc;
        }
        __syncthreads();
    }
    const uint32_t beta_code = rows[k - 1][L];
    if (lane == 0) {
        beta_out[inst] = (beta_code >= kCodeInf) ? __uint_as_float(kInfBits) : dec[beta_code - kCodeZero];
        for (int s = 0; s < k; ++s) order[s] = perm_at(perm, s);
    }
    // rule T2, latest segment first: the smallest cut of the window that keeps the bottleneck (lanes over the cuts)
    int e = L;
    for (int s = k - 1; s >= 1; --s) {
        const uint16_t* q = q_s[s];
        const int first = lo_s[s][e] > s ? lo_s[s][e] : s;
        int chosen = -1;
        for (int i0 = first; i0 < e && chosen < 0; i0 += 64) {
            const int i = i0 + lane;
            bool keeps = false;
            if (i < e) {
                const uint32_t d = rows[s - 1][i], g = q[i - 1];
                keeps = (d > g ? d : g) <= beta_code;
            }
            const unsigned long long found = __ballot(keeps);
            if (found) chosen = i0 + __ffsll((long long)found) - 1;
        }
        if (lane == 0) cuts[s - 1] = chosen;
        if (chosen < 0) break;  // cannot happen for a key produced by the enumeration
        e = chosen;
    }
}

bool paired_supported(int L, int k);
hipError_t launch_pair_tables(const Layout& y, int n_inst, void* ws, hipStream_t stream);
hipError_t launch_enumerate_paired(const Layout& y, int n_inst, const void* ws, uint32_t rank_begin, uint32_t rank_end,
                                   uint64_t* best_key, float* beta_export, bool bounded, uint64_t* skipped_groups,
                                   hipStream_t stream);

hipError_t launch_precompute(const float* t, const float* m, const float* M, const float* B, const Layout& y,
                             int n_inst, void* ws, hipStream_t stream) {
    hipLaunchKernelGGL(precompute_kernel, dim3(n_inst), dim3(kPreThreads), 0, stream, t, m, M, B, y,
                       static_cast<unsigned char*>(ws));
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || y.L < 2 || y.npairs == 0) return e;   // no link, no quotient
    const int ppb = kPreThreads / (y.L - 1);
    hipLaunchKernelGGL(codes_kernel, dim3((y.npairs + ppb - 1) / ppb, n_inst), dim3(kPreThreads), 0, stream, y,
                       static_cast<unsigned char*>(ws));
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_pair_tables(y, n_inst, ws, stream);
}

hipError_t launch_init_keys(uint64_t* keys, int n_inst, hipStream_t stream) {
    hipLaunchKernelGGL(init_keys_kernel, dim3((n_inst + 255) / 256), dim3(256), 0, stream,
                       reinterpret_cast<unsigned long long*>(keys), n_inst);
    return hipGetLastError();
}

bool grouped_supported(int L, int k);
hipError_t launch_enumerate_grouped(const Layout& y, int n_inst, const void* ws, uint32_t rank_begin,
                                    uint32_t rank_end, uint64_t* best_key, float* beta_export, bool shared_prefix,
                                    uint64_t* skipped_groups, hipStream_t stream);

// 0: pick per shape (grouped kernel when k >= 6 and the rows fit LDS), 1: always the generic kernel
static std::atomic<int> g_enumeration_variant{0};   // read by every launch, set by tests: atomic, so that a set during a launch on another thread is a plain race-free read of either value
void set_enumeration_variant(int v) { g_enumeration_variant.store(v, std::memory_order_relaxed); }

size_t enumerate_lds_bytes(const Layout& y) { return (size_t)y.dec_off + (size_t)(y.L + 1) * kEnumThreads * 2; }

// shared_prefix asks for the bounded mode of the paired or the grouped kernel where one of them applies; elsewhere
// every ordering is evaluated in full
hipError_t launch_enumerate(const Layout& y, int n_inst, const void* ws, uint32_t rank_begin, uint32_t rank_end,
                            uint64_t* best_key, float* beta_export, bool shared_prefix, uint64_t* skipped_groups,
                            hipStream_t stream) {
    const uint32_t span = rank_end - rank_begin;
    if (span == 0 || n_inst == 0) return hipSuccess;
    const int variant = g_enumeration_variant.load(std::memory_order_relaxed);
    if (variant == PPO_ENUM_AUTO && paired_supported(y.L, y.k))
        return launch_enumerate_paired(y, n_inst, ws, rank_begin, rank_end, best_key, beta_export, shared_prefix,
                                       skipped_groups, stream);
    if ((variant == PPO_ENUM_AUTO || variant == PPO_ENUM_GROUPED) && grouped_supported(y.L, y.k))
        return launch_enumerate_grouped(y, n_inst, ws, rank_begin, rank_end, best_key, beta_export, shared_prefix,
                                        skipped_groups, stream);
    const size_t lds = enumerate_lds_bytes(y);
    uint32_t gx = (span + kEnumThreads - 1) / kEnumThreads;
    if (gx > 4096u) gx = 4096u;
    hipError_t e;
    if (beta_export) {
        static std::atomic<uint64_t> lds_allowed{0};
        e = allow_full_lds(reinterpret_cast<const void*>(&enumerate_kernel<true>), lds_allowed);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(enumerate_kernel<true>, dim3(gx, n_inst), dim3(kEnumThreads), lds, stream, y,
                           static_cast<const unsigned char*>(ws), rank_begin, rank_end,
                           reinterpret_cast<unsigned long long*>(best_key), beta_export);
    } else {
        static std::atomic<uint64_t> lds_allowed{0};
        e = allow_full_lds(reinterpret_cast<const void*>(&enumerate_kernel<false>), lds_allowed);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(enumerate_kernel<false>, dim3(gx, n_inst), dim3(kEnumThreads), lds, stream, y,
                           static_cast<const unsigned char*>(ws), rank_begin, rank_end,
                           reinterpret_cast<unsigned long long*>(best_key), beta_export);
    }
    return hipGetLastError();
}

hipError_t launch_traceback(const Layout& y, int n_inst, const void* ws, const uint64_t* best_key, float* beta_out,
                            int32_t* cuts_out, int32_t* order_out, hipStream_t stream) {
    hipLaunchKernelGGL(traceback_kernel, dim3(n_inst), dim3(64), 0, stream, y, static_cast<const unsigned char*>(ws),
                       reinterpret_cast<const unsigned long long*>(best_key), beta_out, cuts_out, order_out);
    return hipGetLastError();
}

}  // namespace ppo
