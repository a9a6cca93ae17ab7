// The search with the compute-time term of Sec. I, Eq. 1: beta is the largest stage of the pipeline, compute
// stages (work of a segment over the speed of its node) and communication stages (Eq. 3) alike.  The paper
// drops the compute stages (Eq. 2); this file keeps them.
//
//   comp(i, e, j) = (float)((Q[e] - Q[i]) / (double)v[j])     Q: binary64 prefix sums of the per-layer work
//   D_0[e] = comp(0, e, pi_0)                                  if layers [0, e) fit node pi_0
//   D_s[e] = min over i in [max(lo[pi_s][e], s), e-1] of max(D_{s-1}[i], q_{pi_{s-1},pi_s}[i-1], comp(i, e, pi_s))
//   beta(pi) = D_{k-1}[L]
//
// The compute stage depends on both ends of a segment, so there are about k L^2 / 2 distinct stage values per
// instance: too many for the 16-bit order codes of the search without the term.  This path therefore works on
// the binary32 values themselves (as unsigned bit patterns: they are non-negative), one ordering per lane, its
// DP row in LDS, the compute stages read from a per-instance table in global memory.  A first, plain version:
// correct at every size, not tuned.
#include "ppo_common.h"

namespace ppo {

struct CtLayout {
    int L, k, npairs;
    uint32_t lo_off, q_off, ct_off, stride;   // bytes within one instance's slice
    __host__ __device__ static CtLayout make(int L, int k) {
        CtLayout y;
        y.L = L;
        y.k = k;
        y.npairs = k * (k - 1) / 2;
        size_t off = 0;
        y.lo_off = (uint32_t)off;                       // lo [k][L+1] u8: first legal segment start
        off = align_up(off + (size_t)k * (L + 1), 16);
        y.q_off = (uint32_t)off;                        // q [npairs][L] f32: t[i] / B[a][b], i < L-1
        off = align_up(off + (size_t)y.npairs * L * 4, 16);
        y.ct_off = (uint32_t)off;                       // ct [k][L+1][L+1] f32: comp(i, e, j) at [j][e][i], i < e
        off = align_up(off + (size_t)k * (L + 1) * (L + 1) * 4, 256);
        y.stride = (uint32_t)off;
        return y;
    }
};

size_t ct_tables_bytes(int L, int k) { return CtLayout::make(L, k).stride; }

constexpr int kCtPreThreads = 256;

__global__ __launch_bounds__(kCtPreThreads) void ct_tables_kernel(const float* __restrict__ t, const float* __restrict__ m,
                                                                  const float* __restrict__ w, const float* __restrict__ M,
                                                                  const float* __restrict__ v, const float* __restrict__ B,
                                                                  CtLayout y, unsigned char* __restrict__ ws) {
    __shared__ double P[PPO_MAX_L + 1], Q[PPO_MAX_L + 1];
    const int L = y.L, k = y.k, inst = blockIdx.x, tid = threadIdx.x, W = L + 1;
    const float* ti = t + (size_t)inst * L;
    const float* mi = m + (size_t)inst * L;
    const float* wi = w + (size_t)inst * L;
    const float* Mi = M + (size_t)inst * k;
    const float* vi = v + (size_t)inst * k;
    const float* Bi = B + (size_t)inst * k * k;
    unsigned char* base = ws + (size_t)inst * y.stride;
    if (tid == 0) {   // the definition fixes the order of the additions
        double a = 0.0, b = 0.0;
        P[0] = 0.0;
        Q[0] = 0.0;
        for (int i = 0; i < L; ++i) {
            a = a + (double)mi[i];
            b = b + (double)wi[i];
            P[i + 1] = a;
            Q[i + 1] = b;
        }
    }
    __syncthreads();
    unsigned char* lo = base + y.lo_off;
    for (int idx = tid; idx < k * W; idx += kCtPreThreads) {
        const int j = idx / W, e = idx - j * W;
        const double cap = (double)Mi[j];
        int i = 0;
        while (i < e && (P[e] - P[i]) > cap) ++i;
        lo[idx] = (unsigned char)i;
    }
    float* q = reinterpret_cast<float*>(base + y.q_off);
    for (int idx = tid; idx < y.npairs * L; idx += kCtPreThreads) {
        const int p = idx / L, i = idx - p * L;
        int a = 0, rem = p;
        while (rem >= k - 1 - a) { rem -= k - 1 - a; ++a; }
        const int b = a + 1 + rem;
        const float tv = ti[i] == 0.0f ? 0.0f : ti[i];   // a zero of either sign is +0
        q[idx] = i < L - 1 ? __fdiv_rn(tv, Bi[a * k + b]) : __uint_as_float(kInfBits);
    }
    float* ct = reinterpret_cast<float*>(base + y.ct_off);
    for (int idx = tid; idx < k * W * W; idx += kCtPreThreads) {
        const int j = idx / (W * W), rest = idx - j * W * W, e = rest / W, i = rest - e * W;
        ct[idx] = i < e ? __double2float_rn(__ddiv_rn(Q[e] - Q[i], (double)vi[j])) : __uint_as_float(kInfBits);
    }
}

// One DP of one ordering, in place in the lane's row (row[e * stride], binary32 bit patterns).
__device__ inline uint32_t ct_dp_one_ordering(uint64_t perm, int L, int k, const unsigned char* lo_s, const uint32_t* q_s,
                                              const uint32_t* __restrict__ ct, uint32_t* row, int stride) {
    const int W = L + 1;
    const int n0 = perm_at(perm, 0);
    const unsigned char* lo0 = lo_s + n0 * W;
    const uint32_t* ct0 = ct + (size_t)n0 * W * W;
    for (int e = 1; e <= L - (k - 1); ++e) row[e * stride] = lo0[e] == 0 ? ct0[e * W] : kInfBits;
    int prev = n0;
    for (int s = 1; s < k; ++s) {
        const int node = perm_at(perm, s);
        const uint32_t* q = q_s + pair_index(prev, node, k) * L;
        const unsigned char* lo = lo_s + node * W;
        const uint32_t* cj = ct + (size_t)node * W * W;
        for (int e = L - k + 1 + s; e >= s + 1; --e) {
            int first = lo[e];
            first = first > s ? first : s;
            uint32_t acc = kInfBits;
            const uint32_t* ce = cj + e * W;
            for (int i = first; i < e; ++i) {
                uint32_t c = row[i * stride];
                const uint32_t g = q[i - 1], h = ce[i];
                c = c > g ? c : g;
                c = c > h ? c : h;
                acc = c < acc ? c : acc;
            }
            row[e * stride] = acc;
        }
        prev = node;
    }
    return row[L * stride];
}

__device__ inline unsigned long long ct_wave_min_u64(unsigned long long v) {
    for (int off = 32; off >= 1; off >>= 1) {
        const unsigned long long o = __shfl_xor(v, off, 64);
        v = o < v ? o : v;
    }
    return v;
}

template <bool EXPORT>
__global__ __launch_bounds__(256) void ct_enumerate_kernel(CtLayout y, const unsigned char* __restrict__ ws,
                                                          uint32_t rank_begin, uint32_t rank_end,
                                                          unsigned long long* __restrict__ best_key,
                                                          float* __restrict__ beta_export) {
    extern __shared__ __align__(16) unsigned char ct_smem[];
    const int L = y.L, k = y.k, inst = blockIdx.y, tid = threadIdx.x, T = blockDim.x;
    const unsigned char* base = ws + (size_t)inst * y.stride;
    // lo and q are contiguous at the start of the slice
    const uint32_t table_bytes = y.ct_off;
    for (uint32_t i = tid * 16u; i < table_bytes; i += (uint32_t)T * 16u)
        *reinterpret_cast<uint4*>(ct_smem + i) = *reinterpret_cast<const uint4*>(base + i);
    __syncthreads();
    const unsigned char* lo_s = ct_smem + y.lo_off;
    const uint32_t* q_s = reinterpret_cast<const uint32_t*>(ct_smem + y.q_off);
    const uint32_t* ct = reinterpret_cast<const uint32_t*>(base + y.ct_off);
    uint32_t* row = reinterpret_cast<uint32_t*>(ct_smem + table_bytes) + tid;
    unsigned long long best = PPO_KEY_NONE;
    const uint32_t span = rank_end - rank_begin;
    for (uint32_t off = blockIdx.x * (uint32_t)T + tid; off < span; off += gridDim.x * (uint32_t)T) {
        const uint32_t r = rank_begin + off;
        const uint32_t bits = ct_dp_one_ordering(unrank_packed(r, k), L, k, lo_s, q_s, ct, row, T);
        if (EXPORT) beta_export[off] = __uint_as_float(bits);
        const unsigned long long key = ((unsigned long long)bits << 32) | r;
        best = key < best ? key : best;
    }
    if (!EXPORT) {
        best = ct_wave_min_u64(best);
        if ((tid & 63) == 0 && best != PPO_KEY_NONE) atomicMin(best_key + inst, best);
    }
}

// The winner's DP with every row kept (lanes over the segment end), then the cut rule: latest segment first,
// the smallest start whose stages (row below, link, compute) stay within beta.
__global__ __launch_bounds__(64) void ct_traceback_kernel(CtLayout y, const unsigned char* __restrict__ ws,
                                                         const unsigned long long* __restrict__ best_key,
                                                         float* __restrict__ beta_out, int32_t* __restrict__ cuts_out,
                                                         int32_t* __restrict__ order_out) {
    __shared__ uint32_t rows[PPO_MAX_K][PPO_MAX_L + 1];
    const int L = y.L, k = y.k, inst = blockIdx.x, lane = threadIdx.x, W = L + 1;
    const unsigned char* base = ws + (size_t)inst * y.stride;
    const unsigned char* lo_t = base + y.lo_off;
    const uint32_t* q_t = reinterpret_cast<const uint32_t*>(base + y.q_off);
    const uint32_t* ct = reinterpret_cast<const uint32_t*>(base + y.ct_off);
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
    const uint64_t perm = unrank_packed(r, k);
    auto stage = [&](int s, int i, int e) -> uint32_t {   // candidate i -> e of row s >= 1
        const int node = perm_at(perm, s);
        uint32_t c = rows[s - 1][i];
        const uint32_t g = q_t[pair_index(perm_at(perm, s - 1), node, k) * L + i - 1];
        const uint32_t h = ct[((size_t)node * W + e) * W + i];
        c = c > g ? c : g;
        return c > h ? c : h;
    };
    for (int e = lane; e <= L; e += 64) {
        const int n0 = perm_at(perm, 0);
        rows[0][e] = (e >= 1 && e <= L - (k - 1) && lo_t[n0 * W + e] == 0) ? ct[((size_t)n0 * W + e) * W] : kInfBits;
    }
    __syncthreads();
    for (int s = 1; s < k; ++s) {
        const unsigned char* lo = lo_t + perm_at(perm, s) * W;
        for (int e = lane; e <= L; e += 64) {
            uint32_t acc = kInfBits;
            if (e >= s + 1 && e <= L - (k - 1 - s)) {
                const int first = lo[e] > s ? lo[e] : s;
                for (int i = first; i < e; ++i) {
                    const uint32_t c = stage(s, i, e);
                    acc = c < acc ? c : acc;
                }
            }
            rows[s][e] = acc;
        }
        __syncthreads();
    }
    const uint32_t beta = rows[k - 1][L];
    if (lane == 0) {
        beta_out[inst] = __uint_as_float(beta);
        for (int s = 0; s < k; ++s) order[s] = perm_at(perm, s);
    }
    int e = L;
    for (int s = k - 1; s >= 1; --s) {
        const unsigned char* lo = lo_t + perm_at(perm, s) * W;
        const int first = lo[e] > s ? lo[e] : s;
        int chosen = -1;
        for (int i0 = first; i0 < e && chosen < 0; i0 += 64) {
            const int i = i0 + lane;
            const bool keeps = i < e && stage(s, i, e) <= beta;
            const unsigned long long found = __ballot(keeps);
            if (found) chosen = i0 + __ffsll((long long)found) - 1;
        }
        if (lane == 0) cuts[s - 1] = chosen;
        if (chosen < 0) break;   // cannot happen for a key produced by the enumeration
        e = chosen;
    }
}

hipError_t launch_ct_tables(const float* t, const float* m, const float* w, const float* M, const float* v, const float* B,
                            int L, int k, int n_inst, void* ws, hipStream_t stream) {
    const CtLayout y = CtLayout::make(L, k);
    hipLaunchKernelGGL(ct_tables_kernel, dim3(n_inst), dim3(kCtPreThreads), 0, stream, t, m, w, M, v, B, y,
                       static_cast<unsigned char*>(ws));
    return hipGetLastError();
}

hipError_t launch_ct_enumerate(int L, int k, int n_inst, const void* ws, uint32_t rank_begin, uint32_t rank_end,
                               uint64_t* best_key, float* beta_export, hipStream_t stream) {
    const uint32_t span = rank_end - rank_begin;
    if (span == 0 || n_inst == 0) return hipSuccess;
    const CtLayout y = CtLayout::make(L, k);
    // a lane's row takes (L + 1) words of LDS: 256 lanes per workgroup where that fits beside the tables, else 128
    int threads = 256;
    if ((size_t)y.ct_off + (size_t)(L + 1) * threads * 4 > (size_t)kLdsBytesPerCU) threads = 128;
    const size_t lds = (size_t)y.ct_off + (size_t)(L + 1) * threads * 4;
    if (lds > (size_t)kLdsBytesPerCU) return hipErrorInvalidValue;
    uint32_t gx = (span + threads - 1) / threads;
    if (gx > 4096u) gx = 4096u;
    hipError_t e;
    if (beta_export) {
        static std::atomic<uint64_t> lds_allowed{0};
        e = allow_full_lds(reinterpret_cast<const void*>(&ct_enumerate_kernel<true>), lds_allowed);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(ct_enumerate_kernel<true>, dim3(gx, n_inst), dim3(threads), lds, stream, y,
                           static_cast<const unsigned char*>(ws), rank_begin, rank_end,
                           reinterpret_cast<unsigned long long*>(best_key), beta_export);
    } else {
        static std::atomic<uint64_t> lds_allowed{0};
        e = allow_full_lds(reinterpret_cast<const void*>(&ct_enumerate_kernel<false>), lds_allowed);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(ct_enumerate_kernel<false>, dim3(gx, n_inst), dim3(threads), lds, stream, y,
                           static_cast<const unsigned char*>(ws), rank_begin, rank_end,
                           reinterpret_cast<unsigned long long*>(best_key), beta_export);
    }
    return hipGetLastError();
}

hipError_t launch_ct_traceback(int L, int k, int n_inst, const void* ws, const uint64_t* best_key, float* beta_out,
                               int32_t* cuts_out, int32_t* order_out, hipStream_t stream) {
    const CtLayout y = CtLayout::make(L, k);
    hipLaunchKernelGGL(ct_traceback_kernel, dim3(n_inst), dim3(64), 0, stream, y, static_cast<const unsigned char*>(ws),
                       reinterpret_cast<const unsigned long long*>(best_key), beta_out, cuts_out, order_out);
    return hipGetLastError();
}

}  // namespace ppo
