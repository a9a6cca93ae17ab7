// The paper's partitioning step on its own (Sec. III-B1, Alg. 1): cut the chain into segments that each fit a
// node of capacity kappa so that the SUM of the transfer sizes at the cuts is least (the path of least cost
// through the partition graph, whose vertices are the contiguous runs of partition points that fit and whose
// edge weights are the transfer sizes).  With f[i] = least sum for layers [i, L):
//     f[L] = 0,   f[i] = min over e in (i, L] with layers [i, e) fitting   of   (e < L ? t[e-1] : 0) + f[e].
// One wave per instance; lanes over the candidate ends e; sums in binary64, added from the chain's end.
#include "ppo_common.h"

namespace ppo {

__global__ __launch_bounds__(64) void min_sum_partition_kernel(const float* __restrict__ t, const float* __restrict__ m,
                                                               int L, const float* __restrict__ kappa,
                                                               int32_t* __restrict__ segs_out,
                                                               int32_t* __restrict__ cuts_out,
                                                               double* __restrict__ sum_out) {
    __shared__ double P[PPO_MAX_L + 1];
    __shared__ double fs[PPO_MAX_L + 1];        // least sum from layer i on (+inf: no partition)
    __shared__ int fc[PPO_MAX_L + 1];           // number of segments of that partition
    __shared__ int next_s[PPO_MAX_L + 1];       // its first segment's end
    const int inst = blockIdx.x, lane = threadIdx.x;
    const float* ti = t + (size_t)inst * L;
    const float* mi = m + (size_t)inst * L;
    const double cap = (double)kappa[inst];
    const double inf = __longlong_as_double(0x7FF0000000000000ll);
    if (lane == 0) {
        double acc = 0.0;
        P[0] = 0.0;
        for (int i = 0; i < L; ++i) {
            acc = acc + (double)mi[i];
            P[i + 1] = acc;
        }
        fs[L] = 0.0;
        fc[L] = 0;
        next_s[L] = L;
    }
    __syncthreads();
    for (int i = L - 1; i >= 0; --i) {
        // candidates: e = lane + 1 + i and that plus 64; best = least (sum, segments, e)
        double bs = inf;
        uint32_t bt = 0xFFFFFFFFu;
        for (int e = i + 1 + lane; e <= L; e += 64) {
            if (!((P[e] - P[i]) <= cap)) break;              // the sum only grows with e
            const double tail = fs[e];
            if (tail == inf) continue;
            const double s = (e < L ? (double)ti[e - 1] : 0.0) + tail;
            const uint32_t tie = ((uint32_t)(fc[e] + 1) << 8) | (uint32_t)e;
            if (s < bs || (s == bs && tie < bt)) { bs = s; bt = tie; }
        }
        for (int off = 32; off >= 1; off >>= 1) {
            const double os = __shfl_xor(bs, off, 64);
            const uint32_t ot = (uint32_t)__shfl_xor((int)bt, off, 64);
            if (os < bs || (os == bs && ot < bt)) { bs = os; bt = ot; }
        }
        if (lane == 0) {
            fs[i] = bs;
            fc[i] = bs == inf ? 0 : (int)(bt >> 8);
            next_s[i] = bs == inf ? L : (int)(bt & 0xFFu);
        }
        __syncthreads();
    }
    int32_t* cuts = cuts_out + (size_t)inst * (L - 1);
    for (int i = lane; i < L - 1; i += 64) cuts[i] = -1;
    __syncthreads();
    if (lane == 0) {
        sum_out[inst] = fs[0];
        segs_out[inst] = fs[0] == inf ? 0 : fc[0];
        if (fs[0] != inf) {
            int s = 0;
            for (int e = next_s[0]; e < L; e = next_s[e]) cuts[s++] = e;
        }
    }
}

hipError_t launch_min_sum_partition(const float* t, const float* m, int L, const float* kappa, int n_inst,
                                    int32_t* segs_out, int32_t* cuts_out, double* sum_out, hipStream_t stream) {
    hipLaunchKernelGGL(min_sum_partition_kernel, dim3(n_inst), dim3(64), 0, stream, t, m, L, kappa, segs_out, cuts_out,
                       sum_out);
    return hipGetLastError();
}

}  // namespace ppo
