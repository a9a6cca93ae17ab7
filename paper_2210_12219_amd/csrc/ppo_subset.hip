// Stage 2 by dynamic programming over node subsets: the same best key as the enumeration of all k!
// orderings, in k 2^(k-1) rows instead of k! DPs.
//
// The bottleneck of a solution is a maximum over its links, so what remains to be paid after the segment
// on node j ends at layer e depends only on j, e and the set R of nodes not yet used, not on the order
// of the nodes before.  For R non-empty, j' in R and a cut e:
//     A[R][j'][e] = min over e' in (e, L-(|R|-1)] with layers [e, e') fitting node j'   of  rest[R\j'][j'][e']
//     rest[R'][j'][e'] = (R' empty) ? (e' == L ? 0 : inf)
//                                   : min over j'' in R' of max(q_{j',j''}[e'-1], A[R'][j''][e'])
// i.e. A[R][j'][e] is the least bottleneck of everything after cut e if node j' takes the next segment and
// the nodes of R (j' among them) the rest of the chain.  The optimum is
//     beta* = min over j, e >= 1 with layers [0,e) fitting j  of  rest[All\j][j][e].
// The lowest-rank ordering among the optimal ones (the tie rule of the key) is the lexicographically
// smallest: position by position, the smallest unused node for which the forward row of the prefix so far
// (the same recurrence as in the enumeration) combined with `rest` still reaches beta*.
//
// One workgroup per instance; rows of A live in global scratch (2^k * k rows of L+2 codes), layer by layer
// in |R|; one wave per row.  Everything is done on the 16-bit order codes of the precompute kernel.
#include "ppo_common.h"

namespace ppo {

constexpr int kSubThreads = 1024;
constexpr int kSubWaves = kSubThreads / 64;

size_t subset_scratch_bytes_per_instance(int L, int k) { return ((size_t)k << k) * (size_t)(L + 2) * sizeof(uint16_t); }

__global__ __launch_bounds__(kSubThreads) void subset_kernel(Layout y, const unsigned char* __restrict__ ws,
                                                             uint16_t* __restrict__ scratch,
                                                             unsigned long long* __restrict__ best_key) {
    __shared__ unsigned char lo_s[PPO_MAX_K * (PPO_MAX_L + 1)];
    __shared__ uint16_t rest_s[kSubWaves][PPO_MAX_L + 2];   // one row of `rest` per wave
    __shared__ uint16_t fwd_s[2][PPO_MAX_L + 2];            // forward rows of the reconstruction
    const int L = y.L, k = y.k, inst = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int RS = L + 2;
    const unsigned char* base = ws + (size_t)inst * y.stride;
    const uint16_t* __restrict__ qc = reinterpret_cast<const uint16_t*>(base + y.qc_off);
    const float* __restrict__ dec = reinterpret_cast<const float*>(base + y.dec_off);
    uint16_t* A = scratch + (size_t)inst * ((size_t)k << k) * RS;
    for (int i = tid; i < k * (L + 1); i += kSubThreads) lo_s[i] = base[y.lo_off + i];
    __syncthreads();
    auto lo = [&](int j, int e) -> int { return lo_s[j * (L + 1) + e]; };
    auto arow = [&](uint32_t mask, int j) -> uint16_t* { return A + ((size_t)mask * k + j) * RS; };
    const uint32_t all = (1u << k) - 1u;

    // rest[R'][j'][e'] for e' = lane, lane+64, ... into `out` (one wave)
    auto rest_row = [&](uint32_t rprime, int jp, uint16_t* out) {
        for (int e = lane; e <= L; e += 64) {
            uint32_t v = kCodeInf;
            if (rprime == 0u) {
                v = e == L ? kCodeZero : kCodeInf;
            } else if (e >= 1 && e <= L - 1) {
                for (int j2 = 0; j2 < k; ++j2) {
                    if (!((rprime >> j2) & 1u)) continue;
                    const uint32_t q = qc[pair_index(jp, j2, k) * L + (e - 1)];
                    const uint32_t a = arow(rprime, j2)[e];
                    const uint32_t c = q > a ? q : a;
                    v = c < v ? c : v;
                }
            }
            out[e] = (uint16_t)v;
        }
    };

    // ---- layers |R| = 1 .. k-1 (the rows for |R| = k are not needed: the first node has no link before it)
    for (int r = 1; r <= k - 1; ++r) {
        for (uint32_t mask = (uint32_t)wave; mask <= all; mask += kSubWaves) {
            if (__popc(mask) != r) continue;
            for (int jp = 0; jp < k; ++jp) {
                if (!((mask >> jp) & 1u)) continue;
                uint16_t* rest = rest_s[wave];
                rest_row(mask & ~(1u << jp), jp, rest);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                uint16_t* out = arow(mask, jp);
                const int emax = L - (r - 1);
                for (int e = lane; e <= L; e += 64) {
                    uint32_t v = kCodeInf;
                    for (int e2 = e + 1; e2 <= emax; ++e2) {
                        if (lo(jp, e2) > e) break;   // lo is non-decreasing in its second argument
                        const uint32_t h = rest[e2];
                        v = h < v ? h : v;
                    }
                    out[e] = (uint16_t)v;
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
        __threadfence_block();
        __syncthreads();
    }

    // ---- the optimum and the lowest-rank ordering that reaches it: wave 0
    if (wave != 0) return;
    uint16_t* rest = rest_s[0];
    auto wave_min = [&](uint32_t v) -> uint32_t {
        for (int off = 32; off >= 1; off >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)v, off, 64);
            v = o < v ? o : v;
        }
        return v;
    };
    // least bottleneck over completions of a prefix whose forward row is `f`, last node j, remaining set rem
    auto completion = [&](const uint16_t* f, int j, uint32_t rem) -> uint32_t {
        rest_row(rem, j, rest);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        uint32_t v = kCodeInf;
        for (int e = lane; e <= L; e += 64) {
            const uint32_t a = f[e], b = rest[e];
            const uint32_t c = a > b ? a : b;
            v = c < v ? c : v;
        }
        __builtin_amdgcn_wave_barrier();
        return wave_min(v);
    };
    // forward row of the first segment on node j
    auto first_row = [&](int j, uint16_t* f) {
        for (int e = lane; e <= L; e += 64) f[e] = (uint16_t)((e >= 1 && e <= L - (k - 1) && lo(j, e) == 0) ? kCodeZero : kCodeInf);
    };
    // forward row of segment s on node jn after node jl: f2[e2] = min over e in [max(lo,s), e2-1] of max(f[e], q[e-1])
    auto next_row = [&](const uint16_t* f, int jl, int jn, int s, uint16_t* f2) {
        const uint16_t* q = qc + pair_index(jl, jn, k) * L;
        for (int e2 = lane; e2 <= L; e2 += 64) {
            uint32_t v = kCodeInf;
            if (e2 >= s + 1 && e2 <= L - (k - 1 - s)) {
                const int l = lo(jn, e2);
                for (int e = l > s ? l : s; e < e2; ++e) {
                    const uint32_t a = f[e], b = q[e - 1];
                    const uint32_t c = a > b ? a : b;
                    v = c < v ? c : v;
                }
            }
            f2[e2] = (uint16_t)v;
        }
    };

    uint32_t best = kCodeInf;
    for (int j = 0; j < k; ++j) {
        first_row(j, fwd_s[0]);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const uint32_t v = completion(fwd_s[0], j, all & ~(1u << j));
        best = v < best ? v : best;
    }
    if (best >= kCodeInf) {
        if (lane == 0) best_key[inst] = ((unsigned long long)kInfBits << 32);
        return;
    }
    uint32_t used = 0, rank = 0;
    int last = -1, cur = 0;
    for (int s = 0; s < k; ++s) {
        int chosen = -1;
        for (int j = 0; j < k && chosen < 0; ++j) {
            if ((used >> j) & 1u) continue;
            uint16_t* f2 = fwd_s[cur ^ 1];
            if (s == 0) first_row(j, f2);
            else next_row(fwd_s[cur], last, j, s, f2);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if (completion(f2, j, all & ~used & ~(1u << j)) == best) chosen = j;
        }
        // chosen >= 0: some completion of the prefix reaches `best`, so some next node does
        const uint32_t smaller = (uint32_t)__popc(~used & ((1u << chosen) - 1u));
        rank += smaller * factorial_u32(k - 1 - s);
        used |= 1u << chosen;
        last = chosen;
        cur ^= 1;
    }
    if (lane == 0) {
        const uint32_t bits = __float_as_uint(dec[best - kCodeZero]);
        best_key[inst] = ((unsigned long long)bits << 32) | rank;
    }
}

hipError_t launch_subset(const Layout& y, int n_inst, const void* ws, void* scratch, uint64_t* best_key,
                         hipStream_t stream) {
    if (n_inst == 0) return hipSuccess;
    hipLaunchKernelGGL(subset_kernel, dim3(n_inst), dim3(kSubThreads), 0, stream, y, static_cast<const unsigned char*>(ws),
                       static_cast<uint16_t*>(scratch), reinterpret_cast<unsigned long long*>(best_key));
    return hipGetLastError();
}

}  // namespace ppo
