// Measurement aid, not part of the search: how fast the vector ALUs of this chip really issue the kind of
// instruction the enumeration kernel is made of (packed 16-bit minimum / maximum), so that the fraction of the
// nominal peak (one wave instruction per 4 clocks per SIMD) can be quoted beside a measured one.
// One workgroup per compute unit (its LDS request keeps a second one out), W waves on each of the four SIMDs,
// every wave a loop of 64 packed operations per trip on eight independent accumulators (the loop's own counter,
// compare and branch are 3 scalar instructions in 67), no memory traffic in the loop.
#include <hip/hip_runtime.h>

#include <cstdint>

namespace ppo {

constexpr int kProbeUnits = 256;              // workgroups = compute units of the chip
constexpr uint32_t kProbeLds = 96u * 1024u;   // more than half of a compute unit's LDS

__global__ __launch_bounds__(1024) void valu_probe_kernel(uint32_t* __restrict__ sink, int iters) {
    extern __shared__ uint32_t probe_lds[];
    uint32_t a0 = threadIdx.x, a1 = threadIdx.x * 3u, a2 = threadIdx.x * 5u, a3 = threadIdx.x * 7u;
    uint32_t a4 = threadIdx.x * 11u, a5 = threadIdx.x * 13u, a6 = threadIdx.x * 17u, a7 = threadIdx.x * 19u;
    const uint32_t x = blockIdx.x * 0x00010001u + 0x00030005u, y = 0x7F007F00u ^ threadIdx.x;
    if (iters < 0) probe_lds[threadIdx.x] = a0;   // never taken: keeps the LDS request alive
#define PPO_PROBE_8(op, src)                                                                                    \
    op " %0, %0, " src "\n" op " %1, %1, " src "\n" op " %2, %2, " src "\n" op " %3, %3, " src "\n"             \
    op " %4, %4, " src "\n" op " %5, %5, " src "\n" op " %6, %6, " src "\n" op " %7, %7, " src "\n"
#define PPO_PROBE_16 PPO_PROBE_8("v_pk_max_u16", "%8") PPO_PROBE_8("v_pk_min_u16", "%9")
    for (int i = 0; i < iters; ++i) {
        asm volatile(PPO_PROBE_16 PPO_PROBE_16 PPO_PROBE_16 PPO_PROBE_16
                     : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7)
                     : "v"(x), "v"(y));
    }
#undef PPO_PROBE_16
#undef PPO_PROBE_8
    sink[blockIdx.x * blockDim.x + threadIdx.x] = a0 + a1 + a2 + a3 + a4 + a5 + a6 + a7;
}

hipError_t launch_valu_probe(int waves_per_simd, int iters, uint32_t* sink, hipStream_t stream) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&valu_probe_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)kProbeLds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(valu_probe_kernel, dim3(kProbeUnits), dim3(256 * waves_per_simd), kProbeLds, stream, sink, iters);
    return hipGetLastError();
}

}  // namespace ppo
