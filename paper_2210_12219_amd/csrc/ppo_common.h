// Shared declarations of the ppo HIP library: workspace layout, value codes, small device helpers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "ppo.h"
#include "ppo_chain_asm.h"

namespace ppo {

// Every latency that can occur in an instance is one of the npairs*(L-1) quotients t[i]/B[a][b]
// (Eq. 3), or 0 (no link crossed yet), or +inf (infeasible).  The precompute kernel replaces each
// by a 16-bit code that orders exactly like the value (equal values, equal codes), so the DP can
// run on 16-bit integers; the winner's code is mapped back to the binary32 quotient afterwards.
// Codes are also valid positive normal binary16 patterns, which order like unsigned integers.
constexpr uint32_t kCodeZero = 0x0400u;  // value +0
constexpr uint32_t kCodeInf = 0x7C00u;   // value +inf
constexpr uint32_t kInfBits = 0x7F800000u;

__host__ __device__ inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// A kernel that asks for more than 64 KB of dynamic LDS has to have its limit raised first.  The limit is a
// property of the kernel on a device, shared by every thread of the process, so it is raised once (per kernel
// and device; `done` holds one bit per device) to all the LDS a compute unit has, never to a launch's own
// size: two host threads launching different shapes then cannot lower each other's limit.
constexpr int kLdsBytesPerCU = 160 * 1024;
inline hipError_t allow_full_lds(const void* kernel, std::atomic<uint64_t>& done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesPerCU);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return e;
}

// Per-instance tables written by the precompute kernel and read by the enumeration and traceback.
//   lo  [k][L+1] u8   lo[j][e] = first layer i such that layers [i,e) fit on node j (== e: none)
//   qc  [npairs][L] u16   qc[p][i] = code of t[i] / B[a][b] for the unordered pair p = {a,b}, i < L-1
//   dec [npairs*(L-1)+2] f32   dec[code - kCodeZero] = value of the code
//   low [k][L+1] u32  the lo table again, one dword per entry (for scalar loads)
//   wt  [k][k-2][wt_cols/4][4][4] u32   chain descriptors for the grouped kernel: for node j, DP row
//       s = 1..k-2 and output dword jj (positions e = 2jj+s and e+1 of row s), from the window lengths
//       w = e - max(lo[j][e], s) if s+1 <= e <= L-k+1+s, else 0 (wx for e, wy for e+1), see WinDesc;
//       the four words of the four outputs of a chunk are stored word by word (ctrl x4, below x4, ...)
//   qa  [npairs][qa_cols] u32   the codes of qc again, two per dword, in both alignments, for the
//       grouped kernel: column a < QD holds (q[2a], q[2a+1]); column QD+1+a holds (q[2a+1], q[2a+2])
//       for a = -1 .. QD-1, where QD = L/2+1 and codes outside 0..L-2 read as +inf
//   d0  [k][wt_cols] u32   row 0 of the DP for first node j, two codes per dword: code of 0 at
//       index i if 1 <= i <= L-k+1 and layers [0,i) fit node j, else +inf (index i = 2*col, 2*col+1)
//   pt  [k][k-1][48] u32   for node j and DP row s = 1..k-1: where the paired kernel enters its code for each
//       output of the row (see ppo_paired.hip)
//   qv  [npairs][L-1] f32   the quotients themselves, each link's row in increasing order (between the two
//       kernels that make the tables);  ord [L-1] u8  the layers in increasing order of t: entry r of a row
//       of qv belongs to layer ord[r]
// Chain descriptor of one output dword (positions x = e and y = e+1) of the grouped kernel, four words.
// The kernel works on chunks of kChunkPairs output dwords and holds the input dword at an output's own
// index and the kChainDepth dwords below it in registers.  The entries of the row below are counted
// downwards from x's first candidate: u = 0, 1, ...; entry u is candidate u of x (wanted if u < wx) and
// candidate u+1 of y (wanted if u+1 < wy); entry u = -1 is y's first candidate.  Dword a below the output's
// index holds entry 2a in its lower half and entry 2a-1 in its upper half.  Because wy <= wx+1, the entries
// both positions want are u = 0 .. C-1 with C = wy-1 (0 if wy = 0).  n = C/2 steps fold two of them each
// into both halves; then one masked step offers entries 2n and 2n+1; what x wants beyond that (entries
// 2n+2 .. wx-1) is folded separately.
//   ctrl      bit  0      wx > 2n+2 (entries left for the separate fold)
//             bit  1      n > depth (the chain continues below the registers), depth = chain_depth(c) for the
//                         output's chunk c of its job: later chunks have more of the job's fetch below them
//             bit  2      bit 0 or bit 1 is set in some descriptor of this output's chunk
//             bits 3..7   ctrl & 0xF8 = PPO_CHAIN_ENTRY0 + 8 * (depth - min(n, depth)): the byte distance
//                         the chain's computed jump adds to reach the first step to execute
//             bits 8..14  for the separate fold: wx/2 - (n+1), the number of dwords it reads beyond dword n+1
//             bit  15     wx is even (the lower half of the last of these dwords is not wanted)
//             bits 16..31 0 if y wants entry -1 (wy >= 1), else +inf: upper half of the accumulator's
//                         initial mask (the lower half is +inf: x does not want entry -1)
//   below     byte distance, in the lane's row (128 bytes per dword), from the first dword the task fetches
//             (kChainDepth below the chunk's first output) to the dword n+1 below this output; may be
//             negative (two's complement)
//   maskA     for entry 2n: per half, 0 if that position wants it, else +inf (max(v, mask) keeps or drops)
//   maskB     for entry 2n+1: lower half as above; upper half +inf (y never wants it)
constexpr int kChunkPairs = 4;
constexpr int kChainDepth = PPO_CHAIN_DEPTH;
constexpr int kJobChunks = 3;                         // chunks of a job of the grouped kernel
constexpr int kJobPairs = kJobChunks * kChunkPairs;   // its output dwords: a part of a row
__host__ __device__ constexpr int chain_depth(int c) { return PPO_CHAIN_DEPTH + c * PPO_CHAIN_DEPTH_STEP; }
static_assert(PPO_CHAIN_DEPTH_STEP == kChunkPairs, "a later chunk gains the dwords of the chunks before it");
static_assert(PPO_CHAIN_ENTRY0 % 8 == 0 && PPO_CHAIN_ENTRY0 + 8 * chain_depth(kJobChunks - 1) <= 0xF8, "jump distance must fit bits 3..7");
struct WinDesc {
    static constexpr uint32_t kFold = 0x1u, kDeepChain = 0x2u, kChunkRare = 0x4u, kJumpMask = 0xF8u, kWxEven = 0x8000u;
    static constexpr int kWords = 4;
    __host__ __device__ static uint32_t fold_dwords(uint32_t ctrl) { return (ctrl >> 8) & 0x7Fu; }
    // number of steps, from the second word and the output's place t in its chunk
    __host__ __device__ static uint32_t steps(uint32_t below, uint32_t t) {
        return t + (uint32_t)kChainDepth - 1u - (uint32_t)((int32_t)below >> 7);
    }
    // descriptor of output column jj, in chunk c of its job, from the two window lengths (without bit 2 of ctrl)
    __host__ __device__ static void pack(uint32_t jj, int c, uint32_t wx, uint32_t wy, uint32_t& ctrl, uint32_t& below,
                                         uint32_t& maskA, uint32_t& maskB) {
        const uint32_t inf = kCodeInf;
        const uint32_t C = wy >= 1u ? (wx < wy - 1u ? wx : wy - 1u) : 0u;
        const uint32_t depth = (uint32_t)chain_depth(c);
        const uint32_t n = C >> 1, nc = n < depth ? n : depth;
        const bool fold = wx > 2u * n + 2u;
        ctrl = (fold ? kFold : 0u) | (n > depth ? kDeepChain : 0u) |
               ((uint32_t)PPO_CHAIN_ENTRY0 + 8u * (depth - nc)) |
               (fold ? (((wx >> 1) - (n + 1u)) << 8) | ((wx & 1u) ? 0u : kWxEven) : 0u) | ((wy >= 1u ? 0u : inf) << 16);
        below = ((jj % kChunkPairs) + (uint32_t)kChainDepth - 1u - n) * 128u;
        maskA = (wx > 2u * n ? 0u : inf) | ((C > 2u * n ? 0u : inf) << 16);
        maskB = (wx > 2u * n + 1u ? 0u : inf) | (inf << 16);
    }
    // dword offset of word `word` of output column jj within the descriptor row of a (node, DP row)
    __host__ __device__ static uint32_t offset(uint32_t jj, uint32_t word) {
        return (jj / kChunkPairs) * (uint32_t)(kWords * kChunkPairs) + word * kChunkPairs + (jj % kChunkPairs);
    }
};

// Entry offsets of the paired enumeration kernel for one (node, DP row): where the chain of every output of
// the row starts in that kernel's unrolled code, 16 bits each, outputs 2x+1 and 2x+2 in dword x.
constexpr int kPairTableDwords = 48;

struct Layout {
    int L, k, npairs, wt_cols, qa_cols;
    uint32_t lo_off, qc_off, dec_off, low_off, wt_off, qa_off, d0_off, qv_off, ord_off, pt_off, stride;  // bytes within one instance's slice

    __host__ __device__ static Layout make(int L, int k) {
        Layout y;
        y.L = L;
        y.k = k;
        y.npairs = k * (k - 1) / 2;
        size_t off = 0;
        y.lo_off = (uint32_t)off;
        off = align_up(off + (size_t)k * (L + 1), 16);
        y.qc_off = (uint32_t)off;
        off = align_up(off + (size_t)y.npairs * L * 2, 16);
        y.dec_off = (uint32_t)off;
        off = align_up(off + ((size_t)y.npairs * (L - 1) + 2) * 4, 16);
        y.low_off = (uint32_t)off;
        off = align_up(off + (size_t)k * (L + 1) * 4, 16);
        off = align_up(off, 64);
        y.wt_off = (uint32_t)off;
        y.wt_cols = (int)align_up((size_t)((L - k + 2 + 1) / 2), 4);
        off = align_up(off + (size_t)k * (k > 2 ? k - 2 : 0) * y.wt_cols * WinDesc::kWords * 4, 16);
        y.qa_off = (uint32_t)off;
        y.qa_cols = 2 * (L / 2 + 1) + 2;
        off = align_up(off + (size_t)y.npairs * y.qa_cols * 4, 16);
        y.d0_off = (uint32_t)off;
        off = align_up(off + (size_t)k * y.wt_cols * 4, 16);
        y.qv_off = (uint32_t)off;
        off = align_up(off + (size_t)y.npairs * (L > 1 ? L - 1 : 0) * 4, 16);
        y.ord_off = (uint32_t)off;
        off = align_up(off + (size_t)L, 64);
        y.pt_off = (uint32_t)off;   // entry offsets of the paired kernel: [k][k-1][kPairTableDwords] u32
        off = align_up(off + (size_t)k * (k > 1 ? k - 1 : 0) * kPairTableDwords * 4, 256);
        y.stride = (uint32_t)off;
        return y;
    }
};

// index of the unordered pair {a,b}, a != b, among the k(k-1)/2 pairs in row-major upper-triangle order
__host__ __device__ inline int pair_index(int a, int b, int k) {
    int lo = a < b ? a : b, hi = a < b ? b : a;
    return lo * k - lo * (lo + 1) / 2 + (hi - lo - 1);
}

__host__ __device__ inline uint32_t factorial_u32(int n) {
    uint32_t f = 1;
    for (int i = 2; i <= n; ++i) f *= (uint32_t)i;
    return f;
}

// The permutation of 0..k-1 with lexicographic rank r, packed four bits per position
// (position p in bits [4p, 4p+4)).  Digit p of r in the factorial number system selects the
// digit-th smallest node not used by positions 0..p-1.
__device__ inline uint64_t unrank_packed(uint32_t r, int k) {
    uint64_t avail = 0xBA9876543210ull;  // nibble j = j-th smallest unused node
    uint64_t perm = 0;
    for (int p = 0; p < k; ++p) {
        uint32_t f = factorial_u32(k - 1 - p);
        uint32_t d = r / f;
        r -= d * f;
        uint32_t sh = 4u * d;
        uint64_t node = (avail >> sh) & 0xFull;
        uint64_t low = avail & ((1ull << sh) - 1ull);
        avail = low | ((avail >> 4) & ~((1ull << sh) - 1ull));
        perm |= node << (4 * p);
    }
    return perm;
}

__device__ inline int perm_at(uint64_t perm, int p) { return (int)((perm >> (4 * p)) & 0xFull); }

}  // namespace ppo
