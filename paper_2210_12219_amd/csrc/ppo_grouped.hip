// Grouped enumeration kernel for k >= 6: the hot loop of the search.
//
// One workgroup evaluates the 360 orderings that share a prefix of k-6 nodes and whose arrangement
// sigma of the six remaining nodes has one parity.  Every ordering still runs its own k DP rows; what
// the grouping buys is that the rows are *scheduled* so that all 60 working lanes of a wave, at any
// moment, handle orderings that put the same node at the current DP row.  The memory window
// [lo[node][e], e-1] is then the same for the whole wave: loop bounds are scalar, nothing is
// predicated per lane, and the only vector work left is the min/max arithmetic itself, done two
// positions at a time on packed 16-bit order codes.
//
// Data layout.  Each ordering owns a "slot": a DP row of NE = L-k+2 codes held in LDS as NP =
// ceil(NE/2) dwords (two codes per dword).  There are two row buffers (read one, write the other).
// Dword a of slot (index, class) sits at ((index*NP + a)*32 + class): the LDS bank of every access
// is the slot's class, and the lane/slot schedule (ppo_group_tables.h) gives the lanes of each
// half-wave 32 distinct banks.
//
// Row convention.  While row s is being computed, the input buffer holds
//     g_s[i] = max(D_{s-1}[i], q_{pi_{s-1},pi_s}[i-1])        at index u = i - s + 1
// and the output buffer receives g_{s+1}[e] = max(D_s[e], q_{pi_s,pi_{s+1}}[e-1]) at index
// u' = e - s, where D_s[e] = min over i in [max(lo[pi_s][e], s), e-1] of g_s[i], that is, over the
// input indices (u' - w, u'] with w = e - max(lo[pi_s][e], s).  Index 0 is always +inf.  The max
// with the next link's quotients is folded into the write, so each row is one pass.  The last row
// needs only D_{k-1}[L].
//
// Work split.  A row is 6 lane sets (one per node that can sit at that row); the output dwords of a lane
// set's row are cut into parts of kJobPairs, and a job = (lane set, part).  A wave runs two jobs per row.
// A job fetches the input dwords it needs into registers once and works through chunks of four output
// dwords; per output dword a chain of n steps over those registers (entered by a computed jump, see
// ppo_chain_asm.h), one masked step and, rarely, a longer tail from LDS.  Everything that decides control
// flow comes from a descriptor table written by the precompute kernel (WinDesc in ppo_common.h).
#include "ppo_common.h"
#include "ppo_group_tables.h"

#include <type_traits>

namespace ppo {

constexpr int kGrpWaves = 12;
constexpr int kGrpThreads = kGrpWaves * 64;
constexpr int kGrpMaxPairs = 4 * kJobPairs;          // a wave runs two jobs per row: at most four parts per lane set
constexpr int kDeep = kChainDepth;                   // chain steps available from prefetched registers
constexpr uint32_t kInf2 = kCodeInf | (kCodeInf << 16);

typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_min(uint32_t a, uint32_t b) {
    ushort2_t x = __builtin_bit_cast(ushort2_t, a), y = __builtin_bit_cast(ushort2_t, b);
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(x, y));
}
__device__ __forceinline__ uint32_t pk_max(uint32_t a, uint32_t b) {
    ushort2_t x = __builtin_bit_cast(ushort2_t, a), y = __builtin_bit_cast(ushort2_t, b);
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(x, y));
}
// Codes are positive normal binary16 patterns (or +inf), which order like the unsigned integers they
// are, so the three-input packed binary16 minimum of gfx950 does two comparisons per position.
__device__ __forceinline__ uint32_t pk_min3(uint32_t a, uint32_t b, uint32_t c) {
    half2_t x = __builtin_bit_cast(half2_t, a), y = __builtin_bit_cast(half2_t, b), z = __builtin_bit_cast(half2_t, c);
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_minimum(__builtin_elementwise_minimum(x, y), z));
}
// LDS accesses by 32-bit LDS byte address
typedef __attribute__((address_space(3))) uint32_t lds_u32_t;
__device__ __forceinline__ uint32_t lds_addr(const uint32_t* p) { return (uint32_t)(uintptr_t)(const lds_u32_t*)p; }
__device__ __forceinline__ uint32_t lds_load(uint32_t byte_addr) { return *(const lds_u32_t*)(uintptr_t)byte_addr; }
// (hi:lo) >> 16: the dword made of the upper code of lo and the lower code of hi
__device__ __forceinline__ uint32_t align16(uint32_t hi, uint32_t lo) { return __builtin_amdgcn_alignbit(hi, lo, 16); }

struct GroupedShape {
    int NE, NP, QD, QROW, QPITCH, nA, nB, nQ;
    uint32_t buf_off, buf_dwords, q_off, slot_off, d0_off, srow_off, total_bytes;  // offsets in dwords
    __host__ __device__ static GroupedShape make(int L, int k) {
        GroupedShape g;
        g.NE = L - k + 2;
        g.NP = (g.NE + 1) >> 1;
        g.QD = L / 2 + 1;
        g.QROW = 2 * g.QD + 2;
        g.QPITCH = g.QROW | 1;   // rows of the table in LDS an odd number of dwords apart: lanes that gather the same
                                 // column of different rows (their own links) then hit different banks
        const int p0 = k - 6;
        g.nA = p0 > 1 ? p0 - 1 : 0;   // links inside the prefix
        g.nB = p0 > 0 ? 6 : 0;        // links from the last prefix node to each remaining node
        g.nQ = g.nA + g.nB + 15;      // plus the links among the six remaining nodes
        g.buf_off = (uint32_t)(kDeep + 1) * 32u;   // room for the fixed-depth fetches and the masked step below dword 0
        g.buf_dwords = 12u * g.NP * 32u;
        g.q_off = g.buf_off + 2u * g.buf_dwords;
        g.slot_off = g.q_off + (uint32_t)(g.nQ * g.QPITCH);
        g.d0_off = g.slot_off + 42u * 64u / 2u;   // schedule entries are 16 bits
        g.srow_off = g.d0_off + (uint32_t)(k * align_up((size_t)g.NP, 4));
        g.total_bytes = (g.srow_off + 3u * (uint32_t)g.NP + 3u) * 4u;   // two shared rows, their linked form (one dword below it), two flags
        return g;
    }
};

bool grouped_supported(int L, int k) {
    if (k < 6) return false;
    GroupedShape g = GroupedShape::make(L, k);
    return g.NP <= kGrpMaxPairs && g.total_bytes <= 160u * 1024u;
}

// 16-bit LDS load and 32-bit LDS store by byte address
__device__ __forceinline__ uint32_t lds_load_u16(uint32_t addr) {
    return *reinterpret_cast<const __attribute__((address_space(3))) uint16_t*>((uintptr_t)addr);
}
__device__ __forceinline__ void lds_store(uint32_t addr, uint32_t v) {
    *reinterpret_cast<__attribute__((address_space(3))) uint32_t*>((uintptr_t)addr) = v;
}
// One step of a chain folds two entries into both halves of the accumulator: the lower half of `hi` and
// the upper half of `lo_`.
__device__ __forceinline__ uint32_t chain_step(uint32_t acc, uint32_t hi, uint32_t lo_) {
    asm(PPO_STEP_ASM : "+v"(acc) : "v"(hi), "v"(lo_));
    return acc;
}
// Start of an accumulator: +inf for x, and for y its first candidate (the upper half of b0) unless the
// upper half of ctrl says +inf.  init_mask holds +inf in its lower half and 0 in its upper half.
__device__ __forceinline__ uint32_t chain_init(uint32_t b0, uint32_t ctrl, uint32_t init_mask) {
    uint32_t r;
    asm("v_pk_maximum3_f16 %0, %1, %2, %3 op_sel:[0,1,0] op_sel_hi:[1,1,1]" : "=v"(r) : "v"(b0), "s"(ctrl), "v"(init_mask));
    return r;
}
// the same with ctrl in a vector register
__device__ __forceinline__ uint32_t chain_init_v(uint32_t b0, uint32_t ctrl, uint32_t init_mask) {
    uint32_t r;
    asm("v_pk_maximum3_f16 %0, %1, %2, %3 op_sel:[0,1,0] op_sel_hi:[1,1,1]" : "=v"(r) : "v"(b0), "v"(ctrl), "v"(init_mask));
    return r;
}
// packed maximum with a mask, of the lower half of v in both halves
__device__ __forceinline__ uint32_t pk_max_lower(uint32_t v, uint32_t mask) {
    uint32_t r;
    asm("v_pk_max_u16 %0, %1, %2 op_sel:[0,0] op_sel_hi:[0,1]" : "=v"(r) : "v"(v), "v"(mask));
    return r;
}
// packed maximum with a mask, of the upper half of v in both halves
__device__ __forceinline__ uint32_t pk_max_upper(uint32_t v, uint32_t mask) {
    uint32_t r;
    asm("v_pk_max_u16 %0, %1, %2 op_sel:[1,0] op_sel_hi:[1,1]" : "=v"(r) : "v"(v), "v"(mask));
    return r;
}

// MODE: kGrpPlain  every ordering runs all of its DP rows (what the headline figure counts);
//       kGrpExport the same, and beta of every ordering is written out;
//       kGrpShared the rows of the prefix, which are the same for all orderings of a group, are computed once
//                  per group, and a group is skipped when the least entry of its last shared row exceeds the
//                  best beta known so far (every later row's entries are at least that, so no ordering of
//                  the group can win or tie).  Same results; not the headline's unit of work.
enum { kGrpPlain = 0, kGrpExport = 1, kGrpShared = 2 };

template <int MODE>
__global__ __launch_bounds__(kGrpThreads) void enumerate_grouped_kernel(
    Layout y, const unsigned char* __restrict__ ws, uint32_t rank_begin, uint32_t rank_end, uint32_t group_begin,
    uint32_t group_end, uint32_t groups_per_block, unsigned long long* __restrict__ best_key,
    float* __restrict__ beta_export, unsigned long long* __restrict__ skipped_groups) {
    constexpr bool EXPORT = MODE == kGrpExport;
    extern __shared__ __align__(16) uint32_t lds[];
    const int L = y.L, k = y.k, inst = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int p0 = k - 6;
    const GroupedShape gs = GroupedShape::make(L, k);
    const int NP = gs.NP, QD = gs.QD, QROW = gs.QROW, QPITCH = gs.QPITCH, nA = gs.nA, nB = gs.nB;
    // A workgroup handles groups_per_block groups of one parity, one after the other (group_begin is even,
    // so the parity of a group is the parity of its index); the schedule table is staged once.
    const uint32_t par = blockIdx.x & 1u;
    const uint32_t group_first = group_begin + par + 2u * (blockIdx.x >> 1) * groups_per_block;

    const unsigned char* base = ws + (size_t)inst * y.stride;
    const float* __restrict__ dec = reinterpret_cast<const float*>(base + y.dec_off);
    const uint32_t* __restrict__ low = reinterpret_cast<const uint32_t*>(base + y.low_off);
    const uint32_t* __restrict__ wt = reinterpret_cast<const uint32_t*>(base + y.wt_off);
    const uint32_t* __restrict__ qa = reinterpret_cast<const uint32_t*>(base + y.qa_off);

    uint32_t* const buf0 = lds + gs.buf_off;
    uint32_t* const buf1 = buf0 + gs.buf_dwords;
    uint32_t* const qtab = lds + gs.q_off;
    uint16_t* const slotTab = reinterpret_cast<uint16_t*>(lds + gs.slot_off);

    {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(&kLaneSlot[par][0][0]);
        for (int i = tid; i < 42 * 64 / 2; i += kGrpThreads) lds[gs.slot_off + i] = src[i];
        for (int i = tid; i < (int)gs.buf_off; i += kGrpThreads) lds[i] = kInf2;
        // Every dword a chain can read has to hold two valid codes, wanted or not: an unwanted entry is dropped
        // by a maximum with +inf, and the three-input minimum that follows is a binary16 one, which a stray
        // pattern above +inf (a NaN) or with the sign bit set would win.  Below a row's first dword lie the
        // margin just filled and, for the first slot of the second buffer, the end of the first buffer.  When
        // every ordering starts at row 0, that buffer has been written by then; with shared prefix rows the
        // first row computed may read the second buffer while the first has never been written.
        if (MODE == kGrpShared) {
            const int tail = (int)gs.buf_dwords < kDeep * 32 ? (int)gs.buf_dwords : kDeep * 32;
            for (int i = tid; i < tail; i += kGrpThreads) buf0[(int)gs.buf_dwords - tail + i] = kInf2;
        }
        // the first rows of all nodes (two codes per dword), the same for every group of the instance
        const uint32_t* d0src = reinterpret_cast<const uint32_t*>(base + y.d0_off);
        for (int i = tid; i < k * y.wt_cols; i += kGrpThreads) lds[gs.d0_off + i] = d0src[i];
    }
    // best (code of beta, rank) of this lane so far: within an instance codes order like the values they stand
    // for, so the value is looked up once, at the end (the per-ordering export looks every value up)
    unsigned long long best = PPO_KEY_NONE;
    uint32_t vzero;   // a zero the compiler cannot see through, kept in a vector register
    asm volatile("v_mov_b32 %0, 0" : "=v"(vzero));
    uint32_t init_mask = kCodeInf;   // kept in a vector register: the instruction using it takes one scalar operand
    asm volatile("" : "+v"(init_mask));

    // ---- prefix of a group: positions 0..p0-1 from the Lehmer digits of its index (weights (k-1-p)!/6!);
    //      `avail` ends up holding the six remaining nodes in ascending order, four bits each
    auto decode_group = [&](uint32_t pr, uint64_t& prefix_out, uint64_t& avail_out) {
        uint64_t avail_ = 0xBA9876543210ull, prefix_ = 0;
        // The digits of pr in the factorial number system, four bits each.  Position p has k - p values, so the
        // last position of the prefix has base 7, the one before it 8, ...: taken from the least significant end
        // the divisors are the constants 7 .. 12 (a multiplication each), not (k-1-p)!/720.
        uint32_t digits = 0, rem = pr;
#pragma unroll
        for (int q = 0; q < PPO_MAX_K - 6; ++q) {
            if (q < p0) {
                const uint32_t base = 7u + (uint32_t)q;
                const uint32_t next = rem / base;
                digits |= (rem - next * base) << (4 * (p0 - 1 - q));
                rem = next;
            }
        }
        for (int p = 0; p < p0; ++p) {
            const uint32_t d = (digits >> (4 * p)) & 15u;
            const uint32_t sh = 4u * d;
            const uint64_t node = (avail_ >> sh) & 0xFull;
            const uint64_t lowbits = avail_ & ((1ull << sh) - 1ull);
            avail_ = lowbits | ((avail_ >> 4) & ~((1ull << sh) - 1ull));
            prefix_ |= node << (4 * p);
        }
        prefix_out = prefix_;
        avail_out = avail_;
    };
    // ---- the quotient rows of the links a group can cross: wave w fetches rows w, w+12, ... into registers
    //      (a group ahead of their use) and writes them to LDS when the group starts
    constexpr int kQRows = (PPO_MAX_K - 7 + 6 + 15 + kGrpWaves - 1) / kGrpWaves, kQCols = (2 * (PPO_MAX_L / 2 + 1) + 2 + 63) / 64;
    auto fetch_quotients = [&](uint64_t prefix, uint64_t avail, uint32_t (&qreg)[kQRows * kQCols]) {
        auto pnode = [=](int p) { return (int)((prefix >> (4 * p)) & 0xFull); };
        auto rnode = [=](int c) { return (int)((avail >> (4 * c)) & 0xFull); };
#pragma unroll
        for (int r = 0; r < kQRows; ++r) {
            const int row = wave + r * kGrpWaves;
            if (row < gs.nQ) {
                int a, b;
                if (row < nA) {
                    a = pnode(row); b = pnode(row + 1);
                } else if (row < nA + nB) {
                    a = pnode(p0 - 1); b = rnode(row - nA);
                } else {
                    int pi = row - nA - nB, ca = 0;
                    while (pi >= 5 - ca) { pi -= 5 - ca; ++ca; }
                    a = rnode(ca); b = rnode(ca + 1 + pi);
                }
                const uint32_t* qsrc = qa + pair_index(a, b, k) * y.qa_cols;
#pragma unroll
                for (int c = 0; c < kQCols; ++c) {
                    const int col = lane + 64 * c;
                    if (col < QROW) qreg[r * kQCols + c] = qsrc[col];
                }
            }
        }
    };
    auto store_quotients = [&](const uint32_t (&qreg)[kQRows * kQCols]) {
#pragma unroll
        for (int r = 0; r < kQRows; ++r) {
            const int row = wave + r * kGrpWaves;
            if (row < gs.nQ) {
#pragma unroll
                for (int c = 0; c < kQCols; ++c) {
                    const int col = lane + 64 * c;
                    if (col < QROW) qtab[row * QPITCH + col] = qreg[r * kQCols + c];
                }
            }
        }
    };
    uint32_t qreg[kQRows * kQCols];
    uint64_t next_prefix = 0, next_avail = 0;
    uint64_t shared_prefix_done = 0;   // prefix whose shared rows are in LDS (kGrpShared)
    if (!(MODE == kGrpShared && p0 >= 1) && group_first < group_end) {
        decode_group(group_first >> 1, next_prefix, next_avail);
        fetch_quotients(next_prefix, next_avail, qreg);
    }

    for (uint32_t gi = 0; gi < groups_per_block; ++gi) {
    const uint32_t group = group_first + 2u * gi;
    if (group >= group_end) break;
    const uint32_t pr = group >> 1;
    if (MODE == kGrpShared && p0 >= 1) {
        // no group ahead here: a group may be skipped.  Only wave 0, which decides that, needs the prefix now;
        // the other waves decode it (and everybody fetches the quotient rows) once the group is known to stay.
        if (wave == 0) decode_group(pr, next_prefix, next_avail);
    }
    if (!(MODE == kGrpShared && p0 >= 1)) {
        store_quotients(qreg);
        __syncthreads();
    }

    // column of the quotient row holding (q[e-1], q[e]) for the output dword jj of row s (e = 2jj + s)
    auto link_col = [&](int s) -> int { return (s & 1) ? (s - 1) / 2 : QD + s / 2; };
    // DP row the per-ordering work starts after: row 0, or the last row of the prefix when it is shared
    const int s_first = (MODE == kGrpShared && p0 >= 1) ? p0 - 1 : 0;
    if (MODE == kGrpShared && p0 >= 1) {
        // ---- the rows D_0 .. D_{p0-1} of the prefix, once for the group: wave 0, one output dword per lane,
        //      in the same packed, sliding layout and from the same descriptors as the rows below, but with
        //      every lane walking its own window through LDS.  Rows D_s alternate between two buffers; the
        //      input of row s is a third buffer holding max(D_{s-1}, quotients of the link s-1 -> s), with one
        //      +inf dword below it.  When only the last node of the prefix differs from the previous group's,
        //      rows 0 .. p0-2 are still there and only the last row is computed.
        uint32_t* const srow = lds + gs.srow_off;
        uint32_t* const linked = srow + 2 * NP + 1;
        uint32_t* const skip_flag = srow + 3 * NP + 1 + (gi & 1u);   // two flags in turn: one barrier per group suffices
        const uint64_t prefix = next_prefix;   // wave 0's; the other waves do not use it in this block
        auto prefix_node = [=](int p) { return (int)((prefix >> (4 * p)) & 0xFull); };
        if (wave == 0) {
            const uint32_t known = (uint32_t)(__atomic_load_n(best_key + inst, __ATOMIC_RELAXED) >> 32);
            const bool live = lane < NP;
            const uint64_t parent_mask = (1ull << (4 * (p0 - 1))) - 1ull;
            const bool same_parent = p0 >= 2 && gi > 0 && ((prefix ^ shared_prefix_done) & parent_mask) == 0ull;
            if (lane == 0) linked[-1] = kInf2;
            if (!same_parent && live) srow[lane] = lds[gs.d0_off + prefix_node(0) * y.wt_cols + lane];
            for (int s = same_parent ? p0 - 1 : 1; s <= p0 - 1; ++s) {
                const uint32_t* prev = srow + ((s - 1) & 1) * NP;
                uint32_t* out = srow + (s & 1) * NP;
                uint32_t res = kInf2;
                // quotient row s-1: the link between prefix nodes s-1 and s
                // (read from global memory: the quotient rows of this group are not staged in LDS yet)
                if (live)
                    linked[lane] = pk_max(prev[lane], qa[pair_index(prefix_node(s - 1), prefix_node(s), k) * y.qa_cols +
                                                         link_col(s - 1) + lane]);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                if (live) {
                    const uint32_t t = (uint32_t)lane % kChunkPairs;
                    const uint32_t* dp = wt + (uint32_t)(prefix_node(s) * (k - 2) * y.wt_cols * WinDesc::kWords) +
                                         (uint32_t)((s - 1) * y.wt_cols * WinDesc::kWords) +
                                         (uint32_t)(lane / kChunkPairs) * (WinDesc::kWords * kChunkPairs) + t;
                    const uint32_t ctrl = dp[0], below = dp[kChunkPairs], maskA = dp[2 * kChunkPairs], maskB = dp[3 * kChunkPairs];
                    const uint32_t n = WinDesc::steps(below, t);
                    const uint32_t* own = linked + lane;   // the input dword at the output's own index
                    uint32_t acc = chain_init_v(own[0], ctrl, init_mask);
                    {
                        // four steps per round, their LDS reads issued together
                        uint32_t cur = own[0], i = 1;
                        for (; i + 3u <= n; i += 4u) {
                            const uint32_t b1 = own[-(int)i], b2 = own[-(int)(i + 1)], b3 = own[-(int)(i + 2)], b4 = own[-(int)(i + 3)];
                            acc = chain_step(acc, cur, b1);
                            acc = chain_step(acc, b1, b2);
                            acc = chain_step(acc, b2, b3);
                            acc = chain_step(acc, b3, b4);
                            cur = b4;
                        }
                        for (; i <= n; ++i) {
                            const uint32_t b1 = own[-(int)i];
                            acc = chain_step(acc, cur, b1);
                            cur = b1;
                        }
                    }
                    acc = pk_min3(acc, pk_max_lower(own[-(int)n], maskA), pk_max_upper(own[-(int)(n + 1)], maskB));
                    if (ctrl & WinDesc::kFold) {
                        const uint32_t cnt = WinDesc::fold_dwords(ctrl);
                        uint32_t tacc = kInf2;
                        for (uint32_t i = 0; i < cnt; ++i) tacc = pk_min(tacc, own[-(int)(n + 1 + i)]);
                        tacc = pk_min(tacc, pk_max(own[-(int)(n + 1 + cnt)], (ctrl & WinDesc::kWxEven) ? kCodeInf : 0u));
                        tacc = pk_min(tacc, align16(tacc, tacc));
                        acc = pk_min(acc, pk_max(tacc, kCodeInf << 16));
                    }
                    res = acc;
                }
                if (live) out[lane] = res;
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
            // least entry of the last shared row: a lower bound on beta of every ordering of the group
            uint32_t lb = kCodeInf;
            if (live) {
                const uint32_t v = srow[(s_first & 1) * NP + lane];
                lb = (v & 0xFFFFu) < (v >> 16) ? (v & 0xFFFFu) : (v >> 16);
            }
            for (int off = 32; off >= 1; off >>= 1) {
                const uint32_t o = (uint32_t)__shfl_xor((int)lb, off, 64);
                lb = o < lb ? o : lb;
            }
            const uint32_t lb_bits = lb >= kCodeInf ? kInfBits : __float_as_uint(dec[lb - kCodeZero]);
            if (lane == 0) {
                *skip_flag = lb_bits > known ? 1u : 0u;
                if (lb_bits > known && skipped_groups) atomicAdd(skipped_groups + inst, 1ull);
            }
        }
        shared_prefix_done = prefix;
        __syncthreads();
        if (*skip_flag) continue;
        if (wave != 0) decode_group(pr, next_prefix, next_avail);
        fetch_quotients(next_prefix, next_avail, qreg);
        store_quotients(qreg);
        __syncthreads();
    }
    const uint64_t avail = next_avail, prefix = next_prefix;
    auto rest_node = [=](int c) { return (int)((avail >> (4 * c)) & 0xFull); };
    // node at DP row s for the lane set of remaining-node index c
    auto row_node = [=](int s, int c) {
        const uint64_t packed = s < p0 ? prefix : avail;
        const int idx = s < p0 ? s : c;
        return (int)((packed >> (4 * idx)) & 0xFull);
    };

    // quotient row used when row s is written (the link between the nodes of rows s and s+1), from the
    // lane's schedule entry
    auto link_row = [&](int s, uint32_t ent) -> int {
        if (s + 1 < p0) return s;
        if (s + 1 == p0) return nA + (int)((ent >> 13) & 7u);
        return nA + nB + (int)((ent >> 9) & 15u);
    };
    auto slot_dword = [&](uint32_t ent) -> uint32_t {
        return __umul24((ent >> 5) & 15u, (uint32_t)(NP * 32)) + (ent & 31u);
    };

    // what the last row needs from global memory is requested now, a whole group's work ahead of its use
    uint32_t last_ent = 0, last_perm = 0, last_lo = 0;
    if (wave < 6) {
        last_ent = slotTab[(5 * 6 + wave) * 64 + lane];
        last_perm = (&kSlotPerm[par][0] + vzero)[last_ent & 511u];
        last_lo = (low + vzero)[rest_node(wave) * (L + 1) + L];
    }

    // ---- row 0: g_1[i] = max(D_0[i], q_{pi_0,pi_1}[i-1]) at index i, D_0[i] = 0 if layers [0,i) fit node pi_0.
    //      With a shared prefix: the same for its last row s_first, from the row computed above.
    {
        const int c = wave % 6, half = wave / 6;
        const int set = p0 > 0 ? 36 + c : c;
        const uint32_t ent = slotTab[set * 64 + lane];
        uint32_t* out = ((s_first & 1) ? buf1 : buf0) + slot_dword(ent);
        const uint32_t* qrow = qtab + link_row(s_first, ent) * QPITCH + link_col(s_first);
        const int j0 = half * ((NP + 1) / 2), j1 = half ? NP : (NP + 1) / 2;
        // the initial row of the node, or the last row of the shared prefix
        const uint32_t* first_row = (MODE == kGrpShared && p0 >= 1) ? lds + gs.srow_off + (s_first & 1) * NP
                                                                    : lds + gs.d0_off + row_node(0, c) * y.wt_cols;
        int jj = j0;
        // four dwords at a time, all eight reads before the first write (the compiler cannot tell that the
        // writes leave the tables alone and would otherwise wait for each read in turn)
        for (; jj + 4 <= j1; jj += 4) {
            const uint32_t e0 = first_row[jj], e1 = first_row[jj + 1], e2 = first_row[jj + 2], e3 = first_row[jj + 3];
            const uint32_t q0 = qrow[jj], q1 = qrow[jj + 1], q2 = qrow[jj + 2], q3 = qrow[jj + 3];
            out[jj * 32] = pk_max(e0, q0);
            out[(jj + 1) * 32] = pk_max(e1, q1);
            out[(jj + 2) * 32] = pk_max(e2, q2);
            out[(jj + 3) * 32] = pk_max(e3, q3);
        }
        for (; jj < j1; ++jj) out[jj * 32] = pk_max(first_row[jj], qrow[jj]);
    }

    // ---- rows 1 .. k-2.  The output dwords of a lane set's row are cut into parts of kJobPairs dwords; a job
    //      = (lane set, part).  With the parts numbered from the top, a wave runs part wave/6 and the part two
    //      below it (the top part is short and the bottom one has short windows, so that the two sums come out
    //      about even), of lane sets wave%6 and (wave+3)%6, at most two jobs in a row of the DP.  A job fetches
    //      the input dwords from (first - kDeep) to (first + kJobPairs - 1) of the lane's row into registers, once, and then
    //      works through its chunks of four output dwords; each chunk's descriptors and next-link quotients
    //      are requested one chunk ahead.
    constexpr int kNB = kJobPairs + kDeep;
    struct ChunkIn {
        uint4 ctrl, below, maskA, maskB;   // descriptors of the four outputs, word by word
        uint32_t qv[kChunkPairs];          // quotients of the next link for the four outputs
    };
    struct Job {
        uint32_t ent;        // the lane's schedule entry for the job's lane set
        uint32_t fbase;      // LDS byte address of the first input dword fetched
        uint32_t out_addr;   // LDS byte address of the first output dword
        uint32_t qa_addr;    // LDS byte address of the quotient dword of the first output
        uint32_t desc_base;  // dword offset of the job's first chunk in the descriptor table (wave-uniform)
    };
    const uint32_t buf0_addr = lds_addr(buf0), buf1_addr = lds_addr(buf1), qtab_addr = lds_addr(qtab);
    const uint32_t desc_node_stride = (uint32_t)((k - 2) * y.wt_cols * WinDesc::kWords);
    uint32_t ent_lane = lds_addr(lds + gs.slot_off) + 2u * (uint32_t)lane;   // the lane's column of the schedule table
    asm volatile("" : "+v"(ent_lane));
    const int nparts = (NP + kJobPairs - 1) / kJobPairs;
    // the wave's two jobs: lane set and first output dword
    const int job_part[2] = {nparts - 1 - wave / 6, nparts - 3 - wave / 6};
    const bool job_valid[2] = {job_part[0] >= 0, job_part[1] >= 0};
    int job_set[2], job_first[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        job_set[j] = (wave + 3 * j) % 6;
        job_first[j] = (job_valid[j] ? job_part[j] : 0) * kJobPairs;
    }
    // Descriptors and quotients of chunk c of job j in row s.  The descriptors are the same for every lane,
    // but they are fetched with vector loads on purpose: scalar loads complete under the same counter as LDS
    // reads, out of order, so one in flight would make every wait for an LDS result a wait for everything.
    // (a wave's second job is never the row's last part: all its chunks have outputs)
    auto chunk_live = [&](int j, int c) { return job_valid[j] && (j == 1 || job_first[j] + c * kChunkPairs < NP); };
    auto request_chunk = [&](int c, const Job& J, ChunkIn& D) {
        const uint4* dp = reinterpret_cast<const uint4*>(wt + J.desc_base + (uint32_t)(c * (WinDesc::kWords * kChunkPairs))) + vzero;
        // ctrl is used first: requested last, its arrival means that all four words are there
        D.below = dp[1];
        D.maskA = dp[2];
        D.maskB = dp[3];
        D.ctrl = dp[0];
#pragma unroll
        for (int t = 0; t < kChunkPairs; ++t) D.qv[t] = lds_load(J.qa_addr + (uint32_t)((c * kChunkPairs + t) * 4));
    };
    // the parts of a job's addresses that do not depend on the buffers' roles: descriptors of (node, row, part),
    // and the quotient row from the schedule entry
    // What a job's set-up needs and only the group, the row and the job decide, for all rows at once: lane
    // 2 (s - 1) + j works out the values of job j in row s (about thirty scalar instructions per job and row
    // otherwise), and the row loop picks them with a lane read.
    //   job_desc: dword offset of the job's first chunk in the descriptor table
    //   job_link: the row of the quotient table is a base (bits 0-7) plus the field of the schedule entry
    //             at a shift (bits 8-15) under a mask (bits 16-23)
    //   job_misc: byte offset of the job's row in the schedule table (bits 0-15); byte offset of the quotient
    //             dword of the job's first output within a row of the quotient table (bits 16-31)
    uint32_t job_desc, job_link, job_misc;
    {
        const int s_ = (lane >> 1) + 1, j_ = lane & 1;
        const int set_ = j_ ? job_set[1] : job_set[0], first_ = j_ ? job_first[1] : job_first[0];
        const uint64_t packed = s_ < p0 ? prefix : avail;
        const int idx = (s_ < p0 ? s_ : set_) & 15;
        const uint32_t node = (uint32_t)((packed >> (4 * idx)) & 0xFull);
        job_desc = node * desc_node_stride + (uint32_t)((s_ - 1) * y.wt_cols * WinDesc::kWords) +
                   (uint32_t)((first_ / kChunkPairs) * (WinDesc::kWords * kChunkPairs));
        const uint32_t lr_base = s_ + 1 < p0 ? (uint32_t)s_ : s_ + 1 == p0 ? (uint32_t)nA : (uint32_t)(nA + nB);
        const uint32_t lr_shift = s_ + 1 == p0 ? 13u : 9u, lr_mask = s_ + 1 < p0 ? 0u : s_ + 1 == p0 ? 7u : 15u;
        job_link = (lr_base & 0xFFu) | (lr_shift << 8) | (lr_mask << 16);
        // the schedule table holds the six lane sets of every row from p0 on, then (from 36) those of the prefix rows
        const uint32_t ent_row = (uint32_t)((s_ < p0 ? 36 : (s_ - p0) * 6) + set_) * 128u;
        const uint32_t qcol = 4u * (uint32_t)(((s_ & 1) ? (s_ - 1) / 2 : QD + s_ / 2) + first_);
        job_misc = (ent_row & 0xFFFFu) | (qcol << 16);
    }
    auto load_job_ent = [&](int s, int j) -> uint32_t {
        const uint32_t misc = (uint32_t)__builtin_amdgcn_readlane((int)job_misc, 2 * (s - 1) + j);
        return (uint32_t)lds_load_u16(ent_lane + (misc & 0xFFFFu));
    };
    auto job_quotients = [&](int s, int j, Job& J) {
        const int r = 2 * (s - 1) + j;
        J.desc_base = (uint32_t)__builtin_amdgcn_readlane((int)job_desc, r);
        const uint32_t link = (uint32_t)__builtin_amdgcn_readlane((int)job_link, r);
        const uint32_t lr = (link & 0xFFu) + ((J.ent >> ((link >> 8) & 0xFFu)) & (link >> 16));
        const uint32_t misc = (uint32_t)__builtin_amdgcn_readlane((int)job_misc, r);
        J.qa_addr = __umul24(lr, (uint32_t)(QPITCH * 4)) + (qtab_addr + (misc >> 16));
    };

    // addresses of job j in row s (the buffers swap roles from row to row)
    auto job_addresses = [&](int s, int j, Job& J) {
        const uint32_t slot_b = slot_dword(J.ent) * 4u;
        J.out_addr = ((s & 1) ? buf1_addr : buf0_addr) + (uint32_t)(job_first[j] * 128) + slot_b;
        J.fbase = ((s & 1) ? buf0_addr : buf1_addr) + (uint32_t)((job_first[j] - kDeep) * 128) + slot_b;
        asm volatile("" : "+v"(J.fbase));
    };

    // what the first chunk of the next row needs and does not depend on the row before it is requested
    // ahead of the barrier that ends that row
    Job J0, J1;
    ChunkIn DA, DB;
    J0.ent = load_job_ent(s_first + 1, 0);
    J1.ent = load_job_ent(s_first + 1, 1);
    job_quotients(s_first + 1, 0, J0);
    job_addresses(s_first + 1, 0, J0);
    request_chunk(0, J0, DA);
    __syncthreads();

    for (int s = s_first + 1; s <= k - 2; ++s) {
        // the next group's quotient rows are requested one row of the DP before this group ends
        if (!(MODE == kGrpShared && p0 >= 1) && s == k - 2 && gi + 1 < groups_per_block && group + 2u < group_end) {
            decode_group((group + 2u) >> 1, next_prefix, next_avail);
            fetch_quotients(next_prefix, next_avail, qreg);
        }
        uint32_t B0[kNB], B1[kNB];
        // Fetch of a job's input dwords [from, to).  Chunk c reads the dwords 4c .. 4c + kDeep + 3: the first
        // chunk's are fetched before the job starts and four more during each of its first two chunks.
        auto fetch = [&](const Job& J, uint32_t (&B)[kNB], auto from_tag, auto to_tag) {
#pragma unroll
            for (int i = decltype(from_tag)::value; i < decltype(to_tag)::value; ++i) B[i] = lds_load(J.fbase + (uint32_t)i * 128u);
        };

        // chunk c of a job: B holds the job's input dwords, D the chunk's descriptors and quotients
        // b(t, i): the input dword i below the index of output t of the chunk (i = 0: the dword at that index)
#define PPO_B(t, i) B[c * kChunkPairs + (t) + kDeep - (i)]
        auto run_chunk = [&](int j, auto c_tag, const Job& J, const uint32_t (&B)[kNB], const ChunkIn& X) {
            constexpr int c = decltype(c_tag)::value;
            const int np = NP - (job_first[j] + c * kChunkPairs);   // outputs beyond the row end are not stored
            const uint32_t cbase = J.fbase + (uint32_t)(c * kChunkPairs * 128);   // first dword fetched for this chunk
            const uint32_t ctrl[kChunkPairs] = {
                (uint32_t)__builtin_amdgcn_readfirstlane(X.ctrl.x), (uint32_t)__builtin_amdgcn_readfirstlane(X.ctrl.y),
                (uint32_t)__builtin_amdgcn_readfirstlane(X.ctrl.z), (uint32_t)__builtin_amdgcn_readfirstlane(X.ctrl.w)};
            const uint32_t below[kChunkPairs] = {X.below.x, X.below.y, X.below.z, X.below.w};
            const uint32_t maskA[kChunkPairs] = {X.maskA.x, X.maskA.y, X.maskA.z, X.maskA.w};
            const uint32_t maskB[kChunkPairs] = {X.maskB.x, X.maskB.y, X.maskB.z, X.maskB.w};
            // the two dwords of the masked step, n and n+1 below the output's index, wherever they are
            uint32_t bn[kChunkPairs], bn1[kChunkPairs];
#pragma unroll
            for (int t = 0; t < kChunkPairs; ++t) {
                const uint32_t a = cbase + below[t];
                bn1[t] = lds_load(a);
                bn[t] = lds_load(a + 128u);
            }
            uint32_t acc[kChunkPairs];
#pragma unroll
            for (int t = 0; t < kChunkPairs; ++t) {
                // y's first candidate is the upper half of the dword at the output's own index: the block starts
                // the accumulator from it, then runs steps min(n, depth) .. 1 from registers (see
                // ppo_chain_asm.h); chunk c has depth 16 + 4c
                uint32_t a;
#define PPO_B4(t, i) "v"(PPO_B(t, i)), "v"(PPO_B(t, i + 1)), "v"(PPO_B(t, i + 2)), "v"(PPO_B(t, i + 3))
                if constexpr (c == 0) {
                    asm volatile(PPO_CHAIN_ASM_0
                                 : "=&v"(a)
                                 : "s"(ctrl[t] & WinDesc::kJumpMask), PPO_B4(t, 0), PPO_B4(t, 4), PPO_B4(t, 8),
                                   PPO_B4(t, 12), "v"(PPO_B(t, 16)), "s"(ctrl[t]), "v"(init_mask)
                                 : "s98", "s99", "scc");
                } else if constexpr (c == 1) {
                    asm volatile(PPO_CHAIN_ASM_1
                                 : "=&v"(a)
                                 : "s"(ctrl[t] & WinDesc::kJumpMask), PPO_B4(t, 0), PPO_B4(t, 4), PPO_B4(t, 8),
                                   PPO_B4(t, 12), PPO_B4(t, 16), "v"(PPO_B(t, 20)), "s"(ctrl[t]), "v"(init_mask)
                                 : "s98", "s99", "scc");
                } else {
                    asm volatile(PPO_CHAIN_ASM_2
                                 : "=&v"(a)
                                 : "s"(ctrl[t] & WinDesc::kJumpMask), PPO_B4(t, 0), PPO_B4(t, 4), PPO_B4(t, 8),
                                   PPO_B4(t, 12), PPO_B4(t, 16), PPO_B4(t, 20), "v"(PPO_B(t, 24)), "s"(ctrl[t]),
                                   "v"(init_mask)
                                 : "s98", "s99", "scc");
                }
#undef PPO_B4
                // the masked step: entry 2n (lower half of dword n) for both, entry 2n+1 (upper half of dword n+1) for x
                acc[t] = pk_min3(a, pk_max_lower(bn[t], maskA[t]), pk_max_upper(bn1[t], maskB[t]));
            }
            // the rare rest: chains deeper than the registers and entries only x wants
            if (ctrl[0] & WinDesc::kChunkRare) {
#pragma unroll
                for (int t = 0; t < kChunkPairs; ++t) {
                    if ((ctrl[t] & (WinDesc::kDeepChain | WinDesc::kFold)) == 0u) continue;
                    if (ctrl[t] & WinDesc::kDeepChain) {
                        // the rest of a long chain walks further down the row
                        const uint32_t n = WinDesc::steps((uint32_t)__builtin_amdgcn_readfirstlane(below[t]), (uint32_t)t);
                        uint32_t a = acc[t];
                        // the deepest dword in registers, chain_depth(c) below the output's index, is the
                        // t-th of the job's fetch
                        uint32_t pa = J.fbase + (uint32_t)t * 128u;
                        uint32_t cur = PPO_B(t, chain_depth(c));
                        uint32_t m = n - (uint32_t)chain_depth(c);
                        while (m >= 4u) {
                            pa -= 512u;
                            const uint32_t b1 = lds_load(pa + 384u), b2 = lds_load(pa + 256u),
                                           b3 = lds_load(pa + 128u), b4 = lds_load(pa);
                            a = chain_step(a, cur, b1);
                            a = chain_step(a, b1, b2);
                            a = chain_step(a, b2, b3);
                            a = chain_step(a, b3, b4);
                            cur = b4;
                            m -= 4u;
                        }
                        while (m >= 1u) {
                            pa -= 128u;
                            const uint32_t b1 = lds_load(pa);
                            a = chain_step(a, cur, b1);
                            cur = b1;
                            m -= 1u;
                        }
                        acc[t] = a;
                    }
                    if (ctrl[t] & WinDesc::kFold) {
                        // x wants entries 2n+2 .. wx-1 as well: fold the dwords n+1 .. wx/2 below the output
                        // (what else they hold lies inside x's window, except the lower half of the last one
                        // when wx is even), then across the two halves, into x's half only.  The last dword is
                        // read whatever the count (it is dword n+1 again if there is no other), so that the
                        // common short cases run straight through.
                        const uint32_t cnt = WinDesc::fold_dwords(ctrl[t]);
                        const uint32_t last_mask = (ctrl[t] & WinDesc::kWxEven) ? kCodeInf : 0u;
                        const uint32_t first = cbase + below[t];   // dword n+1
                        const uint32_t last = lds_load(first - cnt * 128u);
                        uint32_t tacc = cnt == 0u ? kInf2 : bn1[t];
                        for (uint32_t i = 1; i < cnt; ++i) tacc = pk_min(tacc, lds_load(first - i * 128u));
                        // last dword under its mask, both halves folded into one, into x's half of the result.  One
                        // block: between packed instructions written one by one the compiler puts a wait state
                        // each (it takes their high-half operand selectors for a partial write of the result),
                        // which these full-width results do not need.
                        uint32_t t1, t2;
                        asm("v_pk_max_u16 %1, %3, %4\n"
                            "v_pk_min_u16 %1, %5, %1\n"
                            "v_alignbit_b32 %2, %1, %1, 16\n"
                            "v_pk_min_u16 %1, %1, %2\n"
                            "v_pk_max_u16 %1, %1, %6\n"
                            "v_pk_min_u16 %0, %0, %1"
                            : "+v"(acc[t]), "=&v"(t1), "=&v"(t2)
                            : "v"(last), "s"(last_mask), "v"(tacc), "s"((uint32_t)(kCodeInf << 16)));
                    }
                }
            }
            const uint32_t obase = J.out_addr + (uint32_t)(c * kChunkPairs * 128);
            // only a row's last part can be short, and that part is always a wave's first job: the second job's
            // chunks are whole (j is a constant at every place this is expanded)
            if (j == 1 || np >= kChunkPairs) {
#pragma unroll
                for (int t = 0; t < kChunkPairs; ++t) lds_store(obase + (uint32_t)t * 128u, pk_max(acc[t], X.qv[t]));
            } else {
#pragma unroll
                for (int t = 0; t < kChunkPairs; ++t)
                    if (t < np) lds_store(obase + (uint32_t)t * 128u, pk_max(acc[t], X.qv[t]));
                // keeps the compiler from sinking "the last store" of both branches into one block behind a
                // chain of selects (which the full chunk, the common case, would then pay for as well)
                asm volatile("" ::: "memory");
            }
        };
#undef PPO_B

        // The six chunks in turn, each requesting what the next one needs before it starts.  The requests are
        // unconditional (a dead chunk has null descriptors and its fetches stay inside LDS), so that the waits
        // the compiler places count exactly the requests made since.
        using C0 = std::integral_constant<int, 0>;
        using C1 = std::integral_constant<int, 1>;
        using C2 = std::integral_constant<int, 2>;
        using F0 = std::integral_constant<int, 0>;
        using F1 = std::integral_constant<int, kDeep + kChunkPairs>;
        using F2 = std::integral_constant<int, kDeep + 2 * kChunkPairs>;
        using F3 = std::integral_constant<int, kDeep + 3 * kChunkPairs>;
        static_assert(kJobChunks == 3, "the sequence below is written for three chunks per job");
        fetch(J0, B0, F0{}, F1{});
        request_chunk(1, J0, DB);
        fetch(J0, B0, F1{}, F2{});
        if (chunk_live(0, 0)) run_chunk(0, C0{}, J0, B0, DA);
        request_chunk(2, J0, DA);
        fetch(J0, B0, F2{}, F3{});
        job_quotients(s, 1, J1);
        job_addresses(s, 1, J1);
        if (chunk_live(0, 1)) run_chunk(0, C1{}, J0, B0, DB);
        request_chunk(0, J1, DB);
        fetch(J1, B1, F0{}, F1{});
        if (chunk_live(0, 2)) run_chunk(0, C2{}, J0, B0, DA);
        request_chunk(1, J1, DA);
        fetch(J1, B1, F1{}, F2{});
        if (chunk_live(1, 0)) run_chunk(1, C0{}, J1, B1, DB);
        request_chunk(2, J1, DB);
        fetch(J1, B1, F2{}, F3{});
        if (s + 1 <= k - 2) {
            J0.ent = load_job_ent(s + 1, 0);
            J1.ent = load_job_ent(s + 1, 1);
        }
        if (chunk_live(1, 1)) run_chunk(1, C1{}, J1, B1, DA);
        if (chunk_live(1, 2)) run_chunk(1, C2{}, J1, B1, DB);
        if (s + 1 <= k - 2) {
            job_quotients(s + 1, 0, J0);
            job_addresses(s + 1, 0, J0);
            request_chunk(0, J0, DA);
        }
        __syncthreads();
    }

    // ---- row k-1: only D_{k-1}[L] is needed; then the key of each ordering, folded into the lane's best
    if (wave < 6) {
        const int sl_ = k - 1;
        const uint32_t* in = (sl_ & 1) ? buf0 : buf1;
        const uint32_t ent = last_ent;
        const uint32_t slot_dw = slot_dword(ent);
        const uint32_t perm = last_perm;
        const bool active = (perm >> 31) != 0u;   // idle lanes sit on the two unused bank columns
        const int l = (int)__builtin_amdgcn_readfirstlane(last_lo);
        const int w = L - (l > sl_ ? l : sl_);
        // input indices (NE-1-w, NE-1]
        const int ulo = gs.NE - w, uhi = gs.NE - 1;
        uint32_t acc = kInf2;
        for (int jj = uhi >> 1; jj >= (ulo >> 1) && w > 0; --jj) {
            const uint32_t mask = (2 * jj >= ulo ? 0u : kCodeInf) | (2 * jj + 1 <= uhi ? 0u : (kCodeInf << 16));
            acc = pk_min(acc, pk_max(in[slot_dw + jj * 32], mask));
        }
        const uint32_t cx = acc & 0xFFFFu, cy = acc >> 16;
        const uint32_t code = cx < cy ? cx : cy;
        const uint32_t r = pr * 720u + ((perm >> 18) & 1023u);
        if (active && r >= rank_begin && r < rank_end) {
            if (EXPORT) {
                const uint32_t bits = code >= kCodeInf ? kInfBits : __float_as_uint(dec[code - kCodeZero]);
                beta_export[r - rank_begin] = __uint_as_float(bits);
            }
            const unsigned long long key = ((unsigned long long)code << 32) | r;
            best = key < best ? key : best;
        }
    }
    __syncthreads();   // the next group's first row overwrites the buffer this row reads
    }  // groups of this workgroup

    if (!EXPORT) {
        for (int off = 32; off >= 1; off >>= 1) {
            const unsigned long long o = __shfl_xor(best, off, 64);
            best = o < best ? o : best;
        }
        if (lane == 0 && best != PPO_KEY_NONE) {
            const uint32_t code = (uint32_t)(best >> 32);
            const uint32_t bits = code >= kCodeInf ? kInfBits : __float_as_uint(dec[code - kCodeZero]);
            const unsigned long long key = ((unsigned long long)bits << 32) | (best & 0xFFFFFFFFull);
            if (key < best_key[inst]) atomicMin(best_key + inst, key);
        }
    }
}

template <int MODE>
static hipError_t launch_mode(const dim3& grid, const GroupedShape& gs, hipStream_t stream, const Layout& y, const void* ws,
                              uint32_t rank_begin, uint32_t rank_end, uint32_t gbeg, uint32_t gend, uint32_t gpb,
                              uint64_t* best_key, float* beta_export, uint64_t* skipped_groups) {
    static std::atomic<uint64_t> lds_allowed{0};
    hipError_t e = allow_full_lds(reinterpret_cast<const void*>(&enumerate_grouped_kernel<MODE>), lds_allowed);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(enumerate_grouped_kernel<MODE>, grid, dim3(kGrpThreads), gs.total_bytes, stream, y,
                       static_cast<const unsigned char*>(ws), rank_begin, rank_end, gbeg, gend, gpb,
                       reinterpret_cast<unsigned long long*>(best_key), beta_export,
                       reinterpret_cast<unsigned long long*>(skipped_groups));
    return hipGetLastError();
}

// shared_prefix: compute the rows of a group's prefix once and skip groups that cannot win (see kGrpShared);
// skipped_groups (device, one counter per instance, may be null) is incremented per skipped group
hipError_t launch_enumerate_grouped(const Layout& y, int n_inst, const void* ws, uint32_t rank_begin,
                                    uint32_t rank_end, uint64_t* best_key, float* beta_export, bool shared_prefix,
                                    uint64_t* skipped_groups, hipStream_t stream) {
    if (rank_end <= rank_begin || n_inst == 0) return hipSuccess;
    const GroupedShape gs = GroupedShape::make(y.L, y.k);
    const uint32_t gbeg = 2u * (rank_begin / 720u), gend = 2u * ((rank_end + 719u) / 720u);
    // groups per workgroup: enough workgroups to fill the chip several times over, else as many as 8; 16 where
    // that leaves no ragged last workgroup and still many workgroups per compute unit (a workgroup's start-up
    // is then paid half as often).  The bounded mode stays at 8: its bound tightens between workgroups; so
    // does the mode that exports beta per ordering, which never runs at such sizes.
    const uint32_t pairs = (gend - gbeg) / 2;
    uint32_t gpb = 8;
    while (gpb > 1 && (uint64_t)(pairs / gpb) * 2u * (uint64_t)n_inst < 4096u) gpb >>= 1;
    if (!shared_prefix && !beta_export && pairs % 16u == 0 && (uint64_t)(pairs / 16u) * 2u * (uint64_t)n_inst >= 16384u) gpb = 16;
    const dim3 grid(2u * ((pairs + gpb - 1) / gpb), n_inst);
    if (beta_export)
        return launch_mode<kGrpExport>(grid, gs, stream, y, ws, rank_begin, rank_end, gbeg, gend, gpb, best_key, beta_export, nullptr);
    if (shared_prefix)
        return launch_mode<kGrpShared>(grid, gs, stream, y, ws, rank_begin, rank_end, gbeg, gend, gpb, best_key, nullptr, skipped_groups);
    return launch_mode<kGrpPlain>(grid, gs, stream, y, ws, rank_begin, rank_end, gbeg, gend, gpb, best_key, nullptr, nullptr);
}

}  // namespace ppo
