// Grouped enumeration kernel for k >= 6: the hot loop of the search.
//
// One workgroup evaluates the 360 orderings that share a prefix of k-6 nodes and whose arrangement
// sigma of the six remaining nodes has one parity.  Every ordering still runs its own k DP rows; what
// the grouping buys is that the rows are *scheduled* so that all 60 lanes of a wave, at any moment,
// work on orderings that put the same node at the current DP row.  The memory window
// [lo[node][e], e-1] is then the same for the whole wave: loop bounds are scalar, nothing is
// predicated per lane, and the only vector work left is the min/max arithmetic itself, done two
// positions at a time on packed 16-bit order codes.
//
// Data layout.  Each ordering owns a "slot": a DP row of NE = L-k+2 codes held in LDS as NP =
// ceil(NE/2) dwords (two codes per dword).  There are two row buffers (read one, write the other).
// Dword a of slot (index, class) sits at ((index*NP + a)*32 + class): the LDS bank of every access
// is the slot's class, and the lane/slot schedule (ppo_group_tables.h) gives the lanes of each
// half-wave 30 distinct classes.
//
// Row convention.  While row s is being computed, the input buffer holds
//     g_s[i] = max(D_{s-1}[i], q_{pi_{s-1},pi_s}[i-1])        at index u = i - s + 1
// and the output buffer receives g_{s+1}[e] = max(D_s[e], q_{pi_s,pi_{s+1}}[e-1]) at index
// u' = e - s, where D_s[e] = min over i in [max(lo[pi_s][e], s), e-1] of g_s[i], that is, over the
// input indices (u' - w, u'] with w = e - max(lo[pi_s][e], s).  Index 0 is always +inf.  The max
// with the next link's quotients is folded into the write, so each row is one pass.  The last row
// needs only D_{k-1}[L].
#include "ppo_common.h"
#include "ppo_group_tables.h"

namespace ppo {

constexpr int kGrpWaves = 12;
constexpr int kGrpThreads = kGrpWaves * 64;
constexpr int kChunkPairs = 4;                      // target dwords (pairs of positions) per task
constexpr int kGrpMaxPairs = 6 * 2 * kChunkPairs;   // six rounds of two chunks cover at most 48 dwords
constexpr uint32_t kInf2 = kCodeInf | (kCodeInf << 16);

typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));

__device__ inline uint32_t pk_min(uint32_t a, uint32_t b) {
    ushort2_t x = __builtin_bit_cast(ushort2_t, a), y = __builtin_bit_cast(ushort2_t, b);
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(x, y));
}
__device__ inline uint32_t pk_max(uint32_t a, uint32_t b) {
    ushort2_t x = __builtin_bit_cast(ushort2_t, a), y = __builtin_bit_cast(ushort2_t, b);
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(x, y));
}
// Codes are positive normal binary16 patterns (or +inf), which order like the unsigned integers they
// are, so the three-input packed binary16 minimum of gfx950 can do two comparisons per position.
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
__device__ inline uint32_t pk_min3(uint32_t a, uint32_t b, uint32_t c) {
    half2_t x = __builtin_bit_cast(half2_t, a), y = __builtin_bit_cast(half2_t, b), z = __builtin_bit_cast(half2_t, c);
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_minimum(__builtin_elementwise_minimum(x, y), z));
}
// (hi:lo) >> 16: the dword made of the upper code of lo and the lower code of hi
__device__ inline uint32_t align16(uint32_t hi, uint32_t lo) { return __builtin_amdgcn_alignbit(hi, lo, 16); }

struct GroupedShape {
    int NE, NP, QD, QROW, nA, nB, nQ;
    uint32_t buf_dwords, q_off, slot_off, perm_off, total_bytes;  // offsets in dwords
    __host__ __device__ static GroupedShape make(int L, int k) {
        GroupedShape g;
        g.NE = L - k + 2;
        g.NP = (g.NE + 1) >> 1;
        g.QD = L / 2 + 1;
        g.QROW = 2 * g.QD + 2;
        const int p0 = k - 6;
        g.nA = p0 > 1 ? p0 - 1 : 0;   // links inside the prefix
        g.nB = p0 > 0 ? 6 : 0;        // links from the last prefix node to each remaining node
        g.nQ = g.nA + g.nB + 15;      // plus the links among the six remaining nodes
        g.buf_dwords = 12u * g.NP * 32u;
        g.q_off = 2u * g.buf_dwords;
        g.slot_off = g.q_off + (uint32_t)(g.nQ * g.QROW);
        g.perm_off = g.slot_off + 42u * 64u / 2u;
        g.total_bytes = (g.perm_off + 384u) * 4u;
        return g;
    }
};

bool grouped_supported(int L, int k) {
    if (k < 6) return false;
    GroupedShape g = GroupedShape::make(L, k);
    return g.NP <= kGrpMaxPairs && g.total_bytes <= 160u * 1024u;
}

template <bool EXPORT>
__global__ __launch_bounds__(kGrpThreads) void enumerate_grouped_kernel(
    Layout y, const unsigned char* __restrict__ ws, uint32_t rank_begin, uint32_t rank_end, uint32_t group_begin,
    unsigned long long* __restrict__ best_key, float* __restrict__ beta_export) {
    extern __shared__ __align__(16) uint32_t lds[];
    const int L = y.L, k = y.k, inst = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int p0 = k - 6;
    const GroupedShape gs = GroupedShape::make(L, k);
    const int NP = gs.NP, QD = gs.QD, QROW = gs.QROW, nA = gs.nA, nB = gs.nB;
    const uint32_t group = group_begin + blockIdx.x;
    const uint32_t par = group & 1u, pr = group >> 1;

    const unsigned char* base = ws + (size_t)inst * y.stride;
    const uint16_t* __restrict__ qc = reinterpret_cast<const uint16_t*>(base + y.qc_off);
    const float* __restrict__ dec = reinterpret_cast<const float*>(base + y.dec_off);
    const uint32_t* __restrict__ low = reinterpret_cast<const uint32_t*>(base + y.low_off);

    uint32_t* const buf0 = lds;
    uint32_t* const buf1 = lds + gs.buf_dwords;
    uint32_t* const qtab = lds + gs.q_off;
    uint16_t* const slotTab = reinterpret_cast<uint16_t*>(lds + gs.slot_off);
    uint32_t* const permTab = lds + gs.perm_off;

    // ---- prefix: positions 0..p0-1 from the Lehmer digits of pr (weights (k-1-p)!/6!); `avail` ends up
    //      holding the six remaining nodes in ascending order, four bits each
    uint64_t avail = 0xBA9876543210ull, prefix = 0;
    {
        uint32_t rem = pr;
        for (int p = 0; p < p0; ++p) {
            const uint32_t f = factorial_u32(k - 1 - p) / 720u;
            const uint32_t d = rem / f;
            rem -= d * f;
            const uint32_t sh = 4u * d;
            const uint64_t node = (avail >> sh) & 0xFull;
            const uint64_t lowbits = avail & ((1ull << sh) - 1ull);
            avail = lowbits | ((avail >> 4) & ~((1ull << sh) - 1ull));
            prefix |= node << (4 * p);
        }
    }
    auto prefix_node = [&](int p) { return (int)((prefix >> (4 * p)) & 0xFull); };
    auto rest_node = [&](int c) { return (int)((avail >> (4 * c)) & 0xFull); };

    // ---- stage the schedule tables and the quotient rows of the links this group can cross
    {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(&kLaneSlot[par][0][0]);
        uint32_t* dst = lds + gs.slot_off;
        for (int i = tid; i < 42 * 64 / 2; i += kGrpThreads) dst[i] = src[i];
        for (int i = tid; i < 384; i += kGrpThreads) permTab[i] = kSlotPerm[par][i];
        const int total = gs.nQ * QROW;
        for (int idx = tid; idx < total; idx += kGrpThreads) {
            const int row = idx / QROW, col = idx - row * QROW;
            int a, b;
            if (row < nA) {
                a = prefix_node(row); b = prefix_node(row + 1);
            } else if (row < nA + nB) {
                a = prefix_node(p0 - 1); b = rest_node(row - nA);
            } else {
                int pi = row - nA - nB, ca = 0;
                while (pi >= 5 - ca) { pi -= 5 - ca; ++ca; }
                a = rest_node(ca); b = rest_node(ca + 1 + pi);
            }
            const uint16_t* qrow = qc + pair_index(a, b, k) * L;
            // columns [0,QD): (q[2a], q[2a+1]);  columns [QD, 2QD+2): (q[2a+1], q[2a+2]) for a = col-QD-1
            const int i0 = col < QD ? 2 * col : 2 * (col - QD - 1) + 1;
            const uint32_t v0 = (i0 >= 0 && i0 <= L - 2) ? qrow[i0] : kCodeInf;
            const uint32_t v1 = (i0 + 1 >= 0 && i0 + 1 <= L - 2) ? qrow[i0 + 1] : kCodeInf;
            qtab[idx] = v0 | (v1 << 16);
        }
    }
    __syncthreads();

    // quotient row used when row s is written: the link between the nodes of rows s and s+1
    auto link_row = [&](int s, uint32_t perm) -> int {
        if (s + 1 < p0) return s;
        if (s + 1 == p0) return nA + (int)(perm & 7u);
        const int r = s - p0;
        const int a = (int)((perm >> (3 * r)) & 7u), b = (int)((perm >> (3 * r + 3)) & 7u);
        return nA + nB + pair_index(a, b, 6);
    };
    // column of the quotient row holding (q[e-1], q[e]) for the output dword jj of row s (e = 2jj + s)
    auto link_col = [&](int s) -> int { return (s & 1) ? (s - 1) / 2 : QD + s / 2; };

    // ---- row 0: g_1[i] = max(D_0[i], q_{pi_0,pi_1}[i-1]) at index i, D_0[i] = 0 if layers [0,i) fit node pi_0
    {
        const int c = wave % 6, half = wave / 6;
        const int node = p0 > 0 ? prefix_node(0) : rest_node(c);
        const int set = p0 > 0 ? 36 + c : c;
        const uint32_t sl = slotTab[set * 64 + lane];
        const uint32_t perm = permTab[sl];
        uint32_t* out = buf0 + (sl >> 5) * (uint32_t)(NP * 32) + (sl & 31u);
        const uint32_t* qrow = qtab + link_row(0, perm) * QROW + link_col(0);
        const uint32_t* lowrow = low + node * (L + 1);
        const int j0 = half * ((NP + 1) / 2), j1 = half ? NP : (NP + 1) / 2;
        for (int jj = j0; jj < j1; ++jj) {
            const int ix = 2 * jj, iy = 2 * jj + 1;
            const uint32_t dx = (ix >= 1 && ix <= L - k + 1 && lowrow[ix] == 0u) ? kCodeZero : kCodeInf;
            const uint32_t dy = (iy <= L - k + 1 && lowrow[iy] == 0u) ? kCodeZero : kCodeInf;
            out[jj * 32] = pk_max(dx | (dy << 16), qrow[jj]);
        }
    }
    __syncthreads();

    // ---- rows 1 .. k-2
    const uint16_t* __restrict__ wt = reinterpret_cast<const uint16_t*>(base + y.wt_off);
    for (int s = 1; s <= k - 2; ++s) {
        const uint32_t* in = (s & 1) ? buf0 : buf1;
        uint32_t* outb = (s & 1) ? buf1 : buf0;
        const int col = link_col(s);
        for (int q = 0; q < 6; ++q) {
            int c = wave + q;
            c = c >= 12 ? c - 12 : c;
            c = c >= 6 ? c - 6 : c;
            const int chunk = 2 * q + (wave >= 6 ? 1 : 0);
            const int jbeg = chunk * kChunkPairs;
            if (jbeg >= NP) continue;
            const int node = s < p0 ? prefix_node(s) : rest_node(c);
            const int set = s < p0 ? 36 + c : (s - p0) * 6 + c;
            // window lengths of the task's four output dwords: one 8-byte scalar load
            const uint2 wpack = *reinterpret_cast<const uint2*>(wt + ((node * (k - 2) + (s - 1)) * y.wt_cols + jbeg));
            const uint32_t sl = slotTab[set * 64 + lane];
            const uint32_t perm = permTab[sl];
            const uint32_t slot_dw = (sl >> 5) * (uint32_t)(NP * 32) + (sl & 31u);
            const uint32_t* qrow = qtab + link_row(s, perm) * QROW + col;
            const int jend = jbeg + kChunkPairs < NP ? jbeg + kChunkPairs : NP;
#pragma unroll
            for (int t = 0; t < kChunkPairs; ++t) {
                const int jj = jbeg + t;
                if (jj >= jend) break;
                const uint32_t wboth = ((t < 2 ? wpack.x : wpack.y) >> (16 * (t & 1))) & 0xFFFFu;
                const int wx = (int)(wboth & 0xFFu), wy = (int)(wboth >> 8);
                const int nmin = wx < wy ? wx : wy, nmax = wx < wy ? wy : wx;
                // p walks down the input row; p[0] is the dword holding input indices (2a, 2a+1)
                const uint32_t* p = in + slot_dw + jj * 32;
                uint32_t acc = kInf2;
                uint32_t cur = p[0];
                int n = nmin >> 1;   // steps in which both positions take both offsets 2m and 2m+1
                while (n >= 4) {
                    p -= 128;
                    const uint32_t l1 = p[96], l2 = p[64], l3 = p[32], l4 = p[0];
                    acc = pk_min3(acc, cur, align16(cur, l1));
                    acc = pk_min3(acc, l1, align16(l1, l2));
                    acc = pk_min3(acc, l2, align16(l2, l3));
                    acc = pk_min3(acc, l3, align16(l3, l4));
                    cur = l4;
                    n -= 4;
                }
                if (n & 2) {
                    p -= 64;
                    const uint32_t l1 = p[32], l2 = p[0];
                    acc = pk_min3(acc, cur, align16(cur, l1));
                    acc = pk_min3(acc, l1, align16(l1, l2));
                    cur = l2;
                }
                if (n & 1) {
                    p -= 32;
                    const uint32_t l1 = p[0];
                    acc = pk_min3(acc, cur, align16(cur, l1));
                    cur = l1;
                }
                if (nmin & 1) acc = pk_min(acc, cur);   // offset nmin-1 is even and valid for both
                if (nmax > nmin) {
                    // offsets nmin .. nmax-1 exist only for the position with the longer window
                    const uint32_t mask = wx > wy ? (kCodeInf << 16) : kCodeInf;
                    const uint32_t* p0w = in + slot_dw + jj * 32;
                    for (int d = nmin; d < nmax; ++d) {
                        uint32_t v;
                        if (d & 1) {
                            const int a = (d + 1) >> 1;
                            v = align16(p0w[-(a - 1) * 32], p0w[-a * 32]);
                        } else {
                            v = p0w[-(d >> 1) * 32];
                        }
                        acc = pk_min(acc, pk_max(v, mask));
                    }
                }
                outb[slot_dw + jj * 32] = pk_max(acc, qrow[jj]);
            }
        }
        __syncthreads();
    }

    // ---- row k-1: only D_{k-1}[L] is needed; then the key of each ordering and the block minimum
    unsigned long long best = PPO_KEY_NONE;
    if (wave < 6) {
        const int s = k - 1, c = wave;
        const uint32_t* in = (s & 1) ? buf0 : buf1;
        const int node = rest_node(c);
        const int set = 5 * 6 + c;
        const uint32_t sl = slotTab[set * 64 + lane];
        const uint32_t perm = permTab[sl];
        const bool active = (perm >> 31) != 0u;   // idle lanes sit on the two unused bank columns
        const uint32_t slot_dw = (sl >> 5) * (uint32_t)(NP * 32) + (sl & 31u);
        const int l = (int)low[node * (L + 1) + L];
        const int w = L - (l > s ? l : s);
        // input indices (NE-1-w, NE-1]
        const int ulo = gs.NE - w, uhi = gs.NE - 1;
        uint32_t acc = kInf2;
        for (int jj = uhi >> 1; jj >= (ulo >> 1) && w > 0; --jj) {
            const uint32_t mask = (2 * jj >= ulo ? 0u : kCodeInf) | (2 * jj + 1 <= uhi ? 0u : (kCodeInf << 16));
            acc = pk_min(acc, pk_max(in[slot_dw + jj * 32], mask));
        }
        const uint32_t cx = acc & 0xFFFFu, cy = acc >> 16;
        const uint32_t code = cx < cy ? cx : cy;
        const uint32_t bits = code >= kCodeInf ? kInfBits : __float_as_uint(dec[code - kCodeZero]);
        const uint32_t r = pr * 720u + ((perm >> 18) & 1023u);
        if (active && r >= rank_begin && r < rank_end) {
            if (EXPORT) beta_export[r - rank_begin] = __uint_as_float(bits);
            best = ((unsigned long long)bits << 32) | r;
        }
    }
    if (!EXPORT) {
        for (int off = 32; off >= 1; off >>= 1) {
            const unsigned long long o = __shfl_xor(best, off, 64);
            best = o < best ? o : best;
        }
        if (lane == 0 && best != PPO_KEY_NONE) {
            if (best < best_key[inst]) atomicMin(best_key + inst, best);
        }
    }
}

hipError_t launch_enumerate_grouped(const Layout& y, int n_inst, const void* ws, uint32_t rank_begin,
                                    uint32_t rank_end, uint64_t* best_key, float* beta_export, hipStream_t stream) {
    if (rank_end <= rank_begin || n_inst == 0) return hipSuccess;
    const GroupedShape gs = GroupedShape::make(y.L, y.k);
    const uint32_t gbeg = 2u * (rank_begin / 720u), gend = 2u * ((rank_end + 719u) / 720u);
    const dim3 grid(gend - gbeg, n_inst), block(kGrpThreads);
    hipError_t e;
    if (beta_export) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&enumerate_grouped_kernel<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)gs.total_bytes);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(enumerate_grouped_kernel<true>, grid, block, gs.total_bytes, stream, y,
                           static_cast<const unsigned char*>(ws), rank_begin, rank_end, gbeg,
                           reinterpret_cast<unsigned long long*>(best_key), beta_export);
    } else {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&enumerate_grouped_kernel<false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)gs.total_bytes);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(enumerate_grouped_kernel<false>, grid, block, gs.total_bytes, stream, y,
                           static_cast<const unsigned char*>(ws), rank_begin, rank_end, gbeg,
                           reinterpret_cast<unsigned long long*>(best_key), beta_export);
    }
    return hipGetLastError();
}

}  // namespace ppo
