// Paired enumeration kernel for k >= 6: two orderings per lane, the DP row in registers.
//
// A team of six waves evaluates the 720 orderings that share a prefix of k-6 nodes (a workgroup is two teams, each
// on a group of its own).  Every ordering runs all of its k DP rows (the unit the headline figure counts).  Wave c holds, at every row, the orderings that
// put the c-th of the six remaining nodes at that row: the memory window [lo[node][e], e-1] is then the same for
// the whole wave, and since a lane's two orderings (one per 16-bit half of its registers) are chosen to share
// that node as well, every instruction works on both halves alike: one packed three-input minimum folds two
// candidates into two orderings at once, with no masks and no per-lane control.
//
// Row convention.  Entry u of a row (1 <= u <= NE-1, NE = L-k+2) stands for the segment end e = u + s of DP
// row s.  A lane keeps entry u in register v[PPO_PAIR_RB + u].  Before row s is computed the registers hold
//     g_s[i] = max(D_{s-1}[i], q_{pi_{s-1},pi_s}[i-1])       at u = i - s + 1
// and D_s[e] = min over i in [max(lo[pi_s][e], s), e-1] of g_s[i] is the minimum of the w = e - max(lo, s)
// entries u, u-1, .., u-w+1 with u = e - s; it replaces entry u in place (the outputs are worked from the
// highest u down).  Outputs whose windows start at the same entry form a run: a chain folds the window of the
// lowest, and each one above it is the minimum of the output below it and its own entry.  Chains and run steps
// are generated code entered by computed jumps (ppo_pair_asm.h); the jump targets of a (node, row) come from a
// table written by pair_tables_kernel below (ppo_pair_program.h).
//
// Which orderings a lane holds changes from row to row (the node at the row must be the wave's), so between
// rows the entries go through LDS: slot = pair, entries 2h and 2h+1 side by side (64 bits), the next two a fixed
// distance on, the bank of a slot being its coset class (ppo_pair_tables.h), conflict free by construction.  The rows of the shared prefix and the first
// row after it need no exchange: all orderings of a lane set keep their node there.  The pairing changes once,
// before the row of position 4 of the six: only upper halves move (see gen_pair_tables.py).
#include "ppo_common.h"
#include "ppo_pair_asm.h"
#include "ppo_pair_program.h"
#include "ppo_pair_tables.h"

namespace ppo {

constexpr int kPairWaves = 6;                    // waves of a team: one per node that can sit at a row
constexpr int kPairTeams = 2;                    // two teams per workgroup, each on a group of its own
constexpr int kPairThreads = kPairTeams * kPairWaves * 64;
constexpr int kPairSlots = 384;   // 12 indices x 32 banks; banks 30 and 31 hold the spare slots

struct PairedShape {
    int NE, QD, QROW, QPITCH, nA, nB, nQ;
    uint32_t q_off, q_dwords, sync_off, total_bytes;   // offsets in dwords
    __host__ __device__ static PairedShape make(int L, int k) {
        PairedShape g;
        g.NE = L - k + 2;
        g.QD = L / 2 + 1;
        g.QROW = 2 * g.QD + 2;
        g.QPITCH = g.QROW | 1;
        const int p0 = k - 6;
        g.nA = p0 > 1 ? p0 - 1 : 0;
        g.nB = p0 > 0 ? 6 : 0;
        g.nQ = g.nA + g.nB + 15;
        g.q_off = (uint32_t)((g.NE - 1) / 2 + 1) * 2u * kPairSlots;   // pairs of entries (2h, 2h+1), h = 0 .. (NE-1)/2
        g.q_dwords = (uint32_t)(g.nQ * g.QPITCH);          // one quotient table per team
        g.sync_off = g.q_off + kPairTeams * g.q_dwords;    // then the counters the teams synchronise with
        // 64 dwords behind the tables: the quotient reads of a row always take 48 dwords from their first column
        g.total_bytes = (g.sync_off + 64u) * 4u;
        return g;
    }
};

bool paired_supported(int L, int k) {
    if (k < 6) return false;
    const PairedShape g = PairedShape::make(L, k);
    return g.NE - 1 <= PPO_PAIR_UMAX && g.total_bytes <= (uint32_t)kLdsBytesPerCU;
}

// spare slot that holds the first DP row of node j (both halves the same); the spare slots 30, 31, 62, 63 are the
// idle lanes'; eight more keep prefix rows in the bounded mode (team t, row 1 .. 4)
__host__ __device__ inline uint32_t pair_d0_slot(int j) { return (uint32_t)(2 + j / 2) * 32u + 30u + (uint32_t)(j & 1); }
__host__ __device__ inline uint32_t pair_kept_slot(int team, int row) { return (uint32_t)(7 + row) * 32u + 30u + (uint32_t)team; }
static_assert(PPO_MAX_K - 6 - 2 <= 4, "one spare slot per team for each of the prefix rows 1 .. p0-2");
// dword of entry u of a slot: entries 2h and 2h+1 side by side, the next pair of entries 2 * kPairSlots dwords on
__host__ __device__ inline uint32_t pair_entry_dword(uint32_t slot, uint32_t u) { return (u >> 1) * (2u * kPairSlots) + slot * 2u + (u & 1u); }

// ---------------------------------------------------------------------------------------------
// The jump tables of one node's DP rows s = 1 .. k-1, one thread per output position (ppo_pair_program.h).
// ---------------------------------------------------------------------------------------------
static_assert(kPairTableDwords * 2 == kPairSlots16, "two 16-bit entries per dword of the table");
constexpr int kPairTableThreads = 256;
// one workgroup per (node, instance): the rows s = 1 .. k-1 of that node
__global__ __launch_bounds__(kPairTableThreads) void pair_tables_kernel(Layout y, unsigned char* __restrict__ ws) {
    __shared__ unsigned char lo_s[PPO_MAX_L + 1];
    __shared__ __align__(4) uint16_t entry_s[(PPO_MAX_K - 1) * kPairSlots16];
    __shared__ __align__(4) PairOffsets off_s;   // a copy close by: every position looks a few offsets up
    __shared__ unsigned char below_s[(PPO_MAX_K - 1) * kPairSlots16];   // see pair_below
    const int L = y.L, k = y.k, j = blockIdx.x, inst = blockIdx.y, tid = threadIdx.x;
    unsigned char* base = ws + (size_t)inst * y.stride;
    const unsigned char* lo = base + y.lo_off + (size_t)j * (L + 1);
    uint32_t* pt = reinterpret_cast<uint32_t*>(base + y.pt_off) + (size_t)j * (k - 1) * kPairTableDwords;
    for (int i = tid; i <= L; i += kPairTableThreads) lo_s[i] = lo[i];
    {
        const uint16_t* src = reinterpret_cast<const uint16_t*>(&pair_offsets());
        uint16_t* dst = reinterpret_cast<uint16_t*>(&off_s);
        for (int i = tid; i < (int)(sizeof(PairOffsets) / 2); i += kPairTableThreads) dst[i] = src[i];
    }
    uint32_t* fill = reinterpret_cast<uint32_t*>(entry_s);
    for (int i = tid; i < (k - 1) * kPairTableDwords; i += kPairTableThreads) fill[i] = kPairEnd | (kPairEnd << 16);
    __syncthreads();
    const int top = L - k + 1;
    for (int idx = tid; idx < (k - 1) * top; idx += kPairTableThreads) {
        const int row = idx / top, u = idx - row * top + 1;
        below_s[row * kPairSlots16 + u] = pair_below(row + 1, lo_s, u);
    }
    __syncthreads();
    // every output position of every row writes the entries it is responsible for: one writer per entry
    for (int idx = tid; idx < (k - 1) * top; idx += kPairTableThreads) {
        const int row = idx / top, u = idx - row * top + 1;
        pair_row_program_at(off_s, top, row + 1 == k - 1, below_s + row * kPairSlots16, u, entry_s + row * kPairSlots16);
    }
    __syncthreads();
    const uint32_t* src = reinterpret_cast<const uint32_t*>(entry_s);
    for (int i = tid; i < (k - 1) * kPairTableDwords; i += kPairTableThreads) pt[i] = src[i];
}

hipError_t launch_pair_tables(const Layout& y, int n_inst, void* ws, hipStream_t stream) {
    if (!paired_supported(y.L, y.k)) return hipSuccess;   // nothing reads the tables then
    hipLaunchKernelGGL(pair_tables_kernel, dim3(y.k, n_inst), dim3(kPairTableThreads), 0, stream, y, static_cast<unsigned char*>(ws));
    return hipGetLastError();
}

typedef __attribute__((address_space(3))) uint32_t pair_lds_u32_t;
__device__ __forceinline__ uint32_t pair_lds_addr(const uint32_t* p) { return (uint32_t)(uintptr_t)(const pair_lds_u32_t*)p; }

// The row steps.  Every block works on fixed registers (the row in v[PPO_PAIR_RB + 1 ..], see the generator) that
// are declared clobbered here; the values live in them from one block to the next, and the build step checks in
// the compiled code that nothing between the blocks touches them.
#define PPO_PAIR_CLOBBERS PPO_PAIR_CLOBBER_V, PPO_PAIR_CLOBBER_S, "memory"
__device__ __forceinline__ void pair_load(uint32_t addr, uint32_t skip) {
    asm volatile(PPO_PAIR_LOAD_ASM : : [addr] "v"(addr), [skip] "s"(skip) : PPO_PAIR_CLOBBERS);
}
__device__ __forceinline__ void pair_load_exchange(uint32_t addr, uint32_t addr2, uint32_t skip) {
    asm volatile(PPO_PAIR_LOADX_ASM : : [addr] "v"(addr), [addr2] "v"(addr2), [skip] "s"(skip) : PPO_PAIR_CLOBBERS);
}
__device__ __forceinline__ void pair_store(uint32_t addr, uint32_t skip) {
    asm volatile("s_waitcnt lgkmcnt(0)\n" PPO_PAIR_STORE_ASM : : [addr] "v"(addr), [skip] "s"(skip) : PPO_PAIR_CLOBBERS);
}
__device__ __forceinline__ void pair_row(uint32_t qaddr, const uint32_t* desc, uint32_t skip) {
    asm volatile(PPO_PAIR_ROW_ASM : : [qaddr] "v"(qaddr), [desc] "s"(desc), [skip] "s"(skip) : PPO_PAIR_CLOBBERS);
}
__device__ __forceinline__ uint32_t pair_rowmin(uint32_t skip) {
    uint32_t res;
    asm volatile(PPO_PAIR_ROWMIN_ASM : [res] "=&v"(res) : [skip] "s"(skip) : PPO_PAIR_CLOBBERS);
    return res;
}
__device__ __forceinline__ uint32_t pair_extract(uint32_t skip) {
    uint32_t res;
    asm volatile("s_waitcnt lgkmcnt(0)\n" PPO_PAIR_EXTRACT_ASM : [res] "=v"(res) : [skip] "s"(skip) : PPO_PAIR_CLOBBERS);
    return res;
}

// Synchronisation of the two teams.  A team (six waves) works on one group; its rows 0 .. p0 need no LDS, its
// later rows go through the one row buffer of the workgroup.  The teams take turns at the buffer: while one
// exchanges rows, the other computes the register-only rows of its next group, so that every SIMD has waves of
// both kinds to issue from.  Waves of a team meet at a counter in LDS (the hardware barrier would stop the other
// team as well); the buffer passes to the next group when every wave of the group before it has fetched its last
// row.  All counters only grow; a wave compares them with counts of its own.
struct PairSync {
    uint32_t team[kPairTeams];   // waves of the team that have reached their n-th meeting, summed over n
    uint32_t done;               // waves that are through with the row buffer, summed over the groups in turn
    uint32_t bound[kPairTeams];  // bounded mode: bits of the best beta known when the team's group started
};
__device__ __forceinline__ void pair_spin_until(volatile uint32_t* counter, uint32_t target) {
    while (__hip_atomic_load(const_cast<uint32_t*>(counter), __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < target)
        __builtin_amdgcn_s_sleep(1);
}
__device__ __forceinline__ void pair_arrive(uint32_t* counter) {
    if ((threadIdx.x & 63) == 0) __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// beta_export: null for the search; else beta of every ordering of the range is written out as well (one kernel
// for both: a second instantiation would be a second copy of the generated code).
// bounded: a group whose last prefix row (the same for all its orderings) has no entry at or below the best beta
// known when the group starts cannot hold the optimum or a tie with it (no entry of a DP row is below the least
// entry of the row before it) and is left after that row; every wave of the team takes the same decision from the
// same row and from one published copy of the best beta.  Waves publish what they find after every group.
// (A template parameter rather than an argument: the plain search must not carry the other mode's code in its loop.)
template <bool bounded>
__global__ __launch_bounds__(kPairThreads) void enumerate_paired_kernel(
    Layout y, const unsigned char* __restrict__ ws, uint32_t rank_begin, uint32_t rank_end, uint32_t prefix_begin,
    uint32_t prefix_end, uint32_t prefixes_per_block, unsigned long long* __restrict__ best_key,
    float* __restrict__ beta_export, unsigned long long* __restrict__ skipped_groups) {
    extern __shared__ __align__(16) uint32_t lds[];
    const bool EXPORT = beta_export != nullptr;
    const int L = y.L, k = y.k, inst = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
    const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int team = wave_id / kPairWaves, wave = wave_id - team * kPairWaves;
    const int p0 = k - 6;
    const PairedShape ps = PairedShape::make(L, k);
    const int NE = ps.NE, QD = ps.QD, QROW = ps.QROW, QPITCH = ps.QPITCH, nA = ps.nA, nB = ps.nB;
    // what the blocks leave out at the top of their unrolled ranges: entries (compute, extract), pairs of entries (load, store)
    const uint32_t skip = (uint32_t)__builtin_amdgcn_readfirstlane(PPO_PAIR_UMAX - (NE - 1));
    const uint32_t skip_pairs = (uint32_t)__builtin_amdgcn_readfirstlane(PPO_PAIR_HMAX - (NE - 1) / 2);

    const unsigned char* base = ws + (size_t)inst * y.stride;
    const float* __restrict__ dec = reinterpret_cast<const float*>(base + y.dec_off);
    const uint32_t* __restrict__ qa = reinterpret_cast<const uint32_t*>(base + y.qa_off);
    const uint32_t* __restrict__ pt = reinterpret_cast<const uint32_t*>(base + y.pt_off);
    uint32_t* const qtab = lds + ps.q_off + (uint32_t)team * ps.q_dwords;
    PairSync* const sync = reinterpret_cast<PairSync*>(lds + ps.sync_off);
    const uint32_t buf_addr = pair_lds_addr(lds), qtab_addr = pair_lds_addr(qtab);

    // the lane's schedule: which pair it holds at the row of each of the six positions
    const uint32_t lc0 = kPairLane[wave][lane][0], lc1 = kPairLane[wave][lane][1], lc2 = kPairLane[wave][lane][2],
                   lc3 = kPairLane[wave][lane][3];
    auto slot_addr = [&](int r) -> uint32_t {
        const uint32_t s = ((r < 3 ? lc0 >> (9 * r) : lc1 >> (9 * (r - 3))) & 511u);
        return buf_addr + s * 8u;
    };
    // first DP rows of all nodes into their spare slots, and +inf into the spare slots of the idle lanes
    {
        const uint32_t* d0src = reinterpret_cast<const uint32_t*>(base + y.d0_off);
        for (int idx = tid; idx < k * (NE - 1); idx += kPairThreads) {
            const int j = idx / (NE - 1), u = idx - j * (NE - 1) + 1;
            const uint32_t c = (d0src[j * y.wt_cols + (u >> 1)] >> (16 * (u & 1))) & 0xFFFFu;
            lds[pair_entry_dword(pair_d0_slot(j), (uint32_t)u)] = c | (c << 16);
        }
        for (int idx = tid; idx < 4 * (NE - 1); idx += kPairThreads) {
            const int n = idx & 3, u = (idx >> 2) + 1;
            lds[pair_entry_dword(30u + (uint32_t)(n & 1) + 32u * (uint32_t)(n >> 1), (uint32_t)u)] = kCodeInf | (kCodeInf << 16);
        }
        if (tid < (int)(sizeof(PairSync) / 4)) lds[ps.sync_off + tid] = 0u;
    }
    __syncthreads();   // the only hardware barrier: from here on the teams run on their own
    unsigned long long best = PPO_KEY_NONE;
    uint64_t prev_prefix = 0;   // bounded mode: the prefix of the team's previous group
    bool prev_valid = false;
    uint32_t meetings = 0;   // meetings of this wave's team so far
    auto team_meet = [&]() {
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        pair_arrive(&sync->team[team]);
        ++meetings;
        pair_spin_until(&sync->team[team], meetings * (uint32_t)kPairWaves);
    };

    // prefix of a group from the Lehmer digits of its index (weights (k-1-p)!/6!); `avail` ends up holding the
    // six remaining nodes in ascending order, four bits each
    auto decode_group = [&](uint32_t pr, uint64_t& prefix_out, uint64_t& avail_out) {
        uint64_t avail_ = 0xBA9876543210ull, prefix_ = 0;
        uint32_t digits = 0, rem = pr;
#pragma unroll
        for (int q = 0; q < PPO_MAX_K - 6; ++q) {
            if (q < p0) {
                const uint32_t b = 7u + (uint32_t)q;
                const uint32_t next = rem / b;
                digits |= (rem - next * b) << (4 * (p0 - 1 - q));
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
    auto link_col = [&](int s) -> int { return (s & 1) ? (s - 1) / 2 : QD + s / 2; };

    // the groups of this workgroup in turn, even ones to team 0, odd ones to team 1
    const uint32_t prefix_first = prefix_begin + blockIdx.x * prefixes_per_block;
    for (uint32_t gi = (uint32_t)team; gi < prefixes_per_block; gi += kPairTeams) {
        const uint32_t pr = prefix_first + gi;
        if (pr >= prefix_end) break;
        uint64_t prefix, avail;
        decode_group(pr, prefix, avail);
        auto pnode = [=](int p) { return (int)((prefix >> (4 * p)) & 0xFull); };
        auto rnode = [=](int c) { return (int)((avail >> (4 * c)) & 0xFull); };
        team_meet();   // the team is done with the quotient rows of its previous group
        // quotient rows of the links this group can cross: wave w stages rows w, w+6, ...
        for (int row = wave; row < ps.nQ; row += kPairWaves) {
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
            for (int col = lane; col < QROW; col += 64) qtab[row * QPITCH + col] = qsrc[col];
        }
        if (bounded && wave == 0 && lane == 0)
            sync->bound[team] = (uint32_t)(__hip_atomic_load(best_key + inst, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >> 32);
        team_meet();

        // The k rows in turn.  Rows 0 .. p0 stay in registers (the node of each is the same for all orderings of
        // the wave whatever the lane holds); from the row of position 1 on, a row is loaded from the slots its
        // lanes hold now, and every row but the last is stored for the next one.  One copy of each block per
        // kernel: the generated code is large.
        const uint32_t d0_addr = buf_addr + pair_d0_slot(p0 > 0 ? pnode(0) : rnode(wave)) * 8u;
        // Bounded mode: the rows 1 .. p0-2 of the prefix (the same in every lane) are kept in spare slots of the
        // row buffer, one per team and row, and the group starts from the deepest of them that its prefix shares
        // with the team's previous group.
        int s_first = 0;
        if (bounded) {
            const uint64_t diff = prefix ^ prev_prefix;
            const int shared = !prev_valid ? 0 : diff ? (__ffsll((long long)diff) - 1) / 4 : p0;   // leading nodes in common
            if (shared >= 2 && p0 >= 3) s_first = shared - 1 < p0 - 2 ? shared - 1 : p0 - 2;
            prev_prefix = prefix;
            prev_valid = true;
        }
        auto kept_addr = [&](int row) -> uint32_t { return buf_addr + pair_kept_slot(team, row) * 8u; };
        bool left = false;
#pragma unroll 1
        for (int s = s_first; s < k; ++s) {
            const int r = s - p0;
            if (s == s_first || r >= 1) {
                const uint32_t a = s == s_first ? (s == 0 ? d0_addr : kept_addr(s)) : slot_addr(r);
                if (r == 4) {
                    pair_load_exchange(a, buf_addr + (lc2 & 511u) * 8u, skip_pairs);
                    team_meet();   // every upper half has been fetched before a slot is overwritten
                } else {
                    pair_load(a, skip_pairs);
                }
            }
            if (s >= 1 && s != s_first) {
                // the link between the nodes of rows s-1 and s, and the node of row s
                uint32_t qrow;
                int node;
                if (s < p0) {
                    qrow = (uint32_t)(s - 1);
                    node = pnode(s);
                } else if (s == p0) {
                    qrow = (uint32_t)(nA + wave);
                    node = rnode(wave);
                } else {
                    qrow = (uint32_t)(nA + nB) + ((lc2 >> (9 + 4 * (r - 1))) & 15u);
                    node = rnode(wave);
                }
                const uint32_t* desc = pt + (uint32_t)__builtin_amdgcn_readfirstlane((node * (k - 1) + (s - 1)) * kPairTableDwords);
                pair_row(qtab_addr + qrow * (uint32_t)(QPITCH * 4) + (uint32_t)link_col(s) * 4u, desc, skip);
                if (s == k - 1) pair_arrive(&sync->done);   // the last row has been fetched: the buffer can go on
            }
            if (bounded && s >= 1 && s <= p0 - 2 && s != s_first && wave == 0 && lane == 0)
                pair_store(kept_addr(s), skip_pairs);   // for the team's next groups (they meet before they read it)
            if (bounded && s == p0 - 1) {
                // the last row of the prefix: the same in every lane of every wave of the team
                const uint32_t code = (uint32_t)__builtin_amdgcn_readfirstlane(pair_rowmin(skip)) & 0xFFFFu;
                const uint32_t bits = code >= kCodeInf ? kInfBits : __float_as_uint(dec[code - kCodeZero]);
                if (bits > (uint32_t)__builtin_amdgcn_readfirstlane((int)sync->bound[team])) {
                    left = true;
                    break;
                }
            }
            // the row goes to LDS where the next row has to fetch it from other lanes (rows of positions 0 .. 4)
            if (r >= 1 && s < k - 1) pair_store(slot_addr(r), skip_pairs);
            if (r == 0 && s < k - 1) {
                // the group's first row in LDS waits for the buffer: every wave of the group before it has fetched its last row
                pair_spin_until(&sync->done, gi * (uint32_t)kPairWaves);
                pair_store(slot_addr(0), skip_pairs);
            }
            if (r >= 0 && s < k - 1) team_meet();
        }
        if (left) {
            // nothing of this group touches the row buffer: it counts as through with it at once
            pair_arrive(&sync->done);
            if (skipped_groups && wave == 0 && lane == 0) atomicAdd(skipped_groups + inst, 2ull);   // in units of 360 orderings
            continue;
        }
        const uint32_t res = pair_extract(skip);   // D[L] of the lane's two orderings
        if (lc3 >> 31) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t code = (res >> (16 * h)) & 0xFFFFu;
                const uint32_t r = pr * 720u + ((lc3 >> (10 * h)) & 1023u);
                if (r >= rank_begin && r < rank_end) {
                    if (EXPORT) {
                        const uint32_t bits = code >= kCodeInf ? kInfBits : __float_as_uint(dec[code - kCodeZero]);
                        beta_export[r - rank_begin] = __uint_as_float(bits);
                    }
                    const unsigned long long key = ((unsigned long long)code << 32) | r;
                    best = key < best ? key : best;
                }
            }
        }
        if (bounded) {
            // what this wave has found so far, for the groups that start after this one
            unsigned long long w = best;
            for (int off = 32; off >= 1; off >>= 1) {
                const unsigned long long o = __shfl_xor(w, off, 64);
                w = o < w ? o : w;
            }
            if (lane == 0 && w != PPO_KEY_NONE) {
                const uint32_t code = (uint32_t)(w >> 32);
                const uint32_t bits = code >= kCodeInf ? kInfBits : __float_as_uint(dec[code - kCodeZero]);
                const unsigned long long key = ((unsigned long long)bits << 32) | (w & 0xFFFFFFFFull);
                if (key < __hip_atomic_load(best_key + inst, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMin(best_key + inst, key);
            }
        }
    }

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

hipError_t launch_enumerate_paired(const Layout& y, int n_inst, const void* ws, uint32_t rank_begin, uint32_t rank_end,
                                   uint64_t* best_key, float* beta_export, bool bounded, uint64_t* skipped_groups,
                                   hipStream_t stream) {
    if (rank_end <= rank_begin || n_inst == 0) return hipSuccess;
    const PairedShape ps = PairedShape::make(y.L, y.k);
    const uint32_t pbeg = rank_begin / 720u, pend = (rank_end + 719u) / 720u;
    const uint32_t count = pend - pbeg;
    // groups per workgroup (its two teams take them in turn): as many as 16, fewer where the grid would fall
    // under a few thousand workgroups, never fewer than two
    uint32_t ppb = 16;
    while (ppb > 2 && (uint64_t)(count / ppb) * (uint64_t)n_inst < 4096u) ppb >>= 1;
    const dim3 grid((count + ppb - 1) / ppb, n_inst);
    if (bounded && !beta_export) {
        static std::atomic<uint64_t> lds_allowed{0};
        const hipError_t e = allow_full_lds(reinterpret_cast<const void*>(&enumerate_paired_kernel<true>), lds_allowed);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(enumerate_paired_kernel<true>, grid, dim3(kPairThreads), ps.total_bytes, stream, y,
                           static_cast<const unsigned char*>(ws), rank_begin, rank_end, pbeg, pend, ppb,
                           reinterpret_cast<unsigned long long*>(best_key), beta_export,
                           reinterpret_cast<unsigned long long*>(skipped_groups));
    } else {
        static std::atomic<uint64_t> lds_allowed{0};
        const hipError_t e = allow_full_lds(reinterpret_cast<const void*>(&enumerate_paired_kernel<false>), lds_allowed);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(enumerate_paired_kernel<false>, grid, dim3(kPairThreads), ps.total_bytes, stream, y,
                           static_cast<const unsigned char*>(ws), rank_begin, rank_end, pbeg, pend, ppb,
                           reinterpret_cast<unsigned long long*>(best_key), beta_export,
                           reinterpret_cast<unsigned long long*>(skipped_groups));
    }
    return hipGetLastError();
}

}  // namespace ppo
