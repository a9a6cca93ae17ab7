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
// position from the cuts the prefix reaches within beta* and the rows of A, then the cuts by the fixed-k cut rule.
#include <array>
#include <utility>

#include "ppo_common.h"

namespace ppo {

// Codes as in the fixed-k kernels: kCodeZero for the value 0, kCodeZero + 1 + #{smaller quotients}, kCodeInf for
// +inf: positive normal binary16 patterns, so the three-input binary16 minimum acts as an integer minimum.
// Everything these kernels read as a code is written by them as one (a stray pattern could win that minimum).
constexpr uint32_t kClZero = kCodeZero, kClInf = kCodeInf;
constexpr int kClPreThreads = 1024;
static_assert((int)kClZero + (PPO_CLUSTER_MAX_N * (PPO_CLUSTER_MAX_N - 1) / 2) * (PPO_MAX_L - 1) + 1 < (int)kClInf,
              "codes stay below +inf");
static_assert(((unsigned long long)PPO_CLUSTER_MAX_N << (PPO_CLUSTER_MAX_N - 1)) * ((PPO_MAX_L + 1) / 2) < (1ull << 32),
              "the dwords of one instance's rows are counted in 32 bits");

struct ClusterLayout {
    int L, n, npairs, nq, rs;                       // rs: entries per row of A: 0..L-1 (entry L is never finite
                                                    // and not stored), rounded up to even
    uint32_t hi_off, qc_off, dec_off, qv_off, ord_off, img_off, stride;   // bytes within one instance's tables

    __host__ __device__ static ClusterLayout make(int L, int n) {
        ClusterLayout y;
        y.L = L;
        y.n = n;
        y.npairs = n * (n - 1) / 2;
        y.nq = y.npairs * (L - 1);
        y.rs = (L + 1) & ~1;
        size_t off = 0;
        y.hi_off = (uint32_t)off;
        off = align_up(off + (size_t)n * (L + 1), 16);
        y.qc_off = (uint32_t)off;
        off = align_up(off + (size_t)y.npairs * L * 2, 16);
        y.dec_off = (uint32_t)off;
        off = align_up(off + ((size_t)y.nq + 1) * 4, 16);
        y.qv_off = (uint32_t)off;
        off = align_up(off + (size_t)y.nq * 4, 16);
        y.ord_off = (uint32_t)off;   // the layers 0 .. L-2 in increasing order of t (one byte each)
        off = align_up(off + (size_t)L, 256);
        // what the level kernel keeps in LDS, ready to be copied: quotient rows of every ordered pair (rs / 2
        // dwords each, the pitch of the rows of A), then the window queries of every (node, entry) (128 dwords
        // per node)
        y.img_off = (uint32_t)off;
        off = align_up(off + q_image_bytes(n, y.rs) + (size_t)n * 512, 256);
        y.stride = (uint32_t)off;
        return y;
    }
    // bytes of the quotient rows in the LDS image (the window queries follow, 16-byte aligned)
    __host__ __device__ static size_t q_image_bytes(int n, int rs) { return align_up((size_t)n * n * (rs / 2) * 4, 16); }
    // rows A[R][j] exist for j in R only: n 2^(n-1) of them per instance
    __host__ __device__ size_t rows_per_instance() const { return (size_t)n << (n - 1); }
    __host__ __device__ size_t rows_bytes() const { return rows_per_instance() * (size_t)rs * sizeof(uint16_t); }
};

// Row number of A[R][j], j in R: the rows of the sets before R in numeric order (the sum of their sizes),
// then the members of R in increasing order.  The sum of the sizes of all sets below R: a member b of R
// with h members above it stands for the 2^b sets that agree with R above b and lack b; they have
// h + (a free choice below b) members: h 2^b + b 2^(b-1) in all (b 2^(b-1) written (b << b) >> 1: no case for b = 0).
__host__ __device__ inline uint32_t cluster_first_row(uint32_t R, int n) {
    uint32_t rows = 0, above = 0;
    for (int b = n - 1; b >= 0; --b) {
        if (!((R >> b) & 1u)) continue;
        rows += (above << b) + (((uint32_t)b << b) >> 1);
        ++above;
    }
    return rows;
}
size_t cluster_tables_bytes(int L, int n) { return ClusterLayout::make(L, n).stride; }
size_t cluster_rows_bytes(int L, int n) { return ClusterLayout::make(L, n).rows_bytes(); }

// ---------------------------------------------------------------------------------------------
// Tables of one instance: hi[j][e] = last e' such that layers [e, e') fit node j (e if none; the memory
// rule with binary64 prefix sums) and the quotients of Eq. 3; then, in a second kernel over slices of
// the quotients, their order codes (1 + the number of strictly smaller quotients of the instance).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kClPreThreads) void cluster_tables_kernel(const float* __restrict__ t,
                                                                      const float* __restrict__ m,
                                                                      const float* __restrict__ M,
                                                                      const float* __restrict__ B, ClusterLayout y,
                                                                      unsigned char* __restrict__ ws) {
    __shared__ double P[PPO_MAX_L + 1];
    const int L = y.L, n = y.n, inst = blockIdx.x, tid = threadIdx.x;
    const float* ti = t + (size_t)inst * L;
    const float* mi = m + (size_t)inst * L;
    const float* Mi = M + (size_t)inst * n;
    const float* Bi = B + (size_t)inst * n * n;
    unsigned char* base = ws + (size_t)inst * y.stride;
    unsigned char* hi = base + y.hi_off;
    float* dec = reinterpret_cast<float*>(base + y.dec_off);
    float* qv = reinterpret_cast<float*>(base + y.qv_off);
    if (tid == 0) {
        double acc = 0.0;
        P[0] = 0.0;
        for (int i = 0; i < L; ++i) {
            acc = acc + (double)mi[i];
            P[i + 1] = acc;
        }
        dec[0] = 0.0f;
    }
    __syncthreads();
    for (int idx = tid; idx < n * (L + 1); idx += kClPreThreads) {
        const int j = idx / (L + 1), e = idx - j * (L + 1);
        const double cap = (double)Mi[j];
        int e2 = e;
        while (e2 < L && (P[e2 + 1] - P[e]) <= cap) ++e2;
        hi[idx] = (unsigned char)e2;
    }
    // The quotients of one link, t[i] / B, are in the order of the t[i] (a correctly rounded division by a
    // positive number is monotone), so each link's row is written sorted: position r holds the quotient of the
    // layer with the r-th smallest t (ties by index).  Ranking a quotient among all of them is then a binary
    // search per link instead of a comparison with every quotient.
    __shared__ float t_s[PPO_MAX_L];
    __shared__ unsigned char ord_s[PPO_MAX_L];
    for (int i = tid; i < L - 1; i += kClPreThreads) t_s[i] = ti[i] == 0.0f ? 0.0f : ti[i];   // -0 is a size of zero: +0
    __syncthreads();
    for (int i = tid; i < L - 1; i += kClPreThreads) {
        const float x = t_s[i];
        int pos = 0;
        for (int i2 = 0; i2 < L - 1; ++i2) pos += (t_s[i2] < x || (t_s[i2] == x && i2 < i)) ? 1 : 0;
        ord_s[pos] = (unsigned char)i;
        base[y.ord_off + pos] = (unsigned char)i;
    }
    __syncthreads();
    for (int idx = tid; idx < y.nq; idx += kClPreThreads) {
        const int p = idx / (L - 1), r = idx - p * (L - 1);
        int a = 0, rem = p;
        while (rem >= n - 1 - a) { rem -= n - 1 - a; ++a; }
        const int b = a + 1 + rem;
        qv[idx] = __fdiv_rn(t_s[ord_s[r]], Bi[a * n + b]);
    }
}

// Order codes: grid.x slices of 256 quotients, grid.y = instance.  All sorted rows are staged in LDS; a thread
// adds up, over the links, how many of a link's quotients are strictly below its own (a binary search each).
constexpr int kClCountThreads = 256;
__global__ __launch_bounds__(kClCountThreads) void cluster_count_kernel(ClusterLayout y, unsigned char* __restrict__ ws) {
    extern __shared__ __align__(16) float cl_rows[];   // [npairs][L-1]
    const int L = y.L, nq = y.nq, len = L - 1, inst = blockIdx.y, tid = threadIdx.x;
    unsigned char* base = ws + (size_t)inst * y.stride;
    const float* __restrict__ qv = reinterpret_cast<const float*>(base + y.qv_off);
    for (int i = tid; i < nq; i += kClCountThreads) cl_rows[i] = qv[i];
    __syncthreads();
    const int idx = blockIdx.x * kClCountThreads + tid;
    if (idx >= nq) return;
    const float x = cl_rows[idx];
    int below = 0;
    // four links at a time, so that four reads are in flight at every step of the searches
    for (int p0 = 0; p0 < y.npairs; p0 += 4) {
        int pos[4] = {0, 0, 0, 0};   // number of entries of each row below x
        const float* row[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) row[u] = cl_rows + (p0 + u < y.npairs ? p0 + u : p0) * len;
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
    const int p = idx / len, r = idx - p * len;
    const int i = base[y.ord_off + r];
    reinterpret_cast<uint16_t*>(base + y.qc_off)[p * L + i] = (uint16_t)(kClZero + 1 + below);
    reinterpret_cast<float*>(base + y.dec_off)[1 + below] = x;
}

// ---------------------------------------------------------------------------------------------
// One level: every row A[R][j] with |R| = level.  The unit of work of a wave is a set R' with |R'| =
// level - 1: it loads the rows A[R'][j''] once (two entries per lane) and produces A[R' + j][j] for every
// j outside R'.  For each j: the `rest` row (quotients from a copy of the table in LDS, shifted so that
// entry e holds q[e-1]), then a table of minima over runs of 1, 2, 4 .. 64 entries of it in LDS, from which
// the minimum over the window (e, hi[j][e]] is two reads.  grid.x waves share the sets, grid.y = instance.
// ---------------------------------------------------------------------------------------------
constexpr int kClRunLevels = 7;    // runs of 2^0 .. 2^6 entries
constexpr int kClRunRow = 160;     // entries per run-minimum row: 128 computed per set, the rest constant
static_assert(kClRunRow / 2 >= 64 + (1 << (kClRunLevels - 3)) && kClRunRow % 2 == 0,
              "the longest runs (2^(levels-1) entries) are built from dwords up to 2^(levels-3) beyond a lane's own");
constexpr int kClQueryRow = 128;   // window queries per node in LDS: one dword per entry e

typedef unsigned short cl_ushort2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t cl_pk_min(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(cl_ushort2, a), __builtin_bit_cast(cl_ushort2, b)));
}
__device__ __forceinline__ uint32_t cl_pk_max(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(cl_ushort2, a), __builtin_bit_cast(cl_ushort2, b)));
}

// Binomial coefficients C(i, j), i, j <= PPO_CLUSTER_MAX_N, and the set of a given size with a given index:
// sets of c nodes are numbered by sum over their members b_c > ... > b_1 of C(b_i, i) (the combinatorial
// number system), so that the sets of one level can be dealt out evenly to the waves.
struct ClusterBinomials {
    uint32_t c[PPO_CLUSTER_MAX_N + 1][PPO_CLUSTER_MAX_N + 1];
    constexpr ClusterBinomials() : c{} {
        for (int i = 0; i <= PPO_CLUSTER_MAX_N; ++i) {
            c[i][0] = 1;
            for (int j = 1; j <= i; ++j) c[i][j] = c[i - 1][j - 1] + (j <= i - 1 ? c[i - 1][j] : 0u);
        }
    }
};
constexpr ClusterBinomials kClBinomialsHost = ClusterBinomials();
__constant__ ClusterBinomials kClBinomials = ClusterBinomials();

// also gives the set's first row (cluster_first_row), gathered on the way: members come out highest first
__device__ __forceinline__ uint32_t cluster_set_at(uint32_t index, int size, int n, uint32_t& first_row) {
    uint32_t set = 0, rows = 0, above = 0;
    int b = n;
    for (int i = size; i >= 1; --i) {
        do { --b; } while (kClBinomials.c[b][i] > index);
        set |= 1u << b;
        index -= kClBinomials.c[b][i];
        rows += (above << b) + (((uint32_t)b << b) >> 1);
        ++above;
    }
    first_row = rows;
    return set;
}

// LDS of the level kernel: the quotient rows of every ORDERED pair of nodes, rs / 2 dwords each (so that the row
// of (j, j'') is a fixed distance from the row of (j, 0); lanes beyond a row read on into the next one, or into
// the queries after the last, and drop what they read), the window queries of every (node, entry), and the
// run-minimum tables of each wave.
struct ClusterLds {
    uint32_t hi_off, run_off, total;
    int waves;
    __host__ __device__ static ClusterLds make(const ClusterLayout& y, int waves) {
        ClusterLds s;
        s.waves = waves;
        s.hi_off = (uint32_t)ClusterLayout::q_image_bytes(y.n, y.rs);
        s.run_off = (uint32_t)align_up((size_t)s.hi_off + (size_t)y.n * kClQueryRow * 4, 16);
        s.total = s.run_off + (uint32_t)waves * kClRunLevels * kClRunRow * 2;
        return s;
    }
    // as many waves on a compute unit as its 160 KB of LDS allow (a row is a chain of dependent steps, so what
    // counts is the number of rows in flight): two workgroups of 16 if they fit, else two of 8, else one of 16
    __host__ static ClusterLds choose(const ClusterLayout& y) {
        const ClusterLds big = make(y, 16), small = make(y, 8);
        if (2u * big.total <= 160u * 1024u) return big;
        return 2u * small.total <= 160u * 1024u ? small : big;
    }
};

__device__ __forceinline__ uint32_t cl_pk_min3(uint32_t a, uint32_t b, uint32_t c) {
    uint32_t r;
    asm("v_pk_minimum3_f16 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// C = |R'| = level - 1: the rows of the set's members sit in C registers, in the order of the members
template <int C>
__global__ __launch_bounds__(1024) void cluster_level_kernel(ClusterLayout y,
                                                             const unsigned char* __restrict__ ws,
                                                             uint16_t* __restrict__ rows, int pmax, int exact) {
    extern __shared__ __align__(16) unsigned char cl_smem[];
    constexpr int level = C + 1, CA = C > 0 ? C : 1;
    const int L = y.L, n = y.n, rd = y.rs / 2;
    const int inst = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same in all lanes: keeps the set in scalar registers
    const int threads = blockDim.x, waves = threads >> 6;
    const ClusterLds lds = ClusterLds::make(y, waves);
    const unsigned char* base = ws + (size_t)inst * y.stride;
    const uint32_t* q32 = reinterpret_cast<const uint32_t*>(cl_smem);
    const uint32_t* query = reinterpret_cast<const uint32_t*>(cl_smem + lds.hi_off);
    uint16_t* run = reinterpret_cast<uint16_t*>(cl_smem + lds.run_off) + wave * (kClRunLevels * kClRunRow);
    uint32_t* A32 = reinterpret_cast<uint32_t*>(rows) + (size_t)inst * (y.rows_per_instance() * rd);
    const bool more = n - level + 1 < pmax;   // segments up to and including this row's: n - level + 1
    // quotient rows and window queries: a straight copy of the image the tables kernels left (16 bytes a thread)
    {
        const uint4* img = reinterpret_cast<const uint4*>(base + y.img_off);
        uint4* dst = reinterpret_cast<uint4*>(cl_smem);
        const int qrows16 = (int)(lds.hi_off / 16u);
        const int first = more ? 0 : qrows16, count = qrows16 + n * 32;   // the quotient rows only if used
        for (int i = first + tid; i < count; i += threads) dst[i] = img[i];
    }
    // entries 128.. of the run-minimum rows never change: rest[L] = 0 if L = 128, +inf beyond the chain
    for (int i = lane; i < kClRunLevels * (kClRunRow - 128); i += 64) {
        const int k = i / (kClRunRow - 128), e = 128 + i % (kClRunRow - 128);
        run[k * kClRunRow + e] = (uint16_t)(e == L ? kClZero : kClInf);
    }
    __syncthreads();
    const uint32_t inf2 = kClInf | (kClInf << 16);
    const uint32_t all = (1u << n) - 1u;
    const int e0 = 2 * lane, e1 = e0 + 1;
    // rest[L] = 0: the half of entry L is cleared and set to the code of 0
    const uint32_t end_keep = (e0 == L ? 0u : 0xFFFFu) | (e1 == L ? 0u : 0xFFFF0000u);
    const uint32_t end_set = (e0 == L ? kClZero : 0u) | (e1 == L ? kClZero << 16 : 0u);
    const uint32_t after_last = L == 128 ? kClZero : kClInf;   // entry 128 of rest
    uint32_t* run32 = reinterpret_cast<uint32_t*>(run);
    // A wave takes a run of consecutive sets: the first from its index (binomial table, a chain of dependent
    // scalar loads), each further one from the one before (the next larger number with as many bits set).
    const uint32_t nsets = kClBinomials.c[n][C];
    const uint32_t total_waves = gridDim.x * waves;
    const uint32_t per_wave = (nsets + total_waves - 1u) / total_waves;
    uint32_t u = (blockIdx.x * waves + wave) * per_wave;
    const uint32_t u_end = u + per_wave < nsets ? u + per_wave : nsets;
    uint32_t mp = 0, first_row = 0;
    if (u < u_end) mp = cluster_set_at(u, C, n, first_row);
    for (; u < u_end; ++u) {
        uint32_t a[CA];      // row A[R'][member m], two entries per lane
        uint32_t moff[CA];   // dword offset of member m's quotient row from the row of (j, 0)
        {
            const uint32_t* arow = A32 + (size_t)(first_row * (uint32_t)rd) + lane;   // 32 bits hold an instance's dwords
            uint32_t bits = mp;
#pragma unroll
            for (int m = 0; m < C; ++m) {
                moff[m] = (uint32_t)(__ffs(bits) - 1) * (uint32_t)rd;
                bits &= bits - 1u;
                a[m] = (more && lane < rd) ? arow[m * rd] : inf2;
            }
        }
        // with every node to be used (exact), the chain may end (rest[L] = 0) only after the last node
        const bool may_end = !exact || mp == 0u;
        const uint32_t keep_here = may_end ? end_keep : 0xFFFFFFFFu, set_here = may_end ? end_set : 0u;
        const uint32_t after_here = may_end ? after_last : kClInf;
        if (exact && L == 128) {   // rest[L] sits in the constant part of the run-minimum rows
            if (lane < kClRunLevels) run[lane * kClRunRow + 128] = (uint16_t)after_here;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        // Where the rows of this set go: lane j works out the dword offset of row A[R' + j][j], once per set, and
        // the loop below picks it with a lane read instead of a dozen scalar instructions per row.  The first row
        // of R' + j from the first row of R' (j not in R'): the sets counted gain j's own term, and every member of
        // R' below j has one more member above it (their terms grow by 2^b each: `below` in all); then j's place
        // among the members.
        uint32_t out_off;
        {
            const uint32_t jl = (uint32_t)lane & 31u;
            const uint32_t below = mp & ((1u << jl) - 1u);
            const uint32_t above = (uint32_t)__popc((mp >> jl) >> 1);
            out_off = (first_row + (above << jl) + ((jl << jl) >> 1) + below + (uint32_t)__popc(below)) * (uint32_t)rd;
        }
        for (uint32_t jb = all & ~mp; jb; jb &= jb - 1u) {
            const int j = __ffs(jb) - 1;
            uint32_t v = inf2;
            if (more) {
                const uint32_t* qj = q32 + (j * n) * rd + lane;
                uint32_t x[CA];
#pragma unroll
                for (int m = 0; m < C; ++m) x[m] = cl_pk_max(qj[moff[m]], a[m]);
#pragma unroll
                for (int m = 0; m + 1 < C; m += 2) v = cl_pk_min3(v, x[m], x[m + 1]);
                if (C & 1) v = cl_pk_min(v, x[C - 1]);
            }
            v = (v & keep_here) | set_here;
            // minima over runs of 2^k entries starting at each entry
            run32[lane] = v;
            // the dword of the next lane (wave shift left by one: lane i reads lane i + 1; lane 63 keeps the
            // first operand, the entry after the last one)
            const uint32_t next = (uint32_t)__builtin_amdgcn_update_dpp((int)after_here, (int)v, 0x130, 0xF, 0xF, false);
            uint32_t cur = cl_pk_min(v, (v >> 16) | (next << 16));
            run32[(kClRunRow / 2) + lane] = cur;
            {
                // runs of 4 and of 8: the dwords one and two lanes up come by wave shifts too; what enters at
                // lane 63 are the entries 128 .. 131 of the row before, known beforehand
                const uint32_t tail = after_here | (kClInf << 16);
                const uint32_t up1 = (uint32_t)__builtin_amdgcn_update_dpp((int)tail, (int)cur, 0x130, 0xF, 0xF, false);
                cur = cl_pk_min(cur, up1);
                run32[2 * (kClRunRow / 2) + lane] = cur;
                const uint32_t s1 = (uint32_t)__builtin_amdgcn_update_dpp((int)tail, (int)cur, 0x130, 0xF, 0xF, false);
                const uint32_t up2 = (uint32_t)__builtin_amdgcn_update_dpp((int)inf2, (int)s1, 0x130, 0xF, 0xF, false);
                cur = cl_pk_min(cur, up2);
                run32[3 * (kClRunRow / 2) + lane] = cur;
            }
#pragma unroll
            for (int k = 4; k < kClRunLevels; ++k) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                cur = cl_pk_min(cur, run32[(k - 1) * (kClRunRow / 2) + lane + (1 << (k - 2))]);
                run32[k * (kClRunRow / 2) + lane] = cur;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            const uint2 qd = *reinterpret_cast<const uint2*>(query + j * kClQueryRow + e0);
            const unsigned char* runb = reinterpret_cast<const unsigned char*>(run);
            uint32_t res[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t d = h ? qd.y : qd.x;
                const uint32_t r1 = *reinterpret_cast<const uint16_t*>(runb + (d & 0xFFFFu));
                const uint32_t r2 = *reinterpret_cast<const uint16_t*>(runb + (d >> 16));
                res[h] = r1 < r2 ? r1 : r2;
            }
            // row of j within R' + j: after the members below it
            const uint32_t row_off = (uint32_t)__builtin_amdgcn_readlane((int)out_off, j);
            if (lane < rd) A32[(size_t)row_off + lane] = res[0] | (res[1] << 16);
            __builtin_amdgcn_wave_barrier();
        }
        if (C > 0 && u + 1u < u_end) {
            const uint32_t low = mp & (0u - mp), up = mp + low;
            mp = (((up ^ mp) >> 2) >> (__ffs(mp) - 1)) | up;
            first_row = 0;
            uint32_t above = 0;
            for (uint32_t bits = mp; bits; ++above) {
                const int b = 31 - __clz(bits);
                bits ^= 1u << b;
                first_row += (above << b) + (((uint32_t)b << b) >> 1);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// The optimum, the smallest optimal sequence and its cuts: one workgroup per instance.  With beta* known
// (the least A[All][j][0]) every further question is a yes or no, "can this be done with all links at most
// beta*", so the walk keeps sets of cuts as bit masks: F = cuts that the chosen prefix reaches (all its links
// at most beta*), G_j = those of F whose link into candidate j is at most beta*.  Candidate j at a position
// completes to an optimum iff A[unused][j][e] <= beta* for some e in G_j (one row of A, one wave per
// candidate); the smallest such node is taken, and F for the next position is the set of cuts that a window
// of that node starting in G_j covers.  hi[j][.] does not decrease, so the latest start below a cut decides.
// ---------------------------------------------------------------------------------------------
constexpr int kClTraceWaves = 16;   // at most; a launch uses min(n, 16) waves per workgroup

__global__ __launch_bounds__(kClTraceWaves * 64) void cluster_trace_kernel(ClusterLayout y,
                                                                          const unsigned char* __restrict__ ws,
                                                                          const uint16_t* __restrict__ rows, int pmax,
                                                                          int exact,
                                                                          unsigned long long* __restrict__ key_out,
                                                                          float* __restrict__ beta_out,
                                                                          int32_t* __restrict__ segs_out,
                                                                          int32_t* __restrict__ cuts_out,
                                                                          int32_t* __restrict__ order_out) {
    __shared__ unsigned char hi_s[PPO_CLUSTER_MAX_N * (PPO_MAX_L + 1)];
    __shared__ unsigned long long cand_s[PPO_CLUSTER_MAX_N][2];    // G_j of every candidate of this position
    __shared__ unsigned long long start_s[PPO_CLUSTER_MAX_N][2];   // G of the node chosen at every position
    __shared__ uint32_t ok_s[PPO_CLUSTER_MAX_N];
    __shared__ int seq[PPO_CLUSTER_MAX_N];
    const int L = y.L, n = y.n, inst = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const unsigned char* base = ws + (size_t)inst * y.stride;
    const uint16_t* __restrict__ qc = reinterpret_cast<const uint16_t*>(base + y.qc_off);
    const float* __restrict__ dec = reinterpret_cast<const float*>(base + y.dec_off);
    const uint16_t* A = rows + (size_t)inst * (y.rows_per_instance() * y.rs);
    // either the key alone (exact: bits of beta, rank of the permutation) or beta, segments, cuts, order
    float* beta = beta_out ? beta_out + inst : nullptr;
    int32_t* order = order_out ? order_out + (size_t)inst * n : nullptr;
    int32_t* cuts = cuts_out ? cuts_out + (size_t)inst * (n - 1) : nullptr;
    const int threads = blockDim.x, waves = threads >> 6;
    for (int i = tid; i < n * (L + 1); i += threads) hi_s[i] = base[y.hi_off + i];
    if (order)
        for (int i = tid; i < n; i += threads) order[i] = -1;
    if (cuts)
        for (int i = tid; i < n - 1; i += threads) cuts[i] = -1;
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
    // every wave takes the minimum itself: the same value in all of them
    const uint32_t best = wave_min(lane < n ? (uint32_t)A[((size_t)cluster_first_row(all, n) + lane) * y.rs] : kClInf);
    if (best >= kClInf) {
        if (tid == 0) {
            if (key_out) key_out[inst] = (unsigned long long)kInfBits << 32;
            if (beta) *beta = __uint_as_float(kInfBits);
            if (segs_out) segs_out[inst] = 0;
        }
        return;
    }
    // is cut e2 (1 <= e2 <= L) inside the window of node j that starts at the latest cut of (g0, g1) below e2?
    auto covered = [&](unsigned long long g0, unsigned long long g1, int j, int e2) -> bool {
        unsigned long long m0 = g0, m1 = 0;
        if (e2 < 64)
            m0 = g0 & ((1ull << e2) - 1ull);
        else
            m1 = e2 >= 128 ? g1 : g1 & ((1ull << (e2 - 64)) - 1ull);
        const int from = m1 ? 127 - __clzll((long long)m1) : m0 ? 63 - __clzll((long long)m0) : -1;
        return from >= 0 && hi(j, from) >= e2;
    };
    unsigned long long F0 = 1ull, F1 = 0ull;   // the first segment starts at 0
    uint32_t used = 0;
    int last = -1, p = 0;
    for (int s = 0; s < pmax; ++s) {
        const uint32_t unused = all & ~used;
        const uint32_t first_row = cluster_first_row(unused, n);
        for (int j = wave; j < n; j += waves) {
            if ((used >> j) & 1u) {
                if (lane == 0) ok_s[j] = 0u;
                continue;
            }
            const uint16_t* __restrict__ a = A + (size_t)(first_row + (uint32_t)__popc(unused & ((1u << j) - 1u))) * y.rs;
            const uint16_t* __restrict__ q = qc + (s ? pair_index(last, j, n) * L : 0);
            unsigned long long g[2], ok[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int e = lane + 64 * h;
                bool in_g = false, in_ok = false;
                if ((((h ? F1 : F0) >> lane) & 1ull) && e < L) {
                    in_g = s == 0 || (uint32_t)q[e - 1] <= best;   // beyond the first position F holds no cut 0
                    in_ok = in_g && (uint32_t)a[e] <= best;
                }
                g[h] = __ballot(in_g);
                ok[h] = __ballot(in_ok);
            }
            if (lane == 0) {
                cand_s[j][0] = g[0];
                cand_s[j][1] = g[1];
                ok_s[j] = (ok[0] | ok[1]) != 0ull ? 1u : 0u;
            }
        }
        __syncthreads();
        int chosen = -1;
        for (int j = n - 1; j >= 0; --j)
            if (ok_s[j]) chosen = j;
        if (chosen < 0) break;   // cannot happen: some completion of the prefix reaches `best`
        const unsigned long long G0 = cand_s[chosen][0], G1 = cand_s[chosen][1];
        if (tid == 0) {
            seq[s] = chosen;
            start_s[s][0] = G0;
            start_s[s][1] = G1;
        }
        // the prefix itself is optimal: it sorts before its extensions (exact: only a full permutation ends)
        const bool complete = exact ? s == n - 1 : covered(G0, G1, chosen, L);
        F0 = __ballot(lane >= 1 && lane < L && covered(G0, G1, chosen, lane));
        F1 = __ballot(lane + 64 < L && covered(G0, G1, chosen, lane + 64));
        __syncthreads();
        used |= 1u << chosen;
        last = chosen;
        p = s + 1;
        if (complete) break;
    }
    if (wave != 0) return;
    if (key_out && lane == 0) {
        // lexicographic rank of the permutation: digit s counts the smaller nodes not used before position s
        uint32_t rank = 0, seen = 0;
        for (int s = 0; s < p; ++s) {
            rank += (uint32_t)__popc(~seen & ((1u << seq[s]) - 1u)) * factorial_u32(n - 1 - s);
            seen |= 1u << seq[s];
        }
        key_out[inst] = ((unsigned long long)__float_as_uint(dec[best - kClZero]) << 32) | rank;
    }
    if (!cuts && !beta) return;
    // cuts: latest segment first, each time the smallest start (reached by the prefix, link at most beta*)
    // whose window covers the end
    int e = L;
    for (int s = p - 1; s >= 1 && cuts; --s) {
        const int js = seq[s];
        const unsigned long long m0 = __ballot(((start_s[s][0] >> lane) & 1ull) && lane < e && hi(js, lane) >= e);
        const unsigned long long m1 =
            __ballot(((start_s[s][1] >> lane) & 1ull) && lane + 64 < e && hi(js, lane + 64 < L ? lane + 64 : L) >= e);
        if (!(m0 | m1)) break;   // cannot happen: e was reached from such a start
        const int first = m0 ? __ffsll((long long)m0) - 1 : 63 + __ffsll((long long)m1);
        if (lane == 0) cuts[s - 1] = (int32_t)first;
        e = first;
    }
    if (lane == 0) {
        if (beta) *beta = dec[best - kClZero];
        if (segs_out) segs_out[inst] = p;
        if (order)
            for (int s = 0; s < p; ++s) order[s] = seq[s];
    }
}

// ---------------------------------------------------------------------------------------------
// The tables of this file from those of the fixed-k precompute kernel (window starts lo, quotient codes from
// kCodeZero + 1 up): hi[j][e] = last e' with lo[j][e'] <= e; codes and dec are the same.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void cluster_tables_from_prepared_kernel(Layout f, const unsigned char* __restrict__ fixed_ws,
                                                                           ClusterLayout y, unsigned char* __restrict__ ws) {
    const int L = y.L, n = y.n, inst = blockIdx.x, tid = threadIdx.x;
    const unsigned char* src = fixed_ws + (size_t)inst * f.stride;
    unsigned char* dst = ws + (size_t)inst * y.stride;
    __shared__ unsigned char lo[PPO_MAX_K * (PPO_MAX_L + 1)];
    for (int idx = tid; idx < n * (L + 1); idx += 256) lo[idx] = src[f.lo_off + idx];
    __syncthreads();
    for (int idx = tid; idx < n * (L + 1); idx += 256) {
        const int j = idx / (L + 1), e = idx - j * (L + 1);
        int e2 = e;
        while (e2 < L && lo[j * (L + 1) + e2 + 1] <= e) ++e2;
        dst[y.hi_off + idx] = (unsigned char)e2;
    }
    const uint16_t* qsrc = reinterpret_cast<const uint16_t*>(src + f.qc_off);
    uint16_t* qdst = reinterpret_cast<uint16_t*>(dst + y.qc_off);
    for (int idx = tid; idx < y.npairs * L; idx += 256) {
        const int i = idx % L;
        qdst[idx] = (uint16_t)(i < L - 1 ? qsrc[idx] : kClInf);
    }
    const float* dsrc = reinterpret_cast<const float*>(src + f.dec_off);
    float* ddst = reinterpret_cast<float*>(dst + y.dec_off);
    for (int idx = tid; idx <= y.nq; idx += 256) ddst[idx] = dsrc[idx];
}

// The image of the level kernel's LDS tables (needs hi and the codes): one workgroup per instance.
//   quotient rows: entry e of the row of (j, j''): q_{j,j''}[e-1] for 1 <= e <= L-1 (the cuts with a link), else +inf;
//   window queries: the window (e, hi[j][e]] of node j at entry e is covered by two runs of 2^k entries, k the
//   largest with 2^k <= its length: the one starting at e + 1 and the one ending at hi.  The table holds the byte
//   offsets of their minima within a wave's run-minimum rows, 16 bits each; no window: twice an entry that is +inf.
__global__ __launch_bounds__(kClPreThreads) void cluster_image_kernel(ClusterLayout y, unsigned char* __restrict__ ws) {
    const int L = y.L, n = y.n, inst = blockIdx.x, tid = threadIdx.x;
    unsigned char* base = ws + (size_t)inst * y.stride;
    const uint16_t* __restrict__ qc = reinterpret_cast<const uint16_t*>(base + y.qc_off);
    uint16_t* q16 = reinterpret_cast<uint16_t*>(base + y.img_off);
    uint32_t* query = reinterpret_cast<uint32_t*>(base + y.img_off + ClusterLayout::q_image_bytes(n, y.rs));
    for (int i = tid; i < (int)(ClusterLayout::q_image_bytes(n, y.rs) / 2); i += kClPreThreads) {
        const int e = i % y.rs, jj = i / y.rs, j = jj / n, j2 = jj - j * n;   // jj = n * n: the padding
        q16[i] = (uint16_t)((jj < n * n && j != j2 && e >= 1 && e <= L - 1) ? qc[pair_index(j, j2, n) * L + e - 1] : kClInf);
    }
    for (int i = tid; i < n * kClQueryRow; i += kClPreThreads) {
        const int j = i / kClQueryRow, e = i - j * kClQueryRow;
        const int top = e < L ? (int)base[y.hi_off + j * (L + 1) + e] : 0;
        uint32_t o1 = kClRunRow - 2, o2 = kClRunRow - 2;   // run row 0, beyond the chain
        if (top > e) {
            int k = 31 - __clz(top - e);
            k = k > kClRunLevels - 1 ? kClRunLevels - 1 : k;
            o1 = (uint32_t)(k * kClRunRow + e + 1);
            o2 = (uint32_t)(k * kClRunRow + top - (1 << k) + 1);
        }
        query[i] = (o1 * 2u) | ((o2 * 2u) << 16);
    }
}

hipError_t launch_cluster_tables(const float* t, const float* m, const float* M, const float* B, int L, int n,
                                 int n_inst, void* ws, hipStream_t stream) {
    const ClusterLayout y = ClusterLayout::make(L, n);
    unsigned char* w = static_cast<unsigned char*>(ws);
    hipLaunchKernelGGL(cluster_tables_kernel, dim3(n_inst), dim3(kClPreThreads), 0, stream, t, m, M, B, y, w);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (y.nq > 0) {
        const int slices = (y.nq + kClCountThreads - 1) / kClCountThreads;
        const uint32_t lds_bytes = (uint32_t)y.nq * 4u;
        static std::atomic<uint64_t> lds_allowed{0};
        e = allow_full_lds(reinterpret_cast<const void*>(&cluster_count_kernel), lds_allowed);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(cluster_count_kernel, dim3(slices, n_inst), dim3(kClCountThreads), lds_bytes, stream, y, w);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(cluster_image_kernel, dim3(n_inst), dim3(kClPreThreads), 0, stream, y, w);
    return hipGetLastError();
}

// rows of `n_inst` instances (tables at ws, rows at `rows`), levels n - pmax + 1 .. n, then the trace
// one instantiation of the level kernel per set size
using ClLevelLaunch = hipError_t (*)(dim3, dim3, uint32_t, hipStream_t, const ClusterLayout&, const unsigned char*,
                                     uint16_t*, int, int);
template <int C>
static hipError_t cluster_launch_level(dim3 grid, dim3 block, uint32_t lds_bytes, hipStream_t stream, const ClusterLayout& y,
                                       const unsigned char* ws, uint16_t* rows, int pmax, int exact) {
    static std::atomic<uint64_t> lds_allowed{0};
    const hipError_t e = allow_full_lds(reinterpret_cast<const void*>(&cluster_level_kernel<C>), lds_allowed);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(cluster_level_kernel<C>, grid, block, lds_bytes, stream, y, ws, rows, pmax, exact);
    return hipGetLastError();
}
template <int... Cs>
static constexpr std::array<ClLevelLaunch, sizeof...(Cs)> cluster_level_table(std::integer_sequence<int, Cs...>) {
    return {{&cluster_launch_level<Cs>...}};
}
static const std::array<ClLevelLaunch, PPO_CLUSTER_MAX_N> kClLevelLaunch =
    cluster_level_table(std::make_integer_sequence<int, PPO_CLUSTER_MAX_N>{});

// exact: every node has to be used (pmax = n); key_out (may be null): bits of beta and rank of the permutation
hipError_t launch_cluster_solve(int L, int n, int n_inst, int pmax, bool exact, const void* ws, void* rows,
                                uint64_t* key_out, float* beta_out, int32_t* segs_out, int32_t* cuts_out,
                                int32_t* order_out, hipStream_t stream) {
    const ClusterLayout y = ClusterLayout::make(L, n);
    const unsigned char* w = static_cast<const unsigned char*>(ws);
    uint16_t* r = static_cast<uint16_t*>(rows);
    const ClusterLds lds = ClusterLds::choose(y);
    const uint32_t per_cu = (160u * 1024u) / lds.total;   // workgroups a compute unit holds: 1 or 2 (or more for small n)
    const uint32_t resident = 256u * (per_cu < 1u ? 1u : per_cu > 4u ? 4u : per_cu);
    hipError_t e = hipSuccess;
    for (int level = n - pmax + 1; level <= n; ++level) {
        // a set per wave at most; no more workgroups than stay resident (each stages the quotient table once)
        uint32_t blocks = (kClBinomialsHost.c[n][level - 1] + (uint32_t)lds.waves - 1u) / (uint32_t)lds.waves;
        const uint32_t cap = (resident + (uint32_t)n_inst - 1u) / (uint32_t)n_inst;
        if (blocks > cap) blocks = cap;
        e = kClLevelLaunch[level - 1](dim3(blocks, n_inst), dim3(lds.waves * 64), lds.total, stream, y, w, r, pmax,
                                      exact ? 1 : 0);
        if (e != hipSuccess) return e;
    }
    const int trace_waves = n < kClTraceWaves ? n : kClTraceWaves;   // one wave per candidate node
    hipLaunchKernelGGL(cluster_trace_kernel, dim3(n_inst), dim3(trace_waves * 64), 0, stream, y, w, r, pmax,
                       exact ? 1 : 0, reinterpret_cast<unsigned long long*>(key_out), beta_out, segs_out, cuts_out,
                       order_out);
    return hipGetLastError();
}

hipError_t launch_cluster_tables_from_prepared(const Layout& f, const void* fixed_ws, int n_inst, void* ws,
                                               hipStream_t stream) {
    const ClusterLayout y = ClusterLayout::make(f.L, f.k);
    hipLaunchKernelGGL(cluster_tables_from_prepared_kernel, dim3(n_inst), dim3(256), 0, stream, f,
                       static_cast<const unsigned char*>(fixed_ws), y, static_cast<unsigned char*>(ws));
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(cluster_image_kernel, dim3(n_inst), dim3(kClPreThreads), 0, stream, y, static_cast<unsigned char*>(ws));
    return hipGetLastError();
}

}  // namespace ppo
