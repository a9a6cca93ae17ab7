// C ABI of the ppo library (declared in include/ppo.h): argument checks, workspace carving, launches.
#include <mutex>
#include <string>

#include "ppo_common.h"

namespace ppo {
hipError_t launch_precompute(const float*, const float*, const float*, const float*, const Layout&, int, void*,
                             hipStream_t);
hipError_t launch_init_keys(uint64_t*, int, hipStream_t);
hipError_t launch_enumerate(const Layout&, int, const void*, uint32_t, uint32_t, uint64_t*, float*, bool, uint64_t*,
                            hipStream_t);
hipError_t launch_traceback(const Layout&, int, const void*, const uint64_t*, float*, int32_t*, int32_t*,
                            hipStream_t);
void set_enumeration_variant(int);
size_t cluster_tables_bytes(int L, int n);
bool cluster_few_supported(int L, int n, int pmax);
size_t cluster_few_tables_bytes(int L, int n, int pmax);
size_t cluster_few_rows_bytes(int L, int n, int pmax);
hipError_t launch_cluster_few_tables(const float*, const float*, const float*, const float*, int, int, int, int, void*, void*,
                                     hipStream_t);
hipError_t launch_cluster_few_solve(int, int, int, int, void*, void*, float*, int32_t*, int32_t*, int32_t*, hipStream_t);
size_t cluster_rows_bytes(int L, int n);
hipError_t launch_cluster_tables(const float*, const float*, const float*, const float*, int, int, int, void*,
                                 hipStream_t);
hipError_t launch_cluster_solve(int, int, int, int, bool, const void*, void*, uint64_t*, float*, int32_t*, int32_t*,
                                int32_t*, hipStream_t);
hipError_t launch_cluster_tables_from_prepared(const Layout&, const void*, int, void*, hipStream_t);
hipError_t launch_min_sum_partition(const float*, const float*, int, const float*, int, int32_t*, int32_t*, double*,
                                    hipStream_t);
hipError_t launch_valu_probe(int, int, uint32_t*, hipStream_t);
hipError_t launch_heuristic(const float*, const float*, int, const float*, const float*, int, int, int, int, const float*,
                            int, const int32_t*, const int32_t*, float*, int32_t*, int32_t*, int32_t*, int32_t*, hipStream_t);
size_t ct_tables_bytes(int L, int k);
hipError_t launch_ct_tables(const float*, const float*, const float*, const float*, const float*, const float*, int, int,
                            int, void*, hipStream_t);
hipError_t launch_ct_enumerate(int, int, int, const void*, uint32_t, uint32_t, uint64_t*, float*, hipStream_t);
hipError_t launch_ct_traceback(int, int, int, const void*, const uint64_t*, float*, int32_t*, int32_t*, hipStream_t);
}  // namespace ppo

namespace {

thread_local std::string g_hip_error = "no HIP error recorded";

int hip_fail(hipError_t e, const char* where) {
    g_hip_error = std::string("HIP error in ") + where + ": " + hipGetErrorString(e);
    return PPO_EHIP;
}

#define PPO_HIP(call, where)                            \
    do {                                                \
        hipError_t e_ = (call);                         \
        if (e_ != hipSuccess) return hip_fail(e_, where); \
    } while (0)

int check_shape(int L, int k, int n_inst) {
    if (L < 1 || k < 1 || k > L || n_inst < 0) return PPO_EINVAL;
    if (k > PPO_MAX_K || L > PPO_MAX_L) return PPO_ETOOBIG;
    return PPO_OK;
}

// One launch covers at most this many instances (grid y dimension).
constexpr int kInstPerLaunch = 32768;

size_t tables_bytes(const ppo::Layout& y, int n_inst) { return (size_t)y.stride * (size_t)n_inst; }

int run_prepare(const float* t, const float* m, int L, const float* M, const float* B, int k, int n_inst, void* ws,
                hipStream_t stream) {
    const ppo::Layout y = ppo::Layout::make(L, k);
    for (int first = 0; first < n_inst; first += kInstPerLaunch) {
        const int n = (n_inst - first < kInstPerLaunch) ? n_inst - first : kInstPerLaunch;
        unsigned char* wsi = static_cast<unsigned char*>(ws) + (size_t)first * y.stride;
        PPO_HIP(ppo::launch_precompute(t + (size_t)first * L, m + (size_t)first * L, M + (size_t)first * k,
                                       B + (size_t)first * k * k, y, n, wsi, stream),
                "precompute launch");
    }
    return PPO_OK;
}

int run_range(int L, int k, int n_inst, const void* ws, uint32_t rank_begin, uint32_t rank_end, uint64_t* best_key,
              bool shared_prefix, uint64_t* skipped_groups, hipStream_t stream) {
    const ppo::Layout y = ppo::Layout::make(L, k);
    for (int first = 0; first < n_inst; first += kInstPerLaunch) {
        const int n = (n_inst - first < kInstPerLaunch) ? n_inst - first : kInstPerLaunch;
        const unsigned char* wsi = static_cast<const unsigned char*>(ws) + (size_t)first * y.stride;
        PPO_HIP(ppo::launch_enumerate(y, n, wsi, rank_begin, rank_end, best_key + first, nullptr, shared_prefix,
                                      skipped_groups ? skipped_groups + first : nullptr, stream),
                "enumerate launch");
    }
    return PPO_OK;
}

int run_finalize(int L, int k, int n_inst, const void* ws, const uint64_t* best_key, float* beta_out,
                 int32_t* cuts_out, int32_t* order_out, hipStream_t stream) {
    const ppo::Layout y = ppo::Layout::make(L, k);
    for (int first = 0; first < n_inst; first += kInstPerLaunch) {
        const int n = (n_inst - first < kInstPerLaunch) ? n_inst - first : kInstPerLaunch;
        const unsigned char* wsi = static_cast<const unsigned char*>(ws) + (size_t)first * y.stride;
        PPO_HIP(ppo::launch_traceback(y, n, wsi, best_key + first, beta_out + first,
                                      cuts_out + (size_t)first * (k - 1), order_out + (size_t)first * k, stream),
                "traceback launch");
    }
    return PPO_OK;
}

}  // namespace

// The kernels read the tables with 16-byte loads at offsets that are multiples of 16 within the workspace
// and update the keys with 64-bit atomics: pointers that break these alignments are refused here.
static bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }
static bool bad_workspace(const void* ws) { return !ws || misaligned(ws, 256); }
static bool bad_keys(const void* keys) { return !keys || misaligned(keys, 8); }

extern "C" {

int ppo_version(void) { return 204; }

int ppo_set_enumeration(int variant) {
    if (variant != PPO_ENUM_AUTO && variant != PPO_ENUM_GENERIC && variant != PPO_ENUM_GROUPED) return PPO_EINVAL;
    ppo::set_enumeration_variant(variant);
    return PPO_OK;
}

const char* ppo_strerror(int code) {
    switch (code) {
        case PPO_OK: return "ok";
        case PPO_EINVAL: return "invalid argument";
        case PPO_ETOOBIG: return "k or L beyond the compiled limits";
        case PPO_EHIP: return g_hip_error.c_str();
        case PPO_ENOSPC: return "workspace too small";
        default: return "unknown ppo error code";
    }
}

size_t ppo_workspace_bytes(int L, int k, int n_inst) {
    if (check_shape(L, k, n_inst) != PPO_OK) return 0;
    const ppo::Layout y = ppo::Layout::make(L, k);
    // tables of every instance, then one key per instance (used by ppo_solve_ws)
    return tables_bytes(y, n_inst) + ppo::align_up((size_t)n_inst * sizeof(uint64_t), 256);
}

int ppo_prepare(const float* t, const float* m, int L, const float* M, const float* B, int k, int n_inst,
                void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_shape(L, k, n_inst);
    if (rc) return rc;
    if (n_inst == 0) return PPO_OK;
    if (!t || !m || !M || !B || bad_workspace(workspace)) return PPO_EINVAL;
    if (workspace_bytes < ppo_workspace_bytes(L, k, n_inst)) return PPO_ENOSPC;
    return run_prepare(t, m, L, M, B, k, n_inst, workspace, static_cast<hipStream_t>(stream));
}

int ppo_init_keys(uint64_t* best_key, int n_inst, void* stream) {
    if (n_inst < 0) return PPO_EINVAL;
    if (n_inst == 0) return PPO_OK;
    if (bad_keys(best_key)) return PPO_EINVAL;
    PPO_HIP(ppo::launch_init_keys(best_key, n_inst, static_cast<hipStream_t>(stream)), "init_keys launch");
    return PPO_OK;
}

int ppo_solve_range(int L, int k, int n_inst, const void* workspace, size_t workspace_bytes, uint64_t rank_begin,
                    uint64_t rank_end, uint64_t* best_key, void* stream) {
    int rc = check_shape(L, k, n_inst);
    if (rc) return rc;
    if (rank_begin > rank_end || rank_end > (uint64_t)ppo::factorial_u32(k)) return PPO_EINVAL;
    if (n_inst == 0) return PPO_OK;
    if (bad_keys(best_key) || bad_workspace(workspace)) return PPO_EINVAL;
    if (workspace_bytes < ppo_workspace_bytes(L, k, n_inst)) return PPO_ENOSPC;
    return run_range(L, k, n_inst, workspace, (uint32_t)rank_begin, (uint32_t)rank_end, best_key, false, nullptr,
                     static_cast<hipStream_t>(stream));
}

int ppo_solve_range_bounded(int L, int k, int n_inst, const void* workspace, size_t workspace_bytes,
                            uint64_t rank_begin, uint64_t rank_end, uint64_t* best_key, uint64_t* skipped_groups,
                            void* stream) {
    int rc = check_shape(L, k, n_inst);
    if (rc) return rc;
    if (rank_begin > rank_end || rank_end > (uint64_t)ppo::factorial_u32(k)) return PPO_EINVAL;
    if (n_inst == 0) return PPO_OK;
    if (bad_keys(best_key) || bad_workspace(workspace) || (skipped_groups && misaligned(skipped_groups, 8))) return PPO_EINVAL;
    if (workspace_bytes < ppo_workspace_bytes(L, k, n_inst)) return PPO_ENOSPC;
    return run_range(L, k, n_inst, workspace, (uint32_t)rank_begin, (uint32_t)rank_end, best_key, true, skipped_groups,
                     static_cast<hipStream_t>(stream));
}

int ppo_solve_subsets(int L, int k, int n_inst, const void* workspace, size_t workspace_bytes, uint64_t* best_key,
                      void* stream) {
    int rc = check_shape(L, k, n_inst);
    if (rc) return rc;
    if (n_inst == 0) return PPO_OK;
    if (bad_keys(best_key) || bad_workspace(workspace)) return PPO_EINVAL;
    if (workspace_bytes < ppo_workspace_bytes(L, k, n_inst)) return PPO_ENOSPC;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const ppo::Layout y = ppo::Layout::make(L, k);
    // the engine of the cluster form with every node to be used: its own copy of the tables and the DP rows,
    // for as many instances at a time as fit in 1 GiB
    const size_t tables = ppo::cluster_tables_bytes(L, k), rows = ppo::cluster_rows_bytes(L, k);
    size_t batch = ((size_t)1 << 30) / (tables + rows);
    if (batch < 1) batch = 1;
    if (batch > (size_t)n_inst) batch = (size_t)n_inst;
    if (batch > (size_t)kInstPerLaunch) batch = (size_t)kInstPerLaunch;
    unsigned char* scratch = nullptr;
    PPO_HIP(hipMallocAsync(reinterpret_cast<void**>(&scratch), (tables + rows) * batch, s), "hipMallocAsync (subset DP rows)");
    hipError_t e = hipSuccess;
    for (size_t first = 0; first < (size_t)n_inst && e == hipSuccess; first += batch) {
        const int n = (int)(((size_t)n_inst - first < batch) ? (size_t)n_inst - first : batch);
        e = ppo::launch_cluster_tables_from_prepared(y, static_cast<const unsigned char*>(workspace) + first * y.stride, n,
                                                     scratch, s);
        if (e == hipSuccess)
            e = ppo::launch_cluster_solve(L, k, n, k, true, scratch, scratch + tables * batch, best_key + first, nullptr,
                                          nullptr, nullptr, nullptr, s);
    }
    const hipError_t e2 = hipFreeAsync(scratch, s);
    PPO_HIP(e, "subset DP launch");
    PPO_HIP(e2, "hipFreeAsync (subset DP rows)");
    return PPO_OK;
}

static int check_cluster_shape(int L, int n, int n_inst) {
    if (L < 1 || n < 1 || n_inst < 0) return PPO_EINVAL;
    if (n > PPO_CLUSTER_MAX_N || L > PPO_MAX_L) return PPO_ETOOBIG;
    return PPO_OK;
}

size_t ppo_cluster_workspace_bytes(int L, int n, int n_inst) {
    if (check_cluster_shape(L, n, n_inst) != PPO_OK) return 0;
    const size_t rows = ppo::cluster_rows_bytes(L, n);
    size_t together = ((size_t)16 << 30) / rows;
    if (together < 1) together = 1;
    if (together > (size_t)n_inst) together = (size_t)n_inst;
    return ppo::cluster_tables_bytes(L, n) * (size_t)n_inst + rows * together;
}

int ppo_solve_cluster(const float* t, const float* m, int L, const float* M, const float* B, int n, int n_inst,
                      int max_segments, float* beta_out, int32_t* segs_out, int32_t* cuts_out, int32_t* order_out,
                      void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_cluster_shape(L, n, n_inst);
    if (rc) return rc;
    if (max_segments < 1 || max_segments > n) return PPO_EINVAL;
    if (n_inst == 0) return PPO_OK;
    if (!t || !m || !M || !B || !beta_out || !segs_out || !order_out || (n > 1 && !cuts_out) || bad_workspace(workspace))
        return PPO_EINVAL;
    const size_t tables = ppo::cluster_tables_bytes(L, n), rows = ppo::cluster_rows_bytes(L, n);
    if (workspace_bytes < tables * (size_t)n_inst + rows) return PPO_ENOSPC;
    size_t together = (workspace_bytes - tables * (size_t)n_inst) / rows;
    if (together > (size_t)kInstPerLaunch) together = (size_t)kInstPerLaunch;
    if (together > (size_t)n_inst) together = (size_t)n_inst;
    hipStream_t s = static_cast<hipStream_t>(stream);
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    unsigned char* row_area = ws + tables * (size_t)n_inst;   // tables is a multiple of 256
    const int pmax = max_segments < L ? max_segments : L;
    for (int first = 0; first < n_inst; first += kInstPerLaunch) {
        const int cnt = n_inst - first < kInstPerLaunch ? n_inst - first : kInstPerLaunch;
        PPO_HIP(ppo::launch_cluster_tables(t + (size_t)first * L, m + (size_t)first * L, M + (size_t)first * n,
                                           B + (size_t)first * n * n, L, n, cnt, ws + tables * (size_t)first, s),
                "cluster tables launch");
    }
    for (size_t first = 0; first < (size_t)n_inst; first += together) {
        const int cnt = (int)(((size_t)n_inst - first < together) ? (size_t)n_inst - first : together);
        PPO_HIP(ppo::launch_cluster_solve(L, n, cnt, pmax, false, ws + tables * first, row_area, nullptr, beta_out + first,
                                          segs_out + first, cuts_out ? cuts_out + first * (size_t)(n - 1) : nullptr,
                                          order_out + first * (size_t)n, s),
                "cluster DP launch");
    }
    return PPO_OK;
}

static int check_few_shape(int L, int n, int max_segments, int n_inst) {
    if (L < 1 || n < 1 || n_inst < 0 || max_segments < 1 || max_segments > n) return PPO_EINVAL;
    if (L > PPO_MAX_L || n > PPO_CLUSTER_FEW_MAX_N) return PPO_ETOOBIG;
    const int pmax = max_segments < L ? max_segments : L;
    if (pmax > PPO_CLUSTER_FEW_MAX_SEGMENTS || !ppo::cluster_few_supported(L, n, pmax)) return PPO_ETOOBIG;
    return PPO_OK;
}

size_t ppo_cluster_few_workspace_bytes(int L, int n, int max_segments, int n_inst) {
    if (check_few_shape(L, n, max_segments, n_inst) != PPO_OK) return 0;
    const int pmax = max_segments < L ? max_segments : L;
    const size_t rows = ppo::cluster_few_rows_bytes(L, n, pmax);
    size_t together = ((size_t)16 << 30) / rows;
    if (together < 1) together = 1;
    if (together > (size_t)n_inst) together = (size_t)n_inst;
    if (together < 1) together = 1;
    return ppo::cluster_few_tables_bytes(L, n, pmax) * (size_t)(n_inst > 0 ? n_inst : 1) + rows * together;
}

int ppo_solve_cluster_few(const float* t, const float* m, int L, const float* M, const float* B, int n, int n_inst,
                          int max_segments, float* beta_out, int32_t* segs_out, int32_t* cuts_out, int32_t* order_out,
                          void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_few_shape(L, n, max_segments, n_inst);
    if (rc) return rc;
    if (n_inst == 0) return PPO_OK;
    if (!t || !m || !M || !B || !beta_out || !segs_out || !order_out || (n > 1 && !cuts_out) || bad_workspace(workspace))
        return PPO_EINVAL;
    const int pmax = max_segments < L ? max_segments : L;
    const size_t tables = ppo::cluster_few_tables_bytes(L, n, pmax), rows = ppo::cluster_few_rows_bytes(L, n, pmax);
    if (workspace_bytes < tables * (size_t)n_inst + rows) return PPO_ENOSPC;
    size_t together = (workspace_bytes - tables * (size_t)n_inst) / rows;
    if (together > (size_t)kInstPerLaunch) together = (size_t)kInstPerLaunch;
    if (together > (size_t)n_inst) together = (size_t)n_inst;
    hipStream_t s = static_cast<hipStream_t>(stream);
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    unsigned char* row_area = ws + tables * (size_t)n_inst;   // tables is a multiple of 256
    for (size_t first = 0; first < (size_t)n_inst; first += together) {
        const int cnt = (int)(((size_t)n_inst - first < together) ? (size_t)n_inst - first : together);
        // the tables kernel also writes the rows of the one-node sets, so it runs with the rows it belongs to
        PPO_HIP(ppo::launch_cluster_few_tables(t + first * L, m + first * L, M + first * n, B + first * n * n, L, n, pmax, cnt,
                                               ws + tables * first, row_area, s),
                "cluster tables launch");
        PPO_HIP(ppo::launch_cluster_few_solve(L, n, pmax, cnt, ws + tables * first, row_area, beta_out + first,
                                              segs_out + first, cuts_out ? cuts_out + first * (size_t)(n - 1) : nullptr,
                                              order_out + first * (size_t)n, s),
                "cluster DP launch");
    }
    return PPO_OK;
}

int ppo_min_sum_partition(const float* t, const float* m, int L, const float* kappa, int n_inst, int32_t* segs_out,
                          int32_t* cuts_out, double* sum_out, void* stream) {
    if (L < 1 || n_inst < 0) return PPO_EINVAL;
    if (L > PPO_MAX_L) return PPO_ETOOBIG;
    if (n_inst == 0) return PPO_OK;
    if (!t || !m || !kappa || !segs_out || !sum_out || (L > 1 && !cuts_out) || misaligned(sum_out, 8)) return PPO_EINVAL;
    for (int first = 0; first < n_inst; first += kInstPerLaunch) {
        const int cnt = n_inst - first < kInstPerLaunch ? n_inst - first : kInstPerLaunch;
        PPO_HIP(ppo::launch_min_sum_partition(t + (size_t)first * L, m + (size_t)first * L, L, kappa + first, cnt,
                                              segs_out + first, cuts_out ? cuts_out + (size_t)first * (L - 1) : nullptr,
                                              sum_out + first, static_cast<hipStream_t>(stream)),
                "min-sum partition launch");
    }
    return PPO_OK;
}

int ppo_finalize(int L, int k, int n_inst, const void* workspace, size_t workspace_bytes, const uint64_t* best_key,
                 float* beta_out, int32_t* cuts_out, int32_t* order_out, void* stream) {
    int rc = check_shape(L, k, n_inst);
    if (rc) return rc;
    if (n_inst == 0) return PPO_OK;
    if (bad_workspace(workspace) || bad_keys(best_key) || !beta_out || !order_out || (k > 1 && !cuts_out)) return PPO_EINVAL;
    if (workspace_bytes < ppo_workspace_bytes(L, k, n_inst)) return PPO_ENOSPC;
    return run_finalize(L, k, n_inst, workspace, best_key, beta_out, cuts_out, order_out,
                        static_cast<hipStream_t>(stream));
}

int ppo_solve_ws(const float* t, const float* m, int L, const float* M, const float* B, int k, int n_inst,
                 float* beta_out, int32_t* cuts_out, int32_t* order_out, void* workspace, size_t workspace_bytes,
                 void* stream) {
    int rc = check_shape(L, k, n_inst);
    if (rc) return rc;
    if (n_inst == 0) return PPO_OK;
    if (!t || !m || !M || !B || !beta_out || !order_out || (k > 1 && !cuts_out) || bad_workspace(workspace)) return PPO_EINVAL;
    if (workspace_bytes < ppo_workspace_bytes(L, k, n_inst)) return PPO_ENOSPC;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const ppo::Layout y = ppo::Layout::make(L, k);
    uint64_t* keys = reinterpret_cast<uint64_t*>(static_cast<unsigned char*>(workspace) + tables_bytes(y, n_inst));
    rc = run_prepare(t, m, L, M, B, k, n_inst, workspace, s);
    if (rc) return rc;
    PPO_HIP(ppo::launch_init_keys(keys, n_inst, s), "init_keys launch");
    rc = run_range(L, k, n_inst, workspace, 0u, ppo::factorial_u32(k), keys, false, nullptr, s);
    if (rc) return rc;
    return run_finalize(L, k, n_inst, workspace, keys, beta_out, cuts_out, order_out, s);
}

int ppo_solve(const float* t, const float* m, int L, const float* M, const float* B, int k, int n_inst,
              float* beta_out, int32_t* cuts_out, int32_t* order_out, void* stream) {
    int rc = check_shape(L, k, n_inst);
    if (rc) return rc;
    if (n_inst == 0) return PPO_OK;
    if (!t || !m || !M || !B || !beta_out || !order_out || (k > 1 && !cuts_out)) return PPO_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t bytes = ppo_workspace_bytes(L, k, n_inst);
    void* ws = nullptr;
    PPO_HIP(hipMallocAsync(&ws, bytes, s), "hipMallocAsync");
    rc = ppo_solve_ws(t, m, L, M, B, k, n_inst, beta_out, cuts_out, order_out, ws, bytes, stream);
    hipError_t e = hipFreeAsync(ws, s);
    if (rc == PPO_OK && e != hipSuccess) rc = hip_fail(e, "hipFreeAsync");
    return rc;
}

// Scratch of ppo_solve_static: one array per GPU, part of the library's code object, held until the process
// ends.  In host code this name only stands for the symbol; the device address comes from
// hipGetSymbolAddress, once per device, and that pointer is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[PPO_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device (looked up at the first call on that device)
int static_scratch(void** out) {
    int dev = -1;
    PPO_HIP(hipGetDevice(&dev), "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return PPO_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        PPO_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress (static scratch)");
        if (!p) return PPO_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return PPO_OK;
}
}  // namespace

int ppo_solve_static(const float* t, const float* m, int L, const float* M, const float* B, int k, int n_inst,
                     float* beta_out, int32_t* cuts_out, int32_t* order_out, void* stream) {
    int rc = check_shape(L, k, n_inst);
    if (rc) return rc;
    if (n_inst == 0) return PPO_OK;
    if (!t || !m || !M || !B || !beta_out || !order_out || (k > 1 && !cuts_out)) return PPO_EINVAL;
    if (ppo_workspace_bytes(L, k, n_inst) > (size_t)PPO_STATIC_SCRATCH_BYTES) return PPO_ENOSPC;
    void* ws = nullptr;
    rc = static_scratch(&ws);
    if (rc) return rc;
    // every table a kernel reads is written by the stage before it and the keys are set by a fill kernel, so
    // whatever the previous call left in the array does not matter
    return ppo_solve_ws(t, m, L, M, B, k, n_inst, beta_out, cuts_out, order_out, ws, (size_t)PPO_STATIC_SCRATCH_BYTES, stream);
}

int ppo_eval_orderings(const float* t, const float* m, int L, const float* M, const float* B, int k,
                       uint64_t rank_begin, uint64_t rank_end, float* beta_per_ordering, void* stream) {
    int rc = check_shape(L, k, 1);
    if (rc) return rc;
    if (rank_begin > rank_end || rank_end > (uint64_t)ppo::factorial_u32(k)) return PPO_EINVAL;
    if (rank_begin == rank_end) return PPO_OK;
    if (!t || !m || !M || !B || !beta_per_ordering) return PPO_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const ppo::Layout y = ppo::Layout::make(L, k);
    void* ws = nullptr;
    PPO_HIP(hipMallocAsync(&ws, tables_bytes(y, 1), s), "hipMallocAsync");
    hipError_t e = ppo::launch_precompute(t, m, M, B, y, 1, ws, s);
    if (e == hipSuccess)
        e = ppo::launch_enumerate(y, 1, ws, (uint32_t)rank_begin, (uint32_t)rank_end, nullptr, beta_per_ordering, false,
                                  nullptr, s);
    if (e != hipSuccess) rc = hip_fail(e, "eval_orderings launch");
    hipError_t e2 = hipFreeAsync(ws, s);
    if (rc == PPO_OK && e2 != hipSuccess) rc = hip_fail(e2, "hipFreeAsync");
    return rc;
}

// The search with the compute-time term: tables, one DP per ordering, traceback, all on scratch from the
// stream-ordered allocator (tables of every instance, then one key each).
int ppo_solve_ct(const float* t, const float* m, const float* w, int L, const float* M, const float* v, const float* B,
                 int k, int n_inst, float* beta_out, int32_t* cuts_out, int32_t* order_out, void* stream) {
    int rc = check_shape(L, k, n_inst);
    if (rc) return rc;
    if (n_inst == 0) return PPO_OK;
    if (!t || !m || !w || !M || !v || !B || !beta_out || !order_out || (k > 1 && !cuts_out)) return PPO_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t tables = ppo::ct_tables_bytes(L, k);
    unsigned char* ws = nullptr;
    PPO_HIP(hipMallocAsync(reinterpret_cast<void**>(&ws), tables * (size_t)n_inst + (size_t)n_inst * sizeof(uint64_t), s),
            "hipMallocAsync (compute-term tables)");
    uint64_t* keys = reinterpret_cast<uint64_t*>(ws + tables * (size_t)n_inst);   // tables is a multiple of 256
    hipError_t e = ppo::launch_init_keys(keys, n_inst, s);
    for (int first = 0; first < n_inst && e == hipSuccess; first += kInstPerLaunch) {
        const int n = n_inst - first < kInstPerLaunch ? n_inst - first : kInstPerLaunch;
        unsigned char* wsi = ws + tables * (size_t)first;
        e = ppo::launch_ct_tables(t + (size_t)first * L, m + (size_t)first * L, w + (size_t)first * L, M + (size_t)first * k,
                                  v + (size_t)first * k, B + (size_t)first * k * k, L, k, n, wsi, s);
        if (e == hipSuccess) e = ppo::launch_ct_enumerate(L, k, n, wsi, 0u, ppo::factorial_u32(k), keys + first, nullptr, s);
        if (e == hipSuccess)
            e = ppo::launch_ct_traceback(L, k, n, wsi, keys + first, beta_out + first, cuts_out + (size_t)first * (k - 1),
                                         order_out + (size_t)first * k, s);
    }
    const hipError_t e2 = hipFreeAsync(ws, s);
    PPO_HIP(e, "compute-term search launch");
    PPO_HIP(e2, "hipFreeAsync (compute-term tables)");
    return PPO_OK;
}

int ppo_eval_orderings_ct(const float* t, const float* m, const float* w, int L, const float* M, const float* v,
                          const float* B, int k, uint64_t rank_begin, uint64_t rank_end, float* beta_per_ordering,
                          void* stream) {
    int rc = check_shape(L, k, 1);
    if (rc) return rc;
    if (rank_begin > rank_end || rank_end > (uint64_t)ppo::factorial_u32(k)) return PPO_EINVAL;
    if (rank_begin == rank_end) return PPO_OK;
    if (!t || !m || !w || !M || !v || !B || !beta_per_ordering) return PPO_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    void* ws = nullptr;
    PPO_HIP(hipMallocAsync(&ws, ppo::ct_tables_bytes(L, k), s), "hipMallocAsync (compute-term tables)");
    hipError_t e = ppo::launch_ct_tables(t, m, w, M, v, B, L, k, 1, ws, s);
    if (e == hipSuccess)
        e = ppo::launch_ct_enumerate(L, k, 1, ws, (uint32_t)rank_begin, (uint32_t)rank_end, nullptr, beta_per_ordering, s);
    const hipError_t e2 = hipFreeAsync(ws, s);
    PPO_HIP(e, "compute-term per-ordering launch");
    PPO_HIP(e2, "hipFreeAsync (compute-term tables)");
    return PPO_OK;
}

static int check_place_shape(int L, int n, int n_inst) {
    if (L < 1 || n < 1 || n_inst < 0) return PPO_EINVAL;
    if (L > PPO_MAX_L || n > PPO_HEURISTIC_MAX_N) return PPO_ETOOBIG;
    return PPO_OK;
}

int ppo_place_kpath(const float* t, const float* m, int L, const float* kappa, const float* B, int n, int n_inst,
                    int n_classes, float* beta_out, int32_t* segs_out, int32_t* cuts_out, int32_t* order_out,
                    int32_t* classes_out, void* stream) {
    int rc = check_place_shape(L, n, n_inst);
    if (rc) return rc;
    if (n_classes < 1) return PPO_EINVAL;
    if (n_inst == 0) return PPO_OK;
    if (!t || !m || !kappa || !B || !beta_out || !segs_out || !order_out || (L > 1 && !cuts_out)) return PPO_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    double* sums = nullptr;   // the partitioning step's sums: not part of this call's results
    PPO_HIP(hipMallocAsync(reinterpret_cast<void**>(&sums), sizeof(double) * (size_t)n_inst, s), "hipMallocAsync (partition sums)");
    hipError_t e = hipSuccess;
    for (int first = 0; first < n_inst && e == hipSuccess; first += kInstPerLaunch) {
        const int cnt = n_inst - first < kInstPerLaunch ? n_inst - first : kInstPerLaunch;
        int32_t* cuts = cuts_out ? cuts_out + (size_t)first * (L - 1) : nullptr;
        e = ppo::launch_min_sum_partition(t + (size_t)first * L, m + (size_t)first * L, L, kappa + first, cnt, segs_out + first,
                                          cuts, sums + first, s);
        if (e == hipSuccess)
            e = ppo::launch_heuristic(t + (size_t)first * L, m + (size_t)first * L, L, kappa + first, B + (size_t)first * n * n, n,
                                      cnt, n_classes, 0, nullptr, 0, segs_out + first, cuts, beta_out + first, segs_out + first,
                                      cuts, order_out + (size_t)first * n, classes_out ? classes_out + first : nullptr, s);
    }
    const hipError_t e2 = hipFreeAsync(sums, s);
    PPO_HIP(e, "placement heuristic launch");
    PPO_HIP(e2, "hipFreeAsync (partition sums)");
    return PPO_OK;
}

int ppo_place_baseline(const float* t, const float* m, int L, const float* kappa, const float* B, int n, int n_inst,
                       int kind, const float* draws, int n_draws, float* beta_out, int32_t* segs_out, int32_t* cuts_out,
                       int32_t* order_out, void* stream) {
    int rc = check_place_shape(L, n, n_inst);
    if (rc) return rc;
    if (kind != PPO_BASELINE_JOINT && kind != PPO_BASELINE_RANDOM) return PPO_EINVAL;
    if (kind == PPO_BASELINE_RANDOM && (n_draws < 2 || !draws)) return PPO_EINVAL;
    if (n_inst == 0) return PPO_OK;
    if (!t || !m || !kappa || !B || !beta_out || !segs_out || !order_out || (L > 1 && !cuts_out)) return PPO_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    for (int first = 0; first < n_inst; first += kInstPerLaunch) {
        const int cnt = n_inst - first < kInstPerLaunch ? n_inst - first : kInstPerLaunch;
        PPO_HIP(ppo::launch_heuristic(t + (size_t)first * L, m + (size_t)first * L, L, kappa + first, B + (size_t)first * n * n, n,
                                      cnt, 1, kind, draws ? draws + (size_t)first * n_draws : nullptr, n_draws, nullptr, nullptr,
                                      beta_out + first, segs_out + first, cuts_out ? cuts_out + (size_t)first * (L - 1) : nullptr,
                                      order_out + (size_t)first * n, nullptr, s),
                "comparison system launch");
    }
    return PPO_OK;
}

int ppo_probe_valu(int waves_per_simd, int iters, uint32_t* sink, void* stream) {
    if (waves_per_simd < 1 || waves_per_simd > 4 || iters < 1 || sink == nullptr) return PPO_EINVAL;
    PPO_HIP(ppo::launch_valu_probe(waves_per_simd, iters, sink, static_cast<hipStream_t>(stream)), "valu probe launch");
    return PPO_OK;
}

}  // extern "C"
