// C ABI of the rank-order search library: argument checks, workspace carving, launches.
// Declarations and contracts: include/cc.h.
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <mutex>

#include "../../include/cc.h"
#include "cc_internal.h"

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    return CC_ERR_HIP;
}

#define CC_HIP(expr)                                  \
    do {                                              \
        hipError_t e_ = (expr);                       \
        if (e_ != hipSuccess) return hip_fail(e_);    \
    } while (0)

bool is_pow2(int n) { return n > 0 && (n & (n - 1)) == 0; }

size_t align256(size_t x) { return (x + 255u) & ~(size_t)255u; }

// Workspace layout of cc_2opt_search_ex:
// [flags 256 B][costs int64 R][moves int32 R][tours int32 R*N][16-bit matrix copy, N > 256 only]
struct WsLayout {
    size_t flags, costs, moves, tours, mat16, total;
};

WsLayout ws_layout(int N, int restarts) {
    WsLayout w;
    w.flags = 0;
    w.costs = 256;
    w.moves = w.costs + align256(sizeof(int64_t) * (size_t)restarts);
    w.tours = w.moves + align256(sizeof(int32_t) * (size_t)restarts);
    w.mat16 = w.tours + align256(sizeof(int32_t) * (size_t)restarts * (size_t)N);
    w.total = w.mat16 + (N > 256 ? align256(sizeof(uint16_t) * (size_t)N * (size_t)N) : 0);
    return w;
}

int check_matrix_args(const int32_t* c, int N) {
    if (!c) return CC_ERR_INVALID_ARG;
    if (N < 2 || N > CC_MAX_N) return CC_ERR_UNSUPPORTED_N;
    return CC_OK;
}

// Debug aid.  With CC_LDS_POISON=1 in the environment (read at every call) each call first fills the LDS of every
// compute unit with 0x7f bytes, so that a kernel that reads LDS it has not written gets large garbage instead of
// whatever an earlier kernel left there (often the very data it expects), and a parity test fails.  LDS keeps its
// contents between workgroups; a workgroup that asks for all of a compute unit's LDS has the unit to itself, and far
// more such workgroups than compute units are launched, so every unit is reached.
constexpr int kLdsBytesPerCu = 160 * 1024;
__global__ __launch_bounds__(1024) void lds_poison_kernel() {
    extern __shared__ uint32_t lds_words[];
    volatile uint32_t* p = lds_words;
    for (int i = threadIdx.x; i < kLdsBytesPerCu / 4; i += 1024) p[i] = 0x7f7f7f7fu;
}

hipError_t poison_lds_if_asked(hipStream_t s) {
    const char* v = getenv("CC_LDS_POISON");
    if (!v || v[0] != '1') return hipSuccess;
    hipError_t e = hipFuncSetAttribute((const void*)lds_poison_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       kLdsBytesPerCu);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(lds_poison_kernel, dim3(2048), dim3(1024), kLdsBytesPerCu, s);
    return hipGetLastError();
}

// Device memory of cc_2opt_search_noalloc: one array per GPU, part of the code object, there from the moment the
// library is loaded on a device until the process ends.  In host code the name `scratch` is only a handle for
// hipGetSymbolAddress; the array's memory is reached through the per-device pointer that call returns.
static __device__ __align__(256) unsigned char scratch[CC_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Address of the current device's scratch array (looked up once per device, with that device current).
int static_scratch(void** out) {
    int dev = -1;
    CC_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return CC_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        CC_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || ((uintptr_t)ptr & 255u)) return CC_ERR_WORKSPACE;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return CC_OK;
}

}  // namespace

extern "C" {

int cc_ring_cost_batch(const int32_t* cost_matrix, int32_t N, int32_t objective, const int32_t* perms, int64_t B,
                       int64_t* out_costs, void* stream) {
    if (int rc = check_matrix_args(cost_matrix, N)) return rc;
    if (objective < 0 || objective > 3 || B < 0) return CC_ERR_INVALID_ARG;
    if (B == 0) return CC_OK;
    if (!perms || !out_costs) return CC_ERR_INVALID_ARG;
    if (((uintptr_t)perms & 3u) || ((uintptr_t)out_costs & 7u) || ((uintptr_t)cost_matrix & 3u)) return CC_ERR_INVALID_ARG;
    CC_HIP(poison_lds_if_asked((hipStream_t)stream));
    CC_HIP(cc::launch_ring_cost_batch(cost_matrix, N, (objective & 1) != 0, perms, B, out_costs, (hipStream_t)stream));
    return CC_OK;
}

int cc_ring_cost_batch_u8(const int32_t* cost_matrix, int32_t N, int32_t objective, const uint8_t* perms, int64_t B,
                          int64_t* out_costs, void* stream) {
    if (int rc = check_matrix_args(cost_matrix, N)) return rc;
    if (N > 256) return CC_ERR_UNSUPPORTED_N;
    if (objective < 0 || objective > 3 || B < 0) return CC_ERR_INVALID_ARG;
    if (B == 0) return CC_OK;
    if (!perms || !out_costs) return CC_ERR_INVALID_ARG;
    if (((uintptr_t)out_costs & 7u) || ((uintptr_t)cost_matrix & 3u)) return CC_ERR_INVALID_ARG;
    CC_HIP(poison_lds_if_asked((hipStream_t)stream));
    CC_HIP(cc::launch_ring_cost_batch_u8(cost_matrix, N, (objective & 1) != 0, perms, B, out_costs, (hipStream_t)stream));
    return CC_OK;
}

int cc_ring_cost_batch_u16(const int32_t* cost_matrix, int32_t N, int32_t objective, const uint16_t* perms, int64_t B,
                           int64_t* out_costs, void* stream) {
    if (int rc = check_matrix_args(cost_matrix, N)) return rc;
    if (objective < 0 || objective > 3 || B < 0) return CC_ERR_INVALID_ARG;
    if (B == 0) return CC_OK;
    if (!perms || !out_costs) return CC_ERR_INVALID_ARG;
    if (((uintptr_t)perms & 1u) || ((uintptr_t)out_costs & 7u) || ((uintptr_t)cost_matrix & 3u)) return CC_ERR_INVALID_ARG;
    CC_HIP(poison_lds_if_asked((hipStream_t)stream));
    CC_HIP(cc::launch_ring_cost_batch_u16(cost_matrix, N, (objective & 1) != 0, perms, B, out_costs, (hipStream_t)stream));
    return CC_OK;
}

int cc_rd_cost_batch(const int32_t* cost_matrix, int32_t N, const int32_t* perms, int64_t B, int64_t* out_costs,
                     void* stream) {
    if (int rc = check_matrix_args(cost_matrix, N)) return rc;
    if (!is_pow2(N)) return CC_ERR_UNSUPPORTED_N;
    if (B < 0) return CC_ERR_INVALID_ARG;
    if (B == 0) return CC_OK;
    if (!perms || !out_costs) return CC_ERR_INVALID_ARG;
    if (((uintptr_t)perms & 3u) || ((uintptr_t)out_costs & 7u) || ((uintptr_t)cost_matrix & 3u)) return CC_ERR_INVALID_ARG;
    CC_HIP(poison_lds_if_asked((hipStream_t)stream));
    CC_HIP(cc::launch_rd_cost_batch(cost_matrix, N, nullptr, perms, B, out_costs, (hipStream_t)stream));
    return CC_OK;
}

size_t cc_rd_batch_workspace_bytes(int32_t N) {
    if (N < 2 || N > CC_MAX_N) return 0;
    return 256 + align256(sizeof(uint16_t) * (size_t)N * (size_t)N);        // flags, folded 16-bit matrix
}

int cc_rd_cost_batch_ex(const int32_t* cost_matrix, int32_t N, const int32_t* perms, int64_t B, int64_t* out_costs,
                        void* workspace, size_t workspace_bytes, void* stream) {
    if (int rc = check_matrix_args(cost_matrix, N)) return rc;
    if (!is_pow2(N)) return CC_ERR_UNSUPPORTED_N;
    if (B < 0) return CC_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < cc_rd_batch_workspace_bytes(N) || ((uintptr_t)workspace & 255u))
        return CC_ERR_WORKSPACE;
    if (B == 0) return CC_OK;
    if (!perms || !out_costs) return CC_ERR_INVALID_ARG;
    if (((uintptr_t)perms & 3u) || ((uintptr_t)out_costs & 7u) || ((uintptr_t)cost_matrix & 3u)) return CC_ERR_INVALID_ARG;
    char* base = (char*)workspace;
    CC_HIP(poison_lds_if_asked((hipStream_t)stream));
    CC_HIP(cc::launch_rd_cost_batch(cost_matrix, N, nullptr, perms, B, out_costs, (hipStream_t)stream, (int32_t*)base,
                                    (uint16_t*)(base + 256)));
    return CC_OK;
}

static int bcube_batch(const int32_t* cost_matrix, int32_t N, int32_t base, const int32_t* weights, bool weighted,
                       const int32_t* perms, int64_t B, int64_t* out_costs, void* stream, void* workspace = nullptr) {
    if (int rc = check_matrix_args(cost_matrix, N)) return rc;
    if (base < 2) return CC_ERR_INVALID_ARG;
    int64_t power = 1;
    while (power < N) power *= base;
    if (power != N) return CC_ERR_UNSUPPORTED_N;
    if (B < 0 || (weighted && (!weights || ((uintptr_t)weights & 3u)))) return CC_ERR_INVALID_ARG;
    if (B == 0) return CC_OK;
    if (!perms || !out_costs) return CC_ERR_INVALID_ARG;
    if (((uintptr_t)perms & 3u) || ((uintptr_t)out_costs & 7u) || ((uintptr_t)cost_matrix & 3u)) return CC_ERR_INVALID_ARG;
    char* ws = (char*)workspace;
    CC_HIP(poison_lds_if_asked((hipStream_t)stream));
    CC_HIP(cc::launch_bcube_cost_batch(cost_matrix, N, base, weights, perms, B, out_costs, (hipStream_t)stream,
                                       (int32_t*)ws, ws ? (uint16_t*)(ws + 256) : nullptr));
    return CC_OK;
}

int cc_bcube_cost_batch(const int32_t* cost_matrix, int32_t N, int32_t base, const int32_t* perms, int64_t B,
                        int64_t* out_costs, void* stream) {
    return bcube_batch(cost_matrix, N, base, nullptr, false, perms, B, out_costs, stream);
}

int cc_bcube_cost_batch_weighted(const int32_t* cost_matrix, int32_t N, int32_t base, const int32_t* round_weights,
                                 const int32_t* perms, int64_t B, int64_t* out_costs, void* stream) {
    return bcube_batch(cost_matrix, N, base, round_weights, true, perms, B, out_costs, stream);
}

int cc_bcube_cost_batch_ex(const int32_t* cost_matrix, int32_t N, int32_t base, const int32_t* round_weights,
                           const int32_t* perms, int64_t B, int64_t* out_costs, void* workspace, size_t workspace_bytes,
                           void* stream) {
    if (int rc = check_matrix_args(cost_matrix, N)) return rc;
    if (!workspace || workspace_bytes < cc_rd_batch_workspace_bytes(N) || ((uintptr_t)workspace & 255u))
        return CC_ERR_WORKSPACE;
    if (round_weights && ((uintptr_t)round_weights & 3u)) return CC_ERR_INVALID_ARG;
    return bcube_batch(cost_matrix, N, base, round_weights, false, perms, B, out_costs, stream, workspace);
}

int cc_dbt_cost_batch(const int32_t* cost_matrix, int32_t N, const int32_t* perms, int64_t B, int64_t* out_costs,
                      void* stream) {
    if (int rc = check_matrix_args(cost_matrix, N)) return rc;
    if (B < 0) return CC_ERR_INVALID_ARG;
    if (B == 0) return CC_OK;
    if (!perms || !out_costs) return CC_ERR_INVALID_ARG;
    if (((uintptr_t)perms & 3u) || ((uintptr_t)out_costs & 7u) || ((uintptr_t)cost_matrix & 3u)) return CC_ERR_INVALID_ARG;
    CC_HIP(poison_lds_if_asked((hipStream_t)stream));
    CC_HIP(cc::launch_dbt_cost_batch(cost_matrix, N, perms, B, out_costs, (hipStream_t)stream));
    return CC_OK;
}

size_t cc_2opt_workspace_bytes(int32_t N, int32_t objective, int32_t restarts) {
    if (N < 2 || N > CC_MAX_N || objective < 0 || objective > 3 || restarts < 1) return 0;
    return ws_layout(N, restarts).total;
}

// Which move classes go with which objective (cc.h, cc_local_search).
static bool classes_ok(int objective, int classes) {
    if (classes == CC_MOVES_2OPT) return true;
    if (classes == CC_MOVES_OROPT || classes == (CC_MOVES_2OPT | CC_MOVES_OROPT)) return objective == CC_RING_SUM;
    if (classes == (CC_MOVES_2OPT | CC_MOVES_FLIP)) return (objective & 2) != 0;
    return false;
}

static int ring_search_ex(const int32_t* cost_matrix, int32_t N, int32_t objective, int32_t classes, int32_t restarts,
                          uint64_t seed, const int32_t* init_tours, int32_t* best_perm, int64_t* best_cost,
                          int32_t* best_restart, int64_t* restart_costs, int32_t* restart_tours,
                          int32_t* restart_moves, void* workspace, size_t workspace_bytes, void* stream) {
    if (int rc = check_matrix_args(cost_matrix, N)) return rc;
    if (objective < 0 || objective > 3 || restarts < 1 || !classes_ok(objective, classes)) return CC_ERR_INVALID_ARG;
    // either both best_* outputs, or neither and then the per-restart costs and orders
    if ((best_perm == nullptr) != (best_cost == nullptr)) return CC_ERR_INVALID_ARG;
    if (!best_perm && (best_restart || !restart_costs || !restart_tours)) return CC_ERR_INVALID_ARG;
    const WsLayout w = ws_layout(N, restarts);
    if (!workspace || workspace_bytes < w.total || ((uintptr_t)workspace & 255u)) return CC_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    char* base = (char*)workspace;
    int32_t* flags = (int32_t*)(base + w.flags);
    int64_t* costs = restart_costs ? restart_costs : (int64_t*)(base + w.costs);
    int32_t* moves = restart_moves ? restart_moves : (int32_t*)(base + w.moves);
    int32_t* tours = restart_tours ? restart_tours : (int32_t*)(base + w.tours);
    if (init_tours && init_tours != tours)
        CC_HIP(hipMemcpyAsync(tours, init_tours, sizeof(int32_t) * (size_t)restarts * (size_t)N,
                              hipMemcpyDeviceToDevice, s));
    CC_HIP(poison_lds_if_asked((hipStream_t)stream));
    CC_HIP(cc::launch_2opt(cost_matrix, N, objective, classes, restarts, seed, init_tours != nullptr, tours, costs,
                           moves, flags, (uint16_t*)(base + w.mat16), best_perm, best_cost, best_restart, s));
    return CC_OK;
}

static int ring_search(const int32_t* cost_matrix, int32_t N, int32_t objective, int32_t classes, int32_t restarts,
                       uint64_t seed, int32_t* best_perm, int64_t* best_cost, void* stream) {
    if (int rc = check_matrix_args(cost_matrix, N)) return rc;
    if (objective < 0 || objective > 3 || restarts < 1 || !best_perm || !best_cost || !classes_ok(objective, classes))
        return CC_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const size_t bytes = cc_2opt_workspace_bytes(N, objective, restarts);
    void* ws = nullptr;
    CC_HIP(hipMallocAsync(&ws, bytes, s));
    const int rc = ring_search_ex(cost_matrix, N, objective, classes, restarts, seed, nullptr, best_perm, best_cost,
                                  nullptr, nullptr, nullptr, nullptr, ws, bytes, stream);
    const hipError_t e = hipFreeAsync(ws, s);   // stream-ordered: released after the search has run
    if (rc != CC_OK) return rc;
    if (e != hipSuccess) return hip_fail(e);
    return CC_OK;
}

int cc_2opt_search_ex(const int32_t* cost_matrix, int32_t N, int32_t objective, int32_t restarts, uint64_t seed,
                      const int32_t* init_tours, int32_t* best_perm, int64_t* best_cost, int32_t* best_restart,
                      int64_t* restart_costs, int32_t* restart_tours, int32_t* restart_moves, void* workspace,
                      size_t workspace_bytes, void* stream) {
    return ring_search_ex(cost_matrix, N, objective, CC_MOVES_2OPT, restarts, seed, init_tours, best_perm, best_cost,
                          best_restart, restart_costs, restart_tours, restart_moves, workspace, workspace_bytes, stream);
}

int cc_local_search_ex(const int32_t* cost_matrix, int32_t N, int32_t objective, int32_t move_classes,
                       int32_t restarts, uint64_t seed, const int32_t* init_tours, int32_t* best_perm,
                       int64_t* best_cost, int32_t* best_restart, int64_t* restart_costs, int32_t* restart_tours,
                       int32_t* restart_moves, void* workspace, size_t workspace_bytes, void* stream) {
    return ring_search_ex(cost_matrix, N, objective, move_classes, restarts, seed, init_tours, best_perm, best_cost,
                          best_restart, restart_costs, restart_tours, restart_moves, workspace, workspace_bytes, stream);
}

int cc_local_search(const int32_t* cost_matrix, int32_t N, int32_t objective, int32_t move_classes, int32_t restarts,
                    uint64_t seed, int32_t* best_perm, int64_t* best_cost, void* stream) {
    return ring_search(cost_matrix, N, objective, move_classes, restarts, seed, best_perm, best_cost, stream);
}

int cc_best_of_restarts(const int64_t* restart_costs, const int32_t* restart_tours, int32_t N, int32_t restarts,
                        int32_t* best_perm, int64_t* best_cost, int32_t* best_restart, void* stream) {
    if (N < 2 || N > CC_MAX_N) return CC_ERR_UNSUPPORTED_N;
    if (!restart_costs || !restart_tours || restarts < 1 || !best_perm || !best_cost) return CC_ERR_INVALID_ARG;
    CC_HIP(poison_lds_if_asked((hipStream_t)stream));
    CC_HIP(cc::launch_best_restart(restart_costs, restart_tours, N, restarts, best_perm, best_cost, best_restart,
                                   (hipStream_t)stream));
    return CC_OK;
}

int cc_2opt_search(const int32_t* cost_matrix, int32_t N, int32_t objective, int32_t restarts, uint64_t seed,
                   int32_t* best_perm, int64_t* best_cost, void* stream) {
    return ring_search(cost_matrix, N, objective, CC_MOVES_2OPT, restarts, seed, best_perm, best_cost, stream);
}

int cc_2opt_search_noalloc(const int32_t* cost_matrix, int32_t N, int32_t objective, int32_t restarts, uint64_t seed,
                           int32_t* best_perm, int64_t* best_cost, void* stream) {
    if (int rc = check_matrix_args(cost_matrix, N)) return rc;
    if (objective < 0 || objective > 3 || restarts < 1 || !best_perm || !best_cost) return CC_ERR_INVALID_ARG;
    const size_t bytes = cc_2opt_workspace_bytes(N, objective, restarts);
    if (bytes == 0 || bytes > (size_t)CC_STATIC_SCRATCH_BYTES) return CC_ERR_SCRATCH_LIMIT;
    void* ws = nullptr;
    if (int rc = static_scratch(&ws)) return rc;
    return ring_search_ex(cost_matrix, N, objective, CC_MOVES_2OPT, restarts, seed, nullptr, best_perm, best_cost,
                          nullptr, nullptr, nullptr, nullptr, ws, bytes, stream);
}

size_t cc_rd_swap_workspace_bytes(int32_t N, int32_t restarts) {
    if (N < 2 || N > CC_MAX_N || !is_pow2(N) || restarts < 1) return 0;
    return ws_layout(N, restarts).total;       // flags, costs, moves, tours, folded 16-bit matrix (N > 256)
}

int cc_rd_swap_search_ex(const int32_t* cost_matrix, int32_t N, int32_t restarts, uint64_t seed,
                         const int32_t* init_tours, int32_t* best_perm, int64_t* best_cost, int32_t* best_restart,
                         int64_t* restart_costs, int32_t* restart_tours, int32_t* restart_moves, void* workspace,
                         size_t workspace_bytes, void* stream) {
    if (int rc = check_matrix_args(cost_matrix, N)) return rc;
    if (!is_pow2(N)) return CC_ERR_UNSUPPORTED_N;
    if (restarts < 1 || !best_perm || !best_cost) return CC_ERR_INVALID_ARG;
    const WsLayout w = ws_layout(N, restarts);
    if (!workspace || workspace_bytes < w.total || ((uintptr_t)workspace & 255u)) return CC_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    char* base = (char*)workspace;
    int64_t* costs = restart_costs ? restart_costs : (int64_t*)(base + w.costs);
    int32_t* moves = restart_moves ? restart_moves : (int32_t*)(base + w.moves);
    int32_t* tours = restart_tours ? restart_tours : (int32_t*)(base + w.tours);
    if (init_tours && init_tours != tours)
        CC_HIP(hipMemcpyAsync(tours, init_tours, sizeof(int32_t) * (size_t)restarts * (size_t)N,
                              hipMemcpyDeviceToDevice, s));
    CC_HIP(poison_lds_if_asked((hipStream_t)stream));
    CC_HIP(cc::launch_rdswap(cost_matrix, N, restarts, seed, init_tours != nullptr, tours, costs, moves,
                             (int32_t*)(base + w.flags), (uint16_t*)(base + w.mat16), s));
    CC_HIP(cc::launch_best_restart(costs, tours, N, restarts, best_perm, best_cost, best_restart, s));
    return CC_OK;
}

int cc_rd_swap_search(const int32_t* cost_matrix, int32_t N, int32_t restarts, uint64_t seed, int32_t* best_perm,
                      int64_t* best_cost, void* stream) {
    if (int rc = check_matrix_args(cost_matrix, N)) return rc;
    if (!is_pow2(N)) return CC_ERR_UNSUPPORTED_N;
    if (restarts < 1 || !best_perm || !best_cost) return CC_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const size_t bytes = cc_rd_swap_workspace_bytes(N, restarts);
    void* ws = nullptr;
    CC_HIP(hipMallocAsync(&ws, bytes, s));
    const int rc = cc_rd_swap_search_ex(cost_matrix, N, restarts, seed, nullptr, best_perm, best_cost, nullptr, nullptr,
                                        nullptr, nullptr, ws, bytes, stream);
    const hipError_t e = hipFreeAsync(ws, s);
    if (rc != CC_OK) return rc;
    if (e != hipSuccess) return hip_fail(e);
    return CC_OK;
}

size_t cc_sa_workspace_bytes(int32_t N, int32_t chains) {
    if (N < 2 || N > CC_MAX_N || chains < 1) return 0;
    return ws_layout(N, chains).mat16;       // flags, costs, accepted counts, orders
}

// Both annealing searches: ring sum with sub-array reversals, or halving-doubling with pair exchanges.
static int sa_search_ex(bool halving_doubling, const int32_t* cost_matrix, int32_t N, int32_t chains, int64_t steps,
                        int32_t t_start, int32_t t_end, uint64_t seed, const int32_t* init_tours, int32_t* best_perm,
                        int64_t* best_cost, int32_t* best_chain, int64_t* chain_costs, int32_t* chain_tours,
                        int32_t* chain_accepted, void* workspace, size_t workspace_bytes, void* stream) {
    if (int rc = check_matrix_args(cost_matrix, N)) return rc;
    if (halving_doubling && !is_pow2(N)) return CC_ERR_UNSUPPORTED_N;
    if (chains < 1 || steps < 0 || steps > CC_SA_MAX_STEPS || t_start < 0 || t_start > CC_COST_MAX || t_end < 0 ||
        t_end > CC_COST_MAX || !best_perm || !best_cost)
        return CC_ERR_INVALID_ARG;
    const WsLayout w = ws_layout(N, chains);
    if (!workspace || workspace_bytes < w.mat16 || ((uintptr_t)workspace & 255u)) return CC_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    char* base = (char*)workspace;
    int64_t* costs = chain_costs ? chain_costs : (int64_t*)(base + w.costs);
    int32_t* acc = chain_accepted ? chain_accepted : (int32_t*)(base + w.moves);
    int32_t* tours = chain_tours ? chain_tours : (int32_t*)(base + w.tours);
    if (init_tours && init_tours != tours)
        CC_HIP(hipMemcpyAsync(tours, init_tours, sizeof(int32_t) * (size_t)chains * (size_t)N, hipMemcpyDeviceToDevice, s));
    CC_HIP(poison_lds_if_asked(s));
    if (halving_doubling)
        CC_HIP(cc::launch_sa_rd(cost_matrix, N, chains, steps, t_start, t_end, seed, init_tours == nullptr, tours, costs,
                                acc, s));
    else
        CC_HIP(cc::launch_sa_ring(cost_matrix, N, chains, steps, t_start, t_end, seed, init_tours == nullptr, tours,
                                  costs, acc, s));
    CC_HIP(cc::launch_best_restart(costs, tours, N, chains, best_perm, best_cost, best_chain, s));
    return CC_OK;
}

static int sa_search(bool halving_doubling, const int32_t* cost_matrix, int32_t N, int32_t chains, int64_t steps,
                     int32_t t_start, int32_t t_end, uint64_t seed, int32_t* best_perm, int64_t* best_cost,
                     void* stream) {
    if (int rc = check_matrix_args(cost_matrix, N)) return rc;
    if (halving_doubling && !is_pow2(N)) return CC_ERR_UNSUPPORTED_N;
    if (chains < 1 || !best_perm || !best_cost) return CC_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const size_t bytes = cc_sa_workspace_bytes(N, chains);
    void* ws = nullptr;
    CC_HIP(hipMallocAsync(&ws, bytes, s));
    const int rc = sa_search_ex(halving_doubling, cost_matrix, N, chains, steps, t_start, t_end, seed, nullptr, best_perm,
                                best_cost, nullptr, nullptr, nullptr, nullptr, ws, bytes, stream);
    const hipError_t e = hipFreeAsync(ws, s);
    if (rc != CC_OK) return rc;
    if (e != hipSuccess) return hip_fail(e);
    return CC_OK;
}

int cc_sa_search_ex(const int32_t* cost_matrix, int32_t N, int32_t chains, int64_t steps, int32_t t_start, int32_t t_end,
                    uint64_t seed, const int32_t* init_tours, int32_t* best_perm, int64_t* best_cost, int32_t* best_chain,
                    int64_t* chain_costs, int32_t* chain_tours, int32_t* chain_accepted, void* workspace,
                    size_t workspace_bytes, void* stream) {
    return sa_search_ex(false, cost_matrix, N, chains, steps, t_start, t_end, seed, init_tours, best_perm, best_cost,
                        best_chain, chain_costs, chain_tours, chain_accepted, workspace, workspace_bytes, stream);
}

int cc_sa_search(const int32_t* cost_matrix, int32_t N, int32_t chains, int64_t steps, int32_t t_start, int32_t t_end,
                 uint64_t seed, int32_t* best_perm, int64_t* best_cost, void* stream) {
    return sa_search(false, cost_matrix, N, chains, steps, t_start, t_end, seed, best_perm, best_cost, stream);
}

int cc_sa_rd_search_ex(const int32_t* cost_matrix, int32_t N, int32_t chains, int64_t steps, int32_t t_start,
                       int32_t t_end, uint64_t seed, const int32_t* init_tours, int32_t* best_perm, int64_t* best_cost,
                       int32_t* best_chain, int64_t* chain_costs, int32_t* chain_tours, int32_t* chain_accepted,
                       void* workspace, size_t workspace_bytes, void* stream) {
    return sa_search_ex(true, cost_matrix, N, chains, steps, t_start, t_end, seed, init_tours, best_perm, best_cost,
                        best_chain, chain_costs, chain_tours, chain_accepted, workspace, workspace_bytes, stream);
}

int cc_sa_rd_search(const int32_t* cost_matrix, int32_t N, int32_t chains, int64_t steps, int32_t t_start, int32_t t_end,
                    uint64_t seed, int32_t* best_perm, int64_t* best_cost, void* stream) {
    return sa_search(true, cost_matrix, N, chains, steps, t_start, t_end, seed, best_perm, best_cost, stream);
}

int cc_init_tours(int32_t N, int64_t first, int64_t count, uint64_t seed, int32_t* tours, void* stream) {
    if (N < 2 || N > CC_MAX_N) return CC_ERR_UNSUPPORTED_N;
    if (first < 0 || count < 0 || first + count > (int64_t)1 << 32) return CC_ERR_INVALID_ARG;
    if (count == 0) return CC_OK;
    if (!tours || ((uintptr_t)tours & 3u)) return CC_ERR_INVALID_ARG;
    CC_HIP(poison_lds_if_asked((hipStream_t)stream));
    CC_HIP(cc::launch_init_tours(N, first, count, seed, tours, (hipStream_t)stream));
    return CC_OK;
}

int cc_cost_matrix_from_probes(const int32_t* samples, int32_t N, int32_t K, int32_t percentile, int32_t symmetrize,
                               int32_t* cost_matrix, void* stream) {
    if (!samples || !cost_matrix || ((uintptr_t)samples & 3u) || ((uintptr_t)cost_matrix & 3u)) return CC_ERR_INVALID_ARG;
    if (N < 1 || N > CC_MAX_N) return CC_ERR_UNSUPPORTED_N;
    if (K < 1 || K > CC_MAX_PROBES || percentile < 0 || percentile > 100) return CC_ERR_INVALID_ARG;
    int64_t rank = ((int64_t)percentile * K + 99) / 100;
    if (rank < 1) rank = 1;
    CC_HIP(poison_lds_if_asked((hipStream_t)stream));
    CC_HIP(cc::launch_probes_percentile(samples, N, K, (int)rank, symmetrize != 0, cost_matrix, (hipStream_t)stream));
    return CC_OK;
}

int cc_validate_matrix(const int32_t* cost_matrix, int32_t N, int32_t require_symmetric, void* stream) {
    if (int rc = check_matrix_args(cost_matrix, N)) return rc;
    hipStream_t s = (hipStream_t)stream;
    int32_t* flags = nullptr;
    CC_HIP(hipMalloc((void**)&flags, sizeof(int32_t)));
    int32_t host = 0;
    hipError_t e = hipMemsetAsync(flags, 0, sizeof(int32_t), s);
    if (e == hipSuccess) e = cc::launch_validate(cost_matrix, N, require_symmetric != 0, flags, s);
    if (e == hipSuccess) e = hipMemcpyAsync(&host, flags, sizeof(int32_t), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    (void)hipFree(flags);
    if (e != hipSuccess) return hip_fail(e);
    if (host & 1) return CC_ERR_COST_RANGE;
    if (host & 2) return CC_ERR_NOT_SYMMETRIC;
    return CC_OK;
}

const char* cc_status_string(int status) {
    switch (status) {
        case CC_OK: return "ok";
        case CC_ERR_INVALID_ARG: return "invalid argument";
        case CC_ERR_UNSUPPORTED_N: return "unsupported N";
        case CC_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case CC_ERR_HIP: return "HIP runtime error";
        case CC_ERR_NOT_SYMMETRIC: return "cost matrix is not symmetric";
        case CC_ERR_COST_RANGE: return "cost matrix entry out of range";
        case CC_ERR_SCRATCH_LIMIT: return "search too large for the static scratch array (CC_STATIC_SCRATCH_BYTES)";
        default: return "unknown status";
    }
}

int cc_last_hip_error(void) { return g_last_hip_error; }

int cc_version(void) { return 501; }

}  // extern "C"
