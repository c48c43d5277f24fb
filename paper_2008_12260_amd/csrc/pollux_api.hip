// C ABI of the library (see include/pollux.h): argument checks on the host,
// device check, then the launch functions.

#include <hip/hip_runtime.h>
#include <math.h>
#include <string.h>

#include <atomic>
#include <mutex>

#include "../../include/pollux.h"
#include "pollux_host.h"

// ---- scratch memory owned by the library (pollux_fitness_static) -------------------------------------------
// One array per GPU, part of the code object: every device the library runs on holds its own copy, at its own
// address, from the moment the code object is loaded there until the process ends.  In host code the name
// `scratch` only stands for the symbol; the address kernels can use is looked up once per device, with that
// device current, and kept.
static __device__ __align__(256) unsigned char scratch[POLLUX_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
// Per device: 0 unknown, 1 gfx950, -1 something else.  A cache of a property that never changes: two threads
// that find it unknown both query the device and store the same value.
std::atomic<int> g_arch_ok[kMaxDevices];

int check_device(int *device = nullptr)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return PX_E_HIP;
    if (dev < 0 || dev >= kMaxDevices) return PX_E_HIP;
    if (device) *device = dev;
    int ok = g_arch_ok[dev].load(std::memory_order_relaxed);
    if (ok == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return PX_E_HIP;
        ok = strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : -1;
        g_arch_ok[dev].store(ok, std::memory_order_relaxed);
    }
    return ok == 1 ? PX_OK : PX_E_UNSUPPORTED_ARCH;
}

void *g_scratch_ptr[kMaxDevices];     // device address of `scratch` on each device, null until looked up
std::mutex g_scratch_lock;

int static_scratch(int dev, void **out)
{
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return PX_E_HIP;
        if (((uintptr_t)ptr & 255u) != 0) return PX_E_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return PX_OK;
}

bool dims_ok(const pollux_dims *d, bool need_grid)
{
    if (!d) return false;
    if (d->P <= 0 || d->J <= 0 || d->N <= 0) return false;
    if (need_grid && (d->Gm <= 0 || d->Gs <= 0)) return false;
    if (d->precision != 0 && d->precision != 1) return false;
    if ((d->flags & PX_FLAG_SAMPLE_M) && d->precision != 0) return false;   // the sampling argmax exists in fp64 only
    if (d->N >= (1 << 30)) return false;   // node counts share a 32-bit word with a flag
    // flat indices of (candidate, job) pairs and of grid points are kept in 32 bits
    if ((long long)d->P * d->J > 0x7FFFFFFFll) return false;
    if (need_grid && (long long)d->Gm * d->Gs > 0x7FFFFFFFll) return false;
    if (need_grid && (d->Gm > (1 << 20) || d->Gs > (1 << 14))) return false;   // chunk ids are packed into one word
    if (need_grid && (long long)d->J * d->Gm > 0x7FFFFFFFll) return false;
    // offsets inside one job's tables (last pass [2,64,Gm], lane masks [64,Gm/64,Gs up to 32]) are kept in 32 bits
    if (need_grid && ((long long)d->Gm + 63) * (((long long)d->Gs + 31) / 32 * 32) > (1ll << 28)) return false;
    return true;
}

int check_workspace(const pollux_dims *d, const void *ws, size_t bytes)
{
    if (!ws || ((uintptr_t)ws & 255u) != 0) return PX_E_WORKSPACE;
    if (bytes < px::workspace_layout(*d).total) return PX_E_WORKSPACE;
    return PX_OK;
}

}  // namespace

extern "C" {

int pollux_version(void) { return POLLUX_VERSION; }

const char *pollux_strerror(int code)
{
    switch (code) {
        case PX_OK: return "success";
        case PX_E_INVALID_ARG: return "invalid argument";
        case PX_E_WORKSPACE: return "workspace missing, misaligned or too small";
        case PX_E_UNSUPPORTED_ARCH: return "current device is not gfx950";
        case PX_E_HIP: return "HIP runtime error";
        default: return "unknown error code";
    }
}

int pollux_workspace_size(const pollux_dims *dims, size_t *bytes)
{
    if (!bytes || !dims_ok(dims, false)) return PX_E_INVALID_ARG;
    *bytes = px::workspace_layout(*dims).total;
    return PX_OK;
}

namespace {

int fitness_call(const pollux_dims *dims, const int32_t *population, const double *job_params, const int32_t *m_grid,
                 const int32_t *fair_share, const int32_t *current_alloc, const int32_t *node_capacity, double p,
                 double delta, void *workspace, size_t workspace_bytes, double *fitness, int32_t *best_m,
                 int32_t *best_s, double *best_goodput, double *speedup, int32_t *violations, hipEvent_t sweep_start,
                 hipEvent_t sweep_stop, void *hip_stream)
{
    if (!dims_ok(dims, true)) return PX_E_INVALID_ARG;
    if (!population || !job_params || !m_grid || !fair_share || !current_alloc || !node_capacity || !fitness ||
        (best_m == nullptr) != (best_s == nullptr))
        return PX_E_INVALID_ARG;
    if (!isfinite(p) || !isfinite(delta) || delta < 0.0) return PX_E_INVALID_ARG;
    int rc = check_workspace(dims, workspace, workspace_bytes);
    if (rc != PX_OK) return rc;
    rc = check_device();
    if (rc != PX_OK) return rc;
    return px::launch_fitness(dims, population, job_params, m_grid, fair_share, current_alloc, node_capacity, p, delta,
                              workspace, fitness, best_m, best_s, best_goodput, speedup, violations, sweep_start,
                              sweep_stop, 0, false, (hipStream_t)hip_stream);
}

}  // namespace

int pollux_fitness(const pollux_dims *dims, const int32_t *population, const double *job_params, const int32_t *m_grid,
                   const int32_t *fair_share, const int32_t *current_alloc, const int32_t *node_capacity, double p,
                   double delta, void *workspace, size_t workspace_bytes, double *fitness, int32_t *best_m,
                   int32_t *best_s, double *best_goodput, double *speedup, int32_t *violations, void *hip_stream)
{
    return fitness_call(dims, population, job_params, m_grid, fair_share, current_alloc, node_capacity, p, delta,
                        workspace, workspace_bytes, fitness, best_m, best_s, best_goodput, speedup, violations, nullptr,
                        nullptr, hip_stream);
}

int pollux_fitness_timed(const pollux_dims *dims, const int32_t *population, const double *job_params,
                         const int32_t *m_grid, const int32_t *fair_share, const int32_t *current_alloc,
                         const int32_t *node_capacity, double p, double delta, void *workspace, size_t workspace_bytes,
                         double *fitness, int32_t *best_m, int32_t *best_s, double *best_goodput, double *speedup,
                         int32_t *violations, void *sweep_start_event, void *sweep_stop_event, void *hip_stream)
{
    if (!sweep_start_event || !sweep_stop_event) return PX_E_INVALID_ARG;
    return fitness_call(dims, population, job_params, m_grid, fair_share, current_alloc, node_capacity, p, delta,
                        workspace, workspace_bytes, fitness, best_m, best_s, best_goodput, speedup, violations,
                        (hipEvent_t)sweep_start_event, (hipEvent_t)sweep_stop_event, hip_stream);
}

int pollux_fitness_static(const pollux_dims *dims, const int32_t *population, const double *job_params,
                          const int32_t *m_grid, const int32_t *fair_share, const int32_t *current_alloc,
                          const int32_t *node_capacity, double p, double delta, double *fitness, int32_t *best_m,
                          int32_t *best_s, double *best_goodput, double *speedup, int32_t *violations,
                          int32_t *status, void *hip_stream)
{
    if (!dims_ok(dims, true)) return PX_E_INVALID_ARG;
    if (!population || !job_params || !m_grid || !fair_share || !current_alloc || !node_capacity || !fitness ||
        (best_m == nullptr) != (best_s == nullptr))
        return PX_E_INVALID_ARG;
    if (!isfinite(p) || !isfinite(delta) || delta < 0.0) return PX_E_INVALID_ARG;
    // the problem must fit the library's array: checked on the host, before any device is touched
    if (px::workspace_layout(*dims).total > (size_t)POLLUX_STATIC_SCRATCH_BYTES) return PX_E_WORKSPACE;
    int dev = 0;
    int rc = check_device(&dev);
    if (rc != PX_OK) return rc;
    void *ws = nullptr;
    rc = static_scratch(dev, &ws);
    if (rc != PX_OK) return rc;
    rc = px::launch_fitness(dims, population, job_params, m_grid, fair_share, current_alloc, node_capacity, p, delta,
                            ws, fitness, best_m, best_s, best_goodput, speedup, violations, nullptr, nullptr, 0, false,
                            (hipStream_t)hip_stream);
    if (rc != PX_OK) return rc;
    return status ? px::launch_copy_status(ws, status, (hipStream_t)hip_stream) : PX_OK;
}

int pollux_ga_step(const pollux_dims *dims, const int32_t *parents, const double *fitness,
                   const int32_t *node_capacity, const pollux_ga_params *params, void *workspace,
                   size_t workspace_bytes, int32_t *children, void *hip_stream)
{
    if (!dims_ok(dims, false)) return PX_E_INVALID_ARG;
    if (!parents || !fitness || !node_capacity || !params || !children) return PX_E_INVALID_ARG;
    if (params->elite_k < 1u || params->elite_k > (uint32_t)dims->P) return PX_E_INVALID_ARG;
    if (!px::ga_shapes_fit(dims->J, dims->N)) return PX_E_INVALID_ARG;   // per-job and per-node bookkeeping lives in LDS
    const size_t bytes = sizeof(int32_t) * (size_t)dims->P * dims->J * dims->N;
    const char *a = (const char *)parents, *b = (const char *)children;
    if (params->flags & ~(uint32_t)PX_GA_IN_PLACE) return PX_E_INVALID_ARG;
    if (params->flags & PX_GA_IN_PLACE) {
        if (a != b) return PX_E_INVALID_ARG;
    } else if (a < b + bytes && b < a + bytes) {
        return PX_E_INVALID_ARG;
    }
    int rc = check_workspace(dims, workspace, workspace_bytes);
    if (rc != PX_OK) return rc;
    rc = check_device();
    if (rc != PX_OK) return rc;
    return px::launch_ga_step(dims, parents, fitness, node_capacity, params, workspace, children, false,
                              (hipStream_t)hip_stream);
}

int pollux_generation(const pollux_dims *dims, int32_t *population, const double *job_params, const int32_t *m_grid,
                      const int32_t *fair_share, const int32_t *current_alloc, const int32_t *node_capacity, double p,
                      double delta, const pollux_ga_params *params, void *workspace, size_t workspace_bytes,
                      double *fitness, int32_t *best_m, int32_t *best_s, double *best_goodput, double *speedup,
                      int32_t *violations, void *hip_stream)
{
    if (!dims_ok(dims, true)) return PX_E_INVALID_ARG;
    if (!population || !job_params || !m_grid || !fair_share || !current_alloc || !node_capacity || !params || !fitness ||
        (best_m == nullptr) != (best_s == nullptr))
        return PX_E_INVALID_ARG;
    if (!isfinite(p) || !isfinite(delta) || delta < 0.0) return PX_E_INVALID_ARG;
    if (params->elite_k < 1u || params->elite_k > (uint32_t)dims->P) return PX_E_INVALID_ARG;
    // the step is in place by definition here
    if (params->flags != (uint32_t)PX_GA_IN_PLACE && params->flags != (uint32_t)(PX_GA_IN_PLACE | PX_GA_INHERIT_ROWS))
        return PX_E_INVALID_ARG;
    const bool inherit_rows = (params->flags & PX_GA_INHERIT_ROWS) != 0;
    // the per-pair results a memoised call leaves in the workspace only on request
    if (inherit_rows && (dims->flags & PX_FLAG_MEMOISE) && !(dims->flags & PX_FLAG_PAIR_RESULTS)) return PX_E_INVALID_ARG;
    if (!px::ga_shapes_fit(dims->J, dims->N)) return PX_E_INVALID_ARG;
    int rc = check_workspace(dims, workspace, workspace_bytes);
    if (rc != PX_OK) return rc;
    rc = check_device();
    if (rc != PX_OK) return rc;
    rc = px::launch_ga_step(dims, population, fitness, node_capacity, params, workspace, population, inherit_rows,
                            (hipStream_t)hip_stream);
    if (rc != PX_OK) return rc;
    pollux_dims kept = *dims;
    kept.flags |= PX_FLAG_KEEP_JOB_TABLES;
    return px::launch_fitness(&kept, population, job_params, m_grid, fair_share, current_alloc, node_capacity, p, delta,
                              workspace, fitness, best_m, best_s, best_goodput, speedup, violations, nullptr, nullptr,
                              (int)params->elite_k, inherit_rows, (hipStream_t)hip_stream);
}

int pollux_apply_best(const pollux_dims *dims, const int32_t *population, const double *fitness, int32_t *current_alloc,
                      int32_t *best, int32_t *K, int32_t *nodes, int32_t *changed, void *hip_stream)
{
    if (!dims_ok(dims, false)) return PX_E_INVALID_ARG;
    if (!population || !fitness || !current_alloc || !best || !K || !nodes || !changed) return PX_E_INVALID_ARG;
    const int rc = check_device();
    if (rc != PX_OK) return rc;
    return px::launch_apply_best(dims, population, fitness, current_alloc, best, K, nodes, changed, (hipStream_t)hip_stream);
}

namespace {

// dims of the calls that use the job-level tables only: the grid sweep in fp64, no flags
bool query_dims_ok(const pollux_dims *d)
{
    return dims_ok(d, true) && d->precision == 0 && d->flags == 0;
}

}  // namespace

int pollux_goodput_per_gpu(const pollux_dims *dims, const double *job_params, const int32_t *m_grid,
                           int32_t gpus_per_node, int32_t max_nodes, void *workspace, size_t workspace_bytes,
                           double *per_gpu, void *hip_stream)
{
    if (!query_dims_ok(dims) || !job_params || !m_grid || !per_gpu) return PX_E_INVALID_ARG;
    if (gpus_per_node < 1 || max_nodes < 1) return PX_E_INVALID_ARG;
    if ((long long)gpus_per_node * max_nodes > 0x7FFFFFFFll || (long long)dims->J * (max_nodes + 1ll) > 0x7FFFFFFFll)
        return PX_E_INVALID_ARG;
    int rc = check_workspace(dims, workspace, workspace_bytes);
    if (rc != PX_OK) return rc;
    rc = check_device();
    if (rc != PX_OK) return rc;
    return px::launch_goodput_per_gpu(dims, job_params, m_grid, gpus_per_node, max_nodes, workspace, per_gpu,
                                      (hipStream_t)hip_stream);
}

int pollux_autoscale(int32_t J, int32_t max_nodes, const double *per_gpu, const int32_t *nodes_now, double U, double L,
                     int32_t *nodes_new, void *hip_stream)
{
    if (J < 1 || max_nodes < 1 || !per_gpu || !nodes_now || !nodes_new) return PX_E_INVALID_ARG;
    if (!isfinite(U) || !isfinite(L)) return PX_E_INVALID_ARG;
    const int rc = check_device();
    if (rc != PX_OK) return rc;
    return px::launch_autoscale(J, max_nodes, per_gpu, nodes_now, U, L, nodes_new, (hipStream_t)hip_stream);
}

int pollux_sim_tick(const pollux_dims *dims, const double *job_params, const int32_t *m_grid, const int32_t *K,
                    const int32_t *nodes, const int32_t *changed, const double *target, double dt, double restart_delay,
                    void *workspace, size_t workspace_bytes, double *progress, double *goodput, int32_t *finished,
                    void *hip_stream)
{
    if (!query_dims_ok(dims) || !job_params || !m_grid || !K || !nodes || !changed || !target || !progress || !goodput ||
        !finished)
        return PX_E_INVALID_ARG;
    if (!isfinite(dt) || !isfinite(restart_delay) || dt < 0.0 || restart_delay < 0.0) return PX_E_INVALID_ARG;
    int rc = check_workspace(dims, workspace, workspace_bytes);
    if (rc != PX_OK) return rc;
    rc = check_device();
    if (rc != PX_OK) return rc;
    return px::launch_sim_tick(dims, job_params, m_grid, K, nodes, changed, target, dt, restart_delay, workspace,
                               progress, goodput, finished, (hipStream_t)hip_stream);
}

int pollux_fit_theta(int32_t J, int32_t max_obs, const int32_t *obs_count, const int32_t *obs_K,
                     const int32_t *obs_nodes, const int32_t *obs_m, const int32_t *obs_s, const double *obs_T,
                     const double *theta_init, int32_t max_iter, int32_t n_starts, double *theta, double *rmsle,
                     int32_t *iterations, void *hip_stream)
{
    if (J < 1 || max_obs < 1 || max_iter < 0 || n_starts < 1 || n_starts > 5) return PX_E_INVALID_ARG;
    if ((long long)J * max_obs > 0x7FFFFFFFll) return PX_E_INVALID_ARG;
    if (!obs_count || !obs_K || !obs_nodes || !obs_m || !obs_s || !obs_T || !theta || !rmsle) return PX_E_INVALID_ARG;
    const int rc = check_device();
    if (rc != PX_OK) return rc;
    return px::launch_fit_theta(J, max_obs, max_iter, n_starts, obs_count, obs_K, obs_nodes, obs_m, obs_s, obs_T, theta_init,
                                theta, rmsle, iterations, (hipStream_t)hip_stream);
}

int pollux_last_status(const void *workspace, void *hip_stream, int32_t *host_out)
{
    if (!workspace || !host_out) return PX_E_INVALID_ARG;
    const char *ws = (const char *)workspace;
    pollux_dims d = {1, 1, 1, 1, 1, 0, 0};
    const size_t off = px::workspace_layout(d).status;    // the status word sits at a fixed offset
    if (hipMemcpyAsync(host_out, ws + off, sizeof(int32_t), hipMemcpyDeviceToHost, (hipStream_t)hip_stream) != hipSuccess)
        return PX_E_HIP;
    if (hipStreamSynchronize((hipStream_t)hip_stream) != hipSuccess) return PX_E_HIP;
    return PX_OK;
}

}  // extern "C"
