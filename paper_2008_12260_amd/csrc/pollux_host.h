// Host-side declarations shared by the translation units of the library:
// workspace layout and the launch functions behind the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/pollux.h"

namespace px {

// The last pass of Eq. 10 is tabled for GPU counts K = 1..kTableK; larger K are computed in place.
constexpr int kTableK = 64;

// Byte offsets of the sections of the caller's workspace (each 256-byte aligned).  The sections whose size
// depends on P, J and N only come first, so that their offsets are the same for every grid: the search step
// (which ignores Gm and Gs) and a fitness call that keeps the job tables may then share one workspace
// whatever grid dimensions the former is given.
struct WorkspaceLayout {
    size_t status;    // int32 status word
    size_t k1;        // int32            the tables of the "one node" class cover K <= this (largest node capacity)
    size_t order;     // int32  [P]       candidates by rank (search step)
    size_t redo;      // int32  [P]       memoised mode: candidates with a row beyond the memo table
    size_t curmask;   // uint64 [J]       16-byte groups of the job's current row that hold a non-zero entry
    size_t zeros;     // 64 zero bytes
    size_t rk;        // double [256]     1/K
    size_t denom;     // double [J]       fair-share goodput
    size_t factor;    // double [J]       re-allocation factor
    size_t running;   // int32  [J]       job holds GPUs in current_alloc
    size_t G;         // double [P,J]     best goodput of the pair
    size_t meta;      // int32  [P,J]     nodes occupied by the row | changed flag
    size_t memo;      // 16 bytes [J,2,kTableK]  best point per (job, one node?, K) in memoised mode
    size_t colpack;   // uint64 [P,N]     per node of each candidate: GPUs asked + multi-node jobs << 40
    // row inheritance of pollux_generation (child k = the candidate of rank elite_k + k)
    size_t src_row;   // int32  [P,J]     the candidate whose row j child k holds unchanged, or -1
    size_t odd;       // int32  [P]       child k may violate a constraint: nothing about it is taken for granted
    size_t dirty_count;  // int32 [J]     rows of job j to sweep
    size_t dirty;     // int32  [J,P]     the candidates those rows belong to (row stride: the number of children)
    // from here on the offsets depend on the grid
    size_t rs;        // double [Gs up to a multiple of 32]  1/(s+1)
    size_t rsf;       // float  [Gs up to a multiple of 32]  the same in fp32
    size_t tg;        // double [J,Gm,2]  T_grad(m_i) and its reciprocal
    size_t lntg;      // double [J,Gm]    ln T_grad(m_i)
    size_t pu;        // double [J,Gm]    phi / m_i
    size_t qh5;       // double [J,Gm]    floor(M_max / m_i) + 1/2
    size_t ql5;       // double [J,Gm]    ceil(M0 / m_i) - 1/2
    size_t lt;        // double [J,2,kTableK,Gm]  last pass of Eq. 10 by (job, one node?, K)
    size_t ca;        // double [J,2,kTableK,Gm,2]  the sweep's (C, A0) by (job, one node?, K, grid point)
    size_t srange;    // int32  [J,kTableK,Gm]  feasible accumulation counts of grid point i with K GPUs:
                      //                  first | last << 16 (first > last: none)
    size_t total;
};

inline WorkspaceLayout workspace_layout(const pollux_dims &d)
{
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    WorkspaceLayout L;
    size_t o = 0;
    const size_t P = (size_t)d.P, J = (size_t)d.J, Gm = (size_t)(d.Gm > 0 ? d.Gm : 1), Gs = (size_t)(d.Gs > 0 ? d.Gs : 1);
    L.status = o;  o = up(o + 256);
    L.k1 = o;      o = up(o + 256);
    L.order = o;   o = up(o + 4 * P);
    L.redo = o;    o = up(o + 4 * P);
    L.curmask = o; o = up(o + 8 * J);
    L.zeros = o;   o = up(o + 64);
    L.rk = o;      o = up(o + 8 * 256);
    L.denom = o;   o = up(o + 8 * J);
    L.factor = o;  o = up(o + 8 * J);
    L.running = o; o = up(o + 4 * J);
    L.G = o;       o = up(o + 8 * P * J);
    L.meta = o;    o = up(o + 4 * P * J);
    L.memo = o;    o = up(o + 16 * J * 2 * kTableK);
    L.colpack = o; o = up(o + 8 * P * (size_t)d.N);
    L.src_row = o; o = up(o + 4 * P * J);
    L.odd = o;     o = up(o + 4 * P);
    L.dirty_count = o; o = up(o + 4 * J);
    L.dirty = o;   o = up(o + 4 * P * J);
    L.rs = o;      o = up(o + 8 * ((Gs + 31) / 32) * 32);
    L.rsf = o;     o = up(o + 4 * ((Gs + 31) / 32) * 32);
    L.tg = o;      o = up(o + 16 * J * Gm);
    L.lntg = o;    o = up(o + 8 * J * Gm);
    L.pu = o;      o = up(o + 8 * J * Gm);
    L.qh5 = o;     o = up(o + 8 * J * Gm);
    L.ql5 = o;     o = up(o + 8 * J * Gm);
    L.lt = o;      o = up(o + 8 * J * 2 * kTableK * Gm);
    L.ca = o;      o = up(o + 16 * J * 2 * kTableK * Gm);
    L.srange = o;  o = up(o + 4 * J * kTableK * Gm);
    L.total = o;
    return L;
}

int launch_fitness(const pollux_dims *d, const int32_t *population, const double *job_params, const int32_t *m_grid,
                   const int32_t *fair_share, const int32_t *current_alloc, const int32_t *node_capacity, double p,
                   double delta, void *workspace, double *fitness, int32_t *best_m, int32_t *best_s,
                   double *best_goodput, double *speedup, int32_t *violations, hipEvent_t sweep_start,
                   hipEvent_t sweep_stop, int first_rank, bool inherit_rows, hipStream_t stream);
// the two events, if given, bracket the grid-sweep kernel; first_rank > 0 evaluates only the candidates of that
// rank and beyond in the order the last search step left in the workspace (dims must carry PX_FLAG_KEEP_JOB_TABLES);
// inherit_rows (with first_rank > 0, after launch_ga_step with inherit_rows): rows a child holds unchanged take over
// their parent's results, only the others are swept

// Copies the status word of `workspace` to *status_out (device memory) on the stream.
int launch_copy_status(const void *workspace, int32_t *status_out, hipStream_t stream);

int launch_ga_step(const pollux_dims *d, const int32_t *parents, const double *fitness, const int32_t *node_capacity,
                   const pollux_ga_params *ga, void *workspace, int32_t *children, bool inherit_rows, hipStream_t stream);
// inherit_rows (in place only): the step also leaves, in the workspace, where every row of every child comes from
// (WorkspaceLayout::src_row, odd) and clears the count of rows to sweep, for launch_fitness with inherit_rows

// True when the search step's per-job and per-node bookkeeping for J jobs and N nodes fits the LDS of a workgroup.
bool ga_shapes_fit(int J, int N);

int launch_apply_best(const pollux_dims *d, const int32_t *population, const double *fitness, int32_t *current_alloc,
                      int32_t *best, int32_t *K, int32_t *nodes, int32_t *changed, hipStream_t stream);

int launch_goodput_per_gpu(const pollux_dims *d, const double *job_params, const int32_t *m_grid, int gpus_per_node,
                           int max_nodes, void *workspace, double *per_gpu, hipStream_t stream);

int launch_autoscale(int J, int max_nodes, const double *per_gpu, const int32_t *nodes_now, double U, double L,
                     int32_t *nodes_new, hipStream_t stream);

int launch_sim_tick(const pollux_dims *d, const double *job_params, const int32_t *m_grid, const int32_t *K,
                    const int32_t *nodes, const int32_t *changed, const double *target, double dt, double restart_delay,
                    void *workspace, double *progress, double *goodput, int32_t *finished, hipStream_t stream);

int launch_fit_theta(int J, int max_obs, int max_iter, int n_starts, const int32_t *count, const int32_t *K, const int32_t *nodes,
                     const int32_t *m, const int32_t *s, const double *T, const double *init, double *theta,
                     double *rmsle, int32_t *iterations, hipStream_t stream);

}  // namespace px
