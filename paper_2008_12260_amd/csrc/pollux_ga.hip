// One generation of the population search on gfx950 (Pollux, arXiv 2008.12260,
// Sec. 4.3: candidate allocation matrices are perturbed and combined, then
// modified to satisfy node capacity and interference avoidance, Sec. 4.2).
// The operators are the ones documented at pollux_ga_step in pollux.h; all
// arithmetic is integer.
//
// Kernels
//   rank_kernel                 order[] = candidates by (fitness desc, index asc)
//   children_kernel             one workgroup per child, one wavefront per row:
//                               elite copy, or row-wise crossover + mutation
//   repair_capacity_kernel      one workgroup per child, one thread per node
//   repair_interference_kernel  one workgroup per child: nodes in order, jobs in
//                               parallel, integer LDS atomics (order independent)

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/pollux.h"
#include "pollux_device.h"
#include "pollux_host.h"

namespace px {

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds of two 32x32->64
// multiplications whose high halves are mixed with the other counter words and
// the key; the key advances by a Weyl sequence between rounds.
struct U4 { uint32_t x, y, z, w; };

__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    return U4{c0, c1, c2, c3};
}

enum { kTagParent = 0, kTagCross = 1, kTagMutDecide = 2, kTagMutArgs = 3, kTagRepair = 4 };

__device__ __forceinline__ uint32_t below(uint32_t r, uint32_t n) { return __umulhi(r, n); }

struct GaArgs {
    int P, J, N;
    const int32_t *parents, *node_capacity;
    const double *fitness;
    int32_t *children, *order;
    uint32_t key0, key1, generation, elite_k, mut_threshold;
};

// ---- rank ----------------------------------------------------------------------
// rank(c) = number of candidates that come before c; ranks are distinct, so
// order[rank(c)] = c is a permutation.
__global__ void __launch_bounds__(256) rank_kernel(GaArgs a)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= a.P) return;
    double f = a.fitness[c];
    if (!(f == f)) f = -__builtin_inf();
    int before = 0;
    for (int o = 0; o < a.P; ++o) {
        double g = a.fitness[o];
        if (!(g == g)) g = -__builtin_inf();
        before += (g > f) || (g == f && o < c);
    }
    a.order[before] = c;
}

// ---- children ------------------------------------------------------------------
__global__ void __launch_bounds__(256) children_kernel(GaArgs a)
{
    const int c = blockIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int waves = blockDim.x >> 6;
    const int lane = lane_id();
    const size_t JN = (size_t)a.J * a.N;
    int32_t *__restrict__ child = a.children + (size_t)c * JN;

    if ((uint32_t)c < a.elite_k) {
        const int32_t *__restrict__ src = a.parents + (size_t)a.order[c] * JN;
        for (size_t e = threadIdx.x; e < JN; e += blockDim.x) child[e] = src[e];
        return;
    }
    const U4 pr = philox4x32_10(a.generation, (uint32_t)c, 0u, kTagParent, a.key0, a.key1);
    const int32_t *__restrict__ pa = a.parents + (size_t)a.order[below(pr.x, a.elite_k)] * JN;
    const int32_t *__restrict__ pb = a.parents + (size_t)a.order[below(pr.y, a.elite_k)] * JN;

    for (int j = wave; j < a.J; j += waves) {
        const U4 cr = philox4x32_10(a.generation, (uint32_t)c, (uint32_t)j, kTagCross, a.key0, a.key1);
        const int32_t *__restrict__ src = ((cr.x & 1u) ? pb : pa) + (size_t)j * a.N;
        int32_t *__restrict__ dst = child + (size_t)j * a.N;
        const U4 md = philox4x32_10(a.generation, (uint32_t)c, (uint32_t)j, kTagMutDecide, a.key0, a.key1);
        int move = -1, target = -1;
        if (md.x < a.mut_threshold) {
            const U4 ma = philox4x32_10(a.generation, (uint32_t)c, (uint32_t)j, kTagMutArgs, a.key0, a.key1);
            move = (int)(ma.x % 3u);
            target = (int)below(ma.y, (uint32_t)a.N);
        }
        if (move == 2) {
            // re-pack: the whole row goes to one node, as far as that node's capacity allows
            long long k = 0;
            for (int n = lane; n < a.N; n += kWave) k += src[n];
            k = wave_sum(k);
            if (k < 0) k = 0;
            const long long cap = a.node_capacity[target];
            const int32_t put = (int32_t)(k < cap ? k : cap);
            for (int n = lane; n < a.N; n += kWave) dst[n] = (n == target) ? put : 0;
        } else {
            for (int n = lane; n < a.N; n += kWave) {
                int32_t v = src[n];
                if (n == target) {
                    if (move == 0) v += 1;
                    else if (v > 0) v -= 1;     // move == 1
                }
                dst[n] = v;
            }
        }
    }
}

// ---- repair: node capacity -------------------------------------------------------
__global__ void __launch_bounds__(256) repair_capacity_kernel(GaArgs a)
{
    const int c = blockIdx.x + (int)a.elite_k;      // elites are kept verbatim
    int32_t *__restrict__ A = a.children + (size_t)c * a.J * a.N;
    for (int n = threadIdx.x; n < a.N; n += blockDim.x) {
        long long total = 0;
        for (int j = 0; j < a.J; ++j) total += A[(size_t)j * a.N + n];
        long long excess = total - (long long)a.node_capacity[n];
        if (excess <= 0) continue;
        const U4 r = philox4x32_10(a.generation, (uint32_t)c, (uint32_t)n, kTagRepair, a.key0, a.key1);
        int j = (int)below(r.x, (uint32_t)a.J);
        for (int t = 0; t < a.J && excess > 0; ++t) {
            const long long have = A[(size_t)j * a.N + n];
            if (have > 0) {
                const long long take = have < excess ? have : excess;
                A[(size_t)j * a.N + n] = (int32_t)(have - take);
                excess -= take;
            }
            j = (j + 1 == a.J) ? 0 : j + 1;
        }
    }
}

// ---- repair: at most one multi-node job per node ------------------------------------
__global__ void __launch_bounds__(256) repair_interference_kernel(GaArgs a)
{
    extern __shared__ int32_t nodes_of[];           // [J] nodes occupied by each job
    __shared__ int count;                           // multi-node jobs present on the current node
    __shared__ unsigned long long keep;             // (GPUs there) << 32 | ~job: maximum = most GPUs, lowest job
    const int c = blockIdx.x + (int)a.elite_k;
    int32_t *__restrict__ A = a.children + (size_t)c * a.J * a.N;
    const int wave = threadIdx.x >> 6, waves = blockDim.x >> 6, lane = lane_id();

    for (int j = wave; j < a.J; j += waves) {
        int cnt = 0;
        for (int n0 = 0; n0 < a.N; n0 += kWave) {
            const int n = n0 + lane;
            cnt += __popcll(__ballot(n < a.N && A[(size_t)j * a.N + n] > 0));
        }
        if (lane == 0) nodes_of[j] = cnt;
    }
    if (threadIdx.x == 0) { count = 0; keep = 0ull; }
    __syncthreads();

    for (int n = 0; n < a.N; ++n) {
        for (int j = threadIdx.x; j < a.J; j += blockDim.x) {
            const int32_t v = A[(size_t)j * a.N + n];
            if (v > 0 && nodes_of[j] >= 2) {
                atomicAdd(&count, 1);
                atomicMax(&keep, ((unsigned long long)(uint32_t)v << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)j));
            }
        }
        __syncthreads();
        const int cnt = count;
        const int keeper = (int)(0xFFFFFFFFu - (uint32_t)(keep & 0xFFFFFFFFull));
        __syncthreads();
        if (cnt > 1) {
            for (int j = threadIdx.x; j < a.J; j += blockDim.x) {
                if (j == keeper) continue;
                if (A[(size_t)j * a.N + n] > 0 && nodes_of[j] >= 2) {
                    A[(size_t)j * a.N + n] = 0;
                    nodes_of[j] -= 1;
                }
            }
        }
        if (threadIdx.x == 0) { count = 0; keep = 0ull; }
        __syncthreads();
    }
}

int launch_ga_step(const pollux_dims *d, const int32_t *parents, const double *fitness, const int32_t *node_capacity,
                   const pollux_ga_params *ga, void *workspace, int32_t *children, hipStream_t stream)
{
    const WorkspaceLayout L = workspace_layout(*d);
    GaArgs a;
    a.P = d->P; a.J = d->J; a.N = d->N;
    a.parents = parents; a.node_capacity = node_capacity; a.fitness = fitness;
    a.children = children;
    a.order = (int32_t *)((char *)workspace + L.order);
    a.key0 = (uint32_t)(ga->seed & 0xFFFFFFFFull);
    a.key1 = (uint32_t)(ga->seed >> 32);
    a.generation = ga->generation; a.elite_k = ga->elite_k; a.mut_threshold = ga->mut_threshold;

    hipLaunchKernelGGL(rank_kernel, dim3((unsigned)((d->P + 255) / 256)), dim3(256), 0, stream, a);
    hipLaunchKernelGGL(children_kernel, dim3((unsigned)d->P), dim3(256), 0, stream, a);
    const int bred = d->P - (int)ga->elite_k;
    if (bred > 0) {
        hipLaunchKernelGGL(repair_capacity_kernel, dim3((unsigned)bred), dim3(256), 0, stream, a);
        hipLaunchKernelGGL(repair_interference_kernel, dim3((unsigned)bred), dim3(256), sizeof(int32_t) * (size_t)d->J,
                           stream, a);
    }
    return hipGetLastError() == hipSuccess ? PX_OK : PX_E_HIP;
}

}  // namespace px
