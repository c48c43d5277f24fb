// One generation of the population search on gfx950 (Pollux, arXiv 2008.12260,
// Sec. 4.3: candidate allocation matrices are perturbed and combined, then
// modified to satisfy node capacity and interference avoidance, Sec. 4.2).
// The operators are the ones documented at pollux_ga_step in pollux.h; all
// arithmetic is integer.
//
// Kernels
//   rank_kernel                 order[] = candidates by (fitness desc, index asc)
//   generation_kernel           one workgroup per child: elite copy, or row-wise
//                               crossover + mutation, then both repairs, with the
//                               per-node bookkeeping in LDS

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

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
    const int32_t *job_gpu_cap;    // [J] or null
    const double *fitness;
    int32_t *children, *order;
    uint32_t key0, key1, generation, elite_k, mut_threshold;
    int max_entries;   // capacity of the per-node entry lists in LDS
    int in_place;      // children == parents: only children c >= elite_k are formed, child c goes to slot order[c]
    // Row inheritance (in place only; all three null otherwise).  Child c = elite_k + k:
    int32_t *src_row;      // [P - elite_k, J]: the candidate whose row j the child holds unchanged, or -1 if a move or a
                           // repair has changed the row
    int32_t *odd;          // [P - elite_k]: 1 if the child may violate a constraint or hold a negative entry (a negative
                           // entry was met, a node could not be brought within its capacity, or the node lists
                           // overflowed), so that nothing about it may be taken for granted
    int32_t *dirty_count;  // [J], set to zero by the step: the rows to be swept are counted there afterwards, per job
};

// ---- rank ----------------------------------------------------------------------
// rank(c) = number of candidates that come before c; ranks are distinct, so
// order[rank(c)] = c is a permutation.
__global__ void __launch_bounds__(256) rank_kernel(GaArgs a)
{
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int c = blockIdx.x * 4 + wave;           // one wavefront per candidate, lanes over the others
    if (a.dirty_count && blockIdx.x == 0) {
        for (int j = threadIdx.x; j < a.J; j += blockDim.x) a.dirty_count[j] = 0;
    }
    if (c >= a.P) return;
    const int lane = lane_id();
    double f = a.fitness[c];
    if (!(f == f)) f = -__builtin_inf();
    // every lane counts among the candidates o = lane, lane + 64, ...; eight loads are requested together
    // (past the end the last candidate is read again and not counted)
    constexpr int kBatch = 8;
    int mine = 0;
    for (int o0 = 0; o0 < a.P; o0 += kBatch * kWave) {
        double g[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int o = o0 + u * kWave + lane;
            g[u] = a.fitness[o < a.P ? o : a.P - 1];
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int o = o0 + u * kWave + lane;
            const double gu = (g[u] == g[u]) ? g[u] : -__builtin_inf();
            const bool first = (gu > f) | ((gu == f) & (o < c));
            mine += (int)((o < a.P) & first);
        }
    }
    const int before = wave_sum(mine);
    if (lane == 0) a.order[before] = c;
}

// ---- one child per workgroup: build, repair capacity, repair interference ---------
//
// Allocation matrices are sparse (a job sits on a few of the N nodes), so while the
// rows are built every positive entry is also threaded into a per-node list in LDS:
// entry e = (job, GPUs, next entry of the same node).  Both repairs then work on those
// lists and touch global memory only to write the entries they change.
//
// LDS (dynamic): colsum[N] GPUs asked per node (64-bit); nodes_of[J] nodes occupied by
// each row; colcnt[N] multi-node jobs per node; dist[J] indices of multi-node jobs;
// dec[J], decx[J] the drawn decisions of each row; head[N] and the entry arrays.
//
// Step A  one thread per job draws the row's decisions (Philox), then one wavefront
//         per row: crossover source, mutation, write the row, count its nodes, add
//         its entries to colsum and to the node lists.
// Step B  one thread per node over capacity: visit the jobs present in cyclic order
//         from the drawn start and take GPUs away until the node fits.
// Step C  the nodes are taken in ascending order: among the multi-node jobs present the
//         largest holder stays (lowest job on ties) and the others are zeroed there.
//         Sequential by definition: a job that loses a node may stop being multi-node,
//         which later nodes must see.  One thread per node first lists the node's
//         multi-node entries (up to four) in LDS; one wavefront then visits only the nodes
//         that list two or more, four lanes looking at a node's entries together.
// When a matrix has more positive entries than the lists hold (dense matrices) steps
// B and C run the same rules on columns read from memory instead.
// Matrices of at most 64 nodes (the instances with FOUR) keep, instead of the lists, an array of
// entries per node (kNodeCap each; more: the column path).  Step B then gives half a wavefront to a
// node: lane k holds its k-th entry, and what a job gives up, min(its GPUs, the excess less the
// GPUs of the jobs before it in the cyclic order), needs a sum over the entries with a smaller
// cyclic distance, which every lane forms for itself: no walk, no second pass.  Step C lists the
// multi-node entries of every node from the arrays, and the wavefront that takes the nodes in order
// holds the listed entries of sixteen nodes in registers, four lanes a node.
//
// A workgroup re-reads global memory written by its own wavefronts only in that
// fallback; __syncthreads() orders those accesses (one CU, one L1).

constexpr int kGaThreads = 512;     // eight wavefronts keep enough row loads in flight to approach copy bandwidth
// Capacity of the per-node entry lists: one and a half entries per job (allocations hold a little more than one
// node per job), in steps of 256, between 512 and 3072.  Fewer entries mean less LDS per workgroup and more
// workgroups per CU, i.e. more rows in flight; a matrix with more positive entries takes the column path.
inline int ga_max_entries(int J)
{
    long long e = (((long long)J * 3 / 2 + 255) / 256) * 256;
    return (int)(e < 512 ? 512 : (e > 3072 ? 3072 : e));
}

constexpr int kNodeSlots = 4;       // multi-node entries listed per node for step C (more: that node's list is walked)
// Rows of at most 64 nodes (the instances with FOUR): instead of the lists every node keeps its entries as an array,
// which 32 lanes read together, so that neither repair walks anything.  A node with more entries than its array
// holds sends the child down the column path.
constexpr int kNodeCap = 32;
constexpr int kArrayNodes = 64;     // the arrays exist for matrices of at most this many nodes

struct GaShared {
    unsigned long long *colsum;
    int32_t *nodes_of, *colcnt, *dist, *dec, *decx, *head;
    int32_t *ent_j, *ent_v, *ent_next;
    uint16_t *slot;                 // [N, kNodeSlots] entry indices; shares the memory of dec / decx, which step A is done with
    // N <= kArrayNodes only: entries per node; per node and position the job and its GPUs there
    int32_t *ncnt, *arr_j, *arr_v;
};

__device__ __forceinline__ GaShared carve_shared(unsigned char *base, int J, int N, int max_entries)
{
    GaShared sh;
    sh.colsum = (unsigned long long *)base;                         // 8-byte aligned first
    sh.nodes_of = (int32_t *)(sh.colsum + N);
    sh.colcnt = sh.nodes_of + J;
    sh.dist = sh.colcnt + N;
    sh.dec = sh.dist + J;
    sh.decx = sh.dec + J;
    sh.head = sh.decx + J;
    sh.ent_j = sh.head + N;
    sh.ent_v = sh.ent_j + max_entries;
    sh.ent_next = sh.ent_v + max_entries;
    // 2 * kNodeSlots bytes per node: inside dec / decx (8 bytes per job) when J >= N, else behind the entry arrays
    sh.slot = J >= N ? (uint16_t *)sh.dec : (uint16_t *)(sh.ent_next + max_entries);
    sh.ncnt = sh.ent_next + max_entries + (J >= N ? 0 : (2 * kNodeSlots * N) / 4);
    sh.arr_j = sh.ncnt + N;
    sh.arr_v = sh.arr_j + N * kNodeCap;
    return sh;
}

inline size_t ga_shared_bytes(int J, int N)
{
    return 16 * (size_t)N + 16 * (size_t)J + 12 * (size_t)ga_max_entries(J) + (J >= N ? 0 : 2 * kNodeSlots * (size_t)N) +
           (N <= kArrayNodes ? 4 * (size_t)N + 8 * (size_t)N * kNodeCap : 0);
}

// What a workgroup may use: the 160 KB of a compute unit less the kernel's few static variables, rounded down.
constexpr size_t kGaMaxShared = 159 * 1024;
constexpr int kGaDevices = 64;

bool ga_shapes_fit(int J, int N) { return ga_shared_bytes(J, N) <= kGaMaxShared; }

// Number of positive entries of a row; every lane returns the same value.
__device__ __forceinline__ int count_occupied(const int32_t *__restrict__ row, int N, int lane)
{
    int occupied = 0;
    for (int n0 = 0; n0 < N; n0 += kWave) {
        const int n = n0 + lane;
        occupied += __popcll(__ballot(n < N && row[n] > 0));
    }
    return occupied;
}

// Index of the pick-th positive entry of a row in ascending order (pick < number of positive entries).
__device__ __forceinline__ int kth_occupied(const int32_t *__restrict__ row, int N, int lane, int pick)
{
    int seen = 0;
    for (int n0 = 0; n0 < N; n0 += kWave) {
        const int n = n0 + lane;
        unsigned long long mask = __ballot(n < N && row[n] > 0);
        const int here = __popcll(mask);
        if (pick < seen + here) {
            for (int t = pick - seen; t > 0; --t) mask &= mask - 1;       // drop the lower set bits
            return n0 + (__ffsll(mask) - 1);
        }
        seen += here;
    }
    return -1;
}

// (GPUs there) << 32 | ~job: the maximum is the largest holder, lowest job index on ties
__device__ __forceinline__ unsigned long long holder_key(int32_t v, int j)
{
    return ((unsigned long long)(uint32_t)v << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)j);
}

// FOUR: the host has checked that rows are 16-byte groups of at most 64 nodes and no per-job GPU limit is given.
// INHERIT: the step also records where every row of the child comes from (GaArgs::src_row, odd); an instance of its
// own, so that the plain step pays nothing for it (a few scalar registers more would cost it a workgroup per CU).
template <bool FOUR, bool INHERIT>
__global__ void __launch_bounds__(kGaThreads) __attribute__((amdgpu_num_sgpr(96))) generation_kernel(GaArgs a)
{
    extern __shared__ __align__(16) unsigned char ga_lds[];
    __shared__ int count, n_dist, n_ent;
    __shared__ int odd;             // see GaArgs::odd
    __shared__ int spill;           // FOUR: a node has more entries than its array holds
    __shared__ unsigned long long keep;

    const int c = a.in_place ? (int)(blockIdx.x + a.elite_k) : (int)blockIdx.x;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int waves = kGaThreads >> 6;
    const int lane = lane_id();
    const size_t JN = (size_t)a.J * a.N;
    int32_t *__restrict__ child = a.children + (size_t)(a.in_place ? a.order[c] : c) * JN;

    if ((uint32_t)c < a.elite_k) {
        // survivors are copied verbatim, in rank order
        const int32_t *__restrict__ src = a.parents + (size_t)a.order[c] * JN;
        if ((JN & 3) == 0 && (((uintptr_t)src | (uintptr_t)child) & 15) == 0) {
            const int4 *__restrict__ s4 = (const int4 *)src;
            int4 *__restrict__ d4 = (int4 *)child;
            for (size_t e = tid; e < (JN >> 2); e += kGaThreads) d4[e] = s4[e];
        } else {
            for (size_t e = tid; e < JN; e += kGaThreads) child[e] = src[e];
        }
        return;
    }

    const GaShared sh = carve_shared(ga_lds, a.J, a.N, a.max_entries);
    for (int n = tid; n < a.N; n += kGaThreads) {
        sh.colsum[n] = 0ull; sh.colcnt[n] = 0; sh.head[n] = -1;
        if constexpr (FOUR) sh.ncnt[n] = 0;
    }
    if (tid == 0) { count = 0; n_dist = 0; n_ent = 0; keep = 0ull; odd = 0; spill = 0; }
    // row inheritance: where the child's rows come from (see GaArgs)
    int32_t *__restrict__ src_row = INHERIT ? a.src_row + (size_t)(c - (int)a.elite_k) * a.J : nullptr;

    // ---- step A ----
    // decisions of every row, one thread per job: dec[j] = source parent | (move + 1) << 1, decx[j] = the
    // second word of the mutation draw (which node)
    for (int j = tid; j < a.J; j += kGaThreads) {
        const U4 cr = philox4x32_10(a.generation, (uint32_t)c, (uint32_t)j, kTagCross, a.key0, a.key1);
        const U4 md = philox4x32_10(a.generation, (uint32_t)c, (uint32_t)j, kTagMutDecide, a.key0, a.key1);
        int d = (int)(cr.x & 1u);
        uint32_t x = 0u;
        if (md.x < a.mut_threshold) {
            const U4 ma = philox4x32_10(a.generation, (uint32_t)c, (uint32_t)j, kTagMutArgs, a.key0, a.key1);
            d |= (int)((ma.x % 3u) + 1u) << 1;
            x = ma.y;
        }
        sh.dec[j] = d;
        sh.decx[j] = (int32_t)x;
    }
    const U4 pr = philox4x32_10(a.generation, (uint32_t)c, 0u, kTagParent, a.key0, a.key1);
    const int32_t *__restrict__ pa = a.parents + (size_t)a.order[below(pr.x, a.elite_k)] * JN;
    // half of the children have a single parent (mutation only)
    const int32_t *__restrict__ pb = (pr.z & 1u) ? pa : a.parents + (size_t)a.order[below(pr.y, a.elite_k)] * JN;
    // the two parents as candidates (what src_row names)
    int cand_a = 0, cand_b = 0;
    if constexpr (INHERIT) {
        cand_a = a.order[below(pr.x, a.elite_k)];
        cand_b = (pr.z & 1u) ? cand_a : a.order[below(pr.y, a.elite_k)];
    }
    const bool vec4 = (a.N & 3) == 0 && (((uintptr_t)a.parents | (uintptr_t)a.children) & 15) == 0;
    __syncthreads();

    // a positive entry of the child: per-node total and node list
    auto record = [&](int j, int n, int32_t v) {
        atomicAdd(&sh.colsum[n], (unsigned long long)(long long)v);
        if (INHERIT && v < 0) odd = 1;
        if (v > 0) {
            if constexpr (FOUR) {
                const int k = atomicAdd(&sh.ncnt[n], 1);
                if (k < kNodeCap) {
                    sh.arr_j[n * kNodeCap + k] = j;
                    sh.arr_v[n * kNodeCap + k] = v;
                } else {
                    spill = 1;
                }
            } else {
                const int e = atomicAdd(&n_ent, 1);
                if (e < a.max_entries) {
                    sh.ent_j[e] = j;
                    sh.ent_v[e] = v;
                    sh.ent_next[e] = atomicExch(&sh.head[n], e);
                }
            }
        }
    };

    // Rows of at most 64 nodes that are copied unchanged (no move drawn, no GPU limit to apply): four rows per
    // load of the wavefront, 16 lanes each.  The loop after this one then takes only the rows with a move.
    if constexpr (FOUR) {
        const int n4 = a.N >> 2;
        const int g = lane >> 4, l16 = lane & 15;
        for (int j0 = 4 * wave; j0 < a.J; j0 += 4 * waves) {
            const int j = j0 + g;
            const int d = j < a.J ? sh.dec[j] : 2;
            const bool plain = (d >> 1) == 0;
            int4 v = {0, 0, 0, 0};
            if (plain && l16 < n4) {
                v = ((const int4 *)(((d & 1) ? pb : pa) + (size_t)j * a.N))[l16];
                ((int4 *)(child + (size_t)j * a.N))[l16] = v;
                const int n = 4 * l16;
                if (v.x != 0) record(j, n, v.x);
                if (v.y != 0) record(j, n + 1, v.y);
                if (v.z != 0) record(j, n + 2, v.z);
                if (v.w != 0) record(j, n + 3, v.w);
            }
            const int nodes = row16_sum((v.x > 0 ? 1 : 0) + (v.y > 0 ? 1 : 0) + (v.z > 0 ? 1 : 0) + (v.w > 0 ? 1 : 0));
            if (plain && l16 == 0) {
                sh.nodes_of[j] = nodes;
                if (nodes >= 2) sh.dist[atomicAdd(&n_dist, 1)] = j;
                if (INHERIT) src_row[j] = (d & 1) ? cand_b : cand_a;
            }
        }
    }

    // one row by one wavefront: the move (if any), the job's GPU limit, the copy, the bookkeeping
    auto row_by_wavefront = [&](int j, int d) {
        const int32_t *__restrict__ src = ((d & 1) ? pb : pa) + (size_t)j * a.N;
        int32_t *__restrict__ dst = child + (size_t)j * a.N;
        const int move = ((d >> 1) & 3) - 1;
        int target = -1, delta = 0;
        int32_t put = 0;
        if (move == 2) {
            // re-pack: the whole row goes to one drawn node, as far as that node's capacity allows
            target = (int)below((uint32_t)__builtin_amdgcn_readfirstlane(sh.decx[j]), (uint32_t)a.N);
            long long k = 0;
            for (int n = lane; n < a.N; n += kWave) k += src[n];
            k = wave_sum(k);
            if (k < 0) k = 0;
            const long long cap = a.node_capacity[target];
            put = (int32_t)(k < cap ? k : cap);
        } else if (move >= 0) {
            // grow / shrink by one GPU on one of the nodes the job occupies (a job without GPUs grows on a drawn node)
            const uint32_t x = (uint32_t)__builtin_amdgcn_readfirstlane(sh.decx[j]);
            const int occupied = count_occupied(src, a.N, lane);
            if (occupied > 0) {
                target = kth_occupied(src, a.N, lane, (int)below(x, (uint32_t)occupied));
                delta = move == 0 ? 1 : -1;
            } else if (move == 0) {
                target = (int)below(x, (uint32_t)a.N);
                delta = 1;
            }
        }
        // the entry of node n after the move
        auto moved = [&](int n, int32_t v) -> int32_t {
            if (move == 2) return (n == target) ? put : 0;
            return n == target ? v + delta : v;
        };
        int nodes = 0;
        // GPU limit of the job: needed only when the row after the move holds more than the limit (rare);
        // that row is then written by the slower path below, which keeps GPUs in ascending node order.
        bool over_limit = false;
        long long limit = 0;
        if (a.job_gpu_cap) {
            limit = a.job_gpu_cap[j];
            if (limit < 0) limit = 0;
            long long k = 0;
            for (int n = lane; n < a.N; n += kWave) {
                const int32_t v = moved(n, src[n]);
                k += v > 0 ? v : 0;
            }
            over_limit = wave_sum(k) > limit;
        }
        if (over_limit) {
            long long kept = 0;                       // GPUs kept on the nodes before this group of 64
            for (int n0 = 0; n0 < a.N; n0 += kWave) {
                const int n = n0 + lane;
                int32_t v = n < a.N ? moved(n, src[n]) : 0;
                const long long pos = v > 0 ? v : 0;
                long long before = kept;              // plus the positive entries of the lower lanes
                for (int l = 0; l < kWave; ++l) {
                    const long long other = wave_broadcast(pos, l);
                    if (l < lane) before += other;
                    kept += other;
                }
                if (n < a.N) {
                    if (v > 0) {
                        const long long room = limit - before;
                        if (v > room) v = (int32_t)(room > 0 ? room : 0);
                    }
                    dst[n] = v;
                    if (v != 0) record(j, n, v);
                }
                nodes += __popcll(__ballot(v > 0));
            }
        } else if (vec4) {
            const int4 *__restrict__ s4 = (const int4 *)src;
            int4 *__restrict__ d4 = (int4 *)dst;
            const int n4 = a.N >> 2;
            for (int q0 = 0; q0 < n4; q0 += kWave) {
                const int q = q0 + lane;
                int4 v = {0, 0, 0, 0};
                if (q < n4) {
                    v = s4[q];
                    const int n = q * 4;
                    v.x = moved(n, v.x); v.y = moved(n + 1, v.y); v.z = moved(n + 2, v.z); v.w = moved(n + 3, v.w);
                    d4[q] = v;
                    if (v.x != 0) record(j, n, v.x);
                    if (v.y != 0) record(j, n + 1, v.y);
                    if (v.z != 0) record(j, n + 2, v.z);
                    if (v.w != 0) record(j, n + 3, v.w);
                }
                nodes += __popcll(__ballot(v.x > 0)) + __popcll(__ballot(v.y > 0)) + __popcll(__ballot(v.z > 0)) +
                         __popcll(__ballot(v.w > 0));
            }
        } else {
            for (int n0 = 0; n0 < a.N; n0 += kWave) {
                const int n = n0 + lane;
                int32_t v = 0;
                if (n < a.N) {
                    v = moved(n, src[n]);
                    dst[n] = v;
                    if (v != 0) record(j, n, v);
                }
                nodes += __popcll(__ballot(v > 0));
            }
        }
        if (lane == 0) sh.nodes_of[j] = nodes;
        if (nodes >= 2 && lane == 0) sh.dist[atomicAdd(&n_dist, 1)] = j;
        if (INHERIT && lane == 0) src_row[j] = (move < 0 && !over_limit) ? ((d & 1) ? cand_b : cand_a) : -1;
    };
    if constexpr (FOUR) {
        // only the rows with a move are left: every wavefront reads the decisions 64 at a time and takes, of the rows
        // that have one, those whose number is its own modulo the number of wavefronts (a few per child: walking
        // all rows to find them cost one LDS round trip per row)
        static_assert(kGaThreads / kWave == 8, "the pattern below picks every eighth row");
        for (int jb = 0; jb < a.J; jb += kWave) {
            const int jj = jb + lane;
            const int dd = jj < a.J ? sh.dec[jj] : 0;
            unsigned long long mine = __ballot((dd >> 1) != 0) & (0x0101010101010101ull << wave);
            while (mine != 0ull) {
                const int b = __builtin_ctzll(mine);
                mine &= mine - 1ull;
                row_by_wavefront(jb + b, __builtin_amdgcn_readlane(dd, b));
            }
        }
    } else {
        for (int j = wave; j < a.J; j += waves) row_by_wavefront(j, __builtin_amdgcn_readfirstlane(sh.dec[j]));
    }
    __syncthreads();

    if constexpr (FOUR) {
      if (spill == 0) {
        static_assert(kNodeCap == 32 && kWave == 64 && kArrayNodes == 64 && kGaThreads == 512,
                      "a half of a wavefront per node, four nodes per half");
        const int half = lane >> 5, k = lane & 31;
        // the entries this lane looks after: the k-th of nodes 2 wave + half, + 16, + 32, + 48
        int ej[4], ev[4], en[4], have[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            en[r] = 16 * r + 2 * wave + half;
            ej[r] = 0;
            ev[r] = 0;
            have[r] = en[r] < a.N ? sh.ncnt[en[r]] : 0;
            if (k < have[r]) {
                ej[r] = sh.arr_j[en[r] * kNodeCap + k];
                ev[r] = sh.arr_v[en[r] * kNodeCap + k];
            }
        }
        // ---- step B on the node arrays.  In the cyclic order from the drawn start a job gives up
        // min(its GPUs, what is still to take after the jobs before it), and "before it" is a sum over the
        // entries with a smaller distance: every lane forms its own, no walk, no second pass.
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int n = en[r];
            const long long excess = n < a.N ? (long long)sh.colsum[n] - (long long)a.node_capacity[n] : 0ll;
            const bool over = excess > 0;
            if (__ballot(over) == 0ull) continue;
            int dist = 0x7FFFFFFF;                      // cyclic distance of the job from the start; no job: last
            if (over && ev[r] > 0) {
                const U4 rr = philox4x32_10(a.generation, (uint32_t)c, (uint32_t)n, kTagRepair, a.key0, a.key1);
                const int j0 = (int)below(rr.x, (uint32_t)a.J);
                dist = ej[r] >= j0 ? ej[r] - j0 : ej[r] - j0 + a.J;
            }
            long long before = 0, present = 0;
            const int most = max(__builtin_amdgcn_readlane(have[r], 0), __builtin_amdgcn_readlane(have[r], 32));
            for (int i = 0; i < most; ++i) {
                const int from = ((lane & 32) + i) << 2;
                const int di = __builtin_amdgcn_ds_bpermute(from, dist), vi = __builtin_amdgcn_ds_bpermute(from, ev[r]);
                if (di != 0x7FFFFFFF) {
                    present += vi;
                    if (di < dist) before += vi;
                }
            }
            const long long room = excess - before;
            if (dist != 0x7FFFFFFF && room > 0) {
                const int32_t left = (long long)ev[r] <= room ? 0 : (int32_t)((long long)ev[r] - room);
                ev[r] = left;
                child[(size_t)ej[r] * a.N + n] = left;
                if (INHERIT) src_row[ej[r]] = -1;
                if (left == 0) atomicSub(&sh.nodes_of[ej[r]], 1);
            }
            if (INHERIT && over && present < excess) odd = 1;     // nothing left to take away: the node stays over its capacity
        }
        __syncthreads();
        if (INHERIT && tid == 0) a.odd[c - (int)a.elite_k] = odd;   // final: step C only removes entries
        // ---- step C on the node arrays: first the listing, which multi-node jobs each node holds now (their positions
        // in the node's array, up to kNodeSlots of them) ...
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const bool multi = ev[r] > 0 && sh.nodes_of[ej[r]] >= 2;
            const unsigned long long both = __ballot(multi);
            const unsigned mine = half ? (unsigned)(both >> 32) : (unsigned)both;
            const int pos = __popc(mine & ((1u << k) - 1u));
            if (multi && pos < kNodeSlots) sh.slot[en[r] * kNodeSlots + pos] = (uint16_t)(en[r] * kNodeCap + k);
            if (en[r] < a.N && k == 0) sh.colcnt[en[r]] = __popc(mine);
            // (step B's outcome, for the walk below of a node that lists more than kNodeSlots)
            if (k < have[r]) sh.arr_v[en[r] * kNodeCap + k] = ev[r];
        }
        __syncthreads();
        if (wave != 0) return;
        // ... then one wavefront takes the nodes in ascending order, 16 at a time: four lanes hold a node's listed
        // entries, so a node that lists two or more costs one look at its jobs' node counts (which the nodes before
        // it may have lowered), a maximum over four lanes and the writes.
        for (int n0 = 0; n0 < a.N; n0 += 16) {
            const int n = n0 + (lane >> 2), q = lane & 3;
            const int listed_n = n < a.N ? sh.colcnt[n] : 0;
            int j = 0;
            int32_t v = 0;
            const bool has = q < listed_n && q < kNodeSlots;
            if (has) {
                const int at = sh.slot[n * kNodeSlots + q];
                j = sh.arr_j[at];
                v = sh.arr_v[at];
            }
            unsigned long long conflicts = __ballot(q == 0 && listed_n > 1);
            while (conflicts != 0ull) {
                const int first = __builtin_ctzll(conflicts);          // the node's first lane
                conflicts &= conflicts - 1ull;
                const int nn = n0 + (first >> 2);
                const int listed = __builtin_amdgcn_readlane(listed_n, first);
                if (listed <= kNodeSlots) {
                    const bool multi = has && (lane >> 2) == (first >> 2) && sh.nodes_of[j] >= 2;
                    if (__popcll(__ballot(multi)) > 1) {
                        long long key = multi ? (long long)holder_key(v, j) : 0ll;      // below 2^63: v is positive
                        long long other = exchange<0>(key);
                        key = other > key ? other : key;
                        other = exchange<1>(key);
                        key = other > key ? other : key;                                  // the four lanes agree
                        const int keeper = (int)(0xFFFFFFFFu - (uint32_t)((unsigned long long)key & 0xFFFFFFFFull));
                        if (multi && j != keeper) {
                            child[(size_t)j * a.N + nn] = 0;
                            if (INHERIT) src_row[j] = -1;
                            sh.nodes_of[j] -= 1;
                        }
                    }
                } else if (lane == 0) {
                    const int entries = sh.ncnt[nn];
                    int cnt = 0;
                    unsigned long long best = 0ull;
                    for (int t = 0; t < entries; ++t) {
                        const int jt = sh.arr_j[nn * kNodeCap + t];
                        const int32_t vt = sh.arr_v[nn * kNodeCap + t];
                        if (vt > 0 && sh.nodes_of[jt] >= 2) {
                            cnt++;
                            const unsigned long long key = holder_key(vt, jt);
                            best = key > best ? key : best;
                        }
                    }
                    if (cnt > 1) {
                        const int keeper = (int)(0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull));
                        for (int t = 0; t < entries; ++t) {
                            const int jt = sh.arr_j[nn * kNodeCap + t];
                            if (jt != keeper && sh.arr_v[nn * kNodeCap + t] > 0 && sh.nodes_of[jt] >= 2) {
                                child[(size_t)jt * a.N + nn] = 0;
                                if (INHERIT) src_row[jt] = -1;
                                sh.nodes_of[jt] -= 1;
                            }
                        }
                    }
                }
            }
        }
        return;
      }
    }

    if (!FOUR && n_ent <= a.max_entries) {
        // ---- step B on the node lists ----
        for (int n = tid; n < a.N; n += kGaThreads) {
            long long excess = (long long)sh.colsum[n] - (long long)a.node_capacity[n];
            if (excess <= 0) continue;
            const U4 r = philox4x32_10(a.generation, (uint32_t)c, (uint32_t)n, kTagRepair, a.key0, a.key1);
            const int j0 = (int)below(r.x, (uint32_t)a.J);
            int last = -1;                                  // cyclic distance from j0 of the job visited last
            while (excess > 0) {
                int pick = -1, pick_dist = 0x7FFFFFFF;
                for (int e = sh.head[n]; e >= 0; e = sh.ent_next[e]) {
                    if (sh.ent_v[e] <= 0) continue;
                    const int j = sh.ent_j[e];
                    const int dist = j >= j0 ? j - j0 : j - j0 + a.J;
                    if (dist > last && dist < pick_dist) { pick = e; pick_dist = dist; }
                }
                if (pick < 0) break;
                const long long have = sh.ent_v[pick];
                const long long take = have < excess ? have : excess;
                const int j = sh.ent_j[pick];
                sh.ent_v[pick] = (int32_t)(have - take);
                child[(size_t)j * a.N + n] = (int32_t)(have - take);
                if (INHERIT) src_row[j] = -1;
                excess -= take;
                if (take == have) atomicSub(&sh.nodes_of[j], 1);
                last = pick_dist;
            }
            if (INHERIT && excess > 0) odd = 1;             // nothing left to take away: the node stays over its capacity
        }
        __syncthreads();
        if (INHERIT && tid == 0) a.odd[c - (int)a.elite_k] = odd;   // final: step C only removes entries
        // ---- step C on the node lists ----
        // which multi-node jobs each node holds now (later removals can only take some away)
        for (int n = tid; n < a.N; n += kGaThreads) {
            int cnt = 0;
            for (int e = sh.head[n]; e >= 0; e = sh.ent_next[e]) {
                if (sh.ent_v[e] > 0 && sh.nodes_of[sh.ent_j[e]] >= 2) {
                    if (cnt < kNodeSlots) sh.slot[n * kNodeSlots + cnt] = (uint16_t)e;
                    cnt++;
                }
            }
            sh.colcnt[n] = cnt;
        }
        __syncthreads();
        if (wave != 0) return;
        for (int n0 = 0; n0 < a.N; n0 += kWave) {
            unsigned long long conflicts = __ballot(n0 + lane < a.N && sh.colcnt[n0 + lane < a.N ? n0 + lane : 0] > 1);
            while (conflicts) {
                const int n = n0 + __ffsll(conflicts) - 1;
                conflicts &= conflicts - 1;
                const int listed = __builtin_amdgcn_readfirstlane(sh.colcnt[n]);
                if (listed <= kNodeSlots) {
                    // lane k < listed looks at the k-th listed entry
                    int j = 0;
                    int32_t v = 0;
                    bool multi = false;
                    if (lane < listed) {
                        const int e = sh.slot[n * kNodeSlots + lane];
                        j = sh.ent_j[e];
                        v = sh.ent_v[e];
                        multi = sh.nodes_of[j] >= 2;
                    }
                    if (__popcll(__ballot(multi)) > 1) {
                        long long key = multi ? (long long)holder_key(v, j) : 0ll;      // below 2^63: v is positive
                        long long other = exchange<0>(key);
                        key = other > key ? other : key;
                        other = exchange<1>(key);
                        key = other > key ? other : key;                                  // the four lanes agree
                        const int keeper = (int)(0xFFFFFFFFu - (uint32_t)((unsigned long long)key & 0xFFFFFFFFull));
                        if (multi && j != keeper) {
                            child[(size_t)j * a.N + n] = 0;
                            if (INHERIT) src_row[j] = -1;
                            sh.nodes_of[j] -= 1;
                        }
                    }
                } else if (lane == 0) {
                    int cnt = 0;
                    unsigned long long best = 0ull;
                    for (int e = sh.head[n]; e >= 0; e = sh.ent_next[e]) {
                        const int j = sh.ent_j[e];
                        if (sh.ent_v[e] > 0 && sh.nodes_of[j] >= 2) {
                            cnt++;
                            const unsigned long long key = holder_key(sh.ent_v[e], j);
                            best = key > best ? key : best;
                        }
                    }
                    if (cnt > 1) {
                        const int keeper = (int)(0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull));
                        for (int e = sh.head[n]; e >= 0; e = sh.ent_next[e]) {
                            const int j = sh.ent_j[e];
                            if (j != keeper && sh.ent_v[e] > 0 && sh.nodes_of[j] >= 2) {
                                child[(size_t)j * a.N + n] = 0;
                                if (INHERIT) src_row[j] = -1;
                                sh.nodes_of[j] -= 1;
                            }
                        }
                    }
                }
            }
        }
        return;
    }

    // ---- dense fallback: step B on columns read from memory ----
    if (INHERIT && tid == 0) a.odd[c - (int)a.elite_k] = 1;     // evaluated in full afterwards: src_row is not kept up
    for (int n = tid; n < a.N; n += kGaThreads) {
        long long excess = (long long)sh.colsum[n] - (long long)a.node_capacity[n];
        if (excess <= 0) continue;
        const U4 r = philox4x32_10(a.generation, (uint32_t)c, (uint32_t)n, kTagRepair, a.key0, a.key1);
        int j = (int)below(r.x, (uint32_t)a.J);
        for (int t = 0; t < a.J && excess > 0; ++t) {
            const long long have = child[(size_t)j * a.N + n];
            if (have > 0) {
                const long long take = have < excess ? have : excess;
                child[(size_t)j * a.N + n] = (int32_t)(have - take);
                excess -= take;
                if (take == have) atomicSub(&sh.nodes_of[j], 1);
            }
            j = (j + 1 == a.J) ? 0 : j + 1;
        }
    }
    __syncthreads();
    // ---- dense fallback: step C, integer LDS atomics (order independent) ----
    const int nd = n_dist;
    for (int k = wave; k < nd; k += waves) {
        const int j = sh.dist[k];
        if (__builtin_amdgcn_readfirstlane(sh.nodes_of[j]) < 2) continue;      // capacity repair left it on one node
        for (int n = lane; n < a.N; n += kWave)
            if (child[(size_t)j * a.N + n] > 0) atomicAdd(&sh.colcnt[n], 1);
    }
    __syncthreads();
    for (int n = 0; n < a.N; ++n) {
        if (__builtin_amdgcn_readfirstlane(sh.colcnt[n]) <= 1) continue;
        for (int k = tid; k < nd; k += kGaThreads) {
            const int j = sh.dist[k];
            const int32_t v = child[(size_t)j * a.N + n];
            if (v > 0 && sh.nodes_of[j] >= 2) {
                atomicAdd(&count, 1);
                atomicMax(&keep, holder_key(v, j));
            }
        }
        __syncthreads();
        const int cnt = count;
        const int keeper = (int)(0xFFFFFFFFu - (uint32_t)(keep & 0xFFFFFFFFull));
        __syncthreads();
        if (cnt > 1) {
            for (int k = tid; k < nd; k += kGaThreads) {
                const int j = sh.dist[k];
                if (j == keeper) continue;
                if (child[(size_t)j * a.N + n] > 0 && sh.nodes_of[j] >= 2) {
                    child[(size_t)j * a.N + n] = 0;
                    sh.nodes_of[j] -= 1;
                }
            }
        }
        if (tid == 0) { count = 0; keep = 0ull; }
        __syncthreads();
    }
}

// ---- applying the outcome of a search --------------------------------------------------
// The matrix PolluxSched applies at the end of a scheduling interval is the candidate of highest fitness
// (Sec. 4.3), i.e. the first in the order of rank_kernel: fitness descending, index ascending, NaN last.
__global__ void __launch_bounds__(256) best_kernel(int P, const double *__restrict__ fitness, int32_t *__restrict__ best)
{
    __shared__ double red_f[256];
    __shared__ int red_c[256];
    const int t = threadIdx.x;
    double f = -__builtin_inf();
    int c = 0x7FFFFFFF;
    for (int o = t; o < P; o += 256) {
        double g = fitness[o];
        if (!(g == g)) g = -__builtin_inf();
        if (c == 0x7FFFFFFF || g > f) { f = g; c = o; }        // ascending o: an equal value keeps the lower index
    }
    red_f[t] = f;
    red_c[t] = c;
    __syncthreads();
    for (int half = 128; half > 0; half >>= 1) {
        if (t < half) {
            const double g = red_f[t + half];
            const int o = red_c[t + half];
            if (o != 0x7FFFFFFF && (red_c[t] == 0x7FFFFFFF || g > red_f[t] || (g == red_f[t] && o < red_c[t]))) {
                red_f[t] = g;
                red_c[t] = o;
            }
        }
        __syncthreads();
    }
    if (t == 0) *best = red_c[0];
}

// One wavefront per job: the job's row of the best candidate becomes its current row; K, nodes and the
// re-allocation flag (row differs from the previous current row, which held at least one GPU) are reported.
__global__ void __launch_bounds__(256) apply_kernel(int J, int N, const int32_t *__restrict__ population,
                                                    const int32_t *__restrict__ best, int32_t *__restrict__ current,
                                                    int32_t *__restrict__ K_out, int32_t *__restrict__ nodes_out,
                                                    int32_t *__restrict__ changed_out)
{
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int j = blockIdx.x * 4 + wave;
    if (j >= J) return;
    const int lane = lane_id();
    const int32_t *__restrict__ row = population + ((size_t)*best * J + j) * N;
    int32_t *__restrict__ cur = current + (size_t)j * N;
    long long k = 0, held = 0;
    int nodes = 0;
    bool differs = false;
    for (int n0 = 0; n0 < N; n0 += kWave) {
        const int n = n0 + lane;
        const int32_t v = n < N ? row[n] : 0, was = n < N ? cur[n] : 0;
        k += v;
        held += was;
        nodes += __popcll(__ballot(v > 0));
        differs |= __ballot(v != was) != 0;
        if (n < N) cur[n] = v;
    }
    k = wave_sum(k);
    held = wave_sum(held);
    if (lane == 0) {
        K_out[j] = (int32_t)k;
        nodes_out[j] = nodes;
        changed_out[j] = (differs && held > 0) ? 1 : 0;
    }
}

int launch_apply_best(const pollux_dims *d, const int32_t *population, const double *fitness, int32_t *current_alloc,
                      int32_t *best, int32_t *K, int32_t *nodes, int32_t *changed, hipStream_t stream)
{
    hipLaunchKernelGGL(best_kernel, dim3(1), dim3(256), 0, stream, d->P, fitness, best);
    hipLaunchKernelGGL(apply_kernel, dim3((unsigned)((d->J + 3) / 4)), dim3(256), 0, stream, d->J, d->N, population, best,
                       current_alloc, K, nodes, changed);
    return hipGetLastError() == hipSuccess ? PX_OK : PX_E_HIP;
}

int launch_ga_step(const pollux_dims *d, const int32_t *parents, const double *fitness, const int32_t *node_capacity,
                   const pollux_ga_params *ga, void *workspace, int32_t *children, bool inherit_rows, hipStream_t stream)
{
    const WorkspaceLayout L = workspace_layout(*d);
    GaArgs a;
    a.P = d->P; a.J = d->J; a.N = d->N;
    a.parents = parents; a.node_capacity = node_capacity; a.fitness = fitness;
    a.children = children;
    a.job_gpu_cap = ga->job_gpu_cap;
    a.order = (int32_t *)((char *)workspace + L.order);
    a.key0 = (uint32_t)(ga->seed & 0xFFFFFFFFull);
    a.key1 = (uint32_t)(ga->seed >> 32);
    a.generation = ga->generation; a.elite_k = ga->elite_k; a.mut_threshold = ga->mut_threshold;
    a.in_place = (ga->flags & PX_GA_IN_PLACE) ? 1 : 0;
    a.max_entries = ga_max_entries(d->J);
    a.src_row = nullptr; a.odd = nullptr; a.dirty_count = nullptr;
    if (inherit_rows && a.in_place) {
        a.src_row = (int32_t *)((char *)workspace + L.src_row);
        a.odd = (int32_t *)((char *)workspace + L.odd);
        a.dirty_count = (int32_t *)((char *)workspace + L.dirty_count);
    }

    hipLaunchKernelGGL(rank_kernel, dim3((unsigned)((d->P + 3) / 4)), dim3(256), 0, stream, a);
    const size_t lds = ga_shared_bytes(d->J, d->N);
    const bool four = (d->N & 3) == 0 && d->N <= kWave && !a.job_gpu_cap && (((uintptr_t)a.parents | (uintptr_t)a.children) & 15) == 0;
    const bool inherit = a.src_row != nullptr;
    const int instance = (four ? 1 : 0) + (inherit ? 2 : 0);
    const void *kernels[4] = {(const void *)generation_kernel<false, false>, (const void *)generation_kernel<true, false>,
                              (const void *)generation_kernel<false, true>, (const void *)generation_kernel<true, true>};
    if (lds > 48 * 1024) {
        // Beyond 48 KB a kernel must be allowed its dynamic LDS explicitly.  The allowance is raised per kernel
        // instance and device, and only when a call needs more than any earlier one did.
        static std::mutex lock;
        static size_t allowed[4][kGaDevices];
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kGaDevices) return PX_E_HIP;
        std::lock_guard<std::mutex> hold(lock);
        if (allowed[instance][dev] < lds) {
            if (hipFuncSetAttribute(kernels[instance], hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return PX_E_HIP;
            allowed[instance][dev] = lds;
        }
    }
    const unsigned children_formed = a.in_place ? (unsigned)d->P - ga->elite_k : (unsigned)d->P;
    if (children_formed > 0) {
        const dim3 grid(children_formed), block(kGaThreads);
        if (instance == 0) hipLaunchKernelGGL((generation_kernel<false, false>), grid, block, lds, stream, a);
        else if (instance == 1) hipLaunchKernelGGL((generation_kernel<true, false>), grid, block, lds, stream, a);
        else if (instance == 2) hipLaunchKernelGGL((generation_kernel<false, true>), grid, block, lds, stream, a);
        else hipLaunchKernelGGL((generation_kernel<true, true>), grid, block, lds, stream, a);
    }
    return hipGetLastError() == hipSuccess ? PX_OK : PX_E_HIP;
}

}  // namespace px
