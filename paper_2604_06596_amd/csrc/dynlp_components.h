// Label initialisation of a batch's inserted vertices: Alg. 2 Step 1 ("sparsification": the
// batch-internal graph G' keeps the batch edges between two inserted vertices whose weight exceeds
// tau; its connected components are the supernodes) and Step 2 (every supernode starts at its
// share of edge weight towards each labelled class).
//
// The paper flags sub-threshold entries in a device CSR of the batch and runs vertex-centric
// Shiloach-Vishkin hook / jump kernels over it.  Here the batch arrives as an edge list, so the
// kept edges are compacted into a list once and the hook step is edge-centric: an edge whose two
// ends have different parents hooks the larger parent under the smaller one (atomicMin), the jump
// step then compresses every path completely, and the pair repeats until a hook step finds every
// edge inside one tree.  Parents only ever decrease and always stay inside the vertex's component,
// so at the end every vertex points at the smallest id of its component, whatever order the
// atomics took.  Batch-local ids (global id - first inserted id) are used throughout.
#pragma once

#include "dynlp_device.h"

namespace dynlp {

// Device-side counters of one initialisation.
struct InitCtr {
    unsigned int kept;        // |E'|
    unsigned int components;  // number of roots
    unsigned int pad[2];
    unsigned int changed[kInitChain];  // changed[i] != 0: hook step i of the running chain moved a parent
};

// weight sum per block of rows, for the mean edge weight (fixed assignment of rows to threads and a
// fixed reduction order: the result does not depend on timing)
__global__ void __launch_bounds__(kBlock) k_weight_partial(int64_t n, const RowMeta* __restrict__ meta,
                                                          const Edge* __restrict__ pool,
                                                          double* __restrict__ partial) {
    __shared__ double red[kBlock / kWave];
    constexpr int G = 16;
    const int sub = threadIdx.x & (G - 1);
    const int64_t group = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / G;
    const int64_t groups = (int64_t)gridDim.x * kBlock / G;
    double acc = 0.0;
    for (int64_t u = group; u < n; u += groups) {
        const RowMeta rm = meta[u];
        for (int j = sub; j < rm.len; j += G) acc += (double)pool[rm.off + j].w;
    }
    acc = wave_sum(acc);
    if (lane_id() == 0) red[threadIdx.x / kWave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int i = 0; i < kBlock / kWave; ++i) t += red[i];
        partial[blockIdx.x] = t;
    }
}

__global__ void __launch_bounds__(kBlock) k_cc_reset(int64_t k, int32_t* __restrict__ par) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < k) par[i] = (int32_t)i;
}

// E': batch edges with both ends inserted in this batch and weight > tau, as pairs of batch-local
// ids, appended in arbitrary order (a workgroup takes kAppendItems * kBlock edges and reserves its
// output range with one counter atomic).
__global__ void __launch_bounds__(kBlock) k_cc_filter(int64_t m, int64_t n0, int64_t k, const int32_t* __restrict__ eu,
                                                     const int32_t* __restrict__ ev, const float* __restrict__ ew,
                                                     float tau, int2* __restrict__ kept, InitCtr* ctr) {
    __shared__ unsigned int smem[kBlock / kWave + 1];
    const int64_t base = (int64_t)blockIdx.x * kBlock * kAppendItems;
    int2 pairs[kAppendItems];
    unsigned int keepmask = 0;
#pragma unroll
    for (int q = 0; q < kAppendItems; ++q) {
        const int64_t e = base + (int64_t)q * kBlock + threadIdx.x;
        pairs[q] = make_int2(0, 0);
        if (e < m) {
            const int64_t la = (int64_t)eu[e] - n0, lb = (int64_t)ev[e] - n0;
            if (la >= 0 && la < k && lb >= 0 && lb < k && ew[e] > tau) {
                keepmask |= 1u << q;
                pairs[q] = make_int2((int)la, (int)lb);
            }
        }
    }
    unsigned int slot = block_reserve(&ctr->kept, (unsigned int)__popc(keepmask), smem);
#pragma unroll
    for (int q = 0; q < kAppendItems; ++q)
        if ((keepmask >> q) & 1u) kept[slot++] = pairs[q];
}

// Hook step `iter` of a chain.  Skipped when the previous hook step of the chain changed nothing.
// Before every hook step all paths are fully compressed, so the parents read here are roots (or
// were at the start of the step; a root that another lane has just hooked is still in the same
// component, and atomicMin keeps the smaller parent).
__global__ void __launch_bounds__(kBlock) k_cc_hook(int iter, const int2* __restrict__ kept, int32_t* par,
                                                   InitCtr* ctr) {
    if (iter > 0 && __atomic_load_n(&ctr->changed[iter - 1], __ATOMIC_RELAXED) == 0u) return;
    const unsigned int count = ctr->kept;
    const unsigned int stride = gridDim.x * kBlock;
    bool any = false;
    for (unsigned int e = blockIdx.x * kBlock + threadIdx.x; e < count; e += stride) {
        const int2 ab = kept[e];
        const int pa = __atomic_load_n(&par[ab.x], __ATOMIC_RELAXED);
        const int pb = __atomic_load_n(&par[ab.y], __ATOMIC_RELAXED);
        if (pa != pb) {
            const int hi = pa > pb ? pa : pb, lo = pa > pb ? pb : pa;
            // many edges of a large component name the same two roots: only the first of them needs the atomic
            if (__atomic_load_n(&par[hi], __ATOMIC_RELAXED) > lo) atomicMin(&par[hi], lo);
            any = true;
        }
    }
    if (__ballot(any) != 0ull && lane_id() == 0) __atomic_store_n(&ctr->changed[iter], 1u, __ATOMIC_RELAXED);
}

// Jump step: every vertex follows its parents to the root and points at it.  No parent of a root
// changes during this kernel, so the root a walk ends at is final for this step.
__global__ void __launch_bounds__(kBlock) k_cc_jump(int iter, int64_t k, int32_t* par, const InitCtr* ctr) {
    if (__atomic_load_n(&ctr->changed[iter], __ATOMIC_RELAXED) == 0u) return;
    const int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= k) return;
    int p = __atomic_load_n(&par[v], __ATOMIC_RELAXED);
    for (;;) {
        const int q = __atomic_load_n(&par[p], __ATOMIC_RELAXED);
        if (q == p) break;
        p = q;
    }
    __atomic_store_n(&par[v], p, __ATOMIC_RELAXED);
}

// Dense component numbers in ascending order of the root id (= smallest member), three steps:
// roots per block of kBlock vertices; exclusive scan of the block counts by one workgroup; dense id
// of every root.  k_cc_label then gives every vertex the dense id of its root.
__global__ void __launch_bounds__(kBlock) k_cc_count_roots(int64_t k, const int32_t* __restrict__ par,
                                                          unsigned int* __restrict__ block_sum) {
    const int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int is_root = v < k && par[v] == (int32_t)v;
    const int cnt = __syncthreads_count(is_root);
    if (threadIdx.x == 0) block_sum[blockIdx.x] = (unsigned int)cnt;
}

__global__ void __launch_bounds__(kBlock) k_cc_scan_blocks(int64_t nb, unsigned int* __restrict__ block_sum,
                                                          InitCtr* ctr) {
    __shared__ unsigned int smem[kBlock / kWave + 1];
    unsigned int carry = 0;
    for (int64_t base = 0; base < nb; base += kBlock) {
        const int64_t i = base + threadIdx.x;
        const unsigned int v = i < nb ? block_sum[i] : 0u;
        unsigned int total;
        const unsigned int ex = block_exclusive_scan(v, smem, &total);
        if (i < nb) block_sum[i] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) ctr->components = carry;
}

__global__ void __launch_bounds__(kBlock) k_cc_number_roots(int64_t k, const int32_t* __restrict__ par,
                                                           const unsigned int* __restrict__ block_off,
                                                           int32_t* __restrict__ dense) {
    __shared__ unsigned int smem[kBlock / kWave + 1];
    const int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const unsigned int is_root = (v < k && par[v] == (int32_t)v) ? 1u : 0u;
    unsigned int total;
    const unsigned int ex = block_exclusive_scan(is_root, smem, &total);
    if (is_root) dense[v] = (int32_t)(block_off[blockIdx.x] + ex);
}

__global__ void __launch_bounds__(kBlock) k_cc_label(int64_t k, const int32_t* __restrict__ par,
                                                    const int32_t* __restrict__ dense, int32_t* __restrict__ comp) {
    const int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (v < k) comp[v] = dense[par[v]];
}

__global__ void __launch_bounds__(kBlock) k_fill_f64(int64_t count, double* __restrict__ p, double value) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < count) p[i] = value;
}

// Step 2, sums: W[comp(u)][j] += w(u,v) for every inserted vertex u (labelled or not) and every
// neighbour v labelled j.  16 lanes walk one row.  Labelled neighbours are rare, but when the batch-internal graph
// percolates nearly all of them belong to one giant supernode, and atomics on one address run at about 1e8 per
// second (2.2M of them took 22 of this kernel's 26 ms on the 50M-vertex graph).  So a workgroup takes kSwRows
// consecutive rows, collects their contributions (supernode, class, weight) in LDS, adds up those with the same
// target and issues one binary64 atomic per distinct target (a list that overflows goes straight to memory).
// The order of the additions changes a sum by rounding in the 16th digit only, far below the binary32 result.
constexpr int kSwRows = 1024;  // rows per workgroup
constexpr int kSwCap = 1024;   // contributions a workgroup can hold

__global__ void __launch_bounds__(kBlock) k_supernode_weights(int64_t n0, int64_t k, int C,
                                                             const RowMeta* __restrict__ meta,
                                                             const Edge* __restrict__ pool,
                                                             const int32_t* __restrict__ seed_class,
                                                             const int32_t* __restrict__ comp, double* W) {
    __shared__ int32_t s_comp[kSwCap];
    __shared__ int32_t s_cls[kSwCap];
    __shared__ double s_w[kSwCap];
    __shared__ unsigned int s_n;
    if (threadIdx.x == 0) s_n = 0u;
    __syncthreads();
    constexpr int G = 16;
    const int sub = threadIdx.x & (G - 1);
    const int64_t base = (int64_t)blockIdx.x * kSwRows;
    for (int r = threadIdx.x / G; r < kSwRows; r += kBlock / G) {
        const int64_t i = base + r;
        if (i >= k) break;
        const RowMeta rm = meta[n0 + i];
        const int32_t ci = comp[i];
        for (int j = sub; j < rm.len; j += G) {
            const Edge e = pool[rm.off + j];
            const int cls = seed_class[e.col];
            if (cls >= 0) {
                const unsigned int slot = atomicAdd(&s_n, 1u);
                if (slot < (unsigned int)kSwCap) {
                    s_comp[slot] = ci;
                    s_cls[slot] = cls;
                    s_w[slot] = (double)e.w;
                } else {
                    atomicAdd(&W[(int64_t)ci * C + cls], (double)e.w);
                }
            }
        }
    }
    __syncthreads();
    const int L = (int)(s_n < (unsigned int)kSwCap ? s_n : (unsigned int)kSwCap);
    for (int t = threadIdx.x; t < L; t += kBlock) {
        const int32_t ci = s_comp[t], cls = s_cls[t];
        bool first = true;
        for (int q = 0; q < t && first; ++q) first = !(s_comp[q] == ci && s_cls[q] == cls);
        if (!first) continue;
        double sum = s_w[t];
        for (int q = t + 1; q < L; ++q)
            if (s_comp[q] == ci && s_cls[q] == cls) sum += s_w[q];
        atomicAdd(&W[(int64_t)ci * C + cls], sum);
    }
}

// Step 2, rows: F_u[j] = W[comp(u)][j] / sum_j W[comp(u)][j] for every unlabelled inserted vertex,
// 1/C when the supernode has no labelled neighbour; padding columns stay 0.  One lane per stored
// column; every lane adds the C sums in class order.
__global__ void __launch_bounds__(kBlock) k_supernode_rows(int64_t n0, int64_t k, int C, int Cs, int coff, int CP,
                                                          const int32_t* __restrict__ seed_class,
                                                          const int32_t* __restrict__ comp,
                                                          const double* __restrict__ W, float* __restrict__ F) {
    const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t i = t / CP;
    const int j = (int)(t % CP);
    if (i >= k) return;
    const int64_t u = n0 + i;
    if (seed_class[u] >= 0) return;
    const double* Wc = W + (int64_t)comp[i] * C;
    double tot = 0.0;
    for (int c = 0; c < C; ++c) tot += Wc[c];
    float out = 0.f;
    if (j < Cs) out = tot > 0.0 ? (float)(Wc[j + coff] / tot) : 1.0f / (float)C;  // stored column j = class j + coff
    F[u * CP + j] = out;
}

}  // namespace dynlp
