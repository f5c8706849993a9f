// HIP kernels of the DynLP hot path for gfx950 (wave64, no MFMA: the path is a sparse gather).
#pragma once

#include "dynlp_device.h"

namespace dynlp {

// =================================================================================================
// Slack-CSR construction (mutable CSR with per-row slack)
// =================================================================================================
__host__ __device__ inline int32_t row_capacity(int64_t len, float slack) {
    int64_t a = (int64_t)((double)len * (double)slack + 0.999999);
    int64_t b = len + 4;
    int64_t c = a > b ? a : b;
    c = (c + (kRowAlign - 1)) / kRowAlign * kRowAlign;
    return (int32_t)c;
}

// row_ptr must start at 0, never decrease and end at nnz.
__global__ void __launch_bounds__(kBlock) k_validate_row_ptr(int64_t n, const int64_t* __restrict__ row_ptr,
                                                            int64_t nnz, BatchCtr* bc) {
    const int64_t u = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (u >= n) return;
    const int64_t a = row_ptr[u], b = row_ptr[u + 1];
    if ((u == 0 && a != 0) || a > b || b > nnz || a < 0 || (b - a) > 0x7fffffff - 64) report_error(bc, kErrRowPtr, u);
}

// len, cap of every row and the per-block sums of the capacities.
__global__ void __launch_bounds__(kBlock) k_row_caps(int64_t n, const int64_t* __restrict__ row_ptr, float slack,
                                                    RowMeta* __restrict__ meta, int64_t* __restrict__ block_sums) {
    __shared__ int64_t sm[kBlock / kWave + 1];
    const int64_t u = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    int64_t cap = 0;
    if (u < n) {
        const int64_t len = row_ptr[u + 1] - row_ptr[u];
        cap = row_capacity(len, slack);
        meta[u].len = (int32_t)len;
        meta[u].cap = (int32_t)cap;
    }
    int64_t total;
    block_exclusive_scan<int64_t>(cap, sm, &total);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

// Exclusive scan of nb values in place by one workgroup; *grand_total receives the sum.
__global__ void __launch_bounds__(kBlock) k_scan_block_sums(int64_t nb, int64_t* __restrict__ sums,
                                                           unsigned long long* grand_total) {
    __shared__ int64_t sm[kBlock / kWave + 1];
    const int64_t per = (nb + kBlock - 1) / kBlock;
    const int64_t lo = (int64_t)threadIdx.x * per;
    const int64_t hi = lo + per < nb ? lo + per : nb;
    int64_t local = 0;
    for (int64_t i = lo; i < hi; ++i) local += sums[i];
    int64_t total;
    int64_t run = block_exclusive_scan<int64_t>(local, sm, &total);
    for (int64_t i = lo; i < hi; ++i) {
        const int64_t t = sums[i];
        sums[i] = run;
        run += t;
    }
    if (threadIdx.x == 0 && grand_total) *grand_total = (unsigned long long)total;
}

__global__ void __launch_bounds__(kBlock) k_row_offsets(int64_t n, RowMeta* __restrict__ meta,
                                                       const int64_t* __restrict__ block_offsets) {
    __shared__ int64_t sm[kBlock / kWave + 1];
    const int64_t u = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t cap = u < n ? meta[u].cap : 0;
    int64_t total;
    const int64_t ex = block_exclusive_scan<int64_t>(cap, sm, &total);
    if (u < n) meta[u].off = block_offsets[blockIdx.x] + ex;
}

// One thread per CSR entry: find its row, check it, store it in the pool.
__global__ void __launch_bounds__(kBlock) k_scatter_entries(int64_t nnz, int64_t n, const int64_t* __restrict__ row_ptr,
                                                           const int32_t* __restrict__ col,
                                                           const float* __restrict__ w,
                                                           const RowMeta* __restrict__ meta, Edge* __restrict__ pool,
                                                           BatchCtr* bc) {
    const int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (j >= nnz) return;
    int64_t lo = 0, hi = n;  // largest u with row_ptr[u] <= j
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (row_ptr[mid] <= j) lo = mid; else hi = mid;
    }
    const int64_t u = lo;
    const int32_t c = col[j];
    const float ww = w[j];
    if (c < 0 || c >= n) { report_error(bc, kErrColRange, j); return; }
    if (c == u) { report_error(bc, kErrSelfLoop, j); return; }
    if (!(ww > 0.f) || !isfinite(ww)) { report_error(bc, kErrWeight, j); return; }
    Edge e;
    e.col = c;
    e.w = ww;
    pool[meta[u].off + (j - row_ptr[u])] = e;
}

// Degree d(u) = sum of the row's weights, in stored order (deterministic for a given order).
__global__ void __launch_bounds__(kBlock) k_row_degree(int64_t n, const RowMeta* __restrict__ meta,
                                                      const Edge* __restrict__ pool, float* __restrict__ deg) {
    constexpr int G = 16;
    const int64_t u = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / G;
    const int gl = threadIdx.x % G;
    if (u >= n) return;
    const RowMeta m = meta[u];
    float s = 0.f;
    for (int j = gl; j < m.len; j += G) s += pool[m.off + j].w;
#pragma unroll
    for (int d = G / 2; d > 0; d >>= 1) s += __shfl_xor(s, d, G);
    if (gl == 0) deg[u] = s;
}

// =================================================================================================
// Labels: initialisation, seed clamping, argmax, packing
// =================================================================================================
// Rows [u0, u1): seed rows one-hot, others uniform 1/C, padding columns 0.
// Stored column c holds class c + coff: coff = 0 and Cs = C normally; the binary scalar layout
// (C = 2) stores only class 1 (Cs = 1, coff = 1), class 0 being 1 - F_u.
__global__ void __launch_bounds__(kBlock) k_init_labels(int64_t u0, int64_t u1, int C, int Cs, int coff, int CP,
                                                       const int32_t* __restrict__ seed_class,
                                                       float* __restrict__ F) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t u = u0 + i / CP;
    const int c = (int)(i % CP);
    if (u >= u1) return;
    const int sc = seed_class[u];
    float v = 0.f;
    if (c < Cs) v = sc < 0 ? 1.0f / (float)C : (c + coff == sc ? 1.0f : 0.0f);
    F[u * CP + c] = v;
}

__global__ void __launch_bounds__(kBlock) k_fill_i32(int64_t u0, int64_t u1, int32_t* __restrict__ a, int32_t v) {
    const int64_t i = u0 + (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < u1) a[i] = v;
}

__global__ void __launch_bounds__(kBlock) k_init_meta(int64_t u0, int64_t u1, RowMeta* __restrict__ meta,
                                                     float* __restrict__ deg) {
    const int64_t i = u0 + (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < u1) {
        RowMeta m;
        m.off = 0;
        m.len = 0;
        m.cap = 0;
        meta[i] = m;
        deg[i] = 0.f;
    }
}

// Seeds: range checks, clash with an existing label, two classes for one vertex in this list.
// tmp is an all-zero int32 scratch (n_total entries) that k_clear_seed_tmp restores afterwards.
__global__ void __launch_bounds__(kBlock) k_validate_seeds(int64_t s, int64_t n_total, int64_t n_existing, int C,
                                                          const int32_t* __restrict__ sv,
                                                          const int32_t* __restrict__ sc,
                                                          const int32_t* __restrict__ seed_class,
                                                          int32_t* __restrict__ tmp, BatchCtr* bc) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= s) return;
    const int32_t v = sv[i], c = sc[i];
    if (v < 0 || v >= n_total) { report_error(bc, kErrSeedVertex, i); return; }
    if (c < 0 || c >= C) { report_error(bc, kErrSeedClass, i); return; }
    if (v < n_existing && seed_class[v] >= 0 && seed_class[v] != c) { report_error(bc, kErrRelabel, i); return; }
    const int32_t old = atomicCAS(&tmp[v], 0, c + 1);
    if (old != 0 && old != c + 1) report_error(bc, kErrSeedConflict, i);
}

__global__ void __launch_bounds__(kBlock) k_clear_seed_tmp(int64_t s, int64_t n_total, const int32_t* __restrict__ sv,
                                                          int32_t* __restrict__ tmp) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= s) return;
    const int32_t v = sv[i];
    if (v >= 0 && v < n_total) tmp[v] = 0;
}

__global__ void __launch_bounds__(kBlock) k_set_seed_class(int64_t s, const int32_t* __restrict__ sv,
                                                          const int32_t* __restrict__ sc,
                                                          int32_t* __restrict__ seed_class) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < s) seed_class[sv[i]] = sc[i];
}

// New seeds of a batch: clamp the row one-hot (the row is never updated again) and put the
// neighbours into V_aff.  16 lanes per seed.
__global__ void __launch_bounds__(kBlock) k_apply_seeds(int64_t s, const int32_t* __restrict__ sv,
                                                       const int32_t* __restrict__ sc, int Cs, int coff, int CP,
                                                       int32_t* __restrict__ seed_class, float* __restrict__ F,
                                                       const RowMeta* __restrict__ meta,
                                                       const Edge* __restrict__ pool, uint8_t* __restrict__ flag) {
    constexpr int G = 16;
    const int64_t i = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / G;
    const int gl = threadIdx.x % G;
    if (i >= s) return;
    const int32_t v = sv[i], c = sc[i];
    if (gl == 0) seed_class[v] = c;
    for (int k = gl; k < CP; k += G) F[(int64_t)v * CP + k] = (k < Cs && k + coff == c) ? 1.0f : 0.0f;
    const RowMeta m = meta[v];
    for (int j = gl; j < m.len; j += G) flag[pool[m.off + j].col] = 1;
}

// hard[u] = argmax_c F[u][c], lowest index on ties.  A row of CP >= 4 floats is read by CP/4 adjacent
// lanes as one float4 each (a coalesced 16*L-byte segment per row); the lanes' (value, index) pairs
// are then merged with xor shuffles.  CP < 4 rows are read by one lane.
__global__ void __launch_bounds__(kBlock) k_argmax(int64_t n, int C, int CP, const float* __restrict__ F,
                                                  int32_t* __restrict__ hard) {
    const int L = CP >= 4 ? CP / 4 : 1;  // lanes per row: 1, 2, 4, 8 or 16
    const int64_t u = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / L;
    const int sub = threadIdx.x & (L - 1);
    const bool live = u < n;
    float bv = -1.0f;  // label values are >= 0
    int best = 0;
    if (live) {
        const float* row = F + u * CP;
        if (CP >= 4) {
            const float4 q = *reinterpret_cast<const float4*>(row + 4 * sub);
            const float v[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int c = 4 * sub + k;
                if (c < C && v[k] > bv) { bv = v[k]; best = c; }
            }
        } else {
            bv = row[0];
            for (int c = 1; c < C; ++c)
                if (row[c] > bv) { bv = row[c]; best = c; }
        }
    }
    for (int d = L >> 1; d > 0; d >>= 1) {
        const float ov = __shfl_xor(bv, d);
        const int ob = __shfl_xor(best, d);
        if (ov > bv || (ov == bv && ob < best)) { bv = ov; best = ob; }
    }
    if (live && sub == 0) hard[u] = best;
}

__global__ void __launch_bounds__(kBlock) k_pack_soft(int64_t n, int C, int CP, const float* __restrict__ F,
                                                     float* __restrict__ soft) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n * C) return;
    soft[i] = F[(i / C) * CP + (i % C)];
}

// Binary scalar layout: hard label = the paper's 0.5 cut-off (class 1 iff F_u > 0.5, i.e. iff class 1
// beats class 0; a tie goes to class 0 like the argmax), soft row = (1 - F_u, F_u).
__global__ void __launch_bounds__(kBlock) k_scalar_hard(int64_t n, const float* __restrict__ F,
                                                       int32_t* __restrict__ hard) {
    const int64_t u = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (u < n) hard[u] = F[u] > 0.5f ? 1 : 0;
}

__global__ void __launch_bounds__(kBlock) k_scalar_soft(int64_t n, const float* __restrict__ F,
                                                       float* __restrict__ soft) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= 2 * n) return;
    const float f = F[i >> 1];
    soft[i] = (i & 1) ? f : 1.0f - f;
}

// =================================================================================================
// Edge insertion (Alg. 2 Step 1 for insertions) into the slack CSR
// =================================================================================================
// index_base: position of eu[0] in the caller's batch (the arrays may be one chunk of it), for the error report.
__global__ void __launch_bounds__(kBlock) k_validate_edges(int64_t m, int64_t n_total, const int32_t* __restrict__ eu,
                                                          const int32_t* __restrict__ ev,
                                                          const float* __restrict__ ew, BatchCtr* bc,
                                                          int64_t index_base = 0) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= m) return;
    const int32_t a = eu[i], b = ev[i];
    const float ww = ew[i];
    if (a < 0 || a >= n_total || b < 0 || b >= n_total) { report_error(bc, kErrEndpoint, index_base + i); return; }
    if (a == b) { report_error(bc, kErrSelfLoop, index_base + i); return; }
    if (!(ww > 0.f) || !isfinite(ww)) report_error(bc, kErrWeight, index_base + i);
}

// Half-edge i < m has source eu[i]; half-edge m + i has source ev[i].  Count the entries each row
// will receive and list every row that receives any ("touched" rows).  Out-of-range sources are
// skipped (the validation kernel reports them).  A workgroup takes kAppendItems * kBlock half-edges
// and appends its first-touched rows with one counter atomic.
// rank_u / rank_v (both or neither): what the counting atomic returned for half-edge i / m + i, i.e. the
// half-edge's place among the entries this batch appends to its row; k_write_halfedges then needs no second atomic.
__global__ void __launch_bounds__(kBlock) k_count_halfedges(int64_t m, int64_t n_total, const int32_t* __restrict__ eu,
                                                           const int32_t* __restrict__ ev,
                                                           int32_t* __restrict__ add_cnt,
                                                           int32_t* __restrict__ touched, BatchCtr* bc,
                                                           int32_t* __restrict__ rank_u, int32_t* __restrict__ rank_v) {
    __shared__ unsigned int smem[kBlock / kWave + 1];
    const int64_t base = (int64_t)blockIdx.x * kBlock * kAppendItems;
    int32_t srcs[kAppendItems];
    unsigned int firstmask = 0;
#pragma unroll
    for (int k = 0; k < kAppendItems; ++k) {
        const int64_t i = base + (int64_t)k * kBlock + threadIdx.x;
        int32_t src = -1;
        if (i < 2 * m) {
            src = i < m ? eu[i] : ev[i - m];
            if (src >= 0 && src < n_total) {
                const int32_t r = atomicAdd(&add_cnt[src], 1);
                if (r == 0) firstmask |= 1u << k;
                if (rank_u) (i < m ? rank_u[i] : rank_v[i - m]) = r;
            }
        }
        srcs[k] = src;
    }
    unsigned int slot = block_reserve(&bc->touched, (unsigned int)__popc(firstmask), smem);
#pragma unroll
    for (int k = 0; k < kAppendItems; ++k)
        if ((firstmask >> k) & 1u) touched[slot++] = srcs[k];
}

// Rows whose slack cannot take the new entries get room at the pool tail (one tail atomic per workgroup: atomics
// on one address run at about 1e8 per second); reloc_off[t] is the new offset or -1.  Touches no row: bc->pool_tail
// afterwards tells the host how large the pool has to be before k_relocate may run.
__global__ void __launch_bounds__(kBlock) k_plan_reserve(unsigned int nt, const int32_t* __restrict__ touched,
                                                        const RowMeta* __restrict__ meta,
                                                        const int32_t* __restrict__ add_cnt, float slack,
                                                        int64_t* __restrict__ reloc_off, BatchCtr* bc) {
    __shared__ unsigned long long smem[kBlock / kWave + 1];
    __shared__ unsigned long long sbase;
    const unsigned int t = blockIdx.x * kBlock + threadIdx.x;
    unsigned long long cap = 0;
    if (t < nt) {
        const int32_t u = touched[t];
        const RowMeta m = meta[u];
        const int64_t need = (int64_t)m.len + add_cnt[u];
        if (need > m.cap) cap = (unsigned long long)row_capacity(need, slack);
    }
    unsigned long long total;
    const unsigned long long ex = block_exclusive_scan<unsigned long long>(cap, smem, &total);
    const int nrel = __syncthreads_count(cap != 0);
    if (threadIdx.x == 0) {
        sbase = total ? atomicAdd(&bc->pool_tail, total) : 0ull;
        if (nrel) atomicAdd(&bc->relocated, (unsigned int)nrel);
    }
    __syncthreads();
    if (t < nt) reloc_off[t] = cap ? (int64_t)(sbase + ex) : -1;
}

// Give every relocated row its new place.  One lane per touched row; rows that already hold entries (few, but
// hubs among them) are copied by the whole wave, one row after the other.
__global__ void __launch_bounds__(kBlock) k_relocate(unsigned int nt, const int32_t* __restrict__ touched,
                                                    RowMeta* __restrict__ meta, const int32_t* __restrict__ add_cnt,
                                                    float slack, const int64_t* __restrict__ reloc_off,
                                                    Edge* __restrict__ pool) {
    const unsigned int t = blockIdx.x * kBlock + threadIdx.x;
    const int64_t noff = t < nt ? reloc_off[t] : -1;
    int64_t ooff = 0;
    int len = 0;
    if (noff >= 0) {
        const int32_t u = touched[t];
        const RowMeta m = meta[u];
        ooff = m.off;
        len = m.len;
        RowMeta r;
        r.off = noff;
        r.len = m.len;
        r.cap = row_capacity((int64_t)m.len + add_cnt[u], slack);
        meta[u] = r;
    }
    unsigned long long todo = __ballot(len > 0);
    const int lane = lane_id();
    while (todo) {
        const int l = __ffsll((long long)todo) - 1;
        todo &= todo - 1;
        const int64_t from = __shfl(ooff, l), to = __shfl(noff, l);
        const int n = __shfl(len, l);
        for (int j = lane; j < n; j += kWave) pool[to + j] = pool[from + j];
    }
}

// Append both directions of every new edge.  With ranks (k_count_halfedges): the entry goes to position
// len + rank of its row and the row's length stays as it was (k_sort_finish adds the batch's count); without: the
// position comes from an atomic on the length.  Either way the order of one batch's entries inside a row is
// unspecified until they are sorted.
__global__ void __launch_bounds__(kBlock) k_write_halfedges(int64_t m, const int32_t* __restrict__ eu,
                                                           const int32_t* __restrict__ ev,
                                                           const float* __restrict__ ew, RowMeta* __restrict__ meta,
                                                           Edge* __restrict__ pool, const int32_t* __restrict__ rank) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= 2 * m) return;
    const int64_t k = i < m ? i : i - m;
    const int32_t src = i < m ? eu[k] : ev[k];
    const int32_t dst = i < m ? ev[k] : eu[k];
    Edge e;
    e.col = dst;
    e.w = ew[k];
    if (rank) {
        const RowMeta r = meta[src];
        pool[r.off + r.len + rank[i]] = e;
    } else {
        const int slot = atomicAdd(&meta[src].len, 1);
        pool[meta[src].off + slot] = e;
    }
}

// The entries one batch appends to a row land in the order their atomics happened to take.  Sorting
// the appended segment by (neighbour id, weight bits) makes the stored row, and with it every sum
// over the row, a function of the batch alone.  16 lanes per touched row; segments of up to
// 16 * kSortRegs entries are rank-sorted in registers (every key is broadcast to the group once),
// longer ones are queued for k_sort_long_segments (and finished by k_finish_rows afterwards).
__device__ inline unsigned long long edge_key(const Edge& e) {
    return ((unsigned long long)(unsigned int)e.col << 32) | (unsigned long long)__float_as_uint(e.w);
}

__device__ inline Edge key_edge(unsigned long long k) {
    Edge e;
    e.col = (int32_t)(unsigned int)(k >> 32);
    e.w = __uint_as_float((unsigned int)(k & 0xffffffffull));
    return e;
}

// ... and, for the same rows, what ends Step 1: d(u) recomputed from the stored row (entries added in position
// order, lane j mod 16 takes entry j), the counting scratch cleared, the row put into V_aff (both endpoints of every
// inserted edge are affected).  The sorted weights go through LDS so that the sum needs no second pass over the row.
// len_is_old: the rows' lengths do not yet include the appended entries (k_write_halfedges with ranks); the kernel
// then stores the new length.  Rows with long appended segments only get their length and are listed.
__global__ void __launch_bounds__(kBlock) k_sort_finish(unsigned int nt, const int32_t* __restrict__ touched,
                                                       RowMeta* __restrict__ meta, Edge* __restrict__ pool,
                                                       int32_t* __restrict__ add_cnt, int len_is_old,
                                                       int32_t* __restrict__ long_list, BatchCtr* bc,
                                                       float* __restrict__ deg, uint8_t* __restrict__ flag) {
    constexpr int G = 16;
    __shared__ float sorted_w[kBlock / G][G * kSortRegs];
    const unsigned int t = (blockIdx.x * kBlock + threadIdx.x) / G;
    const int grp = threadIdx.x / G;
    const int gl = threadIdx.x % G;
    int32_t u = 0;
    int a = 0, len_old = 0;
    RowMeta m;
    m.off = 0;
    m.len = 0;
    m.cap = 0;
    bool is_long = false;
    if (t < nt) {
        u = touched[t];
        a = add_cnt[u];
        m = meta[u];
        len_old = len_is_old ? m.len : m.len - a;
        is_long = a > G * kSortRegs;
    }
    const bool sorts = t < nt && !is_long;
    Edge* seg = pool + m.off + len_old;
    if (sorts) {
        const int slots = (a + G - 1) / G;  // uniform in the group
        unsigned long long key[kSortRegs];
#pragma unroll
        for (int r = 0; r < kSortRegs; ++r) {
            const int j = r * G + gl;
            key[r] = (r < slots && j < a) ? edge_key(seg[j]) : ~0ull;
        }
        int rank[kSortRegs];
#pragma unroll
        for (int r = 0; r < kSortRegs; ++r) rank[r] = r * G + gl;
        if (a > 1) {
#pragma unroll
            for (int r = 0; r < kSortRegs; ++r) rank[r] = 0;
#pragma unroll
            for (int r2 = 0; r2 < kSortRegs; ++r2) {
                if (r2 < slots) {
                    for (int l = 0; l < G; ++l) {
                        const unsigned int hi = __shfl((unsigned int)(key[r2] >> 32), l, G);
                        const unsigned int lo = __shfl((unsigned int)(key[r2] & 0xffffffffull), l, G);
                        const unsigned long long other = ((unsigned long long)hi << 32) | lo;
                        const int oj = r2 * G + l;
#pragma unroll
                        for (int r = 0; r < kSortRegs; ++r) {
                            const int j = r * G + gl;
                            rank[r] += (other < key[r] || (other == key[r] && oj < j)) ? 1 : 0;
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int r = 0; r < kSortRegs; ++r) {
            const int j = r * G + gl;
            if (r < slots && j < a) {
                const Edge e = key_edge(key[r]);
                if (a > 1) seg[rank[r]] = e;
                sorted_w[grp][rank[r]] = e.w;
            }
        }
    }
    __syncthreads();
    if (t >= nt) return;
    if (is_long) {
        if (gl == 0) {
            if (len_is_old) meta[u].len = len_old + a;
            long_list[atomicAdd(&bc->sort_long, 1u)] = u;
        }
        return;
    }
    const int len_new = len_old + a;
    float s = 0.f;
    // (a row may be a hub of tens of thousands of entries that received a few: several loads in flight, added in order)
    constexpr int UN = 4;
    for (int j0 = gl; j0 < len_new; j0 += UN * G) {
        float wv[UN];
#pragma unroll
        for (int q = 0; q < UN; ++q) {
            const int j = j0 + q * G;
            wv[q] = j < len_old ? pool[m.off + j].w : (j < len_new ? sorted_w[grp][j - len_old] : 0.f);
        }
#pragma unroll
        for (int q = 0; q < UN; ++q)
            if (j0 + q * G < len_new) s += wv[q];
    }
#pragma unroll
    for (int d = G / 2; d > 0; d >>= 1) s += __shfl_xor(s, d, G);
    if (gl == 0) {
        if (len_is_old) meta[u].len = len_new;
        deg[u] = s;
        add_cnt[u] = 0;
        if (flag) flag[u] = 1;
    }
}

// Long appended segments: one workgroup of kSortThreads per row sorts the segment with a bitonic network whose
// compare-exchanges all point the same way (the first step of every merge pairs i with its mirror image inside
// the block), so positions past the end act as +infinity.  The network runs on tiles of kSortTile keys in LDS:
// a segment of one tile (a power-law hub that receives a few thousand entries from one batch) never goes to memory
// in between; a longer one (a new hub vertex arriving with tens of thousands of entries) is first sorted tile by
// tile, and of every later merge only the steps whose partners lie in different tiles run in memory (6 of 136 steps
// for 50,000 entries), UN disjoint pairs in flight per lane.
constexpr int kSortThreads = 1024;
constexpr int kSortTile = 8192;

// steps j = j_first, j_first / 2, ..., 1 of the network on the first `len` positions (a power of two) of a tile held
// in LDS; mirror: the first of them pairs i with its mirror image inside blocks of 2 * j_first
__device__ inline void sort_tile_steps(unsigned long long* keys, unsigned int len, unsigned int j_first, bool mirror) {
    for (unsigned int j = j_first; j > 0; j >>= 1) {
        const unsigned int mask = (mirror && j == j_first) ? (2 * j_first - 1) : j;
        for (unsigned int i = threadIdx.x; i < len; i += kSortThreads) {
            const unsigned int l = i ^ mask;
            if (l > i) {
                const unsigned long long x = keys[i], y = keys[l];
                if (y < x) {
                    keys[i] = y;
                    keys[l] = x;
                }
            }
        }
        __syncthreads();
    }
}

__global__ void __launch_bounds__(kSortThreads) k_sort_long_segments(const int32_t* __restrict__ long_list,
                                                                    const RowMeta* __restrict__ meta, Edge* pool,
                                                                    const int32_t* __restrict__ add_cnt,
                                                                    const BatchCtr* bc) {
    __shared__ unsigned long long keys[kSortTile];
    constexpr unsigned int T = kSortTile;
    const unsigned int count = bc->sort_long;
    for (unsigned int q = blockIdx.x; q < count; q += gridDim.x) {  // uniform per workgroup
        const int32_t u = long_list[q];
        const unsigned int a = (unsigned int)add_cnt[u];
        const RowMeta m = meta[u];
        Edge* seg = pool + m.off + (m.len - (int)a);
        unsigned int P = 2;
        while (P < a) P <<= 1;
        const unsigned int L = P < T ? P : T;  // positions of a tile the network works on (all of it from T keys on)
        const unsigned int tiles = (a + T - 1) / T;
        auto load_tile = [&](unsigned int t) {
            for (unsigned int i = threadIdx.x; i < L; i += kSortThreads)
                keys[i] = t * T + i < a ? edge_key(seg[t * T + i]) : ~0ull;
            __syncthreads();
        };
        auto store_tile = [&](unsigned int t) {
            for (unsigned int i = threadIdx.x; i < L; i += kSortThreads)
                if (t * T + i < a) seg[t * T + i] = key_edge(keys[i]);
            __syncthreads();
        };
        // every tile on its own: merges of blocks of 2, 4, ..., L keys
        for (unsigned int t = 0; t < tiles; ++t) {
            load_tile(t);
            for (unsigned int k = 2; k <= L; k <<= 1) sort_tile_steps(keys, L, k >> 1, true);
            store_tile(t);
        }
        // merges of blocks of 2T, 4T, ..., P keys: partners in different tiles meet in memory, the rest in LDS
        for (unsigned int k = 2 * T; k <= P; k <<= 1) {
            for (unsigned int j = k >> 1; j >= T; j >>= 1) {
                const unsigned int mask = (j == (k >> 1)) ? (k - 1) : j;
                constexpr int UN = 8;
                for (unsigned int i0 = threadIdx.x; i0 < a; i0 += UN * kSortThreads) {
                    Edge x[UN], y[UN];
                    bool pair[UN];
#pragma unroll
                    for (int r = 0; r < UN; ++r) {
                        const unsigned int i = i0 + r * kSortThreads, l = i ^ mask;
                        pair[r] = i < a && l > i && l < a;
                        if (pair[r]) {
                            x[r] = seg[i];
                            y[r] = seg[l];
                        }
                    }
#pragma unroll
                    for (int r = 0; r < UN; ++r) {
                        const unsigned int i = i0 + r * kSortThreads, l = i ^ mask;
                        if (pair[r] && edge_key(y[r]) < edge_key(x[r])) {
                            seg[i] = y[r];
                            seg[l] = x[r];
                        }
                    }
                }
                __syncthreads();
            }
            for (unsigned int t = 0; t < tiles; ++t) {
                load_tile(t);
                sort_tile_steps(keys, T, T >> 1, false);
                store_tile(t);
            }
        }
    }
}

// The rows k_sort_long_segments has sorted (their number is bc->sort_long): recompute d(u) from the stored row in
// the same order as k_sort_finish, clear the counting scratch, and put the row into V_aff.
__global__ void __launch_bounds__(kBlock) k_finish_rows(const int32_t* __restrict__ list, const BatchCtr* bc,
                                                       const RowMeta* __restrict__ meta,
                                                       const Edge* __restrict__ pool, int32_t* __restrict__ add_cnt,
                                                       float* __restrict__ deg, uint8_t* __restrict__ flag) {
    constexpr int G = 16;
    const unsigned int count = bc->sort_long;
    const int gl = threadIdx.x % G;
    for (unsigned int t = (blockIdx.x * kBlock + threadIdx.x) / G; t < count; t += gridDim.x * (kBlock / G)) {
        const int32_t u = list[t];
        const RowMeta m = meta[u];
        float s = 0.f;
        // these are hub rows of up to tens of thousands of entries: 8 loads in flight per lane, added in order
        constexpr int UN = 8;
        for (int j0 = gl; j0 < m.len; j0 += UN * G) {
            float wv[UN];
#pragma unroll
            for (int q = 0; q < UN; ++q) wv[q] = j0 + q * G < m.len ? pool[m.off + j0 + q * G].w : 0.f;
#pragma unroll
            for (int q = 0; q < UN; ++q)
                if (j0 + q * G < m.len) s += wv[q];
        }
#pragma unroll
        for (int d = G / 2; d > 0; d >>= 1) s += __shfl_xor(s, d, G);
        if (gl == 0) {
            deg[u] = s;
            add_cnt[u] = 0;
            if (flag) flag[u] = 1;
        }
    }
}

// Undo k_count_halfedges after a failed validation.
__global__ void __launch_bounds__(kBlock) k_clear_counts(unsigned int nt, const int32_t* __restrict__ touched,
                                                        int32_t* __restrict__ add_cnt) {
    const unsigned int t = blockIdx.x * kBlock + threadIdx.x;
    if (t < nt) add_cnt[touched[t]] = 0;
}

// =================================================================================================
// Vertex deletion (Alg. 2 Step 1 for Delta^Del): V_aff <- V_aff U N(u), then u and its edges go
// =================================================================================================
constexpr int32_t kDeletedMark = -2;  // seed_class value of a vertex while its batch deletes it

__global__ void __launch_bounds__(kBlock) k_validate_deleted(int64_t nd, int64_t n, const int32_t* __restrict__ del,
                                                            BatchCtr* bc) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= nd) return;
    const int32_t u = del[i];
    if (u < 0 || u >= n) report_error(bc, kErrDeleted, i);
}

__global__ void __launch_bounds__(kBlock) k_mark_deleted(int64_t nd, const int32_t* __restrict__ del,
                                                        int32_t* __restrict__ seed_class, int32_t value) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < nd) seed_class[del[i]] = value;
}

// One 16-lane group per listed vertex.  The group that swaps the row length to 0 owns the row (a
// vertex listed twice is handled once): every surviving neighbour v is put into V_aff (flag) and, on
// first touch, into the list of rows that must drop their entries towards deleted vertices.  The
// deleted row keeps its place and capacity in the pool (a later batch may give the id edges again);
// its label row becomes the neutral 1/C.
__global__ void __launch_bounds__(kBlock) k_delete_rows(int64_t nd, const int32_t* __restrict__ del, int C, int Cs, int CP,
                                                       RowMeta* meta, const Edge* __restrict__ pool,
                                                       const int32_t* __restrict__ seed_class,
                                                       uint8_t* __restrict__ flag, int32_t* __restrict__ add_cnt,
                                                       int32_t* __restrict__ touched, float* __restrict__ deg,
                                                       float* __restrict__ F, BatchCtr* bc) {
    constexpr int G = 16;
    const int64_t i = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / G;
    const int gl = threadIdx.x % G;
    int len = 0;
    int32_t u = 0;
    int64_t off = 0;
    if (i < nd) {
        u = del[i];
        if (gl == 0) len = atomicExch(&meta[u].len, 0);
        len = __shfl(len, 0, G);
        off = meta[u].off;
    }
    // all 64 lanes of the wave walk together (wave_reserve needs every lane)
    int maxlen = len;
#pragma unroll
    for (int d = G; d < kWave; d <<= 1) maxlen = max(maxlen, __shfl_xor(maxlen, d, kWave));
    unsigned long long removed = 0;
    for (int base = 0; base < maxlen; base += G) {
        const int j = base + gl;
        bool first = false;
        int32_t v = -1;
        if (j < len) {
            v = pool[off + j].col;
            removed += 1;
            if (seed_class[v] != kDeletedMark) {
                flag[v] = 1;
                removed += 1;  // the entry v -> u goes as well
                first = atomicAdd(&add_cnt[v], 1) == 0;
            }
        }
        const unsigned int slot = wave_reserve(&bc->touched, first);
        if (first) touched[slot] = v;
    }
    removed = wave_sum(removed);
    if (lane_id() == 0 && removed) atomicAdd(&bc->removed, removed);
    if (i < nd) {  // also for a vertex that had no edges, or is listed twice: the same values again
        if (gl == 0) deg[u] = 0.f;
        for (int c = gl; c < CP; c += G) F[(size_t)u * CP + c] = c < Cs ? 1.0f / (float)C : 0.f;
    }
}

// Touched rows: drop the entries that point at deleted vertices, keeping the order of the others,
// then recompute d(v) from the stored row (same summation order as k_finish_rows) and clear the
// counting scratch.  16 lanes per row; a chunk is loaded completely before any of it is written
// back, and the write position never passes the read position.
__global__ void __launch_bounds__(kBlock) k_drop_deleted_entries(unsigned int nt, const int32_t* __restrict__ touched,
                                                                RowMeta* __restrict__ meta, Edge* __restrict__ pool,
                                                                const int32_t* __restrict__ seed_class,
                                                                int32_t* __restrict__ add_cnt,
                                                                float* __restrict__ deg) {
    constexpr int G = 16;
    const unsigned int t = (blockIdx.x * kBlock + threadIdx.x) / G;
    const int gl = threadIdx.x % G;
    const int gshift = (lane_id() / G) * G;
    if (t >= nt) return;
    const int32_t v = touched[t];
    const RowMeta m = meta[v];
    int out = 0;
    // UN chunks of G entries per step (the row may be a hub of tens of thousands of entries): their loads and the
    // lookups of their neighbours are in flight together; the kept ones are written in order, always to positions
    // that lie before everything the step has read
    constexpr int UN = 4;
    for (int base = 0; base < m.len; base += UN * G) {
        Edge e[UN];
        bool keep[UN];
#pragma unroll
        for (int q = 0; q < UN; ++q) {
            const int j = base + q * G + gl;
            e[q].col = 0;
            e[q].w = 0.f;
            if (j < m.len) e[q] = pool[m.off + j];
        }
#pragma unroll
        for (int q = 0; q < UN; ++q) keep[q] = base + q * G + gl < m.len && seed_class[e[q].col] != kDeletedMark;
#pragma unroll
        for (int q = 0; q < UN; ++q) {
            const unsigned int mask = (unsigned int)((__ballot(keep[q]) >> gshift) & 0xffffull);
            if (keep[q]) pool[m.off + out + __popc(mask & ((1u << gl) - 1u))] = e[q];
            out += __popc(mask);
        }
    }
    float s = 0.f;
    for (int j0 = gl; j0 < out; j0 += 8 * G) {  // the same order of additions as k_sort_finish / k_finish_rows
        float wv[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) wv[q] = j0 + q * G < out ? pool[m.off + j0 + q * G].w : 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if (j0 + q * G < out) s += wv[q];
    }
#pragma unroll
    for (int d = G / 2; d > 0; d >>= 1) s += __shfl_xor(s, d, G);
    if (gl == 0) {
        meta[v].len = out;
        deg[v] = s;
        add_cnt[v] = 0;
    }
}

// =================================================================================================
// Storage compaction: rows laid out again in id order with fresh slack (reclaims what relocations
// and deletions left behind)
// =================================================================================================
__global__ void __launch_bounds__(kBlock) k_recap_rows(int64_t n, const RowMeta* __restrict__ meta_old, float slack,
                                                      RowMeta* __restrict__ meta_new,
                                                      int64_t* __restrict__ block_sums) {
    __shared__ int64_t sm[kBlock / kWave + 1];
    const int64_t u = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    int64_t cap = 0;
    if (u < n) {
        const int32_t len = meta_old[u].len;
        cap = row_capacity(len, slack);
        meta_new[u].len = len;
        meta_new[u].cap = (int32_t)cap;
    }
    int64_t total;
    block_exclusive_scan<int64_t>(cap, sm, &total);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

__global__ void __launch_bounds__(kBlock) k_copy_rows(int64_t n, const RowMeta* __restrict__ meta_old,
                                                     const RowMeta* __restrict__ meta_new,
                                                     const Edge* __restrict__ pool_old, Edge* __restrict__ pool_new) {
    constexpr int G = 16;
    const int64_t u = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / G;
    const int gl = threadIdx.x % G;
    if (u >= n) return;
    const RowMeta a = meta_old[u], b = meta_new[u];
    for (int j = gl; j < a.len; j += G) pool_new[b.off + j] = pool_old[a.off + j];
}

// =================================================================================================
// Yardstick: a plain streaming copy (what this chip sustains when every byte is used once)
// =================================================================================================
__global__ void __launch_bounds__(kBlock) k_stream_copy(int64_t n16, const float4* __restrict__ src,
                                                       float4* __restrict__ dst) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// Read-only counterpart (the row update reads about 40 times what it writes): every thread sums what
// it reads and stores one float, so that the loads cannot be dropped.
__global__ void __launch_bounds__(kBlock) k_stream_read(int64_t n16, const float4* __restrict__ src,
                                                       float* __restrict__ sink) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    float acc = 0.f;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n16; i += stride) {
        const float4 v = src[i];
        acc += (v.x + v.y) + (v.z + v.w);
    }
    sink[(int64_t)blockIdx.x * kBlock + threadIdx.x] = acc;
}

// Yardstick for the gathers of the row update: every group of LPN adjacent lanes reads whole rows of 16 * LPN
// bytes at pseudo-random places of a table (the row number is a multiplicative hash of a running index, so the
// kernel reads no index array: its only memory traffic is the gathers), eight independent rows in flight per
// group, the values summed so that the loads cannot be dropped.  What it sustains is the ceiling of "one
// neighbour row per CSR entry" for rows of that size in a table of that footprint.
template <int LPN>
__global__ void __launch_bounds__(kBlock) k_gather_probe(const float4* __restrict__ table, unsigned int rows,
                                                        unsigned long long gathers, float* __restrict__ sink) {
    constexpr int UN = 8;
    const unsigned long long groups = (unsigned long long)gridDim.x * (kBlock / LPN);
    const unsigned long long g = (unsigned long long)blockIdx.x * (kBlock / LPN) + threadIdx.x / LPN;
    const unsigned int part = threadIdx.x % LPN;
    float acc = 0.f;
    for (unsigned long long i = g; i < gathers; i += groups * UN) {
        float4 v[UN];
#pragma unroll
        for (int t = 0; t < UN; ++t) {
            const unsigned long long idx = i + (unsigned long long)t * groups;
            const unsigned int h = (unsigned int)((idx * 0x9E3779B97F4A7C15ull) >> 32);
            const unsigned int r = (unsigned int)(((unsigned long long)h * rows) >> 32);
            v[t] = idx < gathers ? table[(unsigned long long)r * LPN + part] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int t = 0; t < UN; ++t) acc += (v[t].x + v[t].y) + (v[t].z + v[t].w);
    }
    sink[(unsigned long long)blockIdx.x * kBlock + threadIdx.x] = acc;
}

// =================================================================================================
// Export (inspection / tests)
// =================================================================================================
__global__ void __launch_bounds__(kBlock) k_row_lens(int64_t n, const RowMeta* __restrict__ meta,
                                                    int64_t* __restrict__ lens, int64_t* __restrict__ block_sums) {
    __shared__ int64_t sm[kBlock / kWave + 1];
    const int64_t u = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t len = u < n ? meta[u].len : 0;
    if (u < n) lens[u] = len;
    int64_t total;
    block_exclusive_scan<int64_t>(len, sm, &total);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

// lens[] (in) becomes the exclusive prefix (out); row_ptr[n] is written by the host.
__global__ void __launch_bounds__(kBlock) k_lens_to_row_ptr(int64_t n, int64_t* __restrict__ lens,
                                                           const int64_t* __restrict__ block_offsets) {
    __shared__ int64_t sm[kBlock / kWave + 1];
    const int64_t u = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t len = u < n ? lens[u] : 0;
    int64_t total;
    const int64_t ex = block_exclusive_scan<int64_t>(len, sm, &total);
    if (u < n) lens[u] = block_offsets[blockIdx.x] + ex;
}

__global__ void __launch_bounds__(kBlock) k_export_rows(int64_t n, const RowMeta* __restrict__ meta,
                                                       const Edge* __restrict__ pool,
                                                       const int64_t* __restrict__ row_ptr, int32_t* __restrict__ col,
                                                       float* __restrict__ w) {
    constexpr int G = 16;
    const int64_t u = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / G;
    const int gl = threadIdx.x % G;
    if (u >= n) return;
    const RowMeta m = meta[u];
    const int64_t o = row_ptr[u];
    for (int j = gl; j < m.len; j += G) {
        const Edge e = pool[m.off + j];
        col[o + j] = e.col;
        w[o + j] = e.w;
    }
}

}  // namespace dynlp
