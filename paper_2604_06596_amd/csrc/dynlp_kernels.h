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
__global__ void __launch_bounds__(kBlock) k_init_labels(int64_t u0, int64_t u1, int C, int CP,
                                                       const int32_t* __restrict__ seed_class,
                                                       float* __restrict__ F) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t u = u0 + i / CP;
    const int c = (int)(i % CP);
    if (u >= u1) return;
    const int sc = seed_class[u];
    float v = 0.f;
    if (c < C) v = sc < 0 ? 1.0f / (float)C : (c == sc ? 1.0f : 0.0f);
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
                                                       const int32_t* __restrict__ sc, int C, int CP,
                                                       int32_t* __restrict__ seed_class, float* __restrict__ F,
                                                       const RowMeta* __restrict__ meta,
                                                       const Edge* __restrict__ pool, uint8_t* __restrict__ flag) {
    constexpr int G = 16;
    const int64_t i = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / G;
    const int gl = threadIdx.x % G;
    if (i >= s) return;
    const int32_t v = sv[i], c = sc[i];
    if (gl == 0) seed_class[v] = c;
    for (int k = gl; k < CP; k += G) F[(int64_t)v * CP + k] = (k == c) ? 1.0f : 0.0f;
    const RowMeta m = meta[v];
    for (int j = gl; j < m.len; j += G) flag[pool[m.off + j].col] = 1;
}

// hard[u] = argmax_c F[u][c], lowest index on ties.
__global__ void __launch_bounds__(kBlock) k_argmax(int64_t n, int C, int CP, const float* __restrict__ F,
                                                  int32_t* __restrict__ hard) {
    const int64_t u = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (u >= n) return;
    const float* row = F + u * CP;
    int best = 0;
    float bv = row[0];
    for (int c = 1; c < C; ++c) {
        const float v = row[c];
        if (v > bv) { bv = v; best = c; }
    }
    hard[u] = best;
}

__global__ void __launch_bounds__(kBlock) k_pack_soft(int64_t n, int C, int CP, const float* __restrict__ F,
                                                     float* __restrict__ soft) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n * C) return;
    soft[i] = F[(i / C) * CP + (i % C)];
}

// =================================================================================================
// Edge insertion (Alg. 2 Step 1 for insertions) into the slack CSR
// =================================================================================================
__global__ void __launch_bounds__(kBlock) k_validate_edges(int64_t m, int64_t n_total, const int32_t* __restrict__ eu,
                                                          const int32_t* __restrict__ ev,
                                                          const float* __restrict__ ew, BatchCtr* bc) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= m) return;
    const int32_t a = eu[i], b = ev[i];
    const float ww = ew[i];
    if (a < 0 || a >= n_total || b < 0 || b >= n_total) { report_error(bc, kErrEndpoint, i); return; }
    if (a == b) { report_error(bc, kErrSelfLoop, i); return; }
    if (!(ww > 0.f) || !isfinite(ww)) report_error(bc, kErrWeight, i);
}

// Half-edge i < m has source eu[i]; half-edge m + i has source ev[i].  Count the entries each row
// will receive and list every row that receives any ("touched" rows).  Out-of-range sources are
// skipped (the validation kernel reports them).
__global__ void __launch_bounds__(kBlock) k_count_halfedges(int64_t m, int64_t n_total, const int32_t* __restrict__ eu,
                                                           const int32_t* __restrict__ ev,
                                                           int32_t* __restrict__ add_cnt,
                                                           int32_t* __restrict__ touched, BatchCtr* bc) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    bool first = false;
    int32_t src = -1;
    if (i < 2 * m) {
        src = i < m ? eu[i] : ev[i - m];
        if (src >= 0 && src < n_total) first = atomicAdd(&add_cnt[src], 1) == 0;
    }
    const unsigned int slot = wave_reserve(&bc->touched, first);
    if (first) touched[slot] = src;
}

// Rows whose slack cannot take the new entries: total capacity they need at the pool tail.
__global__ void __launch_bounds__(kBlock) k_plan_sum(unsigned int nt, const int32_t* __restrict__ touched,
                                                    const RowMeta* __restrict__ meta,
                                                    const int32_t* __restrict__ add_cnt, float slack,
                                                    BatchCtr* bc) {
    const unsigned int t = blockIdx.x * kBlock + threadIdx.x;
    unsigned long long need_cap = 0;
    if (t < nt) {
        const int32_t u = touched[t];
        const RowMeta m = meta[u];
        const int64_t need = (int64_t)m.len + add_cnt[u];
        if (need > m.cap) need_cap = (unsigned long long)row_capacity(need, slack);
    }
    need_cap = wave_sum(need_cap);
    if (lane_id() == 0 && need_cap) atomicAdd(&bc->reloc_need, need_cap);
}

// Reserve tail space for every overflowing touched row (one atomic per wave); reloc_off[t] is the
// new offset or -1.
__global__ void __launch_bounds__(kBlock) k_plan_reserve(unsigned int nt, const int32_t* __restrict__ touched,
                                                        const RowMeta* __restrict__ meta,
                                                        const int32_t* __restrict__ add_cnt, float slack,
                                                        int64_t* __restrict__ reloc_off, BatchCtr* bc) {
    const unsigned int t = blockIdx.x * kBlock + threadIdx.x;
    unsigned long long cap = 0;
    if (t < nt) {
        const int32_t u = touched[t];
        const RowMeta m = meta[u];
        const int64_t need = (int64_t)m.len + add_cnt[u];
        if (need > m.cap) cap = (unsigned long long)row_capacity(need, slack);
    }
    const unsigned long long inc = wave_inclusive_scan(cap);
    const unsigned long long total = __shfl(inc, kWave - 1, kWave);
    unsigned long long base = 0;
    if (lane_id() == kWave - 1 && total) base = atomicAdd(&bc->pool_tail, total);
    base = __shfl(base, kWave - 1, kWave);
    const unsigned long long nrel = __popcll(__ballot(cap != 0));
    if (lane_id() == 0 && nrel) atomicAdd(&bc->relocated, (unsigned int)nrel);
    if (t < nt) reloc_off[t] = cap ? (int64_t)(base + inc - cap) : -1;
}

// Move the valid entries of every relocated row to its new place (16 lanes per row).
__global__ void __launch_bounds__(kBlock) k_relocate(unsigned int nt, const int32_t* __restrict__ touched,
                                                    RowMeta* __restrict__ meta, const int32_t* __restrict__ add_cnt,
                                                    float slack, const int64_t* __restrict__ reloc_off,
                                                    Edge* __restrict__ pool) {
    constexpr int G = 16;
    const unsigned int t = (blockIdx.x * kBlock + threadIdx.x) / G;
    const int gl = threadIdx.x % G;
    if (t >= nt) return;
    const int64_t noff = reloc_off[t];
    if (noff < 0) return;
    const int32_t u = touched[t];
    const RowMeta m = meta[u];
    for (int j = gl; j < m.len; j += G) pool[noff + j] = pool[m.off + j];
    if (gl == 0) {
        RowMeta r;
        r.off = noff;
        r.len = m.len;
        r.cap = row_capacity((int64_t)m.len + add_cnt[u], slack);
        meta[u] = r;
    }
}

// Append both directions of every new edge; the slot inside the row comes from an atomic on its
// length, so the order of one batch's entries inside a row is unspecified.
__global__ void __launch_bounds__(kBlock) k_write_halfedges(int64_t m, const int32_t* __restrict__ eu,
                                                           const int32_t* __restrict__ ev,
                                                           const float* __restrict__ ew, RowMeta* __restrict__ meta,
                                                           Edge* __restrict__ pool) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= 2 * m) return;
    const int64_t k = i < m ? i : i - m;
    const int32_t src = i < m ? eu[k] : ev[k];
    const int32_t dst = i < m ? ev[k] : eu[k];
    const int slot = atomicAdd(&meta[src].len, 1);
    Edge e;
    e.col = dst;
    e.w = ew[k];
    pool[meta[src].off + slot] = e;
}

// Touched rows: recompute d(u) from the stored row, clear the counting scratch, and put the row
// into V_aff (both endpoints of every inserted edge are affected).
__global__ void __launch_bounds__(kBlock) k_finish_rows(unsigned int nt, const int32_t* __restrict__ touched,
                                                       const RowMeta* __restrict__ meta,
                                                       const Edge* __restrict__ pool, int32_t* __restrict__ add_cnt,
                                                       float* __restrict__ deg, uint8_t* __restrict__ flag) {
    constexpr int G = 16;
    const unsigned int t = (blockIdx.x * kBlock + threadIdx.x) / G;
    const int gl = threadIdx.x % G;
    if (t >= nt) return;
    const int32_t u = touched[t];
    const RowMeta m = meta[u];
    float s = 0.f;
    for (int j = gl; j < m.len; j += G) s += pool[m.off + j].w;
#pragma unroll
    for (int d = G / 2; d > 0; d >>= 1) s += __shfl_xor(s, d, G);
    if (gl == 0) {
        deg[u] = s;
        add_cnt[u] = 0;
        if (flag) flag[u] = 1;
    }
}

// Undo k_count_halfedges after a failed validation.
__global__ void __launch_bounds__(kBlock) k_clear_counts(unsigned int nt, const int32_t* __restrict__ touched,
                                                        int32_t* __restrict__ add_cnt) {
    const unsigned int t = blockIdx.x * kBlock + threadIdx.x;
    if (t < nt) add_cnt[touched[t]] = 0;
}

// =================================================================================================
// Frontier compaction (+ commit of the staged rows of the round that just ran)
// =================================================================================================
constexpr int kFlagsPerThread = 16;
constexpr int kFlagsPerBlock = kBlock * kFlagsPerThread;  // 4096

// Blocks [0, commit_blocks): copy staged rows Fq[i] -> F[queue_cur[i]] (the Jacobi commit).
// Blocks [commit_blocks, ...): each scans kFlagsPerBlock flag bytes, keeps the vertices that
// may be updated (unlabelled, at least one edge), reserves a range of the next queue with one
// atomic, writes the ids in ascending order inside the range, and clears the flags it read.
// all_rows != 0 ignores the flags and lists every updatable vertex (static solve).
__global__ void __launch_bounds__(kBlock) k_commit_compact(const int32_t* __restrict__ queue_cur, unsigned int nq,
                                                          const float* __restrict__ Fq, float* __restrict__ F, int CP,
                                                          unsigned int commit_blocks, unsigned int n,
                                                          uint8_t* __restrict__ flag,
                                                          const int32_t* __restrict__ seed_class,
                                                          const RowMeta* __restrict__ meta,
                                                          int32_t* __restrict__ queue_next,
                                                          unsigned int* __restrict__ next_count, int all_rows) {
    if (blockIdx.x < commit_blocks) {
        if (CP >= 4) {
            const unsigned int vpr = CP / 4;
            const unsigned long long total = (unsigned long long)nq * vpr;
            const float4* src = reinterpret_cast<const float4*>(Fq);
            float4* dst = reinterpret_cast<float4*>(F);
            for (unsigned long long i = (unsigned long long)blockIdx.x * kBlock + threadIdx.x; i < total;
                 i += (unsigned long long)commit_blocks * kBlock) {
                const unsigned int qi = (unsigned int)(i / vpr);
                const unsigned int ch = (unsigned int)(i % vpr);
                dst[(unsigned long long)queue_cur[qi] * vpr + ch] = src[i];
            }
        } else {
            const unsigned long long total = (unsigned long long)nq * CP;
            for (unsigned long long i = (unsigned long long)blockIdx.x * kBlock + threadIdx.x; i < total;
                 i += (unsigned long long)commit_blocks * kBlock) {
                const unsigned int qi = (unsigned int)(i / CP);
                F[(unsigned long long)queue_cur[qi] * CP + (i % CP)] = Fq[i];
            }
        }
        return;
    }
    __shared__ unsigned int sm[kBlock / kWave + 1];
    __shared__ unsigned int sbase;
    const unsigned int b = blockIdx.x - commit_blocks;
    const unsigned int v0 = b * kFlagsPerBlock + threadIdx.x * kFlagsPerThread;
    unsigned int keep = 0;  // bit k: vertex v0+k enters the queue
    bool any = false;
    if (v0 < n) {
        if (all_rows) {
            for (int k = 0; k < kFlagsPerThread; ++k) {
                const unsigned int v = v0 + k;
                if (v < n && seed_class[v] < 0 && meta[v].len > 0) keep |= 1u << k;
            }
        } else {
            const uint4 f = *reinterpret_cast<const uint4*>(flag + v0);
            const unsigned int wds[4] = {f.x, f.y, f.z, f.w};
            any = (f.x | f.y | f.z | f.w) != 0;
            if (any) {
#pragma unroll
                for (int k = 0; k < kFlagsPerThread; ++k) {
                    if ((wds[k >> 2] >> ((k & 3) * 8)) & 0xffu) {
                        const unsigned int v = v0 + k;
                        if (v < n && seed_class[v] < 0 && meta[v].len > 0) keep |= 1u << k;
                    }
                }
                *reinterpret_cast<uint4*>(flag + v0) = make_uint4(0, 0, 0, 0);
            }
        }
    }
    const unsigned int cnt = __popc(keep);
    unsigned int total;
    const unsigned int ex = block_exclusive_scan<unsigned int>(cnt, sm, &total);
    if (threadIdx.x == 0) sbase = total ? atomicAdd(next_count, total) : 0u;
    __syncthreads();
    unsigned int pos = sbase + ex;
    while (keep) {
        const int k = __ffs(keep) - 1;
        keep &= keep - 1;
        queue_next[pos++] = (int32_t)(v0 + k);
    }
}

// =================================================================================================
// Frontier row update: the hot kernel (Alg. 2 Step 3 inner loop / one ItLP sweep of Eq. (1))
// =================================================================================================
// G lanes cooperate on one frontier row u.  A neighbour row of CP floats is read by LPN = CP/VEC
// adjacent lanes (VEC = 4 floats = 16 bytes per lane), so the group gathers SLOTS = G/LPN
// neighbour rows at once, each as one contiguous CP*4-byte segment.  The row's (col, w) pairs
// are first read G at a time with one coalesced 8-byte load per lane and handed round with
// lane shuffles.  Every lane keeps the partial sums of its slot; a butterfly over the slot bits
// finishes acc = sum_j w_j F[col_j] and s = sum_j w_j; F'_u = acc / s.
//   STATIC : F' is written to row u of F_out (ping-pong buffer); no frontier bookkeeping.
//   dynamic: F' is staged at row g of F_out (g = position in the queue) so that every row of
//            this round reads the round-start F (Jacobi); if max_c |F'_u - F_u| > tol the row
//            marks itself and its neighbours in flag[] for the next round (Alg. 2 Step 3).
// The kernel is grid-strided so that each workgroup issues one set of counter atomics.
template <int CP, int G, bool STATIC>
__global__ void __launch_bounds__(kBlock) k_row_update(const int32_t* __restrict__ queue, unsigned int nq,
                                                      const RowMeta* __restrict__ meta,
                                                      const Edge* __restrict__ pool,
                                                      const float* __restrict__ F_in, float* __restrict__ F_out,
                                                      uint8_t* __restrict__ flag, float tol,
                                                      RoundCtr* __restrict__ ctr, RoundCtr* __restrict__ ctr_zero) {
    constexpr int VEC = CP >= 4 ? 4 : CP;
    constexpr int LPN = CP / VEC;
    constexpr int SLOTS = G / LPN;
    constexpr int GPB = kBlock / G;
    static_assert(G % LPN == 0 && SLOTS >= 1, "group must hold whole neighbour rows");

    if (ctr_zero && blockIdx.x == 0 && threadIdx.x == 0) {
        ctr_zero->next_count = 0;
        ctr_zero->resid_bits = 0;
        ctr_zero->changed = 0;
        ctr_zero->edges = 0;
    }

    const int gl = threadIdx.x % G;
    const int slot = gl / LPN;
    const int chunk = gl % LPN;
    float rmax = 0.f;
    unsigned long long edges = 0;
    unsigned int changed = 0;

    for (unsigned int g = blockIdx.x * GPB + threadIdx.x / G; g < nq; g += gridDim.x * GPB) {
        const int32_t u = queue[g];
        const RowMeta m = meta[u];
        const Edge* __restrict__ row = pool + m.off;
        Vec<VEC> acc;
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc.v[k] = 0.f;
        float s = 0.f;
        Edge e;
        e.col = u;
        e.w = 0.f;
        for (int base = 0; base < m.len; base += G) {
            const int idx = base + gl;
            if (idx < m.len) {
                e = row[idx];
            } else {  // a harmless stand-in: own row, weight 0
                e.col = u;
                e.w = 0.f;
            }
            const int cnt = m.len - base;
#pragma unroll
            for (int j0 = 0; j0 < G; j0 += SLOTS) {
                if (j0 < cnt) {  // uniform across the group
                    const int32_t c = __shfl(e.col, j0 + slot, G);
                    const float w = __shfl(e.w, j0 + slot, G);
                    const Vec<VEC> f = load_vec<VEC>(F_in + (size_t)c * CP + chunk * VEC);
#pragma unroll
                    for (int k = 0; k < VEC; ++k) acc.v[k] = fmaf(w, f.v[k], acc.v[k]);
                    s += w;
                }
            }
        }
#pragma unroll
        for (int d = LPN; d < G; d <<= 1) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) acc.v[k] += __shfl_xor(acc.v[k], d, G);
            s += __shfl_xor(s, d, G);
        }
        const Vec<VEC> old = load_vec<VEC>(F_in + (size_t)u * CP + chunk * VEC);
        Vec<VEC> fn;
        float r = 0.f;
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            fn.v[k] = acc.v[k] / s;
            r = fmaxf(r, fabsf(fn.v[k] - old.v[k]));
        }
#pragma unroll
        for (int d = 1; d < LPN; d <<= 1) r = fmaxf(r, __shfl_xor(r, d, G));
        if (slot == 0) store_vec<VEC>(F_out + (size_t)(STATIC ? (unsigned int)u : g) * CP + chunk * VEC, fn);
        const bool big = r > tol;
        if (!STATIC && big) {
            // V_aff <- V_aff U {u} U N(u); the last chunk of the row is still in registers
            if (gl == 0) flag[u] = 1;
            if (e.w != 0.f && !flag[e.col]) flag[e.col] = 1;
            const int last_base = ((m.len - 1) / G) * G;
            for (int idx = gl; idx < last_base; idx += G) {
                const int32_t c = row[idx].col;
                if (!flag[c]) flag[c] = 1;
            }
        }
        if (gl == 0) {
            rmax = fmaxf(rmax, r);
            edges += (unsigned long long)m.len;
            changed += big ? 1u : 0u;
        }
    }

    __shared__ float sm_r[kBlock / kWave];
    __shared__ unsigned long long sm_e[kBlock / kWave];
    __shared__ unsigned int sm_c[kBlock / kWave];
    rmax = wave_max(rmax);
    edges = wave_sum(edges);
    changed = wave_sum(changed);
    if (lane_id() == 0) {
        sm_r[threadIdx.x / kWave] = rmax;
        sm_e[threadIdx.x / kWave] = edges;
        sm_c[threadIdx.x / kWave] = changed;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < kBlock / kWave; ++i) {
            rmax = fmaxf(rmax, sm_r[i]);
            edges += sm_e[i];
            changed += sm_c[i];
        }
        atomicMax(&ctr->resid_bits, __float_as_uint(rmax));
        if (edges) atomicAdd(&ctr->edges, edges);
        if (changed) atomicAdd(&ctr->changed, changed);
    }
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
