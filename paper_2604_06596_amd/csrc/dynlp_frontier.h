// Frontier kernels of DynLP for gfx950: compaction of V_aff into queues, the frontier row update
// (the hot kernel), the Jacobi commit of staged rows and the expansion of V_aff (Alg. 2 Step 3).
#pragma once

#include "dynlp_device.h"

namespace dynlp {

constexpr int kFlagsPerThread = 16;
constexpr int kFlagsPerBlock = kBlock * kFlagsPerThread;  // 4096
constexpr int kLongRow = 128;  // rows longer than this get a whole workgroup

#ifndef DYNLP_UN_CAP
#define DYNLP_UN_CAP 8
#endif

// A frontier is stored in one int32 array of n_cap entries: "short" rows (len <= kLongRow) from
// the front, position i at front[i]; "long" rows from the back, position j at back[-j] with
// back = front + n_cap - 1.  The two never meet because a frontier has at most n entries.
// Row i of the frontier (short rows first, then long rows) has *position* i; staged label rows
// are indexed by position.
__device__ inline int32_t frontier_vertex(const int32_t* front, const int32_t* back, unsigned int ns,
                                          unsigned int pos) {
    return pos < ns ? front[pos] : back[-(long long)(pos - ns)];
}

// =================================================================================================
// Compaction: flag bytes -> next frontier
// =================================================================================================
// Each workgroup scans SEG * kFlagsPerBlock flag bytes (SEG runs of kFlagsPerBlock, 16 consecutive bytes per
// thread and run), keeps the vertices that may be updated (unlabelled, at least one edge), reserves ranges of
// the short and the long queue with one atomic each, writes the ids inside its ranges, and clears the flags it
// read.  The order of a frontier list has no influence on results.  SEG: atomics on one address run at about 1e8
// per second, so the 12,000 workgroups of a 50M-vertex graph at SEG = 1 spend 0.12 ms queueing for the counter;
// the host picks SEG = 4 from 16M vertices on and SEG = 1 (more workgroups) below.
// all_rows != 0 ignores the flags and lists every updatable vertex (static solve, and the count of
// updatable vertices).
template <int SEG>
__global__ void __launch_bounds__(kBlock) k_compact(unsigned int n, uint8_t* __restrict__ flag,
                                                   const int32_t* __restrict__ seed_class,
                                                   const RowMeta* __restrict__ meta, int all_rows,
                                                   int32_t* __restrict__ front, int32_t* __restrict__ back,
                                                   unsigned int* __restrict__ count_short,
                                                   unsigned int* __restrict__ count_long) {
    __shared__ unsigned long long sm[kBlock / kWave + 1];
    __shared__ unsigned int sbase[2];
    unsigned int keep[SEG], is_long[SEG];  // bit k: vertex v0+k enters the frontier / as a long row
    unsigned int n_short = 0, n_long = 0;
#pragma unroll
    for (int q = 0; q < SEG; ++q) {
        const unsigned int v0 = (blockIdx.x * SEG + q) * kFlagsPerBlock + threadIdx.x * kFlagsPerThread;
        keep[q] = 0;
        is_long[q] = 0;
        if (v0 < n) {
            unsigned int cand = 0;
            if (all_rows) {
                cand = 0xffffu;
            } else {
                const uint4 f = *reinterpret_cast<const uint4*>(flag + v0);
                if ((f.x | f.y | f.z | f.w) != 0) {
                    const unsigned int wds[4] = {f.x, f.y, f.z, f.w};
#pragma unroll
                    for (int k = 0; k < kFlagsPerThread; ++k)
                        if ((wds[k >> 2] >> ((k & 3) * 8)) & 0xffu) cand |= 1u << k;
                    *reinterpret_cast<uint4*>(flag + v0) = make_uint4(0, 0, 0, 0);
                }
            }
            while (cand) {
                const int k = __ffs(cand) - 1;
                cand &= cand - 1;
                const unsigned int v = v0 + k;
                if (v < n && seed_class[v] < 0) {
                    const int len = meta[v].len;
                    if (len > 0) {
                        keep[q] |= 1u << k;
                        if (len > kLongRow) is_long[q] |= 1u << k;
                    }
                }
            }
        }
        n_short += (unsigned int)__popc(keep[q] & ~is_long[q]);
        n_long += (unsigned int)__popc(is_long[q]);
    }
    const unsigned long long cnt = (unsigned long long)n_short | ((unsigned long long)n_long << 32);
    unsigned long long total;
    const unsigned long long ex = block_exclusive_scan<unsigned long long>(cnt, sm, &total);
    if (threadIdx.x == 0) {
        const unsigned int ts = (unsigned int)total, tl = (unsigned int)(total >> 32);
        sbase[0] = ts ? atomicAdd(count_short, ts) : 0u;
        sbase[1] = tl ? atomicAdd(count_long, tl) : 0u;
    }
    __syncthreads();
    unsigned int ps = sbase[0] + (unsigned int)ex;
    unsigned int pl = sbase[1] + (unsigned int)(ex >> 32);
#pragma unroll
    for (int q = 0; q < SEG; ++q) {
        const unsigned int v0 = (blockIdx.x * SEG + q) * kFlagsPerBlock + threadIdx.x * kFlagsPerThread;
        unsigned int kp = keep[q];
        while (kp) {
            const int k = __ffs(kp) - 1;
            kp &= kp - 1;
            if ((is_long[q] >> k) & 1u) back[-(long long)(pl++)] = (int32_t)(v0 + k);
            else front[ps++] = (int32_t)(v0 + k);
        }
    }
}

// =================================================================================================
// Commit of staged rows (staged rounds) and the next frontier after a ping-pong round
// =================================================================================================
// F[vertex at position i] = Fq[i] for all positions: the Jacobi commit of a staged round.
__global__ void __launch_bounds__(kBlock) k_commit(const RoundCtr* __restrict__ prev,
                                                  const int32_t* __restrict__ front,
                                                  const int32_t* __restrict__ back,
                                                  const float* __restrict__ Fq, float* __restrict__ F, int CP) {
    const unsigned int ns = prev->next_count, nl = prev->next_long;
    const unsigned int nq = ns + nl;
    if (CP >= 4) {
        const unsigned int vpr = CP / 4;
        const unsigned long long total = (unsigned long long)nq * vpr;
        const float4* src = reinterpret_cast<const float4*>(Fq);
        float4* dst = reinterpret_cast<float4*>(F);
        for (unsigned long long i = (unsigned long long)blockIdx.x * kBlock + threadIdx.x; i < total;
             i += (unsigned long long)gridDim.x * kBlock) {
            const unsigned int pos = (unsigned int)(i / vpr);
            const unsigned int ch = (unsigned int)(i % vpr);
            dst[(unsigned long long)frontier_vertex(front, back, ns, pos) * vpr + ch] = src[i];
        }
    } else {
        const unsigned long long total = (unsigned long long)nq * CP;
        for (unsigned long long i = (unsigned long long)blockIdx.x * kBlock + threadIdx.x; i < total;
             i += (unsigned long long)gridDim.x * kBlock) {
            const unsigned int pos = (unsigned int)(i / CP);
            F[(unsigned long long)frontier_vertex(front, back, ns, pos) * CP + (i % CP)] = Fq[i];
        }
    }
}

__device__ inline void mark(uint8_t* __restrict__ flag, int32_t v) {
    if (!flag[v]) flag[v] = 1;
}

// Next V_aff after a ping-pong round, computed by *pulling* instead of marking, and written straight
// into the next frontier (no flag bytes, no separate compaction).  The update kernels of a ping-pong
// round set one bit per row that moved by more than tol (moved[], 1 bit per vertex: 125 KB per million
// vertices, so the neighbour look-ups below stay in cache).  Alg. 2 Step 3 puts u into the next V_aff
// iff u moved or one of its neighbours moved; this kernel evaluates exactly that for every updatable
// vertex u (the universe list, short rows first, long rows from the back): one bit read, and only
// when u itself did not move a scan of N(u)'s bits that stops at the first hit.  A row that does not
// make it into the next V_aff gets its current value copied into F_old if the two buffers differ
// (it was updated in this round), so that they keep agreeing on every row outside V_aff (the
// invariant ping-pong rounds rely on).  The kernel also clears the bitmap of the next round.
// Workgroups [0, long_blocks): long rows, one wave per row, 64 neighbours per step.  The others:
// short rows, one lane per row.  A workgroup handles chunks of consecutive universe positions and
// reserves the output range of a whole chunk with ONE atomic (atomics on one address run at only
// ~10^8 per second device-wide, so they are kept to a few hundred per launch); kept ids are written
// in universe order inside the chunk's range.
__device__ inline bool moved_bit(const unsigned int* __restrict__ moved, int32_t v) {
    return (moved[(unsigned int)v >> 5] >> ((unsigned int)v & 31u)) & 1u;
}

// COH: read past the caches (the bitmap was written by other workgroups earlier in the same launch)
template <bool COH>
__device__ inline bool moved_bit_c(const unsigned int* moved, int32_t v) {
    if constexpr (!COH) return moved_bit(moved, v);
    else
        return (__hip_atomic_load(&moved[(unsigned int)v >> 5], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >>
                ((unsigned int)v & 31u)) & 1u;
}

// kPullSub = sub-steps per workgroup chunk (one queue atomic per chunk of kPullSub * kBlock positions).
// Small chunks mean more workgroups (the kernel is latency-bound on small and on low-degree graphs),
// large chunks mean fewer atomics on the one queue counter (which run at about 1e8 per second and show
// once every row also scans tens of neighbours): the host picks 4 or 16.
template <int kPullSub>
__global__ void __launch_bounds__(kBlock) k_pull_frontier(unsigned int ns, unsigned int nl, unsigned int long_blocks,
                                                         const int32_t* __restrict__ ufront,
                                                         const int32_t* __restrict__ uback,
                                                         const unsigned int* __restrict__ moved,
                                                         unsigned int* __restrict__ moved_next, unsigned int words,
                                                         const float* __restrict__ F_new, float* __restrict__ F_old,
                                                         int CP, const RowMeta* __restrict__ meta,
                                                         const Edge* __restrict__ pool,
                                                         int32_t* __restrict__ front, int32_t* __restrict__ back,
                                                         unsigned int* __restrict__ count_short,
                                                         unsigned int* __restrict__ count_long) {
    constexpr int NW = kBlock / kWave;
    __shared__ unsigned int cnt[kPullSub][NW];  // kept items per sub-step and wave, then their offsets
    __shared__ unsigned int sbase;
    const int wave = threadIdx.x / kWave;
    const int lane = lane_id();
    for (unsigned int w = blockIdx.x * kBlock + threadIdx.x; w < words; w += gridDim.x * kBlock) moved_next[w] = 0u;

    if (blockIdx.x < long_blocks) {
        // long rows: one wave per row, kPullSub rows per wave and chunk
        constexpr unsigned int CH = NW * kPullSub;
        for (unsigned int c0 = blockIdx.x * CH; c0 < nl; c0 += long_blocks * CH) {  // uniform per workgroup
            unsigned int keepmask = 0;
            for (int sub = 0; sub < kPullSub; ++sub) {
                const unsigned int j = c0 + sub * NW + wave;
                bool keep = false;
                if (j < nl) {
                    const int32_t u = uback[-(long long)j];
                    keep = moved_bit(moved, u);
                    if (!keep) {
                        const RowMeta m = meta[u];
                        const Edge* __restrict__ row = pool + m.off;
                        for (int base = 0; base < m.len; base += kWave) {  // uniform per wave
                            const int idx = base + lane;
                            const bool hit = idx < m.len && moved_bit(moved, row[idx].col);
                            if (__ballot(hit)) {
                                keep = true;
                                break;
                            }
                        }
                        if (!keep && F_old) {
                            for (int k = lane; k < CP; k += kWave) {
                                const float a = F_new[(size_t)u * CP + k];
                                if (a != F_old[(size_t)u * CP + k]) F_old[(size_t)u * CP + k] = a;
                            }
                        }
                    }
                }
                if (keep) keepmask |= 1u << sub;
                if (lane == 0) cnt[sub][wave] = keep ? 1u : 0u;
            }
            __syncthreads();
            if (threadIdx.x == 0) {
                unsigned int run = 0;
                for (int sub = 0; sub < kPullSub; ++sub)
                    for (int q = 0; q < NW; ++q) {
                        const unsigned int t = cnt[sub][q];
                        cnt[sub][q] = run;
                        run += t;
                    }
                sbase = run ? atomicAdd(count_long, run) : 0u;
            }
            __syncthreads();
            if (lane == 0) {
                for (int sub = 0; sub < kPullSub; ++sub)
                    if ((keepmask >> sub) & 1u)
                        back[-(long long)(sbase + cnt[sub][wave])] = uback[-(long long)(c0 + sub * NW + wave)];
            }
            __syncthreads();
        }
        return;
    }
    // short rows: one lane per row, kPullSub * kBlock consecutive universe positions per chunk
    constexpr unsigned int CH = kBlock * kPullSub;
    const unsigned int nb = gridDim.x - long_blocks;
    const unsigned int bid = blockIdx.x - long_blocks;
    for (unsigned int c0 = bid * CH; c0 < ns; c0 += nb * CH) {  // uniform per workgroup
        // all ids of the chunk first, then all their bits: two memory round trips instead of 2 * kPullSub
        int32_t us[kPullSub];
#pragma unroll
        for (int sub = 0; sub < kPullSub; ++sub) {
            const unsigned int pos = c0 + sub * kBlock + threadIdx.x;
            us[sub] = pos < ns ? ufront[pos] : -1;
        }
        unsigned int keepmask = 0;
#pragma unroll
        for (int sub = 0; sub < kPullSub; ++sub)
            if (us[sub] >= 0 && moved_bit(moved, us[sub])) keepmask |= 1u << sub;
#pragma unroll
        for (int sub = 0; sub < kPullSub; ++sub) {
            const int32_t u = us[sub];
            bool keep = (keepmask >> sub) & 1u;
            if (u >= 0 && !keep) {
                const RowMeta m = meta[u];
                const Edge* __restrict__ row = pool + m.off;
                // eight independent look-ups per step (the lane waits once per step, not once per entry)
                for (int j = 0; j < m.len && !keep; j += 8) {
                    unsigned int hit = 0;
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        const int jj = j + q < m.len ? j + q : m.len - 1;
                        hit |= moved_bit(moved, row[jj].col) ? 1u : 0u;
                    }
                    keep = hit != 0;
                }
                if (keep) {
                    keepmask |= 1u << sub;
                } else if (F_old) {
                    for (int k = 0; k < CP; ++k) {
                        const float a = F_new[(size_t)u * CP + k];
                        if (a != F_old[(size_t)u * CP + k]) F_old[(size_t)u * CP + k] = a;
                    }
                }
            }
            const unsigned long long b = __ballot(keep);
            if (lane == 0) cnt[sub][wave] = (unsigned int)__popcll(b);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            unsigned int run = 0;
            for (int sub = 0; sub < kPullSub; ++sub)
                for (int q = 0; q < NW; ++q) {
                    const unsigned int t = cnt[sub][q];
                    cnt[sub][q] = run;
                    run += t;
                }
            sbase = run ? atomicAdd(count_short, run) : 0u;
        }
        __syncthreads();
#pragma unroll
        for (int sub = 0; sub < kPullSub; ++sub) {
            const bool keep = (keepmask >> sub) & 1u;
            const unsigned long long b = __ballot(keep);
            if (keep) {
                const unsigned int rank = (unsigned int)__popcll(b & ((1ull << lane) - 1ull));
                front[sbase + cnt[sub][wave] + rank] = us[sub];
            }
        }
        __syncthreads();
    }
}

// =================================================================================================
// Frontier row update: the hot kernels (Alg. 2 Step 3 inner loop / one ItLP sweep of Eq. (1))
// =================================================================================================
// G lanes cooperate on one frontier row u.  A neighbour row of CP floats is read by LPN = CP/VEC
// adjacent lanes (VEC = 4 floats = 16 bytes per lane), so the group gathers SLOTS = G/LPN neighbour
// rows at once, each as one contiguous CP*4-byte segment.  The row's (col, w) pairs are read G at
// a time with one coalesced 8-byte load per lane and handed round with lane shuffles; UN gathers
// are issued back to back before their values are used.  Every lane keeps the partial sums of its
// slot; a butterfly over the slot bits finishes acc = sum_j w_j F[col_j] and s = sum_j w_j.
template <int CP>
struct RowShape {
    static constexpr int VEC = CP >= 4 ? 4 : CP;
    static constexpr int LPN = CP / VEC;
};

// Accumulate the chunks first_chunk, first_chunk + chunk_step, ... (G entries each) of one row.
// Lanes past the end of the row carry a stand-in entry (own row, weight 0).  On return e holds the
// last chunk this group loaded (or the stand-in if it loaded none).
template <int CP, int G, bool COH = false>
__device__ inline void accumulate_row(const Edge* __restrict__ row, int len, int first_chunk, int chunk_step,
                                      int32_t u, const float* F_in, int gl,
                                      Vec<RowShape<CP>::VEC>& acc, float& s, Edge& e) {
    constexpr int VEC = RowShape<CP>::VEC;
    constexpr int LPN = RowShape<CP>::LPN;
    constexpr int SLOTS = G / LPN;
    constexpr int UN = LPN < DYNLP_UN_CAP ? LPN : DYNLP_UN_CAP;
    static_assert(G % LPN == 0 && SLOTS >= 1, "group must hold whole neighbour rows");
    static_assert(G % (SLOTS * UN) == 0, "a chunk of G entries is a whole number of gather blocks");
    const int slot = gl / LPN;
    const int chunk = gl % LPN;
    for (int base = first_chunk * G; base < len; base += chunk_step * G) {
        const int idx = base + gl;
        if (idx < len) {
            e = row[idx];
        } else {
            e.col = u;
            e.w = 0.f;
        }
        const int cnt = len - base;
#pragma unroll
        for (int j0 = 0; j0 < G; j0 += SLOTS * UN) {
            if (j0 < cnt) {  // uniform across the group
                int32_t c[UN];
                float w[UN];
                Vec<VEC> f[UN];
#pragma unroll
                for (int t = 0; t < UN; ++t) {
                    c[t] = __shfl(e.col, j0 + t * SLOTS + slot, G);
                    w[t] = __shfl(e.w, j0 + t * SLOTS + slot, G);
                }
#pragma unroll
                for (int t = 0; t < UN; ++t) f[t] = load_row<VEC, COH>(F_in + (size_t)c[t] * CP + chunk * VEC);
#pragma unroll
                for (int t = 0; t < UN; ++t) {
#pragma unroll
                    for (int k = 0; k < VEC; ++k) acc.v[k] = fmaf(w[t], f[t].v[k], acc.v[k]);
                    s += w[t];
                }
            }
        }
    }
#pragma unroll
    for (int d = LPN; d < G; d <<= 1) {
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc.v[k] += __shfl_xor(acc.v[k], d, G);
        s += __shfl_xor(s, d, G);
    }
}

// Per-workgroup totals -> one set of atomics on one of the round's partial records.
// Returns (in thread 0) the number of rows the workgroup moved.
__device__ inline unsigned int flush_round_counters(float rmax, unsigned long long edges, unsigned int changed,
                                                    RoundCtr* __restrict__ ctr, bool long_rows, unsigned int rows = 0) {
    __shared__ float sm_r[kBlock / kWave];
    __shared__ unsigned long long sm_e[kBlock / kWave];
    __shared__ unsigned int sm_c[kBlock / kWave];
    __shared__ unsigned int sm_n[kBlock / kWave];
    rmax = wave_max(rmax);
    edges = wave_sum(edges);
    changed = wave_sum(changed);
    rows = wave_sum(rows);
    if (lane_id() == 0) {
        sm_r[threadIdx.x / kWave] = rmax;
        sm_e[threadIdx.x / kWave] = edges;
        sm_c[threadIdx.x / kWave] = changed;
        sm_n[threadIdx.x / kWave] = rows;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < kBlock / kWave; ++i) {
            rmax = fmaxf(rmax, sm_r[i]);
            edges += sm_e[i];
            changed += sm_c[i];
            rows += sm_n[i];
        }
        RoundPart* p = &ctr->part[blockIdx.x & (kCtrLanes - 1)];
        if (rmax > 0.f) atomicMax(&p->resid_bits, __float_as_uint(rmax));
        if (edges) atomicAdd(long_rows ? &p->edges_long : &p->edges, edges);
        if (changed) {
            atomicAdd(&p->changed, changed);
            ctr->any_moved = 1u;
        }
        if (rows) atomicAdd(long_rows ? &p->rows_long : &p->rows_short, rows);
    }
    return changed;
}

// Short rows: G lanes per row, grid-strided (body; k_row_update dispatches to it).
//   STAGED = false (static sweep / ping-pong round): F'_u is written to row u of F_out, the
//            ping-pong partner of F_in; a row that moved by more than tol sets its bit in moved[]
//            (if not NULL; see k_pull_frontier).
//   STAGED = true (partial round): F'_u is staged at row pos of F_out so that every row of this
//            round reads the round-start F (Jacobi); a row that moved by > tol marks itself and
//            its neighbours in flag[] for the next round.  by_vertex is a set of flags.  kRowByVertex: the
//            row is written to row u of F_out instead (in-place rounds, F_out == F_in: nothing to commit).
//            kRowLazy: the new row is the mean of the old row and the weighted mean of the neighbours (same
//            fixed point; the host asks for it when rounds repeat themselves exactly, a period-2 cycle
//            that float32 rounding keeps alive in a nearly bipartite, weakly tied component).
// F_in and F_out may be the same array (in-place mode): a row then reads whatever its neighbours
// hold at that moment.  Reads and writes are whole 16-byte segments, columns are independent linear
// systems, and the update is a contraction per column, so mixed old/new reads only change the path
// to the fixed point, not the fixed point.
//   PULL (with STAGED = false): front lists every updatable vertex and the round itself decides which of them
//            are in V_aff: u is updated iff u or one of its neighbours moved by more than tol in the previous
//            round (bitmap moved_prev) - Alg. 2 Step 3's V_aff, evaluated where the row is read anyway.  A row
//            outside V_aff is copied to F_out when that is another buffer, so the two keep agreeing there.
constexpr int kRowByVertex = 1, kRowLazy = 2;

template <int CP, int G, bool STAGED, bool PULL = false, bool COH = false>
__device__ inline unsigned int row_update_short(unsigned int bid, unsigned int nblocks, const int32_t* __restrict__ front,
                                        unsigned int ns, const RowMeta* __restrict__ meta,
                                        const Edge* __restrict__ pool, const float* F_in,
                                        float* F_out, int by_vertex, uint8_t* __restrict__ flag,
                                        unsigned int* __restrict__ moved, float tol,
                                        RoundCtr* __restrict__ ctr,
                                        const unsigned int* moved_prev = nullptr) {
    constexpr int VEC = RowShape<CP>::VEC;
    constexpr int LPN = RowShape<CP>::LPN;
    constexpr int GPB = kBlock / G;
    const int gl = threadIdx.x % G;
    const int slot = gl / LPN;
    const int chunk = gl % LPN;
    float rmax = 0.f;
    unsigned long long edges = 0;
    unsigned int nchanged = 0;
    unsigned int nrows = 0;

    for (unsigned int g = bid * GPB + threadIdx.x / G; g < ns; g += nblocks * GPB) {
        const int32_t u = front[g];
        const RowMeta m = meta[u];
        const Edge* __restrict__ row = pool + m.off;
        if (PULL) {
            bool in_front = moved_bit_c<COH>(moved_prev, u);
            for (int base = 0; base < m.len && !in_front; base += G) {  // uniform in the group
                const int idx = base + gl;
                const bool hit = idx < m.len && moved_bit_c<COH>(moved_prev, row[idx].col);
                const unsigned long long b = __ballot(hit);
                const unsigned long long mine = G == kWave ? b : (b >> ((lane_id() / G) * G)) & ((1ull << (G & 63)) - 1ull);
                in_front = mine != 0ull;
            }
            if (!in_front) {
                if (F_out != F_in && slot == 0)
                    store_row<VEC, COH>(F_out + (size_t)u * CP + chunk * VEC, load_row<VEC, COH>(F_in + (size_t)u * CP + chunk * VEC));
                continue;
            }
            if (gl == 0) nrows += 1;
        }
        Vec<VEC> acc;
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc.v[k] = 0.f;
        float s = 0.f;
        Edge e;
        e.col = u;
        e.w = 0.f;
        accumulate_row<CP, G, COH>(row, m.len, 0, 1, u, F_in, gl, acc, s, e);
        const Vec<VEC> old = load_row<VEC, COH>(F_in + (size_t)u * CP + chunk * VEC);
        Vec<VEC> fn;
        float r = 0.f;
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            fn.v[k] = acc.v[k] / s;
            if (by_vertex & kRowLazy) fn.v[k] = 0.5f * (fn.v[k] + old.v[k]);
            r = fmaxf(r, fabsf(fn.v[k] - old.v[k]));
        }
#pragma unroll
        for (int d = 1; d < LPN; d <<= 1) r = fmaxf(r, __shfl_xor(r, d, G));
        if (slot == 0) store_row<VEC, COH>(F_out + (size_t)(STAGED && !(by_vertex & kRowByVertex) ? g : (unsigned int)u) * CP + chunk * VEC, fn);
        const bool big = r > tol;
        if (STAGED) {
            if (big) {  // V_aff <- V_aff U {u} U N(u); the last chunk of the row is still in registers
                if (gl == 0) flag[u] = 1;
                if (e.w != 0.f) mark(flag, e.col);
                const int last_base = ((m.len - 1) / G) * G;
                for (int idx = gl; idx < last_base; idx += G) mark(flag, row[idx].col);
            }
        } else if (moved) {
            // one atomic per distinct bitmap word among the rows of this wave (consecutive list positions are mostly
            // consecutive vertices: the wave's kWave / G rows usually share a word)
            const unsigned int word = (unsigned int)u >> 5;
            unsigned int bits = (big && gl == 0) ? 1u << ((unsigned int)u & 31u) : 0u;
            bool lowest = true;
#pragma unroll
            for (int k = 0; k < kWave / G; ++k) {
                const unsigned int ow = __shfl(word, k * G);
                const unsigned int ob = __shfl((big && gl == 0) ? 1u << ((unsigned int)u & 31u) : 0u, k * G);
                if (ow == word && k * G != (lane_id() / G) * G) {
                    bits |= ob;
                    if (k * G < (lane_id() / G) * G && ob) lowest = false;
                }
            }
            if (gl == 0 && big && lowest) atomicOr(&moved[word], bits);
        }
        if (gl == 0) {
            rmax = fmaxf(rmax, r);
            edges += (unsigned long long)m.len;
            nchanged += big ? 1u : 0u;
        }
    }
    return flush_round_counters(rmax, edges, nchanged, ctr, false, nrows);
}

// Long rows: one workgroup per row (body; k_row_update dispatches to it).  Its kBlock/G groups take the row's chunks round-robin; their
// partial sums meet in LDS and are added in group order (a fixed order: results do not depend on
// timing).  Position of long row j is pos_base + j.
template <int CP, bool STAGED, bool PULL = false, bool COH = false>
__device__ inline unsigned int row_update_long(unsigned int bid, unsigned int nblocks, const int32_t* __restrict__ back,
                                       unsigned int nl, unsigned int pos_base, const RowMeta* __restrict__ meta,
                                       const Edge* __restrict__ pool, const float* F_in,
                                       float* F_out, int by_vertex, uint8_t* __restrict__ flag,
                                       unsigned int* __restrict__ moved, float tol,
                                       RoundCtr* __restrict__ ctr,
                                       const unsigned int* moved_prev = nullptr) {
    constexpr int VEC = RowShape<CP>::VEC;
    constexpr int LPN = RowShape<CP>::LPN;
    constexpr int G = LPN > 16 ? LPN : 16;
    constexpr int NG = kBlock / G;
    __shared__ float part[NG][CP + 1];
    __shared__ float part_s[NG];
    __shared__ int sh_big;
    const int gi = threadIdx.x / G;
    const int gl = threadIdx.x % G;
    const int slot = gl / LPN;
    const int chunk = gl % LPN;
    float rmax = 0.f;
    unsigned long long edges = 0;
    unsigned int nchanged = 0;

    unsigned int nrows = 0;
    for (unsigned int j = bid; j < nl; j += nblocks) {
        const int32_t u = back[-(long long)j];
        const RowMeta m = meta[u];
        const Edge* __restrict__ row = pool + m.off;
        if (PULL) {  // every decision below is uniform across the workgroup
            bool in_front = moved_bit_c<COH>(moved_prev, u);
            for (int base = 0; base < m.len && !in_front; base += kBlock) {
                const int idx = base + (int)threadIdx.x;
                in_front = __syncthreads_or(idx < m.len && moved_bit_c<COH>(moved_prev, row[idx].col)) != 0;
            }
            if (!in_front) {
                if (F_out != F_in && gi == 0 && slot == 0)
                    store_row<VEC, COH>(F_out + (size_t)u * CP + chunk * VEC, load_row<VEC, COH>(F_in + (size_t)u * CP + chunk * VEC));
                continue;
            }
            if (threadIdx.x == 0) nrows += 1;
        }
        Vec<VEC> acc;
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc.v[k] = 0.f;
        float s = 0.f;
        Edge e;
        e.col = u;
        e.w = 0.f;
        accumulate_row<CP, G, COH>(row, m.len, gi, NG, u, F_in, gl, acc, s, e);
        if (slot == 0) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) part[gi][chunk * VEC + k] = acc.v[k];
            if (gl == 0) part_s[gi] = s;
        }
        __syncthreads();
        if (gi == 0 && slot == 0) {
            Vec<VEC> tot;
#pragma unroll
            for (int k = 0; k < VEC; ++k) tot.v[k] = 0.f;
            float st = 0.f;
            for (int q = 0; q < NG; ++q) {
#pragma unroll
                for (int k = 0; k < VEC; ++k) tot.v[k] += part[q][chunk * VEC + k];
                st += part_s[q];
            }
            const Vec<VEC> old = load_row<VEC, COH>(F_in + (size_t)u * CP + chunk * VEC);
            Vec<VEC> fn;
            float r = 0.f;
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                fn.v[k] = tot.v[k] / st;
                if (by_vertex & kRowLazy) fn.v[k] = 0.5f * (fn.v[k] + old.v[k]);
                r = fmaxf(r, fabsf(fn.v[k] - old.v[k]));
            }
#pragma unroll
            for (int d = 1; d < LPN; d <<= 1) r = fmaxf(r, __shfl_xor(r, d, G));
            store_row<VEC, COH>(F_out + (size_t)(STAGED && !(by_vertex & kRowByVertex) ? pos_base + j : (unsigned int)u) * CP + chunk * VEC, fn);
            if (gl == 0) {
                const bool big = r > tol;
                sh_big = big ? 1 : 0;
                if (!STAGED && moved && big) atomicOr(&moved[(unsigned int)u >> 5], 1u << ((unsigned int)u & 31u));
                rmax = fmaxf(rmax, r);
                edges += (unsigned long long)m.len;
                nchanged += big ? 1u : 0u;
            }
        }
        __syncthreads();
        if (STAGED && sh_big) {
            if (threadIdx.x == 0) flag[u] = 1;
            for (int idx = threadIdx.x; idx < m.len; idx += kBlock) mark(flag, row[idx].col);
        }
        __syncthreads();
    }
    return flush_round_counters(rmax, edges, nchanged, ctr, true, nrows);
}

// One launch per round.  The frontier's size comes from the previous round's counter slot (prev), so
// that rounds can be queued back to back without the host reading anything.  Workgroups
// [0, long_blocks) take the long rows (started first: they are the long poles; long_blocks =
// min(long rows, long_blocks_max)), the rest take the short rows.  Workgroup 0 clears the counter slot of the next round and records what this round
// worked on.  stop_bits: a static sweep does nothing if the previous sweep already met the stop rule
// (max change <= tol, as float bits) or did not run; frontier rounds pass 0xffffffff... never stop.
template <int CP, int G, bool STAGED>
__global__ void __launch_bounds__(kBlock) k_row_update(const RoundCtr* __restrict__ prev, int static_stop,
                                                      unsigned int stop_bits, unsigned int long_blocks_max,
                                                      const int32_t* __restrict__ front,
                                                      const int32_t* __restrict__ back,
                                                      const RowMeta* __restrict__ meta,
                                                      const Edge* __restrict__ pool,
                                                      const float* F_in, float* F_out, int by_vertex,
                                                      uint8_t* __restrict__ flag, unsigned int* __restrict__ moved,
                                                      float tol,
                                                      RoundCtr* __restrict__ ctr,
                                                      RoundCtr* __restrict__ ctr_zero) {
    if (ctr_zero && blockIdx.x == 0) {
        if (threadIdx.x == 0) {
            ctr_zero->next_count = 0;
            ctr_zero->next_long = 0;
            ctr_zero->executed = 0;
            ctr_zero->rows_short = 0;
            ctr_zero->rows_long = 0;
            ctr_zero->any_moved = 0;
        }
        if (threadIdx.x < kCtrLanes) {
            RoundPart* p = &ctr_zero->part[threadIdx.x];
            p->resid_bits = 0;
            p->changed = 0;
            p->edges = 0;
            p->edges_long = 0;
            p->rows_short = 0;
            p->rows_long = 0;
        }
    }
    const unsigned int ns = prev->next_count, nl = prev->next_long;
    if (ns + nl == 0) return;
    if (static_stop) {
        unsigned int prev_resid = 0xffffffffu;
        if (static_stop == 2) {  // max change of the previous sweep: maximum over its partial records
            const int lane = lane_id();
            prev_resid = lane < kCtrLanes ? prev->part[lane].resid_bits : 0u;
#pragma unroll
            for (int d = kWave / 2; d > 0; d >>= 1) {
                const unsigned int o = __shfl_xor(prev_resid, d, kWave);
                prev_resid = o > prev_resid ? o : prev_resid;
            }
        }
        if (static_stop == 2 && (!prev->executed || prev_resid <= stop_bits)) {
            // keep the frontier for whoever reads this slot next
            if (blockIdx.x == 0 && threadIdx.x == 0) {
                ctr->next_count = ns;
                ctr->next_long = nl;
            }
            return;
        }
        if (blockIdx.x == 0 && threadIdx.x == 0) {  // a static sweep's frontier never changes
            ctr->next_count = ns;
            ctr->next_long = nl;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        ctr->executed = 1;
        ctr->rows_short = ns;
        ctr->rows_long = nl;
    }
    const unsigned int long_blocks = nl < long_blocks_max ? nl : long_blocks_max;
    if (blockIdx.x < long_blocks)
        row_update_long<CP, STAGED>(blockIdx.x, long_blocks, back, nl, ns, meta, pool, F_in, F_out, by_vertex, flag, moved,
                                    tol, ctr);
    else
        row_update_short<CP, G, STAGED>(blockIdx.x - long_blocks, gridDim.x - long_blocks, front, ns, meta, pool, F_in,
                                        F_out, by_vertex, flag, moved, tol, ctr);
}

// A round over nearly all updatable vertices that finds its own V_aff (no frontier list, no separate pull):
// (front, back, ns, nl) is the list of all updatable vertices; moved_prev has the bits of the rows that moved
// in the previous round, moved_cur receives this round's, moved_clear (the bitmap of the round after) is
// zeroed.  The round does nothing if the previous one did not run or moved no row (V_aff is empty then).
template <int CP, int G>
__global__ void __launch_bounds__(kBlock) k_row_update_pull(const RoundCtr* __restrict__ prev, unsigned int long_blocks_max,
                                                           const int32_t* __restrict__ front,
                                                           const int32_t* __restrict__ back, unsigned int ns,
                                                           unsigned int nl, const RowMeta* __restrict__ meta,
                                                           const Edge* __restrict__ pool, const float* F_in,
                                                           float* F_out, const unsigned int* __restrict__ moved_prev,
                                                           unsigned int* __restrict__ moved_cur,
                                                           unsigned int* __restrict__ moved_clear, unsigned int words,
                                                           float tol, RoundCtr* __restrict__ ctr,
                                                           RoundCtr* __restrict__ ctr_zero) {
    if (ctr_zero && blockIdx.x == 0) {
        if (threadIdx.x == 0) {
            ctr_zero->next_count = 0;
            ctr_zero->next_long = 0;
            ctr_zero->executed = 0;
            ctr_zero->rows_short = 0;
            ctr_zero->rows_long = 0;
            ctr_zero->any_moved = 0;
        }
        if (threadIdx.x < kCtrLanes) {
            RoundPart* p = &ctr_zero->part[threadIdx.x];
            p->resid_bits = 0;
            p->changed = 0;
            p->edges = 0;
            p->edges_long = 0;
            p->rows_short = 0;
            p->rows_long = 0;
        }
    }
    // did the previous round move a row?  (one word of its header instead of its 32 partial records: thousands of
    // short-lived workgroups each reading 32 lines was a fifth of the launch on a 100K-vertex graph)
    if (!prev->executed || prev->any_moved == 0u) return;
    for (unsigned int w = blockIdx.x * kBlock + threadIdx.x; w < words; w += gridDim.x * kBlock) moved_clear[w] = 0u;
    if (blockIdx.x == 0 && threadIdx.x == 0) ctr->executed = 1;
    const unsigned int long_blocks = nl < long_blocks_max ? nl : long_blocks_max;
    if (blockIdx.x < long_blocks)
        row_update_long<CP, false, true>(blockIdx.x, long_blocks, back, nl, ns, meta, pool, F_in, F_out, 1, nullptr,
                                         moved_cur, tol, ctr, moved_prev);
    else
        row_update_short<CP, G, false, true>(blockIdx.x - long_blocks, gridDim.x - long_blocks, front, ns, meta, pool,
                                             F_in, F_out, 1, nullptr, moved_cur, tol, ctr, moved_prev);
}

// =================================================================================================
// Several rounds in one launch, for graphs whose rounds are too short to be worth a launch each
// =================================================================================================
// On a graph of a few hundred thousand rows a round over all rows takes tens of microseconds, of which the
// work is a small part: the rest is the launch, the ramp-up of thousands of short-lived workgroups and the
// drain before the next launch may start.  k_rounds_persistent runs up to `rounds` consecutive rounds of the kind
// k_row_update_pull runs (every updatable vertex decides from the previous round's bitmap whether it is in V_aff)
// with a grid of workgroups that are all resident at once and a barrier across the grid between rounds.
//
// What crosses the barrier (label rows, bitmap words, counters) is read and written with device-scope accesses
// (load_row / store_row / moved_bit_c with COH): every XCD has an L2 of its own, and writing back and invalidating
// whole caches at every barrier costs ten times the round.
//
// The barrier is a two-level tree, so that no address is polled by more than kBarGroup workgroups (a word polled by
// a thousand workgroups answers so slowly that the barrier alone took 100 us): a workgroup arrives at its group's
// counter; the last arrival of a group arrives at the global counter; the last arrival there writes the release
// word of every group, and every workgroup waits for the release word of its group only.  The arrivals carry along
// whether the workgroup moved a row in the round, so that the release word also says whether any row moved at all:
// if none did, V_aff is empty and every workgroup leaves the kernel.
//
// The wait is bounded.  After spin_limit polls a workgroup tries to give the barrier up for the whole grid: a
// compare-and-swap sets the top bit of the global counter, and only succeeds while the last group has not arrived
// there; the last arrival, in turn, does not release when it finds that bit set.  So either every workgroup is
// released from barrier k or none is, and no round is ever run by a part of the grid.  Every workgroup completes the
// work of a round before it looks at the barrier; whenever the kernel ends - all rounds done, V_aff empty, or a
// barrier given up - the rounds whose counter slots say "executed" have been executed in full, and the host goes
// on from there with ordinary launches.
constexpr unsigned int kBarGroup = 32;              // workgroups per group
constexpr unsigned int kBarWordsPerLine = 16;       // every counter and release word has a 64-byte line of its own
constexpr unsigned int kBarMaxGroups = 128;
constexpr unsigned int kBarGivenUp = 0x80000000u;   // global counter: the barrier was given up
constexpr unsigned int kBarMovedUnit = 0x10000u;    // counters: arrivals in the low 16 bits, arrivals that moved rows above
constexpr unsigned int kRelStop = 0x40000000u;      // release word: no row moved in the round
constexpr unsigned int kRelFail = 0x80000000u;      // release word: the barrier was given up
// words: [0] global counter, [1] "a barrier was given up" for the host, then one line per group counter, then one
// line per release word
constexpr unsigned int kBarWords = kBarWordsPerLine * (1 + 2 * kBarMaxGroups);

struct PersistArgs {
    RoundCtr* ring;               // kRing slots
    int t0;                       // round number of the first round (>= 1)
    int rounds;
    unsigned int long_blocks_max;
    const int32_t* front;         // list of all updatable vertices: short rows from the front, long rows from the back
    const int32_t* back;
    unsigned int ns, nl;
    const RowMeta* meta;
    const Edge* pool;
    float* buf0;                  // round t0 + r reads buf[r & 1] and writes buf[(r + 1) & 1] (one array in place)
    float* buf1;
    unsigned int* moved0;         // the three bitmaps; the round with stretch index q reads (q - 1) % 3, sets q % 3
    unsigned int* moved1;         // and clears (q + 1) % 3
    unsigned int* moved2;
    int q0;                       // stretch index of the first round (>= 1)
    unsigned int words;
    float tol;
    unsigned int* barrier;        // kBarWords words, all zero at launch
    unsigned int ngroups;         // ceil(gridDim.x / kBarGroup) <= kBarMaxGroups
    unsigned int spin_limit;
};

__device__ inline unsigned int load_fresh(const unsigned int* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ inline void store_through(unsigned int* p, unsigned int v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Barrier number k (1, 2, ...) of the launch.  moved: this workgroup moved at least one row in the round (thread 0's
// value counts).  Returns 1: released, some row moved; 2: released, no row moved anywhere; 0: given up.
__device__ inline int grid_barrier(unsigned int* bar, unsigned int k, unsigned int ngroups, bool moved,
                                   unsigned int spin_limit) {
    __shared__ int sh_res;
    // every wave: its stores and atomics of this round (all of them device-scope, write-through accesses) have been
    // acknowledged before the workgroup reports its arrival
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int g = blockIdx.x / kBarGroup;
        const unsigned int first = g * kBarGroup;
        const unsigned int gsize = gridDim.x - first < kBarGroup ? gridDim.x - first : kBarGroup;
        unsigned int* global = bar;
        unsigned int* gctr = bar + kBarWordsPerLine * (1 + g);
        unsigned int* rel = bar + kBarWordsPerLine * (1 + ngroups + g);
        auto release_all = [&](unsigned int word) {
            for (unsigned int i = 0; i < ngroups; ++i) store_through(bar + kBarWordsPerLine * (1 + ngroups + i), word);
        };
        const unsigned int add = 1u + (moved ? kBarMovedUnit : 0u);
        const unsigned int in_group = atomicAdd(gctr, add) + add;
        if ((in_group & 0xffffu) == gsize * k) {
            // last of the group: take the group's "moved" count out again and arrive at the global counter
            const unsigned int group_moved = in_group & 0xffff0000u;
            if (group_moved) atomicSub(gctr, group_moved);
            const unsigned int gadd = 1u + (group_moved ? kBarMovedUnit : 0u);
            const unsigned int old = atomicAdd(global, gadd);
            const unsigned int now = old + gadd;
            if (old & kBarGivenUp) {
                release_all(kRelFail | k);
            } else if ((now & 0xffffu) == ngroups * k) {
                // last of all: nobody else touches the global counter until the next round's arrivals
                const unsigned int any_moved = now & 0x7fff0000u;
                if (any_moved) atomicSub(global, any_moved);
                release_all(k | (any_moved ? 0u : kRelStop));
            }
        }
        int res = -1;
        unsigned int spins = 0;
        while (res < 0) {
            const unsigned int w = load_fresh(rel);
            if (w & kRelFail) {
                res = 0;
            } else if ((w & 0xffffu) == k) {
                res = (w & kRelStop) ? 2 : 1;
            } else if (++spins > spin_limit) {
                // give up for everybody, unless the last group has arrived by now (then the release is on its way)
                const unsigned int v = load_fresh(global);
                if (v & kBarGivenUp) {
                    res = 0;
                } else if ((v & 0xffffu) >= ngroups * k) {
                    spins = 0;
                } else if (atomicCAS(global, v, v | kBarGivenUp) == v) {
                    release_all(kRelFail | k);
                    res = 0;
                }
            } else {
                __builtin_amdgcn_s_sleep(16);
            }
        }
        if (res == 0) store_through(&bar[1], 1u);  // for the host
        sh_res = res;
    }
    __syncthreads();
    const int res = sh_res;
    __syncthreads();  // sh_res may be rewritten by the next barrier
    return res;
}

template <int CP, int G>
__global__ void __launch_bounds__(kBlock) k_rounds_persistent(PersistArgs a) {
    __shared__ unsigned int sh_go;
    unsigned int* const moved[3] = {a.moved0, a.moved1, a.moved2};
    float* const buf[2] = {a.buf0, a.buf1};
    const unsigned int long_blocks = a.nl < a.long_blocks_max ? a.nl : a.long_blocks_max;
    {
        // the round before the launch: did it run, and did it move a row?  (every later round learns this from the
        // barrier)
        const RoundCtr* prev = a.ring + ((a.t0 - 1) % kRing);
        if (threadIdx.x < kWave) {
            unsigned int prev_changed = lane_id() < kCtrLanes ? load_fresh(&prev->part[lane_id()].changed) : 0u;
            prev_changed = wave_sum(prev_changed);
            if (threadIdx.x == 0) sh_go = (load_fresh(&prev->executed) != 0u && prev_changed != 0u) ? 1u : 0u;
        }
        __syncthreads();
        if (sh_go == 0u) return;  // the same for every workgroup
    }
    for (int r = 0; r < a.rounds; ++r) {
        const int t = a.t0 + r;
        RoundCtr* ctr = a.ring + (t % kRing);
        RoundCtr* ctr_zero = a.ring + ((t + 1) % kRing);
        if (blockIdx.x == 0) {  // write-through stores: the slot's next user may sit on another XCD
            auto put64 = [](unsigned long long* p, unsigned long long v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
            if (threadIdx.x == 0) {
                store_through(&ctr_zero->next_count, 0u);
                store_through(&ctr_zero->next_long, 0u);
                store_through(&ctr_zero->executed, 0u);
                store_through(&ctr_zero->rows_short, 0u);
                store_through(&ctr_zero->rows_long, 0u);
                store_through(&ctr_zero->any_moved, 0u);
                store_through(&ctr->executed, 1u);
            }
            if (threadIdx.x < kCtrLanes) {
                RoundPart* p = &ctr_zero->part[threadIdx.x];
                store_through(&p->resid_bits, 0u);
                store_through(&p->changed, 0u);
                put64(&p->edges, 0ull);
                put64(&p->edges_long, 0ull);
                store_through(&p->rows_short, 0u);
                store_through(&p->rows_long, 0u);
            }
        }
        const int q = a.q0 + r;
        unsigned int* moved_clear = moved[(q + 1) % 3];
        for (unsigned int w = blockIdx.x * kBlock + threadIdx.x; w < a.words; w += gridDim.x * kBlock)
            store_through(&moved_clear[w], 0u);
        const float* F_in = buf[r & 1];
        float* F_out = buf[(r + 1) & 1];
        unsigned int block_moved;
        if (blockIdx.x < long_blocks)
            block_moved = row_update_long<CP, false, true, true>(blockIdx.x, long_blocks, a.back, a.nl, a.ns, a.meta, a.pool,
                                                                 F_in, F_out, 1, nullptr, moved[q % 3], a.tol, ctr,
                                                                 moved[(q + 2) % 3]);
        else
            block_moved = row_update_short<CP, G, false, true, true>(blockIdx.x - long_blocks, gridDim.x - long_blocks, a.front,
                                                                     a.ns, a.meta, a.pool, F_in, F_out, 1, nullptr,
                                                                     moved[q % 3], a.tol, ctr, moved[(q + 2) % 3]);
        if (r + 1 == a.rounds) return;
        if (grid_barrier(a.barrier, (unsigned int)(r + 1), a.ngroups, block_moved != 0u, a.spin_limit) != 1) return;
    }
}

}  // namespace dynlp
