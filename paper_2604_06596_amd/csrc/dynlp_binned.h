// Binned rounds for scalar labels (one float per vertex): Alg. 2 Step 3 / Eq. (1) over nearly all vertices
// without random accesses to memory.
//
// With one float per vertex a gather of F[v] for a random neighbour v costs a whole 128-byte line for 4
// useful bytes; on a graph whose labels do not fit the L2 the ordinary row update moves about ten times its
// algorithmic bytes.  While the graph does not change (all rounds of one batch) the same sums can be
// formed from two streaming passes ("propagation blocking"):
//
//   scatter   every vertex u (labelled ones too: they are sources) sends its label, with the "moved in the
//             previous round" flag in the sign bit (labels are >= 0), to one slot per stored entry (u, v).
//             Slots are grouped by the bin of the receiving vertex v (bin = v >> bin_bits) and, inside a bin,
//             ordered by chunks of kPbChunk consecutive entries of the sources' rows.  A workgroup takes one
//             chunk, sorts its values by slot inside LDS (the permutation is fixed when the slots are laid out)
//             and writes them out so that neighbouring lanes write neighbouring slots: one write transaction
//             per (chunk, bin) run rather than one per entry.  (Written straight from the entries, one 4-byte
//             store each, the pass ran at the speed of the random gathers it was meant to replace.)
//   gather    one workgroup per bin streams the bin's slots (receiver's offset in the bin, weight divided by
//             the receiver's degree, value) and adds w/deg * F into an LDS accumulator per receiver; a second
//             LDS bitmap collects "a neighbour moved".  Then every receiver of the bin that is in V_aff (it
//             moved itself or a neighbour did: Alg. 2 Step 3) takes the sum as its new label, exactly one
//             Jacobi update of Eq. (1) from the labels the scatter pass saw.
//
// The accumulator is a 32-bit fixed-point number (terms w/deg * F lie in [0, 1] and sum to at most 1, one
// unit = 2^-30): integer additions commute, so the result does not depend on the order of the LDS atomics nor
// on where the build step happened to place an entry inside its run.  Rounding each term to 2^-31 is finer
// than the float32 arithmetic of the ordinary row update.
#pragma once

#include "dynlp_device.h"

namespace dynlp {

constexpr int kPbMaxBinBits = 15;                  // receivers per bin: at most 32,768 (128 KB of accumulators)
constexpr int kPbMinBinBits = 8;                   // small bins: for tests on small graphs
constexpr int kPbMaxBins = 4096;                   // bin histograms live in LDS during the build
constexpr unsigned int kPbNone = 0xffffffffu;      // slot of an entry whose receiver is never updated
constexpr int kPbChunk = 16384;                    // entries per chunk: 64 KB of staged values (8K / 16K / 32K entries:
                                                   // 1.74 / 1.63 / 1.82 ms per round on 250M entries)
constexpr float kPbUnit = 1073741824.0f;           // 2^30
constexpr int kPbMaxParts = 16;                    // in-place mode: vertex ranges updated one after the other in a round

// receivers: len[v] = row length if v is updatable (unlabelled, at least one entry), else 0; the same as one
// bit per vertex in upd[] (the build passes test it for every entry; 1 bit per vertex stays in the L2).
__global__ void __launch_bounds__(kBlock) k_pb_receivers(int64_t n, const RowMeta* __restrict__ meta,
                                                        const int32_t* __restrict__ seed_class,
                                                        int32_t* __restrict__ len, unsigned int* __restrict__ upd) {
    const int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    int l = 0;
    if (v < n && seed_class[v] < 0) l = meta[v].len;
    if (v < n) len[v] = l;
    const unsigned long long b = __ballot(l > 0);
    const int lane = lane_id();
    if ((lane == 0 || lane == 32) && v < ((n + 31) & ~(int64_t)31)) upd[v >> 5] = (unsigned int)(lane == 0 ? b : b >> 32);
}

__device__ inline bool pb_bit(const unsigned int* __restrict__ bits, int32_t v) {
    return (bits[(unsigned int)v >> 5] >> ((unsigned int)v & 31u)) & 1u;
}

// first[u] = number of stored entries in rows 0 .. u-1 (first[n] = all of them): entry j of row u is entry
// first[u] + j of the stream the scatter pass reads, whatever the order of the rows in the pool.  Three steps:
// entries per block of kBlock rows, exclusive scan of the block sums by one workgroup, offsets inside every block.
__global__ void __launch_bounds__(kBlock) k_pb_row_blocks(int64_t n, const RowMeta* __restrict__ meta,
                                                         unsigned int* __restrict__ block_sum) {
    __shared__ unsigned int smem[kBlock / kWave + 1];
    const int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    unsigned int total;
    (void)block_exclusive_scan<unsigned int>(v < n ? (unsigned int)meta[v].len : 0u, smem, &total);
    if (threadIdx.x == 0) block_sum[blockIdx.x] = total;
}

__global__ void __launch_bounds__(kBlock) k_pb_scan_blocks(int64_t nb, unsigned int* __restrict__ block_sum) {
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
}

__global__ void __launch_bounds__(kBlock) k_pb_row_first(int64_t n, const RowMeta* __restrict__ meta,
                                                        const unsigned int* __restrict__ block_off,
                                                        unsigned int* __restrict__ first) {
    __shared__ unsigned int smem[kBlock / kWave + 1];
    const int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const unsigned int l = v < n ? (unsigned int)meta[v].len : 0u;
    unsigned int total;
    const unsigned int ex = block_exclusive_scan<unsigned int>(l, smem, &total);
    if (v < n) first[v] = block_off[blockIdx.x] + ex;
    if (v == n - 1) first[n] = block_off[blockIdx.x] + ex + l;
}

// Entry i of the stream (rows in vertex order): its row, its neighbour and its weight.  16 lanes per row.
__global__ void __launch_bounds__(kBlock) k_pb_expand(int64_t n, const RowMeta* __restrict__ meta,
                                                     const Edge* __restrict__ pool,
                                                     const unsigned int* __restrict__ first,
                                                     unsigned int* __restrict__ src, unsigned int* __restrict__ ecol,
                                                     float* __restrict__ ew) {
    constexpr int G = 16;
    const int gl = threadIdx.x % G;
    const int64_t u = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / G;
    if (u >= n) return;
    const RowMeta m = meta[u];
    const unsigned int a = first[u];
    for (int j = gl; j < m.len; j += G) {
        const Edge e = pool[m.off + j];
        src[a + j] = (unsigned int)u;
        ecol[a + j] = (unsigned int)e.col;
        ew[a + j] = e.w;
    }
}

// The build step orders a bin's slots by chunk: a table of entry counts per (chunk, bin) is turned into the
// first slot of every chunk in every bin.
//
// Entries per (chunk, bin): table[chunk * nbins + bin].  One workgroup per chunk.
__global__ void __launch_bounds__(kBlock) k_pb_count(const unsigned int* __restrict__ num_entries, int bin_bits, int nbins,
                                                    const unsigned int* __restrict__ ecol,
                                                    const unsigned int* __restrict__ upd,
                                                    unsigned int* __restrict__ table) {
    __shared__ unsigned int hist[kPbMaxBins];
    for (int b = threadIdx.x; b < nbins; b += kBlock) hist[b] = 0u;
    __syncthreads();
    const int64_t E = (int64_t)*num_entries;
    const int64_t base = (int64_t)blockIdx.x * kPbChunk;
    for (int k = threadIdx.x; k < kPbChunk; k += kBlock) {
        const int64_t i = base + k;
        if (i >= E) break;
        const unsigned int v = ecol[i];
        if (pb_bit(upd, (int32_t)v)) atomicAdd(&hist[v >> bin_bits], 1u);
    }
    __syncthreads();
    unsigned int* __restrict__ mine = table + (size_t)blockIdx.x * nbins;
    for (int b = threadIdx.x; b < nbins; b += kBlock) mine[b] = hist[b];
}

// table[chunk][bin] -> entries of the bin in earlier chunks; bin_count[bin] = entries of the bin.  One thread per
// bin walks the chunks (neighbouring threads read neighbouring words).
__global__ void __launch_bounds__(kBlock) k_pb_chunk_bases(int nbins, int chunks, unsigned int* __restrict__ table,
                                                          unsigned int* __restrict__ bin_count) {
    const int b = blockIdx.x * kBlock + threadIdx.x;
    if (b >= nbins) return;
    unsigned int run = 0;
    for (int c = 0; c < chunks; ++c) {
        const size_t i = (size_t)c * nbins + b;
        const unsigned int t = table[i];
        table[i] = run;
        run += t;
    }
    bin_count[b] = run;
}

// bin_off = exclusive scan of bin_count (nbins + 1 values).  One workgroup.
__global__ void __launch_bounds__(kBlock) k_pb_offsets(int nbins, const unsigned int* __restrict__ bin_count,
                                                      unsigned int* __restrict__ bin_off) {
    __shared__ unsigned int smem[kBlock / kWave + 1];
    unsigned int carry = 0;
    for (int base = 0; base < nbins; base += kBlock) {
        const int i = base + (int)threadIdx.x;
        const unsigned int v = i < nbins ? bin_count[i] : 0u;
        unsigned int total;
        const unsigned int ex = block_exclusive_scan(v, smem, &total);
        if (i < nbins) bin_off[i] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) bin_off[nbins] = carry;
}

// Slots.  One workgroup per chunk c: its entries of bin b take the slots bin_off[b] + table[c][b] + 0, 1, ... in the
// order an LDS counter hands them out.  Sorted by slot, the chunk's entries have positions 0 .. (its number of
// entries with a slot) - 1: lpos[i] is entry i's position, oslot[c * kPbChunk + position] the slot behind it
// (kPbNone for positions past the last slot: entries whose receiver is never updated come last).  The per-slot
// arrays get the receiver's offset in its bin and the raw weight.
__global__ void __launch_bounds__(kBlock) k_pb_place(const unsigned int* __restrict__ num_entries, int bin_bits, int nbins,
                                                    const unsigned int* __restrict__ ecol, const float* __restrict__ ew,
                                                    const unsigned int* __restrict__ upd,
                                                    const unsigned int* __restrict__ table,
                                                    const unsigned int* __restrict__ bin_off,
                                                    unsigned short* __restrict__ lpos, unsigned int* __restrict__ oslot,
                                                    unsigned short* __restrict__ dst, float* __restrict__ wn) {
    __shared__ unsigned int cnt[kPbMaxBins];   // entries per bin, then handed-out count
    __shared__ unsigned int loff[kPbMaxBins];  // position of the bin's first entry in the sorted chunk
    __shared__ unsigned int smem[kBlock / kWave + 1];
    __shared__ unsigned int none_count;
    for (int b = threadIdx.x; b < nbins; b += kBlock) cnt[b] = 0u;
    if (threadIdx.x == 0) none_count = 0u;
    __syncthreads();
    const int64_t E = (int64_t)*num_entries;
    const int64_t base = (int64_t)blockIdx.x * kPbChunk;
    for (int k = threadIdx.x; k < kPbChunk; k += kBlock) {
        const int64_t i = base + k;
        if (i >= E) break;
        const unsigned int v = ecol[i];
        if (pb_bit(upd, (int32_t)v)) atomicAdd(&cnt[v >> bin_bits], 1u);
    }
    __syncthreads();
    // exclusive scan of cnt over the bins: every thread takes a run of consecutive bins
    const int per = (nbins + kBlock - 1) / kBlock;
    const int b0 = (int)threadIdx.x * per;
    unsigned int mine = 0;
    for (int b = b0; b < b0 + per && b < nbins; ++b) mine += cnt[b];
    unsigned int with_slot;
    unsigned int run = block_exclusive_scan(mine, smem, &with_slot);
    for (int b = b0; b < b0 + per && b < nbins; ++b) {
        loff[b] = run;
        run += cnt[b];
        cnt[b] = 0u;
    }
    __syncthreads();
    const unsigned int* __restrict__ before = table + (size_t)blockIdx.x * nbins;
    const unsigned int mask = (1u << bin_bits) - 1u;
    for (int k = threadIdx.x; k < kPbChunk; k += kBlock) {
        const int64_t i = base + k;
        if (i >= E) break;
        const unsigned int v = ecol[i];
        unsigned int pos, s = kPbNone;
        if (pb_bit(upd, (int32_t)v)) {
            const unsigned int b = v >> bin_bits;
            const unsigned int r = atomicAdd(&cnt[b], 1u);
            pos = loff[b] + r;
            s = bin_off[b] + before[b] + r;
            dst[s] = (unsigned short)(v & mask);
            wn[s] = ew[i];
        } else {
            pos = with_slot + atomicAdd(&none_count, 1u);
        }
        lpos[i] = (unsigned short)pos;
        oslot[base + pos] = s;
    }
    // positions past the chunk's last entry (last chunk only)
    const int64_t in_chunk = E - base < kPbChunk ? E - base : kPbChunk;
    for (int64_t k = in_chunk + threadIdx.x; k < kPbChunk; k += kBlock) oslot[base + k] = kPbNone;
}

// wn[s] /= deg[receiver]: one pass over the slots, one workgroup per bin (the degrees of a bin's receivers
// are a window of at most 128 KB).
__global__ void __launch_bounds__(kBlock) k_pb_normalise(int bin_bits, const unsigned int* __restrict__ bin_off,
                                                        const unsigned short* __restrict__ dst,
                                                        const float* __restrict__ deg, float* __restrict__ wn) {
    const unsigned int lo = bin_off[blockIdx.x], hi = bin_off[blockIdx.x + 1];
    const int64_t first = (int64_t)blockIdx.x << bin_bits;
    for (unsigned int i = lo + threadIdx.x; i < hi; i += kBlock) wn[i] = wn[i] / deg[first + dst[i]];
}

// Early-exit test shared by both passes: a round runs iff the previous one ran and moved at least one row.
__device__ inline bool pb_round_runs(const RoundCtr* __restrict__ prev) {
    unsigned int prev_changed = lane_id() < kCtrLanes ? prev->part[lane_id()].changed : 0u;
    prev_changed = wave_sum(prev_changed);
    return prev->executed && prev_changed != 0u;
}

// Scatter pass, one workgroup per chunk: stage[lpos[i]] = F[src[i]] (sign bit: src[i] moved in the previous round)
// for the chunk's entries i, then val[oslot[position]] = stage[position].  Also clears the counter slot and the
// moved-bitmap of the next round.
//
// Workgroups reach the 8 XCDs round-robin by index; chunks are mapped so that XCD x works through the x-th
// eighth of the chunks in order: the runs that consecutive chunks write into a bin are neighbours, and a line
// shared by two runs is completed from the same L2.
constexpr int kPbScatterThreads = 1024;  // two workgroups of this size and 64 KB fill a CU (256 / 512 / 1024 threads:
                                         // 2.25 / 1.75 / 1.63 ms per round on 250M entries)

__global__ void __launch_bounds__(kPbScatterThreads) k_pb_scatter(const RoundCtr* __restrict__ prev,
                                                      const unsigned int* __restrict__ num_entries, unsigned int chunk0,
                                                      unsigned int chunks,
                                                      const unsigned int* __restrict__ src,
                                                      const unsigned short* __restrict__ lpos,
                                                      const unsigned int* __restrict__ oslot, const float* F_in,
                                                      const unsigned int* __restrict__ moved_prev,
                                                      const unsigned int* __restrict__ moved_also,
                                                      unsigned int* __restrict__ moved_clear, unsigned int words,
                                                      unsigned int* __restrict__ val, RoundCtr* __restrict__ ctr_zero) {
    // chunks chunk0 .. chunk0 + chunks - 1; moved_prev (and moved_also, if not NULL): the bitmaps whose bits travel
    // with the labels ("the sender moved"); moved_clear / ctr_zero may be NULL
    __shared__ unsigned int stage[kPbChunk];
    if (ctr_zero && blockIdx.x == 0) {
        if (threadIdx.x == 0) {
            ctr_zero->next_count = 0;
            ctr_zero->next_long = 0;
            ctr_zero->executed = 0;
            ctr_zero->rows_short = 0;
            ctr_zero->rows_long = 0;
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
    if (!pb_round_runs(prev)) return;
    constexpr int T = kPbScatterThreads;
    if (moved_clear)
        for (unsigned int w = blockIdx.x * T + threadIdx.x; w < words; w += gridDim.x * T) moved_clear[w] = 0u;
    const unsigned int per_xcd = (chunks + 7u) / 8u;
    const unsigned int local = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
    if ((blockIdx.x >> 3) >= per_xcd || local >= chunks) return;
    const unsigned int chunk = chunk0 + local;
    const int64_t E = (int64_t)*num_entries;
    const int64_t base = (int64_t)chunk * kPbChunk;
    constexpr int UN = 4;
    for (int k0 = 0; k0 < kPbChunk; k0 += UN * T) {
        unsigned int u[UN], p[UN];
#pragma unroll
        for (int q = 0; q < UN; ++q) {
            const int64_t i = base + k0 + q * T + threadIdx.x;
            const bool ok = i < E;
            u[q] = ok ? src[i] : 0xffffffffu;
            p[q] = ok ? lpos[i] : 0u;
        }
#pragma unroll
        for (int q = 0; q < UN; ++q)
            if (u[q] != 0xffffffffu)
                stage[p[q]] = __float_as_uint(F_in[u[q]]) |
                              ((pb_bit(moved_prev, (int32_t)u[q]) || (moved_also && pb_bit(moved_also, (int32_t)u[q]))) ? 0x80000000u : 0u);
    }
    __syncthreads();
    for (int k0 = 0; k0 < kPbChunk; k0 += UN * T) {
        unsigned int s[UN];
#pragma unroll
        for (int q = 0; q < UN; ++q) s[q] = oslot[base + k0 + q * T + threadIdx.x];
#pragma unroll
        for (int q = 0; q < UN; ++q)
            if (s[q] != kPbNone) val[s[q]] = stage[k0 + q * T + threadIdx.x];
    }
}

// Gather pass: one workgroup of kPbGatherThreads per bin (the accumulators take most of a CU's LDS, so the
// one resident workgroup is made as wide as the hardware allows).
constexpr int kPbGatherThreads = 1024;

__global__ void __launch_bounds__(kPbGatherThreads) k_pb_gather(const RoundCtr* __restrict__ prev, int64_t n, int bin_bits,
                                                               unsigned int bin0,
                                                               const unsigned int* __restrict__ bin_off,
                                                               const unsigned short* __restrict__ dst,
                                                               const float* __restrict__ wn,
                                                               const unsigned int* __restrict__ val,
                                                               const int32_t* __restrict__ len, const float* F_in,
                                                               float* F_out, const unsigned int* __restrict__ moved_prev,
                                                               unsigned int* __restrict__ moved_cur, float tol,
                                                               RoundCtr* __restrict__ ctr) {
    constexpr int T = kPbGatherThreads;
    constexpr int NW = T / kWave;
    __shared__ unsigned int acc[1 << kPbMaxBinBits];
    __shared__ unsigned int nb[(1 << kPbMaxBinBits) / 32];
    __shared__ float sm_r[NW];
    __shared__ unsigned long long sm_e[NW];
    __shared__ unsigned int sm_c[NW], sm_n[NW];
    // a static sweep finds the size of its row list in its predecessor's slot: hand it on (0 in batch rounds)
    // (one workgroup per bin of the range that starts at bin0)
    const unsigned int bin = bin0 + blockIdx.x;
    if (bin == 0 && threadIdx.x == 0) {
        ctr->next_count = prev->next_count;
        ctr->next_long = prev->next_long;
    }
    if (!pb_round_runs(prev)) return;
    if (bin == 0 && threadIdx.x == 0) ctr->executed = 1;
    const int size = 1 << bin_bits;
    for (int d = threadIdx.x; d < size; d += T) acc[d] = 0u;
    for (int d = threadIdx.x; d < size / 32; d += T) nb[d] = 0u;
    __syncthreads();
    const unsigned int lo = bin_off[bin], hi = bin_off[bin + 1];
    constexpr int UN = 4;  // independent slot reads in flight per lane
    for (unsigned int i0 = lo; i0 < hi; i0 += UN * T) {
        unsigned int d[UN], x[UN];
        float w[UN];
#pragma unroll
        for (int q = 0; q < UN; ++q) {
            const unsigned int i = i0 + q * T + threadIdx.x;
            const bool ok = i < hi;
            d[q] = ok ? dst[i] : 0u;
            x[q] = ok ? val[i] : 0u;
            w[q] = ok ? wn[i] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < UN; ++q) {
            const float term = w[q] * __uint_as_float(x[q] & 0x7fffffffu);
            const unsigned int units = (unsigned int)(term * kPbUnit + 0.5f);
            if (units) atomicAdd(&acc[d[q]], units);
            if (x[q] >> 31) atomicOr(&nb[d[q] >> 5], 1u << (d[q] & 31u));
        }
    }
    __syncthreads();
    const int64_t first = (int64_t)bin << bin_bits;
    const int64_t n_words_end = (n + 31) & ~(int64_t)31;
    float rmax = 0.f;
    unsigned long long edges = 0;
    unsigned int nchanged = 0, nrows = 0;
    for (int d0 = 0; d0 < size; d0 += T) {
        const int d = d0 + (int)threadIdx.x;  // d < size is uniform per wave: size is a multiple of 64
        const int64_t v = first + d;
        bool big = false;
        const int l = (d < size && v < n) ? len[v] : 0;
        if (l > 0) {
            const float old = F_in[v];
            const bool in_front = pb_bit(moved_prev, (int32_t)v) || ((nb[d >> 5] >> (d & 31)) & 1u);
            if (in_front) {
                const float fn = fminf((float)acc[d] * (1.0f / kPbUnit), 1.0f);
                const float r = fabsf(fn - old);
                F_out[v] = fn;
                big = r > tol;
                rmax = fmaxf(rmax, r);
                edges += (unsigned long long)l;
                nchanged += big ? 1u : 0u;
                nrows += 1u;
            } else if (F_out != F_in) {
                F_out[v] = old;
            }
        }
        // this workgroup owns every word of the bitmap that covers its bin
        const unsigned long long b = __ballot(big);
        const int lane = lane_id();
        if ((lane == 0 || lane == 32) && d < size && v < n_words_end)
            moved_cur[v >> 5] = (unsigned int)(lane == 0 ? b : b >> 32);
    }
    rmax = wave_max(rmax);
    edges = wave_sum(edges);
    nchanged = wave_sum(nchanged);
    nrows = wave_sum(nrows);
    if (lane_id() == 0) {
        sm_r[threadIdx.x / kWave] = rmax;
        sm_e[threadIdx.x / kWave] = edges;
        sm_c[threadIdx.x / kWave] = nchanged;
        sm_n[threadIdx.x / kWave] = nrows;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < NW; ++i) {
            rmax = fmaxf(rmax, sm_r[i]);
            edges += sm_e[i];
            nchanged += sm_c[i];
            nrows += sm_n[i];
        }
        RoundPart* p = &ctr->part[bin & (kCtrLanes - 1)];
        if (rmax > 0.f) atomicMax(&p->resid_bits, __float_as_uint(rmax));
        if (edges) atomicAdd(&p->edges, edges);
        if (nchanged) atomicAdd(&p->changed, nchanged);
        if (nrows) atomicAdd(&p->rows_short, nrows);
    }
}

}  // namespace dynlp
