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

// Entry i of the stream (rows in vertex order): its row, its neighbour and its weight; and for every chunk of the
// stream the row of its first entry.  16 lanes per row.
__global__ void __launch_bounds__(kBlock) k_pb_expand(int64_t n, const RowMeta* __restrict__ meta,
                                                     const Edge* __restrict__ pool,
                                                     const unsigned int* __restrict__ first,
                                                     unsigned int* __restrict__ src, unsigned int* __restrict__ ecol,
                                                     float* __restrict__ ew, unsigned int* __restrict__ chunk_row0) {
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
        if ((a + j) % kPbChunk == 0) chunk_row0[(a + j) / kPbChunk] = (unsigned int)u;
    }
}

// What the scatter pass reads per entry, in one word: the entry's row as a 16-bit offset from the row of its
// chunk's first entry (high half) and its position in the sorted chunk (low half): 4 instead of 6 bytes per entry
// and round, and one load instead of two (two-byte loads alone, row offsets next to positions, were slower than the
// 32-bit rows: 1.72 against 1.59 ms per round on 250M entries).  A chunk whose 16,384 entries span 65,536 rows or
// more (long runs of vertices without entries) cannot be written that way: *too_wide is set and the scatter pass
// reads the 32-bit rows and the positions instead.
__global__ void __launch_bounds__(kBlock) k_pb_pack(const unsigned int* __restrict__ num_entries,
                                                   const unsigned int* __restrict__ src,
                                                   const unsigned short* __restrict__ lpos,
                                                   const unsigned int* __restrict__ chunk_row0,
                                                   unsigned int* __restrict__ packed, unsigned int* __restrict__ too_wide) {
    const int64_t E = (int64_t)*num_entries;
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= E) return;
    const unsigned int off = src[i] - chunk_row0[i / kPbChunk];
    packed[i] = (off << 16) | (unsigned int)lpos[i];
    if (off > 0xffffu) *too_wide = 1u;
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

// table[chunk][bin] -> entries of the bin in earlier chunks; table[chunks][bin] = bin_count[bin] = entries of the bin
// (so that the entries of (chunk, bin) are table[chunk + 1][bin] - table[chunk][bin] for every chunk).  A thread
// walks one bin's column (neighbouring threads read neighbouring words); the chunks are cut into kPbSegs segments
// so that no walk is longer than chunks / kPbSegs + kPbSegs steps: sums per segment, scan of the segment sums,
// running sums inside every segment.
constexpr int kPbSegs = 128;

__global__ void __launch_bounds__(kBlock) k_pb_seg_sums(int nbins, int chunks, const unsigned int* __restrict__ table,
                                                       unsigned int* __restrict__ seg) {
    const int b = blockIdx.x * kBlock + threadIdx.x;
    if (b >= nbins) return;
    const int per = (chunks + kPbSegs - 1) / kPbSegs;
    const int c0 = (int)blockIdx.y * per, c1 = min(chunks, c0 + per);
    unsigned int run = 0;
    for (int c = c0; c < c1; ++c) run += table[(size_t)c * nbins + b];
    seg[(size_t)blockIdx.y * nbins + b] = run;
}

__global__ void __launch_bounds__(kBlock) k_pb_seg_scan(int nbins, int chunks, unsigned int* __restrict__ seg,
                                                       unsigned int* __restrict__ table,
                                                       unsigned int* __restrict__ bin_count) {
    const int b = blockIdx.x * kBlock + threadIdx.x;
    if (b >= nbins) return;
    unsigned int run = 0;
    for (int s = 0; s < kPbSegs; ++s) {
        const size_t i = (size_t)s * nbins + b;
        const unsigned int t = seg[i];
        seg[i] = run;
        run += t;
    }
    table[(size_t)chunks * nbins + b] = run;
    bin_count[b] = run;
}

__global__ void __launch_bounds__(kBlock) k_pb_chunk_bases(int nbins, int chunks, const unsigned int* __restrict__ seg,
                                                          unsigned int* __restrict__ table) {
    const int b = blockIdx.x * kBlock + threadIdx.x;
    if (b >= nbins) return;
    const int per = (chunks + kPbSegs - 1) / kPbSegs;
    const int c0 = (int)blockIdx.y * per, c1 = min(chunks, c0 + per);
    unsigned int run = seg[(size_t)blockIdx.y * nbins + b];
    for (int c = c0; c < c1; ++c) {
        const size_t i = (size_t)c * nbins + b;
        const unsigned int t = table[i];
        table[i] = run;
        run += t;
    }
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
// entries with a slot) - 1, bin after bin: lpos[i] is entry i's position (entries whose receiver is never updated
// come last).  The slot behind a position needs no array: the positions of bin b start at the sum of the chunk's
// counts of the bins before b, which the scatter pass recomputes from the table.  The per-slot arrays get the
// receiver's offset in its bin and the raw weight; both are sorted by position in LDS first and leave as one run
// of consecutive words per (chunk, bin) (written entry by entry, each store was a memory transaction of its own
// and the pass took 17 ms instead of 4 on 250M entries).
constexpr int kPbPlaceThreads = 1024;

// The chunk's run starts from the table: loff[b] = entries of the chunk in bins < b (loff[nbins] = all with a slot),
// first_slot[b] = bin_off[b] + table[chunk][b].  All threads of a T-thread workgroup call it; nbins <= 4 * T.
template <int T>
__device__ inline void pb_chunk_runs(int nbins, const unsigned int* __restrict__ before,
                                     const unsigned int* __restrict__ bin_off, unsigned short* loff,
                                     unsigned int* first_slot, unsigned int* wave_tot) {
    constexpr int NW = T / kWave;
    const unsigned int* __restrict__ upto = before + nbins;
    const int per = (nbins + T - 1) / T;
    const int b0 = (int)threadIdx.x * per;
    unsigned int bef[4], cnt[4], off[4];
    unsigned int mine = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int b = b0 + q;
        const bool ok = q < per && b < nbins;
        bef[q] = ok ? before[b] : 0u;
        cnt[q] = ok ? upto[b] - bef[q] : 0u;
        off[q] = ok ? bin_off[b] : 0u;
        mine += cnt[q];
    }
    const unsigned int inc = wave_inclusive_scan(mine);
    if (lane_id() == kWave - 1) wave_tot[threadIdx.x / kWave] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned int run = 0;
        for (int i = 0; i < NW; ++i) {
            const unsigned int t = wave_tot[i];
            wave_tot[i] = run;
            run += t;
        }
        wave_tot[NW] = run;
    }
    __syncthreads();
    unsigned int run = inc - mine + wave_tot[threadIdx.x / kWave];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int b = b0 + q;
        if (q < per && b < nbins) {
            loff[b] = (unsigned short)run;  // a chunk holds 16,384 entries: fits 16 bits
            first_slot[b] = off[q] + bef[q];
            run += cnt[q];
        }
    }
    if (threadIdx.x == 0) loff[nbins] = (unsigned short)wave_tot[NW];
    __syncthreads();
}

__global__ void __launch_bounds__(kPbPlaceThreads) k_pb_place(const unsigned int* __restrict__ num_entries, int bin_bits,
                                                             int nbins, int lg_group,
                                                             const unsigned int* __restrict__ ecol,
                                                             const float* __restrict__ ew,
                                                             const unsigned int* __restrict__ upd,
                                                             const unsigned int* __restrict__ table,
                                                             const unsigned int* __restrict__ bin_off,
                                                             unsigned short* __restrict__ lpos,
                                                             unsigned short* __restrict__ dst, float* __restrict__ wn) {
    constexpr int T = kPbPlaceThreads;
    __shared__ float st_w[kPbChunk];
    __shared__ unsigned short st_d[kPbChunk];
    __shared__ unsigned int cur[kPbMaxBins];         // next free position of the bin
    __shared__ unsigned int first_slot[kPbMaxBins];
    __shared__ unsigned short loff[kPbMaxBins + 2];
    __shared__ unsigned int wave_tot[T / kWave + 1];
    __shared__ unsigned int none_next;
    pb_chunk_runs<T>(nbins, table + (size_t)blockIdx.x * nbins, bin_off, loff, first_slot, wave_tot);
    for (int b = threadIdx.x; b < nbins; b += T) cur[b] = loff[b];
    if (threadIdx.x == 0) none_next = loff[nbins];
    __syncthreads();
    const int64_t E = (int64_t)*num_entries;
    const int64_t base = (int64_t)blockIdx.x * kPbChunk;
    const unsigned int mask = (1u << bin_bits) - 1u;
    constexpr int UN = 4;
    for (int k0 = 0; k0 < kPbChunk; k0 += UN * T) {
        unsigned int v[UN];
        float w[UN];
#pragma unroll
        for (int q = 0; q < UN; ++q) {
            const int64_t i = base + k0 + q * T + threadIdx.x;
            v[q] = i < E ? ecol[i] : 0xffffffffu;
            w[q] = i < E ? ew[i] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < UN; ++q) {
            if (v[q] == 0xffffffffu) continue;
            unsigned int pos;
            if (pb_bit(upd, (int32_t)v[q])) {
                pos = atomicAdd(&cur[v[q] >> bin_bits], 1u);
                st_d[pos] = (unsigned short)(v[q] & mask);
                st_w[pos] = w[q];
            } else {
                pos = atomicAdd(&none_next, 1u);
            }
            lpos[base + k0 + q * T + threadIdx.x] = (unsigned short)pos;
        }
    }
    __syncthreads();
    const int gl = (int)threadIdx.x & ((1 << lg_group) - 1);
    const int G = 1 << lg_group;
    for (int b = (int)threadIdx.x >> lg_group; b < nbins; b += T >> lg_group) {
        const unsigned int lo = loff[b], hi = loff[b + 1];
        const unsigned int s0 = first_slot[b];
        for (unsigned int p = lo + gl; p < hi; p += G) {
            dst[s0 + (p - lo)] = st_d[p];
            wn[s0 + (p - lo)] = st_w[p];
        }
    }
}

// wn[s] /= deg[receiver]: one pass over the slots; kPbNormParts workgroups share a bin (the degrees of a bin's
// receivers are a window of at most 128 KB).
constexpr int kPbNormParts = 16;

__global__ void __launch_bounds__(kBlock) k_pb_normalise(int bin_bits, const unsigned int* __restrict__ bin_off,
                                                        const unsigned short* __restrict__ dst,
                                                        const float* __restrict__ deg, float* __restrict__ wn) {
    const unsigned int bin = blockIdx.x / kPbNormParts, part = blockIdx.x % kPbNormParts;
    const unsigned int lo = bin_off[bin], hi = bin_off[bin + 1];
    const int64_t first = (int64_t)bin << bin_bits;
    constexpr int UN = 4;
    for (unsigned int i0 = lo + part * (UN * kBlock); i0 < hi; i0 += kPbNormParts * UN * kBlock) {
        float w[UN], dg[UN];
#pragma unroll
        for (int q = 0; q < UN; ++q) {
            const unsigned int i = i0 + q * kBlock + threadIdx.x;
            w[q] = i < hi ? wn[i] : 0.f;
            dg[q] = i < hi ? deg[first + dst[i]] : 1.f;
        }
#pragma unroll
        for (int q = 0; q < UN; ++q) {
            const unsigned int i = i0 + q * kBlock + threadIdx.x;
            if (i < hi) wn[i] = w[q] / dg[q];
        }
    }
}

// Early-exit test shared by both passes: a round runs iff the previous one ran and moved at least one row.
__device__ inline bool pb_round_runs(const RoundCtr* __restrict__ prev) { return prev->executed && prev->any_moved != 0u; }

// Scatter pass, one workgroup per chunk: stage[lpos[i]] = F[src[i]] (sign bit: src[i] moved in the previous round)
// for the chunk's entries i; then the staged values of bin b (positions loff[b] .. loff[b + 1] - 1, loff = running
// sum of the chunk's entries per bin) go to the slots bin_off[b] + table[chunk][b] + 0, 1, ...: one run of
// consecutive words per (chunk, bin), written by 2^lg_group neighbouring lanes.  Also clears the counter slot and
// the moved-bitmap of the next round.
//
// NB: capacity of the per-bin LDS tables (nbins <= NB).  With NB = 2048 (67M vertices at 32,768 per bin) two
// workgroups share a CU; with kPbMaxBins one does.
//
// Workgroups reach the 8 XCDs round-robin by index; chunks are mapped so that XCD x works through the x-th
// eighth of the chunks in order: the runs that consecutive chunks write into a bin are neighbours, and a line
// shared by two runs is completed from the same L2.
constexpr int kPbScatterThreads = 1024;  // two workgroups of this size and 64 KB fill a CU (256 / 512 / 1024 threads:
                                         // 2.25 / 1.75 / 1.63 ms per round on 250M entries)

template <int NB, bool PACKED>
__global__ void __launch_bounds__(kPbScatterThreads) k_pb_scatter(const RoundCtr* __restrict__ prev,
                                                      const unsigned int* __restrict__ num_entries, unsigned int chunk0,
                                                      unsigned int chunks, int nbins, int lg_group,
                                                      const unsigned int* __restrict__ src,
                                                      const unsigned int* __restrict__ chunk_row0,
                                                      const unsigned short* __restrict__ lpos,
                                                      const unsigned int* __restrict__ table,
                                                      const unsigned int* __restrict__ bin_off, const float* F_in,
                                                      const unsigned int* __restrict__ moved_prev,
                                                      const unsigned int* __restrict__ moved_also,
                                                      unsigned int* __restrict__ moved_clear, unsigned int words,
                                                      unsigned int* __restrict__ val, RoundCtr* __restrict__ ctr_zero) {
    // chunks chunk0 .. chunk0 + chunks - 1; moved_prev (and moved_also, if not NULL): the bitmaps whose bits travel
    // with the labels ("the sender moved"); moved_clear / ctr_zero may be NULL
    __shared__ unsigned int stage[kPbChunk];
    __shared__ unsigned int first_slot[NB];    // slot of the chunk's first entry of the bin
    __shared__ unsigned short loff[NB + 2];    // its position in the sorted chunk; loff[nbins] = entries with a slot
    constexpr int T = kPbScatterThreads;
    constexpr int NW = T / kWave;
    __shared__ unsigned int wave_tot[NW + 1];
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
    if (!pb_round_runs(prev)) return;
    if (moved_clear)
        for (unsigned int w = blockIdx.x * T + threadIdx.x; w < words; w += gridDim.x * T) moved_clear[w] = 0u;
    const unsigned int per_xcd = (chunks + 7u) / 8u;
    const unsigned int local = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
    if ((blockIdx.x >> 3) >= per_xcd || local >= chunks) return;
    const unsigned int chunk = chunk0 + local;
    const int64_t E = (int64_t)*num_entries;
    const int64_t base = (int64_t)chunk * kPbChunk;
    pb_chunk_runs<T>(nbins, table + (size_t)chunk * nbins, bin_off, loff, first_slot, wave_tot);
    constexpr int UN = 4;
    // PACKED: src holds (row - row of the chunk's first entry) << 16 | position; else rows in src, positions in lpos
    const unsigned int row0 = PACKED ? chunk_row0[chunk] : 0u;
    for (int k0 = 0; k0 < kPbChunk; k0 += UN * T) {
        unsigned int u[UN], p[UN];
#pragma unroll
        for (int q = 0; q < UN; ++q) {
            const int64_t i = base + k0 + q * T + threadIdx.x;
            const bool ok = i < E;
            const unsigned int x = ok ? src[i] : 0u;
            u[q] = ok ? (PACKED ? row0 + (x >> 16) : x) : 0xffffffffu;
            p[q] = PACKED ? (x & 0xffffu) : (ok ? lpos[i] : 0u);
        }
#pragma unroll
        for (int q = 0; q < UN; ++q)
            if (u[q] != 0xffffffffu)
                stage[p[q]] = __float_as_uint(F_in[u[q]]) |
                              ((pb_bit(moved_prev, (int32_t)u[q]) || (moved_also && pb_bit(moved_also, (int32_t)u[q]))) ? 0x80000000u : 0u);
    }
    __syncthreads();
    const int gl = (int)threadIdx.x & ((1 << lg_group) - 1);
    const int G = 1 << lg_group;
    for (int b = (int)threadIdx.x >> lg_group; b < nbins; b += T >> lg_group) {
        const unsigned int lo = loff[b], hi = loff[b + 1];  // a full chunk of one bin: hi = 16384 fits 16 bits
        const unsigned int s0 = first_slot[b];
        for (unsigned int p = lo + gl; p < hi; p += G) val[s0 + (p - lo)] = stage[p];
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
    __shared__ unsigned int own[(1 << kPbMaxBinBits) / 32];
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
    const int64_t first = (int64_t)bin << bin_bits;
    const int64_t n_words_end = (n + 31) & ~(int64_t)31;
    for (int d = threadIdx.x; d < size; d += T) acc[d] = 0u;
    // nb: "a neighbour moved"; own: the receiver itself moved (it is in V_aff whatever its neighbours did, so the
    // stream below need not record their moves for it: while most rows move, hardly any flag is recorded)
    for (int d = threadIdx.x; d < size / 32; d += T) {
        nb[d] = 0u;
        const int64_t v0 = first + (int64_t)d * 32;
        own[d] = v0 < n_words_end ? moved_prev[v0 >> 5] : 0u;
    }
    __syncthreads();
    const unsigned int lo = bin_off[bin], hi = bin_off[bin + 1];
    // independent slot reads in flight per lane: 2 / 4 / 8 give 1.74 / 1.71 / 1.72 ms per round; two neighbouring slots
    // per lane with 4- and 8-byte loads instead of 2- and 4-byte ones: no gain either (1.52 against 1.51 ms)
    constexpr int UN = 4;
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
            if ((x[q] >> 31) && !((own[d[q] >> 5] >> (d[q] & 31u)) & 1u)) atomicOr(&nb[d[q] >> 5], 1u << (d[q] & 31u));
        }
    }
    __syncthreads();
    float rmax = 0.f;
    unsigned long long edges = 0;
    unsigned int nchanged = 0, nrows = 0;
    constexpr int UF = 4;  // receivers per lane whose reads are in flight together
    for (int d0 = 0; d0 < size; d0 += UF * T) {
        int l[UF];
        float old[UF];
#pragma unroll
        for (int q = 0; q < UF; ++q) {
            const int d = d0 + q * T + (int)threadIdx.x;  // d < size is uniform per wave: size is a multiple of 64
            const int64_t v = first + d;
            const bool ok = d < size && v < n;
            l[q] = ok ? len[v] : 0;
            old[q] = ok ? F_in[v] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < UF; ++q) {
            const int d = d0 + q * T + (int)threadIdx.x;
            const int64_t v = first + d;
            bool big = false;
            if (l[q] > 0) {
                const bool in_front = ((own[d >> 5] | nb[d >> 5]) >> (d & 31)) & 1u;
                if (in_front) {
                    const float fn = fminf((float)acc[d] * (1.0f / kPbUnit), 1.0f);
                    const float r = fabsf(fn - old[q]);
                    F_out[v] = fn;
                    big = r > tol;
                    rmax = fmaxf(rmax, r);
                    edges += (unsigned long long)l[q];
                    nchanged += big ? 1u : 0u;
                    nrows += 1u;
                } else if (F_out != F_in) {
                    F_out[v] = old[q];
                }
            }
            // this workgroup owns every word of the bitmap that covers its bin
            const unsigned long long b = __ballot(big);
            const int lane = lane_id();
            if ((lane == 0 || lane == 32) && d < size && v < n_words_end)
                moved_cur[v >> 5] = (unsigned int)(lane == 0 ? b : b >> 32);
        }
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
        if (nchanged) {
            atomicAdd(&p->changed, nchanged);
            ctr->any_moved = 1u;
        }
        if (nrows) atomicAdd(&p->rows_short, nrows);
    }
}

}  // namespace dynlp
