// Device-side building blocks shared by the DynLP kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dynlp {

constexpr int kWave = 64;
constexpr int kBlock = 256;       // threads per workgroup for every kernel here
constexpr int kRowAlign = 8;      // row capacities are multiples of 8 entries = 64 bytes
constexpr int kRing = 64;         // per-round counter slots
constexpr int kSortRegs = 8;      // appended entries per lane the in-register segment sort can hold (16 lanes per row)
constexpr int kAppendItems = 8;   // items per thread in kernels that append to a list (one counter atomic per 2,048 items)
constexpr int kInitChain = 4;     // hook/jump steps of the component search queued per host round trip

// One CSR entry of the slack pool: neighbour id and weight side by side, so that a single
// 8-byte load brings both.
struct __attribute__((aligned(8))) Edge {
    int32_t col;
    float w;
};

// Where row u lives in the pool: entries [off, off+len) are valid, [off+len, off+cap) is slack.
struct __attribute__((aligned(16))) RowMeta {
    int64_t off;
    int32_t len;
    int32_t cap;
};

// Counters one propagation round leaves for the host (one slot of a small ring).
// Rounds are launched in chains without a host round trip: the kernels of round t read the size of
// their frontier from the slot of round t-1 and leave their own results in the slot of round t.
//
// What every workgroup of the row update contributes (max change, rows moved, entries traversed) goes
// to one of kCtrLanes partial records, each in a cache line of its own: atomics on one address (or one
// line) run at about 1e8 per second, so 2,048 workgroups hitting one record would cost more than a
// whole sweep over a 100K-vertex graph.  The host folds the partial records into the header fields
// after copying a slot; on the device only the static stop rule needs the maximum over them.
constexpr int kCtrLanes = 32;

struct __attribute__((aligned(64))) RoundPart {
    unsigned int resid_bits;        // max change, float bits (non-negative floats order as uints)
    unsigned int changed;           // rows whose change exceeded tol
    unsigned long long edges;       // CSR entries traversed in short rows
    unsigned long long edges_long;  // CSR entries traversed in long rows
    unsigned int rows_short;        // rows updated, where the round itself decides which rows are in V_aff
    unsigned int rows_long;         // (k_row_update_pull); 0 otherwise
    unsigned int pad[8];
};

struct __attribute__((aligned(64))) RoundCtr {
    unsigned int next_count;   // short rows of V_aff for the next round (written by compaction)
    unsigned int next_long;    // long rows of V_aff for the next round
    unsigned int resid_bits;   // header copies of the folded partial records (filled on the host)
    unsigned int changed;
    unsigned long long edges;
    unsigned long long edges_long;
    unsigned int executed;     // 1 if the round updated anything (0: frontier was empty / already converged)
    unsigned int rows_short;   // the frontier this round worked on
    unsigned int rows_long;
    unsigned int any_moved;    // set (plain store of 1) by every workgroup that moved a row: "did the round move
                               // anything" for the next round without folding the partial records
    unsigned int pad[4];
    RoundPart part[kCtrLanes];
};

// Scalars of the insertion step and error reporting.
struct __attribute__((aligned(64))) BatchCtr {
    unsigned long long pool_tail;    // first free pool entry
    unsigned int touched;            // rows that receive at least one new entry
    unsigned int relocated;          // rows moved by the last insertion
    int err_code;                    // 0 = none; first validation error wins
    int err_pad;
    long long err_index;             // index of the offending item
    unsigned int init_count;         // first frontier: short rows
    unsigned int init_long;          //                 long rows
    unsigned long long scan_total;   // grand total of the last block-sum scan
    unsigned int upd_short;          // updatable vertices (unlabelled, >= 1 edge): short rows
    unsigned int upd_long;           //                                              long rows
    unsigned long long removed;      // CSR entries removed by the deletion step
    unsigned int sort_long;          // touched rows whose appended segment is sorted by a whole workgroup
    unsigned int sort_pad;
};

enum ValidationError : int {
    kErrNone = 0,
    kErrRowPtr = 1,
    kErrColRange = 2,
    kErrSelfLoop = 3,
    kErrWeight = 4,
    kErrSeedVertex = 5,
    kErrSeedClass = 6,
    kErrSeedConflict = 7,
    kErrEndpoint = 8,
    kErrRelabel = 9,
    kErrDeleted = 10,
};

__device__ inline void report_error(BatchCtr* bc, int code, long long index) {
    if (atomicCAS(&bc->err_code, 0, code) == 0) bc->err_index = index;
}

__device__ inline int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

// ---- wave / block reductions and scans --------------------------------------------------------
template <typename T>
__device__ inline T wave_sum(T v) {
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) v += __shfl_xor(v, d, kWave);
    return v;
}

__device__ inline float wave_max(float v) {
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) v = fmaxf(v, __shfl_xor(v, d, kWave));
    return v;
}

// Inclusive scan across the 64 lanes of a wave.
template <typename T>
__device__ inline T wave_inclusive_scan(T v) {
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        T o = __shfl_up(v, d, kWave);
        if (lane >= d) v += o;
    }
    return v;
}

// Exclusive scan over the kBlock threads of a workgroup; *total receives the block sum.
// smem must hold kBlock / kWave + 1 elements.  Contains barriers: call from all threads.
template <typename T>
__device__ inline T block_exclusive_scan(T v, T* smem, T* total) {
    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    constexpr int nw = kBlock / kWave;
    T inc = wave_inclusive_scan(v);
    if (lane == kWave - 1) smem[wave] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        T run = 0;
        for (int i = 0; i < nw; ++i) {
            T t = smem[i];
            smem[i] = run;
            run += t;
        }
        smem[nw] = run;
    }
    __syncthreads();
    T res = inc - v + smem[wave];
    *total = smem[nw];
    __syncthreads();
    return res;
}

// Append-slot reservation with one atomic per wave: lanes with pred get consecutive slots.
__device__ inline unsigned int wave_reserve(unsigned int* counter, bool pred) {
    const unsigned long long mask = __ballot(pred);
    const int lane = lane_id();
    unsigned int base = 0;
    const int leader = __ffsll((long long)mask) - 1;
    if (pred && lane == leader) base = atomicAdd(counter, (unsigned int)__popcll(mask));
    base = __shfl(base, leader < 0 ? 0 : leader, kWave);
    return base + (unsigned int)__popcll(mask & ((1ull << lane) - 1ull));
}

// Append-slot reservation with one atomic per workgroup: every thread asks for `count` consecutive
// slots (0 allowed) and gets the index of its first one.  smem must hold kBlock / kWave + 1 elements.
// Contains barriers: call from all threads of the workgroup.
__device__ inline unsigned int block_reserve(unsigned int* counter, unsigned int count, unsigned int* smem) {
    __shared__ unsigned int base;
    unsigned int total;
    const unsigned int ex = block_exclusive_scan<unsigned int>(count, smem, &total);
    if (threadIdx.x == 0) base = total ? atomicAdd(counter, total) : 0u;
    __syncthreads();
    const unsigned int r = base + ex;
    __syncthreads();
    return r;
}

// ---- small vectors of floats for row chunks ---------------------------------------------------
template <int V>
struct Vec {
    float v[V];
};

template <int V>
__device__ inline Vec<V> load_vec(const float* p);
template <>
__device__ inline Vec<1> load_vec<1>(const float* p) {
    Vec<1> r;
    r.v[0] = *p;
    return r;
}
template <>
__device__ inline Vec<2> load_vec<2>(const float* p) {
    float2 t = *reinterpret_cast<const float2*>(p);
    Vec<2> r;
    r.v[0] = t.x;
    r.v[1] = t.y;
    return r;
}
template <>
__device__ inline Vec<4> load_vec<4>(const float* p) {
    float4 t = *reinterpret_cast<const float4*>(p);
    Vec<4> r;
    r.v[0] = t.x;
    r.v[1] = t.y;
    r.v[2] = t.z;
    r.v[3] = t.w;
    return r;
}

template <int V>
__device__ inline void store_vec(float* p, const Vec<V>& a);
template <>
__device__ inline void store_vec<1>(float* p, const Vec<1>& a) {
    *p = a.v[0];
}
template <>
__device__ inline void store_vec<2>(float* p, const Vec<2>& a) {
    *reinterpret_cast<float2*>(p) = make_float2(a.v[0], a.v[1]);
}
template <>
__device__ inline void store_vec<4>(float* p, const Vec<4>& a) {
    *reinterpret_cast<float4*>(p) = make_float4(a.v[0], a.v[1], a.v[2], a.v[3]);
}

// ---- the same row chunks, read and written coherently across the whole device -------------------------------
// A kernel that runs several rounds (k_rounds_persistent) exchanges label rows between workgroups on different
// XCDs, each of which has an L2 of its own.  Relaxed atomic accesses at device scope are served from / written
// through to the point where the XCDs meet, so that a row written before a grid barrier is what every workgroup
// reads after it, without writing back and invalidating whole caches at every barrier (measured: that costs ten
// times the round itself).  A 16-byte chunk is two 8-byte accesses.
template <int V, bool COH>
__device__ inline Vec<V> load_row(const float* p) {
    if constexpr (!COH) {
        return load_vec<V>(p);
    } else if constexpr (V == 1) {
        Vec<1> r;
        r.v[0] = __uint_as_float(__hip_atomic_load(reinterpret_cast<const unsigned int*>(p), __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT));
        return r;
    } else {
        Vec<V> r;
#pragma unroll
        for (int k = 0; k < V; k += 2) {
            const unsigned long long q = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p + k),
                                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            r.v[k] = __uint_as_float((unsigned int)q);
            r.v[k + 1] = __uint_as_float((unsigned int)(q >> 32));
        }
        return r;
    }
}

template <int V, bool COH>
__device__ inline void store_row(float* p, const Vec<V>& a) {
    if constexpr (!COH) {
        store_vec<V>(p, a);
    } else if constexpr (V == 1) {
        __hip_atomic_store(reinterpret_cast<unsigned int*>(p), __float_as_uint(a.v[0]), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    } else {
#pragma unroll
        for (int k = 0; k < V; k += 2) {
            const unsigned long long q =
                (unsigned long long)__float_as_uint(a.v[k]) | ((unsigned long long)__float_as_uint(a.v[k + 1]) << 32);
            __hip_atomic_store(reinterpret_cast<unsigned long long*>(p + k), q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

}  // namespace dynlp
