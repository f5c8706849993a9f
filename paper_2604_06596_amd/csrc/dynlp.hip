// libdynlp: host side of the DynLP library (context, memory, launch sequencing, C ABI).
// Every step of the path runs in the kernels of dynlp_kernels.h; there is no CPU fallback.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <unordered_map>
#include <unordered_set>
#include <vector>

#include "dynlp.h"
#include "dynlp_kernels.h"
#include "dynlp_frontier.h"
#include "dynlp_components.h"
#include "dynlp_binned.h"

using namespace dynlp;

namespace {

thread_local std::string g_create_error;

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

int padded_classes(int C) {
    if (C <= 1) return 1;
    if (C <= 2) return 2;
    if (C <= 4) return 4;
    if (C <= 8) return 8;
    if (C <= 16) return 16;
    if (C <= 32) return 32;
    return 64;
}

const char* validation_message(int code) {
    switch (code) {
        case kErrRowPtr: return "row_ptr must start at 0, be non-decreasing and end at the entry count (row index %lld)";
        case kErrColRange: return "neighbour id out of range (entry %lld)";
        case kErrSelfLoop: return "self loop (item %lld)";
        case kErrWeight: return "weight must be finite and > 0 (item %lld)";
        case kErrSeedVertex: return "seed vertex out of range (seed %lld)";
        case kErrSeedClass: return "seed class out of range (seed %lld)";
        case kErrSeedConflict: return "one vertex listed with two different classes (seed %lld)";
        case kErrEndpoint: return "edge endpoint out of range (edge %lld)";
        case kErrRelabel: return "vertex is already a seed of another class (seed %lld)";
        case kErrDeleted: return "deleted vertex out of range (item %lld)";
        default: return "validation error %lld";
    }
}

using Clock = std::chrono::steady_clock;
inline float ms_since(Clock::time_point t0) {
    return std::chrono::duration<float, std::milli>(Clock::now() - t0).count();
}

}  // namespace

// Staging area of dynlp_get_labels_static: device memory that exists without any allocation call.  Every GPU
// the library runs on holds its own copy, at its own address, until the process ends.  In host code the name
// `scratch` is only a handle for hipGetSymbolAddress; kernels and copies take the resolved per-device address.
constexpr size_t kStaticScratchBytes = DYNLP_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};        // device address of `scratch` on each device, once resolved
hipError_t g_scratch_err[kMaxDevices] = {};   // what the resolution returned there

// Resolve the address of `scratch` on `device` (which must be the current device).  Once per device.
void resolve_static_scratch(int device) {
    if (device < 0 || device >= kMaxDevices) return;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device]) return;
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    g_scratch_err[device] = e;
    if (e == hipSuccess) g_scratch_ptr[device] = ptr;
    else (void)hipGetLastError();
}

}  // namespace

struct dynlp_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    bool dev_ptrs = false;
    float slack = 1.25f;
    bool time_kernels = false;
    int group_lanes = 0;
    std::unordered_set<void*> live;  // every device array handed out by dev_alloc and not yet freed: whatever an error
                                     // path left behind goes back to the allocator when the context is destroyed
    void* (*alloc_fn)(size_t, void*) = nullptr;
    void (*dealloc_fn)(void*, void*) = nullptr;
    void* alloc_user = nullptr;
    int num_cu = 256;

    int C = 0, CP = 0;
    int Cs = 0, coff = 0;  // stored columns and the class of stored column 0 (binary scalar layout: 1, 1)
    int64_t n = 0, n_cap = 0, flag_cap = 0;
    int64_t entries = 0;  // directed CSR entries stored
    RowMeta* meta = nullptr;
    Edge* pool = nullptr;
    int64_t pool_cap = 0, pool_tail = 0;
    float* F = nullptr;   // current labels, n_cap x CP
    float* F2 = nullptr;  // second buffer: ping-pong partner (static) / staging by queue position (dynamic)
    int32_t* seed_class = nullptr;
    uint8_t* flag = nullptr;
    int32_t* queue[3] = {nullptr, nullptr, nullptr};  // frontier storage: two parities + the list of all
                                                      // updatable vertices (see dynlp_frontier.h)
    int32_t* add_cnt = nullptr;
    float* deg = nullptr;
    unsigned int* moved[3] = {nullptr, nullptr, nullptr};  // 1 bit per vertex: "moved by > tol" of ping-pong rounds;
    int64_t moved_words = 0;                                // round t of a stretch reads t-1's, sets t's, clears t+1's

    int32_t* touched = nullptr;
    int64_t* reloc_off = nullptr;
    int32_t* he_rank = nullptr;  // per half-edge of the batch: its place among the entries appended to its row (or NULL)
    int64_t he_rank_cap = 0;
    int64_t touched_cap = 0;
    int32_t *b_eu = nullptr, *b_ev = nullptr, *b_sv = nullptr, *b_sc = nullptr;
    float* b_ew = nullptr;
    int64_t b_edge_cap = 0, b_seed_cap = 0;

    // pipelined ingest of host-resident batches (see ingest_edges)
    int64_t ingest_chunk = 0;            // edges per chunk
    hipStream_t copy_stream = nullptr;   // default priority, used only for the batch's host-to-device copies
    hipEvent_t ingest_ev[2] = {nullptr, nullptr};
    void* bounce[2] = {nullptr, nullptr};  // pinned staging for callers whose arrays are pageable, 12 bytes per chunk edge
    int64_t bounce_edges = 0;
    int ingest_chunks_last = 0, ingest_pinned_last = 0;  // what the last batch's ingest did (inspection)

    RoundCtr* ring = nullptr;  // kRing round slots + the start slot
    BatchCtr* bc = nullptr;
    RoundCtr* h_slot = nullptr;  // pinned, kRing slots
    unsigned int h_slot_start_long = 0;  // long rows among the updatable vertices of the running static solve
    BatchCtr* h_bc = nullptr;    // pinned

    int update_mode = DYNLP_UPDATE_SYNCHRONOUS;
    bool final_check = false;  // dynlp_set_final_check
    // several rounds per launch (k_rounds_persistent)
    int persist = 0;                  // option: 1 = whenever a stretch allows it, 0 / -1 = never
    unsigned int persist_spin = 1u << 20;  // polls a workgroup waits at the grid barrier before it gives up
    unsigned int* persist_ctl = nullptr;   // device: the words of the grid barrier (kBarWords; [1] = "given up")
    bool persist_failed = false;      // a launch was refused or a barrier was given up: ordinary launches from then on
    int persist_launches_last = 0, persist_aborts_last = 0;  // of the last batch (inspection)
    // binned rounds for scalar labels (dynlp_binned.h)
    int binned = 0;                 // option: 0 = automatic, -1 = never, 8..15 = always, with this many bin bits
    bool pb_built = false;          // the arrays below describe the graph as it stands
    int pb_bits = 0, pb_bins = 0;
    // per stored entry, rows in vertex order
    unsigned int* pb_src = nullptr;    // its row
    unsigned int* pb_sp = nullptr;     // row as an offset from pb_row0 of its chunk << 16 | pb_lpos: what the scatter pass reads
    unsigned int* pb_row0 = nullptr;   // per chunk: the row of its first entry; [chunk capacity]: "an offset needs > 16 bits"
    bool pb_packed_ok = false;
    unsigned short* pb_lpos = nullptr;  // its position in its chunk once sorted by slot
    float* pb_tmp = nullptr;           // build scratch: the entries' weights in stream order
    // per slot
    unsigned short* pb_dst = nullptr;
    float* pb_wn = nullptr;
    unsigned int* pb_val = nullptr;
    int64_t pb_ent_cap = 0;
    int pb_chunks = 0;
    // per vertex
    int32_t* pb_len = nullptr;
    unsigned int* pb_upd = nullptr;
    unsigned int* pb_first = nullptr;  // (+1) first entry of the row in the stream
    unsigned int* pb_block = nullptr;  // per kBlock vertices: scan scratch
    int64_t pb_vcap = 0;
    unsigned int* pb_bin = nullptr;  // bin_count | bin_off (+1), kPbMaxBins + 1 each
    unsigned int* pb_table = nullptr;  // entries per (chunk, bin) during the build
    int64_t pb_table_cap = 0;
    // in-place mode: the vertices are cut into pb_parts ranges of whole bins that are updated one after the other
    // within a round (range i: bins [pb_part_bin[i], pb_part_bin[i+1]), its rows' entries lie in chunks
    // [pb_part_chunk[i][0], pb_part_chunk[i][1]))
    int pb_parts = 1;
    int pb_part_bin[kPbMaxParts + 1] = {};
    int pb_part_chunk[kPbMaxParts][2] = {};
    // label initialisation of inserted vertices (dynlp_components.h)
    int init_mode = DYNLP_INIT_UNIFORM;
    float tau = 0.f;
    int32_t *cc_par = nullptr, *cc_dense = nullptr, *cc_comp = nullptr;
    unsigned int* cc_block = nullptr;
    int64_t cc_vcap = 0;
    int2* cc_kept = nullptr;
    int64_t cc_ecap = 0;
    double* cc_W = nullptr;
    int64_t cc_wcap = 0;
    InitCtr* cc_ctr = nullptr;  // device
    InitCtr* h_cc = nullptr;    // pinned
    hipEvent_t init_ev[2] = {nullptr, nullptr};
    dynlp_init_info last_init = {};  // of the last dynlp_apply_batch; vertices == 0: nothing to report

    float tol = 1e-4f;
    int32_t max_iter = 100000;
    std::vector<dynlp_round_info> log;  // one entry per round of the last solve / batch
    std::vector<hipEvent_t> events;   // pairs: events[2k], events[2k+1] bracket the k-th timed launch
    size_t events_used = 0;               // 2 x the number of timed spans
    size_t events_next = 0;               // events handed out (a span that directly follows another shares its event)
    std::vector<int> ev_first, ev_last;   // event indices of span k
    bool ev_adjacent = false;             // set by a caller: nothing was queued since the previous span was closed
    std::vector<int> ev_round, ev_count;  // rounds [ev_round[k], ev_round[k] + ev_count[k]) ran inside the k-th launch;
                                          // ev_round[k] < 0: the launch found nothing to do (queued past the end)
    hipEvent_t phase_ev[4] = {nullptr, nullptr, nullptr, nullptr};
    std::string err;
    bool poisoned = false;
};

namespace {

struct Fail {
    dynlp_status st;
};

#define HIPCHK(ctx, expr)                                                                              \
    do {                                                                                               \
        hipError_t _e = (expr);                                                                        \
        if (_e != hipSuccess) {                                                                        \
            (ctx)->err = std::string("HIP error: ") + hipGetErrorString(_e) + " in " #expr;            \
            (ctx)->poisoned = true;                                                                    \
            throw Fail{_e == hipErrorOutOfMemory ? DYNLP_ERR_OOM : DYNLP_ERR_DEVICE};                   \
        }                                                                                              \
    } while (0)

// NULL when the allocator has no memory left (nothing else changes).
void* dev_try_alloc(dynlp_ctx* c, size_t bytes) {
    if (bytes == 0) bytes = 256;
    void* p = nullptr;
    if (c->alloc_fn) {
        p = c->alloc_fn(bytes, c->alloc_user);
    } else if (hipMalloc(&p, bytes) != hipSuccess) {
        (void)hipGetLastError();
        p = nullptr;
    }
    if (p) c->live.insert(p);
    return p;
}

void* dev_alloc(dynlp_ctx* c, size_t bytes) {
    void* p = dev_try_alloc(c, bytes);
    if (!p) {
        c->err = "device allocation of " + std::to_string(bytes) + " bytes failed";
        c->poisoned = true;
        throw Fail{DYNLP_ERR_OOM};
    }
    return p;
}

void dev_free(dynlp_ctx* c, void* p) {
    if (!p || c->live.erase(p) == 0) return;  // only what dev_try_alloc handed out and has not been freed yet
    if (c->dealloc_fn) c->dealloc_fn(p, c->alloc_user);
    else (void)hipFree(p);
}

template <typename T>
T* dev_alloc_n(dynlp_ctx* c, int64_t count) {
    return static_cast<T*>(dev_alloc(c, (size_t)std::max<int64_t>(count, 1) * sizeof(T)));
}

// Temporary device array of a call that does not change the context: when the allocator has no memory the call
// ends with DYNLP_ERR_OOM and the context stays usable (nothing in it has changed); freed on scope exit.
struct SoftOom {};
template <typename T>
struct Temp {
    dynlp_ctx* c;
    T* ptr = nullptr;
    Temp(dynlp_ctx* ctx, int64_t count) : c(ctx) {
        ptr = static_cast<T*>(dev_try_alloc(c, (size_t)std::max<int64_t>(count, 1) * sizeof(T)));
        if (!ptr) {
            c->err = "device allocation of " + std::to_string((size_t)std::max<int64_t>(count, 1) * sizeof(T)) +
                     " bytes failed (the context is unchanged)";
            throw SoftOom{};
        }
    }
    ~Temp() { dev_free(c, ptr); }
    Temp(const Temp&) = delete;
    Temp& operator=(const Temp&) = delete;
    T* release() {
        T* p = ptr;
        ptr = nullptr;
        return p;
    }
};

inline unsigned int grid_for(int64_t items) { return (unsigned int)std::max<int64_t>(1, ceil_div(items, kBlock)); }

// A device array argument: either the caller's device pointer, or a temporary device copy of the
// caller's host array (freed by the destructor).
template <typename T>
struct DevIn {
    dynlp_ctx* c;
    const T* ptr = nullptr;
    T* owned = nullptr;
    DevIn(dynlp_ctx* ctx, const T* src, int64_t count) : c(ctx) {
        if (count <= 0 || !src) return;
        if (c->dev_ptrs) {
            ptr = src;
        } else {
            owned = dev_alloc_n<T>(c, count);
            HIPCHK(c, hipMemcpyAsync(owned, src, (size_t)count * sizeof(T), hipMemcpyHostToDevice, c->stream));
            ptr = owned;
        }
    }
    ~DevIn() {
        if (owned) {
            (void)hipStreamSynchronize(c->stream);
            dev_free(c, owned);
        }
    }
};

void read_bc(dynlp_ctx* c) {
    HIPCHK(c, hipMemcpyAsync(c->h_bc, c->bc, sizeof(BatchCtr), hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
}

void write_bc(dynlp_ctx* c) {
    HIPCHK(c, hipMemcpyAsync(c->bc, c->h_bc, sizeof(BatchCtr), hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
}

std::string format_validation(int code, long long index) {
    char buf[256];
    std::snprintf(buf, sizeof buf, validation_message(code), index);
    return buf;
}

// ---- vertex-indexed arrays --------------------------------------------------------------------
void alloc_vertex_arrays(dynlp_ctx* c, int64_t new_cap) {
    const int64_t old_n = c->n;
    const int64_t flag_cap = round_up(new_cap, 4 * kFlagsPerBlock) + 4 * kFlagsPerBlock;
    RowMeta* meta = dev_alloc_n<RowMeta>(c, new_cap);
    float* F = dev_alloc_n<float>(c, new_cap * c->CP);
    float* F2 = dev_alloc_n<float>(c, new_cap * c->CP);
    int32_t* sc = dev_alloc_n<int32_t>(c, new_cap);
    uint8_t* flag = dev_alloc_n<uint8_t>(c, flag_cap);
    int32_t* q0 = dev_alloc_n<int32_t>(c, new_cap);
    int32_t* q1 = dev_alloc_n<int32_t>(c, new_cap);
    int32_t* q2 = dev_alloc_n<int32_t>(c, new_cap);
    int32_t* add = dev_alloc_n<int32_t>(c, new_cap);
    float* deg = dev_alloc_n<float>(c, new_cap);
    const int64_t moved_words = (new_cap + 31) / 32 + 64;
    unsigned int* mv0 = dev_alloc_n<unsigned int>(c, moved_words);
    unsigned int* mv1 = dev_alloc_n<unsigned int>(c, moved_words);
    unsigned int* mv2 = dev_alloc_n<unsigned int>(c, moved_words);
    HIPCHK(c, hipMemsetAsync(flag, 0, (size_t)flag_cap, c->stream));
    HIPCHK(c, hipMemsetAsync(add, 0, (size_t)new_cap * sizeof(int32_t), c->stream));
    if (old_n > 0 && c->meta) {
        HIPCHK(c, hipMemcpyAsync(meta, c->meta, (size_t)old_n * sizeof(RowMeta), hipMemcpyDeviceToDevice, c->stream));
        HIPCHK(c, hipMemcpyAsync(F, c->F, (size_t)old_n * c->CP * sizeof(float), hipMemcpyDeviceToDevice, c->stream));
        HIPCHK(c, hipMemcpyAsync(sc, c->seed_class, (size_t)old_n * sizeof(int32_t), hipMemcpyDeviceToDevice, c->stream));
        HIPCHK(c, hipMemcpyAsync(deg, c->deg, (size_t)old_n * sizeof(float), hipMemcpyDeviceToDevice, c->stream));
    }
    HIPCHK(c, hipStreamSynchronize(c->stream));
    dev_free(c, c->meta);
    dev_free(c, c->F);
    dev_free(c, c->F2);
    dev_free(c, c->seed_class);
    dev_free(c, c->flag);
    dev_free(c, c->queue[0]);
    dev_free(c, c->queue[1]);
    dev_free(c, c->queue[2]);
    dev_free(c, c->add_cnt);
    dev_free(c, c->deg);
    dev_free(c, c->moved[0]);
    dev_free(c, c->moved[1]);
    dev_free(c, c->moved[2]);
    c->moved[0] = mv0;
    c->moved[1] = mv1;
    c->moved[2] = mv2;
    c->moved_words = moved_words;
    c->meta = meta;
    c->F = F;
    c->F2 = F2;
    c->seed_class = sc;
    c->flag = flag;
    c->queue[0] = q0;
    c->queue[1] = q1;
    c->queue[2] = q2;
    c->add_cnt = add;
    c->deg = deg;
    c->n_cap = new_cap;
    c->flag_cap = flag_cap;
}

void grow_pool(dynlp_ctx* c, int64_t min_cap) {
    int64_t new_cap = std::max<int64_t>(min_cap, c->pool_cap + c->pool_cap / 2);
    new_cap = round_up(new_cap, kRowAlign);
    Edge* p = dev_alloc_n<Edge>(c, new_cap);
    if (c->pool && c->pool_tail > 0)
        HIPCHK(c, hipMemcpyAsync(p, c->pool, (size_t)c->pool_tail * sizeof(Edge), hipMemcpyDeviceToDevice, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    dev_free(c, c->pool);
    c->pool = p;
    c->pool_cap = new_cap;
}

void ensure_batch_scratch(dynlp_ctx* c, int64_t m, int64_t s) {
    const int64_t need_t = std::max<int64_t>(1, std::min<int64_t>(2 * m, c->n_cap));
    if (need_t > c->touched_cap) {
        dev_free(c, c->touched);
        dev_free(c, c->reloc_off);
        c->touched = nullptr;
        c->reloc_off = nullptr;
        const int64_t cap = need_t + need_t / 2;
        c->touched = dev_alloc_n<int32_t>(c, cap);
        c->reloc_off = dev_alloc_n<int64_t>(c, cap);
        c->touched_cap = cap;
    }
    // optional (the insertion falls back to a second atomic per half-edge without it)
    if (2 * m > c->he_rank_cap) {
        dev_free(c, c->he_rank);
        c->he_rank_cap = 0;
        c->he_rank = static_cast<int32_t*>(dev_try_alloc(c, (size_t)(3 * m) * sizeof(int32_t)));
        if (c->he_rank) c->he_rank_cap = 3 * m;
    }
    if (!c->dev_ptrs) {
        if (m > c->b_edge_cap) {
            dev_free(c, c->b_eu);
            dev_free(c, c->b_ev);
            dev_free(c, c->b_ew);
            c->b_eu = c->b_ev = nullptr;
            c->b_ew = nullptr;
            const int64_t cap = m + m / 2;
            c->b_eu = dev_alloc_n<int32_t>(c, cap);
            c->b_ev = dev_alloc_n<int32_t>(c, cap);
            c->b_ew = dev_alloc_n<float>(c, cap);
            c->b_edge_cap = cap;
        }
        if (s > c->b_seed_cap) {
            dev_free(c, c->b_sv);
            dev_free(c, c->b_sc);
            c->b_sv = c->b_sc = nullptr;
            const int64_t cap = s + s / 2;
            c->b_sv = dev_alloc_n<int32_t>(c, cap);
            c->b_sc = dev_alloc_n<int32_t>(c, cap);
            c->b_seed_cap = cap;
        }
    }
}

// ---- pipelined ingest of a host-resident batch --------------------------------------------------------------
// The paper overlaps the transfer of a batch with the Step-1 kernels that only need what has already arrived.
// Here the graph lives on the device and only the batch's edge list crosses PCIe; for a batch of more than one
// chunk the list is sent chunk by chunk on a second stream while the main stream validates and counts the
// chunks that have landed (k_validate_edges, k_count_halfedges: the part of Step 1 that needs nothing but the
// chunk).  Caller arrays in pinned memory are sent as they are; pageable arrays go through two pinned staging
// buffers filled by a few host threads, so that filling chunk i+1 overlaps the transfer of chunk i.
constexpr int kIngestThreads = 6;

bool host_pointer_is_pinned(const void* p) {
    hipPointerAttribute_t a;
    if (hipPointerGetAttributes(&a, p) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return a.type == hipMemoryTypeHost;
}

void parallel_copy(void* dst, const void* src, size_t bytes) {
    if (bytes < ((size_t)4 << 20)) {
        std::memcpy(dst, src, bytes);
        return;
    }
    std::thread workers[kIngestThreads];
    const size_t slice = round_up((int64_t)ceil_div((int64_t)bytes, kIngestThreads), 4096);
    int started = 0;
    for (int t = 0; t < kIngestThreads; ++t) {
        const size_t lo = std::min(bytes, slice * t), hi = std::min(bytes, slice * (t + 1));
        if (hi <= lo) break;
        workers[t] = std::thread([=] { std::memcpy(static_cast<char*>(dst) + lo, static_cast<const char*>(src) + lo, hi - lo); });
        ++started;
    }
    for (int t = 0; t < started; ++t) workers[t].join();
}

// Copies eu / ev / ew (host) into c->b_eu / b_ev / b_ew and, per chunk, launches validation and counting on the
// main stream.  bc must have been reset on the main stream before the call.
void ingest_edges(dynlp_ctx* c, int64_t m, int64_t n_total, const int32_t* eu, const int32_t* ev, const float* ew) {
    const int64_t chunk = c->ingest_chunk;
    if (!c->copy_stream) {
        HIPCHK(c, hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking));
        for (hipEvent_t& e : c->ingest_ev) HIPCHK(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
    }
    const bool pinned = host_pointer_is_pinned(eu) && host_pointer_is_pinned(ev) && host_pointer_is_pinned(ew);
    if (!pinned && c->bounce_edges < chunk) {
        for (void*& b : c->bounce) {
            if (b) (void)hipHostFree(b);
            b = nullptr;
        }
        c->bounce_edges = 0;
        for (void*& b : c->bounce) HIPCHK(c, hipHostMalloc(&b, (size_t)chunk * 12, hipHostMallocDefault));
        c->bounce_edges = chunk;
    }
    // the copies must not start before earlier work on the main stream that still reads the device buffers is done
    // (there is none: the previous call ended with a synchronisation), nor before bc has been reset
    HIPCHK(c, hipEventRecord(c->ingest_ev[0], c->stream));
    HIPCHK(c, hipStreamWaitEvent(c->copy_stream, c->ingest_ev[0], 0));
    int chunks = 0;
    bool slot_used[2] = {false, false};
    for (int64_t off = 0; off < m; off += chunk, ++chunks) {
        const int64_t mc = std::min(chunk, m - off);
        const int slot = chunks & 1;
        const int32_t *s_eu = eu + off, *s_ev = ev + off;
        const float* s_ew = ew + off;
        if (!pinned) {
            if (slot_used[slot]) HIPCHK(c, hipEventSynchronize(c->ingest_ev[slot]));  // its last transfer has left the buffer
            char* b = static_cast<char*>(c->bounce[slot]);
            parallel_copy(b, s_eu, (size_t)mc * 4);
            parallel_copy(b + (size_t)chunk * 4, s_ev, (size_t)mc * 4);
            parallel_copy(b + (size_t)chunk * 8, s_ew, (size_t)mc * 4);
            s_eu = reinterpret_cast<const int32_t*>(b);
            s_ev = reinterpret_cast<const int32_t*>(b + (size_t)chunk * 4);
            s_ew = reinterpret_cast<const float*>(b + (size_t)chunk * 8);
        }
        HIPCHK(c, hipMemcpyAsync(c->b_eu + off, s_eu, (size_t)mc * 4, hipMemcpyHostToDevice, c->copy_stream));
        HIPCHK(c, hipMemcpyAsync(c->b_ev + off, s_ev, (size_t)mc * 4, hipMemcpyHostToDevice, c->copy_stream));
        HIPCHK(c, hipMemcpyAsync(c->b_ew + off, s_ew, (size_t)mc * 4, hipMemcpyHostToDevice, c->copy_stream));
        HIPCHK(c, hipEventRecord(c->ingest_ev[slot], c->copy_stream));
        slot_used[slot] = true;
        HIPCHK(c, hipStreamWaitEvent(c->stream, c->ingest_ev[slot], 0));
        hipLaunchKernelGGL(k_validate_edges, dim3(grid_for(mc)), dim3(kBlock), 0, c->stream, mc, n_total, c->b_eu + off,
                           c->b_ev + off, c->b_ew + off, c->bc, off);
        hipLaunchKernelGGL(k_count_halfedges, dim3(grid_for(ceil_div(2 * mc, kAppendItems))), dim3(kBlock), 0, c->stream, mc,
                           n_total, c->b_eu + off, c->b_ev + off, c->add_cnt, c->touched, c->bc,
                           c->he_rank ? c->he_rank + off : nullptr, c->he_rank ? c->he_rank + m + off : nullptr);
        HIPCHK(c, hipGetLastError());
    }
    c->ingest_chunks_last = chunks;
    c->ingest_pinned_last = pinned ? 1 : 0;
}

// ---- frontier launches ---------------------------------------------------------------------------
int lanes_per_neighbour(int CP) { return CP >= 4 ? CP / 4 : 1; }

int choose_group(const dynlp_ctx* c, double avg_len) {
    const int lpn = lanes_per_neighbour(c->CP);
    if (c->group_lanes) return std::max(c->group_lanes, lpn);
    // Measured on MI355X (1M-vertex graph, mean row length 20, C = 4 .. 50): 16 lanes per row is the
    // fastest or within 2% of it for every padded class count; wider groups only pay off when the
    // typical row fills several 16-entry chunks.
    int g = 16;
    // rows of a few entries with one to four label columns (50M vertices of degree 5, one column: 6.2 / 6.3 / 6.5 ms
    // per round over all rows with 4 / 8 / 16 lanes): narrow groups leave fewer lanes idle
    if (avg_len < 8.0 && c->CP <= 4) g = 4;
    if (avg_len >= 96.0) g = 32;
    if (avg_len >= 384.0) g = 64;
    return std::max(g, lpn);
}

// One propagation round's frontier lives in the array of one parity: short rows from the front,
// long rows from the back.  Its size is only on the device (the previous round's counter slot).
struct Frontier {
    int32_t* front = nullptr;
    int32_t* back = nullptr;
    unsigned int ns = 0, nl = 0;  // only meaningful for lists whose size the host has read
    unsigned int size() const { return ns + nl; }
};

Frontier frontier_of(dynlp_ctx* c, int parity, unsigned int ns = 0, unsigned int nl = 0) {
    Frontier f;
    f.front = c->queue[parity];
    f.back = c->queue[parity] + (c->n_cap - 1);
    f.ns = ns;
    f.nl = nl;
    return f;
}

struct UpdateArgs {
    const RoundCtr* prev;  // slot that holds the size of the frontier to work on
    int static_stop;       // 0: frontier round; 1: static sweep; 2: static sweep that checks prev's stop rule
    const float* F_in;
    float* F_out;
    unsigned int* moved;  // "moved by > tol" bitmap of this round (ping-pong rounds), NULL otherwise
    float tol;
    RoundCtr* ctr;
    RoundCtr* ctr_zero;
    int64_t rows_bound;  // upper bounds of the frontier size and of its long rows (they size the grid)
    int64_t long_bound;
    int by_vertex = 0;  // flag-marking rounds only: kRowByVertex (write row u of F_out instead of staging by position), kRowLazy
};

template <int CP, int G, bool STAGED>
void launch_update_inst(dynlp_ctx* c, const Frontier& f, const UpdateArgs& a) {
    constexpr int GPB = kBlock / G;
    const int64_t cap = (int64_t)c->num_cu * 32;
    const unsigned int short_blocks = (unsigned int)std::max<int64_t>(1, std::min<int64_t>(ceil_div(a.rows_bound, GPB), cap));
    const unsigned int long_max = (unsigned int)std::min<int64_t>(a.long_bound, cap / 2);
    unsigned int stop_bits;
    std::memcpy(&stop_bits, &a.tol, sizeof stop_bits);
    hipLaunchKernelGGL((k_row_update<CP, G, STAGED>), dim3(short_blocks + long_max), dim3(kBlock), 0, c->stream, a.prev,
                       a.static_stop, stop_bits, long_max, f.front, f.back, c->meta, c->pool, a.F_in, a.F_out, a.by_vertex, c->flag, a.moved, a.tol,
                       a.ctr, a.ctr_zero);
}

template <int CP, bool STAGED>
void launch_update_cp(dynlp_ctx* c, int G, const Frontier& f, const UpdateArgs& a) {
    constexpr int LPN = CP >= 4 ? CP / 4 : 1;
#define DYNLP_CASE(GV)                                              \
    case GV:                                                        \
        if constexpr (GV >= LPN) {                                  \
            launch_update_inst<CP, GV, STAGED>(c, f, a);            \
            return;                                                 \
        }                                                           \
        break;
    switch (G) {
        DYNLP_CASE(4)
        DYNLP_CASE(8)
        DYNLP_CASE(16)
        DYNLP_CASE(32)
        DYNLP_CASE(64)
        default: break;
    }
#undef DYNLP_CASE
    launch_update_inst<CP, 64, STAGED>(c, f, a);
}

// With kernel timing on, two events bracket every row-update launch; `round` / `count` say which rounds it runs.
// A launch that directly follows the previous timed launch (c->ev_adjacent, set by the caller for this one call)
// takes that launch's closing event as its opening one: an event record costs a few microseconds on the stream,
// which shows once a round takes 40 of them.
hipEvent_t open_timed_span(dynlp_ctx* c, int round, int count) {
    const bool adjacent = c->ev_adjacent && c->events_used > 0;
    c->ev_adjacent = false;
    if (!c->time_kernels) return nullptr;
    while (c->events.size() < c->events_next + 2) {
        hipEvent_t e;
        HIPCHK(c, hipEventCreate(&e));
        c->events.push_back(e);
    }
    const size_t k = c->events_used / 2;
    if (c->ev_round.size() <= k) {
        c->ev_round.resize(k + 1);
        c->ev_count.resize(k + 1);
        c->ev_first.resize(k + 1);
        c->ev_last.resize(k + 1);
    }
    c->ev_round[k] = round;
    c->ev_count[k] = count;
    c->events_used += 2;
    if (adjacent) {
        c->ev_first[k] = c->ev_last[k - 1];
    } else {
        c->ev_first[k] = (int)c->events_next;
        HIPCHK(c, hipEventRecord(c->events[c->events_next++], c->stream));
    }
    c->ev_last[k] = (int)c->events_next;
    return c->events[c->events_next++];
}

void close_timed_span(dynlp_ctx* c, hipEvent_t e1) {
    if (e1) HIPCHK(c, hipEventRecord(e1, c->stream));
}

void reset_timed_spans(dynlp_ctx* c) {
    c->events_used = 0;
    c->events_next = 0;
    c->ev_adjacent = false;
}

// After a chain has been read back: launches of rounds >= first_unexecuted did nothing.
void trim_timed_spans(dynlp_ctx* c, size_t first_pair, int first_unexecuted) {
    for (size_t k = first_pair; k < c->events_used / 2; ++k) {
        if (c->ev_round[k] >= first_unexecuted) c->ev_round[k] = -1;
        else c->ev_count[k] = std::min(c->ev_count[k], first_unexecuted - c->ev_round[k]);
    }
}

// Row update of one frontier: one launch (long rows and short rows share the grid).  With kernel
// timing on, two events per round bracket it.
template <bool STAGED>
void launch_update(dynlp_ctx* c, int G, const Frontier& f, const UpdateArgs& a, int round) {
    hipEvent_t e1 = open_timed_span(c, round, 1);
    switch (c->CP) {
        case 1: launch_update_cp<1, STAGED>(c, G, f, a); break;
        case 2: launch_update_cp<2, STAGED>(c, G, f, a); break;
        case 4: launch_update_cp<4, STAGED>(c, G, f, a); break;
        case 8: launch_update_cp<8, STAGED>(c, G, f, a); break;
        case 16: launch_update_cp<16, STAGED>(c, G, f, a); break;
        case 32: launch_update_cp<32, STAGED>(c, G, f, a); break;
        default: launch_update_cp<64, STAGED>(c, G, f, a); break;
    }
    HIPCHK(c, hipGetLastError());
    close_timed_span(c, e1);
}

// A ping-pong round that evaluates V_aff membership itself (k_row_update_pull): `universe` lists every
// updatable vertex, moved_prev / moved_cur / moved_clear are the bitmaps of the previous, this and the next round.
struct PullRoundArgs {
    const RoundCtr* prev;
    const float* F_in;
    float* F_out;
    const unsigned int* moved_prev;
    unsigned int* moved_cur;
    unsigned int* moved_clear;
    float tol;
    RoundCtr* ctr;
    RoundCtr* ctr_zero;
};

template <int CP, int G>
void launch_update_pull_inst(dynlp_ctx* c, const Frontier& universe, const PullRoundArgs& a) {
    constexpr int GPB = kBlock / G;
    const int64_t cap = (int64_t)c->num_cu * 32;
    const unsigned int short_blocks =
        (unsigned int)std::max<int64_t>(1, std::min<int64_t>(ceil_div((int64_t)universe.ns, GPB), cap));
    const unsigned int long_max = (unsigned int)std::min<int64_t>((int64_t)universe.nl, cap / 2);
    hipLaunchKernelGGL((k_row_update_pull<CP, G>), dim3(short_blocks + long_max), dim3(kBlock), 0, c->stream, a.prev, long_max,
                       universe.front, universe.back, universe.ns, universe.nl, c->meta, c->pool, a.F_in, a.F_out,
                       a.moved_prev, a.moved_cur, a.moved_clear, (unsigned int)c->moved_words, a.tol, a.ctr, a.ctr_zero);
}

template <int CP>
void launch_update_pull_cp(dynlp_ctx* c, int G, const Frontier& universe, const PullRoundArgs& a) {
    constexpr int LPN = CP >= 4 ? CP / 4 : 1;
#define DYNLP_CASE(GV)                                              \
    case GV:                                                        \
        if constexpr (GV >= LPN) {                                  \
            launch_update_pull_inst<CP, GV>(c, universe, a);        \
            return;                                                 \
        }                                                           \
        break;
    switch (G) {
        DYNLP_CASE(4)
        DYNLP_CASE(8)
        DYNLP_CASE(16)
        DYNLP_CASE(32)
        DYNLP_CASE(64)
        default: break;
    }
#undef DYNLP_CASE
    launch_update_pull_inst<CP, 64>(c, universe, a);
}

void launch_update_pull(dynlp_ctx* c, int G, const Frontier& universe, const PullRoundArgs& a, int round) {
    hipEvent_t e1 = open_timed_span(c, round, 1);
    switch (c->CP) {
        case 1: launch_update_pull_cp<1>(c, G, universe, a); break;
        case 2: launch_update_pull_cp<2>(c, G, universe, a); break;
        case 4: launch_update_pull_cp<4>(c, G, universe, a); break;
        case 8: launch_update_pull_cp<8>(c, G, universe, a); break;
        case 16: launch_update_pull_cp<16>(c, G, universe, a); break;
        case 32: launch_update_pull_cp<32>(c, G, universe, a); break;
        default: launch_update_pull_cp<64>(c, G, universe, a); break;
    }
    HIPCHK(c, hipGetLastError());
    close_timed_span(c, e1);
}

// ---- several rounds per launch (k_rounds_persistent) ------------------------------------------------------------
// Whether a stretch of rounds that evaluate V_aff themselves should run many rounds per launch.  Off unless asked
// for: measured on MI355X on a 100,000-vertex kNN graph (10 classes, 2M stored entries) a round inside such a
// launch takes 68 us against 52-58 us as a launch of its own - the label rows that cross the barrier must be
// read past the per-XCD L2s, and a workgroup runs its share of a round's rows one after the other - so that the
// fewer rounds an in-place batch then needs (370 against 500: fewer rows in flight at once) only tie the batch at
// 26 ms, and a synchronous batch loses (46 against 38 ms).
constexpr int kPersistRounds = 32;  // rounds per launch; the ring of counter slots holds kRing = 64

bool persistent_rounds_pay(const dynlp_ctx* c, const Frontier& universe) {
    (void)universe;
    return c->persist > 0 && !c->persist_failed;
}

template <int CP, int G>
bool launch_persistent_inst(dynlp_ctx* c, const Frontier& universe, PersistArgs& a) {
    constexpr int GPB = kBlock / G;
    static int per_cu_cache[64] = {};  // by device ordinal
    int& per_cu = per_cu_cache[c->device & 63];
    if (per_cu == 0) {
        int v = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&v, k_rounds_persistent<CP, G>, kBlock, 0) != hipSuccess || v < 1) {
            (void)hipGetLastError();
            return false;
        }
        per_cu = v;
    }
    const int64_t resident = std::min<int64_t>((int64_t)c->num_cu * per_cu, (int64_t)kBarGroup * kBarMaxGroups);
    const int64_t want = std::max<int64_t>(1, ceil_div((int64_t)universe.ns, GPB)) + std::min<int64_t>(universe.nl, resident / 2);
    const unsigned int grid = (unsigned int)std::min<int64_t>(want, resident);
    a.long_blocks_max = (unsigned int)std::min<int64_t>((int64_t)universe.nl, std::max<int64_t>(grid / 2, universe.ns ? 0 : grid));
    if (a.long_blocks_max >= grid && universe.ns > 0) a.long_blocks_max = grid - 1;
    a.ngroups = (unsigned int)ceil_div((int64_t)grid, (int64_t)kBarGroup);
    // an ordinary launch of a grid that fits the device all at once (a cooperative launch costs milliseconds here);
    // should the grid not be resident as a whole for any reason, the bounded wait at the barrier ends the launch
    hipLaunchKernelGGL((k_rounds_persistent<CP, G>), dim3(grid), dim3(kBlock), 0, c->stream, a);
    if (hipGetLastError() != hipSuccess) return false;
    return true;
}

template <int CP>
bool launch_persistent_cp(dynlp_ctx* c, int G, const Frontier& universe, PersistArgs& a) {
    constexpr int LPN = CP >= 4 ? CP / 4 : 1;
#define DYNLP_CASE(GV)                                                  \
    case GV:                                                            \
        if constexpr (GV >= LPN) return launch_persistent_inst<CP, GV>(c, universe, a); \
        break;
    switch (G) {
        DYNLP_CASE(4)
        DYNLP_CASE(8)
        DYNLP_CASE(16)
        DYNLP_CASE(32)
        DYNLP_CASE(64)
        default: break;
    }
#undef DYNLP_CASE
    return launch_persistent_inst<CP, 64>(c, universe, a);
}

// Rounds [round, round + count) of a stretch in one launch.  False: the launch was refused (nothing was queued);
// the caller queues ordinary rounds instead.
bool launch_persistent(dynlp_ctx* c, int G, const Frontier& universe, PersistArgs& a, int round) {
    HIPCHK(c, hipMemsetAsync(c->persist_ctl, 0, kBarWords * sizeof(unsigned int), c->stream));
    hipEvent_t e1 = open_timed_span(c, round, a.rounds);
    bool ok;
    switch (c->CP) {
        case 1: ok = launch_persistent_cp<1>(c, G, universe, a); break;
        case 2: ok = launch_persistent_cp<2>(c, G, universe, a); break;
        case 4: ok = launch_persistent_cp<4>(c, G, universe, a); break;
        case 8: ok = launch_persistent_cp<8>(c, G, universe, a); break;
        case 16: ok = launch_persistent_cp<16>(c, G, universe, a); break;
        case 32: ok = launch_persistent_cp<32>(c, G, universe, a); break;
        default: ok = launch_persistent_cp<64>(c, G, universe, a); break;
    }
    close_timed_span(c, e1);
    if (!ok && c->time_kernels) c->ev_round[c->events_used / 2 - 1] = -1;
    return ok;
}

// ---- binned rounds (dynlp_binned.h) -----------------------------------------------------------------
// Whether a stretch of rounds over nearly all vertices should run as scatter + gather passes: one label column,
// and either forced by the option or labels well beyond one XCD's L2 (4 MB = 1M labels), so that the ordinary
// round's gathers miss it.  Measured on MI355X, binary labels, one round over all rows, binned against ordinary
// (and whole batches, in-place mode): 50M vertices of degree 5: 1.64 against 6.2 ms (957 against 1,463 ms); 10M
// vertices of mean degree 38: 2.26 against 6.2 ms (1,095 against 1,510 ms); 5M of degree 5: 0.18 against 0.64 ms
// (105 against 164 ms); 2M of degree 5: 0.10 against 0.28 ms (77 against 101 ms); 1M of mean degree 20 (4 MB of
// labels): 0.29 against 0.24 ms, and whole batches twice as slow because the binned rounds are Jacobi rounds
// also in in-place mode.
bool binned_rounds_pay(const dynlp_ctx* c, const Frontier& universe) {
    if (c->CP != 1 || c->binned < 0) return false;
    if (ceil_div(c->n, (int64_t)1 << (c->binned > 0 ? c->binned : kPbMaxBinBits)) > kPbMaxBins) return false;
    if (c->entries >= ((int64_t)1 << 32) - 2 * kPbChunk) return false;  // slots and stream positions are 32-bit
    if (c->binned > 0) return true;
    return universe.size() >= (2u << 20);
}

// Free every array of the binned rounds.
void free_binned(dynlp_ctx* c) {
    void* all[] = {c->pb_src, c->pb_sp, c->pb_row0, c->pb_lpos, c->pb_tmp, c->pb_dst, c->pb_wn, c->pb_val,
                   c->pb_len, c->pb_upd, c->pb_first, c->pb_block, c->pb_bin, c->pb_table};
    for (void* q : all) dev_free(c, q);
    c->pb_src = c->pb_val = c->pb_upd = c->pb_first = c->pb_block = c->pb_bin = c->pb_table = c->pb_row0 = c->pb_sp = nullptr;
    c->pb_lpos = c->pb_dst = nullptr;
    c->pb_tmp = c->pb_wn = nullptr;
    c->pb_len = nullptr;
    c->pb_ent_cap = c->pb_vcap = c->pb_table_cap = 0;
    c->pb_built = false;
}

template <typename T>
bool try_alloc_n(dynlp_ctx* c, T*& p, int64_t count) {
    p = static_cast<T*>(dev_try_alloc(c, (size_t)std::max<int64_t>(count, 1) * sizeof(T)));
    return p != nullptr;
}

// Lanes that share one (chunk, bin) run when it is written out (log2): the mean run length rounded up to a power of
// two, 16 .. 1,024 (8 / 16 / 32 lanes on runs of 11 entries: 1.79 / 1.71 / 1.73 ms per round).
int pb_run_lanes(int nbins) {
    int lg = 4;
    while (lg < 10 && ((int64_t)nbins << lg) < kPbChunk) ++lg;
    return lg;
}

// Slots, per-slot receiver offsets and normalised weights for the graph as it stands.  False (and nothing kept)
// when the arrays cannot be allocated: the caller then runs ordinary rounds.
bool build_binned(dynlp_ctx* c) {
    const int bits = c->binned > 0 ? c->binned : kPbMaxBinBits;
    const int nbins = (int)ceil_div(std::max<int64_t>(c->n, 1), (int64_t)1 << bits);
    const int chunks = (int)ceil_div(std::max<int64_t>(c->entries, 1), kPbChunk);
    bool ok = true;
    if ((int64_t)chunks * kPbChunk > c->pb_ent_cap) {
        void* old[] = {c->pb_src, c->pb_sp, c->pb_row0, c->pb_lpos, c->pb_tmp, c->pb_dst, c->pb_wn, c->pb_val};
        for (void* q : old) dev_free(c, q);
        c->pb_src = c->pb_val = c->pb_row0 = c->pb_sp = nullptr;
        c->pb_lpos = c->pb_dst = nullptr;
        c->pb_tmp = c->pb_wn = nullptr;
        c->pb_ent_cap = 0;
        const int64_t cap = round_up(c->entries + c->entries / 8 + 1, kPbChunk);
        ok = try_alloc_n(c, c->pb_src, cap) && try_alloc_n(c, c->pb_sp, cap) &&
             try_alloc_n(c, c->pb_row0, cap / kPbChunk + 1) && try_alloc_n(c, c->pb_lpos, cap) &&
             try_alloc_n(c, c->pb_tmp, cap) && try_alloc_n(c, c->pb_dst, cap) && try_alloc_n(c, c->pb_wn, cap) &&
             try_alloc_n(c, c->pb_val, cap);
        if (ok) c->pb_ent_cap = cap;
    }
    if (ok && c->n > c->pb_vcap) {
        void* old[] = {c->pb_len, c->pb_upd, c->pb_first, c->pb_block};
        for (void* q : old) dev_free(c, q);
        c->pb_len = nullptr;
        c->pb_upd = c->pb_first = c->pb_block = nullptr;
        c->pb_vcap = 0;
        ok = try_alloc_n(c, c->pb_len, c->n_cap) && try_alloc_n(c, c->pb_upd, c->n_cap / 32 + 64) &&
             try_alloc_n(c, c->pb_first, c->n_cap + 1) && try_alloc_n(c, c->pb_block, c->n_cap / kBlock + 2);
        if (ok) c->pb_vcap = c->n_cap;
    }
    if (ok && !c->pb_bin) ok = try_alloc_n(c, c->pb_bin, 2 * (kPbMaxBins + 1));
    // rows 0 .. chunks of the table, then kPbSegs rows of segment sums
    if (ok && ((int64_t)chunks + 1 + kPbSegs) * nbins > c->pb_table_cap) {
        dev_free(c, c->pb_table);
        c->pb_table = nullptr;
        c->pb_table_cap = 0;
        const int64_t cap = ((int64_t)chunks + 1 + kPbSegs) * nbins + (int64_t)chunks * nbins / 8;
        ok = try_alloc_n(c, c->pb_table, cap);
        if (ok) c->pb_table_cap = cap;
    }
    if (!ok) {
        free_binned(c);
        return false;
    }
    unsigned int* bin_count = c->pb_bin;
    unsigned int* bin_off = c->pb_bin + (kPbMaxBins + 1);
    const unsigned int* num_entries = c->pb_first + c->n;
    const unsigned int vblocks = grid_for(c->n);
    hipLaunchKernelGGL(k_pb_receivers, dim3(grid_for(round_up(c->n, 64))), dim3(kBlock), 0, c->stream, c->n, c->meta,
                       c->seed_class, c->pb_len, c->pb_upd);
    hipLaunchKernelGGL(k_pb_row_blocks, dim3(vblocks), dim3(kBlock), 0, c->stream, c->n, c->meta, c->pb_block);
    hipLaunchKernelGGL(k_pb_scan_blocks, dim3(1), dim3(kBlock), 0, c->stream, (int64_t)vblocks, c->pb_block);
    hipLaunchKernelGGL(k_pb_row_first, dim3(vblocks), dim3(kBlock), 0, c->stream, c->n, c->meta, c->pb_block, c->pb_first);
    HIPCHK(c, hipGetLastError());
    // every array above is sized from the host's count of stored entries: it must be the device's
    unsigned int device_entries = 0;
    HIPCHK(c, hipMemcpyAsync(&device_entries, num_entries, sizeof device_entries, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    if ((int64_t)device_entries != c->entries) {
        c->err = "internal error: the stored rows hold " + std::to_string(device_entries) + " entries, the context counts " +
                 std::to_string(c->entries);
        c->poisoned = true;
        throw Fail{DYNLP_ERR_STATE};
    }
    unsigned int* ecol = c->pb_val;  // scratch until the first scatter pass overwrites it
    unsigned int* too_wide = c->pb_row0 + c->pb_ent_cap / kPbChunk;  // the word after the last chunk's
    HIPCHK(c, hipMemsetAsync(too_wide, 0, sizeof(unsigned int), c->stream));
    hipLaunchKernelGGL(k_pb_expand, dim3(grid_for(c->n * 16)), dim3(kBlock), 0, c->stream, c->n, c->meta, c->pool, c->pb_first,
                       c->pb_src, ecol, c->pb_tmp, c->pb_row0);

    hipLaunchKernelGGL(k_pb_count, dim3(chunks), dim3(kBlock), 0, c->stream, num_entries, bits, nbins, ecol, c->pb_upd,
                       c->pb_table);
    unsigned int* seg = c->pb_table + ((size_t)chunks + 1) * nbins;
    const dim3 col_grid(grid_for(nbins), kPbSegs);
    hipLaunchKernelGGL(k_pb_seg_sums, col_grid, dim3(kBlock), 0, c->stream, nbins, chunks, c->pb_table, seg);
    hipLaunchKernelGGL(k_pb_seg_scan, dim3(grid_for(nbins)), dim3(kBlock), 0, c->stream, nbins, chunks, seg, c->pb_table,
                       bin_count);
    hipLaunchKernelGGL(k_pb_chunk_bases, col_grid, dim3(kBlock), 0, c->stream, nbins, chunks, seg, c->pb_table);
    hipLaunchKernelGGL(k_pb_offsets, dim3(1), dim3(kBlock), 0, c->stream, nbins, bin_count, bin_off);
    hipLaunchKernelGGL(k_pb_place, dim3(chunks), dim3(kPbPlaceThreads), 0, c->stream, num_entries, bits, nbins,
                       pb_run_lanes(nbins), ecol, c->pb_tmp, c->pb_upd, c->pb_table, bin_off, c->pb_lpos, c->pb_dst, c->pb_wn);
    hipLaunchKernelGGL(k_pb_pack, dim3(grid_for(c->entries)), dim3(kBlock), 0, c->stream, num_entries, c->pb_src, c->pb_lpos,
                       c->pb_row0, c->pb_sp, too_wide);
    hipLaunchKernelGGL(k_pb_normalise, dim3(nbins * kPbNormParts), dim3(kBlock), 0, c->stream, bits, bin_off, c->pb_dst,
                       c->deg, c->pb_wn);
    HIPCHK(c, hipGetLastError());
    c->pb_bits = bits;
    c->pb_bins = nbins;
    c->pb_chunks = chunks;
    // In-place mode: the round updates the vertices range by range (whole bins each) and publishes a range's new
    // labels before the next range is updated, which is what "a new row replaces the old one at once" means for
    // two streaming passes; fewer rounds are needed than with all ranges updated from the round-start labels.
    // Synchronous mode: one range.
    // A range's gather runs one workgroup per bin and one workgroup fills a CU: ranges of about one bin per CU keep
    // the whole chip busy (50M vertices, 1,526 bins, in-place batch: 2 / 4 / 6 / 8 / 16 ranges give 802 / 681 / 616 /
    // 622 / 731 ms against 956 ms with one).  Graphs with fewer bins than CUs keep one range.
    const int want_parts = c->update_mode == DYNLP_UPDATE_IN_PLACE ? (int)ceil_div(nbins, std::max(1, c->num_cu)) : 1;
    const int parts = std::max(1, std::min({want_parts, kPbMaxParts, nbins}));
    c->pb_parts = parts;
    std::vector<unsigned int> first_at(parts + 1, 0u);
    unsigned int wide = 1;
    HIPCHK(c, hipMemcpyAsync(&wide, too_wide, sizeof wide, hipMemcpyDeviceToHost, c->stream));
    for (int i = 0; i <= parts; ++i) {
        const int b = (int)(((int64_t)nbins * i) / parts);
        c->pb_part_bin[i] = b;
        const int64_t v = std::min<int64_t>(c->n, (int64_t)b << bits);
        HIPCHK(c, hipMemcpyAsync(&first_at[i], c->pb_first + v, sizeof(unsigned int), hipMemcpyDeviceToHost, c->stream));
    }
    HIPCHK(c, hipStreamSynchronize(c->stream));
    for (int i = 0; i < parts; ++i) {
        c->pb_part_chunk[i][0] = (int)(first_at[i] / kPbChunk);
        c->pb_part_chunk[i][1] = (int)std::min<int64_t>(chunks, ceil_div((int64_t)first_at[i + 1], kPbChunk));
        if (first_at[i + 1] == first_at[i]) c->pb_part_chunk[i][1] = c->pb_part_chunk[i][0];  // no entries: nothing to publish
    }
    c->pb_packed_ok = wide == 0;
    c->pb_built = true;
    return true;
}

// One binned round: scatter pass + gather pass (arguments as for the fused round).
void launch_pb_scatter(dynlp_ctx* c, const RoundCtr* prev, int chunk0, int nchunks, const float* F, const unsigned int* bits,
                       unsigned int* moved_clear, RoundCtr* ctr_zero, const unsigned int* bits_also = nullptr) {
    if (nchunks <= 0 && !ctr_zero && !moved_clear) return;
    const int lg = pb_run_lanes(c->pb_bins);
    const dim3 grid(8 * (unsigned int)std::max<int64_t>(1, ceil_div(nchunks, 8)));
    const unsigned int* bin_off = c->pb_bin + (kPbMaxBins + 1);
#define DYNLP_SCATTER(NB, PACKED, SRC)                                                                                     \
    hipLaunchKernelGGL((k_pb_scatter<NB, PACKED>), grid, dim3(kPbScatterThreads), 0, c->stream, prev, c->pb_first + c->n,      \
                       (unsigned int)chunk0, (unsigned int)std::max(nchunks, 0), c->pb_bins, lg, SRC, c->pb_row0, c->pb_lpos,  \
                       c->pb_table, bin_off, F, bits, bits_also, moved_clear, (unsigned int)c->moved_words, c->pb_val,         \
                       ctr_zero)
    if (c->pb_bins <= 2048 && c->pb_packed_ok) DYNLP_SCATTER(2048, true, c->pb_sp);
    else if (c->pb_bins <= 2048) DYNLP_SCATTER(2048, false, c->pb_src);
    else if (c->pb_packed_ok) DYNLP_SCATTER(kPbMaxBins, true, c->pb_sp);
    else DYNLP_SCATTER(kPbMaxBins, false, c->pb_src);
#undef DYNLP_SCATTER
}

// One binned round (arguments as for the fused round).  `first_of_stretch`: no binned round has run since the slots
// were last brought up to date with the labels.
// One range (synchronous mode): scatter all labels, gather all bins: a Jacobi round.
// Several ranges (in-place mode): the slots are kept up to date between rounds; the round updates range after range,
// each gather followed by the scatter that publishes the range's new labels, so that later ranges of the same round
// already read them.  A published label carries "the sender moved in this round or in the previous one": ranges that
// come later in this round and ranges that come earlier in the next one both have to learn that it moved, and each
// sees only one publication.  V_aff of a round is then a superset of Alg. 2's (a row may be updated once more than
// needed), as with any in-place round that reads rows the same round has already replaced.
void launch_pb_gather(dynlp_ctx* c, const PullRoundArgs& a, int b0, int b1) {
    const unsigned int* bin_off = c->pb_bin + (kPbMaxBins + 1);
    hipLaunchKernelGGL(k_pb_gather, dim3(b1 - b0), dim3(kPbGatherThreads), 0, c->stream, a.prev, c->n, c->pb_bits, (unsigned int)b0,
                       bin_off, c->pb_dst, c->pb_wn, c->pb_val, c->pb_len, a.F_in, a.F_out, a.moved_prev, a.moved_cur, a.tol,
                       a.ctr);
}

void launch_binned_round(dynlp_ctx* c, const PullRoundArgs& a, int round, bool first_of_stretch) {
    hipEvent_t e1 = open_timed_span(c, round, 1);
    if (c->pb_parts <= 1) {
        launch_pb_scatter(c, a.prev, 0, c->pb_chunks, a.F_in, a.moved_prev, a.moved_clear, a.ctr_zero);
        launch_pb_gather(c, a, 0, c->pb_bins);
    } else {
        // bring every slot up to date once (labels and "moved in the previous round" bits); this launch also clears
        // the next round's counter slot and bitmap, as the first launch of every round does
        if (first_of_stretch) launch_pb_scatter(c, a.prev, 0, c->pb_chunks, a.F_in, a.moved_prev, nullptr, nullptr);
        for (int i = 0; i < c->pb_parts; ++i) {
            const int b0 = c->pb_part_bin[i], b1 = c->pb_part_bin[i + 1];
            if (i == 0) launch_pb_scatter(c, a.prev, 0, 0, a.F_in, a.moved_prev, a.moved_clear, a.ctr_zero);
            if (b1 > b0) launch_pb_gather(c, a, b0, b1);
            launch_pb_scatter(c, a.prev, c->pb_part_chunk[i][0], c->pb_part_chunk[i][1] - c->pb_part_chunk[i][0], a.F_out,
                              a.moved_cur, nullptr, nullptr, a.moved_prev);
        }
    }
    HIPCHK(c, hipGetLastError());
    close_timed_span(c, e1);
}

// Resolve the per-round events into the round log; returns the summed device time of all
// row-update launches.
float collect_kernel_ms(dynlp_ctx* c) {
    float total = 0.f;
    for (size_t k = 0; 2 * k + 1 < c->events_used; ++k) {
        float a = 0.f;
        (void)hipEventElapsedTime(&a, c->events[c->ev_first[k]], c->events[c->ev_last[k]]);
        total += a;
        const int first = c->ev_round[k];
        if (first < 0) continue;
        const int last = std::min<int>(first + c->ev_count[k], (int)c->log.size());
        for (int t = first; t < last; ++t) c->log[t].ms_update += a / (float)std::max(1, last - first);
    }
    reset_timed_spans(c);
    return total;
}

dynlp_round_info round_info(const RoundCtr& r, int kind, int G) {
    dynlp_round_info ri;
    std::memset(&ri, 0, sizeof ri);
    ri.rows_short = r.rows_short;
    ri.rows_long = r.rows_long;
    ri.entries_short = (int64_t)r.edges;
    ri.entries_long = (int64_t)r.edges_long;
    std::memcpy(&ri.max_delta, &r.resid_bits, sizeof(float));
    ri.rows_moved = r.changed;
    ri.staged = kind;
    ri.group_lanes = G;
    return ri;
}

// flag bytes (or, with all_rows, every updatable vertex) -> frontier `out`; the two counts land in
// *count_short / *count_long, which must be zero beforehand.
void launch_compact(dynlp_ctx* c, const Frontier& out, unsigned int* count_short, unsigned int* count_long,
                    int all_rows) {
    if (c->n >= (16 << 20)) {
        const unsigned int blocks = (unsigned int)ceil_div(std::max<int64_t>(c->n, 1), 4 * kFlagsPerBlock);
        hipLaunchKernelGGL(k_compact<4>, dim3(blocks), dim3(kBlock), 0, c->stream, (unsigned int)c->n, c->flag, c->seed_class,
                           c->meta, all_rows, out.front, out.back, count_short, count_long);
    } else {
        const unsigned int blocks = (unsigned int)ceil_div(std::max<int64_t>(c->n, 1), kFlagsPerBlock);
        hipLaunchKernelGGL(k_compact<1>, dim3(blocks), dim3(kBlock), 0, c->stream, (unsigned int)c->n, c->flag, c->seed_class,
                           c->meta, all_rows, out.front, out.back, count_short, count_long);
    }
    HIPCHK(c, hipGetLastError());
}

void launch_commit(dynlp_ctx* c, const Frontier& f, const RoundCtr* prev, int64_t rows_bound) {
    const int64_t items = rows_bound * (c->CP >= 4 ? c->CP / 4 : c->CP);
    const unsigned int blocks = (unsigned int)std::max<int64_t>(1, std::min<int64_t>(ceil_div(items, kBlock), (int64_t)c->num_cu * 8));
    hipLaunchKernelGGL(k_commit, dim3(blocks), dim3(kBlock), 0, c->stream, prev, f.front, f.back, c->F2, c->F, c->CP);
    HIPCHK(c, hipGetLastError());
}

// Pull the next V_aff out of the round's "moved" bitmap straight into the frontier `out` (its counts go to
// *count_short / *count_long, zero beforehand); F_new holds the rows just written, F_old the round-start
// rows; `universe` lists every updatable vertex.
template <int SUB>
void launch_pull_frontier_inst(dynlp_ctx* c, const Frontier& universe, const unsigned int* moved, unsigned int* moved_next,
                               const float* F_new, float* F_old, const Frontier& out, unsigned int* count_short,
                               unsigned int* count_long) {
    const int64_t cap = (int64_t)c->num_cu * 8;
    const unsigned int long_blocks =
        (unsigned int)std::min<int64_t>(ceil_div(universe.nl, (kBlock / kWave) * SUB), cap / 2);
    const unsigned int short_blocks =
        (unsigned int)std::max<int64_t>(1, std::min<int64_t>(ceil_div(universe.ns, kBlock * SUB), cap));
    hipLaunchKernelGGL(k_pull_frontier<SUB>, dim3(long_blocks + short_blocks), dim3(kBlock), 0, c->stream, universe.ns,
                       universe.nl, long_blocks, universe.front, universe.back, moved, moved_next, (unsigned int)c->moved_words,
                       F_new, F_old, c->CP,
                       c->meta, c->pool, out.front, out.back, count_short, count_long);
    HIPCHK(c, hipGetLastError());
}

void launch_pull_frontier(dynlp_ctx* c, const Frontier& universe, double avg_len, const unsigned int* moved,
                          unsigned int* moved_next, const float* F_new, float* F_old, const Frontier& out,
                          unsigned int* count_short, unsigned int* count_long) {
    // measured: 10M vertices of mean degree 38 want the large chunks (0.21 vs 0.41 ms per round), 1M vertices of
    // degree 20, 100K vertices and 50M vertices of degree 5 the small ones
    if (universe.size() >= (2u << 20) && avg_len >= 16.0)
        launch_pull_frontier_inst<16>(c, universe, moved, moved_next, F_new, F_old, out, count_short, count_long);
    else
        launch_pull_frontier_inst<4>(c, universe, moved, moved_next, F_new, F_old, out, count_short, count_long);
}

// Whether a ping-pong stretch should run rounds that evaluate V_aff themselves (k_row_update_pull) rather than
// pairs of row update and pull.  The fused round saves the pull's pass over the graph but puts the membership test
// (one more dependent look-up for rows that did not move themselves) in front of every row's gathers.
bool fused_rounds_pay(const dynlp_ctx* c, double avg_len) {
    // Measured on MI355X, batches of 1% new vertices, whole batch, fused against separate: 1M vertices of mean
    // degree 20 with 10 / 32 / 64 classes 68 / 78 / 112 ms against 80 / 89 / 138 ms; 2M vertices of mean degree 38
    // with 10 / 20 classes 611 / 766 ms against 660 / 827 ms; 50M vertices of degree 5, one column, 1.54 s against
    // 1.89 s; but 10M vertices of mean degree 38 with 50 classes 14.9 ms per round against 14.3 + 0.2 ms.  The
    // rule below separates the two groups by the bytes a row's update reads.
    return avg_len * (double)(c->CP * 4 + 8) < 8192.0;
}

// Ping-pong stretches begin when V_aff holds at least kDenseEnter of the updatable vertices and end
// when it falls below kDenseLeave (the pull over all updatable vertices stops paying off).
constexpr double kDenseEnter = 0.90, kDenseLeave = 0.75;
// A binned round costs the same whatever the size of V_aff (two streams over the whole graph), about a quarter of an
// ordinary round over all rows, and a flag-marking round over a third of the rows already costs more: such stretches
// begin and end at smaller V_aff.  50M-vertex random graph, one batch, enter / leave at 0.50 / 0.35 against 0.35 / 0.20:
// synchronous 762 -> 738 ms, with supernode initialisation 367 -> 342 ms, in place with it 332 -> 270 ms (in place
// from uniform rows V_aff collapses within one chain of rounds and nothing changes); 0.20 / 0.10 is no better.
constexpr double kBinnedEnter = 0.35, kBinnedLeave = 0.20;

// The ping-pong partner must agree with F on every row a full sweep does not write (seeds,
// isolated vertices) before it can receive one.
void sync_partner(dynlp_ctx* c) {
    if (c->n > 0)
        HIPCHK(c, hipMemcpyAsync(c->F2, c->F, (size_t)c->n * c->CP * sizeof(float), hipMemcpyDeviceToDevice, c->stream));
}

void zero_ring(dynlp_ctx* c) {
    HIPCHK(c, hipMemsetAsync(c->ring, 0, sizeof(RoundCtr) * (kRing + 1), c->stream));
}

// Slot of round t; round -1 is the start slot that holds the size of the first frontier.
RoundCtr* slot_of(dynlp_ctx* c, int t) { return t < 0 ? c->ring + kRing : c->ring + (t % kRing); }

// Fold a copied slot's partial records into its header fields.
void fold_slot(RoundCtr& r) {
    r.resid_bits = 0;
    r.changed = 0;
    r.edges = 0;
    r.edges_long = 0;
    for (const RoundPart& p : r.part) {
        r.rows_short += p.rows_short;  // only rounds that find their own V_aff count rows here
        r.rows_long += p.rows_long;
        r.resid_bits = std::max(r.resid_bits, p.resid_bits);
        r.changed += p.changed;
        r.edges += p.edges;
        r.edges_long += p.edges_long;
    }
}

// Copy the slots of rounds [t0, t0 + count) to the host (count <= kRing) and wait for them.
void read_slots(dynlp_ctx* c, int t0, int count) {
    for (int i = 0; i < count;) {
        const int idx = (t0 + i) % kRing;
        const int run = std::min(count - i, kRing - idx);
        HIPCHK(c, hipMemcpyAsync(c->h_slot + i, c->ring + idx, sizeof(RoundCtr) * (size_t)run, hipMemcpyDeviceToHost, c->stream));
        i += run;
    }
    HIPCHK(c, hipStreamSynchronize(c->stream));
    for (int i = 0; i < count; ++i) fold_slot(c->h_slot[i]);
}

// Rounds queued per host round trip.
constexpr int kChain = 8;

void read_slots_start(dynlp_ctx* c) {
    HIPCHK(c, hipMemcpyAsync(c->h_slot, c->ring + kRing, sizeof(RoundCtr), hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
}

void fill_stats_zero(dynlp_stats* s) {
    if (s) std::memset(s, 0, sizeof *s);
}

// ---- host-side argument checks (host-pointer mode): errors without touching the device ----------
bool host_check_seeds(std::string& err, int64_t s, int64_t n_total, int C, const int32_t* sv, const int32_t* sc) {
    std::unordered_map<int32_t, int32_t> seen;
    for (int64_t i = 0; i < s; ++i) {
        if (sv[i] < 0 || sv[i] >= n_total) { err = format_validation(kErrSeedVertex, i); return false; }
        if (sc[i] < 0 || sc[i] >= C) { err = format_validation(kErrSeedClass, i); return false; }
        auto it = seen.find(sv[i]);
        if (it != seen.end() && it->second != sc[i]) { err = format_validation(kErrSeedConflict, i); return false; }
        seen[sv[i]] = sc[i];
    }
    return true;
}

bool host_check_csr(std::string& err, int64_t n, const int64_t* row_ptr, const int32_t* col, const float* w) {
    if (row_ptr[0] != 0) { err = format_validation(kErrRowPtr, 0); return false; }
    for (int64_t u = 0; u < n; ++u)
        if (row_ptr[u + 1] < row_ptr[u]) { err = format_validation(kErrRowPtr, u); return false; }
    for (int64_t u = 0; u < n; ++u) {
        for (int64_t j = row_ptr[u]; j < row_ptr[u + 1]; ++j) {
            if (col[j] < 0 || col[j] >= n) { err = format_validation(kErrColRange, j); return false; }
            if (col[j] == u) { err = format_validation(kErrSelfLoop, j); return false; }
            if (!(w[j] > 0.f) || !std::isfinite(w[j])) { err = format_validation(kErrWeight, j); return false; }
        }
    }
    return true;
}

bool host_check_edges(std::string& err, int64_t m, int64_t n_total, const int32_t* eu, const int32_t* ev,
                      const float* ew) {
    for (int64_t i = 0; i < m; ++i) {
        if (eu[i] < 0 || eu[i] >= n_total || ev[i] < 0 || ev[i] >= n_total) {
            err = format_validation(kErrEndpoint, i);
            return false;
        }
        if (eu[i] == ev[i]) { err = format_validation(kErrSelfLoop, i); return false; }
        if (!(ew[i] > 0.f) || !std::isfinite(ew[i])) { err = format_validation(kErrWeight, i); return false; }
    }
    return true;
}

void destroy_ctx(dynlp_ctx* c) {
    if (!c) return;
    (void)hipSetDevice(c->device);
    if (c->stream || c->meta) (void)hipStreamSynchronize(c->stream);
    void* ptrs[] = {c->meta, c->pool, c->F, c->F2, c->seed_class, c->flag, c->queue[0], c->queue[1], c->queue[2], c->moved[0], c->moved[1], c->moved[2], c->add_cnt,
                    c->deg, c->touched, c->reloc_off, c->he_rank, c->b_eu, c->b_ev, c->b_ew, c->b_sv, c->b_sc,
                    c->cc_par, c->cc_dense, c->cc_comp, c->cc_block, c->cc_kept, c->cc_W,
                    c->pb_src, c->pb_sp, c->pb_row0, c->pb_lpos, c->pb_tmp, c->pb_dst, c->pb_wn, c->pb_val, c->pb_len, c->pb_upd,
                    c->pb_first, c->pb_block, c->pb_bin, c->pb_table};
    for (void* p : ptrs) dev_free(c, p);
    const std::vector<void*> left(c->live.begin(), c->live.end());  // arrays an interrupted call never got to free
    for (void* p : left) dev_free(c, p);
    dev_free(c, c->cc_ctr);
    if (c->h_cc) (void)hipHostFree(c->h_cc);
    for (hipEvent_t e : c->init_ev)
        if (e) (void)hipEventDestroy(e);
    dev_free(c, c->ring);
    dev_free(c, c->bc);
    dev_free(c, c->persist_ctl);
    for (void* b : c->bounce)
        if (b) (void)hipHostFree(b);
    for (hipEvent_t e : c->ingest_ev)
        if (e) (void)hipEventDestroy(e);
    if (c->copy_stream) (void)hipStreamDestroy(c->copy_stream);
    if (c->h_slot) (void)hipHostFree(c->h_slot);
    if (c->h_bc) (void)hipHostFree(c->h_bc);
    for (hipEvent_t e : c->events) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->phase_ev)
        if (e) (void)hipEventDestroy(e);
    delete c;
}

// ---- Alg. 2 Step 1 (components of the sparsified batch-internal graph) + Step 2 (supernode rows) ----
void ensure_init_scratch(dynlp_ctx* c, int64_t k, int64_t m) {
    if (!c->cc_ctr) {
        c->cc_ctr = static_cast<InitCtr*>(dev_alloc(c, sizeof(InitCtr)));
        HIPCHK(c, hipHostMalloc(reinterpret_cast<void**>(&c->h_cc), sizeof(InitCtr), hipHostMallocDefault));
        for (hipEvent_t& e : c->init_ev) HIPCHK(c, hipEventCreate(&e));
    }
    if (k > c->cc_vcap) {
        dev_free(c, c->cc_par);
        dev_free(c, c->cc_dense);
        dev_free(c, c->cc_comp);
        dev_free(c, c->cc_block);
        c->cc_par = c->cc_dense = c->cc_comp = nullptr;
        c->cc_block = nullptr;
        c->cc_vcap = 0;
        const int64_t cap = k + k / 2;
        c->cc_par = dev_alloc_n<int32_t>(c, cap);
        c->cc_dense = dev_alloc_n<int32_t>(c, cap);
        c->cc_comp = dev_alloc_n<int32_t>(c, cap);
        c->cc_block = dev_alloc_n<unsigned int>(c, ceil_div(cap, kBlock) + 1);
        c->cc_vcap = cap;
    }
    if (m > c->cc_ecap) {
        dev_free(c, c->cc_kept);
        c->cc_kept = nullptr;
        c->cc_ecap = 0;
        const int64_t cap = m + m / 2;
        c->cc_kept = dev_alloc_n<int2>(c, cap);
        c->cc_ecap = cap;
    }
}

void read_init_ctr(dynlp_ctx* c) {
    HIPCHK(c, hipMemcpyAsync(c->h_cc, c->cc_ctr, sizeof(InitCtr), hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
}

// Runs after the batch's edges are in the CSR and its seeds are clamped; rewrites only the rows of
// the k inserted, unlabelled vertices n0 .. n0+k-1.
void run_supernode_init(dynlp_ctx* c, int64_t n0, int64_t k, int64_t m, const int32_t* d_eu, const int32_t* d_ev,
                        const float* d_ew) {
    ensure_init_scratch(c, k, m);
    HIPCHK(c, hipEventRecord(c->init_ev[0], c->stream));
    HIPCHK(c, hipMemsetAsync(c->cc_ctr, 0, sizeof(InitCtr), c->stream));
    hipLaunchKernelGGL(k_cc_reset, dim3(grid_for(k)), dim3(kBlock), 0, c->stream, k, c->cc_par);
    if (m > 0)
        hipLaunchKernelGGL(k_cc_filter, dim3(grid_for(ceil_div(m, kAppendItems))), dim3(kBlock), 0, c->stream, m, n0, k, d_eu, d_ev, d_ew, c->tau,
                           c->cc_kept, c->cc_ctr);
    const unsigned int hook_grid = (unsigned int)std::min<int64_t>(grid_for(std::max<int64_t>(m, 1)), (int64_t)c->num_cu * 8);
    int hook_steps = 0;
    for (;;) {
        for (int i = 0; i < kInitChain; ++i) {
            hipLaunchKernelGGL(k_cc_hook, dim3(hook_grid), dim3(kBlock), 0, c->stream, i, c->cc_kept, c->cc_par, c->cc_ctr);
            hipLaunchKernelGGL(k_cc_jump, dim3(grid_for(k)), dim3(kBlock), 0, c->stream, i, k, c->cc_par, c->cc_ctr);
        }
        HIPCHK(c, hipGetLastError());
        read_init_ctr(c);
        for (int i = 0; i < kInitChain; ++i)
            if (i == 0 || c->h_cc->changed[i - 1]) ++hook_steps;
        if (c->h_cc->changed[kInitChain - 1] == 0u) break;  // a hook step found every kept edge inside one tree
        HIPCHK(c, hipMemsetAsync(c->cc_ctr->changed, 0, sizeof(unsigned int) * kInitChain, c->stream));
    }
    const int64_t nb = ceil_div(k, kBlock);
    hipLaunchKernelGGL(k_cc_count_roots, dim3((unsigned int)nb), dim3(kBlock), 0, c->stream, k, c->cc_par, c->cc_block);
    hipLaunchKernelGGL(k_cc_scan_blocks, dim3(1), dim3(kBlock), 0, c->stream, nb, c->cc_block, c->cc_ctr);
    hipLaunchKernelGGL(k_cc_number_roots, dim3((unsigned int)nb), dim3(kBlock), 0, c->stream, k, c->cc_par, c->cc_block,
                       c->cc_dense);
    hipLaunchKernelGGL(k_cc_label, dim3(grid_for(k)), dim3(kBlock), 0, c->stream, k, c->cc_par, c->cc_dense, c->cc_comp);
    HIPCHK(c, hipGetLastError());
    read_init_ctr(c);
    const int64_t comps = c->h_cc->components;
    if (comps * c->C > c->cc_wcap) {
        dev_free(c, c->cc_W);
        c->cc_W = nullptr;
        c->cc_wcap = 0;
        const int64_t cap = comps * c->C + comps * c->C / 2;
        c->cc_W = dev_alloc_n<double>(c, cap);
        c->cc_wcap = cap;
    }
    hipLaunchKernelGGL(k_fill_f64, dim3(grid_for(comps * c->C)), dim3(kBlock), 0, c->stream, comps * c->C, c->cc_W, 0.0);
    hipLaunchKernelGGL(k_supernode_weights, dim3((unsigned int)ceil_div(k, kSwRows)), dim3(kBlock), 0, c->stream, n0, k, c->C, c->meta,
                       c->pool, c->seed_class, c->cc_comp, c->cc_W);
    hipLaunchKernelGGL(k_supernode_rows, dim3(grid_for(k * c->CP)), dim3(kBlock), 0, c->stream, n0, k, c->C, c->Cs, c->coff, c->CP,
                       c->seed_class, c->cc_comp, c->cc_W, c->F);
    HIPCHK(c, hipGetLastError());
    HIPCHK(c, hipEventRecord(c->init_ev[1], c->stream));
    c->last_init.vertices = k;
    c->last_init.kept_edges = c->h_cc->kept;
    c->last_init.components = comps;
    c->last_init.hook_steps = hook_steps;
    c->last_init.ms = 0.f;  // filled in after the call's final synchronisation
}

// Prefix offsets of per-row values already stored (caps in meta / lens in an array) need the
// scanned block sums; this runs the middle step and returns the grand total.
int64_t scan_block_sums(dynlp_ctx* c, int64_t nb, int64_t* sums) {
    hipLaunchKernelGGL(k_scan_block_sums, dim3(1), dim3(kBlock), 0, c->stream, nb, sums, &c->bc->scan_total);
    HIPCHK(c, hipGetLastError());
    read_bc(c);
    return (int64_t)c->h_bc->scan_total;
}

// Labels in the caller's format: soft (n x C, no padding) and / or hard (argmax, lowest index on ties) into
// device buffers.  Every row is overwritten, so the buffers need no clearing.
void launch_label_output(dynlp_ctx* c, float* d_soft, int32_t* d_hard) {
    const int64_t n = c->n;
    if (d_soft) {
        if (c->coff)
            hipLaunchKernelGGL(k_scalar_soft, dim3(grid_for(2 * n)), dim3(kBlock), 0, c->stream, n, c->F, d_soft);
        else
            hipLaunchKernelGGL(k_pack_soft, dim3(grid_for(n * c->C)), dim3(kBlock), 0, c->stream, n, c->C, c->CP, c->F, d_soft);
    }
    if (d_hard) {
        if (c->coff)
            hipLaunchKernelGGL(k_scalar_hard, dim3(grid_for(n)), dim3(kBlock), 0, c->stream, n, c->F, d_hard);
        else
            hipLaunchKernelGGL(k_argmax, dim3(grid_for(n * (c->CP >= 4 ? c->CP / 4 : 1))), dim3(kBlock), 0, c->stream, n, c->C, c->CP, c->F, d_hard);
    }
    HIPCHK(c, hipGetLastError());
}

}  // namespace

// =================================================================================================
// C ABI
// =================================================================================================
extern "C" {

void dynlp_default_options(dynlp_options* opt) {
    if (!opt) return;
    std::memset(opt, 0, sizeof *opt);
    opt->slack_factor = 1.25f;
}

const char* dynlp_last_error(const dynlp_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

int64_t dynlp_num_vertices(const dynlp_ctx* ctx) { return ctx ? ctx->n : -1; }
int64_t dynlp_num_entries(const dynlp_ctx* ctx) { return ctx ? ctx->entries : -1; }
int32_t dynlp_num_classes(const dynlp_ctx* ctx) { return ctx ? ctx->C : -1; }

void dynlp_destroy(dynlp_ctx* ctx) { destroy_ctx(ctx); }

dynlp_status dynlp_create(dynlp_ctx** out, int64_t n, const int64_t* row_ptr, const int32_t* col, const float* w,
                          int32_t num_classes, int64_t num_seeds, const int32_t* seed_vertex,
                          const int32_t* seed_class, const dynlp_options* opt) {
    if (out) *out = nullptr;
    g_create_error.clear();
    auto bad = [&](const std::string& msg) {
        g_create_error = msg;
        return DYNLP_ERR_INVALID_ARG;
    };
    if (!out) return bad("out is NULL");
    if (n < 0 || n > 0x7ffffffeLL) return bad("n must be in [0, 2^31-2]");
    if (num_classes < 1 || num_classes > DYNLP_MAX_CLASSES) return bad("num_classes must be in [1, DYNLP_MAX_CLASSES]");
    if (!row_ptr) return bad("row_ptr is NULL");
    if (num_seeds < 0) return bad("num_seeds is negative");
    if (num_seeds > 0 && (!seed_vertex || !seed_class)) return bad("seed arrays are NULL");
    dynlp_options o;
    dynlp_default_options(&o);
    if (opt) o = *opt;
    if (!(o.slack_factor > 1.0f)) o.slack_factor = 1.25f;
    if (o.slack_factor > 8.0f) return bad("slack_factor must be <= 8");
    if (o.reserve_vertices < 0 || o.reserve_edges < 0) return bad("reserve counts must be >= 0");
    if (o.persistent_rounds < -1 || o.persistent_rounds > 1) return bad("persistent_rounds must be -1, 0 or 1");
    if (o.persistent_spin_limit < 0) return bad("persistent_spin_limit must be >= 0");
    if (o.ingest_chunk_edges < 0 || o.ingest_chunk_edges > ((int64_t)1 << 28)) return bad("ingest_chunk_edges must be in [0, 2^28]");
    if ((o.alloc == nullptr) != (o.dealloc == nullptr)) return bad("alloc and dealloc must be given together");
    if (o.binary_scalar != 0 && num_classes != 2) return bad("binary_scalar needs num_classes == 2");
    const int Cs = o.binary_scalar != 0 ? 1 : num_classes;  // stored columns
    const int CP = padded_classes(Cs);
    if (o.binned_rounds != 0 && o.binned_rounds != -1 && (o.binned_rounds < kPbMinBinBits || o.binned_rounds > kPbMaxBinBits))
        return bad("binned_rounds must be 0 (automatic), -1 (never) or a number of bin bits from 8 to 15");
    if (o.group_lanes != 0) {
        const int g = o.group_lanes;
        if (!(g == 4 || g == 8 || g == 16 || g == 32 || g == 64) || g < lanes_per_neighbour(CP))
            return bad("group_lanes must be 0 or one of 4, 8, 16, 32, 64 and at least padded_classes/4");
    }
    // Host-pointer mode: everything that can be checked without a GPU is checked first.
    int64_t nnz = -1;
    if (!o.ptrs_on_device) {
        nnz = row_ptr[n];
        if (nnz < 0) return bad(format_validation(kErrRowPtr, n));
        if (nnz > 0 && (!col || !w)) return bad("col / w are NULL");
        std::string e;
        if (!host_check_csr(e, n, row_ptr, col, w)) return bad(e);
        if (!host_check_seeds(e, num_seeds, n, num_classes, seed_vertex, seed_class)) return bad(e);
    }

    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0 || o.device < 0 || o.device >= ndev) {
        (void)hipGetLastError();
        g_create_error = "no usable GPU (hipGetDeviceCount found " + std::to_string(ndev) + " devices, device " +
                         std::to_string(o.device) + " requested); libdynlp has no CPU path";
        return DYNLP_ERR_DEVICE;
    }
    dynlp_ctx* c = new (std::nothrow) dynlp_ctx;
    if (!c) {
        g_create_error = "host allocation failed";
        return DYNLP_ERR_OOM;
    }
    dynlp_status result = DYNLP_OK;
    int64_t* block_sums = nullptr;
    try {
        c->device = o.device;
        c->stream = static_cast<hipStream_t>(o.stream);
        c->dev_ptrs = o.ptrs_on_device != 0;
        c->slack = o.slack_factor;
        c->time_kernels = o.time_kernels != 0;
        c->group_lanes = o.group_lanes;
        c->binned = o.binned_rounds;
        c->persist = o.persistent_rounds;
        if (o.persistent_spin_limit > 0) c->persist_spin = (unsigned int)o.persistent_spin_limit;
        c->ingest_chunk = o.ingest_chunk_edges > 0 ? o.ingest_chunk_edges : ((int64_t)4 << 20);
        c->alloc_fn = o.alloc;
        c->dealloc_fn = o.dealloc;
        c->alloc_user = o.alloc_user;
        c->C = num_classes;
        c->Cs = Cs;
        c->coff = num_classes - Cs;  // 1 in the binary scalar layout (column 0 holds class 1), else 0
        c->CP = CP;
        HIPCHK(c, hipSetDevice(c->device));
        resolve_static_scratch(c->device);  // for dynlp_get_labels_static; a failure is reported by that call
        hipDeviceProp_t prop;
        HIPCHK(c, hipGetDeviceProperties(&prop, c->device));
        c->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
        c->persist_ctl = static_cast<unsigned int*>(dev_alloc(c, kBarWords * sizeof(unsigned int)));
        c->ring = static_cast<RoundCtr*>(dev_alloc(c, sizeof(RoundCtr) * (kRing + 1)));
        c->bc = static_cast<BatchCtr*>(dev_alloc(c, sizeof(BatchCtr)));
        HIPCHK(c, hipHostMalloc(reinterpret_cast<void**>(&c->h_slot), sizeof(RoundCtr) * kRing, hipHostMallocDefault));
        HIPCHK(c, hipHostMalloc(reinterpret_cast<void**>(&c->h_bc), sizeof(BatchCtr), hipHostMallocDefault));
        for (auto& e : c->phase_ev) HIPCHK(c, hipEventCreate(&e));
        std::memset(c->h_bc, 0, sizeof(BatchCtr));
        write_bc(c);
        zero_ring(c);

        if (c->dev_ptrs) {
            HIPCHK(c, hipMemcpyAsync(&nnz, row_ptr + n, sizeof(int64_t), hipMemcpyDeviceToHost, c->stream));
            HIPCHK(c, hipStreamSynchronize(c->stream));
            if (nnz < 0) {
                c->err = format_validation(kErrRowPtr, n);
                throw Fail{DYNLP_ERR_INVALID_ARG};
            }
            if (nnz > 0 && (!col || !w)) {
                c->err = "col / w are NULL";
                throw Fail{DYNLP_ERR_INVALID_ARG};
            }
        }
        const int64_t reserve_v = o.reserve_vertices > 0 ? o.reserve_vertices : std::max<int64_t>(1024, n / 8);
        c->n = 0;  // nothing to preserve while the arrays are first allocated
        alloc_vertex_arrays(c, n + reserve_v);
        c->n = n;

        DevIn<int64_t> d_rp(c, row_ptr, n + 1);
        DevIn<int32_t> d_col(c, col, nnz);
        DevIn<float> d_w(c, w, nnz);
        DevIn<int32_t> d_sv(c, seed_vertex, num_seeds);
        DevIn<int32_t> d_sc(c, seed_class, num_seeds);

        // validate row_ptr and the seed list
        if (n > 0)
            hipLaunchKernelGGL(k_validate_row_ptr, dim3(grid_for(n)), dim3(kBlock), 0, c->stream, n, d_rp.ptr, nnz, c->bc);
        if (num_seeds > 0) {
            hipLaunchKernelGGL(k_validate_seeds, dim3(grid_for(num_seeds)), dim3(kBlock), 0, c->stream, num_seeds, n,
                               (int64_t)0, c->C, d_sv.ptr, d_sc.ptr, c->seed_class, c->add_cnt, c->bc);
            hipLaunchKernelGGL(k_clear_seed_tmp, dim3(grid_for(num_seeds)), dim3(kBlock), 0, c->stream, num_seeds, n,
                               d_sv.ptr, c->add_cnt);
        }
        HIPCHK(c, hipGetLastError());
        read_bc(c);
        if (c->h_bc->err_code) {
            c->err = format_validation(c->h_bc->err_code, c->h_bc->err_index);
            throw Fail{DYNLP_ERR_INVALID_ARG};
        }

        // slack layout: capacities, offsets (scan), entries
        const int64_t nb = grid_for(n);
        block_sums = dev_alloc_n<int64_t>(c, nb);
        int64_t tail = 0;
        if (n > 0) {
            hipLaunchKernelGGL(k_row_caps, dim3(nb), dim3(kBlock), 0, c->stream, n, d_rp.ptr, c->slack, c->meta, block_sums);
            HIPCHK(c, hipGetLastError());
            tail = scan_block_sums(c, nb, block_sums);
            hipLaunchKernelGGL(k_row_offsets, dim3(nb), dim3(kBlock), 0, c->stream, n, c->meta, block_sums);
            HIPCHK(c, hipGetLastError());
        }
        c->pool_tail = tail;
        const int64_t extra = tail / 4 + 4 * o.reserve_edges + (1 << 16);
        c->pool_cap = 0;
        grow_pool(c, tail + extra);
        c->h_bc->pool_tail = (unsigned long long)tail;
        c->h_bc->err_code = 0;
        write_bc(c);
        if (nnz > 0) {
            hipLaunchKernelGGL(k_scatter_entries, dim3(grid_for(nnz)), dim3(kBlock), 0, c->stream, nnz, n, d_rp.ptr,
                               d_col.ptr, d_w.ptr, c->meta, c->pool, c->bc);
            HIPCHK(c, hipGetLastError());
        }
        read_bc(c);
        if (c->h_bc->err_code) {
            c->err = format_validation(c->h_bc->err_code, c->h_bc->err_index);
            throw Fail{DYNLP_ERR_INVALID_ARG};
        }
        c->entries = nnz;

        // labels
        hipLaunchKernelGGL(k_fill_i32, dim3(grid_for(c->n_cap)), dim3(kBlock), 0, c->stream, (int64_t)0, c->n_cap,
                           c->seed_class, -1);
        if (num_seeds > 0)
            hipLaunchKernelGGL(k_set_seed_class, dim3(grid_for(num_seeds)), dim3(kBlock), 0, c->stream, num_seeds,
                               d_sv.ptr, d_sc.ptr, c->seed_class);
        if (n > 0) {
            hipLaunchKernelGGL(k_init_labels, dim3(grid_for(n * c->CP)), dim3(kBlock), 0, c->stream, (int64_t)0, n, c->C,
                               c->Cs, c->coff, c->CP, c->seed_class, c->F);
            hipLaunchKernelGGL(k_row_degree, dim3(grid_for(n * 16)), dim3(kBlock), 0, c->stream, n, c->meta, c->pool,
                               c->deg);
        }
        HIPCHK(c, hipGetLastError());
        HIPCHK(c, hipStreamSynchronize(c->stream));
    } catch (const Fail& f) {
        result = f.st;
    } catch (const std::bad_alloc&) {
        c->err = "host allocation failed";
        result = DYNLP_ERR_OOM;
    }
    if (block_sums) dev_free(c, block_sums);
    if (result != DYNLP_OK) {
        g_create_error = c->err;
        destroy_ctx(c);
        return result;
    }
    *out = c;
    return DYNLP_OK;
}

dynlp_status dynlp_set_params(dynlp_ctx* ctx, float tol, int32_t max_iter) {
    if (!ctx) return DYNLP_ERR_INVALID_ARG;
    if (!(tol >= 0.f) || !std::isfinite(tol) || max_iter < 0) {
        ctx->err = "tol must be finite and >= 0, max_iter >= 0";
        return DYNLP_ERR_INVALID_ARG;
    }
    ctx->tol = tol;
    ctx->max_iter = max_iter;
    return DYNLP_OK;
}

dynlp_status dynlp_stream_bandwidth(dynlp_ctx* c, int64_t bytes, int32_t repetitions, double* copy_gb_per_s,
                                    double* read_gb_per_s) {
    if (!c) return DYNLP_ERR_INVALID_ARG;
    if (bytes < 16 || repetitions < 1) {
        c->err = "bytes < 16 or repetitions < 1";
        return DYNLP_ERR_INVALID_ARG;
    }
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    try {
        HIPCHK(c, hipSetDevice(c->device));
        const int64_t n16 = bytes / 16;
        const unsigned int blocks = (unsigned int)std::min<int64_t>(grid_for(n16), (int64_t)c->num_cu * 16);
        Temp<float4> src_t(c, n16);
        Temp<float4> dst_t(c, std::max<int64_t>(n16, ceil_div((int64_t)blocks * kBlock * (int64_t)sizeof(float), 16)));
        float4 *src = src_t.ptr, *dst = dst_t.ptr;
        HIPCHK(c, hipMemsetAsync(src, 0, (size_t)n16 * 16, c->stream));
        for (hipEvent_t& e : ev) HIPCHK(c, hipEventCreate(&e));
        hipLaunchKernelGGL(k_stream_copy, dim3(blocks), dim3(kBlock), 0, c->stream, n16, src, dst);  // warm-up
        HIPCHK(c, hipEventRecord(ev[0], c->stream));
        for (int r = 0; r < repetitions; ++r)
            hipLaunchKernelGGL(k_stream_copy, dim3(blocks), dim3(kBlock), 0, c->stream, n16, src, dst);
        HIPCHK(c, hipEventRecord(ev[1], c->stream));
        for (int r = 0; r < repetitions; ++r)
            hipLaunchKernelGGL(k_stream_read, dim3(blocks), dim3(kBlock), 0, c->stream, n16, src,
                               reinterpret_cast<float*>(dst));
        HIPCHK(c, hipEventRecord(ev[2], c->stream));
        HIPCHK(c, hipGetLastError());
        HIPCHK(c, hipEventSynchronize(ev[2]));
        float ms_copy = 0.f, ms_read = 0.f;
        HIPCHK(c, hipEventElapsedTime(&ms_copy, ev[0], ev[1]));
        HIPCHK(c, hipEventElapsedTime(&ms_read, ev[1], ev[2]));
        const double moved = (double)n16 * 16.0 * repetitions;
        if (copy_gb_per_s) *copy_gb_per_s = 2.0 * moved / ((double)ms_copy * 1e6);  // bytes read + bytes written
        if (read_gb_per_s) *read_gb_per_s = moved / ((double)ms_read * 1e6);
        for (hipEvent_t e : ev) (void)hipEventDestroy(e);
        return DYNLP_OK;
    } catch (const SoftOom&) {
        return DYNLP_ERR_OOM;
    } catch (const Fail& f) {
        for (hipEvent_t e : ev)
            if (e) (void)hipEventDestroy(e);
        return f.st;
    }
}

dynlp_status dynlp_gather_bandwidth(dynlp_ctx* c, int64_t table_rows, int32_t row_bytes, int64_t gathers,
                                    int32_t repetitions, double* gathers_per_s, double* gb_per_s) {
    if (!c) return DYNLP_ERR_INVALID_ARG;
    if (table_rows < 1 || table_rows > 0x7fffffffLL || gathers < 1 || repetitions < 1 ||
        !(row_bytes == 16 || row_bytes == 32 || row_bytes == 64 || row_bytes == 128 || row_bytes == 256)) {
        c->err = "table_rows in [1, 2^31), row_bytes one of 16, 32, 64, 128, 256, gathers >= 1, repetitions >= 1";
        return DYNLP_ERR_INVALID_ARG;
    }
    hipEvent_t ev[2] = {nullptr, nullptr};
    try {
        HIPCHK(c, hipSetDevice(c->device));
        const int lpn = row_bytes / 16;
        const unsigned int blocks = (unsigned int)std::min<int64_t>(grid_for(ceil_div(gathers, 8) * lpn), (int64_t)c->num_cu * 32);
        Temp<float4> table(c, table_rows * lpn);
        Temp<float> sink(c, (int64_t)blocks * kBlock);
        HIPCHK(c, hipMemsetAsync(table.ptr, 0, (size_t)table_rows * row_bytes, c->stream));
        for (hipEvent_t& e : ev) HIPCHK(c, hipEventCreate(&e));
        auto launch = [&]() {
            switch (lpn) {
                case 1: hipLaunchKernelGGL(k_gather_probe<1>, dim3(blocks), dim3(kBlock), 0, c->stream, table.ptr, (unsigned int)table_rows, (unsigned long long)gathers, sink.ptr); break;
                case 2: hipLaunchKernelGGL(k_gather_probe<2>, dim3(blocks), dim3(kBlock), 0, c->stream, table.ptr, (unsigned int)table_rows, (unsigned long long)gathers, sink.ptr); break;
                case 4: hipLaunchKernelGGL(k_gather_probe<4>, dim3(blocks), dim3(kBlock), 0, c->stream, table.ptr, (unsigned int)table_rows, (unsigned long long)gathers, sink.ptr); break;
                case 8: hipLaunchKernelGGL(k_gather_probe<8>, dim3(blocks), dim3(kBlock), 0, c->stream, table.ptr, (unsigned int)table_rows, (unsigned long long)gathers, sink.ptr); break;
                default: hipLaunchKernelGGL(k_gather_probe<16>, dim3(blocks), dim3(kBlock), 0, c->stream, table.ptr, (unsigned int)table_rows, (unsigned long long)gathers, sink.ptr); break;
            }
        };
        launch();  // warm-up
        HIPCHK(c, hipEventRecord(ev[0], c->stream));
        for (int r = 0; r < repetitions; ++r) launch();
        HIPCHK(c, hipEventRecord(ev[1], c->stream));
        HIPCHK(c, hipGetLastError());
        HIPCHK(c, hipEventSynchronize(ev[1]));
        float ms = 0.f;
        HIPCHK(c, hipEventElapsedTime(&ms, ev[0], ev[1]));
        const double per_s = (double)gathers * repetitions / ((double)ms * 1e-3);
        if (gathers_per_s) *gathers_per_s = per_s;
        if (gb_per_s) *gb_per_s = per_s * row_bytes / 1e9;
        for (hipEvent_t e : ev) (void)hipEventDestroy(e);
        return DYNLP_OK;
    } catch (const SoftOom&) {
        for (hipEvent_t e : ev)
            if (e) (void)hipEventDestroy(e);
        return DYNLP_ERR_OOM;
    } catch (const Fail& f) {
        for (hipEvent_t e : ev)
            if (e) (void)hipEventDestroy(e);
        return f.st;
    }
}

dynlp_status dynlp_storage_info(const dynlp_ctx* c, int64_t* pool_used, int64_t* pool_capacity) {
    if (!c) return DYNLP_ERR_INVALID_ARG;
    if (pool_used) *pool_used = c->pool_tail;
    if (pool_capacity) *pool_capacity = c->pool_cap;
    return DYNLP_OK;
}

dynlp_status dynlp_compact_storage(dynlp_ctx* c) {
    if (!c) return DYNLP_ERR_INVALID_ARG;
    if (c->poisoned) {
        c->err = "context is unusable after an earlier device or memory error";
        return DYNLP_ERR_STATE;
    }
    if (c->n == 0) return DYNLP_OK;
    try {
        HIPCHK(c, hipSetDevice(c->device));
        const int64_t n = c->n;
        const int64_t nb = grid_for(n);
        // the new layout is built beside the old one; the context switches over only when all of it exists, so
        // running out of memory here leaves graph and labels as they were
        Temp<RowMeta> meta_new(c, c->n_cap);
        Temp<int64_t> block_sums(c, nb);
        hipLaunchKernelGGL(k_recap_rows, dim3(nb), dim3(kBlock), 0, c->stream, n, c->meta, c->slack, meta_new.ptr, block_sums.ptr);
        HIPCHK(c, hipGetLastError());
        const int64_t tail = scan_block_sums(c, nb, block_sums.ptr);
        hipLaunchKernelGGL(k_row_offsets, dim3(nb), dim3(kBlock), 0, c->stream, n, meta_new.ptr, block_sums.ptr);
        const int64_t cap = round_up(tail + tail / 4 + (1 << 16), kRowAlign);
        Temp<Edge> pool_new(c, cap);
        hipLaunchKernelGGL(k_copy_rows, dim3(grid_for(n * 16)), dim3(kBlock), 0, c->stream, n, c->meta, meta_new.ptr, c->pool,
                           pool_new.ptr);
        HIPCHK(c, hipGetLastError());
        HIPCHK(c, hipStreamSynchronize(c->stream));
        dev_free(c, c->meta);
        dev_free(c, c->pool);
        c->meta = meta_new.release();
        c->pool = pool_new.release();
        c->pool_cap = cap;
        c->pool_tail = tail;
        return DYNLP_OK;
    } catch (const SoftOom&) {
        (void)hipStreamSynchronize(c->stream);
        return DYNLP_ERR_OOM;
    } catch (const Fail& f) {
        return f.st;
    } catch (const std::bad_alloc&) {
        c->err = "host allocation failed";
        return DYNLP_ERR_OOM;
    }
}

dynlp_status dynlp_set_update_mode(dynlp_ctx* ctx, int32_t mode) {
    if (!ctx) return DYNLP_ERR_INVALID_ARG;
    if (mode != DYNLP_UPDATE_SYNCHRONOUS && mode != DYNLP_UPDATE_IN_PLACE) {
        ctx->err = "mode must be DYNLP_UPDATE_SYNCHRONOUS or DYNLP_UPDATE_IN_PLACE";
        return DYNLP_ERR_INVALID_ARG;
    }
    ctx->update_mode = mode;
    return DYNLP_OK;
}

dynlp_status dynlp_set_final_check(dynlp_ctx* ctx, int32_t on) {
    if (!ctx) return DYNLP_ERR_INVALID_ARG;
    if (on != 0 && on != 1) {
        ctx->err = "on must be 0 or 1";
        return DYNLP_ERR_INVALID_ARG;
    }
    ctx->final_check = on != 0;
    return DYNLP_OK;
}

dynlp_status dynlp_set_initialiser(dynlp_ctx* ctx, int32_t mode, float tau) {
    if (!ctx) return DYNLP_ERR_INVALID_ARG;
    if (mode != DYNLP_INIT_UNIFORM && mode != DYNLP_INIT_SUPERNODE) {
        ctx->err = "mode must be DYNLP_INIT_UNIFORM or DYNLP_INIT_SUPERNODE";
        return DYNLP_ERR_INVALID_ARG;
    }
    if (mode == DYNLP_INIT_SUPERNODE && (!std::isfinite(tau) || tau < 0.f)) {
        ctx->err = "tau must be finite and >= 0";
        return DYNLP_ERR_INVALID_ARG;
    }
    ctx->init_mode = mode;
    ctx->tau = tau;
    return DYNLP_OK;
}

dynlp_status dynlp_mean_edge_weight(dynlp_ctx* c, double* mean) {
    if (!c) return DYNLP_ERR_INVALID_ARG;
    if (!mean) {
        c->err = "mean is NULL";
        return DYNLP_ERR_INVALID_ARG;
    }
    if (c->poisoned) {
        c->err = "context is unusable after an earlier device or memory error";
        return DYNLP_ERR_STATE;
    }
    *mean = 0.0;
    if (c->entries == 0) return DYNLP_OK;
    try {
        HIPCHK(c, hipSetDevice(c->device));
        const unsigned int blocks = (unsigned int)std::min<int64_t>(grid_for(c->n * 16), (int64_t)c->num_cu * 4);
        Temp<double> d_part(c, blocks);
        std::vector<double> part(blocks);
        hipLaunchKernelGGL(k_weight_partial, dim3(blocks), dim3(kBlock), 0, c->stream, c->n, c->meta, c->pool, d_part.ptr);
        HIPCHK(c, hipGetLastError());
        HIPCHK(c, hipMemcpyAsync(part.data(), d_part.ptr, sizeof(double) * blocks, hipMemcpyDeviceToHost, c->stream));
        HIPCHK(c, hipStreamSynchronize(c->stream));
        double tot = 0.0;
        for (double v : part) tot += v;
        *mean = tot / (double)c->entries;
        return DYNLP_OK;
    } catch (const SoftOom&) {
        return DYNLP_ERR_OOM;
    } catch (const Fail& f) {
        return f.st;
    } catch (const std::bad_alloc&) {
        c->err = "host allocation failed";
        return DYNLP_ERR_OOM;
    }
}

dynlp_status dynlp_last_components(dynlp_ctx* c, int64_t cap, int32_t* comp, dynlp_init_info* info) {
    if (!c) return DYNLP_ERR_INVALID_ARG;
    if (info) *info = c->last_init;
    if (!comp || c->last_init.vertices == 0) return DYNLP_OK;
    if (cap < c->last_init.vertices) {
        c->err = "comp holds fewer entries than the last batch inserted vertices";
        return DYNLP_ERR_INVALID_ARG;
    }
    if (c->poisoned) {
        c->err = "context is unusable after an earlier device or memory error";
        return DYNLP_ERR_STATE;
    }
    try {
        HIPCHK(c, hipSetDevice(c->device));
        HIPCHK(c, hipMemcpyAsync(comp, c->cc_comp, sizeof(int32_t) * (size_t)c->last_init.vertices,
                                 c->dev_ptrs ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost, c->stream));
        HIPCHK(c, hipStreamSynchronize(c->stream));
        return DYNLP_OK;
    } catch (const Fail& f) {
        return f.st;
    }
}

dynlp_status dynlp_static_solve(dynlp_ctx* c, float tol, int32_t max_iter, dynlp_stats* stats) {
    if (!c) return DYNLP_ERR_INVALID_ARG;
    fill_stats_zero(stats);
    if (c->poisoned) {
        c->err = "context is unusable after an earlier device or memory error";
        return DYNLP_ERR_STATE;
    }
    dynlp_status st = dynlp_set_params(c, tol, max_iter);
    if (st != DYNLP_OK) return st;
    const auto t0 = Clock::now();
    try {
        HIPCHK(c, hipSetDevice(c->device));
        c->log.clear();
        reset_timed_spans(c);
        const bool in_place = c->update_mode == DYNLP_UPDATE_IN_PLACE;
        if (!in_place) sync_partner(c);
        zero_ring(c);
        const Frontier f = frontier_of(c, 0);
        RoundCtr* start = slot_of(c, -1);
        launch_compact(c, f, &start->next_count, &start->next_long, 1);
        read_slots_start(c);
        const unsigned int nq = c->h_slot[0].next_count + c->h_slot[0].next_long;
        c->h_slot_start_long = c->h_slot[0].next_long;
        int it = 0;
        float last = 0.f;
        bool converged = nq == 0;
        int64_t edges = 0;
        const int G = choose_group(c, c->n > 0 ? (double)c->entries / (double)std::max<int64_t>(1, nq) : 1.0);
        const auto t_it = Clock::now();
        // synchronous: sweep t reads buf[t & 1], writes buf[(t + 1) & 1]; in place: every sweep reads and writes F
        float* const buf[2] = {c->F, in_place ? c->F : c->F2};
        // sweeps whose max change repeats exactly 16 times are in a float32 limit cycle (a nearly bipartite, weakly
        // tied component): the remaining sweeps average old and new rows (same fixed point, no such cycle)
        int same_run = 0;
        bool lazy = false;
        unsigned int prev_bits = 0xffffffffu;
        // Scalar labels on a large graph: every sweep after the first as a binned round (dynlp_binned.h) in which
        // every updatable vertex counts as moved, so that V_aff is all of them; a binned round does nothing once
        // its predecessor moved no row by more than tol, which is the stop rule of the static solve.
        Frontier all_rows = f;
        all_rows.ns = c->h_slot[0].next_count;
        all_rows.nl = c->h_slot[0].next_long;
        c->pb_built = false;
        const bool binned = !converged && binned_rounds_pay(c, all_rows) && build_binned(c);
        bool pb_fresh = true;  // the slots of the binned rounds do not yet hold the current labels
        if (binned) HIPCHK(c, hipMemsetAsync(c->moved[0], 0xff, (size_t)c->moved_words * sizeof(unsigned int), c->stream));
        while (!converged && it < max_iter) {
            // a chain of sweeps; each checks on the device whether its predecessor already met the stop rule
            const int r = std::min<int>(kChain, max_iter - it);
            const bool chain_binned = binned && !lazy;  // the averaged sweeps of a limit cycle are ordinary ones
            for (int i = 0; i < r; ++i) {
                const int t = it + i;
                c->ev_adjacent = i > 0;  // a chain of sweeps is nothing but these launches
                if (chain_binned && t > 0) {
                    const PullRoundArgs a{slot_of(c, t - 1), buf[t & 1], buf[(t + 1) & 1], c->moved[0], c->moved[1], c->moved[2],
                                          tol, slot_of(c, t), slot_of(c, t + 1)};
                    launch_binned_round(c, a, t, t == 1 || pb_fresh);
                    pb_fresh = false;
                    continue;
                }
                const UpdateArgs a{slot_of(c, t - 1), t == 0 ? 1 : 2, buf[t & 1], buf[(t + 1) & 1], nullptr, tol,
                                   slot_of(c, t), slot_of(c, t + 1), (int64_t)nq, (int64_t)c->h_slot_start_long,
                                   lazy ? kRowLazy : 0};
                launch_update<false>(c, G, f, a, t);
            }
            const size_t first_pair = c->events_used / 2 - (c->time_kernels ? (size_t)r : 0);
            read_slots(c, it, r);
            {
                int done = 0;
                while (done < r && c->h_slot[done].executed) ++done;
                if (c->time_kernels) trim_timed_spans(c, first_pair, it + done);
            }
            if (!c->h_slot[0].executed) break;  // cannot happen while the stop rule is unmet; never spin on it
            for (int i = 0; i < r; ++i) {
                const RoundCtr& rc = c->h_slot[i];
                if (!rc.executed) break;
                std::memcpy(&last, &rc.resid_bits, sizeof(float));
                edges += (int64_t)(rc.edges + rc.edges_long);
                c->log.push_back(round_info(rc, chain_binned && it > 0 ? 3 : 0, G));
                ++it;
                same_run = rc.resid_bits == prev_bits ? same_run + 1 : 0;
                prev_bits = rc.resid_bits;
                if (same_run >= 16) lazy = true;
                if (last <= tol) {
                    converged = true;
                    break;
                }
            }
        }
        // the labels of the last executed sweep
        if (!in_place) {
            c->F = buf[it & 1];
            c->F2 = buf[(it + 1) & 1];
        }
        const float kernel_ms_total = c->time_kernels ? collect_kernel_ms(c) : 0.f;
        if (stats) {
            stats->iterations = it;
            stats->converged = converged ? 1 : 0;
            stats->final_max_delta = last;
            stats->rows_updated = (int64_t)nq * it;
            stats->edges_traversed = edges;
            stats->frontier_initial = nq;
            stats->frontier_peak = nq;
            stats->update_launches = it;
            stats->ms_iterate = ms_since(t_it);
            stats->ms_update_kernel = kernel_ms_total;
            stats->ms_total = ms_since(t0);
        }
        reset_timed_spans(c);
        return converged ? DYNLP_OK : DYNLP_NOT_CONVERGED;
    } catch (const Fail& f) {
        return f.st;
    } catch (const std::bad_alloc&) {
        c->err = "host allocation failed";
        return DYNLP_ERR_OOM;
    }
}

dynlp_status dynlp_apply_batch(dynlp_ctx* c, int64_t k, int64_t m, const int32_t* eu, const int32_t* ev,
                               const float* ew, int64_t s, const int32_t* sv, const int32_t* sc, dynlp_stats* stats) {
    return dynlp_apply_update(c, 0, nullptr, k, m, eu, ev, ew, s, sv, sc, stats);
}

dynlp_status dynlp_apply_update(dynlp_ctx* c, int64_t nd, const int32_t* del, int64_t k, int64_t m, const int32_t* eu,
                                const int32_t* ev, const float* ew, int64_t s, const int32_t* sv, const int32_t* sc,
                                dynlp_stats* stats) {
    if (!c) return DYNLP_ERR_INVALID_ARG;
    fill_stats_zero(stats);
    if (c->poisoned) {
        c->err = "context is unusable after an earlier device or memory error";
        return DYNLP_ERR_STATE;
    }
    auto bad = [&](const std::string& msg) {
        c->err = msg;
        return DYNLP_ERR_INVALID_ARG;
    };
    if (k < 0 || m < 0 || s < 0 || nd < 0) return bad("counts must be >= 0");
    if (nd > 0 && !del) return bad("deleted_vertex is NULL");
    if (m > 0 && (!eu || !ev || !ew)) return bad("edge arrays are NULL");
    if (s > 0 && (!sv || !sc)) return bad("seed arrays are NULL");
    const int64_t n0 = c->n, n1 = c->n + k;
    if (n1 > 0x7ffffffeLL) return bad("vertex count would exceed 2^31-2");
    if (m > 0x3fffffffLL) return bad("too many edges in one batch");
    // a host-resident edge list of more than one chunk is sent in a pipeline (ingest_edges) and checked on the
    // device chunk by chunk as it arrives; a smaller one is checked here, before any device work
    const bool pipelined = !c->dev_ptrs && nd == 0 && m > c->ingest_chunk;
    if (!c->dev_ptrs) {
        std::string e;
        if (!pipelined && !host_check_edges(e, m, n1, eu, ev, ew)) return bad(e);
        if (!host_check_seeds(e, s, n1, c->C, sv, sc)) return bad(e);
        for (int64_t i = 0; i < nd; ++i)
            if (del[i] < 0 || del[i] >= n0) return bad(format_validation(kErrDeleted, i));
    }
    const auto t0 = Clock::now();
    bool mutated = false;
    try {
        HIPCHK(c, hipSetDevice(c->device));
        c->log.clear();
        reset_timed_spans(c);
        // ---- capacity for new vertices; their rows start empty, unlabelled, uniform ----
        if (n1 > c->n_cap) alloc_vertex_arrays(c, n1 + std::max<int64_t>(n1 / 2, 1024));
        ensure_batch_scratch(c, m, s);
        const bool use_rank = c->he_rank != nullptr;
        const int32_t *d_eu = eu, *d_ev = ev, *d_sv = sv, *d_sc = sc;
        const float* d_ew = ew;
        c->ingest_chunks_last = 0;
        if (!c->dev_ptrs) {
            if (m > 0 && !pipelined) {
                HIPCHK(c, hipMemcpyAsync(c->b_eu, eu, (size_t)m * 4, hipMemcpyHostToDevice, c->stream));
                HIPCHK(c, hipMemcpyAsync(c->b_ev, ev, (size_t)m * 4, hipMemcpyHostToDevice, c->stream));
                HIPCHK(c, hipMemcpyAsync(c->b_ew, ew, (size_t)m * 4, hipMemcpyHostToDevice, c->stream));
            }
            if (s > 0) {
                HIPCHK(c, hipMemcpyAsync(c->b_sv, sv, (size_t)s * 4, hipMemcpyHostToDevice, c->stream));
                HIPCHK(c, hipMemcpyAsync(c->b_sc, sc, (size_t)s * 4, hipMemcpyHostToDevice, c->stream));
            }
            d_eu = c->b_eu;
            d_ev = c->b_ev;
            d_ew = c->b_ew;
            d_sv = c->b_sv;
            d_sc = c->b_sc;
        }
        HIPCHK(c, hipEventRecord(c->phase_ev[0], c->stream));

        // ---- deletions come first (Alg. 2 Step 1): the whole batch is validated before anything changes ----
        if (nd > 0) {
            DevIn<int32_t> d_del(c, del, nd);
            if (c->n_cap > c->touched_cap) {  // any vertex may lose an entry
                dev_free(c, c->touched);
                dev_free(c, c->reloc_off);
                c->touched = nullptr;
                c->reloc_off = nullptr;
                c->touched_cap = 0;
                c->touched = dev_alloc_n<int32_t>(c, c->n_cap);
                c->reloc_off = dev_alloc_n<int64_t>(c, c->n_cap);
                c->touched_cap = c->n_cap;
            }
            std::memset(c->h_bc, 0, sizeof(BatchCtr));
            c->h_bc->pool_tail = (unsigned long long)c->pool_tail;
            HIPCHK(c, hipMemcpyAsync(c->bc, c->h_bc, sizeof(BatchCtr), hipMemcpyHostToDevice, c->stream));
            hipLaunchKernelGGL(k_validate_deleted, dim3(grid_for(nd)), dim3(kBlock), 0, c->stream, nd, n0, d_del.ptr, c->bc);
            if (m > 0)
                hipLaunchKernelGGL(k_validate_edges, dim3(grid_for(m)), dim3(kBlock), 0, c->stream, m, n1, d_eu, d_ev, d_ew,
                                   c->bc);
            if (s > 0) {
                hipLaunchKernelGGL(k_validate_seeds, dim3(grid_for(s)), dim3(kBlock), 0, c->stream, s, n1, n0, c->C, d_sv,
                                   d_sc, c->seed_class, c->add_cnt, c->bc);
                hipLaunchKernelGGL(k_clear_seed_tmp, dim3(grid_for(s)), dim3(kBlock), 0, c->stream, s, n1, d_sv, c->add_cnt);
            }
            HIPCHK(c, hipGetLastError());
            read_bc(c);
            if (c->h_bc->err_code) return bad(format_validation(c->h_bc->err_code, c->h_bc->err_index));
            mutated = true;
            hipLaunchKernelGGL(k_mark_deleted, dim3(grid_for(nd)), dim3(kBlock), 0, c->stream, nd, d_del.ptr, c->seed_class,
                               kDeletedMark);
            hipLaunchKernelGGL(k_delete_rows, dim3(grid_for(nd * 16)), dim3(kBlock), 0, c->stream, nd, d_del.ptr, c->C, c->Cs, c->CP,
                               c->meta, c->pool, c->seed_class, c->flag, c->add_cnt, c->touched, c->deg, c->F, c->bc);
            HIPCHK(c, hipGetLastError());
            read_bc(c);
            const unsigned int nt_del = c->h_bc->touched;
            if (nt_del)
                hipLaunchKernelGGL(k_drop_deleted_entries, dim3(grid_for((int64_t)nt_del * 16)), dim3(kBlock), 0, c->stream,
                                   nt_del, c->touched, c->meta, c->pool, c->seed_class, c->add_cnt, c->deg);
            hipLaunchKernelGGL(k_mark_deleted, dim3(grid_for(nd)), dim3(kBlock), 0, c->stream, nd, d_del.ptr, c->seed_class, -1);
            HIPCHK(c, hipGetLastError());
            c->entries -= (int64_t)c->h_bc->removed;
        }

        // ---- validate, count entries per row, plan relocations: one read-back for all three ----
        std::memset(c->h_bc, 0, sizeof(BatchCtr));
        c->h_bc->pool_tail = (unsigned long long)c->pool_tail;
        HIPCHK(c, hipMemcpyAsync(c->bc, c->h_bc, sizeof(BatchCtr), hipMemcpyHostToDevice, c->stream));
        if (m > 0 && !pipelined)
            hipLaunchKernelGGL(k_validate_edges, dim3(grid_for(m)), dim3(kBlock), 0, c->stream, m, n1, d_eu, d_ev, d_ew, c->bc);
        if (s > 0) {
            hipLaunchKernelGGL(k_validate_seeds, dim3(grid_for(s)), dim3(kBlock), 0, c->stream, s, n1, n0, c->C, d_sv,
                               d_sc, c->seed_class, c->add_cnt, c->bc);
            hipLaunchKernelGGL(k_clear_seed_tmp, dim3(grid_for(s)), dim3(kBlock), 0, c->stream, s, n1, d_sv, c->add_cnt);
        }
        if (k > 0) {  // empty rows for the new ids (scratch state only until n is advanced)
            hipLaunchKernelGGL(k_init_meta, dim3(grid_for(k)), dim3(kBlock), 0, c->stream, n0, n1, c->meta, c->deg);
            hipLaunchKernelGGL(k_fill_i32, dim3(grid_for(k)), dim3(kBlock), 0, c->stream, n0, n1, c->seed_class, -1);
        }
        if (pipelined)
            ingest_edges(c, m, n1, eu, ev, ew);
        else if (m > 0)
            hipLaunchKernelGGL(k_count_halfedges, dim3(grid_for(ceil_div(2 * m, kAppendItems))), dim3(kBlock), 0, c->stream, m, n1, d_eu, d_ev,
                               c->add_cnt, c->touched, c->bc, use_rank ? c->he_rank : nullptr,
                               use_rank ? c->he_rank + m : nullptr);
        HIPCHK(c, hipGetLastError());
        read_bc(c);
        unsigned int nt = c->h_bc->touched;
        if (c->h_bc->err_code) {
            if (nt) hipLaunchKernelGGL(k_clear_counts, dim3(grid_for(nt)), dim3(kBlock), 0, c->stream, nt, c->touched, c->add_cnt);
            HIPCHK(c, hipStreamSynchronize(c->stream));
            return bad(format_validation(c->h_bc->err_code, c->h_bc->err_index));
        }
        if (nt) {
            // room at the pool tail for the rows whose slack is too small: planned on the device (no row is touched
            // yet), then the pool is made large enough for the plan
            hipLaunchKernelGGL(k_plan_reserve, dim3(grid_for(nt)), dim3(kBlock), 0, c->stream, nt, c->touched, c->meta,
                               c->add_cnt, c->slack, c->reloc_off, c->bc);
            HIPCHK(c, hipGetLastError());
            read_bc(c);
            const int64_t tail = (int64_t)c->h_bc->pool_tail;
            if (tail > c->pool_cap) grow_pool(c, tail + (tail - c->pool_tail) / 2);
        }
        // ---- from here on the graph changes ----
        mutated = true;
        if (k > 0)
            hipLaunchKernelGGL(k_init_labels, dim3(grid_for(k * c->CP)), dim3(kBlock), 0, c->stream, n0, n1, c->C, c->Cs, c->coff,
                               c->CP, c->seed_class, c->F);
        if (nt) {
            hipLaunchKernelGGL(k_relocate, dim3(grid_for(nt)), dim3(kBlock), 0, c->stream, nt, c->touched, c->meta, c->add_cnt,
                               c->slack, c->reloc_off, c->pool);
            const int32_t* rank = use_rank ? c->he_rank : nullptr;
            hipLaunchKernelGGL(k_write_halfedges, dim3(grid_for(2 * m)), dim3(kBlock), 0, c->stream, m, d_eu, d_ev, d_ew,
                               c->meta, c->pool, rank);
            // the batch's entries of every row in a fixed order, then degree, scratch and V_aff flag of the row (the
            // relocation offsets are no longer needed: their array holds the list of rows with long appended segments)
            int32_t* long_list = reinterpret_cast<int32_t*>(c->reloc_off);
            hipLaunchKernelGGL(k_sort_finish, dim3(grid_for((int64_t)nt * 16)), dim3(kBlock), 0, c->stream, nt, c->touched,
                               c->meta, c->pool, c->add_cnt, use_rank ? 1 : 0, long_list, c->bc, c->deg, c->flag);
            hipLaunchKernelGGL(k_sort_long_segments, dim3(std::min<unsigned int>(nt, 512u)), dim3(kSortThreads), 0, c->stream,
                               long_list, c->meta, c->pool, c->add_cnt, c->bc);
            hipLaunchKernelGGL(k_finish_rows, dim3(std::min<unsigned int>(grid_for((int64_t)nt * 16), 512u)), dim3(kBlock), 0,
                               c->stream, long_list, c->bc, c->meta, c->pool, c->add_cnt, c->deg, c->flag);
            HIPCHK(c, hipGetLastError());
        }
        c->n = n1;
        c->entries += 2 * m;
        HIPCHK(c, hipEventRecord(c->phase_ev[1], c->stream));
        // ---- seeds: clamp one-hot, their neighbours join V_aff; first compaction ----
        if (s > 0)
            hipLaunchKernelGGL(k_apply_seeds, dim3(grid_for(s * 16)), dim3(kBlock), 0, c->stream, s, d_sv, d_sc, c->Cs, c->coff, c->CP,
                               c->seed_class, c->F, c->meta, c->pool, c->flag);
        c->last_init = dynlp_init_info{};
        if (c->init_mode == DYNLP_INIT_SUPERNODE && k > 0) run_supernode_init(c, n0, k, m, d_eu, d_ev, d_ew);
        zero_ring(c);
        // first frontier from the flags (its size goes to the start slot), and the list of all updatable
        // vertices
        RoundCtr* start = slot_of(c, -1);
        launch_compact(c, frontier_of(c, 0), &start->next_count, &start->next_long, 0);
        Frontier universe = frontier_of(c, 2);
        launch_compact(c, universe, &c->bc->upd_short, &c->bc->upd_long, 1);
        read_bc(c);
        read_slots_start(c);
        c->pool_tail = (int64_t)c->h_bc->pool_tail;
        const int64_t relocated = c->h_bc->relocated;
        universe.ns = c->h_bc->upd_short;
        universe.nl = c->h_bc->upd_long;
        unsigned int known = c->h_slot[0].next_count + c->h_slot[0].next_long;  // |V_aff| the host knows of
        HIPCHK(c, hipEventRecord(c->phase_ev[2], c->stream));

        // ---- Step 3: rounds over V_aff, queued in chains of kChain rounds per host round trip ----
        const int64_t frontier_initial = known;
        int64_t peak = known, rows = 0, edges = 0;
        int it = 0, cur = 0;  // round `it` reads the frontier of parity `cur`
        float last = 0.f;
        double avg_len = c->n > 0 ? (double)c->entries / (double)c->n : 1.0;
        bool pingpong = false;
        int stretch_start = 0;  // first round of the running ping-pong stretch
        bool fused = false;     // the stretch's rounds evaluate V_aff themselves (no frontier list, no pull)
        bool binned = false;    // ... as scatter + gather passes (scalar labels)
        bool bin_failed = false;
        // Rounds that repeat themselves exactly (same |V_aff|, rows moved and max change, 16 times in a row) are in
        // a period-2 cycle kept alive by float32 rounding (in-place rounds too: the few rows of such a V_aff run side
        // by side in one wave and read each other's old values); the rest of the batch's flag-marking rounds then
        // average old and new row (kRowLazy), which has the same fixed point and no such cycle.
        int same_run = 0;
        bool lazy = false;
        unsigned int prev_sig[3] = {0xffffffffu, 0xffffffffu, 0xffffffffu};
        c->pb_built = false;    // the batch changed the graph
        c->persist_failed = false;
        c->persist_launches_last = c->persist_aborts_last = 0;
        const bool in_place = c->update_mode == DYNLP_UPDATE_IN_PLACE;
        // dynlp_set_final_check: when V_aff has emptied, one more round over every updatable row; rows it moves by
        // more than tol (and their neighbours) start Step 3 again.  check_round = index of the running check round.
        int final_checks = 0, check_round = -1;
        bool verified = !c->final_check;
        for (;;) {
        while (known > 0 && it < c->max_iter) {
            const int G = choose_group(c, avg_len);
            // A stretch of ping-pong rounds starts when V_aff covers nearly every updatable vertex (one copy
            // of F makes the partner buffer agree on every row outside V_aff) and ends when V_aff has shrunk.
            // Both kinds of round are correct for any V_aff, so the choice is only made between chains.
            // Inside a stretch no frontier list exists: its first round works on the list it was handed, the
            // later ones evaluate V_aff = {u : u or a neighbour moved in the previous round} per row, from
            // the bitmap of moved rows.  Leaving a stretch pulls the list out of the last bitmap once.
            bool can_bin = !bin_failed && binned_rounds_pay(c, universe);
            if (can_bin && !pingpong && !c->pb_built && (double)known >= kBinnedEnter * (double)universe.size() &&
                !build_binned(c)) {
                bin_failed = true;  // no memory for the binned arrays: ordinary rounds for this batch
                can_bin = false;
            }
            // graphs whose rounds run many per launch stay in one stretch from the first round to the last: a round
            // over a small V_aff costs them no more than a launch
            // (not once rounds repeat themselves exactly: the averaged rows that end such a cycle are staged rounds)
            const bool stay = !lazy && !can_bin && fused_rounds_pay(c, avg_len) && persistent_rounds_pay(c, universe);
            if (!pingpong && (stay || (double)known >= (can_bin ? kBinnedEnter : kDenseEnter) * (double)universe.size())) {
                if (!in_place) sync_partner(c);
                for (unsigned int* mv : c->moved)
                    HIPCHK(c, hipMemsetAsync(mv, 0, (size_t)c->moved_words * sizeof(unsigned int), c->stream));
                pingpong = true;
                stretch_start = it;
                binned = can_bin;
                fused = binned || fused_rounds_pay(c, avg_len);
            } else if (pingpong && !(stay && fused && !binned) &&
                       (double)known < (binned ? kBinnedLeave : kDenseLeave) * (double)universe.size()) {
                pingpong = false;
                if (fused) {
                    // rows of the last round are in F (the buffers were swapped to make it so)
                    const int last = it - 1 - stretch_start;
                    RoundCtr* slot = slot_of(c, it - 1);
                    launch_pull_frontier(c, universe, avg_len, c->moved[last % 3], c->moved[(last + 1) % 3], c->F,
                                         in_place ? nullptr : c->F2, frontier_of(c, cur), &slot->next_count, &slot->next_long);
                }
            }
            // a stretch of short rounds runs many rounds per launch (k_rounds_persistent); its first round, which still
            // works on a frontier list, is an ordinary launch
            const bool persist = pingpong && fused && !binned && persistent_rounds_pay(c, universe);
            const int r = std::min<int>(persist ? kPersistRounds : kChain, c->max_iter - it);
            const size_t first_pair = c->events_used / 2;
            // ping-pong: round it+i reads buf[i & 1], writes buf[(i + 1) & 1]; in place: always F
            float* const buf[2] = {c->F, in_place ? c->F : c->F2};
            bool persist_launched = false;
            int persist_first = r;  // chain position of the first round that ran inside a persistent launch
            for (int i = 0; i < r; ++i) {
                const int t = it + i;
                RoundCtr* slot = slot_of(c, t);
                const Frontier f = frontier_of(c, cur);
                if (pingpong) {
                    const int q = t - stretch_start;  // round of the stretch
                    if (!fused) {
                        // new rows go straight into the partner buffer; the next V_aff is pulled from the bitmap
                        // of rows that moved
                        unsigned int* mv = c->moved[q & 1];
                        const UpdateArgs a{slot_of(c, t - 1), 0, buf[i & 1], buf[(i + 1) & 1], mv, c->tol,
                                           slot, slot_of(c, t + 1), (int64_t)universe.size(), (int64_t)universe.nl};
                        launch_update<false>(c, G, f, a, t);
                        launch_pull_frontier(c, universe, avg_len, mv, c->moved[(q + 1) & 1], buf[(i + 1) & 1],
                                             in_place ? nullptr : buf[i & 1], frontier_of(c, cur ^ 1), &slot->next_count,
                                             &slot->next_long);
                        cur ^= 1;
                    } else if (q == 0) {
                        const UpdateArgs a{slot_of(c, t - 1), 0, buf[i & 1], buf[(i + 1) & 1], c->moved[0], c->tol,
                                           slot, slot_of(c, t + 1), (int64_t)universe.size(), (int64_t)universe.nl};
                        launch_update<false>(c, G, f, a, t);
                    } else {
                        c->ev_adjacent = i > 0;  // fused rounds of one chain follow each other with nothing in between
                        if (persist && !c->persist_failed) {
                            // rounds t .. it + r - 1 in one launch
                            PersistArgs pa;
                            pa.ring = c->ring;
                            pa.t0 = t;
                            pa.rounds = r - i;
                            pa.long_blocks_max = 0;
                            pa.front = universe.front;
                            pa.back = universe.back;
                            pa.ns = universe.ns;
                            pa.nl = universe.nl;
                            pa.meta = c->meta;
                            pa.pool = c->pool;
                            pa.buf0 = buf[i & 1];
                            pa.buf1 = buf[(i + 1) & 1];
                            pa.moved0 = c->moved[0];
                            pa.moved1 = c->moved[1];
                            pa.moved2 = c->moved[2];
                            pa.q0 = q;
                            pa.words = (unsigned int)c->moved_words;
                            pa.tol = c->tol;
                            pa.barrier = c->persist_ctl;
                            pa.spin_limit = c->persist_spin;
                            if (launch_persistent(c, G, universe, pa, t)) {
                                persist_launched = true;
                                persist_first = i;
                                ++c->persist_launches_last;
                                break;
                            }
                            c->persist_failed = true;  // refused: ordinary rounds for the rest of the chain and the batch
                        }
                        const PullRoundArgs a{slot_of(c, t - 1), buf[i & 1], buf[(i + 1) & 1], c->moved[(q - 1) % 3],
                                              c->moved[q % 3], c->moved[(q + 1) % 3], c->tol, slot, slot_of(c, t + 1)};
                        if (binned)
                            launch_binned_round(c, a, t, q == 1);
                        else
                            launch_update_pull(c, G, universe, a, t);
                    }
                } else {
                    // rows are staged by frontier position and committed after the kernel; rows that moved mark
                    // themselves and their neighbours
                    // (in-place mode: written straight into F, nothing to commit)
                    const UpdateArgs a{slot_of(c, t - 1), 0, c->F, in_place ? c->F : c->F2, nullptr, c->tol,
                                       slot, slot_of(c, t + 1), (int64_t)universe.size(), (int64_t)universe.nl,
                                       (in_place ? kRowByVertex : 0) | (lazy ? kRowLazy : 0)};
                    launch_update<true>(c, G, f, a, t);
                    if (!in_place) launch_commit(c, f, slot_of(c, t - 1), (int64_t)universe.size());
                    launch_compact(c, frontier_of(c, cur ^ 1), &slot->next_count, &slot->next_long, 0);
                    cur ^= 1;
                }
            }
            if (persist_launched) {
                // did a workgroup give up at the barrier?  (the rounds whose slots say "executed" are complete either way)
                unsigned int ctl[2] = {0, 0};
                HIPCHK(c, hipMemcpyAsync(ctl, c->persist_ctl, sizeof ctl, hipMemcpyDeviceToHost, c->stream));
                HIPCHK(c, hipStreamSynchronize(c->stream));
                if (ctl[1] != 0u) {
                    c->persist_failed = true;
                    ++c->persist_aborts_last;
                }
            }
            read_slots(c, it, r);
            int executed = 0;
            for (int i = 0; i < r; ++i) {
                const RoundCtr& rc = c->h_slot[i];
                if (!rc.executed) break;
                ++executed;
                const unsigned int nq = rc.rows_short + rc.rows_long;
                std::memcpy(&last, &rc.resid_bits, sizeof(float));
                rows += nq;
                edges += (int64_t)(rc.edges + rc.edges_long);
                avg_len = nq ? (double)(rc.edges + rc.edges_long) / (double)nq : avg_len;
                // the first round of a fused stretch still works on a frontier list
                c->log.push_back(round_info(rc, !pingpong ? 1 : (fused && it + i > stretch_start ? (binned ? 3 : i >= persist_first ? 4 : 2) : 0), G));
                // inside a stretch the next V_aff is not counted: this round's size stands in for it while
                // rows still move
                known = pingpong && fused ? (rc.changed ? std::max(nq, 1u) : 0u) : rc.next_count + rc.next_long;
                if (it + i == check_round) verified = rc.changed == 0u;  // the check round moved no row by more than tol
                const unsigned int sig[3] = {nq, rc.changed, rc.resid_bits};
                same_run = std::memcmp(sig, prev_sig, sizeof sig) == 0 ? same_run + 1 : 0;
                std::memcpy(prev_sig, sig, sizeof sig);
                if (same_run >= 16) lazy = true;
                peak = std::max<int64_t>(peak, known);
            }
            if (pingpong && !in_place && (executed & 1)) std::swap(c->F, c->F2);  // the output of the last executed round
            if (c->time_kernels) trim_timed_spans(c, first_pair, it + executed);
            // a persistent launch that gave up at a barrier stops short without V_aff being empty
            const bool cut_short = persist_launched && executed < r && executed > 0 && c->h_slot[executed - 1].changed != 0u;
            it += executed;
            if (cut_short) continue;
            if (executed < r) known = 0;  // a round found V_aff empty
        }
        if (verified || known > 0 || it >= c->max_iter || universe.size() == 0) break;
        // V_aff is empty: make every updatable vertex the frontier of round `it` (list into the current parity's
        // array, sizes into the slot the round reads them from; a slot past the last executed round is all zero)
        {
            pingpong = false;  // the check round starts a stretch of its own (fresh bitmaps, partner buffer in step)
            RoundCtr* slot = slot_of(c, it - 1);
            HIPCHK(c, hipMemsetAsync(slot, 0, sizeof(RoundCtr), c->stream));
            launch_compact(c, frontier_of(c, cur), &slot->next_count, &slot->next_long, 1);
            known = universe.size();
            check_round = it;
            ++final_checks;
        }
        }
        // not converged: max_iter cut the rounds, or cut them before a requested final check had passed
        const unsigned int nq = known > 0 ? known : (verified || universe.size() == 0 ? 0u : 1u);
        HIPCHK(c, hipEventRecord(c->phase_ev[3], c->stream));
        HIPCHK(c, hipStreamSynchronize(c->stream));
        const float kernel_ms_total = c->time_kernels ? collect_kernel_ms(c) : 0.f;
        if (c->last_init.vertices > 0) (void)hipEventElapsedTime(&c->last_init.ms, c->init_ev[0], c->init_ev[1]);
        if (stats) {
            stats->iterations = it;
            stats->converged = nq == 0 ? 1 : 0;
            stats->final_max_delta = last;
            stats->rows_updated = rows;
            stats->edges_traversed = edges;
            stats->frontier_initial = frontier_initial;
            stats->frontier_peak = peak;
            stats->rows_relocated = relocated;
            stats->update_launches = it;
            stats->final_checks = final_checks;
            stats->ingest_chunks = c->ingest_pinned_last ? c->ingest_chunks_last : -c->ingest_chunks_last;
            stats->ms_update_kernel = kernel_ms_total;
            (void)hipEventElapsedTime(&stats->ms_insert, c->phase_ev[0], c->phase_ev[1]);
            (void)hipEventElapsedTime(&stats->ms_seed, c->phase_ev[1], c->phase_ev[2]);
            (void)hipEventElapsedTime(&stats->ms_iterate, c->phase_ev[2], c->phase_ev[3]);
            stats->ms_total = ms_since(t0);
        }
        reset_timed_spans(c);
        return nq == 0 ? DYNLP_OK : DYNLP_NOT_CONVERGED;
    } catch (const Fail& f) {
        if (mutated) c->poisoned = true;
        return f.st;
    } catch (const std::bad_alloc&) {
        c->err = "host allocation failed";
        if (mutated) c->poisoned = true;
        return DYNLP_ERR_OOM;
    }
}

dynlp_status dynlp_get_labels(dynlp_ctx* c, float* soft, int32_t* hard) {
    if (!c) return DYNLP_ERR_INVALID_ARG;
    if (c->poisoned) {
        c->err = "context is unusable after an earlier device or memory error";
        return DYNLP_ERR_STATE;
    }
    const int64_t n = c->n;
    if (n == 0 || (!soft && !hard)) return DYNLP_OK;
    float* d_soft = nullptr;
    int32_t* d_hard = nullptr;
    dynlp_status st = DYNLP_OK;
    try {
        HIPCHK(c, hipSetDevice(c->device));
        // staging of the packed outputs in host-pointer mode; without memory for it the call fails and the context
        // stays usable
        if (soft && !c->dev_ptrs) d_soft = Temp<float>(c, n * c->C).release();
        if (hard && !c->dev_ptrs) d_hard = Temp<int32_t>(c, n).release();
        float* dst_soft = !soft ? nullptr : c->dev_ptrs ? soft : d_soft;
        int32_t* dst_hard = !hard ? nullptr : c->dev_ptrs ? hard : d_hard;
        launch_label_output(c, dst_soft, dst_hard);
        if (!c->dev_ptrs) {
            if (soft) HIPCHK(c, hipMemcpyAsync(soft, dst_soft, (size_t)n * c->C * sizeof(float), hipMemcpyDeviceToHost, c->stream));
            if (hard) HIPCHK(c, hipMemcpyAsync(hard, dst_hard, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
        }
        HIPCHK(c, hipStreamSynchronize(c->stream));
    } catch (const SoftOom&) {
        st = DYNLP_ERR_OOM;
    } catch (const Fail& f) {
        st = f.st;
    }
    dev_free(c, d_soft);
    dev_free(c, d_hard);
    return st;
}

int64_t dynlp_static_scratch_bytes(void) { return (int64_t)kStaticScratchBytes; }

dynlp_status dynlp_get_labels_static(dynlp_ctx* c, float* soft, int32_t* hard) {
    if (!c) return DYNLP_ERR_INVALID_ARG;
    if (c->poisoned) {
        c->err = "context is unusable after an earlier device or memory error";
        return DYNLP_ERR_STATE;
    }
    const int64_t n = c->n;
    if (n == 0 || (!soft && !hard)) return DYNLP_OK;
    // staging layout: [soft: n*C floats][padding to 256 bytes][hard: n int32]
    const size_t soft_bytes = soft ? (size_t)n * c->C * sizeof(float) : 0;
    const size_t hard_off = (size_t)round_up((int64_t)soft_bytes, 256);
    const size_t need = hard_off + (hard ? (size_t)n * sizeof(int32_t) : 0);
    if (need > kStaticScratchBytes) {
        c->err = "dynlp_get_labels_static: the labels of " + std::to_string(n) + " vertices need " + std::to_string(need) +
                 " bytes of staging, the static scratch holds " + std::to_string(kStaticScratchBytes) +
                 "; use dynlp_get_labels";
        return DYNLP_ERR_INVALID_ARG;
    }
    void* base = c->device >= 0 && c->device < kMaxDevices ? g_scratch_ptr[c->device] : nullptr;
    if (!base) {
        c->err = std::string("dynlp_get_labels_static: the address of the static scratch could not be resolved on this device (") +
                 (c->device >= 0 && c->device < kMaxDevices ? hipGetErrorString(g_scratch_err[c->device]) : "device ordinal too large") + ")";
        return DYNLP_ERR_DEVICE;
    }
    try {
        HIPCHK(c, hipSetDevice(c->device));
        float* d_soft = soft ? static_cast<float*>(base) : nullptr;
        int32_t* d_hard = hard ? reinterpret_cast<int32_t*>(static_cast<unsigned char*>(base) + hard_off) : nullptr;
        launch_label_output(c, d_soft, d_hard);
        if (soft) HIPCHK(c, hipMemcpyAsync(soft, d_soft, soft_bytes, hipMemcpyDeviceToHost, c->stream));
        if (hard) HIPCHK(c, hipMemcpyAsync(hard, d_hard, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
        HIPCHK(c, hipStreamSynchronize(c->stream));
        return DYNLP_OK;
    } catch (const Fail& f) {
        return f.st;
    }
}

dynlp_status dynlp_export_graph(dynlp_ctx* c, int64_t* row_ptr, int32_t* col, float* w, float* degree,
                                int32_t* seed_class) {
    if (!c) return DYNLP_ERR_INVALID_ARG;
    if (c->poisoned) {
        c->err = "context is unusable after an earlier device or memory error";
        return DYNLP_ERR_STATE;
    }
    if (!row_ptr || (c->entries > 0 && (!col || !w))) {
        c->err = "row_ptr / col / w are NULL";
        return DYNLP_ERR_INVALID_ARG;
    }
    const int64_t n = c->n, nnz = c->entries;
    int64_t *d_rp = nullptr, *sums = nullptr;
    int32_t* d_col = nullptr;
    float* d_w = nullptr;
    dynlp_status st = DYNLP_OK;
    const hipMemcpyKind kind = c->dev_ptrs ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost;
    try {
        HIPCHK(c, hipSetDevice(c->device));
        const int64_t nb = grid_for(n);
        d_rp = Temp<int64_t>(c, n + 1).release();
        sums = Temp<int64_t>(c, nb).release();
        int64_t total = 0;
        if (n > 0) {
            hipLaunchKernelGGL(k_row_lens, dim3(nb), dim3(kBlock), 0, c->stream, n, c->meta, d_rp, sums);
            HIPCHK(c, hipGetLastError());
            total = scan_block_sums(c, nb, sums);
            hipLaunchKernelGGL(k_lens_to_row_ptr, dim3(nb), dim3(kBlock), 0, c->stream, n, d_rp, sums);
            HIPCHK(c, hipGetLastError());
        }
        HIPCHK(c, hipMemcpyAsync(d_rp + n, &total, sizeof(int64_t), hipMemcpyHostToDevice, c->stream));
        if (total != nnz) {
            c->err = "internal: entry count mismatch";
            throw Fail{DYNLP_ERR_STATE};
        }
        if (nnz > 0) {
            int32_t* ocol = c->dev_ptrs ? col : (d_col = Temp<int32_t>(c, nnz).release());
            float* ow = c->dev_ptrs ? w : (d_w = Temp<float>(c, nnz).release());
            hipLaunchKernelGGL(k_export_rows, dim3(grid_for(n * 16)), dim3(kBlock), 0, c->stream, n, c->meta, c->pool, d_rp,
                               ocol, ow);
            HIPCHK(c, hipGetLastError());
            if (!c->dev_ptrs) {
                HIPCHK(c, hipMemcpyAsync(col, ocol, (size_t)nnz * 4, hipMemcpyDeviceToHost, c->stream));
                HIPCHK(c, hipMemcpyAsync(w, ow, (size_t)nnz * 4, hipMemcpyDeviceToHost, c->stream));
            }
        }
        HIPCHK(c, hipMemcpyAsync(row_ptr, d_rp, (size_t)(n + 1) * sizeof(int64_t), kind, c->stream));
        if (degree && n > 0) HIPCHK(c, hipMemcpyAsync(degree, c->deg, (size_t)n * sizeof(float), kind, c->stream));
        if (seed_class && n > 0)
            HIPCHK(c, hipMemcpyAsync(seed_class, c->seed_class, (size_t)n * sizeof(int32_t), kind, c->stream));
        HIPCHK(c, hipStreamSynchronize(c->stream));
    } catch (const SoftOom&) {
        (void)hipStreamSynchronize(c->stream);
        st = DYNLP_ERR_OOM;
    } catch (const Fail& f) {
        st = f.st;
    }
    dev_free(c, d_rp);
    dev_free(c, sums);
    dev_free(c, d_col);
    dev_free(c, d_w);
    return st;
}

int64_t dynlp_round_log(const dynlp_ctx* ctx, int64_t cap, dynlp_round_info* out) {
    if (!ctx) return -1;
    const int64_t rounds = (int64_t)ctx->log.size();
    const int64_t k = std::max<int64_t>(0, std::min(cap, rounds));
    if (out && k > 0) std::copy(ctx->log.begin(), ctx->log.begin() + k, out);
    return rounds;
}

}  // extern "C"
