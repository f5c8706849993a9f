/*
 * dynlp.h — C ABI of libdynlp: dynamic batched label propagation (DynLP) on one AMD MI355X.
 *
 * The library keeps, in device memory, a weighted undirected graph G=(V,E) in a mutable CSR
 * with per-row slack, the set V^L of labelled (seed) vertices with their classes, and the
 * n x C label matrix F (row u = class distribution of vertex u; the paper's binary scalar label
 * is column 1 of the C=2 case).  It offers
 *   - the static iterative label propagation ItLP (paper Eq. (1)) as the cold start, and
 *   - the batch update of Alg. 2 ("DynLP Update"): insert the batch's vertices and edges
 *     (Step 1), mark the affected set V_aff, and run the frontier-restricted propagation of
 *     Step 3 until V_aff is empty.
 * Every step runs in hand-written HIP kernels for gfx950; there is no CPU fallback: without a
 * usable GPU every call that needs one returns DYNLP_ERR_DEVICE.
 *
 * Conventions
 *   - All functions are thread-compatible: one context must not be used from two threads at
 *     once; different contexts are independent.
 *   - Pointer arguments are HOST pointers unless the context was created with
 *     dynlp_options.ptrs_on_device = 1, in which case every array argument of every call
 *     (inputs and outputs) is a DEVICE pointer on the context's device.  Scalars, the options
 *     and the stats struct are always host memory.
 *   - The caller owns every buffer it passes; the library copies what it needs and keeps no
 *     caller pointer after a call returns.
 *   - Work is enqueued on dynlp_options.stream (a hipStream_t; NULL = the default stream).  Each
 *     call returns after that work has completed, so outputs are readable on return.
 *   - No C++ exception crosses this boundary.  A failed call leaves the context as it was
 *     before the call (arguments are validated before anything is changed), except for
 *     DYNLP_ERR_OOM / DYNLP_ERR_DEVICE, after which the context may only be destroyed.
 *   - Indices are int32 vertex ids; sizes are int64.  Weights and labels are IEEE binary32.
 */
#ifndef DYNLP_H
#define DYNLP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DYNLP_MAX_CLASSES 64 /* largest num_classes the row-update kernel is laid out for */

typedef struct dynlp_ctx dynlp_ctx; /* opaque; owns all device memory it allocates */

typedef enum dynlp_status {
    DYNLP_OK = 0,
    DYNLP_NOT_CONVERGED = 1,    /* max_iter reached; labels are valid but not converged */
    DYNLP_ERR_INVALID_ARG = -1, /* see dynlp_last_error for which argument and why */
    DYNLP_ERR_OOM = -2,         /* device or host allocation failed */
    DYNLP_ERR_DEVICE = -3,      /* no usable GPU, or a HIP call failed */
    DYNLP_ERR_STATE = -4        /* call not allowed in the context's current state */
} dynlp_status;

/* Counters and timings of the last dynlp_static_solve / dynlp_apply_batch (host memory). */
typedef struct dynlp_stats {
    int32_t iterations;       /* propagation rounds executed */
    int32_t converged;        /* 1 if the stop rule was met, 0 if max_iter cut it */
    float final_max_delta;    /* max_u max_c |F'_u - F_u| of the last round */
    int64_t rows_updated;     /* sum over rounds of |V_aff| */
    int64_t edges_traversed;  /* sum over rounds and frontier rows of the row length */
    int64_t frontier_initial; /* |V_aff| after Step 1 (static solve: number of updatable rows) */
    int64_t frontier_peak;
    int64_t rows_relocated;   /* rows moved to the pool tail because their slack ran out */
    int64_t update_launches;  /* launches of the row-update kernel */
    float ms_update_kernel;   /* summed device time of those launches (HIP events on the stream);
                                 0 unless dynlp_options.time_kernels is set */
    float ms_insert;          /* validation + edge insertion + degree update */
    float ms_seed;            /* seed clamping + frontier seeding + first compaction */
    float ms_iterate;         /* the propagation loop */
    float ms_total;           /* whole call, host wall clock */
    int32_t final_checks;     /* rounds over all updatable rows that dynlp_set_final_check added (0 when it is off) */
    int32_t ingest_chunks;    /* chunks a host-resident edge list was sent in while earlier chunks were being validated
                                 and counted (dynlp_options.ingest_chunk_edges); 0: one plain copy, or device pointers;
                                 negative: the caller's arrays were pageable and went through the pinned staging */
} dynlp_stats;

typedef struct dynlp_options {
    int32_t device;          /* HIP device ordinal */
    void* stream;            /* hipStream_t to enqueue on; NULL = default stream */
    int32_t ptrs_on_device;  /* 0: array arguments are host pointers; 1: device pointers */
    float slack_factor;      /* row capacity = max(ceil(len*slack_factor), len+4), rounded up to 8
                                entries; <= 1 selects the default 1.25 */
    int64_t reserve_vertices; /* room for this many vertices beyond n before arrays regrow */
    int64_t reserve_edges;    /* room for this many extra undirected edges at the pool tail */
    int32_t time_kernels;    /* 1: bracket every row-update launch with HIP events */
    int32_t group_lanes;     /* lanes cooperating on one frontier row: 0 = choose from the mean
                                row length, else 4, 8, 16, 32 or 64 (tuning knob) */
    /* Optional allocator for device memory (e.g. a caching allocator); all three NULL selects
       hipMalloc/hipFree.  alloc returns NULL on failure. */
    void* (*alloc)(size_t bytes, void* user);
    void (*dealloc)(void* ptr, void* user);
    void* alloc_user;
    int32_t binary_scalar;   /* 1 (needs num_classes == 2): keep one float per vertex, the paper's scalar
                                label F_u in [0,1] = weight of class 1 (seeds 0 or 1, neutral start 0.5,
                                hard label by the 0.5 cut-off); dynlp_get_labels still returns n x 2 rows
                                (1 - F_u, F_u).  0: n x C rows */
    int32_t binned_rounds;   /* scalar labels only (tuning knob): rounds over nearly all vertices as two streaming
                                passes (scatter labels into bins of receivers, gather per bin) instead of row
                                updates with random gathers.  0: the library decides (graphs of 2M updatable
                                vertices or more); -1: never; 8..15: always, with 2^k receivers per bin */
    int32_t persistent_rounds; /* tuning knob, off by default: 1 = run the rounds of a batch up to 32 per launch, with a
                                barrier across a grid of workgroups that are all resident at once between rounds (for
                                graphs so small that a round is shorter than a launch and its drain; the batch's
                                rounds then all evaluate V_aff per row themselves).  0 or -1: one launch per round.
                                On MI355X it does not pay yet: see the note at persistent_rounds_pay in the source */
    int32_t persistent_spin_limit; /* polls a workgroup waits at that barrier before it gives up (0 = default 2^20, about
                                a quarter of a second).  A workgroup that gives up makes the launch end after the round
                                in progress; the batch continues with one launch per round */
    int64_t ingest_chunk_edges; /* host pointers only: an insertion batch (no deletions) with more edges than this is
                                sent to the device chunk by chunk on a second stream while the chunks that have
                                arrived are validated and counted (the paper's overlap of batch transfer and Step 1
                                kernels, "Overlapping subgraph transfer and kernel execution").  Arrays in pinned host
                                memory are sent as they are; pageable arrays pass through two pinned staging buffers
                                of 12 bytes per chunk edge.  0 selects the default, 4,194,304 edges */
} dynlp_options;

/* Fill *opt with the defaults (device 0, default stream, host pointers). */
void dynlp_default_options(dynlp_options* opt);

/*
 * Build a context from a weighted undirected graph, a seed set and a class count
 * (the inputs of Alg. 2: G_t, F^L; problem statement in "Preliminaries").
 *   n            number of vertices (>= 0)
 *   row_ptr      n+1 ascending offsets, row_ptr[0] = 0           (CSR, both directions of every
 *   col, w       row_ptr[n] neighbour ids and positive weights    edge present: the graph is
 *                                                                undirected; not verified)
 *   num_classes  C, 1 <= C <= DYNLP_MAX_CLASSES
 *   seed_vertex, seed_class   num_seeds labelled vertices and their classes in [0, C)
 *   opt          NULL = defaults
 * Seed rows of F start one-hot, all other rows uniform 1/C.  The CSR is copied into the slack
 * layout; the caller's arrays are not referenced afterwards.
 * DYNLP_ERR_INVALID_ARG on: NULL required pointer, n < 0, n > 2^31-2, C out of range,
 * non-monotone row_ptr, neighbour id outside [0,n), self loop, weight not finite or <= 0,
 * seed vertex / class out of range, the same vertex listed with two different classes.
 * On failure *out is NULL and dynlp_last_error(NULL) describes the problem.
 */
dynlp_status dynlp_create(dynlp_ctx** out, int64_t n, const int64_t* row_ptr, const int32_t* col, const float* w,
                          int32_t num_classes, int64_t num_seeds, const int32_t* seed_vertex,
                          const int32_t* seed_class, const dynlp_options* opt);

/*
 * Static ItLP (Eq. (1)): sweeps (Jacobi, or in place: see dynlp_set_update_mode) over all unlabelled rows
 * with d(u) > 0, starting from the current F, until max_u max_c |F^(k+1) - F^(k)| <= tol or max_iter sweeps.  Also stores tol and
 * max_iter for later dynlp_apply_batch calls.  tol >= 0, max_iter >= 0.  stats may be NULL.
 */
dynlp_status dynlp_static_solve(dynlp_ctx* ctx, float tol, int32_t max_iter, dynlp_stats* stats);

/* Set the threshold delta and the round cap used by dynlp_apply_batch (defaults 1e-4, 100000). */
dynlp_status dynlp_set_params(dynlp_ctx* ctx, float tol, int32_t max_iter);

/*
 * How the rows of one propagation round see each other (Eq. (1) is written with iteration indices,
 * Alg. 2 Step 3 updates F_u inside a parallel loop over V_aff).
 *   DYNLP_UPDATE_SYNCHRONOUS  (default) every row of a round is computed from the labels the round
 *       started with (Jacobi); for a given edge order results are reproducible round by round.
 *   DYNLP_UPDATE_IN_PLACE     a new row replaces the old one at once and later rows of the same round
 *       may already read it, as in the parallel loop of Alg. 2 executed literally.  Same fixed point
 *       and same stop rule (a row leaves V_aff when it moves by <= tol), about 1.5x fewer rounds, no
 *       second label buffer traffic; which mix of old and new neighbour rows a row reads depends on
 *       scheduling, so two runs agree only within the convergence tolerance, not bit for bit.
 * Applies to dynlp_static_solve and dynlp_apply_batch calls that follow.
 */
typedef enum dynlp_update_mode { DYNLP_UPDATE_SYNCHRONOUS = 0, DYNLP_UPDATE_IN_PLACE = 1 } dynlp_update_mode;
dynlp_status dynlp_set_update_mode(dynlp_ctx* ctx, int32_t mode);

/*
 * A guarantee on top of Alg. 2 Step 3 (off by default; the paper stops when V_aff is empty).  Step 3 stops row by
 * row: a row leaves V_aff once it moves by <= tol, and afterwards its neighbours may each keep moving by just under
 * tol per round without bringing it back, so the labels a batch ends with can sit further than tol from satisfying
 * Eq. (1) (the paper reports the effect as hard-label accuracy below 100% for large batches).  With the check on,
 * every time V_aff empties dynlp_apply_batch / dynlp_apply_update run one more round with V_aff = all updatable
 * vertices; if it moves no row by more than tol the call ends, else Step 3 continues from the rows it moved.  The
 * call then ends in the state a static solve ends in: one sweep of Eq. (1) moves no row by more than tol, hence
 * every row is within tol * ||(I - P_UU)^{-1}||_inf of the exact harmonic labels (convergence corollary), where the
 * norm is the largest expected number of random-walk steps to a labelled vertex.  Costs one round over all rows
 * per check (dynlp_stats.final_checks counts them).
 */
dynlp_status dynlp_set_final_check(dynlp_ctx* ctx, int32_t on);

/*
 * Starting rows of the vertices a batch inserts (Alg. 2 Step 1 "sparsification" and Step 2 "label
 * initialisation").  It changes where Step 3 starts, not the labels it converges to.
 *   DYNLP_INIT_UNIFORM    every inserted unlabelled row starts at 1/C (the paper's neutral 0.5).
 *   DYNLP_INIT_SUPERNODE  the batch edges whose two ends are both inserted by this batch and whose
 *                         weight is > tau form the graph G'; each connected component of G' (over all
 *                         inserted vertices; a vertex without such an edge is its own component) is
 *                         a supernode c_i; W[c_i][j] = summed weight of the updated graph's edges
 *                         from any member of c_i to any vertex labelled j (old or new); every
 *                         unlabelled member starts at W[c_i][j] / sum_j W[c_i][j], or 1/C when that
 *                         sum is 0.  For C = 2 column 1 is the paper's
 *                         0.5 - W^{L0}/(2(W^{L0}+W^{L1})) + W^{L1}/(2(W^{L0}+W^{L1})).
 * tau (finite, >= 0; ignored for DYNLP_INIT_UNIFORM): the paper's experiments use the mean edge
 * weight of the data set, which dynlp_mean_edge_weight returns for the graph currently stored.
 * Each listed batch edge is tested on its own weight.  Default: DYNLP_INIT_UNIFORM.
 */
typedef enum dynlp_init_mode { DYNLP_INIT_UNIFORM = 0, DYNLP_INIT_SUPERNODE = 1 } dynlp_init_mode;
dynlp_status dynlp_set_initialiser(dynlp_ctx* ctx, int32_t mode, float tau);

/* Mean weight over the stored CSR entries (= mean over undirected edges), summed in binary64 in a
 * fixed order; 0 for an empty graph.  mean is host memory. */
dynlp_status dynlp_mean_edge_weight(dynlp_ctx* ctx, double* mean);

/* What the supernode initialisation of the last dynlp_apply_batch did (all zero when it did not
 * run: uniform mode, or a batch without new vertices). */
typedef struct dynlp_init_info {
    int64_t vertices;    /* inserted vertices = vertices of G' */
    int64_t kept_edges;  /* |E'|: batch-internal edges with weight > tau */
    int64_t components;  /* connected components of G' */
    int32_t hook_steps;  /* hook/jump iterations of the component search, the final no-change one included */
    float ms;            /* device time of the whole initialisation (part of dynlp_stats.ms_seed) */
} dynlp_init_info;

/*
 * Components found by the last dynlp_apply_batch in DYNLP_INIT_SUPERNODE mode (the set C of Alg. 2):
 * comp[i] = component of inserted vertex i (i-th new id of that batch), numbered 0..components-1 in
 * ascending order of each component's smallest member.  comp (cap >= vertices entries; device or
 * host memory like every array argument) may be NULL to fetch only *info (host memory, may be NULL).
 */
dynlp_status dynlp_last_components(dynlp_ctx* ctx, int64_t cap, int32_t* comp, dynlp_init_info* info);

/*
 * DynLP update for one insertion batch (Alg. 2 Steps 1 and 3).
 *   num_new_vertices   they receive ids n .. n+k-1 in order; rows start as dynlp_set_initialiser chose
 *   eu, ev, ew         num_new_edges undirected edges, each listed once, endpoints in [0, n+k),
 *                      eu != ev, weight finite and > 0; an edge that already exists is legal
 *                      and adds its weight (parallel edge)
 *   seed_vertex/class  num_new_seeds vertices (old or new) that are labelled from now on
 * Step 1: both directions of every edge are appended to their rows (rows whose slack is
 * exhausted move to the pool tail with fresh slack; the appended entries of a row are then put in
 * ascending (neighbour id, weight bits) order, so the stored graph does not depend on timing); degrees are updated; new seeds are clamped
 * one-hot; V_aff = inserted vertices, endpoints of inserted edges and neighbours of new seeds,
 * without seeds and isolated vertices.  Step 3: rounds of F'_u = sum_v w(u,v) F_v / d(u) for
 * u in V_aff from the round-start F; every F'_u is stored; u with max_c |F'_u - F_u| > tol
 * puts itself and N(u) into the next V_aff; stops when V_aff is empty (DYNLP_OK) or after
 * max_iter rounds (DYNLP_NOT_CONVERGED).
 * One safeguard beyond the paper: when 16 consecutive rounds repeat exactly (same |V_aff|, same
 * number of rows moved, same max change) the iteration is in a period-2 cycle that float32
 * rounding keeps alive (a nearly bipartite, weakly tied component); the batch's remaining rounds on
 * small V_aff then store the mean of the old row and F'_u, which has the same fixed point.
 * dynlp_static_solve does the same when the max change of 16 consecutive sweeps is one number.
 * DYNLP_ERR_INVALID_ARG (context unchanged) on: negative counts, NULL array with a positive
 * count, endpoint out of range, self loop, bad weight, seed vertex/class out of range, a vertex
 * given two different classes, relabelling an existing seed with another class.
 */
dynlp_status dynlp_apply_batch(dynlp_ctx* ctx, int64_t num_new_vertices, int64_t num_new_edges, const int32_t* eu,
                               const int32_t* ev, const float* ew, int64_t num_new_seeds,
                               const int32_t* seed_vertex, const int32_t* seed_class, dynlp_stats* stats);

/*
 * DynLP update for one batch with deletions and insertions (Alg. 2 Steps 1 and 3 in full; Delta_t =
 * {Delta^Ins, Delta^Del}).  dynlp_apply_batch is this call with num_deleted = 0; the insertion
 * arguments, Step 3, the statuses and the stats are the same.
 *   deleted_vertex   num_deleted ids of existing vertices (in [0, n) as of before the call; an id
 *                    listed twice is deleted once)
 * Deletions are applied first: every neighbour of a deleted vertex joins V_aff (V_aff <- V_aff U
 * N(u)); all edges of the deleted vertex are removed from both sides (the order of the remaining
 * entries of a row is kept).  Ids are never renumbered: the deleted vertex stays behind as an
 * isolated, unlabelled vertex whose row is 1/C (a deleted seed stops being a seed); it is never
 * updated, and the insertion part of this or a later batch may give it edges again.  A vertex that
 * loses its last edge keeps the label it has.  The pool space of removed entries is not reclaimed.
 * Seed arguments are validated against the state before the call.
 * DYNLP_ERR_INVALID_ARG (context unchanged) additionally on: deleted vertex out of range.
 */
dynlp_status dynlp_apply_update(dynlp_ctx* ctx, int64_t num_deleted, const int32_t* deleted_vertex,
                                int64_t num_new_vertices, int64_t num_new_edges, const int32_t* eu,
                                const int32_t* ev, const float* ew, int64_t num_new_seeds,
                                const int32_t* seed_vertex, const int32_t* seed_class, dynlp_stats* stats);

/*
 * Current labels.  soft: n*C floats row-major (no padding), or NULL.  hard: n int32 =
 * argmax_c F[u][c] with the lowest class index winning ties (for C=2 the paper's 0.5 cut-off), or
 * NULL.  Seed rows are exactly one-hot.
 */
dynlp_status dynlp_get_labels(dynlp_ctx* ctx, float* soft, int32_t* hard);

/*
 * dynlp_get_labels for callers that cannot allocate device memory: code between two stream-capture calls of
 * another part of the program, tight serving loops, harnesses that forbid hipMalloc.  Same results as
 * dynlp_get_labels, bit for bit, but soft and hard are always HOST pointers (whatever ptrs_on_device says), and
 * the device-side staging of the packed rows (soft: n*C floats, then, from the next multiple of 256 bytes, hard:
 * n int32) lives in a static device array of DYNLP_STATIC_SCRATCH_BYTES instead of an allocated buffer.  The call
 * makes no hipMalloc / hipFree and calls no allocator callback.
 *   - A request whose staging exceeds DYNLP_STATIC_SCRATCH_BYTES is rejected with DYNLP_ERR_INVALID_ARG (nothing
 *     is written); dynlp_get_labels has no such limit.  Passing only one of soft / hard halves the need.
 *   - Every context on one GPU shares that GPU's array, which keeps the previous call's contents; each call
 *     overwrites exactly the part it then copies out.  Two calls that overlap in time on one GPU (two threads, two
 *     contexts) race on it: serialise them.
 *   - The array's address is looked up once per GPU, in the first dynlp_create on that GPU; if that look-up
 *     failed the call returns DYNLP_ERR_DEVICE.
 *   - The copies to soft / hard are asynchronous only for pinned host memory; the call returns after they are done.
 * dynlp_static_scratch_bytes returns DYNLP_STATIC_SCRATCH_BYTES as compiled into the library.
 */
#define DYNLP_STATIC_SCRATCH_BYTES (16u << 20)
dynlp_status dynlp_get_labels_static(dynlp_ctx* ctx, float* soft, int32_t* hard);
int64_t dynlp_static_scratch_bytes(void);

/* Current number of vertices / directed CSR entries (2x the undirected edge count); -1 on NULL. */
int64_t dynlp_num_vertices(const dynlp_ctx* ctx);
int64_t dynlp_num_entries(const dynlp_ctx* ctx);
int32_t dynlp_num_classes(const dynlp_ctx* ctx);

/*
 * Copy the graph out as a compact CSR (inspection and tests): row_ptr n+1 offsets, col/w
 * dynlp_num_entries() entries in stored order (within a row: the entries given to dynlp_create in
 * their order, then batch by batch the entries that batch added, each batch's in ascending order
 * of (neighbour id, weight bit pattern); deletions keep the order of what remains); degree: n floats d(u) as maintained by the
 * insertion step, or NULL; seed_class: n int32, -1 for unlabelled, or NULL.
 */
dynlp_status dynlp_export_graph(dynlp_ctx* ctx, int64_t* row_ptr, int32_t* col, float* w, float* degree,
                                int32_t* seed_class);

/*
 * Storage of the mutable CSR.  Rows that outgrow their slack move to the end of the entry pool and
 * deleted entries are only dropped from their rows, so the pool's used part grows with every batch
 * even when the graph does not.  dynlp_storage_info reports the used part and the capacity (in
 * entries of 8 bytes; either pointer may be NULL; host memory).  dynlp_compact_storage lays all rows
 * out again in id order, each with fresh slack, in a new pool of the size that needs (plus a quarter
 * for growth) and releases the old one; graph, labels and every later result are unchanged.  It needs
 * room for both pools at once.
 */
dynlp_status dynlp_storage_info(const dynlp_ctx* ctx, int64_t* pool_used, int64_t* pool_capacity);
dynlp_status dynlp_compact_storage(dynlp_ctx* ctx);

/*
 * Yardsticks for bandwidth figures, measured on the context's stream with two temporary device
 * buffers of `bytes` bytes (rounded down to 16): `repetitions` launches of a plain float4 streaming
 * copy -> *copy_gb_per_s = (bytes read + bytes written) / time; then of a read-only pass that sums
 * what it reads -> *read_gb_per_s = bytes read / time.  Both outputs are host memory, either may be
 * NULL.
 */
dynlp_status dynlp_stream_bandwidth(dynlp_ctx* ctx, int64_t bytes, int32_t repetitions, double* copy_gb_per_s,
                                    double* read_gb_per_s);

/*
 * Yardstick for the neighbour-row gathers of the row update (Alg. 2 Step 3 reads one label row per CSR entry):
 * `repetitions` launches of a kernel that reads `gathers` whole rows of `row_bytes` bytes (16, 32, 64, 128 or 256:
 * the stored row sizes of 4 ... 64 label columns) at pseudo-random places of a temporary table of `table_rows` rows,
 * eight rows in flight per lane group, with no other memory traffic.  *gathers_per_s = rows read per second,
 * *gb_per_s = that times row_bytes; both host memory, either may be NULL.  With table_rows = the number of vertices
 * it is the ceiling of a sweep over a graph without locality.
 */
dynlp_status dynlp_gather_bandwidth(dynlp_ctx* ctx, int64_t table_rows, int32_t row_bytes, int64_t gathers,
                                    int32_t repetitions, double* gathers_per_s, double* gb_per_s);

/* One propagation round of the last dynlp_static_solve / dynlp_apply_batch. */
typedef struct dynlp_round_info {
    int64_t rows_short;    /* |V_aff| of the round, split by how the row was updated: rows of at most 128 */
    int64_t rows_long;     /* entries (a few lanes per row) and longer rows (a workgroup per row)        */
    int64_t entries_short; /* CSR entries those rows hold */
    int64_t entries_long;
    int64_t rows_moved;    /* rows with max_c |F'_u - F_u| > tol */
    float max_delta;       /* max_u max_c |F'_u - F_u| */
    float ms_update;       /* device time of the round's row-update launch (0 unless time_kernels) */
    float reserved;
    int32_t staged;        /* 1: the round marked the next V_aff in per-vertex flags from inside the update
                              kernel (synchronous mode: rows staged by position and committed after the
                              kernel); 0: rows written by vertex and the next V_aff pulled from a bitmap of
                              moved rows (static sweeps, rounds over nearly all vertices); 2: as 0, but the
                              round ran over all updatable vertices and decided per row, from the previous
                              round's bitmap, whether the row is in V_aff (no frontier list in between); 3: as 2,
                              as a binned round (scalar labels: scatter pass + gather pass, see
                              dynlp_options.binned_rounds); 4: as 2, one of several rounds run by one launch
                              (dynlp_options.persistent_rounds; ms_update is that launch's time divided by its rounds) */
    int32_t group_lanes;   /* lanes per row the short-row kernel ran with */
} dynlp_round_info;

/*
 * Per-round log of the last solve / batch: copies the first min(rounds, cap) entries to out (HOST
 * memory regardless of ptrs_on_device; may be NULL).  Returns the number of rounds executed.
 */
int64_t dynlp_round_log(const dynlp_ctx* ctx, int64_t cap, dynlp_round_info* out);

/* Message for the last failed call on ctx (or, with ctx NULL, the last failed dynlp_create on this
 * thread).  Valid until the next call on the same context / thread.  Never NULL. */
const char* dynlp_last_error(const dynlp_ctx* ctx);

/* Release the context and all device memory it owns.  NULL is allowed. */
void dynlp_destroy(dynlp_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* DYNLP_H */
