/*
 * libpancake -- C ABI of the MI355X (gfx950) IVF search / insert hot path.
 *
 * What is computed (paper sections, restated):
 *   Section 2.2   An IVF index partitions vectors into clusters ("lists").  A query
 *                 ranks the clusters by the distance between their centroids and
 *                 itself (coarse search), keeps the best `nprobe`, and searches those
 *                 clusters vector by vector (fine search), returning the best `k`.
 *   Section 3.1 / Section 6.1 ("IVF-Static")
 *                 A new vector is appended to the cluster of its nearest centroid;
 *                 centroids never move, nothing else is maintained.
 *   Section 4.4   Vectors inserted after the build sit in a per-cluster buffer that is
 *                 searched together with the cluster and the partial results merged;
 *                 here the buffer is a chain of device-resident delta pages of the list.
 *   Section 3.2 / Section 5
 *                 One independent index per agent ("memory scope"); operations arrive
 *                 in batches and must not block the caller: every call only enqueues
 *                 work on the caller's HIP stream.
 *
 * Conventions
 *   - Every pointer is marked HOST or DEVICE.  Device buffers belong to the caller
 *     (including arenas); the library owns only the host-side handle and one
 *     grow-only device workspace per handle that it allocates itself (tens of MB for a
 *     batch of 1024 queries: its size follows the batch, k and nprobe, not the index).
 *     The workspace grows (stream synchronisation, hipFree, hipMalloc) only when a call
 *     needs more than it holds.  pk_workspace_reserve sizes it once for every call
 *     within stated limits, inserts to come included; after that no search or insert
 *     within those limits allocates or waits (pk_stats.workspace_grows counts the
 *     growths).  Searches may then be captured into a HIP graph (inserts may not: they
 *     advance host-side counters).  A graph holds pointers into the workspace: growth
 *     invalidates it, so reserve before capturing; a call that would have to grow the
 *     workspace while its stream is capturing fails with PK_ERR_WORKSPACE instead.
 *     Inserts between replays are fine as long as they stay within the reserved
 *     `inserts_ahead` (the graph's tile list bound was taken at capture time).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work
 *     is enqueued on it; outputs are valid once the caller has synchronised the stream.
 *     (A search of 512 queries or more may run one of its kernels on a stream that the
 *     handle owns, forked from and joined to the caller's stream by events inside the
 *     call, at the default priority: to the caller the call stays ordered on `stream`.
 *     Under graph capture and in pk_search_noalloc everything stays on `stream`.)
 *     Calls on one handle must come from one thread and one stream at a time; an
 *     insert enqueued before a search on the same stream is seen by that search.
 *     pk_index_build, pk_index_stats and pk_list_lengths synchronise the stream.
 *   - One metric per index serves coarse ranking, build/insert assignment and fine
 *     search.  PK_METRIC_L2 returns the SQUARED Euclidean distance.
 *   - Result rows are sorted best first (inner product descending, L2 ascending); equal
 *     values are ordered by ascending id; rows with fewer than k candidates are padded
 *     with id -1 and -inf (IP) / +inf (L2).  Centroid ties go to the lower list number.
 *   - Inputs must be finite.  Rows are float32, row-major, densely packed.
 *   - Every function returns PK_OK (0) or a negative pk_status; nothing aborts, throws
 *     or prints.  Argument checks happen on the host before anything is launched.
 */
#ifndef PANCAKE_H
#define PANCAKE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pk_index pk_index; /* opaque per-agent handle (host object) */

typedef enum { PK_METRIC_IP = 0, PK_METRIC_L2 = 1 } pk_metric;
typedef enum { PK_F32 = 0, PK_F16 = 1 } pk_dtype; /* storage type of list vectors */

typedef enum {
    PK_OK = 0,
    PK_ERR_INVALID_ARG = -1,  /* null pointer, size or parameter out of range         */
    PK_ERR_BAD_HANDLE = -2,   /* not a live pk_index                                   */
    PK_ERR_DIM_MISMATCH = -3, /* handles of one multi-agent call differ in d / metric  */
    PK_ERR_NOMEM = -4,        /* arena (or host / workspace memory) exhausted          */
    PK_ERR_HIP = -5,          /* a HIP runtime call failed                             */
    PK_ERR_UNSUPPORTED = -6,  /* valid request outside the limits below                */
    PK_ERR_WORKSPACE = -7     /* the call does not fit the workspace it must use (fixed, or growth under capture) */
} pk_status;

/* Limits (compile-time). */
#define PK_MAX_K 1024        /* k per search                                          */
#define PK_MAX_NPROBE 1024   /* nprobe per search (also <= nlist)                     */
#define PK_MAX_HANDLES 128   /* handles per pk_search_multi call                      */
#define PK_MAX_ARENAS 8      /* arenas per index                                      */
#define PK_MAX_DIM 1536      /* vector dimension                                      */
#define PK_NOALLOC_WORKSPACE_BYTES (64u << 20) /* workspace of pk_search_noalloc, per GPU */

typedef struct {
    int32_t d;               /* vector dimension, >= 1                                 */
    int32_t nlist;           /* number of clusters / inverted lists, >= 1              */
    int32_t metric;          /* pk_metric                                              */
    int32_t storage;         /* pk_dtype: fp16 storage rounds to nearest even once     */
    int32_t page_vecs;       /* vectors per page: multiple of 32 in [32, 1024]; 0 = 128 */
    int32_t max_delta_pages; /* pages a list may grow by after the build; 0 = 1024     */
} pk_config;

typedef struct {
    int64_t n_total;         /* vectors in the index (build + inserts - deletes)       */
    int64_t n_inserted;      /* vectors added by pk_insert                             */
    int64_t pages_total;     /* pages available in all arenas                          */
    int64_t pages_used;      /* pages handed to lists                                  */
    int64_t arena_bytes;     /* sum of arena sizes                                     */
    int64_t workspace_bytes; /* current size of the library-owned search workspace     */
    int64_t workspace_grows; /* times that workspace was (re)allocated since the build  */
    int64_t max_list_len;    /* longest list                                           */
    int32_t device_error;    /* sticky device-side flag: 0 ok, 1 out of pages, 2 list full, 4 work list overflow */
    int32_t n_arenas;
} pk_stats;

/*
 * Bytes of arena needed to build an index over n vectors and then insert
 * n_insert_reserve more in the worst case (every list opening pages of its own).
 * Returns 0 for an invalid config.
 */
size_t pk_arena_bytes(const pk_config *cfg, int64_t n, int64_t n_insert_reserve);

/*
 * Section 2.2 (index) + Section 3.1 (assignment rule).  Creates an index over
 * `n` vectors: each goes to the list of its best centroid under cfg->metric (ties to the
 * lower list number) and is stored list-major in pages carved from `arena`.
 *   centroids  DEVICE [nlist, d] float32, copied into the arena
 *   vectors    DEVICE [n, d] float32 (may be NULL when n == 0); not referenced after return
 *   ids        DEVICE [n] int64, or NULL for 0 .. n-1
 *   arena      DEVICE, 256-byte aligned, arena_bytes long; owned by the caller, must stay
 *              allocated until pk_index_free
 *   out        HOST, receives the handle
 * Synchronises `stream` before returning.  PK_ERR_NOMEM if the arena is too small
 * (pk_arena_bytes gives a sufficient size).
 */
int pk_index_build(const pk_config *cfg, const float *centroids, const float *vectors, const int64_t *ids,
                   int64_t n, void *arena, size_t arena_bytes, void *stream, pk_index **out);

/* Adds page space after PK_ERR_NOMEM.  arena: DEVICE, 256-byte aligned, caller-owned. */
int pk_index_add_arena(pk_index *index, void *arena, size_t arena_bytes, void *stream);

/*
 * Index training on the device (Section 2.2: the clusters of an IVF index come from a
 * k-means over the data; Section 4.4 / 6.1, the IVF-Split variant, re-clusters with a light
 * k-means on the GPU).  `iters` Lloyd iterations under squared L2: every vector goes to its
 * nearest centroid (ties to the lower cluster number: the coarse search with nprobe = 1),
 * every cluster that has members moves to their mean (summed in float64), a cluster without
 * members keeps its centroid.
 *   vectors      DEVICE [n, d] float32
 *   centroids    DEVICE [nlist, d] float32: initial centroids on entry, result on return
 *   assign_out   DEVICE [n] int32 or NULL: the assignment of the last iteration (made with
 *                the centroids that iteration started from)
 *   inertia_out  HOST [iters] float64 or NULL: the sum of squared distances measured by the
 *                assignment step of each iteration
 * Allocates and frees its own scratch memory; synchronises `stream` before returning.
 */
int pk_kmeans(const float *vectors, int64_t n, int32_t d, int32_t nlist, int32_t iters, float *centroids,
              int32_t *assign_out, double *inertia_out, void *stream);

/*
 * Section 4.4, asynchronous cluster expansion (allocate room for the grown cluster, copy
 * the old data and the insertion buffer into it, swap, release the old), done here for
 * the whole index at once: every list is copied, in list order, into one contiguous extent
 * of pages in `arena` (its delta pages folded in), and the index then lives in `arena`
 * alone.  Positions inside a list are kept, so search results do not change; inserts go on
 * as before (tail page first, then new delta pages).
 *   arena   DEVICE, 256-byte aligned, caller-owned, must not overlap a current arena and
 *           must stay allocated until pk_index_free or the next compaction
 * Synchronises `stream` twice: to read the list lengths that fix the extents, and after the
 * copy, so that on return the arenas the index had before are no longer referenced and may
 * be freed or reused by the caller.  PK_ERR_NOMEM if `arena` cannot hold the index
 * (pk_arena_bytes(cfg, n_total, reserve) is sufficient); the index is unchanged then.
 */
int pk_index_compact(pk_index *index, void *arena, size_t arena_bytes, void *stream);

/*
 * Section 3.1 / Section 6.1 "IVF-Static" insert + Section 4.4 insertion buffer.
 * Each of the m vectors is assigned to its best centroid (same rule as the build) and
 * appended to the tail page of that list, opening a delta page when the tail is full.
 *   vectors         DEVICE [m, d] float32
 *   ids             DEVICE [m] int64, or NULL to continue the running counter
 *                   (vectors ever added before the call, +1 per vector)
 *   assigned_lists  DEVICE [m] int32, optional (NULL): receives the chosen lists
 * Asynchronous.  PK_ERR_NOMEM if the arenas may not hold m more vectors (nothing is
 * enqueued then).
 */
int pk_insert(pk_index *index, const float *vectors, const int64_t *ids, int64_t m, int32_t *assigned_lists,
              void *stream);

/*
 * Section 3.2 / Section 5: every agent has its own index and operations arrive in batches.
 * pk_insert for the indexes of several agents in one launch sequence: rows
 * [v_offsets[a], v_offsets[a+1]) of `vectors` (and of ids / assigned_lists) go to handles[a],
 * each assigned with that handle's own centroids.  Same semantics as n_handles pk_insert
 * calls in handle order.
 *   handles    HOST [n_handles] distinct live handles of equal d, metric, storage, page size
 *   v_offsets  HOST [n_handles + 1], v_offsets[0] = 0, non-decreasing
 * Asynchronous.  PK_ERR_NOMEM if any handle may not hold its share (nothing is enqueued).
 * The first handle owns the workspace used.
 */
int pk_insert_multi(pk_index *const *handles, int32_t n_handles, const int64_t *v_offsets, const float *vectors,
                    const int64_t *ids, int32_t *assigned_lists, void *stream);

/*
 * Section 4.4 (on-GPU cluster splitting) / Section 6.1 (the IVF-Split variant): a cluster
 * that has grown past `threshold` vectors is split in two by a light k-means over its
 * members, run on the device.  Done together with a compaction, because the number of
 * lists changes: the index moves into `arena` as in pk_index_compact, and every list that
 * is longer than `threshold` when the call starts is first split: 2-means under squared
 * L2 over its stored vectors (initial centroids: the member with the smallest id and the
 * member with the largest id; `iters` Lloyd iterations as in pk_kmeans), the members of
 * the first side stay in the list, whose centroid becomes the first centroid, the others
 * form a new list appended after the last one (list numbers nlist, nlist + 1, ... in the
 * order of the lists they came from) with the second centroid.  cfg.nlist grows by the
 * number of splits; all other lists and centroids are unchanged.
 *   n_split  HOST, optional: receives the number of lists split
 * Synchronises `stream`; on return the former arenas are no longer referenced.
 * PK_ERR_NOMEM if `arena` cannot hold the index with its new tables (the index is unchanged).
 */
int pk_index_split(pk_index *index, void *arena, size_t arena_bytes, int64_t threshold, int32_t iters,
                   int32_t *n_split, void *stream);

/* Read-back for callers that keep their own copy of the clustering (tests, after a split).
 *   pk_index_centroids  out: DEVICE [nlist, d] float32, the current centroid table
 *   pk_list_ids         out: DEVICE [cap] int64, receives the ids of the first min(cap, length)
 *                       members of `list` in storage order (lengths: pk_list_lengths)
 * Asynchronous. */
int pk_index_centroids(pk_index *index, float *out, void *stream);
int pk_list_ids(pk_index *index, int32_t list, int64_t *out, int64_t cap, void *stream);

/*
 * Section 5 (the interface offers search, insert, delete and update).  Every stored vector
 * whose id is among ids[0..m) is removed, all of them if several carry the id; ids nobody
 * carries are ignored.  A removed row is overwritten by the last row of its list and the
 * list shrinks by one (lists are unordered sets: search results, ordered by value and id,
 * show nothing but the removal; no tombstones are left for searches to skip).  Pages a list
 * no longer reaches stay with the list and are used again when it grows.  An update is a
 * pk_delete followed by a pk_insert on the same stream.
 *   ids        DEVICE [m] int64
 *   n_removed  HOST, optional (NULL): receives the number of vectors removed
 * Synchronises `stream` (the handle keeps the live count).
 */
int pk_delete(pk_index *index, const int64_t *ids, int64_t m, int64_t *n_removed, void *stream);

/* As pk_insert, with the lists given by the caller (DEVICE [m] int32, each in [0, nlist)). */
int pk_insert_assigned(pk_index *index, const float *vectors, const int64_t *ids, int64_t m,
                       const int32_t *lists, void *stream);

/*
 * Section 2.2 coarse + fine search for a batch of queries of one index.
 *   queries   DEVICE [nq, d] float32
 *   k         1 .. PK_MAX_K;  nprobe 1 .. min(nlist, PK_MAX_NPROBE)
 *   out_ids   DEVICE [nq, k] int64;  out_dist DEVICE [nq, k] float32
 * Asynchronous.
 */
int pk_search(pk_index *index, const float *queries, int64_t nq, int32_t k, int32_t nprobe, int64_t *out_ids,
              float *out_dist, void *stream);

/*
 * Section 5 (operations must not block the caller).  Sizes the workspace of handles[0], the
 * handle whose workspace a call uses (the index of a single-handle call, the first handle of
 * a multi-handle call), so that every later pk_search / pk_search_multi / pk_insert /
 * pk_insert_multi / pk_coarse / pk_scan_probes over these handles (any subset, handles[0]
 * first) with at most nq_max queries (or vectors) in total, k <= k_max and nprobe <=
 * nprobe_max finds it large enough, until inserts_ahead more vectors have been inserted into
 * any one of the handles: such calls then never allocate and never wait for the device.
 * The size does not depend on how many candidates the queries meet: a query's emitted
 * candidates live in a region of a few dozen times k entries, and a query that emits more
 * (no usable threshold, or a tie group larger than the region) is selected by rescoring its
 * rows instead, with the same values.
 *   handles   HOST [n_handles] live handles of equal d, metric, storage, page size
 *   nq_max    1 .. 32768;  inserts_ahead >= 0
 * May synchronise `stream` and allocate (once); PK_ERR_NOMEM if the device is out of memory.
 */
int pk_workspace_reserve(pk_index *const *handles, int32_t n_handles, int64_t nq_max, int32_t k_max,
                         int32_t nprobe_max, int64_t inserts_ahead, void *stream);

/* Test seam / tuning: entries of each query's emission region in later searches on this
 * handle (0 = the default, a few dozen times k; the library never uses fewer than k + 1).
 * A small value forces queries down the rescoring path. */
int pk_index_set_emit_cap(pk_index *index, int32_t entries);

/*
 * pk_search for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bit-identical results, but the workspace (prepared queries, centroid scores, probe lists,
 * work list, tiles, emitted candidates: everything pk_search keeps in the handle's
 * grow-only buffer) is a fixed array of PK_NOALLOC_WORKSPACE_BYTES that is part of the
 * library's device image: every GPU the library is loaded on holds one copy until the
 * process ends.  The call never calls hipMalloc / hipFree, never waits for the device and
 * records no stage timing.
 *   PK_ERR_WORKSPACE  the search needs more than the array holds; nothing is enqueued.
 *                     pk_search_noalloc_bytes(index, nq, k, nprobe) tells the need
 *                     beforehand (0: invalid arguments); it grows with nq, k and nprobe
 *                     and, slowly, with the pages the index holds.
 * All calls on one GPU share that GPU's array, whatever the handle: two such calls that
 * overlap in time on one GPU (different streams or threads) race and give wrong results.
 * Calls in stream order are safe; every call clears what it needs cleared itself.
 * Asynchronous.
 */
int pk_search_noalloc(pk_index *index, const float *queries, int64_t nq, int32_t k, int32_t nprobe,
                      int64_t *out_ids, float *out_dist, void *stream);
size_t pk_search_noalloc_bytes(pk_index *index, int64_t nq, int32_t k, int32_t nprobe);

/*
 * Section 3.2 (independent per-agent indexes) + Section 5 (batched operations): queries
 * addressed to many handles are served by one launch sequence.  Segment a = query rows
 * [q_offsets[a], q_offsets[a+1]) is searched in handles[a]; results equal per-handle
 * pk_search calls bit for bit.
 *   handles    HOST [n_handles]; all share d, metric, storage and page_vecs; each at most once
 *   q_offsets  HOST [n_handles + 1], non-decreasing, q_offsets[0] == 0
 *   queries    DEVICE [q_offsets[n_handles], d];  outputs as in pk_search
 */
int pk_search_multi(pk_index *const *handles, int32_t n_handles, const int64_t *q_offsets, const float *queries,
                    int32_t k, int32_t nprobe, int64_t *out_ids, float *out_dist, void *stream);

/*
 * Section 3.2: a request may read the memories of a set of agents (its scope), e.g. the
 * shared memory plus the agent's private one; each index of the scope is searched and the
 * results are merged.  Every query is searched in every handle (coarse + fine search per
 * handle, with that handle's own centroids), and the k best of the union are returned;
 * equal values are ordered by the position of the handle in `handles`, then by id.
 *   handles   HOST [n_handles] distinct live handles of equal d, metric, storage, page size
 *   queries   DEVICE [nq, d] float32
 *   out_src   DEVICE [nq, k] int32: position in `handles` of the index each result came
 *             from (-1 for padding)
 *   out_ids   DEVICE [nq, k] int64;  out_dist DEVICE [nq, k] float32
 * Asynchronous; the work is that of n_handles searches of the batch, in one segmented
 * launch sequence.  The first handle owns the staging buffer (grown on demand).
 */
int pk_search_union(pk_index *const *handles, int32_t n_handles, const float *queries, int64_t nq, int32_t k,
                    int32_t nprobe, int32_t *out_src, int64_t *out_ids, float *out_dist, void *stream);

/*
 * Section 4.2 (multi-level index cache, early termination): the indexes of an agent form
 * levels, every upper level a subset of the one below that follows the agent's recent
 * accesses; a search starts at the top level and skips the levels below as soon as all
 * top-k candidates of the current level are closer than alpha_et * d_agent (d_agent: the
 * agent's mean top-k distance over its recent queries).  This call is that search rule over
 * levels the caller maintains: every query is searched in levels[0]; a query whose row there
 * holds k candidates and whose k-th value is smaller than stop[q] (inner product: greater)
 * keeps that row; the others are searched in levels[1], whose row replaces the upper one,
 * and so on; the last level ends every search.  Below the first level only the queries
 * still open are scanned (the coarse step runs for the whole batch).
 *   levels    HOST [n_levels] distinct live handles of equal d and metric, top level first
 *   nprobes   HOST [n_levels] lists to probe per level, 1 <= nprobes[l] <= nlist of level l
 *   stop      DEVICE [nq] float32: alpha_et * d_agent of each query's agent, in the unit
 *             the index returns (squared distance for L2, score for inner product)
 *   out_level DEVICE [nq] int32 or NULL: the level whose row the query carries
 *   out_ids   DEVICE [nq, k] int64;  out_dist DEVICE [nq, k] float32
 * Asynchronous.  The first handle owns the staging buffer (grown on demand).
 */
int pk_search_levels(pk_index *const *levels, int32_t n_levels, const int32_t *nprobes, const float *queries,
                     int64_t nq, int32_t k, const float *stop, int32_t *out_level, int64_t *out_ids,
                     float *out_dist, void *stream);

/* Stage seams (tests isolate coarse and fine search with them). */

/* Coarse search only: out_probes DEVICE [nq, nprobe] int32, best list first. */
int pk_coarse(pk_index *index, const float *queries, int64_t nq, int32_t nprobe, int32_t *out_probes,
              void *stream);

/* Fine search over caller-given probe lists: probes DEVICE [nq, nprobe] int32, each row
 * without repeats, every entry in [0, nlist). */
int pk_scan_probes(pk_index *index, const float *queries, int64_t nq, int32_t k, int32_t nprobe,
                   const int32_t *probes, int64_t *out_ids, float *out_dist, void *stream);

/* Counters of the index; synchronises `stream`.  out: HOST. */
int pk_index_stats(pk_index *index, pk_stats *out, void *stream);

/* Current length of every list; synchronises `stream`.  out_len: HOST [nlist] int64. */
int pk_list_lengths(pk_index *index, int64_t *out_len, void *stream);

/*
 * Stage timing for benchmarks.  Between pk_profile_begin and pk_profile_end every search
 * launch sequence on this handle is bracketed by HIP events on its stream (at most 1024
 * sequences are recorded) and the device adds up what the work lists contained.
 *   coarse_ms   Section 2.2 coarse search: centroid scoring + top-nprobe
 *   worklist_ms grouping of (query, list) pairs into page tiles
 *   scan_ms     Section 2.2 fine search: the list-scan kernels alone (both launches)
 *   select_ms   per-query top-k over the scored candidates (Section 4.4 merge)
 * scanned_rows counts each probed list once per launch sequence (the rows the scan must
 * read from memory); candidates counts (query, vector) pairs scored, emitted those that
 * passed the running per-query threshold and reached the top-k selection.  pk_profile_end synchronises
 * `stream`.  out: HOST.
 */
typedef struct {
    int32_t launches;
    float coarse_ms, worklist_ms, scan_ms, select_ms; /* sums over the recorded sequences */
    int64_t scanned_rows, candidates, tiles, emitted; /* sums over all sequences          */
    int64_t overflowed;  /* queries whose emission region overflowed (selected by rescoring) */
    int64_t max_emitted; /* most candidates a single query emitted                          */
    float scan_hot_ms;   /* the part of scan_ms spent in the launch for lists probed by many queries */
} pk_profile;
int pk_profile_begin(pk_index *index, void *stream);
int pk_profile_end(pk_index *index, pk_profile *out, void *stream);

/* Frees the host object and the library-owned workspace (not the arenas).  The caller
 * must have synchronised every stream that still uses the index. */
int pk_index_free(pk_index *index);

const char *pk_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* PANCAKE_H */
