// Internal declarations shared by the translation units of libpancake (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <atomic>
#include <stddef.h>
#include <stdint.h>

#include "pancake.h"

// Development builds (-DPK_DEV_TIMING) record the wall clock of workgroup 0's first thread at marked
// points of a kernel; a release build holds none of this.
#ifdef PK_DEV_TIMING
#define PK_DEV_MARKS(name)                                                                      \
    static __device__ unsigned long long name##_marks[64];                                      \
    extern "C" int pk_dev_##name##_marks(unsigned long long *out)                              \
    {                                                                                           \
        return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(name##_marks), sizeof(name##_marks));   \
    }
#define PK_MARK(name, i)                                                                        \
    do {                                                                                        \
        if (blockIdx.x == 0 && threadIdx.x == 0) name##_marks[i] = wall_clock64();              \
    } while (0)
// (mark by the first thread of whichever workgroup `cond` picks)
#define PK_MARK_IF(name, i, cond)                                                               \
    do {                                                                                        \
        if ((cond) && threadIdx.x == 0) name##_marks[i] = wall_clock64();                       \
    } while (0)
#else
#define PK_DEV_MARKS(name)
#define PK_MARK(name, i) do { } while (0)
#define PK_MARK_IF(name, i, cond) do { } while (0)
#endif

namespace pk {

// ------------------------------------------------------------------ constants
constexpr int kWave = 64;
constexpr int kScanThreads = 256;     // 4 waves per workgroup in the scan kernel
constexpr int kRrTileRows = 128;      // rows per tile of the rows-in-registers scan kernel
constexpr int kRrSlots = 512;         // most query slots per tile of that kernel
constexpr int kRowBlock = 32;         // rows one wave scores per pass (two 16-wide MFMA tiles)
constexpr int kIterBytes = 256;       // bytes of one row consumed per inner iteration
constexpr int kQPadBytes = 16;        // LDS row padding of the query tile (bank spread)
constexpr int kCentroidPad = 32;      // the centroid table is zero padded to a multiple of this many rows
constexpr int kSelThreads = 256;
constexpr int kSelVec = 4;            // candidates per thread per round
constexpr int kSelCap = 4096;         // LDS key buffer of the select kernels (K + one round <= cap)
constexpr int kSelChunk = 32768;      // candidates per (query, chunk) workgroup (large batches; small ones cut finer)
constexpr unsigned long long kMaxKey = ~0ull;
constexpr int kHistBins = 64;         // per-query key histogram that tightens the emission threshold

constexpr int kErrPages = 1, kErrListFull = 2, kErrWorklist = 4;

// One arena = npages pages: vectors | norms | ids, each indexed by the local page number.
struct Arena {
    uint32_t first_page, npages;
    char *vec;       // [npages][P][row_bytes]
    float *norm;     // [npages][P]
    int64_t *ids;    // [npages][P]
};

// Device-resident description of one index (lives at the start of its first arena).
struct DevIndex {
    const float *cent;   // [nlist_pad][dpad32] fp32 centroid table, zero padded
    const float *cnorm;  // [nlist_pad] squared norms (L2 only, else zeros)
    uint32_t *list_len;  // [nlist] vectors per list
    uint32_t *main_base; // [nlist] first page of the build-time extent
    uint32_t *main_pages;// [nlist] pages in that extent
    uint32_t *dtab;      // [nlist][max_dp] delta page numbers
    uint32_t *ctr;       // [0] next free page, [1] sticky error flags, [2] pages total
    unsigned long long *stats; // running sums: [0] rows of distinct probed lists, [1] candidates, [2] tiles, [3] emitted,
                               // [4] queries whose emission region overflowed; [5] most candidates one query emitted
    int32_t nlist, nlist_pad, d, dpad32, P, max_dp, metric, storage;
    int32_t row_bytes;   // padded bytes of one stored row
    int32_t n_arenas;
    Arena arenas[PK_MAX_ARENAS];
};

__device__ __forceinline__ const Arena &arena_of(const DevIndex &ix, uint32_t page)
{
    int a = 0;
    while (a + 1 < ix.n_arenas && page >= ix.arenas[a].first_page + ix.arenas[a].npages) ++a;
    return ix.arenas[a];
}

// physical page of logical page `lp` of list `l`
__device__ __forceinline__ uint32_t phys_page(const DevIndex &ix, uint32_t l, uint32_t lp)
{
    uint32_t mp = ix.main_pages[l];
    return lp < mp ? ix.main_base[l] + lp : ix.dtab[(size_t)l * ix.max_dp + (lp - mp)];
}

// A value as an unsigned key whose ascending order is best-first (smaller = better) under
// the metric; exact inverse below.  Padding (-inf for inner product, +inf for L2) maps to
// 0xff800000 under both metrics; finite values map below it.
__device__ __forceinline__ uint32_t order_bits(float v, int metric)
{
    const uint32_t b = __float_as_uint(v);
    const uint32_t asc = b ^ ((b >> 31) ? 0xffffffffu : 0x80000000u);
    return metric == PK_METRIC_L2 ? asc : ~asc;
}

__device__ __forceinline__ float value_of(uint32_t ob, int metric)
{
    const uint32_t asc = metric == PK_METRIC_L2 ? ob : ~ob;
    const uint32_t b = (asc & 0x80000000u) ? (asc ^ 0x80000000u) : ~asc;
    return __uint_as_float(b);
}

constexpr uint32_t kWorstBits = 0xff800000u;

// Bucket of a value on a per-query scale: the distance of the value from the best sampled
// value `lo`, in units of 1/inv, cut into kHistBins-1 equal buckets; everything past the
// sampled range lands in the last bucket.  Monotone in the value (each float operation
// involved is), better values get lower buckets, so "bucket <= b" is a valid cut wherever
// k candidates are known to have bucket <= b.
__device__ __forceinline__ uint32_t bucket_of(float v, float lo, float inv, int metric)
{
    float off = metric == PK_METRIC_L2 ? v - lo : lo - v;
    off = fmaxf(off, 0.f);
    const float t = fminf(off * inv, (float)(kHistBins - 1));
    return (uint32_t)t;
}

// ---- MFMA operand helpers shared by the scan kernels and the exact per-query rescoring
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Pointers taken out of a tile descriptor are generic pointers to the compiler, and loads
// through them would be flat loads: those count on the LDS counter as well, so a wait for
// an LDS read would also wait for the rows being prefetched.  These types say "global".
typedef const char __attribute__((address_space(1))) *gbytes;
typedef const float __attribute__((address_space(1))) *gfloats;
typedef const u32x4 __attribute__((address_space(1))) *gvec4;
__device__ __forceinline__ gbytes in_global(const char *p) { return (gbytes)p; }
__device__ __forceinline__ gfloats in_global(const float *p) { return (gfloats)p; }

// 16 bytes of a query row (A) against 16 bytes of a stored row (B), fp32 accumulation: one
// v_mfma_f32_16x16x32_f16, or four v_mfma_f32_16x16x4_f32.  Every kernel that scores a
// (row, query) pair issues these in the same order over the row, so the value of a pair does
// not depend on the kernel that computed it.
template <int STORAGE>
__device__ __forceinline__ void mfma_step(f32x4 &acc, const u32x4 &qa, const u32x4 &xb)
{
    if constexpr (STORAGE == PK_F16) {
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, qa), __builtin_bit_cast(half8, xb),
                                                     acc, 0, 0, 0);
    } else {
        f32x4 qf = __builtin_bit_cast(f32x4, qa), xf = __builtin_bit_cast(f32x4, xb);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(qf[0], xf[0], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(qf[1], xf[1], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(qf[2], xf[2], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(qf[3], xf[3], acc, 0, 0, 0);
    }
}

// squared L2 distance from the inner product and the two squared norms (one expression, used
// by every kernel that returns a fine-search value)
__device__ __forceinline__ float l2_from_dot(float xn, float dot, float qn) { return fmaxf(xn - 2.f * dot + qn, 0.f); }

// exclusive scan of in[0,n) into out[0,n) by one workgroup (up to 1024 threads); returns the
// total.  A thread takes 4 consecutive elements, so 4096 elements need one round of barriers;
// out may be the same array as in.
__device__ __forceinline__ uint32_t block_exscan(const uint32_t *in, uint32_t *out, uint32_t n, uint32_t *s_wave /*[17]*/)
{
    uint32_t carry = 0;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    for (uint32_t base = 0; base < n; base += 4u * blockDim.x) {
        const uint32_t i = base + 4u * threadIdx.x;
        uint32_t v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = i + j < n ? in[i + j] : 0u;
        const uint32_t t = v[0] + v[1] + v[2] + v[3];
        uint32_t x = t;
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t y = __shfl_up(x, off);
            if (lane >= off) x += y;
        }
        if (lane == 63) s_wave[wave] = x;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t acc = 0;
            for (int w = 0; w < nwaves; ++w) {
                const uint32_t tw = s_wave[w];
                s_wave[w] = acc;
                acc += tw;
            }
            s_wave[16] = acc;
        }
        __syncthreads();
        uint32_t run = carry + s_wave[wave] + x - t;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (i + j < n) out[i + j] = run;
            run += v[j];
        }
        carry += s_wave[16];
        __syncthreads();
    }
    return carry;
}

// One unit of scan work: one page of rows against one group of query slots.
struct Tile {
    const char *x;    // first row of the page
    const float *xn;  // squared norms of the rows (L2), else unused
    uint32_t row0;    // position of the page's first row in the list
    uint32_t qbeg;    // first slot of the group in slot_query / slot_out
    uint16_t nrows;   // rows to score (<= rows per page)
    uint16_t qcnt;    // slots in the group (<= MQ)
    uint32_t pad;
};
static_assert(sizeof(Tile) == 32, "Tile is 32 bytes");

// Handles of one call, passed to kernels by value (fits the 4 KiB kernel-argument space).
struct MultiArgs {
    const DevIndex *ix[PK_MAX_HANDLES];
    uint32_t qlo[PK_MAX_HANDLES + 1];   // handle a owns query rows [qlo[a], qlo[a+1])
    int32_t n;
};

// --------------------------------------------------------------- launch APIs
// (each enqueues on `s` and returns the HIP status of the launch)

hipError_t launch_fill_u32(uint32_t *p, uint32_t v, size_t n, hipStream_t s);
hipError_t launch_copy_i32(const int32_t *src, int32_t *dst, int64_t n, hipStream_t s);

// queries -> storage type, zero padded rows, squared norms of the converted values
hipError_t launch_prep_queries(const float *q, int64_t nq, int d, int storage, int row_bytes, void *qs,
                               float *qnorm, hipStream_t s);

struct ScanArgs {
    const Tile *tiles;
    const uint32_t *ntiles;      // device scalar
    const uint32_t *batch;       // device scalar: tiles taken per grab (>= 1)
    const char *qs;              // prepared queries [nq][row_bytes]
    const float *qnorm;          // [nq]
    const uint32_t *slot_query;  // slot -> query row
    const uint32_t *slot_out;    // slot -> first output element of the (query, list) pair
    float *out;                  // dense mode: values, one per (slot, row)
    // gated mode (tau != NULL): a value is emitted only if its key is <= tau[query]; it is
    // appended as (key << 32 | position) to the query's region of cbuf
    const uint32_t *tau;         // [nq] threshold keys from the sample (never change)
    const float *tlo;            // [nq] best sample value: origin of the bucket scale
    const float *tinv;           // [nq] bucket scale (see bucket_of)
    uint32_t *hist;              // [nq][kHistBins] emitted candidates per bucket (zero before the launch)
    uint32_t *tcur;              // [nq] running bucket limit shared by all workgroups (starts at kHistBins-1)
    uint32_t ecap;               // entries of each query's region of cbuf: query q owns [q * ecap, (q + 1) * ecap)
    uint32_t *ccnt;              // [nq] candidates that passed the gate so far (zero before the launch); those past
                                 // ecap are counted but not stored, and the query is then selected by rescoring
    unsigned long long *cbuf;
    uint32_t *tile_ctr;          // device scalar, zero before the launch: batches handed out after the first round
    int k, use_hist;
    int row_bytes, metric, storage, mq;
};
hipError_t launch_scan(const ScanArgs &a, int grid, hipStream_t s);
hipError_t launch_scan_ks(const ScanArgs &a, int grid, hipStream_t s);
hipError_t launch_scan_rr(const ScanArgs &a, int grid, hipStream_t s);
int scan_rr_lds_bytes();
int scan_lds_bytes(int row_bytes, int mq);
int scan_ks_lds_bytes(int mq);
int scan_max_mq(int row_bytes, int storage, int lds_limit);

// Tile schedule shared by the list-scan kernels.  The first tile of every workgroup is fixed (tile b for
// workgroup b); later batches come from one counter, so uneven tiles still balance while
// the launch does not start with a burst of atomics.  A batch is `grab` tiles; the first batch
// is a single tile so that the emission gates get their first refresh early.  The request for the next
// batch is issued when a batch starts and collected when it ends, and the descriptor of the
// next tile is fetched while the current tile is scored.  Every workgroup stops the first
// time it is handed a batch past the end.
struct Sched {
    uint32_t t, end, ntiles, grab;
    uint32_t nblk; // workgroups that take tiles (all of the launch, unless its first ones do other work)
    int parity;
    bool fresh; // t is the first tile of a batch
    // bid: this workgroup's number among the nblk that take tiles
    __device__ __forceinline__ void start(uint32_t nt, uint32_t g, uint32_t bid, uint32_t nb)
    {
        ntiles = nt;
        grab = g;
        nblk = nb;
        t = bid;
        end = t + 1 < nt ? t + 1 : nt;
        parity = 0;
        fresh = true;
    }
    // one thread asks for the batch after the current one (s_misc[2*parity], [2*parity+1] = start, size)
    __device__ __forceinline__ void request(const ScanArgs &a, uint32_t *s_misc, uint32_t asker = 0u) const
    {
        if (threadIdx.x == asker && nblk < ntiles) {
            // One atomic per batch and no other access to the counter: every workgroup of the
            // grid claims from this one address, and a second access per claim (a load, to
            // size the batch by what is left) measurably slows the whole scan.
            const uint32_t want = grab;
            s_misc[2 * parity] = nblk + atomicAdd(a.tile_ctr, want);
            s_misc[2 * parity + 1] = want;
        }
    }
    // index of the tile after t; at the end of a batch this collects the requested batch (block-wide)
    __device__ __forceinline__ uint32_t peek(const uint32_t *s_misc, uint32_t &next_end, bool &next_fresh) const
    {
        if (t + 1 < end) {
            next_end = end;
            next_fresh = false;
            return t + 1;
        }
        next_fresh = true;
        if (nblk >= ntiles) {
            next_end = ntiles;
            return ntiles;
        }
        __syncthreads();
        const uint32_t st = s_misc[2 * parity], sz = s_misc[2 * parity + 1];
        next_end = st + sz < ntiles ? st + sz : ntiles;
        return st;
    }
};


// Dynamic LDS beyond 64 KB has to be allowed per kernel and device.  Every scan kernel is cleared
// once per device for the most a workgroup can have, so the value never depends on the call
// that happens to come first and threads serving different handles cannot undo each other.
constexpr int kMaxDevices = 64;
struct LdsCleared {
    std::atomic<int> on[kMaxDevices];
};

template <typename K>
inline hipError_t launch_with_lds(K kernel, LdsCleared &c, int lds, const ScanArgs &a, int grid, int threads, hipStream_t s)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < kMaxDevices;
    if (!tracked || c.on[dev].load(std::memory_order_acquire) == 0) {
        int most = 0;
        e = hipDeviceGetAttribute(&most, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, most);
        if (e != hipSuccess) return e;
        if (tracked) c.on[dev].store(1, std::memory_order_release);
    }
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(threads), lds, s, a);
    return hipGetLastError();
}



struct SelectArgs {
    const float *vals;            // candidate values, or NULL when keys are given
    const unsigned long long *keys; // candidate keys (value key << 32 | position)
    const uint32_t *qoff;         // [nq] first candidate of each query
    const uint32_t *qcnt;         // [nq] candidates of each query
    int metric, K, nchunks;
    int chunk;                    // candidates per (query, chunk) workgroup
    unsigned long long *partial;  // [nq][nchunks][K]
};
hipError_t launch_select_partial(const SelectArgs &a, int64_t nq, hipStream_t s);
constexpr int kMaxSamplePages = 64;      // most pages of one query's threshold sample
constexpr uint32_t kWlSmallLists = 2048; // most lists (all handles of a call) whose work list is laid out inside another kernel's launch
constexpr int kDenseSelectMax = 8192; // longest score row the register-resident selection takes

hipError_t launch_select_probes(const unsigned long long *partial, int nchunks, int K, int nprobe, int64_t nq,
                                int32_t *probes, hipStream_t s);

struct FinalArgs {
    int K, k, nprobe, metric, storage, row_bytes;
    const unsigned long long *keys;   // emitted candidates: query q owns [q * ecap, (q + 1) * ecap)
    unsigned long long *spill;        // the same regions, writable: scratch of a query that is rescored
    uint32_t ecap;
    const uint32_t *qcnt;             // [nq] candidates that passed the gate (more than ecap: region overflowed)
    const uint32_t *pair_off;         // [nq][nprobe+1] start of each probe's segment inside the query's range
    const int32_t *probes;            // [nq][nprobe]
    const uint16_t *qagent;           // [nq] handle number
    const char *qs;                   // prepared queries [nq][row_bytes] (storage type), for the rescoring
    const float *qnorm;               // [nq]
    int64_t *out_ids;
    float *out_dist;
};
hipError_t launch_select_final(const FinalArgs &a, const MultiArgs &m, int64_t nq, hipStream_t s);

// Per-query bookkeeping of the coarse step, filled while the queries are prepared.
struct QueryMeta {
    uint32_t stride;               // elements between the score rows of consecutive queries
    uint32_t *cand_off, *cand_cnt; // [nq] score row of each query and its length (nlist of its handle)
    uint16_t *qagent;              // [nq] handle number of each query
    uint32_t *clear;               // words the fine step wants zeroed before it starts (or null)
    uint32_t nclear;
};
// fp32 queries -> zero padded rows and squared norms, plus the bookkeeping above
hipError_t launch_prep_coarse(const float *q, int64_t nq, int d, int row_bytes, void *qs, float *qnorm,
                              const QueryMeta &meta, const MultiArgs &m, hipStream_t s);

// Centroid scoring of small query segments (16 centroids x `chunk` queries per workgroup).
struct CentroidArgs {
    const char *qs;      // prepared fp32 queries [nq][row_bytes]
    const float *qnorm;  // [nq]
    float *out;          // score of (query q, centroid c of q's handle) at out[q * stride + c]
    uint32_t stride;
    int row_bytes, metric;
    int chunk;           // queries per workgroup: 16, 32, 48 or 64
    uint32_t blk[PK_MAX_HANDLES + 1]; // first workgroup of handle a, [n] = all; a handle scored elsewhere owns none
    // Optional extras that save a launch each on small batches:
    //   meta.cand_off != null: this kernel also does the per-query bookkeeping of the coarse step and clears
    //   the words in meta.clear (qs then are the caller's own rows: no padding needed, no norms for inner product);
    //   best != null: instead of writing scores, every query keeps its best (score key << 32 | list) by
    //   atomicMin (top-1 assignment of inserts; best[] must hold ~0 on entry).
    QueryMeta meta;
    unsigned long long *best;
};
hipError_t launch_centroid_scores(const CentroidArgs &a, const MultiArgs &m, hipStream_t s);

// merge of per-handle result rows into one row per query (k <= 1024: rank fits 10 bits, handle 7)
struct UnionArgs {
    const int64_t *ids;  // [n_handles][nq][k] rows of the handles, each sorted best first, -1 padded
    const float *dist;   // [n_handles][nq][k]
    int n_handles, k, metric;
    int64_t nq;
    int32_t *out_src;    // [nq][k] position of the handle in the scope, -1 for padding
    int64_t *out_ids;    // [nq][k]
    float *out_dist;     // [nq][k]
};
hipError_t launch_union_merge(const UnionArgs &a, hipStream_t s);

// Level cascade (early termination): bookkeeping between the searches of two levels.
struct LevelArgs {
    int64_t nq;
    int k, metric, level;
    bool first, last;        // first: every query is open; last: this level ends every search
    const float *stop;       // [nq]
    uint32_t *open;          // [nq] 1 while the query has not ended (written when first)
    int32_t *level_out;      // [nq] or null
    const int64_t *row_ids;  // [nq][k] this level's rows (null when first: they are already in out_*)
    const float *row_dist;   // [nq][k]
    int64_t *out_ids;        // [nq][k]
    float *out_dist;         // [nq][k]
};
// rows of this level -> output for the open queries; closes those the rule (or the last level) ends
hipError_t launch_level_accept(const LevelArgs &a, hipStream_t s);
// probes[q][*] = -1 for queries that are no longer open (their lists are not scanned)
hipError_t launch_level_mask(int32_t *probes, int nprobe, const uint32_t *open, int64_t nq, hipStream_t s);

struct WorklistArgs {
    const int32_t *probes;     // [nq][nprobe]; entries outside [0, nlist) are ignored
    const uint16_t *qagent;    // [nq]
    int64_t nq;
    int nprobe, n_handles, nlist_max, scan_grid, scan_grid_hot, grab_div, hot_grab;
    int mq;                    // slots per group of a regular tile
    int mq_hot;                // slots per group of a hot tile
    int hot_rows;              // rows per hot tile: 0 = a page; else a divisor of the page size (rows-stationary kernel)
    uint32_t hot_from;         // lists probed by more than this many queries of the batch are hot
    uint32_t *lcnt, *lstart, *lfill, *ltile, *lhtile; // [n_handles * nlist_max]
    bool lcnt_cleared;         // the coarse step of the same search has zeroed lcnt already
    uint32_t *pair_off;        // [nq][nprobe+1]
    uint32_t *ccnt;            // [nq] zeroed here (emission counters of the gated scan)
    uint32_t *slot_query, *slot_out; // [nq * nprobe]; slot_out = first position of the pair inside the query's range
    Tile *tiles, *tiles_hot;
    uint32_t tile_cap;
    uint32_t *scalars;         // [0] ntiles [1] tile counter [2] grab size
    uint32_t *scalars_hot;     // [0] hot tiles [1] tile counter [2] grab size
    // one handle only: its list lengths, page size and list count, so that the work-list layout of a small batch
    // reads them without first chasing the handle's descriptor (null / 0 otherwise)
    const uint32_t *len1;
    uint32_t P1, nlist1;
};

// Threshold sampling: the first `sp` pages of each query's first probed list are scored
// densely; the k-th best of them bounds the query's k-th best overall.
struct SampleArgs {
    const int32_t *probes;     // [nq][nprobe]
    const uint16_t *qagent;
    int64_t nq;
    int nprobe, sp, k, metric, scan_grid;
    uint32_t span;             // values per query = sp * rows per page (same for all handles)
    Tile *tiles;               // [nq * sp]
    uint32_t *slot_query;      // [nq] = q
    uint32_t *slot_out;        // [nq] = q * span
    float *vals;               // [nq][span], pre-filled with the padding value by the kernel
    uint32_t *scalars;         // [0] ntiles [1] tile counter [2] grab size
    uint32_t *tau;             // [nq] out: k-th best sample key, or 0xffffffff
    float *tlo;                // [nq] out: best sample value
    float *tinv;               // [nq] out: bucket scale = (kHistBins-1) / |k-th best (or worst) sample value - best|
    uint32_t *hist;            // [nq][kHistBins] zeroed here
    uint32_t *tcur;            // [nq] out: running bucket limit, starts at kHistBins-1
};
hipError_t launch_worklist_count(const WorklistArgs &a, const SampleArgs &sm, const MultiArgs &m, hipStream_t s);
hipError_t launch_worklist_tiles(const WorklistArgs &a, const MultiArgs &m, hipStream_t s);
// wa / ma given (small batches): the launch also builds the second half of the work list (launch_worklist_tiles is not needed)
hipError_t launch_tau(const SampleArgs &a, hipStream_t s, const WorklistArgs *wa = nullptr, const MultiArgs *ma = nullptr);
// small batches: the sample's tiles, the thresholds and the second half of the work list in one launch (in place of
// launch_scan over the sample, launch_tau and launch_worklist_tiles); sm.span at most 4096
hipError_t launch_sample_tau(const ScanArgs &a, const SampleArgs &sm, const WorklistArgs &wa, const MultiArgs &ma, int grid,
                             hipStream_t s);
// wa / sm / ma given: the selection's workgroups also do launch_worklist_count's work for their queries
hipError_t launch_select_dense(const float *vals, const uint32_t *qoff, const uint32_t *qcnt, uint32_t max_cnt, int metric,
                               int K, int64_t nq, int32_t *probes, hipStream_t s, const WorklistArgs *wa = nullptr,
                               const SampleArgs *sm = nullptr, const MultiArgs *ma = nullptr);

// dense coarse scoring on the matrix cores (large query batches, build)
struct GemmArgs {
    const float *q;      // [m][ld] prepared fp32 queries (zero padded rows)
    const float *c;      // [n_pad][ld] centroid table
    const float *qnorm;  // [m]
    const float *cnorm;  // [n_pad]
    float *out;          // [m][stride]
    int m, n, n_pad, n_store, ld, metric;
    uint32_t stride;
};
hipError_t launch_gemm_scores(const GemmArgs &a, hipStream_t s);

// build / insert
hipError_t launch_hist(const int32_t *assign, int64_t n, uint32_t *cnt, hipStream_t s);
hipError_t launch_scatter_build(const DevIndex *ix, const float *x, const int64_t *ids, const int32_t *assign,
                                int64_t n, int64_t id0, uint32_t *fill, hipStream_t s);
hipError_t launch_store_centroids(const float *c, int nlist, int d, int dpad32, int nlist_pad, int metric,
                                  float *cent, float *cnorm, hipStream_t s);
// Removes the rows whose id is among ids[0..m), m <= kDeleteChunk.  One pass removes at most kDeleteChunk
// rows; if more rows carry the ids (several rows under one id), the sticky flag says so and the caller
// runs the pass again.
constexpr int kDeleteChunk = 4096;
constexpr int kDeleteUnit = 1024; // rows of one list that a workgroup examines at a time
struct DeleteArgs {
    const DevIndex *ix;
    int nlist, m, grid;        // grid: workgroups of the search over the rows
    const int64_t *ids;        // [m]
    int64_t *sorted;           // scratch [kDeleteChunk]
    uint32_t *unit_start;      // scratch [nlist + 1]: units of the lists before each one
    unsigned long long *hits;  // scratch [kDeleteChunk]: (list << 32) | position of the rows to go
    uint32_t *hit_len0;        // scratch [kDeleteChunk]: per hit, its list's length before the pass,
    uint32_t *hit_seg0;        //   where the list's hits start in the sorted hits,
    uint32_t *hit_cnt;         //   and how many they are
    uint32_t *scal;            // [0] rows found in this pass, [1] units, [2] sticky: a pass found more than it could take
    unsigned long long *removed; // device counter, added to
};
hipError_t launch_delete(const DeleteArgs &a, hipStream_t s);
// copies every list into the contiguous extents of `dst` (dst's tables are already in place)
// (skip: optional [dst nlist] flags of lists the caller fills itself; lists beyond src's are skipped too)
hipError_t launch_compact_pages(const DevIndex *src, const DevIndex *dst, uint32_t new_pages, const uint8_t *skip,
                                hipStream_t s);
// the first min(len, length of list l) members of list l as dense fp32 rows [.][d] and / or their ids
hipError_t launch_gather_list(const DevIndex *ix, uint32_t l, uint32_t len, float *rows, int64_t *ids, hipStream_t s);
// 2-means of every list to split, all lists in the same launches, straight from the lists' pages
// (Section 4.4: a light k-means on the device decides the split).  Job j splits list job_list[j].
constexpr int kSplitUnit = 1024; // rows of one list that a workgroup assigns at a time
struct SplitArgs {
    const DevIndex *ix;
    int njobs;
    const uint32_t *job_list;  // [njobs]
    const uint32_t *job_len;   // [njobs] members
    const uint32_t *job_unit0; // [njobs + 1] units of the jobs before each one
    const uint32_t *job_row0;  // [njobs] members of the jobs before each one: where the job's part of side[] starts
    double *cent;              // [njobs][2][d] the two centroids
    double *sum;               // [njobs][2][d] sums of the members of each side (zero between the launches)
    unsigned long long *cnt;   // [njobs][2] members of each side (zero between the launches)
    unsigned long long *cnt_out; // [njobs][2] the counts of the last assignment
    int32_t *side;             // [sum of job_len] 0 / 1 per member, by position in its list
};
// first centroids: the member with the smallest id and the member with the largest id
hipError_t launch_split_init(const SplitArgs &a, hipStream_t s);
// one Lloyd iteration: every member to the nearer centroid (ties to the first), then the centroids to the
// means of their members (a centroid without members stays)
hipError_t launch_split_iterate(const SplitArgs &a, uint32_t total_units, int d, hipStream_t s);
// the jobs' centroids into a dense fp32 table [.][d]: row job_list[j] and row nlist0 + j
hipError_t launch_split_centroids(const SplitArgs &a, int nlist0, float *dense, hipStream_t s);
// list l of src split by side[r]: side 0 stays list l of dst, side 1 becomes list lnew of dst (slot: scratch [len])
hipError_t launch_split_list(const DevIndex *src, const DevIndex *dst, uint32_t l, uint32_t lnew, const int32_t *side,
                             uint32_t *slot, uint32_t len, hipStream_t s);
// k-means update step (Lloyd): members of every cluster gathered, then one workgroup per cluster
struct KmeansArgs {
    const float *x;        // [n][d] training rows
    const int32_t *assign; // [n] cluster of each row
    int64_t n;
    int d, nlist;
    uint32_t *cnt, *start, *fill; // [nlist] each (scratch)
    uint32_t *members;     // [n] row numbers in cluster-major order (scratch)
    float *centroids;      // [nlist][d] in: centroids the assignment used; out: means of the members
    double *sums;          // [nlist][d] scratch: per-cluster totals
    double *sq;            // [nlist] scratch: per-cluster totals of |x|^2
    double *inertia;       // one word: receives the sum of squared distances of the assignment
};
hipError_t launch_kmeans_update(const KmeansArgs &a, hipStream_t s);
// Insert: slots for the vectors of every handle of the batch (one workgroup per handle, at most 1024
// vectors each; rows [qlo[a], qlo[a+1]) of assign / slots / assigned_out belong to handle a), then the rows.
// batches of at most this many vectors per handle: reservation and row writes share one launch
constexpr int kFusedAppend = 64;
struct AppendIds {
    int64_t id0[PK_MAX_HANDLES]; // first id of each handle's segment when the caller gives no ids
};
hipError_t launch_reserve(const MultiArgs &ma, const int32_t *assign, uint32_t *slots, int32_t *assigned_out, hipStream_t s);
hipError_t launch_append(const MultiArgs &ma, const AppendIds &idc, const float *x, const int64_t *ids,
                         const int32_t *assign, const uint32_t *slots, hipStream_t s);
// assign == null: the lists are the low words of best[] (left by the centroid kernel), which is reset to ~0
hipError_t launch_reserve_append(const MultiArgs &ma, const AppendIds &idc, const float *x, const int64_t *ids,
                                 const int32_t *assign, unsigned long long *best, uint32_t *slots, int32_t *assigned_out,
                                 hipStream_t s);

} // namespace pk
