// C ABI of libpancake: handle management, arena layout, host-side bounds and the launch
// sequences of build, insert and search.  See include/pancake.h for the contract.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "pk_internal.h"

using namespace pk;

namespace {

constexpr uint64_t kMagic = 0x70616e63616b6531ull;
constexpr uint64_t kRegionBytes = 256ull << 20; // emission regions of one launch sequence (all queries together)
constexpr int kBuildChunk = 16384;          // vectors assigned per coarse pass during the build
constexpr int kInsertFast = 1024;           // most vectors of an insert call that takes the two-launch path

#define PK_HIP(expr)                                   \
    do {                                               \
        if ((expr) != hipSuccess) return PK_ERR_HIP;   \
    } while (0)
#define PK_TRY(expr)                                   \
    do {                                               \
        const int rc_ = (expr);                        \
        if (rc_ != PK_OK) return rc_;                  \
    } while (0)

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Workspace of pk_search_noalloc: a file-scope device array, so that the call needs no
// hipMalloc.  Every GPU the library is loaded on holds its own copy until the process ends.
// In host code the name `scratch` is only a stand-in for the symbol, never a device address:
// the address on the current device comes from hipGetSymbolAddress (scratch_on_device) and
// that pointer is what kernels and copies get.
constexpr size_t kScratchBytes = (size_t)PK_NOALLOC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kScratchDevices = 64;
std::atomic<char *> g_scratch_ptr[kScratchDevices];

// address of this device's copy of `scratch` (resolved once per device, with that device current)
int scratch_on_device(char **out)
{
    int dev = 0;
    PK_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kScratchDevices) return PK_ERR_UNSUPPORTED;
    char *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        void *sym = nullptr;
        if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) {
            (void)hipGetLastError();
            return PK_ERR_HIP;
        }
        p = static_cast<char *>(sym);
        g_scratch_ptr[dev].store(p, std::memory_order_release); // every thread resolves the same address
    }
    *out = p;
    return PK_OK;
}

} // namespace

struct pk_index {
    uint64_t magic;
    pk_config cfg;
    int dpad32, rb32, row_bytes, nlist_pad, P, max_dp;
    size_t page_stride;     // bytes of one page over the three regions
    DevIndex host;          // host copy of the device descriptor
    DevIndex *dev;          // device copy, inside the first arena
    uint32_t pages_total;
    size_t arena_bytes;
    std::vector<uint64_t> top_len; // [j] = total length of the j longest lists when the layout was last fixed (build, compaction)
    int64_t inserted_at_top;       // n_inserted at that moment
    int64_t n_total, n_inserted;
    int64_t n_refused;             // vectors of batches the device refused (found when the stats are read)
    int64_t next_id;               // vectors ever added: the running id counter (deletes do not lower it)
    // page accounting: last page counter read back, and how many vectors were inserted by then
    uint32_t pages_known;
    int64_t inserted_at_known;
    uint32_t *pin_pages;
    hipEvent_t ev;
    bool ev_pending;
    int64_t ev_inserted;
    // library-owned workspace
    char *ws;
    size_t ws_bytes;
    int64_t ws_grows;       // times the workspace was (re)allocated since the build
    int32_t emit_cap;       // entries of a query's emission region set by the caller (0: by k)
    // staging of scope-union searches (replicated queries, per-handle results); grow-only
    char *ubuf;
    size_t ubuf_bytes;
    int lds_limit, num_cu;
    // small inserts: top-1 keys of the batch (kept at ~0 between calls) and the slots the batch got
    unsigned long long *ins_best; // DEVICE [kInsertFast]
    uint32_t *ins_slots;          // DEVICE [kInsertFast]
    // second stream of a search whose lists fall into two tile classes: the kernel for the lists many
    // queries probe is bound by the matrix cores and runs on some of the CUs while the HBM-bound scan of
    // the other lists has the rest (fork and join by events; default priority)
    hipStream_t side;
    hipEvent_t ev_fork, ev_join;
    // stage timing (pk_profile_begin .. pk_profile_end)
    bool prof_on;
    std::vector<hipEvent_t> prof_ev; // 6 events per recorded launch sequence
    std::vector<uint8_t> prof_beside; // per sequence: the two scan kernels ran side by side (the fourth event then
                                      // follows the kernel of the lists many queries probe, not the regular scan)
    size_t prof_used;
};

namespace {

bool live(const pk_index *ix) { return ix && ix->magic == kMagic; }

constexpr size_t kProfEvents = 6;
constexpr size_t kProfMaxLaunches = 1024;

// records the next stage boundary of the current launch sequence, if timing is on
int mark(pk_index *ix, hipStream_t s)
{
    if (!ix->prof_on || ix->prof_used >= kProfEvents * kProfMaxLaunches) return PK_OK;
    if (ix->prof_used == ix->prof_ev.size()) {
        hipEvent_t e;
        PK_HIP(hipEventCreate(&e));
        ix->prof_ev.push_back(e);
    }
    PK_HIP(hipEventRecord(ix->prof_ev[ix->prof_used++], s));
    return PK_OK;
}

struct Carver {
    char *base;
    size_t off;
    template <typename T> T *take(size_t count)
    {
        off = round_up(off, 256);
        T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
        off += count * sizeof(T);
        return p;
    }
};

// true when `s` is being captured into a graph (nothing may wait, free or allocate then)
bool capturing(hipStream_t s)
{
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &st) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return st != hipStreamCaptureStatusNone;
}

int ensure_ws(pk_index *ix, size_t bytes, hipStream_t s)
{
    if (bytes <= ix->ws_bytes) return PK_OK;
    // A captured graph would keep pointers into the buffer that is about to be freed.
    if (capturing(s)) return PK_ERR_WORKSPACE;
    // grow: earlier work on this handle's stream may still use the old buffer
    PK_HIP(hipStreamSynchronize(s));
    if (ix->ws) PK_HIP(hipFree(ix->ws));
    ix->ws = nullptr;
    ix->ws_bytes = 0;
    const size_t want = round_up(bytes + bytes / 8, 1 << 20);
    void *p = nullptr;
    if (hipMalloc(&p, want) != hipSuccess) {
        (void)hipGetLastError();
        return PK_ERR_NOMEM;
    }
    ix->ws = static_cast<char *>(p);
    ix->ws_bytes = want;
    ix->ws_grows += 1;
    return PK_OK;
}

// Pages that `t` more vectors can open at most: one per touched list (its tail page may be
// full) plus one per P vectors.
uint64_t pages_for(const pk_index *ix, uint64_t t)
{
    return (t + ix->P - 1) / ix->P + std::min<uint64_t>(t, (uint64_t)ix->cfg.nlist);
}

uint32_t pages_used_ub(const pk_index *ix, int64_t ahead = 0)
{
    const uint64_t ub =
        (uint64_t)ix->pages_known + pages_for(ix, (uint64_t)(ix->n_inserted - ix->inserted_at_known + ahead));
    return (uint32_t)std::min<uint64_t>(ub, ix->pages_total);
}

// upper bound of one query's candidate range (padded segments) for `nprobe` lists, valid until
// `ahead` more vectors have been inserted
uint64_t wq_ub(const pk_index *ix, int nprobe, int64_t ahead = 0)
{
    const int np = std::min(nprobe, ix->cfg.nlist);
    return round_up(ix->top_len[np] + (uint64_t)(ix->n_inserted - ix->inserted_at_top + ahead) + 15ull * np, 16);
}

// Everything one launch sequence needs, carved out of the owner's workspace.
struct Plan {
    int64_t nq;
    int nprobe, k, nh;
    int mq_f, mq_h, grid_f, grid_h, grid_s, cchunks, K, nlist_max, sp;
    uint32_t hot_from;
    bool hot_rs; // the hot class is scored by the rows-in-registers kernel (tiles of kRrTileRows rows x up to kRrSlots slots)
    double avg_per_list; // queries per list on average (the largest over the handles of the call)
    uint32_t stride, ecap, tile_cap, span;
    uint64_t cbuf_entries; // entries of all emission regions together
    bool need_coarse, need_fine, f16;
    bool raw_queries; // the coarse step reads the caller's query rows directly (no preparation launch)
    bool wl_small;    // the second half of the work list is small enough for one workgroup (rides in the threshold launch)
    // buffers
    char *qs32, *qs;
    float *qn32, *qn, *S, *svals, *tlo, *tinv;
    uint32_t *cand_off, *cand_cnt, *lcnt, *lstart, *lfill, *ltile, *lhtile, *pair_off, *slot_q, *slot_o, *scalars,
        *tau, *tcur, *hist, *ccnt, *sslot_q, *sslot_o;
    uint16_t *qagent;
    Tile *tiles, *tiles_hot, *stiles;
    unsigned long long *cpartial, *cbuf;
    int32_t *probes;
    size_t bytes;
};

void carve(Plan &p, char *base, const pk_index *own)
{
    Carver c{base, 0};
    const size_t nq = (size_t)p.nq;
    p.qs32 = c.take<char>(nq * own->rb32);
    p.qn32 = c.take<float>(nq);
    if (p.f16) {
        p.qs = c.take<char>(nq * own->row_bytes);
        p.qn = c.take<float>(nq);
    } else {
        p.qs = p.qs32;
        p.qn = p.qn32;
    }
    p.qagent = c.take<uint16_t>(nq);
    p.scalars = c.take<uint32_t>(32);
    p.probes = c.take<int32_t>(nq * p.nprobe);
    p.cand_off = c.take<uint32_t>(nq);
    p.cand_cnt = c.take<uint32_t>(nq);
    if (p.need_coarse) {
        p.S = c.take<float>(nq * p.stride + 16);
        p.cpartial = c.take<unsigned long long>(nq * p.cchunks * p.nprobe);
    }
    if (p.need_fine) {
        const size_t nl = (size_t)p.nh * p.nlist_max;
        p.lcnt = c.take<uint32_t>(2 * nl); // pair counters, then the fill marks: cleared together
        p.lfill = p.lcnt ? p.lcnt + nl : nullptr;
        p.lstart = c.take<uint32_t>(nl);
        p.ltile = c.take<uint32_t>(nl);
        p.lhtile = c.take<uint32_t>(nl);
        p.pair_off = c.take<uint32_t>(nq * (p.nprobe + 1));
        p.slot_q = c.take<uint32_t>(nq * p.nprobe);
        p.slot_o = c.take<uint32_t>(nq * p.nprobe);
        p.tiles = c.take<Tile>((size_t)p.tile_cap + 1);
        p.tiles_hot = c.take<Tile>((size_t)p.tile_cap + 1);
        p.tau = c.take<uint32_t>(nq);
        p.tlo = c.take<float>(nq);
        p.tinv = c.take<float>(nq);
        p.tcur = c.take<uint32_t>(nq);
        p.hist = c.take<uint32_t>(nq * kHistBins);
        p.ccnt = c.take<uint32_t>(nq);
        p.sslot_q = c.take<uint32_t>(nq);
        p.sslot_o = c.take<uint32_t>(nq);
        p.stiles = c.take<Tile>(nq * p.sp + 1);
        p.svals = c.take<float>(nq * p.span + 16);
        p.cbuf = c.take<unsigned long long>((size_t)p.cbuf_entries + 16);
    }
    p.bytes = round_up(c.off, 256);
}

// Tuning constants: the measured choices.  A build with -DPK_DEV_TUNABLES reads each of them
// from the environment variable named beside it (once per process), so that a sweep needs no
// rebuild; the shipped library reads no environment variable.
struct Tunables {
    int wgs;      // PK_TUNE_WGS: most scan workgroups per CU
    int mq;       // PK_TUNE_MQ: most query slots per regular tile (0: by expected queries per list)
    int mqh;      // PK_TUNE_MQH: most query slots per tile of the sliced-query kernel
    int ks;       // PK_TUNE_KS: sliced-query kernel 0 never, 1 automatic, 2 every list, 3 lists above one group
    int sp_max;   // PK_TUNE_SP_MAX: most sample pages per query beyond the k rows needed
    int gemm_wgs; // PK_TUNE_GEMM_WGS: fewest 128 x 128 tiles for which the coarse step uses the GEMM
    int densesel; // PK_TUNE_DENSESEL: register top-nprobe selection of the coarse scores (1) or chunked (0)
    int grabdiv;  // PK_TUNE_GRABDIV: tiles per claimed batch = tiles / (grid * this), at most 8
    int hist;     // PK_TUNE_HIST: emission gate tightened by the bucket histogram (1) or sample threshold only (0)
    int rs_from;  // PK_TUNE_RS_FROM: lists probed by more queries than this go to the rows-stationary kernel
                  // (0: lists with more queries than one group of the regular kernel; -1: none)
    int rs_nq;    // PK_TUNE_RS_NQ: fewest queries of a batch for which the rows-stationary class exists
    int hot_grab; // PK_TUNE_HOT_GRAB: tiles per claim of the rows-stationary kernels
    int hot_cus;  // PK_TUNE_HOT_CUS: CUs given to the rows-in-registers kernel while it runs beside the regular
                  // lists' scan (0: one after the other on the caller's stream)
    int wl_aside; // PK_TUNE_WL_ASIDE: large batches build the second half of the work list beside the sample scan
    int fuse_tau; // PK_TUNE_FUSE_TAU: small batches take sample, thresholds and work list in one launch
};

#ifdef PK_DEV_TUNABLES
#define PK_TUNABLES_STORAGE static thread_local
#else
#define PK_TUNABLES_STORAGE static const
#endif

const Tunables &tunables()
{
#ifdef PK_DEV_TUNABLES
    PK_TUNABLES_STORAGE Tunables t;
    t = [] { // read on every call, so one process can sweep
#else
    PK_TUNABLES_STORAGE Tunables t = [] {
#endif
        auto env = [](const char *name, int dflt) {
#ifdef PK_DEV_TUNABLES
            const char *v = getenv(name);
            return v ? atoi(v) : dflt;
#else
            (void)name;
            return dflt;
#endif
        };
        return Tunables{env("PK_TUNE_WGS", 4),       env("PK_TUNE_MQ", 0),        env("PK_TUNE_MQH", 64),
                        env("PK_TUNE_KS", 1),        env("PK_TUNE_SP_MAX", 16),   env("PK_TUNE_GEMM_WGS", 128),
                        env("PK_TUNE_DENSESEL", 1),  env("PK_TUNE_GRABDIV", 8),   env("PK_TUNE_HIST", 1),
                        env("PK_TUNE_RS_FROM", 0),   env("PK_TUNE_RS_NQ", 512),   env("PK_TUNE_HOT_GRAB", 1),
                        env("PK_TUNE_HOT_CUS", 96),  env("PK_TUNE_WL_ASIDE", 1),  env("PK_TUNE_FUSE_TAU", 1)};
    }();
    return t;
}

// a tile of the threshold sample scores one query against one page of its first probed list
constexpr int kSampleSlots = 1;

int grid_for(const pk_index *ix, int row_bytes, int mq)
{
    const int lds = scan_lds_bytes(row_bytes, mq);
    int per_cu = (160 * 1024) / lds;
    per_cu = std::max(1, std::min(per_cu, tunables().wgs));
    return ix->num_cu * per_cu;
}

bool coarse_by_gemm(uint32_t nqa, const pk_index *ix);

uint32_t pow2_at_least(uint64_t v)
{
    uint32_t p = 1;
    while (p < v && p < (1u << 30)) p <<= 1;
    return p;
}

// Entries of one query's emission region.  The gate (sample threshold + running histogram)
// lets a few times k candidates through on evenly sized lists, so a few dozen times k with a
// floor is ample there; a query whose best list is very long lets more through before the
// histogram has tightened (its threshold is a quantile of the sample, and that quantile of a
// 400 000-row list is thousands of rows), so a batch of few queries gets regions of up to
// 32768 entries: all regions of a call together stay near 32 MB.  A query that emits more than
// its region holds is selected by rescoring its rows (select_final_kernel), one workgroup for
// the whole query: the size is a matter of speed, not of correctness.  If every candidate a
// query can have fits, nothing can overflow and the region is just that large.
uint32_t emit_cap_for(const pk_index *own, int K, uint64_t wmax, int64_t nq)
{
    uint64_t e = std::min<uint64_t>(std::max<uint64_t>(pow2_at_least(32ull * (uint64_t)K), 2048), 32768);
    const uint64_t roomy = (4ull << 20) / (uint64_t)std::max<int64_t>(nq, 1); // entries per query at 32 MB in all
    e = std::max(e, std::min<uint64_t>(32768, roomy / 1024 * 1024));
    if (own->emit_cap > 0) e = (uint64_t)own->emit_cap;
    e = std::min<uint64_t>(e, round_up(wmax, 16));
    return (uint32_t)std::max<uint64_t>(e, round_up((uint64_t)K, 16));
}

// Fills the plan for handles hs[0..nh) with query segments qlo (relative to this batch).
// ahead > 0 sizes the buffers for what the same call would need after `ahead` more inserts
// into every handle; worst also takes the largest value of every size that depends on how the
// queries spread (tile groups, sample pages), which is how pk_workspace_reserve sizes the
// workspace for every call within its limits.
int make_plan(Plan &p, pk_index *const *hs, int nh, const uint32_t *qlo, int64_t nq, int k, int nprobe,
              bool need_coarse, bool need_fine, int64_t ahead = 0, bool worst = false)
{
    const pk_index *own = hs[0];
    std::memset(&p, 0, sizeof(p));
    p.nq = nq;
    p.nprobe = nprobe;
    p.k = k;
    p.nh = nh;
    p.need_coarse = need_coarse;
    p.need_fine = need_fine;
    p.f16 = own->cfg.storage == PK_F16;
    p.mq_f = scan_max_mq(own->row_bytes, own->cfg.storage, own->lds_limit);
    {
        // Query slots per scan tile: the smallest group that holds the expected number of
        // queries per probed list; small groups keep the LDS tile small and the occupancy
        // high, and a list probed by more queries is scored once per group (its pages are
        // re-read from L2 / Infinity Cache, which measured faster than larger groups).
        // If even that tile would leave one workgroup per CU (wide fp32 rows), the
        // sliced-query kernel, whose LDS use does not depend on the row length, takes every
        // list.  The ks tunable can force either kernel, or route only lists with more queries
        // than one group to the sliced kernel (3).
        double avg = 0;
        for (int a = 0; a < nh; ++a)
            avg = std::max(avg, (double)(qlo[a + 1] - qlo[a]) * nprobe / hs[a]->cfg.nlist);
        p.avg_per_list = avg;
        const int want = avg <= 6 ? 16 : (avg <= 20 ? 32 : 64);
        p.mq_f = std::min(p.mq_f, tunables().mq > 0 ? tunables().mq : want);
        p.mq_h = own->cfg.storage == PK_F16 ? 64 : 32;
        p.mq_h = std::min(p.mq_h, tunables().mqh);
        const int ks = tunables().ks;
        const bool wide = p.mq_f < 16 || scan_lds_bytes(own->row_bytes, p.mq_f) > 64 * 1024;
        if (ks == 2 || (ks == 1 && wide)) p.hot_from = 0;
        else if (ks == 3) p.hot_from = (uint32_t)p.mq_f;
        else p.hot_from = 0xffffffffu;
        // Large batches over narrow rows: a list probed by more queries than one group holds is scored
        // with its rows stationary in registers, all its queries streaming past them, instead of once
        // per query group (pages must split into tiles of kRrTileRows rows).
        if (p.hot_from == 0xffffffffu && tunables().rs_from >= 0 && nq >= tunables().rs_nq && own->row_bytes <= 1536 &&
            own->P % kRrTileRows == 0 && scan_rr_lds_bytes() <= own->lds_limit) {
            bool same = true; // one tile geometry for all handles of the call
            for (int a = 1; a < nh; ++a) same = same && hs[a]->P == own->P;
            if (same) {
                p.hot_rs = true;
                p.hot_from = tunables().rs_from > 0 ? (uint32_t)tunables().rs_from : (uint32_t)p.mq_f;
                p.mq_h = kRrSlots;
            }
        }
        if (p.hot_from == 0) {
            p.mq_h = std::min(p.mq_h, std::max(want, 16));
            if (p.mq_f < 16) p.mq_f = 16; // unused, but keeps the tile arithmetic defined
        }
    }
    if (p.mq_f < 16) return PK_ERR_UNSUPPORTED;
    p.grid_f = grid_for(own, own->row_bytes, p.mq_f);
    p.grid_h = own->num_cu * std::max(1, std::min((160 * 1024) / scan_ks_lds_bytes(p.mq_h), tunables().wgs));
    if (p.hot_rs) p.grid_h = own->num_cu; // one workgroup of 8 waves per CU (its LDS holds the rows and every slot)
    p.grid_s = grid_for(own, own->row_bytes, kSampleSlots);
    p.K = k + 1;
    p.sp = (k + own->P - 1) / own->P; // sample pages: at least k rows when the first pages are full
    uint64_t tiles = 0, wmax = 0, lmax = 0;
    int nlist_hi = 0, pad_hi = 0;
    const int mq_least = worst ? 16 : std::min(p.mq_f, p.mq_h);
    const bool rs_tiles = worst ? (own->row_bytes <= 1536 && own->P % kRrTileRows == 0) : p.hot_rs;
    for (int a = 0; a < nh; ++a) {
        const pk_index *ix = hs[a];
        const uint64_t nqa = worst ? (uint64_t)nq : qlo[a + 1] - qlo[a];
        nlist_hi = std::max(nlist_hi, ix->cfg.nlist);
        pad_hi = std::max(pad_hi, ix->nlist_pad);
        if (nqa == 0) continue;
        const uint64_t w = wq_ub(ix, nprobe, ahead);
        if (w > 0xfffffff0ull) return PK_ERR_UNSUPPORTED; // positions inside a query's range are 32-bit
        wmax = std::max(wmax, w);
        lmax = std::max(lmax, wq_ub(ix, 1)); // the longest list as it may be now
        const uint64_t pp = w / ix->P + nprobe;
        const uint64_t pages = std::min<uint64_t>(pages_used_ub(ix, ahead), nqa * pp);
        tiles += pages + nqa * pp / mq_least + 1;
        // tiles of the rows-in-registers kernel are parts of a page (P / kRrTileRows times the pages), and a
        // list probed by more than kRrSlots queries has one tile per group of that many
        if (rs_tiles) tiles += (uint64_t)(ix->P / kRrTileRows) * pages * ((uint64_t)(nqa + kRrSlots - 1) / kRrSlots);
    }
    if (tiles > 0xfffffff0ull) return PK_ERR_UNSUPPORTED;
    {
        // Sample pages per query.  A larger sample gives a tighter threshold and a finer bucket
        // scale, hence fewer emitted candidates; it costs one tile per query and page.  Wanted:
        // the k-th best of the sample at most its 40 % quantile (large k).  And for batches of
        // few queries, whose emitted candidates all meet at a handful of counters and serialise
        // there: the query that lands in the longest list emits a share of that list's rows that
        // falls as 1 / pages, about 1 ns of serialised emission per row of the list at one page
        // (measured: 60 k entries from a 444 k-row list, 0.45 ms), while a page costs every query
        // a tile: 0.7 us of latency plus its bytes at 10 TB/s while the tiles fit the chip side by
        // side.  The sum is least at pages = sqrt(first cost / second).
        // Spent: at most 3 % of the scan's tiles, and sp_max pages.
        const uint64_t afford = tiles * 3u / 100u / (uint64_t)std::max<int64_t>(nq, 1);
        const uint64_t by_quantile = ((uint64_t)p.K * 10 + 3 * own->P - 1) / (3 * own->P);
        uint64_t by_size = 0;
        if (nq <= 64) {
            const double emit_us = 1.0e-3 * (double)lmax;
            const double page_us = 0.7 + (double)nq * (double)own->P * (double)own->row_bytes / 1.0e7;
            by_size = (uint64_t)std::llround(std::sqrt(emit_us / page_us));
        }
        uint64_t more = std::min(afford, std::max(by_quantile, by_size));
        more = std::min<uint64_t>(more, (uint64_t)tunables().sp_max);
        if (worst) more = (uint64_t)tunables().sp_max;
        p.sp = std::max(p.sp, (int)more);
    }
    p.sp = std::min(p.sp, kMaxSamplePages); // (a sample of fewer than k rows gives no threshold: slower, not wrong)
    p.span = (uint32_t)(p.sp * own->P);
    p.nlist_max = nlist_hi;
    p.stride = (uint32_t)pad_hi;
    p.cchunks = (nlist_hi + kSelChunk - 1) / kSelChunk;
    // Inner product over rows that need no padding: the coarse step can read the caller's queries as they
    // are (no norms, no zero fill), unless a segment is large enough for the GEMM, which wants the prepared copy.
    p.raw_queries = need_coarse && !worst && own->cfg.metric == PK_METRIC_IP && own->cfg.d * 4 == own->rb32;
    for (int a = 0; a < nh && p.raw_queries; ++a)
        if (coarse_by_gemm(qlo[a + 1] - qlo[a], hs[a])) p.raw_queries = false;
    // few lists, pairs and tiles: the threshold kernel's workgroups lay out slots and tiles as well (see wl_spread)
    p.wl_small = (uint64_t)nh * (uint64_t)nlist_hi <= kWlSmallLists && (uint64_t)nq * (uint64_t)nprobe <= 16384 && tiles <= 65536;
    p.ecap = emit_cap_for(own, p.K, wmax, nq);
    p.cbuf_entries = (uint64_t)nq * p.ecap;
    // a smaller batch has larger regions: none needs more in all than this
    if (worst) p.cbuf_entries = std::max<uint64_t>(p.cbuf_entries, std::min<uint64_t>(32768ull * (uint64_t)nq, 4ull << 20));
    p.tile_cap = (uint32_t)tiles;
    carve(p, nullptr, own);
    return PK_OK;
}

// A query segment goes through the 128 x 128-tile MFMA GEMM when it has enough tiles to
// occupy a good part of the chip; smaller segments take the finely cut centroid kernel.
bool coarse_by_gemm(uint32_t nqa, const pk_index *ix)
{
    const uint64_t wgs = (uint64_t)((nqa + 127) / 128) * (uint64_t)((ix->nlist_pad + 127) / 128);
    return wgs >= (uint64_t)tunables().gemm_wgs;
}

void fill_multi(MultiArgs &m, pk_index *const *hs, int nh, const uint32_t *qlo)
{
    std::memset(&m, 0, sizeof(m));
    m.n = nh;
    for (int a = 0; a < nh; ++a) {
        m.ix[a] = hs[a]->dev;
        m.qlo[a] = qlo[a];
    }
    m.qlo[nh] = qlo[nh];
}

// Arguments of the work-list construction and of the threshold sample of one launch sequence.
void fill_worklist_args(const Plan &p, const pk_index *own, WorklistArgs &w, SampleArgs &sm)
{
    // threshold sampling: k-th best of the first pages of each query's first probed list
    sm = SampleArgs{};
    sm.probes = p.probes;
    sm.qagent = p.qagent;
    sm.nq = p.nq;
    sm.nprobe = p.nprobe;
    sm.sp = p.sp;
    sm.k = p.k;
    sm.metric = own->cfg.metric;
    sm.scan_grid = p.grid_s;
    sm.span = p.span;
    sm.tiles = p.stiles;
    sm.slot_query = p.sslot_q;
    sm.slot_out = p.sslot_o;
    sm.vals = p.svals;
    sm.scalars = p.scalars + 8;
    sm.tau = p.tau;
    sm.tlo = p.tlo;
    sm.tinv = p.tinv;
    sm.tcur = p.tcur;
    sm.hist = p.hist;
    w = WorklistArgs{};
    w.probes = p.probes;
    w.qagent = p.qagent;
    w.nq = p.nq;
    w.nprobe = p.nprobe;
    w.n_handles = p.nh;
    w.nlist_max = p.nlist_max;
    w.mq = p.mq_f;
    w.mq_hot = p.mq_h;
    w.hot_from = p.hot_from;
    w.hot_rows = p.hot_rs ? kRrTileRows : 0;
    w.scan_grid = p.grid_f;
    w.scan_grid_hot = p.grid_h;
    w.grab_div = tunables().grabdiv;
    w.hot_grab = tunables().hot_grab;
    w.lcnt = p.lcnt;
    w.lstart = p.lstart;
    w.lfill = p.lfill;
    w.ltile = p.ltile;
    w.lhtile = p.lhtile;
    w.pair_off = p.pair_off;
    w.ccnt = p.ccnt;
    w.slot_query = p.slot_q;
    w.slot_out = p.slot_o;
    w.tiles = p.tiles;
    w.tiles_hot = p.tiles_hot;
    w.tile_cap = p.tile_cap;
    w.scalars = p.scalars + 4;
    w.scalars_hot = p.scalars + 12;
    w.lcnt_cleared = p.need_coarse;
    if (p.nh == 1) {
        w.len1 = own->host.list_len;
        w.P1 = (uint32_t)own->host.P;
        w.nlist1 = (uint32_t)own->host.nlist;
    }
}

// Coarse search of one batch: probes[nq][nprobe] in the plan's workspace.
// counted (optional): set when the selection also did the first half of the work-list construction for the fine step.
int run_coarse(const Plan &p, const MultiArgs &m, pk_index *const *hs, const float *q, hipStream_t s, bool *counted = nullptr)
{
    if (counted) *counted = false;
    const pk_index *own = hs[0];
    QueryMeta qm{};
    qm.stride = p.stride;
    qm.cand_off = p.cand_off;
    qm.cand_cnt = p.cand_cnt;
    qm.qagent = p.qagent;
    qm.clear = p.need_fine ? p.lcnt : nullptr;
    qm.nclear = p.need_fine ? 2u * (uint32_t)p.nh * (uint32_t)p.nlist_max : 0u; // and the fill marks behind them
    // small segments: one launch of the centroid kernel for all of them
    CentroidArgs ca{};
    if (p.raw_queries) {
        // the caller's rows are usable as they are and no norms are needed: the centroid kernel does the bookkeeping
        ca.qs = reinterpret_cast<const char *>(q);
        ca.qnorm = nullptr;
        ca.meta = qm;
    } else {
        PK_HIP(launch_prep_coarse(q, p.nq, own->cfg.d, own->rb32, p.qs32, p.qn32, qm, m, s));
        ca.qs = p.qs32;
        ca.qnorm = p.qn32;
    }
    ca.out = p.S;
    ca.stride = p.stride;
    ca.row_bytes = own->rb32;
    ca.metric = own->cfg.metric;
    uint32_t longest = 0;
    for (int a = 0; a < m.n; ++a) {
        const uint32_t nqa = m.qlo[a + 1] - m.qlo[a];
        if (!coarse_by_gemm(nqa, hs[a])) longest = std::max(longest, nqa);
    }
    // Queries per workgroup: as many as one workgroup takes (64) when that still leaves a workgroup for every
    // CU; fewer otherwise, since the kernel is a chain of dependent slices and a chip half empty gains nothing
    // from the centroid rows a larger group shares.
    ca.chunk = (int)std::min<uint32_t>(64, (longest + 15) / 16 * 16);
    uint64_t wgs = 0;
    while (true) {
        wgs = 0;
        for (int a = 0; a < m.n; ++a) {
            const uint32_t nqa = m.qlo[a + 1] - m.qlo[a];
            ca.blk[a] = (uint32_t)wgs;
            if (nqa > 0 && !coarse_by_gemm(nqa, hs[a]))
                wgs += (uint64_t)((nqa + ca.chunk - 1) / ca.chunk) * (uint64_t)(hs[a]->nlist_pad / 16);
        }
        if (wgs >= (uint64_t)own->num_cu || ca.chunk <= 16) break;
        ca.chunk -= 16;
    }
    if (wgs > 0x7fffffffull) return PK_ERR_UNSUPPORTED;
    ca.blk[m.n] = (uint32_t)wgs;
    if (wgs > 0) PK_HIP(launch_centroid_scores(ca, m, s));
    for (int a = 0; a < m.n; ++a) {
        const uint32_t nqa = m.qlo[a + 1] - m.qlo[a];
        if (nqa == 0 || !coarse_by_gemm(nqa, hs[a])) continue;
        const pk_index *ix = hs[a];
        GemmArgs g{};
        g.q = reinterpret_cast<const float *>(p.qs32) + (size_t)m.qlo[a] * ix->dpad32;
        g.c = ix->host.cent;
        g.qnorm = p.qn32 + m.qlo[a];
        g.cnorm = ix->host.cnorm;
        g.out = p.S + (size_t)m.qlo[a] * p.stride;
        g.m = (int)nqa;
        g.n = ix->cfg.nlist;
        g.n_pad = ix->nlist_pad;
        g.n_store = ix->nlist_pad;
        g.ld = ix->dpad32;
        g.metric = ix->cfg.metric;
        g.stride = p.stride;
        PK_HIP(launch_gemm_scores(g, s));
    }
    if (p.nlist_max <= kDenseSelectMax && tunables().densesel) {
        if (counted && p.need_fine) {
            // the selection's workgroups go on to count their queries' pairs and lay out the sample
            WorklistArgs w;
            SampleArgs sm;
            fill_worklist_args(p, own, w, sm);
            PK_HIP(launch_select_dense(p.S, p.cand_off, p.cand_cnt, (uint32_t)p.nlist_max, own->cfg.metric, p.nprobe, p.nq,
                                       p.probes, s, &w, &sm, &m));
            *counted = true;
            return PK_OK;
        }
        PK_HIP(launch_select_dense(p.S, p.cand_off, p.cand_cnt, (uint32_t)p.nlist_max, own->cfg.metric, p.nprobe, p.nq,
                                   p.probes, s));
        return PK_OK;
    }
    SelectArgs se{};
    se.vals = p.S;
    se.qoff = p.cand_off;
    se.qcnt = p.cand_cnt;
    se.metric = own->cfg.metric;
    se.K = p.nprobe;
    se.nchunks = p.cchunks;
    se.chunk = kSelChunk;
    se.partial = p.cpartial;
    PK_HIP(launch_select_partial(se, p.nq, s));
    PK_HIP(launch_select_probes(p.cpartial, p.cchunks, p.nprobe, p.nprobe, p.nq, p.probes, s));
    return PK_OK;
}

// Fine search of one batch over p.probes.
int run_fine(const Plan &p, const MultiArgs &m, pk_index *own, const float *q, int64_t *out_ids, float *out_dist,
             hipStream_t s, bool timed, bool counted, bool fixed)
{
    if (p.f16) PK_HIP(launch_prep_queries(q, p.nq, own->cfg.d, PK_F16, own->row_bytes, p.qs, p.qn, s));
    WorklistArgs w;
    SampleArgs sm;
    fill_worklist_args(p, own, w, sm);
    if (!counted) PK_HIP(launch_worklist_count(w, sm, m, s));
    ScanArgs ss{};
    ss.tiles = p.stiles;
    ss.ntiles = p.scalars + 8;
    ss.tile_ctr = p.scalars + 9;
    ss.batch = p.scalars + 10;
    ss.qs = p.qs;
    ss.qnorm = p.qn;
    ss.slot_query = p.sslot_q;
    ss.slot_out = p.sslot_o;
    ss.out = p.svals;
    ss.row_bytes = own->row_bytes;
    ss.metric = own->cfg.metric;
    ss.storage = own->cfg.storage;
    ss.mq = kSampleSlots;
    // Large batches: the second half of the work list (two small, latency-bound kernels) needs the pair counts
    // only, not the thresholds: it runs on the handle's second stream while the sample is scored (HBM-bound).
    // (worth the two cross-stream waits only beside a sample of some length: 400 MB are about 80 us)
    const bool wl_aside = !p.wl_small && tunables().wl_aside && own->side && !fixed && !capturing(s) &&
                          (uint64_t)p.nq * p.span * (uint64_t)own->row_bytes >= (400ull << 20);
    if (wl_aside) {
        PK_HIP(hipEventRecord(own->ev_fork, s));
        PK_HIP(hipStreamWaitEvent(own->side, own->ev_fork, 0));
        PK_HIP(launch_worklist_tiles(w, m, own->side));
        PK_HIP(hipEventRecord(own->ev_join, own->side));
    }
    if (p.wl_small && p.span <= 16u * (uint32_t)kSelThreads && tunables().fuse_tau) {
        // small batches: the sample, the thresholds and the slots and tiles of the work list in one launch
        PK_HIP(launch_sample_tau(ss, sm, w, m, p.grid_s, s));
    } else if (p.wl_small) {
        PK_HIP(launch_scan(ss, p.grid_s, s));
        PK_HIP(launch_tau(sm, s, &w, &m)); // its workgroups also lay out the slots and tiles of the work list
    } else {
        PK_HIP(launch_scan(ss, p.grid_s, s));
        PK_HIP(launch_tau(sm, s));
        if (wl_aside) PK_HIP(hipStreamWaitEvent(s, own->ev_join, 0));
        else PK_HIP(launch_worklist_tiles(w, m, s));
    }
    if (timed) PK_TRY(mark(own, s));
    ScanArgs sa{};
    sa.tiles = p.tiles;
    sa.ntiles = p.scalars + 4;
    sa.tile_ctr = p.scalars + 5;
    sa.batch = p.scalars + 6;
    sa.qs = p.qs;
    sa.qnorm = p.qn;
    sa.slot_query = p.slot_q;
    sa.slot_out = p.slot_o;
    sa.out = nullptr;
    sa.tau = p.tau;
    sa.tlo = p.tlo;
    sa.tinv = p.tinv;
    sa.tcur = p.tcur;
    // The running per-query histogram tightens the gate while a query's tiles follow one another; when every
    // tile of the call runs at once (at most one per workgroup of the grid) it can only cost time.
    sa.use_hist = tunables().hist && p.tile_cap > (uint32_t)p.grid_f;
    sa.hist = p.hist;
    sa.k = p.k;
    sa.ecap = p.ecap;
    sa.ccnt = p.ccnt;
    sa.cbuf = p.cbuf;
    sa.row_bytes = own->row_bytes;
    sa.metric = own->cfg.metric;
    sa.storage = own->cfg.storage;
    sa.mq = p.mq_f;
    // Two tile classes: the rows-in-registers kernel (matrix cores, little HBM traffic) takes hot_cus CUs while the
    // regular lists' scan (HBM) runs on the others.  The first goes to the caller's stream, where it starts at once
    // and has its CUs (it needs whole ones: a wave per SIMD with all its registers) by the time the scan, launched
    // on the handle's second stream behind an event, brings its workgroups; the caller's stream then waits for the
    // scan.  The first only reads the bucket limits the scan publishes (whatever they are by then: a looser gate
    // emits more, never less).  Not under capture, and not for a fixed workspace shared by all handles of the
    // process: there the two run one after the other.
    // Nor when the average list is probed by more queries than a regular tile holds: then most lists are of the
    // first kernel's class, and it should have the whole chip rather than a part of it beside an idle scan.
    const bool beside = p.hot_rs && p.hot_from > 0 && p.hot_from != 0xffffffffu && tunables().hot_cus > 0 &&
                        tunables().hot_cus < own->num_cu && own->side && !fixed && !capturing(s) &&
                        p.avg_per_list < (double)p.hot_from;
    ScanArgs sh = sa;
    sh.tiles = p.tiles_hot;
    sh.ntiles = p.scalars + 12;
    sh.tile_ctr = p.scalars + 13;
    sh.batch = p.scalars + 14;
    sh.mq = p.mq_h;
    if (beside) {
        sh.use_hist = 0;
        PK_HIP(hipEventRecord(own->ev_fork, s));
        PK_HIP(launch_scan_rr(sh, tunables().hot_cus, s));
        PK_HIP(hipStreamWaitEvent(own->side, own->ev_fork, 0));
        PK_HIP(launch_scan(sa, p.grid_f, own->side));
        PK_HIP(hipEventRecord(own->ev_join, own->side));
        if (timed) {
            own->prof_beside.push_back(1);
            PK_TRY(mark(own, s)); // after the kernel of the lists many queries probe
        }
        PK_HIP(hipStreamWaitEvent(s, own->ev_join, 0));
        if (timed) PK_TRY(mark(own, s));
    } else {
        if (p.hot_from > 0) PK_HIP(launch_scan(sa, p.grid_f, s));
        if (timed) {
            own->prof_beside.push_back(0);
            PK_TRY(mark(own, s)); // after the regular lists' scan
        }
        if (p.hot_from != 0xffffffffu) {
            if (p.hot_rs) {
                sh.use_hist = 0; // the regular lists' scan has published its limits; this one only reads them
                PK_HIP(launch_scan_rr(sh, p.grid_h, s));
            } else {
                PK_HIP(launch_scan_ks(sh, p.grid_h, s));
            }
        }
        if (timed) PK_TRY(mark(own, s));
    }
    FinalArgs f{};
    f.K = p.K;
    f.k = p.k;
    f.nprobe = p.nprobe;
    f.metric = own->cfg.metric;
    f.storage = own->cfg.storage;
    f.row_bytes = own->row_bytes;
    f.keys = p.cbuf;
    f.spill = p.cbuf;
    f.ecap = p.ecap;
    f.qcnt = p.ccnt;
    f.pair_off = p.pair_off;
    f.probes = p.probes;
    f.qagent = p.qagent;
    f.qs = p.qs;
    f.qnorm = p.qn;
    f.out_ids = out_ids;
    f.out_dist = out_dist;
    PK_HIP(launch_select_final(f, m, p.nq, s));
    if (timed) PK_TRY(mark(own, s));
    return PK_OK;
}

// qagent for runs that skip the coarse stage (forced probes): one handle only
int set_single_agent(const Plan &p, hipStream_t s)
{
    // uint16 zeros, written as uint32 words (the buffer is 256-byte aligned and padded)
    PK_HIP(launch_fill_u32(reinterpret_cast<uint32_t *>(p.qagent), 0u, ((size_t)p.nq + 1) / 2, s));
    return PK_OK;
}

enum Mode { kFull, kCoarseOnly, kForced };

// fixed_ws: a workspace the call must fit into whole (no growth, no allocation, one launch
// sequence), or null for the handle's own grow-only workspace.
int search_impl(pk_index *const *hs, int nh, const int64_t *q_offsets, const float *queries, int k, int nprobe,
                Mode mode, const int32_t *forced, int32_t *out_probes, int64_t *out_ids, float *out_dist, hipStream_t s,
                char *fixed_ws = nullptr, size_t fixed_bytes = 0)
{
    pk_index *own = hs[0];
    const int64_t nq_all = q_offsets[nh];
    const int d = own->cfg.d;
    // queries per launch sequence: the emission regions of one sequence stay within kRegionBytes
    uint64_t wmax = 1;
    for (int a = 0; a < nh; ++a) wmax = std::max(wmax, wq_ub(hs[a], nprobe));
    const uint64_t per_query = (uint64_t)emit_cap_for(own, k + 1, wmax, 32768) * sizeof(unsigned long long);
    const int64_t step = std::max<int64_t>(1, std::min<int64_t>(32768, (int64_t)(kRegionBytes / per_query)));
    std::vector<uint32_t> qlo(nh + 1);
    for (int64_t q0 = 0; q0 < nq_all; q0 += step) {
        const int64_t nq = std::min(step, nq_all - q0);
        for (int a = 0; a <= nh; ++a)
            qlo[a] = (uint32_t)std::min<int64_t>(std::max<int64_t>(q_offsets[a] - q0, 0), nq);
        Plan p;
        PK_TRY(make_plan(p, hs, nh, qlo.data(), nq, k, nprobe, mode != kForced, mode != kCoarseOnly));
        if (fixed_ws) {
            if (nq != nq_all || p.bytes > fixed_bytes) return PK_ERR_WORKSPACE;
            carve(p, fixed_ws, own);
        } else {
            PK_TRY(ensure_ws(own, p.bytes, s));
            carve(p, own->ws, own);
        }
        MultiArgs m;
        fill_multi(m, hs, nh, qlo.data());
        const float *q = queries + (size_t)q0 * d;
        if (p.raw_queries) { // the fine step reads the same rows (fp16 indexes convert their own copy)
            p.qs32 = const_cast<char *>(reinterpret_cast<const char *>(q));
            if (!p.f16) p.qs = p.qs32;
        }
        const bool timed = mode == kFull && own->prof_on && !fixed_ws; // stage timing creates events
        if (timed) PK_TRY(mark(own, s));
        bool counted = false;
        if (mode == kForced) {
            PK_TRY(set_single_agent(p, s));
            PK_HIP(launch_copy_i32(forced + (size_t)q0 * nprobe, p.probes, nq * nprobe, s));
            if (!p.f16) PK_HIP(launch_prep_queries(q, nq, d, PK_F32, own->rb32, p.qs32, p.qn32, s));
        } else {
            PK_TRY(run_coarse(p, m, hs, q, s, &counted));
        }
        if (timed) PK_TRY(mark(own, s));
        if (mode == kCoarseOnly) {
            PK_HIP(launch_copy_i32(p.probes, out_probes + (size_t)q0 * nprobe, nq * nprobe, s));
        } else {
            PK_TRY(run_fine(p, m, own, q, out_ids + (size_t)q0 * k, out_dist + (size_t)q0 * k, s, timed, counted, fixed_ws != nullptr));
        }
    }
    return PK_OK;
}

int check_search_args(const pk_index *ix, const void *q, int64_t nq, int k, int nprobe)
{
    if (!live(ix)) return PK_ERR_BAD_HANDLE;
    if (nq < 0 || (nq > 0 && !q)) return PK_ERR_INVALID_ARG;
    if (k < 1 || k > PK_MAX_K) return PK_ERR_INVALID_ARG;
    if (nprobe < 1 || nprobe > ix->cfg.nlist || nprobe > PK_MAX_NPROBE) return PK_ERR_INVALID_ARG;
    return PK_OK;
}

bool valid_config(const pk_config *c)
{
    if (!c) return false;
    if (c->d < 1 || c->d > PK_MAX_DIM || c->nlist < 1) return false;
    if (c->metric != PK_METRIC_IP && c->metric != PK_METRIC_L2) return false;
    if (c->storage != PK_F32 && c->storage != PK_F16) return false;
    if (c->page_vecs != 0 && (c->page_vecs < 32 || c->page_vecs > 1024 || c->page_vecs % 32 != 0)) return false;
    if (c->max_delta_pages < 0) return false;
    return true;
}

struct Dims {
    int dpad32, rb32, row_bytes, nlist_pad, P, max_dp;
    size_t header, page_stride;
};

Dims dims_of(const pk_config *c)
{
    Dims x;
    x.rb32 = (int)round_up((size_t)c->d * 4, kIterBytes);
    x.dpad32 = x.rb32 / 4;
    x.row_bytes = c->storage == PK_F16 ? (int)round_up((size_t)c->d * 2, kIterBytes) : x.rb32;
    x.nlist_pad = (int)round_up(c->nlist, kCentroidPad);
    x.P = c->page_vecs ? c->page_vecs : 128;
    x.max_dp = c->max_delta_pages ? c->max_delta_pages : 1024;
    Carver h{nullptr, 0};
    h.take<float>((size_t)x.nlist_pad * x.dpad32);
    h.take<float>(x.nlist_pad);
    h.take<uint32_t>(c->nlist);
    h.take<uint32_t>(c->nlist);
    h.take<uint32_t>(c->nlist);
    h.take<uint32_t>((size_t)c->nlist * x.max_dp);
    h.take<uint32_t>(16);
    h.take<unsigned long long>(8);
    h.take<DevIndex>(1);
    x.header = round_up(h.off, 4096);
    x.page_stride = (size_t)x.P * x.row_bytes + (size_t)x.P * 12;
    return x;
}

// pages that fit into `bytes`, leaving room to align the three regions
uint32_t pages_in(size_t bytes, const Dims &x)
{
    if (bytes < 1024) return 0;
    const size_t n = (bytes - 1024) / x.page_stride;
    return (uint32_t)std::min<size_t>(n, 0x7fffffffu);
}

void place_arena(Arena &a, char *base, uint32_t first_page, uint32_t npages, const Dims &x)
{
    a.first_page = first_page;
    a.npages = npages;
    Carver c{base, 0};
    a.vec = c.take<char>((size_t)npages * x.P * x.row_bytes);
    a.norm = c.take<float>((size_t)npages * x.P);
    a.ids = c.take<int64_t>((size_t)npages * x.P);
}

// Lays the header of an index (centroid table, per-list tables, counters, device descriptor)
// and one arena of pages out in `base`; fills the host descriptor D.  Nothing is written to
// the device.
void place_header(DevIndex &D, DevIndex **dev, uint32_t *pages_total, float **cent, float **cnorm, const pk_config *cfg,
                  char *base, size_t arena_bytes, const Dims &x)
{
    Carver h{base, 0};
    std::memset(&D, 0, sizeof(D));
    *cent = h.take<float>((size_t)x.nlist_pad * x.dpad32);
    *cnorm = h.take<float>(x.nlist_pad);
    D.cent = *cent;
    D.cnorm = *cnorm;
    D.list_len = h.take<uint32_t>(cfg->nlist);
    D.main_base = h.take<uint32_t>(cfg->nlist);
    D.main_pages = h.take<uint32_t>(cfg->nlist);
    D.dtab = h.take<uint32_t>((size_t)cfg->nlist * x.max_dp);
    D.ctr = h.take<uint32_t>(16);
    D.stats = h.take<unsigned long long>(8);
    *dev = h.take<DevIndex>(1);
    D.nlist = cfg->nlist;
    D.nlist_pad = x.nlist_pad;
    D.d = cfg->d;
    D.dpad32 = x.dpad32;
    D.P = x.P;
    D.max_dp = x.max_dp;
    D.metric = cfg->metric;
    D.storage = cfg->storage;
    D.row_bytes = x.row_bytes;
    D.n_arenas = 1;
    *pages_total = pages_in(arena_bytes - x.header, x);
    place_arena(D.arenas[0], base + x.header, 0, *pages_total, x);
}

int snapshot_pages(pk_index *ix, hipStream_t s)
{
    if (ix->ev_pending) {
        const hipError_t e = hipEventQuery(ix->ev);
        if (e == hipSuccess) {
            ix->pages_known = *ix->pin_pages;
            ix->inserted_at_known = ix->ev_inserted;
            ix->ev_pending = false;
        } else if (e != hipErrorNotReady) {
            return PK_ERR_HIP;
        } else {
            (void)hipGetLastError();
        }
    }
    if (!ix->ev_pending) {
        PK_HIP(hipMemcpyAsync(ix->pin_pages, ix->host.ctr, sizeof(uint32_t), hipMemcpyDeviceToHost, s));
        PK_HIP(hipEventRecord(ix->ev, s));
        ix->ev_pending = true;
        ix->ev_inserted = ix->n_inserted;
    }
    return PK_OK;
}

// exact page count (waits for the pending read-back)
int settle_pages(pk_index *ix)
{
    if (ix->ev_pending) {
        PK_HIP(hipEventSynchronize(ix->ev));
        ix->pages_known = *ix->pin_pages;
        ix->inserted_at_known = ix->ev_inserted;
        ix->ev_pending = false;
    }
    return PK_OK;
}

void destroy(pk_index *ix)
{
    if (!ix) return;
    if (ix->ws) (void)hipFree(ix->ws);
    if (ix->ubuf) (void)hipFree(ix->ubuf);
    if (ix->ins_best) (void)hipFree(ix->ins_best);
    if (ix->pin_pages) (void)hipHostFree(ix->pin_pages);
    if (ix->ev) (void)hipEventDestroy(ix->ev);
    if (ix->ev_fork) (void)hipEventDestroy(ix->ev_fork);
    if (ix->ev_join) (void)hipEventDestroy(ix->ev_join);
    if (ix->side) (void)hipStreamDestroy(ix->side);
    for (hipEvent_t e : ix->prof_ev) (void)hipEventDestroy(e);
    ix->magic = 0;
    delete ix;
}

// Host-side capacity check of an insert of m vectors, before anything is enqueued.  Fast
// path: a bound from the last page counter read back.  If that does not clear the batch,
// synchronise, read the exact page counter and list lengths, and test the exact worst case:
// m vectors open the most pages when they first top up the fullest tail pages (cost: free
// slots + 1 each) and then fill whole pages.
int check_capacity(pk_index *ix, int64_t m, hipStream_t s)
{
    if ((uint64_t)ix->pages_known + pages_for(ix, (uint64_t)(ix->n_inserted - ix->inserted_at_known + m)) <=
        ix->pages_total)
        return PK_OK;
    PK_HIP(hipStreamSynchronize(s));
    PK_TRY(settle_pages(ix));
    std::vector<uint32_t> len((size_t)ix->cfg.nlist);
    uint32_t used = 0;
    PK_HIP(hipMemcpy(len.data(), ix->host.list_len, len.size() * 4, hipMemcpyDeviceToHost));
    PK_HIP(hipMemcpy(&used, ix->host.ctr, 4, hipMemcpyDeviceToHost));
    ix->pages_known = used;
    ix->inserted_at_known = ix->n_inserted;
    std::vector<uint32_t> first(len.size());
    const uint32_t P = (uint32_t)ix->P;
    for (size_t l = 0; l < len.size(); ++l) first[l] = (P - len[l] % P) % P + 1;
    std::sort(first.begin(), first.end());
    uint64_t budget = (uint64_t)m, pages = 0;
    for (uint32_t c : first) {
        if (budget < c) break;
        budget -= c;
        ++pages;
    }
    pages += budget / P;
    return (uint64_t)used + pages > ix->pages_total ? PK_ERR_NOMEM : PK_OK;
}

// after an insert: count it, and start a read-back of the page counter once the bound above
// is close enough to the limit that a later batch of 4096 might fail the fast path
int note_inserted(pk_index *ix, int64_t m, hipStream_t s)
{
    ix->n_total += m;
    ix->next_id += m;
    ix->n_inserted += m;
    if ((uint64_t)ix->pages_known + pages_for(ix, (uint64_t)(ix->n_inserted - ix->inserted_at_known + 4096)) <=
        ix->pages_total)
        return PK_OK;
    return snapshot_pages(ix, s);
}

// One launch sequence: top-1 coarse search (unless the lists are given), slot reservation and
// append for the vectors of hs[0..nh), rows [qlo[a], qlo[a+1]) of the batch going to handle a
// (at most 1024 each).  The workspace is that of hs[0].
int insert_batch(pk_index *const *hs, int nh, const uint32_t *qlo, const float *x, const int64_t *ids,
                 const int32_t *forced, int32_t *assigned_out, hipStream_t s)
{
    pk_index *own = hs[0];
    const int64_t m = qlo[nh];
    bool few = forced == nullptr && m <= kInsertFast; // every handle's share small enough for the fused append
    for (int a = 0; a < nh && few; ++a)
        few = qlo[a + 1] - qlo[a] <= (uint32_t)kFusedAppend && !coarse_by_gemm(qlo[a + 1] - qlo[a], hs[a]);
    if (few) {
        // Two launches (three when the rows need preparing), no workspace: the centroid kernel keeps each
        // vector's best (score, list) by atomicMin in the handle's own small buffer, and the kernel that
        // reserves the slots and writes the rows reads the lists from there and resets the words.
        const bool raw = own->cfg.metric == PK_METRIC_IP && own->cfg.d * 4 == own->rb32;
        MultiArgs mm;
        fill_multi(mm, hs, nh, qlo);
        CentroidArgs ca{};
        ca.qs = reinterpret_cast<const char *>(x);
        if (!raw) {
            // prepared rows and norms: the head of the workspace (nothing else of a plan is needed)
            const size_t rows = round_up((size_t)m * own->rb32, 256);
            PK_TRY(ensure_ws(own, rows + round_up((size_t)m * 4, 256), s));
            PK_HIP(launch_prep_queries(x, m, own->cfg.d, PK_F32, own->rb32, own->ws, reinterpret_cast<float *>(own->ws + rows), s));
            ca.qs = own->ws;
            ca.qnorm = reinterpret_cast<float *>(own->ws + rows);
        }
        ca.row_bytes = own->rb32;
        ca.metric = own->cfg.metric;
        ca.best = own->ins_best;
        uint32_t longest = 0;
        for (int a = 0; a < nh; ++a) longest = std::max(longest, qlo[a + 1] - qlo[a]);
        ca.chunk = (int)std::min<uint32_t>(64, (longest + 15) / 16 * 16);
        uint64_t wgs = 0;
        for (int a = 0; a < nh; ++a) {
            const uint32_t ma = qlo[a + 1] - qlo[a];
            ca.blk[a] = (uint32_t)wgs;
            if (ma > 0) wgs += (uint64_t)((ma + ca.chunk - 1) / ca.chunk) * (uint64_t)(hs[a]->nlist_pad / 16);
        }
        if (wgs > 0x7fffffffull) return PK_ERR_UNSUPPORTED;
        ca.blk[nh] = (uint32_t)wgs;
        PK_HIP(launch_centroid_scores(ca, mm, s));
        AppendIds idc{};
        for (int a = 0; a < nh; ++a) idc.id0[a] = hs[a]->next_id;
        PK_HIP(launch_reserve_append(mm, idc, x, ids, nullptr, own->ins_best, own->ins_slots, assigned_out, s));
        for (int a = 0; a < nh; ++a) PK_TRY(note_inserted(hs[a], (int64_t)(qlo[a + 1] - qlo[a]), s));
        return PK_OK;
    }
    Plan p;
    PK_TRY(make_plan(p, hs, nh, qlo, m, 1, 1, forced == nullptr, false));
    const size_t extra = round_up(p.bytes, 256);
    PK_TRY(ensure_ws(own, extra + round_up((size_t)m * 4, 256), s));
    carve(p, own->ws, own);
    uint32_t *slots = reinterpret_cast<uint32_t *>(own->ws + extra);
    MultiArgs mm;
    fill_multi(mm, hs, nh, qlo);
    const int32_t *assign = forced;
    if (!forced) {
        PK_TRY(run_coarse(p, mm, hs, x, s));
        assign = p.probes;
    }
    AppendIds idc{};
    for (int a = 0; a < nh; ++a) idc.id0[a] = hs[a]->next_id;
    bool small = true;
    for (int a = 0; a < nh; ++a) small = small && qlo[a + 1] - qlo[a] <= (uint32_t)kFusedAppend;
    if (small) {
        PK_HIP(launch_reserve_append(mm, idc, x, ids, assign, nullptr, slots, assigned_out, s));
    } else {
        PK_HIP(launch_reserve(mm, assign, slots, assigned_out, s));
        PK_HIP(launch_append(mm, idc, x, ids, assign, slots, s));
    }
    for (int a = 0; a < nh; ++a) PK_TRY(note_inserted(hs[a], (int64_t)(qlo[a + 1] - qlo[a]), s));
    return PK_OK;
}

int insert_impl(pk_index *ix, const float *x, const int64_t *ids, int64_t m, const int32_t *forced,
                int32_t *assigned_out, hipStream_t s)
{
    if (!live(ix)) return PK_ERR_BAD_HANDLE;
    if (m < 0 || (m > 0 && !x)) return PK_ERR_INVALID_ARG;
    if (m == 0) return PK_OK;
    PK_TRY(check_capacity(ix, m, s));
    pk_index *hs[1] = {ix};
    for (int64_t i0 = 0; i0 < m; i0 += 1024) {
        const uint32_t qlo[2] = {0, (uint32_t)std::min<int64_t>(1024, m - i0)};
        PK_TRY(insert_batch(hs, 1, qlo, x + (size_t)i0 * ix->cfg.d, ids ? ids + i0 : nullptr, forced ? forced + i0 : nullptr,
                            assigned_out ? assigned_out + i0 : nullptr, s));
    }
    return PK_OK;
}

} // namespace

// ------------------------------------------------------------------- C ABI

extern "C" {

size_t pk_arena_bytes(const pk_config *cfg, int64_t n, int64_t n_insert_reserve)
{
    if (!valid_config(cfg) || n < 0 || n_insert_reserve < 0) return 0;
    const Dims x = dims_of(cfg);
    const uint64_t pages = (uint64_t)(n + x.P - 1) / x.P + (uint64_t)std::min<int64_t>(n, cfg->nlist) +
                           (uint64_t)(n_insert_reserve + x.P - 1) / x.P +
                           (uint64_t)std::min<int64_t>(n_insert_reserve, cfg->nlist) + 1;
    return x.header + pages * x.page_stride + 4096;
}

int pk_index_build(const pk_config *cfg, const float *centroids, const float *vectors, const int64_t *ids, int64_t n,
                   void *arena, size_t arena_bytes, void *stream, pk_index **out)
{
    if (!out) return PK_ERR_INVALID_ARG;
    *out = nullptr;
    if (!cfg || !centroids || !arena || n < 0 || (n > 0 && !vectors)) return PK_ERR_INVALID_ARG;
    if (cfg->d > PK_MAX_DIM) return PK_ERR_UNSUPPORTED;
    if (!valid_config(cfg)) return PK_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(arena) % 256 != 0) return PK_ERR_INVALID_ARG;
    if (n > 0x7fffffff00ll) return PK_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Dims x = dims_of(cfg);
    if (arena_bytes < x.header + 1024 + x.page_stride) return PK_ERR_NOMEM;

    pk_index *ix = new (std::nothrow) pk_index();
    if (!ix) return PK_ERR_NOMEM;
    ix->magic = kMagic;
    ix->cfg = *cfg;
    ix->dpad32 = x.dpad32;
    ix->rb32 = x.rb32;
    ix->row_bytes = x.row_bytes;
    ix->nlist_pad = x.nlist_pad;
    ix->P = x.P;
    ix->max_dp = x.max_dp;
    ix->cfg.page_vecs = x.P;
    ix->cfg.max_delta_pages = x.max_dp;
    ix->page_stride = x.page_stride;
    ix->arena_bytes = arena_bytes;
    ix->top_len.assign((size_t)cfg->nlist + 1, 0);
    int rc = PK_OK;
    auto fail = [&](int code) {
        (void)hipStreamSynchronize(s);
        destroy(ix);
        return code;
    };

    int dev = 0, lds = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return fail(PK_ERR_HIP);
    ix->lds_limit = lds;
    ix->num_cu = cus > 0 ? cus : 256;
    if (scan_max_mq(x.rb32, PK_F32, lds) < 16 || scan_max_mq(x.row_bytes, cfg->storage, lds) < 16)
        return fail(PK_ERR_UNSUPPORTED);
    if (hipHostMalloc(reinterpret_cast<void **>(&ix->pin_pages), 64, hipHostMallocDefault) != hipSuccess)
        return fail(PK_ERR_HIP);
    if (hipEventCreateWithFlags(&ix->ev, hipEventDisableTiming) != hipSuccess) return fail(PK_ERR_HIP);
    if (hipStreamCreateWithFlags(&ix->side, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&ix->ev_fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&ix->ev_join, hipEventDisableTiming) != hipSuccess)
        return fail(PK_ERR_HIP);
    if (hipMalloc(reinterpret_cast<void **>(&ix->ins_best), (size_t)kInsertFast * 12) != hipSuccess) return fail(PK_ERR_NOMEM);
    ix->ins_slots = reinterpret_cast<uint32_t *>(ix->ins_best + kInsertFast);
    if (launch_fill_u32(reinterpret_cast<uint32_t *>(ix->ins_best), 0xffffffffu, (size_t)kInsertFast * 2, s) != hipSuccess)
        return fail(PK_ERR_HIP);
    {
        // set-up for pk_search_noalloc: resolve this device's copy of its workspace array now, so
        // that the call itself finds the address ready (a failure here is reported by that call)
        char *unused = nullptr;
        (void)scratch_on_device(&unused);
    }

    // header of the first arena
    DevIndex &D = ix->host;
    float *cent = nullptr, *cnorm = nullptr;
    place_header(D, &ix->dev, &ix->pages_total, &cent, &cnorm, cfg, static_cast<char *>(arena), arena_bytes, x);

    if (hipMemcpyAsync(ix->dev, &D, sizeof(D), hipMemcpyHostToDevice, s) != hipSuccess) return fail(PK_ERR_HIP);
    if (launch_fill_u32(D.list_len, 0u, cfg->nlist, s) != hipSuccess ||
        launch_fill_u32(D.main_base, 0u, cfg->nlist, s) != hipSuccess ||
        launch_fill_u32(D.main_pages, 0u, cfg->nlist, s) != hipSuccess ||
        launch_fill_u32(D.dtab, 0xffffffffu, (size_t)cfg->nlist * x.max_dp, s) != hipSuccess ||
        launch_fill_u32(D.ctr, 0u, 16, s) != hipSuccess ||
        launch_fill_u32(reinterpret_cast<uint32_t *>(D.stats), 0u, 16, s) != hipSuccess ||
        launch_fill_u32(D.ctr + 2, ix->pages_total, 1, s) != hipSuccess ||
        launch_store_centroids(centroids, cfg->nlist, cfg->d, x.dpad32, x.nlist_pad, cfg->metric, cent, cnorm, s) !=
            hipSuccess)
        return fail(PK_ERR_HIP);

    std::vector<uint32_t> cnt((size_t)cfg->nlist, 0);
    if (n > 0) {
        int32_t *d_assign = nullptr;
        uint32_t *d_cnt = nullptr;
        if (hipMalloc(reinterpret_cast<void **>(&d_assign), (size_t)n * sizeof(int32_t)) != hipSuccess)
            return fail(PK_ERR_NOMEM);
        if (hipMalloc(reinterpret_cast<void **>(&d_cnt), (size_t)cfg->nlist * 2 * sizeof(uint32_t)) != hipSuccess) {
            (void)hipFree(d_assign);
            return fail(PK_ERR_NOMEM);
        }
        auto fail2 = [&](int code) {
            (void)hipStreamSynchronize(s);
            (void)hipFree(d_assign);
            (void)hipFree(d_cnt);
            destroy(ix);
            return code;
        };
        // assignment: a top-1 coarse search per chunk (Section 3.1 rule = rank-1 probe)
        pk_index *hs[1] = {ix};
        for (int64_t i0 = 0; i0 < n && rc == PK_OK; i0 += kBuildChunk) {
            const int64_t mc = std::min<int64_t>(kBuildChunk, n - i0);
            const uint32_t qlo[2] = {0, (uint32_t)mc};
            Plan p;
            rc = make_plan(p, hs, 1, qlo, mc, 1, 1, true, false);
            if (rc == PK_OK) rc = ensure_ws(ix, p.bytes, s);
            if (rc != PK_OK) break;
            carve(p, ix->ws, ix);
            MultiArgs mm;
            fill_multi(mm, hs, 1, qlo);
            rc = run_coarse(p, mm, hs, vectors + (size_t)i0 * cfg->d, s);
            if (rc == PK_OK && launch_copy_i32(p.probes, d_assign + i0, mc, s) != hipSuccess) rc = PK_ERR_HIP;
        }
        if (rc != PK_OK) return fail2(rc);
        if (launch_fill_u32(d_cnt, 0u, (size_t)cfg->nlist * 2, s) != hipSuccess ||
            launch_hist(d_assign, n, d_cnt, s) != hipSuccess ||
            hipMemcpyAsync(cnt.data(), d_cnt, (size_t)cfg->nlist * sizeof(uint32_t), hipMemcpyDeviceToHost, s) !=
                hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess)
            return fail2(PK_ERR_HIP);
        std::vector<uint32_t> mbase((size_t)cfg->nlist), mpages((size_t)cfg->nlist);
        uint64_t used = 0;
        for (int l = 0; l < cfg->nlist; ++l) {
            mbase[l] = (uint32_t)used;
            mpages[l] = (cnt[l] + x.P - 1) / x.P;
            used += mpages[l];
        }
        if (used > ix->pages_total) return fail2(PK_ERR_NOMEM);
        const uint32_t used32 = (uint32_t)used;
        if (hipMemcpyAsync(D.main_base, mbase.data(), mbase.size() * 4, hipMemcpyHostToDevice, s) != hipSuccess ||
            hipMemcpyAsync(D.main_pages, mpages.data(), mpages.size() * 4, hipMemcpyHostToDevice, s) != hipSuccess ||
            hipMemcpyAsync(D.list_len, cnt.data(), cnt.size() * 4, hipMemcpyHostToDevice, s) != hipSuccess ||
            hipMemcpyAsync(D.ctr, &used32, 4, hipMemcpyHostToDevice, s) != hipSuccess ||
            launch_scatter_build(ix->dev, vectors, ids, d_assign, n, 0, d_cnt + cfg->nlist, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess)
            return fail2(PK_ERR_HIP);
        (void)hipFree(d_assign);
        (void)hipFree(d_cnt);
        ix->pages_known = used32;
    }
    if (hipStreamSynchronize(s) != hipSuccess) return fail(PK_ERR_HIP);
    // the build's own scratch (score matrices of 16 384-vector chunks) is not what searches need
    if (ix->ws) (void)hipFree(ix->ws);
    ix->ws = nullptr;
    ix->ws_bytes = 0;
    ix->ws_grows = 0;
    ix->n_total = n;
    ix->next_id = n;
    ix->n_inserted = 0;
    ix->inserted_at_known = 0;
    ix->inserted_at_top = 0;
    std::vector<uint32_t> sorted(cnt);
    std::sort(sorted.begin(), sorted.end(), [](uint32_t a, uint32_t b) { return a > b; });
    for (int j = 0; j < cfg->nlist; ++j) ix->top_len[j + 1] = ix->top_len[j] + sorted[j];
    *out = ix;
    return PK_OK;
}

int pk_index_add_arena(pk_index *ix, void *arena, size_t arena_bytes, void *stream)
{
    if (!live(ix)) return PK_ERR_BAD_HANDLE;
    if (!arena || reinterpret_cast<uintptr_t>(arena) % 256 != 0) return PK_ERR_INVALID_ARG;
    if (ix->host.n_arenas >= PK_MAX_ARENAS) return PK_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Dims x = dims_of(&ix->cfg);
    const uint32_t np = pages_in(arena_bytes, x);
    if (np == 0 || (uint64_t)ix->pages_total + np > 0x7fffffffu) return PK_ERR_INVALID_ARG;
    DevIndex &D = ix->host;
    place_arena(D.arenas[D.n_arenas], static_cast<char *>(arena), ix->pages_total, np, x);
    D.n_arenas += 1;
    ix->pages_total += np;
    ix->arena_bytes += arena_bytes;
    PK_HIP(hipMemcpyAsync(ix->dev, &D, sizeof(D), hipMemcpyHostToDevice, s));
    PK_HIP(launch_fill_u32(D.ctr + 2, ix->pages_total, 1, s));
    return PK_OK;
}

int pk_delete(pk_index *ix, const int64_t *ids, int64_t m, int64_t *n_removed, void *stream)
{
    if (!live(ix)) return PK_ERR_BAD_HANDLE;
    if (m < 0 || (m > 0 && !ids)) return PK_ERR_INVALID_ARG;
    if (n_removed) *n_removed = 0;
    if (m == 0) return PK_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Carver c{nullptr, 0};
    DeleteArgs da{};
    auto lay = [&](Carver &cv) {
        da.sorted = cv.take<int64_t>(kDeleteChunk);
        da.unit_start = cv.take<uint32_t>((size_t)ix->cfg.nlist + 1);
        da.hits = cv.take<unsigned long long>(kDeleteChunk);
        da.hit_len0 = cv.take<uint32_t>(kDeleteChunk);
        da.hit_seg0 = cv.take<uint32_t>(kDeleteChunk);
        da.hit_cnt = cv.take<uint32_t>(kDeleteChunk);
        da.scal = cv.take<uint32_t>(4);
        da.removed = cv.take<unsigned long long>(1);
    };
    lay(c);
    PK_TRY(ensure_ws(ix, c.off + 256, s));
    c = Carver{ix->ws, 0};
    lay(c);
    da.ix = ix->dev;
    da.nlist = ix->cfg.nlist;
    da.grid = ix->num_cu * 8;
    PK_HIP(launch_fill_u32(da.scal, 0u, 4, s));
    PK_HIP(launch_fill_u32(reinterpret_cast<uint32_t *>(da.removed), 0u, 2, s));
    unsigned long long removed = 0;
    for (int pass = 0; pass < 1 << 20; ++pass) {
        for (int64_t i0 = 0; i0 < m; i0 += kDeleteChunk) {
            da.ids = ids + i0;
            da.m = (int)std::min<int64_t>(kDeleteChunk, m - i0);
            PK_HIP(launch_delete(da, s));
        }
        // more rows carried the ids than one pass takes (several rows under one id): go again
        uint32_t again = 0;
        PK_HIP(hipMemcpyAsync(&removed, da.removed, sizeof(removed), hipMemcpyDeviceToHost, s));
        PK_HIP(hipMemcpyAsync(&again, da.scal + 2, sizeof(again), hipMemcpyDeviceToHost, s));
        PK_HIP(hipStreamSynchronize(s));
        if (!again) break;
        PK_HIP(launch_fill_u32(da.scal + 2, 0u, 1, s));
    }
    ix->n_total -= (int64_t)removed;
    if (n_removed) *n_removed = (int64_t)removed;
    return PK_OK;
}

int pk_kmeans(const float *vectors, int64_t n, int32_t d, int32_t nlist, int32_t iters, float *centroids,
              int32_t *assign_out, double *inertia_out, void *stream)
{
    if (!vectors || !centroids || n < 1 || nlist < 1 || iters < 1) return PK_ERR_INVALID_ARG;
    if (d < 1) return PK_ERR_INVALID_ARG;
    if (d > PK_MAX_DIM || n > 0x7fffffffll) return PK_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // the assignment step is a top-1 coarse search under L2: an index without vectors carries the centroid table
    pk_config cfg{d, nlist, PK_METRIC_L2, PK_F32, 32, 1};
    const size_t abytes = pk_arena_bytes(&cfg, 0, 0);
    char *kbuf = nullptr;
    const size_t nl4 = round_up((size_t)nlist * 4, 256), n4 = round_up((size_t)n * 4, 256);
    const size_t sums8 = round_up((size_t)nlist * d * 8, 256), sq8 = round_up((size_t)nlist * 8, 256);
    const size_t sbytes = round_up(abytes, 256) + 3 * nl4 + 2 * n4 + round_up((size_t)iters * 8, 256) + sums8 + sq8;
    if (hipMalloc(reinterpret_cast<void **>(&kbuf), sbytes) != hipSuccess) {
        (void)hipGetLastError();
        return PK_ERR_NOMEM;
    }
    pk_index *ix = nullptr;
    int rc = pk_index_build(&cfg, centroids, nullptr, nullptr, 0, kbuf, abytes, stream, &ix);
    if (rc != PK_OK) {
        (void)hipFree(kbuf);
        return rc;
    }
    KmeansArgs ka{};
    char *p = kbuf + round_up(abytes, 256);
    ka.cnt = reinterpret_cast<uint32_t *>(p);
    ka.start = reinterpret_cast<uint32_t *>(p + nl4);
    ka.fill = reinterpret_cast<uint32_t *>(p + 2 * nl4);
    ka.members = reinterpret_cast<uint32_t *>(p + 3 * nl4);
    int32_t *assign = reinterpret_cast<int32_t *>(p + 3 * nl4 + n4);
    double *inertia = reinterpret_cast<double *>(p + 3 * nl4 + 2 * n4);
    ka.sums = reinterpret_cast<double *>(p + 3 * nl4 + 2 * n4 + round_up((size_t)iters * 8, 256));
    ka.sq = reinterpret_cast<double *>(p + 3 * nl4 + 2 * n4 + round_up((size_t)iters * 8, 256) + sums8);
    ka.x = vectors;
    ka.assign = assign;
    ka.n = n;
    ka.d = d;
    ka.nlist = nlist;
    ka.centroids = centroids;
    pk_index *hs[1] = {ix};
    auto run = [&]() -> int {
        for (int it = 0; it < iters; ++it) {
            if (it > 0)
                PK_HIP(launch_store_centroids(centroids, nlist, d, ix->dpad32, ix->nlist_pad, PK_METRIC_L2,
                                              const_cast<float *>(ix->host.cent), const_cast<float *>(ix->host.cnorm), s));
            for (int64_t i0 = 0; i0 < n; i0 += kBuildChunk) {
                const int64_t mc = std::min<int64_t>(kBuildChunk, n - i0);
                const uint32_t qlo[2] = {0, (uint32_t)mc};
                Plan pl;
                PK_TRY(make_plan(pl, hs, 1, qlo, mc, 1, 1, true, false));
                PK_TRY(ensure_ws(ix, pl.bytes, s));
                carve(pl, ix->ws, ix);
                MultiArgs mm;
                fill_multi(mm, hs, 1, qlo);
                PK_TRY(run_coarse(pl, mm, hs, vectors + (size_t)i0 * d, s));
                PK_HIP(launch_copy_i32(pl.probes, assign + i0, mc, s));
            }
            ka.inertia = inertia + it;
            PK_HIP(launch_kmeans_update(ka, s));
        }
        if (assign_out) PK_HIP(hipMemcpyAsync(assign_out, assign, (size_t)n * 4, hipMemcpyDeviceToDevice, s));
        if (inertia_out)
            PK_HIP(hipMemcpyAsync(inertia_out, inertia, (size_t)iters * 8, hipMemcpyDeviceToHost, s));
        PK_HIP(hipStreamSynchronize(s));
        return PK_OK;
    };
    rc = run();
    if (rc != PK_OK) (void)hipStreamSynchronize(s);
    destroy(ix);
    (void)hipFree(kbuf);
    return rc;
}

namespace {

// one list that is being split: its 2-means result
struct SplitJob {
    int list;              // the list (keeps side 0); the new list is nlist_old + (position of the job)
    uint32_t len, len_new; // members before the split, members that move to the new list
    int32_t *side;         // DEVICE [len] 0 / 1
};

// Moves the index into `arena`, every list in one contiguous extent.  threshold > 0: lists
// longer than that are split by a 2-means over their members first (the new lists are
// appended after the last one).
int relayout(pk_index *ix, void *arena, size_t arena_bytes, int64_t threshold, int iters, int32_t *n_split_out,
             hipStream_t s)
{
    if (!live(ix)) return PK_ERR_BAD_HANDLE;
    if (!arena || reinterpret_cast<uintptr_t>(arena) % 256 != 0) return PK_ERR_INVALID_ARG;
    if (n_split_out) *n_split_out = 0;
    const pk_config old_cfg = ix->cfg;
    const int d = old_cfg.d, nlist0 = old_cfg.nlist;
    for (int a = 0; a < ix->host.n_arenas; ++a)
        if (ix->host.arenas[a].vec >= static_cast<char *>(arena) &&
            ix->host.arenas[a].vec < static_cast<char *>(arena) + arena_bytes)
            return PK_ERR_INVALID_ARG; // the new arena overlaps a current one
    // exact list lengths decide the new extents
    PK_HIP(hipStreamSynchronize(s));
    PK_TRY(settle_pages(ix));
    std::vector<uint32_t> len((size_t)nlist0);
    PK_HIP(hipMemcpy(len.data(), ix->host.list_len, len.size() * 4, hipMemcpyDeviceToHost));

    // ---- 2-means of the lists to split (Section 4.4: a light k-means on the device)
    std::vector<SplitJob> jobs;
    std::vector<void *> owned; // device scratch freed on every way out
    auto release = [&]() {
        for (void *p : owned) (void)hipFree(p);
        owned.clear();
    };
    auto fail = [&](int code) {
        (void)hipStreamSynchronize(s);
        release();
        return code;
    };
    SplitArgs sp{};
    uint32_t *slots_all = nullptr;       // DEVICE scratch of the scatter, one part per job
    std::vector<uint32_t> job_row0;      // members of the jobs before each one
    if (threshold > 0) {
        std::vector<uint32_t> jl, jn, ju;
        uint64_t rows = 0, units = 0;
        for (int l = 0; l < nlist0; ++l) {
            if ((int64_t)len[l] <= threshold) continue;
            if (nlist0 + (int)jobs.size() + 1 > 0x3fffffff) return fail(PK_ERR_UNSUPPORTED);
            SplitJob j{};
            j.list = l;
            j.len = len[l];
            jobs.push_back(j);
            jl.push_back((uint32_t)l);
            jn.push_back(len[l]);
            ju.push_back((uint32_t)units);
            job_row0.push_back((uint32_t)rows);
            rows += len[l];
            units += (len[l] + kSplitUnit - 1) / kSplitUnit;
        }
        const size_t nj = jobs.size();
        if (nj > 0) {
            if (rows > 0xfffffff0ull || units > 0x7fffffffull) return fail(PK_ERR_UNSUPPORTED);
            ju.push_back((uint32_t)units);
            // one block of scratch for every job: tables, centroids, sums, counts, sides, scatter slots
            Carver cv{nullptr, 0};
            auto lay = [&](Carver &c) {
                sp.job_list = c.take<uint32_t>(nj);
                sp.job_len = c.take<uint32_t>(nj);
                sp.job_unit0 = c.take<uint32_t>(nj + 1);
                sp.job_row0 = c.take<uint32_t>(nj);
                sp.cent = c.take<double>(nj * 2 * d);
                sp.sum = c.take<double>(nj * 2 * d);
                sp.cnt = c.take<unsigned long long>(nj * 2);
                sp.cnt_out = c.take<unsigned long long>(nj * 2);
                sp.side = c.take<int32_t>(rows);
                slots_all = c.take<uint32_t>(rows);
            };
            lay(cv);
            char *block = nullptr;
            if (hipMalloc(reinterpret_cast<void **>(&block), cv.off + 256) != hipSuccess) return fail(PK_ERR_NOMEM);
            owned.push_back(block);
            cv = Carver{block, 0};
            lay(cv);
            sp.ix = ix->dev;
            sp.njobs = (int)nj;
            auto up = [&](const uint32_t *dst, const std::vector<uint32_t> &v) {
                return hipMemcpyAsync(const_cast<uint32_t *>(dst), v.data(), v.size() * 4, hipMemcpyHostToDevice, s);
            };
            if (up(sp.job_list, jl) != hipSuccess || up(sp.job_len, jn) != hipSuccess || up(sp.job_unit0, ju) != hipSuccess ||
                up(sp.job_row0, job_row0) != hipSuccess)
                return fail(PK_ERR_HIP);
            if (launch_split_init(sp, s) != hipSuccess) return fail(PK_ERR_HIP);
            for (int it = 0; it < iters; ++it)
                if (launch_split_iterate(sp, (uint32_t)units, d, s) != hipSuccess) return fail(PK_ERR_HIP);
            std::vector<unsigned long long> cnt(nj * 2);
            if (hipMemcpyAsync(cnt.data(), sp.cnt_out, cnt.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost, s) !=
                    hipSuccess ||
                hipStreamSynchronize(s) != hipSuccess) // also keeps the uploaded tables alive until they are read
                return fail(PK_ERR_HIP);
            for (size_t t = 0; t < nj; ++t) {
                jobs[t].len_new = (uint32_t)cnt[2 * t + 1];
                jobs[t].side = sp.side + job_row0[t];
            }
        }
    }
    const int ns = (int)jobs.size(), nlist1 = nlist0 + ns;

    // ---- new layout
    pk_config cfg = old_cfg;
    cfg.nlist = nlist1;
    const Dims x = dims_of(&cfg);
    if (arena_bytes < x.header + 1024 + x.page_stride) return fail(PK_ERR_NOMEM);
    std::vector<uint32_t> nlen((size_t)nlist1), mbase((size_t)nlist1), mpages((size_t)nlist1);
    std::vector<uint8_t> skip((size_t)nlist1, 0);
    for (int l = 0; l < nlist0; ++l) nlen[l] = len[l];
    for (int t = 0; t < ns; ++t) {
        nlen[jobs[t].list] = jobs[t].len - jobs[t].len_new;
        nlen[nlist0 + t] = jobs[t].len_new;
        skip[jobs[t].list] = skip[nlist0 + t] = 1;
    }
    uint64_t used = 0;
    for (int l = 0; l < nlist1; ++l) {
        mbase[l] = (uint32_t)used;
        mpages[l] = (nlen[l] + x.P - 1) / x.P;
        used += mpages[l];
    }
    DevIndex N;
    DevIndex *ndev = nullptr;
    uint32_t npages = 0;
    float *cent = nullptr, *cnorm = nullptr;
    place_header(N, &ndev, &npages, &cent, &cnorm, &cfg, static_cast<char *>(arena), arena_bytes, x);
    if (used > npages) return fail(PK_ERR_NOMEM);
    const DevIndex &O = ix->host;
    const uint32_t head[3] = {(uint32_t)used, 0u, npages};
    auto enqueue = [&]() -> int {
        PK_HIP(hipMemcpyAsync(ndev, &N, sizeof(N), hipMemcpyHostToDevice, s));
        if (ns == 0) {
            PK_HIP(hipMemcpyAsync(cent, O.cent, (size_t)x.nlist_pad * x.dpad32 * sizeof(float), hipMemcpyDeviceToDevice, s));
            PK_HIP(hipMemcpyAsync(cnorm, O.cnorm, (size_t)x.nlist_pad * sizeof(float), hipMemcpyDeviceToDevice, s));
        } else {
            // dense copy of the centroids, the split lists' rows replaced, the new lists' rows appended,
            // then laid out again (padding, squared norms)
            float *dense = nullptr;
            if (hipMalloc(reinterpret_cast<void **>(&dense), (size_t)nlist1 * d * sizeof(float)) != hipSuccess) {
                (void)hipGetLastError();
                return PK_ERR_NOMEM;
            }
            owned.push_back(dense);
            PK_HIP(hipMemcpy2DAsync(dense, (size_t)d * sizeof(float), O.cent, (size_t)ix->dpad32 * sizeof(float),
                                    (size_t)d * sizeof(float), (size_t)nlist0, hipMemcpyDeviceToDevice, s));
            PK_HIP(launch_split_centroids(sp, nlist0, dense, s));
            PK_HIP(launch_store_centroids(dense, nlist1, d, x.dpad32, x.nlist_pad, cfg.metric, cent, cnorm, s));
        }
        PK_HIP(hipMemcpyAsync(N.list_len, nlen.data(), nlen.size() * 4, hipMemcpyHostToDevice, s));
        PK_HIP(hipMemcpyAsync(N.main_base, mbase.data(), mbase.size() * 4, hipMemcpyHostToDevice, s));
        PK_HIP(hipMemcpyAsync(N.main_pages, mpages.data(), mpages.size() * 4, hipMemcpyHostToDevice, s));
        PK_HIP(launch_fill_u32(N.dtab, 0xffffffffu, (size_t)nlist1 * x.max_dp, s));
        PK_HIP(hipMemcpyAsync(N.ctr, O.ctr, 16 * sizeof(uint32_t), hipMemcpyDeviceToDevice, s)); // keeps the sticky error flags
        PK_HIP(hipMemcpyAsync(N.ctr, head, 4, hipMemcpyHostToDevice, s));
        PK_HIP(hipMemcpyAsync(N.ctr + 2, head + 2, 4, hipMemcpyHostToDevice, s));
        PK_HIP(hipMemcpyAsync(N.stats, O.stats, 8 * sizeof(unsigned long long), hipMemcpyDeviceToDevice, s));
        uint8_t *dskip = nullptr;
        if (ns > 0) {
            if (hipMalloc(reinterpret_cast<void **>(&dskip), skip.size()) != hipSuccess) {
                (void)hipGetLastError();
                return PK_ERR_NOMEM;
            }
            owned.push_back(dskip);
            PK_HIP(hipMemcpyAsync(dskip, skip.data(), skip.size(), hipMemcpyHostToDevice, s));
        }
        PK_HIP(launch_compact_pages(ix->dev, ndev, (uint32_t)used, dskip, s));
        for (int t = 0; t < ns; ++t)
            PK_HIP(launch_split_list(ix->dev, ndev, (uint32_t)jobs[t].list, (uint32_t)(nlist0 + t), jobs[t].side,
                                     slots_all + job_row0[(size_t)t], jobs[t].len, s));
        PK_HIP(hipStreamSynchronize(s)); // the old arenas are out of use from here on
        return PK_OK;
    };
    const int rc = enqueue();
    if (rc != PK_OK) return fail(rc);
    release();
    ix->cfg = cfg;
    ix->nlist_pad = x.nlist_pad;
    ix->host = N;
    ix->dev = ndev;
    ix->pages_total = npages;
    ix->arena_bytes = arena_bytes;
    ix->pages_known = (uint32_t)used;
    ix->inserted_at_known = ix->n_inserted;
    ix->inserted_at_top = ix->n_inserted;
    std::sort(nlen.begin(), nlen.end(), [](uint32_t a, uint32_t b) { return a > b; });
    ix->top_len.assign((size_t)nlist1 + 1, 0);
    for (int j = 0; j < nlist1; ++j) ix->top_len[j + 1] = ix->top_len[j] + nlen[j];
    if (n_split_out) *n_split_out = ns;
    return PK_OK;
}

} // namespace

int pk_index_compact(pk_index *ix, void *arena, size_t arena_bytes, void *stream)
{
    return relayout(ix, arena, arena_bytes, 0, 0, nullptr, static_cast<hipStream_t>(stream));
}

int pk_index_split(pk_index *ix, void *arena, size_t arena_bytes, int64_t threshold, int32_t iters, int32_t *n_split,
                   void *stream)
{
    if (threshold < 1 || iters < 1) return live(ix) ? PK_ERR_INVALID_ARG : PK_ERR_BAD_HANDLE;
    return relayout(ix, arena, arena_bytes, threshold, iters, n_split, static_cast<hipStream_t>(stream));
}

int pk_index_centroids(pk_index *ix, float *out, void *stream)
{
    if (!live(ix)) return PK_ERR_BAD_HANDLE;
    if (!out) return PK_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    PK_HIP(hipMemcpy2DAsync(out, (size_t)ix->cfg.d * sizeof(float), ix->host.cent, (size_t)ix->dpad32 * sizeof(float),
                            (size_t)ix->cfg.d * sizeof(float), (size_t)ix->cfg.nlist, hipMemcpyDeviceToDevice, s));
    return PK_OK;
}

int pk_list_ids(pk_index *ix, int32_t list, int64_t *out, int64_t cap, void *stream)
{
    if (!live(ix)) return PK_ERR_BAD_HANDLE;
    if (list < 0 || list >= ix->cfg.nlist || cap < 0 || (cap > 0 && !out)) return PK_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t most = std::min<int64_t>(cap, std::max<int64_t>(ix->n_total, 0)); // no list is longer than the index
    PK_HIP(launch_gather_list(ix->dev, (uint32_t)list, (uint32_t)std::min<int64_t>(most, 0x7fffffff), nullptr, out, s));
    return PK_OK;
}

int pk_insert(pk_index *ix, const float *vectors, const int64_t *ids, int64_t m, int32_t *assigned_lists, void *stream)
{
    return insert_impl(ix, vectors, ids, m, nullptr, assigned_lists, static_cast<hipStream_t>(stream));
}

int pk_insert_multi(pk_index *const *handles, int32_t n_handles, const int64_t *v_offsets, const float *vectors,
                    const int64_t *ids, int32_t *assigned_lists, void *stream)
{
    if (!handles || !v_offsets || n_handles < 1 || n_handles > PK_MAX_HANDLES) return PK_ERR_INVALID_ARG;
    if (v_offsets[0] != 0) return PK_ERR_INVALID_ARG;
    bool small = true;
    for (int a = 0; a < n_handles; ++a) {
        if (!live(handles[a])) return PK_ERR_BAD_HANDLE;
        if (v_offsets[a + 1] < v_offsets[a]) return PK_ERR_INVALID_ARG;
        for (int b = 0; b < a; ++b)
            if (handles[b] == handles[a]) return PK_ERR_INVALID_ARG;
        const pk_config &c0 = handles[0]->cfg, &c = handles[a]->cfg;
        if (c.d != c0.d || c.metric != c0.metric || c.storage != c0.storage || c.page_vecs != c0.page_vecs)
            return PK_ERR_DIM_MISMATCH;
        small = small && v_offsets[a + 1] - v_offsets[a] <= 1024;
    }
    const int64_t m = v_offsets[n_handles];
    if (m > 0 && !vectors) return PK_ERR_INVALID_ARG;
    if (m == 0) return PK_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int d = handles[0]->cfg.d;
    // all capacity checks first: nothing is enqueued if any handle cannot take its share
    for (int a = 0; a < n_handles; ++a) PK_TRY(check_capacity(handles[a], v_offsets[a + 1] - v_offsets[a], s));
    if (small && m <= 0x7fffffff) {
        std::vector<uint32_t> qlo((size_t)n_handles + 1);
        for (int a = 0; a <= n_handles; ++a) qlo[(size_t)a] = (uint32_t)v_offsets[a];
        return insert_batch(handles, n_handles, qlo.data(), vectors, ids, nullptr, assigned_lists, s);
    }
    for (int a = 0; a < n_handles; ++a) { // long segments: handle by handle
        const int64_t lo = v_offsets[a], ma = v_offsets[a + 1] - lo;
        PK_TRY(insert_impl(handles[a], vectors + (size_t)lo * d, ids ? ids + lo : nullptr, ma, nullptr,
                           assigned_lists ? assigned_lists + lo : nullptr, s));
    }
    return PK_OK;
}

int pk_insert_assigned(pk_index *ix, const float *vectors, const int64_t *ids, int64_t m, const int32_t *lists,
                       void *stream)
{
    if (m > 0 && !lists) return PK_ERR_INVALID_ARG;
    return insert_impl(ix, vectors, ids, m, lists, nullptr, static_cast<hipStream_t>(stream));
}

int pk_search(pk_index *ix, const float *queries, int64_t nq, int32_t k, int32_t nprobe, int64_t *out_ids,
              float *out_dist, void *stream)
{
    PK_TRY(check_search_args(ix, queries, nq, k, nprobe));
    if (nq > 0 && (!out_ids || !out_dist)) return PK_ERR_INVALID_ARG;
    if (nq == 0) return PK_OK;
    pk_index *hs[1] = {ix};
    const int64_t offs[2] = {0, nq};
    return search_impl(hs, 1, offs, queries, k, nprobe, kFull, nullptr, nullptr, out_ids, out_dist,
                       static_cast<hipStream_t>(stream));
}

int pk_search_noalloc(pk_index *ix, const float *queries, int64_t nq, int32_t k, int32_t nprobe, int64_t *out_ids,
                      float *out_dist, void *stream)
{
    PK_TRY(check_search_args(ix, queries, nq, k, nprobe));
    if (nq > 0 && (!out_ids || !out_dist)) return PK_ERR_INVALID_ARG;
    if (nq == 0) return PK_OK;
    char *ws = nullptr;
    PK_TRY(scratch_on_device(&ws));
    pk_index *hs[1] = {ix};
    const int64_t offs[2] = {0, nq};
    return search_impl(hs, 1, offs, queries, k, nprobe, kFull, nullptr, nullptr, out_ids, out_dist,
                       static_cast<hipStream_t>(stream), ws, kScratchBytes);
}

size_t pk_search_noalloc_bytes(pk_index *ix, int64_t nq, int32_t k, int32_t nprobe)
{
    if (!live(ix) || nq < 1 || k < 1 || k > PK_MAX_K || nprobe < 1 || nprobe > ix->cfg.nlist || nprobe > PK_MAX_NPROBE ||
        nq > 0x7fffffff)
        return 0;
    pk_index *hs[1] = {ix};
    const uint32_t qlo[2] = {0, (uint32_t)nq};
    Plan p;
    if (make_plan(p, hs, 1, qlo, nq, k, nprobe, true, true) != PK_OK) return 0;
    return p.bytes;
}

int pk_workspace_reserve(pk_index *const *handles, int32_t n_handles, int64_t nq_max, int32_t k_max, int32_t nprobe_max,
                         int64_t inserts_ahead, void *stream)
{
    if (!handles || n_handles < 1 || n_handles > PK_MAX_HANDLES) return PK_ERR_INVALID_ARG;
    for (int a = 0; a < n_handles; ++a) {
        if (!live(handles[a])) return PK_ERR_BAD_HANDLE;
        const pk_config &c0 = handles[0]->cfg, &c = handles[a]->cfg;
        if (c.d != c0.d || c.metric != c0.metric || c.storage != c0.storage || c.page_vecs != c0.page_vecs)
            return PK_ERR_DIM_MISMATCH;
    }
    if (nq_max < 1 || nq_max > 32768 || k_max < 1 || k_max > PK_MAX_K || nprobe_max < 1 || nprobe_max > PK_MAX_NPROBE ||
        inserts_ahead < 0)
        return PK_ERR_INVALID_ARG;
    // sized as if every handle received all nq_max queries: every size is monotone in a handle's
    // share of the batch, so this covers any split
    std::vector<uint32_t> qlo((size_t)n_handles + 1);
    for (int b = 0; b <= n_handles; ++b) qlo[(size_t)b] = (uint32_t)((nq_max * b) / n_handles);
    int np = nprobe_max;
    for (int a = 0; a < n_handles; ++a) np = std::min(np, handles[a]->cfg.nlist);
    Plan p;
    PK_TRY(make_plan(p, handles, n_handles, qlo.data(), nq_max, k_max, np, true, true, inserts_ahead, true));
    size_t need = p.bytes;
    need += round_up((size_t)nq_max * 4, 256) + 256; // slot array of an insert batch
    return ensure_ws(handles[0], need, static_cast<hipStream_t>(stream));
}

int pk_index_set_emit_cap(pk_index *ix, int32_t entries)
{
    if (!live(ix)) return PK_ERR_BAD_HANDLE;
    if (entries < 0 || entries > (1 << 20)) return PK_ERR_INVALID_ARG;
    ix->emit_cap = entries;
    return PK_OK;
}

int pk_search_multi(pk_index *const *handles, int32_t n_handles, const int64_t *q_offsets, const float *queries,
                    int32_t k, int32_t nprobe, int64_t *out_ids, float *out_dist, void *stream)
{
    if (!handles || !q_offsets || n_handles < 1 || n_handles > PK_MAX_HANDLES) return PK_ERR_INVALID_ARG;
    if (q_offsets[0] != 0) return PK_ERR_INVALID_ARG;
    for (int a = 0; a < n_handles; ++a) {
        if (!live(handles[a])) return PK_ERR_BAD_HANDLE;
        if (q_offsets[a + 1] < q_offsets[a]) return PK_ERR_INVALID_ARG;
        for (int b = 0; b < a; ++b)
            if (handles[b] == handles[a]) return PK_ERR_INVALID_ARG;
        const pk_config &c0 = handles[0]->cfg, &c = handles[a]->cfg;
        if (c.d != c0.d || c.metric != c0.metric || c.storage != c0.storage || c.page_vecs != c0.page_vecs)
            return PK_ERR_DIM_MISMATCH;
        PK_TRY(check_search_args(handles[a], queries, q_offsets[n_handles], k, nprobe));
    }
    const int64_t nq = q_offsets[n_handles];
    if (nq > 0 && (!out_ids || !out_dist || !queries)) return PK_ERR_INVALID_ARG;
    if (nq == 0) return PK_OK;
    return search_impl(handles, n_handles, q_offsets, queries, k, nprobe, kFull, nullptr, nullptr, out_ids, out_dist,
                       static_cast<hipStream_t>(stream));
}

static_assert(PK_MAX_K <= 1024 && PK_MAX_HANDLES <= 128, "union_merge_kernel packs rank and handle into 17 bits");

// grow-only staging buffer of the calls that run several searches (scope union, level cascade)
static int ensure_ubuf(pk_index *own, size_t need, hipStream_t s)
{
    if (need <= own->ubuf_bytes) return PK_OK;
    PK_HIP(hipStreamSynchronize(s)); // earlier work on this stream may still use the old buffer
    if (own->ubuf) PK_HIP(hipFree(own->ubuf));
    own->ubuf = nullptr;
    own->ubuf_bytes = 0;
    void *p = nullptr;
    if (hipMalloc(&p, need) != hipSuccess) {
        (void)hipGetLastError();
        return PK_ERR_NOMEM;
    }
    own->ubuf = static_cast<char *>(p);
    own->ubuf_bytes = need;
    return PK_OK;
}

int pk_search_union(pk_index *const *handles, int32_t n_handles, const float *queries, int64_t nq, int32_t k,
                    int32_t nprobe, int32_t *out_src, int64_t *out_ids, float *out_dist, void *stream)
{
    if (!handles || n_handles < 1 || n_handles > PK_MAX_HANDLES) return PK_ERR_INVALID_ARG;
    for (int a = 0; a < n_handles; ++a) {
        if (!live(handles[a])) return PK_ERR_BAD_HANDLE;
        for (int b = 0; b < a; ++b)
            if (handles[b] == handles[a]) return PK_ERR_INVALID_ARG;
        const pk_config &c0 = handles[0]->cfg, &c = handles[a]->cfg;
        if (c.d != c0.d || c.metric != c0.metric || c.storage != c0.storage || c.page_vecs != c0.page_vecs)
            return PK_ERR_DIM_MISMATCH;
        PK_TRY(check_search_args(handles[a], queries, nq, k, nprobe));
    }
    if (nq > 0 && (!out_src || !out_ids || !out_dist)) return PK_ERR_INVALID_ARG;
    if (nq == 0) return PK_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    pk_index *own = handles[0];
    const int d = own->cfg.d;
    const int64_t H = n_handles;
    // every query is searched in every handle: the segmented launch over H copies of the batch
    const int64_t chunk = std::max<int64_t>(1, std::min<int64_t>(nq, 32768 / H));
    const size_t qb = round_up((size_t)H * chunk * d * sizeof(float), 256);
    const size_t ib = round_up((size_t)H * chunk * k * sizeof(int64_t), 256);
    const size_t need = qb + ib + round_up((size_t)H * chunk * k * sizeof(float), 256);
    PK_TRY(ensure_ubuf(own, need, s));
    float *uq = reinterpret_cast<float *>(own->ubuf);
    int64_t *uids = reinterpret_cast<int64_t *>(own->ubuf + qb);
    float *udist = reinterpret_cast<float *>(own->ubuf + qb + ib);
    std::vector<int64_t> offs((size_t)H + 1);
    for (int64_t q0 = 0; q0 < nq; q0 += chunk) {
        const int64_t nc = std::min(chunk, nq - q0);
        for (int64_t h = 0; h <= H; ++h) offs[(size_t)h] = h * nc;
        for (int64_t h = 0; h < H; ++h)
            PK_HIP(hipMemcpyAsync(uq + (size_t)h * nc * d, queries + (size_t)q0 * d, (size_t)nc * d * sizeof(float),
                                  hipMemcpyDeviceToDevice, s));
        PK_TRY(search_impl(handles, n_handles, offs.data(), uq, k, nprobe, kFull, nullptr, nullptr, uids, udist, s));
        UnionArgs u{};
        u.ids = uids;
        u.dist = udist;
        u.n_handles = n_handles;
        u.k = k;
        u.metric = own->cfg.metric;
        u.nq = nc;
        u.out_src = out_src + (size_t)q0 * k;
        u.out_ids = out_ids + (size_t)q0 * k;
        u.out_dist = out_dist + (size_t)q0 * k;
        PK_HIP(launch_union_merge(u, s));
    }
    return PK_OK;
}

int pk_search_levels(pk_index *const *levels, int32_t n_levels, const int32_t *nprobes, const float *queries,
                     int64_t nq, int32_t k, const float *stop, int32_t *out_level, int64_t *out_ids,
                     float *out_dist, void *stream)
{
    if (!levels || !nprobes || n_levels < 1 || n_levels > PK_MAX_HANDLES) return PK_ERR_INVALID_ARG;
    int np_max = 1;
    for (int l = 0; l < n_levels; ++l) {
        if (!live(levels[l])) return PK_ERR_BAD_HANDLE;
        for (int b = 0; b < l; ++b)
            if (levels[b] == levels[l]) return PK_ERR_INVALID_ARG;
        const pk_config &c0 = levels[0]->cfg, &c = levels[l]->cfg;
        if (c.d != c0.d || c.metric != c0.metric) return PK_ERR_DIM_MISMATCH;
        PK_TRY(check_search_args(levels[l], queries, nq, k, nprobes[l]));
        np_max = std::max(np_max, (int)nprobes[l]);
    }
    if (nq > 0 && (!stop || !out_ids || !out_dist)) return PK_ERR_INVALID_ARG;
    if (nq == 0) return PK_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    pk_index *own = levels[0];
    // staging: open flags, the probes of a lower level, its rows
    const size_t ob = round_up((size_t)nq * sizeof(uint32_t), 256);
    const size_t pb = round_up((size_t)nq * np_max * sizeof(int32_t), 256);
    const size_t ib = round_up((size_t)nq * k * sizeof(int64_t), 256);
    const size_t db = round_up((size_t)nq * k * sizeof(float), 256);
    if (n_levels > 1) PK_TRY(ensure_ubuf(own, ob + pb + ib + db, s));
    else PK_TRY(ensure_ubuf(own, ob, s));
    uint32_t *open = reinterpret_cast<uint32_t *>(own->ubuf);
    int32_t *probes = reinterpret_cast<int32_t *>(own->ubuf + ob);
    int64_t *row_ids = reinterpret_cast<int64_t *>(own->ubuf + ob + pb);
    float *row_dist = reinterpret_cast<float *>(own->ubuf + ob + pb + ib);
    const int64_t offs[2] = {0, nq};
    for (int l = 0; l < n_levels; ++l) {
        pk_index *hs[1] = {levels[l]};
        LevelArgs a{};
        a.nq = nq;
        a.k = k;
        a.metric = own->cfg.metric;
        a.level = l;
        a.first = l == 0;
        a.last = l == n_levels - 1;
        a.stop = stop;
        a.open = open;
        a.level_out = out_level;
        a.out_ids = out_ids;
        a.out_dist = out_dist;
        if (l == 0) {
            PK_TRY(search_impl(hs, 1, offs, queries, k, nprobes[0], kFull, nullptr, nullptr, out_ids, out_dist, s));
        } else {
            // coarse step for the batch, lists of the queries that have ended struck out, fine search
            PK_TRY(search_impl(hs, 1, offs, queries, 1, nprobes[l], kCoarseOnly, nullptr, probes, nullptr, nullptr, s));
            PK_HIP(launch_level_mask(probes, nprobes[l], open, nq, s));
            PK_TRY(search_impl(hs, 1, offs, queries, k, nprobes[l], kForced, probes, nullptr, row_ids, row_dist, s));
            a.row_ids = row_ids;
            a.row_dist = row_dist;
        }
        PK_HIP(launch_level_accept(a, s));
    }
    return PK_OK;
}

int pk_coarse(pk_index *ix, const float *queries, int64_t nq, int32_t nprobe, int32_t *out_probes, void *stream)
{
    PK_TRY(check_search_args(ix, queries, nq, 1, nprobe));
    if (nq > 0 && !out_probes) return PK_ERR_INVALID_ARG;
    if (nq == 0) return PK_OK;
    pk_index *hs[1] = {ix};
    const int64_t offs[2] = {0, nq};
    return search_impl(hs, 1, offs, queries, 1, nprobe, kCoarseOnly, nullptr, out_probes, nullptr, nullptr,
                       static_cast<hipStream_t>(stream));
}

int pk_scan_probes(pk_index *ix, const float *queries, int64_t nq, int32_t k, int32_t nprobe, const int32_t *probes,
                   int64_t *out_ids, float *out_dist, void *stream)
{
    PK_TRY(check_search_args(ix, queries, nq, k, nprobe));
    if (nq > 0 && (!probes || !out_ids || !out_dist)) return PK_ERR_INVALID_ARG;
    if (nq == 0) return PK_OK;
    pk_index *hs[1] = {ix};
    const int64_t offs[2] = {0, nq};
    return search_impl(hs, 1, offs, queries, k, nprobe, kForced, probes, nullptr, out_ids, out_dist,
                       static_cast<hipStream_t>(stream));
}

int pk_index_stats(pk_index *ix, pk_stats *out, void *stream)
{
    if (!live(ix)) return PK_ERR_BAD_HANDLE;
    if (!out) return PK_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t ctr[4] = {0, 0, 0, 0};
    std::vector<uint32_t> len((size_t)ix->cfg.nlist);
    PK_HIP(hipMemcpyAsync(ctr, ix->host.ctr, sizeof(ctr), hipMemcpyDeviceToHost, s));
    PK_HIP(hipMemcpyAsync(len.data(), ix->host.list_len, len.size() * 4, hipMemcpyDeviceToHost, s));
    PK_HIP(hipStreamSynchronize(s));
    PK_TRY(settle_pages(ix));
    std::memset(out, 0, sizeof(*out));
    // The device's list lengths are the truth: a batch the device refused (sticky error flag:
    // a list's delta-page table was full) was counted on the host when it was enqueued.
    // (the host's own count of inserts only serves as an upper bound and stays as it is)
    int64_t held = 0;
    for (uint32_t v : len) held += v;
    const int64_t refused = ctr[1] != 0 ? std::max<int64_t>(0, ix->n_total - held) : 0;
    ix->n_total = held;
    ix->n_refused += refused;
    out->n_total = held;
    out->n_inserted = std::max<int64_t>(0, ix->n_inserted - ix->n_refused);
    out->pages_total = ix->pages_total;
    out->pages_used = ctr[0];
    out->arena_bytes = (int64_t)ix->arena_bytes;
    out->workspace_bytes = (int64_t)ix->ws_bytes;
    out->workspace_grows = ix->ws_grows;
    out->max_list_len = len.empty() ? 0 : *std::max_element(len.begin(), len.end());
    out->device_error = (int32_t)ctr[1];
    out->n_arenas = ix->host.n_arenas;
    return PK_OK;
}

int pk_list_lengths(pk_index *ix, int64_t *out_len, void *stream)
{
    if (!live(ix)) return PK_ERR_BAD_HANDLE;
    if (!out_len) return PK_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    std::vector<uint32_t> len((size_t)ix->cfg.nlist);
    PK_HIP(hipMemcpyAsync(len.data(), ix->host.list_len, len.size() * 4, hipMemcpyDeviceToHost, s));
    PK_HIP(hipStreamSynchronize(s));
    for (size_t i = 0; i < len.size(); ++i) out_len[i] = len[i];
    return PK_OK;
}

int pk_profile_begin(pk_index *ix, void *stream)
{
    if (!live(ix)) return PK_ERR_BAD_HANDLE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    PK_HIP(launch_fill_u32(reinterpret_cast<uint32_t *>(ix->host.stats), 0u, 16, s));
    ix->prof_used = 0;
    ix->prof_beside.clear();
    ix->prof_on = true;
    return PK_OK;
}

int pk_profile_end(pk_index *ix, pk_profile *out, void *stream)
{
    if (!live(ix)) return PK_ERR_BAD_HANDLE;
    if (!out) return PK_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    ix->prof_on = false;
    unsigned long long st[6] = {0, 0, 0, 0, 0, 0};
    PK_HIP(hipMemcpyAsync(st, ix->host.stats, sizeof(st), hipMemcpyDeviceToHost, s));
    PK_HIP(hipStreamSynchronize(s));
    std::memset(out, 0, sizeof(*out));
    const size_t n = ix->prof_used / kProfEvents;
    for (size_t i = 0; i < n; ++i) {
        float ms[5];
        for (int j = 0; j < 5; ++j)
            PK_HIP(hipEventElapsedTime(&ms[j], ix->prof_ev[i * kProfEvents + j], ix->prof_ev[i * kProfEvents + j + 1]));
        out->coarse_ms += ms[0];
        out->worklist_ms += ms[1];
        out->scan_ms += ms[2] + ms[3];
        out->scan_hot_ms += i < ix->prof_beside.size() && ix->prof_beside[i] ? ms[2] : ms[3];
        out->select_ms += ms[4];
    }
    out->launches = (int32_t)n;
    out->scanned_rows = (int64_t)st[0];
    out->candidates = (int64_t)st[1];
    out->tiles = (int64_t)st[2];
    out->emitted = (int64_t)st[3];
    out->overflowed = (int64_t)st[4];
    out->max_emitted = (int64_t)st[5];
    ix->prof_used = 0;
    ix->prof_beside.clear();
    return PK_OK;
}

int pk_index_free(pk_index *ix)
{
    if (!live(ix)) return PK_ERR_BAD_HANDLE;
    destroy(ix);
    return PK_OK;
}

const char *pk_strerror(int status)
{
    switch (status) {
    case PK_OK: return "ok";
    case PK_ERR_INVALID_ARG: return "invalid argument";
    case PK_ERR_BAD_HANDLE: return "bad index handle";
    case PK_ERR_DIM_MISMATCH: return "handles differ in dimension, metric or storage";
    case PK_ERR_NOMEM: return "out of arena, workspace or host memory";
    case PK_ERR_HIP: return "HIP runtime error";
    case PK_ERR_UNSUPPORTED: return "request outside the supported limits";
    case PK_ERR_WORKSPACE: return "the call needs more workspace than the fixed-size one it was given";
    default: return "unknown status";
    }
}

} // extern "C"
