// Device-side pieces of the work-list construction, shared by the kernels that run them on
// their own (pk_worklist.hip) and by the kernels that take them along to save launches on
// small batches (the coarse selection counts the pairs; the first workgroups of the launch
// that scores the threshold sample, or else the threshold kernel's, lay out slots and tiles).
#pragma once

#include "pk_internal.h"

#ifndef PK_WL_MARK
#define PK_WL_MARK(i) do { } while (0)
#endif

namespace pk {

// Work of one query: count the pairs per list, lay the query's candidate range out probe by
// probe; and the tiles of the query's threshold sample: sm.sp pages of its nearest lists, full
// pages before partly filled ones, so that a query whose best lists are short still draws its
// threshold from at least k rows whenever longer lists follow.  Called by every thread of a workgroup.  probes_q: the query's probe list (global
// memory or, straight from the selection, LDS); probes_out: where to store it, or null.
// v: the query's index, read ahead of the caller's own work so that the chain of dependent loads is
// over by now.  Everything is read before anything is written: a load queues behind the stores and
// atomics issued before it, and those take longest.
struct WlIndexView {
    const DevIndex *ix;
    const uint32_t *list_len, *main_pages, *main_base;
    uint32_t ag, P, nlist;
};
__device__ __forceinline__ WlIndexView wl_index_view(const WorklistArgs &a, const MultiArgs &m, uint32_t q)
{
    WlIndexView v;
    v.ag = a.qagent[q];
    v.ix = m.ix[v.ag];
    v.list_len = v.ix->list_len;
    v.main_pages = v.ix->main_pages;
    v.main_base = v.ix->main_base;
    v.P = (uint32_t)v.ix->P;
    v.nlist = (uint32_t)v.ix->nlist;
    return v;
}
struct WlCountLds {
    uint32_t len[PK_MAX_NPROBE];     // rows of each probed list
    uint32_t mp[PK_MAX_NPROBE];      // pages of its build-time extent
    uint32_t mb[PK_MAX_NPROBE];      // first page of that extent
    uint32_t po[PK_MAX_NPROBE + 1];  // candidates of the probed lists before each one
    uint16_t sr[kMaxSamplePages];    // the sample's pages: which probed list,
    uint32_t slp[kMaxSamplePages];   //   and which of its pages
    uint32_t ns;                     // how many there are
};
__device__ __forceinline__ void wl_count_query(const WorklistArgs &a, const SampleArgs &sm, const MultiArgs &m, uint32_t q,
                                               WlCountLds &s, const int32_t *probes_q, int32_t *probes_out,
                                               const WlIndexView &v)
{
    const DevIndex &ix = *v.ix;
    const uint32_t P = v.P;
    for (int r = threadIdx.x; r < a.nprobe; r += blockDim.x) {
        const uint32_t l = (uint32_t)probes_q[r];
        const bool valid = l < v.nlist;
        s.len[r] = valid ? v.list_len[l] : 0u;
        s.mp[r] = valid ? v.main_pages[l] : 0u;
        s.mb[r] = valid ? v.main_base[l] : 0u;
    }
    __syncthreads();
    PK_WL_MARK(5);
    if (threadIdx.x == 0) {
        uint32_t acc = 0;
        for (int r = 0; r < a.nprobe; ++r) {
            s.po[r] = acc;
            acc += (s.len[r] + 15u) & ~15u; // segments are padded to the 16-row MFMA tile
        }
        s.po[a.nprobe] = acc;
        // The sample's pages: full pages first, nearest lists first, then the lists' last, partly filled
        // pages: short lists at the head of the probe list cannot leave the sample with fewer than k
        // rows (and the query without a threshold) while longer lists follow.
        const uint32_t want = (uint32_t)sm.sp;
        uint32_t ns = 0;
        for (int r = 0; r < a.nprobe && ns < want; ++r)
            for (uint32_t lp = 0; lp < s.len[r] / P && ns < want; ++lp) {
                s.sr[ns] = (uint16_t)r;
                s.slp[ns++] = lp;
            }
        for (int r = 0; r < a.nprobe && ns < want; ++r)
            if (s.len[r] % P) {
                s.sr[ns] = (uint16_t)r;
                s.slp[ns++] = s.len[r] / P;
            }
        s.ns = ns;
    }
    __syncthreads();
    PK_WL_MARK(6);
    for (uint32_t p = threadIdx.x; p < (uint32_t)sm.sp; p += blockDim.x) {
        Tile tl;
        tl.x = ix.arenas[0].vec;
        tl.xn = ix.arenas[0].norm;
        tl.row0 = p * P; // position inside the sample, not inside a list
        tl.qbeg = q;
        tl.nrows = 0;
        tl.qcnt = 1;
        tl.pad = 0;
        if (p < s.ns) {
            const int r = s.sr[p];
            const uint32_t l = (uint32_t)probes_q[r];
            const uint32_t lp = s.slp[p];
            const uint32_t pg = lp < s.mp[r] ? s.mb[r] + lp : ix.dtab[(size_t)l * ix.max_dp + (lp - s.mp[r])];
            const Arena &ar = arena_of(ix, pg);
            const size_t local = pg - ar.first_page;
            tl.x = ar.vec + local * P * (size_t)ix.row_bytes;
            tl.xn = ar.norm + local * P;
            const uint32_t left = s.len[r] - lp * P;
            tl.nrows = (uint16_t)(left < P ? left : P);
        }
        sm.tiles[(size_t)q * sm.sp + p] = tl;
    }
    // from here on, stores only
    uint32_t *po = a.pair_off + (size_t)q * (a.nprobe + 1);
    for (int r = threadIdx.x; r <= a.nprobe; r += blockDim.x) {
        po[r] = s.po[r];
        if (r < a.nprobe) {
            const uint32_t l = (uint32_t)probes_q[r];
            if (probes_out) probes_out[r] = (int32_t)l;
            if (l < v.nlist) atomicAdd(&a.lcnt[(size_t)v.ag * a.nlist_max + l], 1u);
        }
    }
    const float worst = sm.metric == PK_METRIC_IP ? -INFINITY : INFINITY;
    float *vals = sm.vals + (size_t)q * sm.span;
    for (uint32_t i = threadIdx.x; i < sm.span; i += blockDim.x) vals[i] = worst;
    if (threadIdx.x == 0) {
        a.ccnt[q] = 0;
        sm.tcur[q] = 0; // until the threshold exists: the query's sample tiles that are done (small batches)
        sm.slot_query[q] = q;
        sm.slot_out[q] = q * sm.span;
        if (q == 0) {
            const uint32_t ntiles = (uint32_t)sm.nq * (uint32_t)sm.sp;
            sm.scalars[0] = ntiles;
            sm.scalars[1] = 0;
            const uint32_t g = ntiles / (uint32_t)(sm.scan_grid * 4);
            sm.scalars[2] = g < 1 ? 1 : (g > 8 ? 8 : g);
        }
    }
}

// One workgroup (any size up to 1024): offsets of the lists' slot ranges and tile ranges.
__device__ __forceinline__ void wl_scan_body(const WorklistArgs &a, const MultiArgs &m, uint32_t *s_wave /*[17]*/)
{
    const uint32_t nl = (uint32_t)a.n_handles * (uint32_t)a.nlist_max;
    block_exscan(a.lcnt, a.lstart, nl, s_wave);
    // tiles per list: regular lists -> ltile, hot lists -> lhtile (counts first, then their scans in place)
    unsigned long long rows = 0;
    for (uint32_t gl = threadIdx.x; gl < nl; gl += blockDim.x) {
        const uint32_t h = gl / (uint32_t)a.nlist_max, l = gl - h * (uint32_t)a.nlist_max;
        uint32_t nt_reg = 0, nt_hot = 0;
        const uint32_t c = a.lcnt[gl];
        if (c > 0) {
            const DevIndex &ix = *m.ix[h];
            const uint32_t len = ix.list_len[l];
            const uint32_t pages = (len + (uint32_t)ix.P - 1) / (uint32_t)ix.P;
            if (c > a.hot_from) {
                // hot tiles of the rows-in-registers kernel cover hot_rows rows, not a page
                const uint32_t units = a.hot_rows ? (len + (uint32_t)a.hot_rows - 1) / (uint32_t)a.hot_rows : pages;
                nt_hot = units * ((c + (uint32_t)a.mq_hot - 1) / (uint32_t)a.mq_hot);
            } else {
                nt_reg = pages * ((c + (uint32_t)a.mq - 1) / (uint32_t)a.mq);
            }
            rows += len;
        }
        a.ltile[gl] = nt_reg;
        a.lhtile[gl] = nt_hot;
    }
    __syncthreads();
    for (int hot = 0; hot < 2; ++hot) {
        // a class no list can fall into (no hot class at all, or every list hot) needs no scan
        const bool none = hot ? a.hot_from == 0xffffffffu : a.hot_from == 0u;
        uint32_t *lt = hot ? a.lhtile : a.ltile;
        const uint32_t ntiles = none ? 0u : block_exscan(lt, lt, nl, s_wave);
        if (threadIdx.x == 0) {
            uint32_t nt = ntiles;
            if (ntiles > a.tile_cap) {
                // cannot happen while the host bounds hold; refuse to scan rather than overrun
                nt = 0;
                atomicOr(&m.ix[0]->ctr[1], (uint32_t)kErrWorklist);
            }
            uint32_t *sc = hot ? a.scalars_hot : a.scalars;
            sc[0] = nt;
            sc[1] = 0;
            // tiles per claimed batch (the rows-in-registers kernel claims its long tiles one by one)
            uint32_t g = nt / (uint32_t)(a.scan_grid * a.grab_div);
            g = g < 1 ? 1 : (g > 8 ? 8 : g);
            sc[2] = hot && a.hot_rows ? (uint32_t)a.hot_grab : g;
            if (nt) atomicAdd(&m.ix[0]->stats[2], (unsigned long long)nt);
        }
        __syncthreads();
    }
    for (int off = 32; off > 0; off >>= 1) rows += __shfl_xor(rows, off); // one atomic per wave
    if ((threadIdx.x & 63) == 0 && rows) atomicAdd(&m.ix[0]->stats[0], rows);
}

// slot of pair i = (query i / nprobe, probe i % nprobe): the next free slot of its list
// (lstart: the lists' first slots, in global memory or LDS)
__device__ __forceinline__ void wl_slot_of_pair(const WorklistArgs &a, const MultiArgs &m, size_t i, const uint32_t *lstart)
{
    const uint32_t q = (uint32_t)(i / a.nprobe), r = (uint32_t)(i - (size_t)q * a.nprobe);
    const uint32_t ag = a.qagent[q];
    if ((uint32_t)a.probes[i] >= (uint32_t)m.ix[ag]->nlist) return;
    const size_t gl = (size_t)ag * a.nlist_max + (uint32_t)a.probes[i];
    const uint32_t slot = lstart[gl] + atomicAdd(&a.lfill[gl], 1u);
    a.slot_query[slot] = q;
    a.slot_out[slot] = a.pair_off[(size_t)q * (a.nprobe + 1) + r];
}

// tile j of list gl (c pairs, hot or regular): tile order inside a list is [query group][unit of rows],
// so that neighbouring tiles share their query group
// (first_slot: where the list's slots start)
__device__ __forceinline__ void wl_write_tile(const WorklistArgs &a, const MultiArgs &m, uint32_t gl, uint32_t c, bool hot,
                                              uint32_t j, Tile *out, uint32_t first_slot)
{
    const uint32_t h = gl / (uint32_t)a.nlist_max, l = gl - h * (uint32_t)a.nlist_max;
    const DevIndex &ix = *m.ix[h];
    const uint32_t len = ix.list_len[l];
    const uint32_t P = (uint32_t)ix.P;
    const uint32_t mq = hot ? (uint32_t)a.mq_hot : (uint32_t)a.mq;
    // rows per tile: a page, or (hot tiles of the rows-in-registers kernel) a fixed part of one
    const uint32_t R = hot && a.hot_rows ? (uint32_t)a.hot_rows : P;
    const uint32_t units = (len + R - 1) / R;
    const uint32_t g = j / units, u = j - g * units;
    const uint32_t first = u * R; // position of the tile's first row in the list
    const uint32_t p = first / P, in_page = first - p * P;
    const uint32_t pg = phys_page(ix, l, p);
    const Arena &ar = arena_of(ix, pg);
    const size_t local = (size_t)(pg - ar.first_page) * P + in_page;
    Tile tl;
    tl.x = ar.vec + local * (size_t)ix.row_bytes;
    tl.xn = ar.norm + local;
    tl.row0 = first;
    tl.qbeg = first_slot + g * mq;
    const uint32_t left = len - first;
    tl.nrows = (uint16_t)(left < R ? left : R);
    const uint32_t ql = c - g * mq;
    tl.qcnt = (uint16_t)(ql < mq ? ql : mq);
    tl.pad = 0;
    out[j] = tl;
}

// all tiles of list gl, by one workgroup
__device__ __forceinline__ void wl_tiles_of_list(const WorklistArgs &a, const MultiArgs &m, uint32_t gl)
{
    const uint32_t c = a.lcnt[gl];
    if (c == 0) return;
    const bool hot = c > a.hot_from;
    if ((hot ? a.scalars_hot[0] : a.scalars[0]) == 0) return; // overflow guard tripped
    Tile *out = (hot ? a.tiles_hot : a.tiles) + (hot ? a.lhtile[gl] : a.ltile[gl]);
    const uint32_t h = gl / (uint32_t)a.nlist_max, l = gl - h * (uint32_t)a.nlist_max;
    const DevIndex &ix = *m.ix[h];
    const uint32_t len = ix.list_len[l];
    const uint32_t R = hot && a.hot_rows ? (uint32_t)a.hot_rows : (uint32_t)ix.P;
    const uint32_t mq = hot ? (uint32_t)a.mq_hot : (uint32_t)a.mq;
    const uint32_t total = ((len + R - 1) / R) * ((c + mq - 1) / mq);
    const uint32_t first_slot = a.lstart[gl];
    for (uint32_t j = threadIdx.x; j < total; j += blockDim.x) wl_write_tile(a, m, gl, c, hot, j, out, first_slot);
}

// Small batches: the second half of the work list (offsets, slots, tiles) as a share of the work of
// every workgroup of another kernel's launch (one workgroup of 256 threads per query), which saves the
// two launches it would otherwise take.  With at most kWlSmallLists lists in all, every workgroup repeats
// the three prefix sums over the lists in LDS (a few microseconds, and no workgroup has to wait for
// another), then places its own query's pairs and writes its share of the tiles.  Workgroup 0 also
// publishes the tile counts.  The pair counters' fill marks (lfill) are zero on entry.
constexpr int kWlPerThread = 8; // lists per thread: 256 threads cover kWlSmallLists in one round

// What a workgroup reads from global memory for its share, requested before the host kernel's own work so
// that the two latencies overlap.
struct WlPrefetch {
    uint32_t c[kWlPerThread], len[kWlPerThread], P[kWlPerThread]; // pairs, rows and page size of the thread's lists
    uint32_t probe, pair_off, ag, nlist;                          // the thread's pair of the query (if any)
};

__device__ __forceinline__ void wl_spread_prefetch(const WorklistArgs &a, const MultiArgs &m, uint32_t q, WlPrefetch &w)
{
    const uint32_t nl = (uint32_t)a.n_handles * (uint32_t)a.nlist_max;
    if (a.len1) { // one handle: nothing to look up first
#pragma unroll
        for (int j = 0; j < kWlPerThread; ++j) {
            const uint32_t gl = threadIdx.x * kWlPerThread + j;
            w.c[j] = w.len[j] = 0;
            w.P[j] = a.P1;
            if (gl < nl) {
                w.c[j] = a.lcnt[gl];
                if (gl < a.nlist1) w.len[j] = a.len1[gl];
            }
        }
        w.ag = 0;
        w.nlist = a.nlist1;
    } else {
#pragma unroll
        for (int j = 0; j < kWlPerThread; ++j) {
            const uint32_t gl = threadIdx.x * kWlPerThread + j;
            w.c[j] = w.len[j] = 0;
            w.P[j] = 1;
            if (gl < nl) {
                const uint32_t h = gl / (uint32_t)a.nlist_max, l = gl - h * (uint32_t)a.nlist_max;
                const DevIndex &ix = *m.ix[h];
                w.c[j] = a.lcnt[gl];
                w.P[j] = (uint32_t)ix.P;
                if (l < (uint32_t)ix.nlist) w.len[j] = ix.list_len[l];
            }
        }
        w.ag = a.qagent[q];
        w.nlist = (uint32_t)m.ix[w.ag]->nlist;
    }
    w.probe = 0xffffffffu;
    w.pair_off = 0;
    if (threadIdx.x < (uint32_t)a.nprobe) {
        w.probe = (uint32_t)a.probes[(size_t)q * a.nprobe + threadIdx.x];
        w.pair_off = a.pair_off[(size_t)q * (a.nprobe + 1) + threadIdx.x];
    }
}

// s_pref: LDS [3][kWlSmallLists + 1]; s_wave: LDS [12]
__device__ __forceinline__ void wl_spread(const WorklistArgs &a, const MultiArgs &m, uint32_t *s_pref, uint32_t *s_wave,
                                          uint32_t q, const WlPrefetch &w)
{
    constexpr int E = kWlPerThread;
    const uint32_t nl = (uint32_t)a.n_handles * (uint32_t)a.nlist_max;
    uint32_t *s_start = s_pref, *s_reg = s_pref + (kWlSmallLists + 1), *s_hot = s_reg + (kWlSmallLists + 1);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t tr[E], th[E];
    unsigned long long rows = 0;
#pragma unroll
    for (int j = 0; j < E; ++j) {
        tr[j] = th[j] = 0;
        const uint32_t c = w.c[j], len = w.len[j];
        if (c > 0) {
            const uint32_t pages = (len + w.P[j] - 1) / w.P[j];
            if (c > a.hot_from) {
                // hot tiles of the rows-in-registers kernel cover hot_rows rows, not a page
                const uint32_t units = a.hot_rows ? (len + (uint32_t)a.hot_rows - 1) / (uint32_t)a.hot_rows : pages;
                th[j] = units * ((c + (uint32_t)a.mq_hot - 1) / (uint32_t)a.mq_hot);
            } else {
                tr[j] = pages * ((c + (uint32_t)a.mq - 1) / (uint32_t)a.mq);
            }
            rows += len;
        }
    }
    PK_WL_MARK(20);
    uint32_t t0 = 0, t1 = 0, t2 = 0;
#pragma unroll
    for (int j = 0; j < E; ++j) {
        t0 += w.c[j];
        t1 += tr[j];
        t2 += th[j];
    }
    uint32_t x0 = t0, x1 = t1, x2 = t2;
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t y0 = __shfl_up(x0, off), y1 = __shfl_up(x1, off), y2 = __shfl_up(x2, off);
        if (lane >= off) {
            x0 += y0;
            x1 += y1;
            x2 += y2;
        }
    }
    if (lane == 63) {
        s_wave[wave] = x0;
        s_wave[4 + wave] = x1;
        s_wave[8 + wave] = x2;
    }
    __syncthreads();
    uint32_t run0 = x0 - t0, run1 = x1 - t1, run2 = x2 - t2, nslots = 0, ntr = 0, nth = 0;
    for (int v = 0; v < 4; ++v) {
        if (v < wave) {
            run0 += s_wave[v];
            run1 += s_wave[4 + v];
            run2 += s_wave[8 + v];
        }
        nslots += s_wave[v];
        ntr += s_wave[4 + v];
        nth += s_wave[8 + v];
    }
#pragma unroll
    for (int j = 0; j < E; ++j) { // entries past the last list hold the totals
        s_start[threadIdx.x * E + j] = run0;
        s_reg[threadIdx.x * E + j] = run1;
        s_hot[threadIdx.x * E + j] = run2;
        run0 += w.c[j];
        run1 += tr[j];
        run2 += th[j];
    }
    if (threadIdx.x == 0) {
        s_start[kWlSmallLists] = nslots;
        s_reg[kWlSmallLists] = ntr;
        s_hot[kWlSmallLists] = nth;
    }
    // cannot happen while the host bounds hold; refuse to scan rather than overrun
    if (ntr > a.tile_cap) ntr = 0xffffffffu;
    if (nth > a.tile_cap) nth = 0xffffffffu;
    if (q == 0) {
        if (threadIdx.x == 0) {
            for (int hot = 0; hot < 2; ++hot) {
                uint32_t nt = hot ? nth : ntr;
                if (nt == 0xffffffffu) {
                    nt = 0;
                    atomicOr(&m.ix[0]->ctr[1], (uint32_t)kErrWorklist);
                }
                uint32_t *sc = hot ? a.scalars_hot : a.scalars;
                sc[0] = nt;
                sc[1] = 0;
                // tiles per claimed batch (the rows-in-registers kernel claims its long tiles one by one)
                uint32_t g = nt / (uint32_t)(a.scan_grid * a.grab_div);
                g = g < 1 ? 1 : (g > 8 ? 8 : g);
                sc[2] = hot && a.hot_rows ? (uint32_t)a.hot_grab : g;
                if (nt) atomicAdd(&m.ix[0]->stats[2], (unsigned long long)nt);
            }
        }
        for (int off = 32; off > 0; off >>= 1) rows += __shfl_xor(rows, off); // one atomic per wave
        if (lane == 0 && rows) atomicAdd(&m.ix[0]->stats[0], rows);
    }
    __syncthreads();
    PK_WL_MARK(21);
    // the query's own pairs: the next free slot of each probed list (stored after the tiles' loads)
    uint32_t my_slot = 0xffffffffu;
    if (threadIdx.x < (uint32_t)a.nprobe && w.probe < w.nlist) {
        const size_t gl = (size_t)w.ag * a.nlist_max + w.probe;
        my_slot = s_start[gl] + atomicAdd(&a.lfill[gl], 1u);
    }
    PK_WL_MARK(22);
    for (int hot = 0; hot < 2; ++hot) {
        const uint32_t ntiles = hot ? nth : ntr;
        if (ntiles == 0u || ntiles == 0xffffffffu) continue;
        const uint32_t *lt = hot ? s_hot : s_reg;
        Tile *tiles = hot ? a.tiles_hot : a.tiles;
        for (uint32_t t = q * blockDim.x + threadIdx.x; t < ntiles; t += (uint32_t)a.nq * blockDim.x) {
            uint32_t lo = 0, hi = nl - 1; // last list whose first tile is at or before t: the list tile t belongs to
            while (lo < hi) {
                const uint32_t mid = (lo + hi + 1) >> 1;
                if (lt[mid] <= t) lo = mid;
                else hi = mid - 1;
            }
            wl_write_tile(a, m, lo, s_start[lo + 1] - s_start[lo], hot != 0, t - lt[lo], tiles + lt[lo], s_start[lo]);
        }
    }
    if (my_slot != 0xffffffffu) {
        a.slot_query[my_slot] = q;
        a.slot_out[my_slot] = w.pair_off;
    }
    for (uint32_t r = threadIdx.x + blockDim.x; r < (uint32_t)a.nprobe; r += blockDim.x) { // more probes than threads
        const uint32_t l = (uint32_t)a.probes[(size_t)q * a.nprobe + r];
        if (l >= w.nlist) continue;
        const size_t gl = (size_t)w.ag * a.nlist_max + l;
        const uint32_t slot = s_start[gl] + atomicAdd(&a.lfill[gl], 1u);
        a.slot_query[slot] = q;
        a.slot_out[slot] = a.pair_off[(size_t)q * (a.nprobe + 1) + r];
    }
}

} // namespace pk
