// Query preparation and work-list construction (device side, no host round trip).
//
// Section 5 of the paper batches operations; Section 3.2 keeps one index per agent and
// Section 4.4 notes that a per-cluster GPU launch is dominated by launch cost.  Here one
// batch (possibly addressed to many agents' indexes) becomes ONE list of fixed-size
// tiles: the (query, probed list) pairs are grouped by list, every list is cut into its
// pages and every page is paired with groups of at most MQ of the queries that probe it.
// Lists therefore are read once per batch, not once per query, and a 400 k-vector list
// is as good a citizen as a 50-vector one.
#include <algorithm>

#include "pk_internal.h"

namespace pk {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------- small utilities

__global__ void fill_u32_kernel(uint32_t *p, uint32_t v, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

hipError_t launch_fill_u32(uint32_t *p, uint32_t v, size_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    const int grid = (int)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
    hipLaunchKernelGGL(fill_u32_kernel, dim3(grid), dim3(256), 0, s, p, v, n);
    return hipGetLastError();
}

// ------------------------------------------------------------ query preparation

// one workgroup per query: convert to the storage type, zero pad to row_bytes, squared norm
// of the converted values (fp32 sum)
__device__ __forceinline__ void prep_row(const float *q, int d, int storage, int row_bytes, char *qs, float *qnorm)
{
    __shared__ float s_part[4];
    const size_t row = blockIdx.x;
    const float *src = q + row * d;
    const int n_el = storage == PK_F16 ? row_bytes / 2 : row_bytes / 4;
    float acc = 0.f;
    for (int i = threadIdx.x; i < n_el; i += blockDim.x) {
        float v = i < d ? src[i] : 0.f;
        if (storage == PK_F16) {
            const _Float16 h = (_Float16)v; // round to nearest even
            reinterpret_cast<_Float16 *>(qs + row * row_bytes)[i] = h;
            v = (float)h;
        } else {
            reinterpret_cast<float *>(qs + row * row_bytes)[i] = v;
        }
        acc += v * v;
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) qnorm[row] = s_part[0] + s_part[1] + s_part[2] + s_part[3];
}

__global__ __launch_bounds__(256) void prep_queries_kernel(const float *q, int d, int storage, int row_bytes, char *qs,
                                                           float *qnorm)
{
    prep_row(q, d, storage, row_bytes, qs, qnorm);
}

// the same for the coarse step (fp32), which also notes which handle each query belongs to
// and where its row of centroid scores lies
__global__ __launch_bounds__(256) void prep_coarse_kernel(const float *q, int d, int row_bytes, char *qs, float *qnorm,
                                                          QueryMeta meta, MultiArgs m)
{
    prep_row(q, d, PK_F32, row_bytes, qs, qnorm);
    // first kernel of a search: also clears the per-list pair counters of the fine step
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < meta.nclear; i += gridDim.x * blockDim.x) meta.clear[i] = 0u;
    if (threadIdx.x == 0) {
        const uint32_t t = blockIdx.x;
        int h = 0;
        while (h + 1 < m.n && t >= m.qlo[h + 1]) ++h;
        meta.cand_off[t] = t * meta.stride;
        meta.cand_cnt[t] = (uint32_t)m.ix[h]->nlist;
        meta.qagent[t] = (uint16_t)h;
    }
}

hipError_t launch_prep_queries(const float *q, int64_t nq, int d, int storage, int row_bytes, void *qs, float *qnorm,
                               hipStream_t s)
{
    if (nq <= 0) return hipSuccess;
    hipLaunchKernelGGL(prep_queries_kernel, dim3((uint32_t)nq), dim3(256), 0, s, q, d, storage, row_bytes,
                       static_cast<char *>(qs), qnorm);
    return hipGetLastError();
}

hipError_t launch_prep_coarse(const float *q, int64_t nq, int d, int row_bytes, void *qs, float *qnorm,
                              const QueryMeta &meta, const MultiArgs &m, hipStream_t s)
{
    if (nq <= 0) return hipSuccess;
    hipLaunchKernelGGL(prep_coarse_kernel, dim3((uint32_t)nq), dim3(256), 0, s, q, d, row_bytes, static_cast<char *>(qs),
                       qnorm, meta, m);
    return hipGetLastError();
}

// ---------------------------------------------------------------- list work list

// per query: count the pairs per list, lay the query's candidate range out probe by probe;
// and the tiles of the query's threshold sample: the first sm.sp pages of that range (the
// pages of its first probed list, then of its second, ...), so that a query whose best list is
// short still draws its threshold from at least k rows whenever it has that many candidates
__global__ __launch_bounds__(256) void wl_count_kernel(WorklistArgs a, SampleArgs sm, MultiArgs m)
{
    __shared__ uint32_t s_len[PK_MAX_NPROBE];    // rows of each probed list
    __shared__ uint32_t s_pg0[PK_MAX_NPROBE + 1]; // pages of the probed lists before each one
    const uint32_t q = blockIdx.x;
    const uint32_t ag = a.qagent[q];
    const DevIndex &ix = *m.ix[ag];
    const uint32_t P = (uint32_t)ix.P;
    for (int r = threadIdx.x; r < a.nprobe; r += blockDim.x) {
        const uint32_t l = (uint32_t)a.probes[(size_t)q * a.nprobe + r];
        uint32_t len = 0;
        if (l < (uint32_t)ix.nlist) {
            atomicAdd(&a.lcnt[(size_t)ag * a.nlist_max + l], 1u);
            len = ix.list_len[l];
        }
        s_len[r] = len;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t acc = 0, pages = 0;
        uint32_t *po = a.pair_off + (size_t)q * (a.nprobe + 1);
        for (int r = 0; r < a.nprobe; ++r) {
            po[r] = acc;
            s_pg0[r] = pages;
            acc += (s_len[r] + 15u) & ~15u; // segments are padded to the 16-row MFMA tile
            pages += (s_len[r] + P - 1) / P;
        }
        po[a.nprobe] = acc;
        s_pg0[a.nprobe] = pages;
        a.ccnt[q] = 0;
        atomicAdd(&m.ix[0]->stats[1], (unsigned long long)acc);
    }
    {
        const float worst = sm.metric == PK_METRIC_IP ? -INFINITY : INFINITY;
        float *v = sm.vals + (size_t)q * sm.span;
        for (uint32_t i = threadIdx.x; i < sm.span; i += blockDim.x) v[i] = worst;
        if (threadIdx.x == 0) {
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
    __syncthreads();
    for (uint32_t p = threadIdx.x; p < (uint32_t)sm.sp; p += blockDim.x) {
        Tile tl;
        tl.x = ix.arenas[0].vec;
        tl.xn = ix.arenas[0].norm;
        tl.row0 = p * P; // position inside the sample, not inside a list
        tl.qbeg = q;
        tl.nrows = 0;
        tl.qcnt = 1;
        tl.pad = 0;
        if (p < s_pg0[a.nprobe]) {
            int r = 0;
            while (s_pg0[r + 1] <= p) ++r; // the probed list that holds page p of the range
            const uint32_t l = (uint32_t)a.probes[(size_t)q * a.nprobe + r];
            const uint32_t lp = p - s_pg0[r];
            const uint32_t pg = phys_page(ix, l, lp);
            const Arena &ar = arena_of(ix, pg);
            const size_t local = pg - ar.first_page;
            tl.x = ar.vec + local * P * (size_t)ix.row_bytes;
            tl.xn = ar.norm + local * P;
            const uint32_t left = s_len[r] - lp * P;
            tl.nrows = (uint16_t)(left < P ? left : P);
        }
        sm.tiles[(size_t)q * sm.sp + p] = tl;
    }
}

// one workgroup: offsets of the lists' slot ranges and tile ranges
__global__ __launch_bounds__(1024) void wl_scan_kernel(WorklistArgs a, MultiArgs m)
{
    __shared__ uint32_t s_wave[17];
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
                // hot tiles of the rows-stationary kernel cover hot_rows rows, not a page
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
            // tiles per claimed batch
            uint32_t g = nt / (uint32_t)(a.scan_grid * a.grab_div);
            g = g < 1 ? 1 : (g > 8 ? 8 : g);
            // a rows-stationary tile is long (all slots of its list) and tiles differ tenfold: one per claim
            sc[2] = hot && a.hot_rows ? (uint32_t)a.hot_grab : g;
            if (nt) atomicAdd(&m.ix[0]->stats[2], (unsigned long long)nt);
        }
        __syncthreads();
    }
    if (rows) atomicAdd(&m.ix[0]->stats[0], rows);
    __syncthreads();
    for (uint32_t gl = threadIdx.x; gl < nl; gl += blockDim.x) a.lfill[gl] = 0;
}

// slots: every (query, probe) pair takes the next free slot of its list (one thread per pair)
__device__ __forceinline__ void wl_slots_block(const WorklistArgs &a, const MultiArgs &m, uint32_t block)
{
    const size_t i = (size_t)block * blockDim.x + threadIdx.x;
    if (i >= (size_t)a.nq * a.nprobe) return;
    const uint32_t q = (uint32_t)(i / a.nprobe), r = (uint32_t)(i - (size_t)q * a.nprobe);
    const uint32_t ag = a.qagent[q];
    if ((uint32_t)a.probes[i] >= (uint32_t)m.ix[ag]->nlist) return;
    const size_t gl = (size_t)ag * a.nlist_max + (uint32_t)a.probes[i];
    const uint32_t slot = a.lstart[gl] + atomicAdd(&a.lfill[gl], 1u);
    a.slot_query[slot] = q;
    a.slot_out[slot] = a.pair_off[(size_t)q * (a.nprobe + 1) + r];
}

// tiles: one workgroup per list; tile order inside a list is [query group][page], so that
// neighbouring tiles share their query group
__device__ __forceinline__ void wl_tiles_block(const WorklistArgs &a, const MultiArgs &m, uint32_t gl)
{
    const uint32_t c = a.lcnt[gl];
    if (c == 0) return;
    const bool hot = c > a.hot_from;
    if ((hot ? a.scalars_hot[0] : a.scalars[0]) == 0) return; // overflow guard tripped
    const uint32_t h = gl / (uint32_t)a.nlist_max, l = gl - h * (uint32_t)a.nlist_max;
    const DevIndex &ix = *m.ix[h];
    const uint32_t len = ix.list_len[l];
    const uint32_t P = (uint32_t)ix.P;
    const uint32_t pages = (len + P - 1) / P;
    const uint32_t mq = hot ? (uint32_t)a.mq_hot : (uint32_t)a.mq;
    const uint32_t groups = (c + mq - 1) / mq;
    Tile *out = (hot ? a.tiles_hot : a.tiles) + (hot ? a.lhtile[gl] : a.ltile[gl]);
    // rows per tile: a page, or (hot tiles of the rows-stationary kernel) a fixed part of one
    const uint32_t R = hot && a.hot_rows ? (uint32_t)a.hot_rows : P;
    const uint32_t units = hot && a.hot_rows ? (len + R - 1) / R : pages;
    for (uint32_t j = threadIdx.x; j < units * groups; j += blockDim.x) {
        const uint32_t g = j / units, u = j - g * units;
        const uint32_t first = u * R;          // position of the tile's first row in the list
        const uint32_t p = first / P, in_page = first - p * P;
        const uint32_t pg = phys_page(ix, l, p);
        const Arena &ar = arena_of(ix, pg);
        const size_t local = (size_t)(pg - ar.first_page) * P + in_page;
        Tile tl;
        tl.x = ar.vec + local * (size_t)ix.row_bytes;
        tl.xn = ar.norm + local;
        tl.row0 = first;
        tl.qbeg = a.lstart[gl] + g * mq;
        const uint32_t left = len - first;
        tl.nrows = (uint16_t)(left < R ? left : R);
        const uint32_t ql = c - g * mq;
        tl.qcnt = (uint16_t)(ql < mq ? ql : mq);
        tl.pad = 0;
        out[j] = tl;
    }
}

// Slots and tiles both need only the offsets wl_scan wrote, not each other: one launch, the
// first slot_blocks workgroups place the pairs, the others write one list's tiles each.
__global__ __launch_bounds__(256) void wl_slots_tiles_kernel(WorklistArgs a, MultiArgs m, uint32_t slot_blocks)
{
    if (blockIdx.x < slot_blocks) wl_slots_block(a, m, blockIdx.x);
    else wl_tiles_block(a, m, blockIdx.x - slot_blocks);
}


// first half of the work list: pairs per list and the candidate layout of every query, and the
// tiles of the threshold sample (which the caller scores next)
hipError_t launch_worklist_count(const WorklistArgs &a, const SampleArgs &sm, const MultiArgs &m, hipStream_t s)
{
    if (!a.lcnt_cleared) {
        const hipError_t e = launch_fill_u32(a.lcnt, 0u, (size_t)a.n_handles * (size_t)a.nlist_max, s);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(wl_count_kernel, dim3((uint32_t)a.nq), dim3(256), 0, s, a, sm, m);
    return hipGetLastError();
}

// second half: slot ranges of the lists, slots of the pairs, tiles
hipError_t launch_worklist_tiles(const WorklistArgs &a, const MultiArgs &m, hipStream_t s)
{
    const uint32_t nl = (uint32_t)a.n_handles * (uint32_t)a.nlist_max;
    hipLaunchKernelGGL(wl_scan_kernel, dim3(1), dim3(1024), 0, s, a, m);
    const uint32_t slot_blocks = (uint32_t)(((size_t)a.nq * a.nprobe + 255) / 256);
    hipLaunchKernelGGL(wl_slots_tiles_kernel, dim3(slot_blocks + nl), dim3(256), 0, s, a, m, slot_blocks);
    return hipGetLastError();
}

} // namespace pk
