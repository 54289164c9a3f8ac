// Index construction and the insert path (device side).
//
// Section 3.1 / Section 6.1 "IVF-Static": a vector is appended to the list of its nearest
// centroid and nothing else changes.  Section 4.4 keeps new vectors of a GPU-resident
// cluster in a CPU-side buffer because a device list cannot grow in place; here a list
// is a chain of fixed-size pages, so growing it means taking the next free page of the
// arena: no reallocation, no copy of old data, no host involvement.
#include "pk_internal.h"

namespace pk {

// centroid table in scan layout: [nlist_pad][dpad32] fp32, zero padded, plus squared norms
__global__ __launch_bounds__(256) void store_centroids_kernel(const float *c, int nlist, int d, int dpad32, int metric,
                                                              float *cent, float *cnorm)
{
    __shared__ float s_part[4];
    const int row = blockIdx.x;
    float acc = 0.f;
    for (int i = threadIdx.x; i < dpad32; i += blockDim.x) {
        const float v = (row < nlist && i < d) ? c[(size_t)row * d + i] : 0.f;
        cent[(size_t)row * dpad32 + i] = v;
        acc += v * v;
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) cnorm[row] = metric == PK_METRIC_L2 ? s_part[0] + s_part[1] + s_part[2] + s_part[3] : 0.f;
}

hipError_t launch_store_centroids(const float *c, int nlist, int d, int dpad32, int nlist_pad, int metric, float *cent,
                                  float *cnorm, hipStream_t s)
{
    hipLaunchKernelGGL(store_centroids_kernel, dim3(nlist_pad), dim3(256), 0, s, c, nlist, d, dpad32, metric, cent,
                       cnorm);
    return hipGetLastError();
}

__global__ void hist_kernel(const int32_t *assign, int64_t n, uint32_t *cnt)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        atomicAdd(&cnt[assign[i]], 1u);
}

hipError_t launch_hist(const int32_t *assign, int64_t n, uint32_t *cnt, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const int grid = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    hipLaunchKernelGGL(hist_kernel, dim3(grid), dim3(256), 0, s, assign, n, cnt);
    return hipGetLastError();
}

// one wave writes one vector into slot `slot` of list `l`: convert (fp16: round to nearest
// even), zero pad the row, squared norm of the stored values, id
__device__ void write_row(const DevIndex &ix, uint32_t l, uint32_t slot, const float *src, int64_t id)
{
    const uint32_t P = (uint32_t)ix.P;
    const uint32_t lp = slot / P;
    const uint32_t pg = phys_page(ix, l, lp);
    const Arena &ar = arena_of(ix, pg);
    const size_t local = (size_t)(pg - ar.first_page) * P + (slot - lp * P);
    char *dst = ar.vec + local * (size_t)ix.row_bytes;
    const int lane = threadIdx.x & 63;
    const int n_el = ix.storage == PK_F16 ? ix.row_bytes / 2 : ix.row_bytes / 4;
    float acc = 0.f;
    constexpr int kBatch = 8; // elements read before the first of them is written: a load queues behind earlier stores
    for (int i0 = lane; i0 < n_el; i0 += 64 * kBatch) {
        float v[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int i = i0 + 64 * u;
            v[u] = i < ix.d ? src[i] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int i = i0 + 64 * u;
            if (i >= n_el) continue;
            if (ix.storage == PK_F16) {
                const _Float16 h = (_Float16)v[u];
                reinterpret_cast<_Float16 *>(dst)[i] = h;
                v[u] = (float)h;
            } else {
                reinterpret_cast<float *>(dst)[i] = v[u];
            }
            acc += v[u] * v[u];
        }
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (lane == 0) {
        ar.norm[local] = acc;
        ar.ids[local] = id;
    }
}

// build: every vector takes the next slot of its list's build-time extent
__global__ __launch_bounds__(256) void scatter_build_kernel(const DevIndex *ixp, const float *x, const int64_t *ids,
                                                            const int32_t *assign, int64_t n, int64_t id0, uint32_t *fill)
{
    const DevIndex &ix = *ixp;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int64_t i = (int64_t)blockIdx.x * 4 + wave; i < n; i += (int64_t)gridDim.x * 4) {
        const uint32_t l = (uint32_t)assign[i];
        uint32_t slot = 0;
        if (lane == 0) slot = atomicAdd(&fill[l], 1u);
        slot = __shfl(slot, 0);
        write_row(ix, l, slot, x + (size_t)i * ix.d, ids ? ids[i] : id0 + i);
    }
}

hipError_t launch_scatter_build(const DevIndex *ix, const float *x, const int64_t *ids, const int32_t *assign, int64_t n,
                                int64_t id0, uint32_t *fill, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const int64_t want = (n + 3) / 4;
    const int grid = (int)(want < 65536 ? want : 65536);
    hipLaunchKernelGGL(scatter_build_kernel, dim3(grid), dim3(256), 0, s, ix, x, ids, assign, n, id0, fill);
    return hipGetLastError();
}

// Insert, step 2: slot reservation for a batch of at most 1024 vectors by one workgroup.
// Vector i takes slot list_len[l] + (number of earlier batch members of the same list), so
// the order inside a list is the arrival order.  A vector whose slot starts a page beyond
// the build-time extent opens a delta page.  If the arena or a list's delta table cannot
// take the whole batch, nothing is changed, every slot is 0xffffffff and the sticky error
// flag is set.  Small batches (x given): the workgroup's 16 waves also write the rows
// (step 3), which saves the launch that would otherwise follow.
__global__ __launch_bounds__(1024) void reserve_kernel(MultiArgs ma, const int32_t *assign, unsigned long long *best,
                                                       uint32_t *slots, int32_t *assigned_out, AppendIds idc,
                                                       const float *x, const int64_t *ids)
{
    __shared__ int32_t s_l[1024];
    __shared__ uint32_t s_slot[1024];
    __shared__ uint32_t s_need, s_bad, s_page0;
    // workgroup a serves handle a: its vectors are rows [qlo[a], qlo[a+1]) of the batch
    const DevIndex &ix = *ma.ix[blockIdx.x];
    const uint32_t row0 = ma.qlo[blockIdx.x];
    const int m = (int)(ma.qlo[blockIdx.x + 1] - row0);
    if (m == 0) return;
    if (assign) assign += row0;
    slots += row0;
    if (assigned_out) assigned_out += row0;
    const int i = threadIdx.x;
    if (i == 0) {
        s_need = 0;
        s_bad = 0;
    }
    int32_t l = -1;
    if (i < m) {
        if (assign) {
            l = assign[i];
        } else { // the top-1 key the centroid kernel left (reset for the next insert on the way out)
            l = (int32_t)(uint32_t)best[row0 + i];
        }
        if (l < 0 || l >= ix.nlist) l = -1;
    }
    s_l[i] = l;
    __syncthreads();
    uint32_t rank = 0, cnt = 0;
    if (l >= 0) {
        for (int j = 0; j < m; ++j) {
            const bool same = s_l[j] == l;
            cnt += same ? 1u : 0u;
            rank += (same && j < i) ? 1u : 0u;
        }
    }
    uint32_t slot = 0xffffffffu, di = 0;
    bool opens = false;
    if (l >= 0) {
        slot = ix.list_len[l] + rank;
        const uint32_t lp = slot / (uint32_t)ix.P;
        if (slot % (uint32_t)ix.P == 0 && lp >= ix.main_pages[l]) {
            di = lp - ix.main_pages[l];
            if (di >= (uint32_t)ix.max_dp) atomicOr(&s_bad, (uint32_t)kErrListFull);
            // a list that shrank (deletes) still owns the delta pages it had: take a new one
            // only where the table has none
            else opens = ix.dtab[(size_t)l * ix.max_dp + di] == 0xffffffffu;
        }
    } else if (i < m) {
        atomicOr(&s_bad, (uint32_t)kErrListFull);
    }
    uint32_t my_page = 0;
    if (opens) my_page = atomicAdd(&s_need, 1u);
    __syncthreads();
    if (i == 0) {
        const uint32_t p0 = ix.ctr[0];
        s_page0 = p0;
        if (p0 + s_need > ix.ctr[2]) s_bad |= (uint32_t)kErrPages;
        if (s_bad) atomicOr(&ix.ctr[1], s_bad);
        else ix.ctr[0] = p0 + s_need;
    }
    __syncthreads();
    const bool ok = s_bad == 0;
    if (ok && opens) ix.dtab[(size_t)l * ix.max_dp + di] = s_page0 + my_page;
    if (ok && l >= 0 && rank == cnt - 1) ix.list_len[l] = slot + 1;
    if (i < m) {
        slots[i] = ok ? slot : 0xffffffffu;
        if (assigned_out) assigned_out[i] = l;
    }
    if (!x) {
        if (best && !assign && i < m) best[row0 + i] = ~0ull;
        return;
    }
    s_slot[i] = ok ? slot : 0xffffffffu;
    __syncthreads(); // slots, and the page table entries just written, are visible to the whole workgroup
    for (int r = i >> 6; r < m; r += 16) {
        if (s_slot[r] == 0xffffffffu) continue;
        const uint32_t row = row0 + (uint32_t)r;
        write_row(ix, (uint32_t)s_l[r], s_slot[r], x + (size_t)row * ix.d,
                  ids ? ids[row] : idc.id0[blockIdx.x] + (int64_t)r);
    }
    if (best && !assign && i < m) best[row0 + i] = ~0ull;
}

hipError_t launch_reserve(const MultiArgs &ma, const int32_t *assign, uint32_t *slots, int32_t *assigned_out, hipStream_t s)
{
    if (ma.n <= 0 || ma.qlo[ma.n] == 0) return hipSuccess;
    for (int a = 0; a < ma.n; ++a)
        if (ma.qlo[a + 1] - ma.qlo[a] > 1024u) return hipErrorInvalidValue;
    hipLaunchKernelGGL(reserve_kernel, dim3(ma.n), dim3(1024), 0, s, ma, assign, nullptr, slots, assigned_out, AppendIds{},
                       nullptr, nullptr);
    return hipGetLastError();
}

// steps 2 and 3 in one launch, for batches of at most kFusedAppend vectors per handle
hipError_t launch_reserve_append(const MultiArgs &ma, const AppendIds &idc, const float *x, const int64_t *ids,
                                 const int32_t *assign, unsigned long long *best, uint32_t *slots, int32_t *assigned_out,
                                 hipStream_t s)
{
    if (ma.n <= 0 || ma.qlo[ma.n] == 0) return hipSuccess;
    if (!x || (!assign && !best)) return hipErrorInvalidValue;
    for (int a = 0; a < ma.n; ++a)
        if (ma.qlo[a + 1] - ma.qlo[a] > (uint32_t)kFusedAppend) return hipErrorInvalidValue;
    hipLaunchKernelGGL(reserve_kernel, dim3(ma.n), dim3(1024), 0, s, ma, assign, best, slots, assigned_out, idc, x, ids);
    return hipGetLastError();
}

// Insert, step 3: write the vectors into their reserved slots
__global__ __launch_bounds__(256) void append_kernel(MultiArgs ma, AppendIds idc, const float *x, const int64_t *ids,
                                                     const int32_t *assign, const uint32_t *slots)
{
    const int wave = threadIdx.x >> 6;
    const uint32_t i = blockIdx.x * 4 + wave;
    if (i >= ma.qlo[ma.n]) return;
    int h = 0;
    while (h + 1 < ma.n && i >= ma.qlo[h + 1]) ++h;
    const DevIndex &ix = *ma.ix[h];
    const uint32_t slot = slots[i];
    if (slot == 0xffffffffu) return;
    write_row(ix, (uint32_t)assign[i], slot, x + (size_t)i * ix.d, ids ? ids[i] : idc.id0[h] + (int64_t)(i - ma.qlo[h]));
}

hipError_t launch_append(const MultiArgs &ma, const AppendIds &idc, const float *x, const int64_t *ids,
                         const int32_t *assign, const uint32_t *slots, hipStream_t s)
{
    const uint32_t m = ma.n > 0 ? ma.qlo[ma.n] : 0u;
    if (m == 0) return hipSuccess;
    hipLaunchKernelGGL(append_kernel, dim3((m + 3) / 4), dim3(256), 0, s, ma, idc, x, ids, assign, slots);
    return hipGetLastError();
}

// probes[:, 0] of a top-1 coarse search -> assignment array (stride nprobe = 1 is the identity;
// kept as a kernel so the copy stays on the stream)
// ------------------------------------------------------------------ delete

// location of position `pos` of list l: arena and row number inside the arena
__device__ __forceinline__ const Arena &locate(const DevIndex &ix, uint32_t l, uint32_t pos, size_t &local)
{
    const uint32_t P = (uint32_t)ix.P, lp = pos / P;
    const uint32_t pg = phys_page(ix, l, lp);
    const Arena &ar = arena_of(ix, pg);
    local = (size_t)(pg - ar.first_page) * P + (pos - lp * P);
    return ar;
}

// Deleting by id (Section 5's interface: delete, and update as delete + insert) in four launches, every
// one of them parallel over what it works on, so that a list of 400 000 rows costs what its share of the
// index's rows costs:
//   prepare  one workgroup: sorts the ids; cuts every list into units of kDeleteUnit rows (prefix sum)
//   find     many workgroups: every row's id is looked up among the sorted ids (held in LDS); the rows
//            to go are noted as (list, position)
//   plan     one workgroup: sorts the noted rows (so a list's rows are neighbours, by position), notes
//            for each where its list's rows start and how long the list was, and shortens the lists
//   move     a list that loses c rows keeps its first len - c positions: the rows to go among them are
//            holes, and as many rows beyond them stay; the i-th row that stays fills the i-th hole.
//            Every move reads and writes rows no other move touches, so they all run at once.
// Lists are unordered sets: no tombstones, nothing for the scan to skip.  The pages a list no longer
// reaches stay its own for later inserts.

__device__ __forceinline__ void sort_keys_lds(unsigned long long *s_keys, int n2)
{
    for (int k = 2; k <= n2; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = threadIdx.x; i < n2; i += blockDim.x) {
                const int p = i ^ j;
                if (p > i) {
                    const unsigned long long a = s_keys[i], b = s_keys[p];
                    if (((i & k) == 0) == (a > b)) {
                        s_keys[i] = b;
                        s_keys[p] = a;
                    }
                }
            }
            __syncthreads();
        }
}

// first index in keys[0, n) whose key is not below `key`
__device__ __forceinline__ uint32_t lower_bound_u64(const unsigned long long *keys, uint32_t n, unsigned long long key)
{
    uint32_t lo = 0, hi = n;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (keys[mid] < key) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

__global__ __launch_bounds__(1024) void delete_prepare_kernel(DeleteArgs a)
{
    __shared__ unsigned long long s_keys[kDeleteChunk];
    __shared__ uint32_t s_wave[17];
    int n2 = 2;
    while (n2 < a.m) n2 <<= 1;
    for (int i = threadIdx.x; i < n2; i += blockDim.x)
        s_keys[i] = i < a.m ? (unsigned long long)a.ids[i] ^ 0x8000000000000000ull : ~0ull; // order of signed values
    __syncthreads();
    sort_keys_lds(s_keys, n2);
    for (int i = threadIdx.x; i < a.m; i += blockDim.x) a.sorted[i] = (int64_t)(s_keys[i] ^ 0x8000000000000000ull);
    const DevIndex &ix = *a.ix;
    for (int l = threadIdx.x; l < a.nlist; l += blockDim.x) a.unit_start[l] = (ix.list_len[l] + kDeleteUnit - 1) / kDeleteUnit;
    __syncthreads();
    const uint32_t units = block_exscan(a.unit_start, a.unit_start, (uint32_t)a.nlist, s_wave);
    if (threadIdx.x == 0) {
        a.unit_start[a.nlist] = units;
        a.scal[0] = 0;
        a.scal[1] = units;
    }
}

__global__ __launch_bounds__(256) void delete_find_kernel(DeleteArgs a)
{
    __shared__ int64_t s_ids[kDeleteChunk];
    const DevIndex &ix = *a.ix;
    for (int i = threadIdx.x; i < a.m; i += blockDim.x) s_ids[i] = a.sorted[i];
    __syncthreads();
    const uint32_t units = a.scal[1];
    for (uint32_t u = blockIdx.x; u < units; u += gridDim.x) {
        uint32_t lo = 0, hi = (uint32_t)a.nlist - 1; // the last list whose units start at or before u
        while (lo < hi) {
            const uint32_t mid = (lo + hi + 1) >> 1;
            if (a.unit_start[mid] <= u) lo = mid;
            else hi = mid - 1;
        }
        const uint32_t l = lo, len = ix.list_len[l];
        const uint32_t base = (u - a.unit_start[l]) * (uint32_t)kDeleteUnit;
#pragma unroll
        for (int j = 0; j < kDeleteUnit / 256; ++j) {
            const uint32_t pos = base + (uint32_t)j * 256u + threadIdx.x;
            if (pos >= len) continue;
            size_t local;
            const Arena &ar = locate(ix, l, pos, local);
            const int64_t id = ar.ids[local];
            int b = 0, e = a.m;
            while (b < e) {
                const int mid = (b + e) >> 1;
                if (s_ids[mid] < id) b = mid + 1;
                else e = mid;
            }
            if (b < a.m && s_ids[b] == id) {
                const uint32_t at = atomicAdd(&a.scal[0], 1u);
                if (at < (uint32_t)kDeleteChunk) a.hits[at] = ((unsigned long long)l << 32) | pos;
            }
        }
    }
}

__global__ __launch_bounds__(1024) void delete_plan_kernel(DeleteArgs a)
{
    __shared__ unsigned long long s_keys[kDeleteChunk];
    const DevIndex &ix = *a.ix;
    const uint32_t found = a.scal[0];
    const uint32_t nh = found < (uint32_t)kDeleteChunk ? found : (uint32_t)kDeleteChunk;
    if (nh == 0) return;
    int n2 = 2;
    while ((uint32_t)n2 < nh) n2 <<= 1;
    for (int i = threadIdx.x; i < n2; i += blockDim.x) s_keys[i] = (uint32_t)i < nh ? a.hits[i] : ~0ull;
    __syncthreads();
    sort_keys_lds(s_keys, n2);
    for (uint32_t g = threadIdx.x; g < nh; g += blockDim.x) {
        const unsigned long long key = s_keys[g];
        const uint32_t l = (uint32_t)(key >> 32);
        const uint32_t seg0 = lower_bound_u64(s_keys, nh, (unsigned long long)l << 32);
        const uint32_t seg1 = lower_bound_u64(s_keys, nh, ((unsigned long long)l + 1ull) << 32);
        a.hits[g] = key;
        a.hit_seg0[g] = seg0;
        a.hit_cnt[g] = seg1 - seg0;
        a.hit_len0[g] = ix.list_len[l];
    }
    __syncthreads(); // every list length has been read (and stored with the hits) before any is changed
    for (uint32_t g = threadIdx.x; g < nh; g += blockDim.x) {
        const uint32_t l = (uint32_t)(s_keys[g] >> 32);
        if (g == 0 || (uint32_t)(s_keys[g - 1] >> 32) != l) {
            const uint32_t seg1 = lower_bound_u64(s_keys, nh, ((unsigned long long)l + 1ull) << 32);
            ix.list_len[l] -= seg1 - g;
        }
    }
    if (threadIdx.x == 0) {
        atomicAdd(a.removed, (unsigned long long)nh);
        if (found > nh) a.scal[2] = 1u;
    }
}

__global__ __launch_bounds__(256) void delete_move_kernel(DeleteArgs a)
{
    __shared__ unsigned long long s_keys[kDeleteChunk];
    __shared__ uint32_t s_list[256], s_src[256], s_dst[256];
    __shared__ uint32_t s_n;
    const DevIndex &ix = *a.ix;
    const uint32_t found = a.scal[0];
    const uint32_t nh = found < (uint32_t)kDeleteChunk ? found : (uint32_t)kDeleteChunk;
    if (blockIdx.x * 256u >= nh) return;
    for (uint32_t i = threadIdx.x; i < nh; i += blockDim.x) s_keys[i] = a.hits[i];
    if (threadIdx.x == 0) s_n = 0;
    __syncthreads();
    const uint32_t g = blockIdx.x * 256u + threadIdx.x;
    if (g < nh) {
        // this thread looks at one position beyond the list's new end: position number t of the c there are
        const uint32_t l = (uint32_t)(s_keys[g] >> 32);
        const uint32_t seg0 = a.hit_seg0[g], c = a.hit_cnt[g], newlen = a.hit_len0[g] - c;
        const unsigned long long *seg = s_keys + seg0;
        const uint32_t t = g - seg0, p = newlen + t;
        const unsigned long long lkey = (unsigned long long)l << 32;
        const uint32_t holes = lower_bound_u64(seg, c, lkey | newlen); // rows to go among the positions that stay
        const uint32_t idx = lower_bound_u64(seg, c, lkey | p);
        if (!(idx < c && seg[idx] == (lkey | p))) {
            // the row stays: it is number t - (rows to go beyond the new end and before it) of those that do
            const uint32_t i = t - (idx - holes);
            const uint32_t at = atomicAdd(&s_n, 1u);
            s_list[at] = l;
            s_src[at] = p;
            s_dst[at] = (uint32_t)seg[i];
        }
    }
    __syncthreads();
    const uint32_t moves = s_n;
    const int row_bytes = ix.row_bytes, lane = threadIdx.x & 63;
    for (uint32_t mv = threadIdx.x >> 6; mv < moves; mv += 4) { // a wave per move
        size_t ls, ld;
        const Arena &as = locate(ix, s_list[mv], s_src[mv], ls);
        const Arena &ad = locate(ix, s_list[mv], s_dst[mv], ld);
        const uint4 *src = reinterpret_cast<const uint4 *>(as.vec + ls * (size_t)row_bytes);
        uint4 *dst = reinterpret_cast<uint4 *>(ad.vec + ld * (size_t)row_bytes);
        for (int i = lane; i < row_bytes / 16; i += 64) dst[i] = src[i];
        if (lane == 0) {
            ad.norm[ld] = as.norm[ls];
            ad.ids[ld] = as.ids[ls];
        }
    }
}

hipError_t launch_delete(const DeleteArgs &a, hipStream_t s)
{
    if (a.m <= 0) return hipSuccess;
    if (a.m > kDeleteChunk || a.nlist < 1 || a.grid < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(delete_prepare_kernel, dim3(1), dim3(1024), 0, s, a);
    hipLaunchKernelGGL(delete_find_kernel, dim3(a.grid), dim3(256), 0, s, a);
    hipLaunchKernelGGL(delete_plan_kernel, dim3(1), dim3(1024), 0, s, a);
    hipLaunchKernelGGL(delete_move_kernel, dim3(kDeleteChunk / 256), dim3(256), 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------ compaction

// One workgroup per page of the new layout: page pg belongs to the list whose new extent
// contains it; its rows, norms and ids are copied from wherever the old layout keeps that
// logical page (build-time extent or delta page, any arena).  Positions inside a list do
// not change.
__global__ __launch_bounds__(256) void compact_pages_kernel(const DevIndex *srcp, const DevIndex *dstp,
                                                            const uint8_t *skip)
{
    __shared__ uint32_t s_list;
    const DevIndex &src = *srcp, &dst = *dstp;
    const uint32_t pg = blockIdx.x;
    if (threadIdx.x == 0) {
        // last list whose extent starts at or before pg (extents are in list order; a list
        // without pages shares its start with the next one and can never be the answer)
        uint32_t lo = 0, hi = (uint32_t)dst.nlist;
        while (hi - lo > 1) {
            const uint32_t mid = (lo + hi) / 2;
            if (dst.main_base[mid] <= pg) lo = mid;
            else hi = mid;
        }
        s_list = lo;
    }
    __syncthreads();
    const uint32_t l = s_list;
    // lists the caller fills itself (split lists and the lists they give rise to)
    if (l >= (uint32_t)src.nlist || (skip && skip[l])) return;
    const uint32_t lp = pg - dst.main_base[l];
    const uint32_t P = (uint32_t)dst.P;
    const uint32_t len = dst.list_len[l];
    if (lp >= dst.main_pages[l] || lp * P >= len) return;
    const uint32_t nrows = len - lp * P < P ? len - lp * P : P;
    const uint32_t opg = phys_page(src, l, lp);
    const Arena &sa = arena_of(src, opg), &da = arena_of(dst, pg);
    const size_t so = opg - sa.first_page, dn = pg - da.first_page;
    const int row_bytes = dst.row_bytes;
    const uint4 *sv = reinterpret_cast<const uint4 *>(sa.vec + so * P * (size_t)row_bytes);
    uint4 *dv = reinterpret_cast<uint4 *>(da.vec + dn * P * (size_t)row_bytes);
    const size_t nvec = (size_t)nrows * row_bytes / 16;
    for (size_t i = threadIdx.x; i < nvec; i += blockDim.x) dv[i] = sv[i];
    for (uint32_t i = threadIdx.x; i < nrows; i += blockDim.x) {
        da.norm[dn * P + i] = sa.norm[so * P + i];
        da.ids[dn * P + i] = sa.ids[so * P + i];
    }
}

hipError_t launch_compact_pages(const DevIndex *src, const DevIndex *dst, uint32_t new_pages, const uint8_t *skip,
                                hipStream_t s)
{
    if (new_pages == 0) return hipSuccess;
    hipLaunchKernelGGL(compact_pages_kernel, dim3(new_pages), dim3(256), 0, s, src, dst, skip);
    return hipGetLastError();
}

// ------------------------------------------------------------------ list read-back and split

// one wave per member of list l: the stored row as fp32 [d] (rows may be NULL) and its id (ids may be NULL)
__global__ __launch_bounds__(256) void gather_list_kernel(const DevIndex *ixp, uint32_t l, uint32_t limit, float *rows,
                                                          int64_t *ids)
{
    const DevIndex &ix = *ixp;
    const uint32_t r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= ix.list_len[l] || r >= limit) return;
    size_t local;
    const Arena &ar = locate(ix, l, r, local);
    const int lane = threadIdx.x & 63;
    if (rows) {
        const char *src = ar.vec + local * (size_t)ix.row_bytes;
        for (int i = lane; i < ix.d; i += 64)
            rows[(size_t)r * ix.d + i] = ix.storage == PK_F16 ? (float)reinterpret_cast<const _Float16 *>(src)[i]
                                                               : reinterpret_cast<const float *>(src)[i];
    }
    if (ids && lane == 0) ids[r] = ar.ids[local];
}

hipError_t launch_gather_list(const DevIndex *ix, uint32_t l, uint32_t len, float *rows, int64_t *ids, hipStream_t s)
{
    if (len == 0) return hipSuccess;
    hipLaunchKernelGGL(gather_list_kernel, dim3((len + 3) / 4), dim3(256), 0, s, ix, l, len, rows, ids);
    return hipGetLastError();
}

// ---- 2-means of the lists to split

// stored row -> element i as fp32
__device__ __forceinline__ float row_element(const char *row, int storage, int i)
{
    return storage == PK_F16 ? (float)reinterpret_cast<const _Float16 *>(row)[i] : reinterpret_cast<const float *>(row)[i];
}

// one workgroup per job: the members with the smallest and the largest id become the first centroids
__global__ __launch_bounds__(1024) void split_init_kernel(SplitArgs a)
{
    __shared__ long long s_id[2][16];
    __shared__ uint32_t s_pos[2][16];
    const DevIndex &ix = *a.ix;
    const uint32_t j = blockIdx.x, l = a.job_list[j], len = a.job_len[j];
    long long lo_id = INT64_MAX, hi_id = INT64_MIN;
    uint32_t lo_pos = 0xffffffffu, hi_pos = 0xffffffffu;
    for (uint32_t r = threadIdx.x; r < len; r += blockDim.x) {
        size_t local;
        const Arena &ar = locate(ix, l, r, local);
        const long long id = ar.ids[local];
        if (id < lo_id || (id == lo_id && r < lo_pos)) {
            lo_id = id;
            lo_pos = r;
        }
        if (id > hi_id || (id == hi_id && r < hi_pos)) {
            hi_id = id;
            hi_pos = r;
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        const long long oi = __shfl_xor(lo_id, off), pi = __shfl_xor(hi_id, off);
        const uint32_t op = __shfl_xor(lo_pos, off), pp = __shfl_xor(hi_pos, off);
        if (oi < lo_id || (oi == lo_id && op < lo_pos)) {
            lo_id = oi;
            lo_pos = op;
        }
        if (pi > hi_id || (pi == hi_id && pp < hi_pos)) {
            hi_id = pi;
            hi_pos = pp;
        }
    }
    if ((threadIdx.x & 63) == 0) {
        s_id[0][threadIdx.x >> 6] = lo_id;
        s_pos[0][threadIdx.x >> 6] = lo_pos;
        s_id[1][threadIdx.x >> 6] = hi_id;
        s_pos[1][threadIdx.x >> 6] = hi_pos;
    }
    __syncthreads();
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) { // every thread folds the waves' results the same way
        if (s_id[0][w] < lo_id || (s_id[0][w] == lo_id && s_pos[0][w] < lo_pos)) {
            lo_id = s_id[0][w];
            lo_pos = s_pos[0][w];
        }
        if (s_id[1][w] > hi_id || (s_id[1][w] == hi_id && s_pos[1][w] < hi_pos)) {
            hi_id = s_id[1][w];
            hi_pos = s_pos[1][w];
        }
    }
    const int d = ix.d;
    for (int side = 0; side < 2; ++side) {
        size_t local;
        const Arena &ar = locate(ix, l, side ? hi_pos : lo_pos, local);
        const char *row = ar.vec + local * (size_t)ix.row_bytes;
        for (int i = threadIdx.x; i < d; i += blockDim.x) {
            a.cent[((size_t)j * 2 + side) * d + i] = (double)row_element(row, ix.storage, i);
            a.sum[((size_t)j * 2 + side) * d + i] = 0.0;
        }
    }
    if (threadIdx.x < 2) a.cnt[(size_t)j * 2 + threadIdx.x] = 0ull;
}

// One workgroup per unit of kSplitUnit members of one job; a wave takes a quarter of them, row by row:
// the lanes share the row's elements, the two squared distances are reduced over the wave (fp32), and the
// row is added to the wave's running sum of its side.  The four waves' sums meet in LDS and go to the
// job's sums as one fp64 atomic per element and unit.
constexpr int kSplitEl = (PK_MAX_DIM + 63) / 64; // elements of a row per lane
__global__ __launch_bounds__(256) void split_assign_kernel(SplitArgs a)
{
    extern __shared__ __align__(16) float s_split[]; // [2][d] centroids, then [4][2][d] the waves' sums
    __shared__ uint32_t s_ones[4];
    const DevIndex &ix = *a.ix;
    const int d = ix.d, storage = ix.storage, row_bytes = ix.row_bytes;
    const uint32_t P = (uint32_t)ix.P;
    uint32_t lo = 0, hi = (uint32_t)a.njobs - 1; // the job this unit belongs to
    while (lo < hi) {
        const uint32_t mid = (lo + hi + 1) >> 1;
        if (a.job_unit0[mid] <= blockIdx.x) lo = mid;
        else hi = mid - 1;
    }
    const uint32_t j = lo, l = a.job_list[j], len = a.job_len[j];
    const uint32_t first = (blockIdx.x - a.job_unit0[j]) * (uint32_t)kSplitUnit;
    float *s_c = s_split, *s_sum = s_split + 2 * d;
    for (int i = threadIdx.x; i < 2 * d; i += blockDim.x) s_c[i] = (float)a.cent[(size_t)j * 2 * d + i];
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float c0[kSplitEl], c1[kSplitEl], acc0[kSplitEl], acc1[kSplitEl];
#pragma unroll
    for (int e = 0; e < kSplitEl; ++e) {
        const int i = lane + 64 * e;
        c0[e] = i < d ? s_c[i] : 0.f;
        c1[e] = i < d ? s_c[d + i] : 0.f;
        acc0[e] = acc1[e] = 0.f;
    }
    uint32_t ones = 0;
    const uint32_t r0 = first + (uint32_t)wave * (kSplitUnit / 4);
    const uint32_t r1 = min(r0 + (uint32_t)(kSplitUnit / 4), len);
    for (uint32_t r = r0; r < r1;) {
        // the rows of one page are neighbours in memory
        const uint32_t lp = r / P, in_page = r - lp * P;
        const uint32_t pg = phys_page(ix, l, lp);
        const Arena &ar = arena_of(ix, pg);
        const char *page = ar.vec + ((size_t)(pg - ar.first_page) * P) * (size_t)row_bytes;
        const uint32_t n = min(P - in_page, r1 - r);
        for (uint32_t t = 0; t < n; ++t) {
            const char *row = page + (size_t)(in_page + t) * row_bytes;
            float x[kSplitEl], s0 = 0.f, s1 = 0.f;
#pragma unroll
            for (int e = 0; e < kSplitEl; ++e) {
                const int i = lane + 64 * e;
                x[e] = i < d ? row_element(row, storage, i) : 0.f;
            }
#pragma unroll
            for (int e = 0; e < kSplitEl; ++e) {
                const float u0 = x[e] - c0[e], u1 = x[e] - c1[e];
                s0 += u0 * u0;
                s1 += u1 * u1;
            }
            for (int off = 32; off > 0; off >>= 1) {
                s0 += __shfl_xor(s0, off);
                s1 += __shfl_xor(s1, off);
            }
            const bool second = s1 < s0; // the same in every lane
            if (second) {
#pragma unroll
                for (int e = 0; e < kSplitEl; ++e) acc1[e] += x[e];
                ++ones;
            } else {
#pragma unroll
                for (int e = 0; e < kSplitEl; ++e) acc0[e] += x[e];
            }
            if (lane == 0) a.side[(size_t)a.job_row0[j] + r + t] = second ? 1 : 0;
        }
        r += n;
    }
#pragma unroll
    for (int e = 0; e < kSplitEl; ++e) {
        const int i = lane + 64 * e;
        if (i < d) {
            s_sum[((size_t)wave * 2 + 0) * d + i] = acc0[e];
            s_sum[((size_t)wave * 2 + 1) * d + i] = acc1[e];
        }
    }
    if (lane == 0) s_ones[wave] = ones;
    __syncthreads();
    for (int i = threadIdx.x; i < 2 * d; i += blockDim.x) {
        const double v = ((double)s_sum[i] + (double)s_sum[2 * d + i]) + ((double)s_sum[4 * d + i] + (double)s_sum[6 * d + i]);
        if (v != 0.0) atomicAdd(&a.sum[(size_t)j * 2 * d + i], v);
    }
    if (threadIdx.x == 0) {
        const uint32_t rows = first < len ? min((uint32_t)kSplitUnit, len - first) : 0u;
        const uint32_t n1 = s_ones[0] + s_ones[1] + s_ones[2] + s_ones[3];
        if (rows - n1) atomicAdd(&a.cnt[(size_t)j * 2], (unsigned long long)(rows - n1));
        if (n1) atomicAdd(&a.cnt[(size_t)j * 2 + 1], (unsigned long long)n1);
    }
}

// one workgroup per job: centroids to the means of their members; sums and counts back to zero
__global__ __launch_bounds__(256) void split_update_kernel(SplitArgs a)
{
    const uint32_t j = blockIdx.x;
    const int d = a.ix->d;
    const unsigned long long n0 = a.cnt[(size_t)j * 2], n1 = a.cnt[(size_t)j * 2 + 1];
    for (int i = threadIdx.x; i < 2 * d; i += blockDim.x) {
        const unsigned long long n = i < d ? n0 : n1;
        const size_t at = (size_t)j * 2 * d + i;
        if (n > 0) a.cent[at] = a.sum[at] / (double)n;
        a.sum[at] = 0.0;
    }
    __syncthreads(); // every thread has read the counts
    if (threadIdx.x < 2) {
        a.cnt_out[(size_t)j * 2 + threadIdx.x] = threadIdx.x ? n1 : n0;
        a.cnt[(size_t)j * 2 + threadIdx.x] = 0ull;
    }
}

__global__ __launch_bounds__(256) void split_centroids_kernel(SplitArgs a, int nlist0, float *dense)
{
    const uint32_t j = blockIdx.x;
    const int d = a.ix->d;
    for (int i = threadIdx.x; i < d; i += blockDim.x) {
        dense[(size_t)a.job_list[j] * d + i] = (float)a.cent[(size_t)j * 2 * d + i];
        dense[(size_t)(nlist0 + j) * d + i] = (float)a.cent[((size_t)j * 2 + 1) * d + i];
    }
}

hipError_t launch_split_init(const SplitArgs &a, hipStream_t s)
{
    if (a.njobs <= 0) return hipSuccess;
    hipLaunchKernelGGL(split_init_kernel, dim3(a.njobs), dim3(1024), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_split_iterate(const SplitArgs &a, uint32_t total_units, int d, hipStream_t s)
{
    if (a.njobs <= 0 || total_units == 0) return hipSuccess;
    if (d > PK_MAX_DIM) return hipErrorInvalidValue;
    const size_t lds = (size_t)10 * d * sizeof(float); // at most 60 KB
    hipLaunchKernelGGL(split_assign_kernel, dim3(total_units), dim3(256), lds, s, a);
    hipLaunchKernelGGL(split_update_kernel, dim3(a.njobs), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_split_centroids(const SplitArgs &a, int nlist0, float *dense, hipStream_t s)
{
    if (a.njobs <= 0) return hipSuccess;
    hipLaunchKernelGGL(split_centroids_kernel, dim3(a.njobs), dim3(256), 0, s, a, nlist0, dense);
    return hipGetLastError();
}

// Stable partition of a list by side[r] in {0, 1}: slot[r] = number of earlier members on the
// same side (one workgroup walks the list)
__global__ __launch_bounds__(1024) void split_slots_kernel(const int32_t *side, uint32_t len, uint32_t *slot)
{
    __shared__ uint32_t s_wave[17];
    __shared__ uint32_t s_in[1024], s_out[1024];
    uint32_t ones = 0;
    for (uint32_t base = 0; base < len; base += 1024) {
        const uint32_t r = base + threadIdx.x;
        const uint32_t b = r < len && side[r] != 0 ? 1u : 0u;
        s_in[threadIdx.x] = b;
        __syncthreads();
        const uint32_t n = len - base < 1024u ? len - base : 1024u;
        const uint32_t total = block_exscan(s_in, s_out, n, s_wave);
        if (r < len) slot[r] = b ? ones + s_out[threadIdx.x] : r - (ones + s_out[threadIdx.x]);
        ones += total;
        __syncthreads();
    }
}

// one wave per member of list l of the old layout: to slot[r] of list l (side 0) or of list lnew (side 1)
// of the new layout, stored bytes, norm and id unchanged
__global__ __launch_bounds__(256) void split_scatter_kernel(const DevIndex *srcp, const DevIndex *dstp, uint32_t l,
                                                            uint32_t lnew, const int32_t *side, const uint32_t *slot,
                                                            uint32_t len)
{
    const DevIndex &src = *srcp, &dst = *dstp;
    const uint32_t r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= len) return;
    size_t ls, ld;
    const Arena &as = locate(src, l, r, ls);
    const Arena &ad = locate(dst, side[r] ? lnew : l, slot[r], ld);
    const int lane = threadIdx.x & 63, row_bytes = src.row_bytes;
    const uint4 *from = reinterpret_cast<const uint4 *>(as.vec + ls * (size_t)row_bytes);
    uint4 *to = reinterpret_cast<uint4 *>(ad.vec + ld * (size_t)row_bytes);
    for (int i = lane; i < row_bytes / 16; i += 64) to[i] = from[i];
    if (lane == 0) {
        ad.norm[ld] = as.norm[ls];
        ad.ids[ld] = as.ids[ls];
    }
}

hipError_t launch_split_list(const DevIndex *src, const DevIndex *dst, uint32_t l, uint32_t lnew, const int32_t *side,
                             uint32_t *slot, uint32_t len, hipStream_t s)
{
    if (len == 0) return hipSuccess;
    hipLaunchKernelGGL(split_slots_kernel, dim3(1), dim3(1024), 0, s, side, len, slot);
    hipLaunchKernelGGL(split_scatter_kernel, dim3((len + 3) / 4), dim3(256), 0, s, src, dst, l, lnew, side, slot, len);
    return hipGetLastError();
}

__global__ void copy_i32_kernel(const int32_t *src, int32_t *dst, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

hipError_t launch_copy_i32(const int32_t *src, int32_t *dst, int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(copy_i32_kernel, dim3((uint32_t)((n + 255) / 256)), dim3(256), 0, s, src, dst, n);
    return hipGetLastError();
}

} // namespace pk
