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
#include "pk_worklist_dev.h"

namespace pk {

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

// per query: pairs per list, candidate layout, tiles of the threshold sample
__global__ __launch_bounds__(256) void wl_count_kernel(WorklistArgs a, SampleArgs sm, MultiArgs m)
{
    __shared__ WlCountLds s;
    wl_count_query(a, sm, m, blockIdx.x, s, a.probes + (size_t)blockIdx.x * a.nprobe, nullptr, wl_index_view(a, m, blockIdx.x));
}

// one workgroup: offsets of the lists' slot ranges and tile ranges
__global__ __launch_bounds__(1024) void wl_scan_kernel(WorklistArgs a, MultiArgs m)
{
    __shared__ uint32_t s_wave[17];
    wl_scan_body(a, m, s_wave);
}

// Slots and tiles both need only the offsets wl_scan wrote, not each other: one launch, the
// first slot_blocks workgroups place the pairs (one thread per pair), the others write one
// list's tiles each.
__global__ __launch_bounds__(256) void wl_slots_tiles_kernel(WorklistArgs a, MultiArgs m, uint32_t slot_blocks)
{
    if (blockIdx.x < slot_blocks) {
        const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
        if (i < (size_t)a.nq * a.nprobe) wl_slot_of_pair(a, m, i, a.lstart);
    } else {
        wl_tiles_of_list(a, m, blockIdx.x - slot_blocks);
    }
}


// first half of the work list: pairs per list and the candidate layout of every query, and the
// tiles of the threshold sample (which the caller scores next)
hipError_t launch_worklist_count(const WorklistArgs &a, const SampleArgs &sm, const MultiArgs &m, hipStream_t s)
{
    if (!a.lcnt_cleared) {
        // the pair counters and, behind them, the fill marks
        const hipError_t e = launch_fill_u32(a.lcnt, 0u, (size_t)2 * (size_t)a.n_handles * (size_t)a.nlist_max, s);
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
