// Lloyd's update step on the device, for index training (Section 2.2: the clusters of an IVF
// index come from k-means; Section 4.4 / 6.1 "IVF-Split" re-runs a light k-means on the GPU).
// The assignment step is the coarse search with nprobe = 1 under L2 (pk_api.hip); this file
// turns an assignment into new centroids: histogram, exclusive scan, scatter of the row
// numbers into cluster-major order, then the members are summed in fp64, 256 at a time per
// workgroup (thread j owns dimensions j, j + 256, ...; rows are read coalesced; partial sums
// meet by fp64 atomics), and every cluster divides its total.  An empty cluster keeps its
// centroid.  The objective of the assignment comes out of the same sums:
// sum_i |x_i - c|^2 = sum |x_i|^2 - 2 <c, sum x_i> + m |c|^2, in fp64.
#include "pk_internal.h"

namespace pk {

__global__ void km_hist_kernel(KmeansArgs a)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < a.n; i += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t l = (uint32_t)a.assign[i];
        if (l < (uint32_t)a.nlist) atomicAdd(&a.cnt[l], 1u);
    }
}

__global__ __launch_bounds__(1024) void km_offsets_kernel(KmeansArgs a)
{
    __shared__ uint32_t s_wave[17];
    block_exscan(a.cnt, a.start, (uint32_t)a.nlist, s_wave);
}

__global__ void km_scatter_kernel(KmeansArgs a)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < a.n; i += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t l = (uint32_t)a.assign[i];
        if (l < (uint32_t)a.nlist) a.members[a.start[l] + atomicAdd(&a.fill[l], 1u)] = (uint32_t)i;
    }
}

constexpr int kKmDims = (PK_MAX_DIM + 255) / 256; // dimensions per thread
constexpr int kKmChunk = 256;                     // members one workgroup sums

// One workgroup per 256 consecutive entries of the cluster-major member array.  The entries
// of one cluster are a contiguous run; the workgroup sums each run it holds (thread j owns
// dimensions j, j + 256, ...) and adds the run's partial sums to the cluster's totals with
// float64 atomics, so a cluster of any size is summed by as many workgroups as it needs.
__global__ __launch_bounds__(256) void km_accumulate_kernel(KmeansArgs a)
{
    const int64_t first = (int64_t)blockIdx.x * kKmChunk;
    // (entries past the last assigned row belong to no cluster: the walk below runs out of clusters first)
    const int64_t last = first + kKmChunk < a.n ? first + kKmChunk : a.n;
    // cluster of the first entry: the last cluster whose start is <= first
    uint32_t lo = 0, hi = (uint32_t)a.nlist;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) / 2;
        if ((int64_t)a.start[mid] <= first) lo = mid;
        else hi = mid;
    }
    uint32_t l = lo;
    int64_t r = first;
    while (r < last && l < (uint32_t)a.nlist) {
        const int64_t end_l = (int64_t)a.start[l] + a.cnt[l];
        if (r >= end_l) { // empty cluster, or the run ended exactly here
            ++l;
            continue;
        }
        const int64_t stop = end_l < last ? end_l : last;
        double sum[kKmDims], sq = 0.0;
#pragma unroll
        for (int t = 0; t < kKmDims; ++t) sum[t] = 0.0;
        for (int64_t e = r; e < stop; ++e) {
            const float *row = a.x + (size_t)a.members[e] * a.d;
#pragma unroll
            for (int t = 0; t < kKmDims; ++t) {
                const int j = (int)threadIdx.x + 256 * t;
                if (j < a.d) {
                    const double v = (double)row[j];
                    sum[t] += v;
                    sq += v * v;
                }
            }
        }
#pragma unroll
        for (int t = 0; t < kKmDims; ++t) {
            const int j = (int)threadIdx.x + 256 * t;
            if (j < a.d) atomicAdd(&a.sums[(size_t)l * a.d + j], sum[t]);
        }
        for (int off = 32; off > 0; off >>= 1) sq += __shfl_xor(sq, off);
        if ((threadIdx.x & 63) == 0) atomicAdd(&a.sq[l], sq);
        r = stop;
        ++l;
    }
}

// one workgroup per cluster: centroid = total / members (an empty cluster keeps its centroid), and the
// cluster's share of the objective of the assignment
__global__ __launch_bounds__(256) void km_finalize_kernel(KmeansArgs a)
{
    __shared__ double s_part[4];
    const uint32_t l = blockIdx.x;
    const uint32_t m = a.cnt[l];
    if (m == 0) return;
    double obj = 0.0;
    for (int j = threadIdx.x; j < a.d; j += 256) {
        float *c = a.centroids + (size_t)l * a.d + j;
        const double c0 = (double)*c, sj = a.sums[(size_t)l * a.d + j];
        obj += (double)m * c0 * c0 - 2.0 * c0 * sj;
        *c = (float)(sj / (double)m);
    }
    for (int off = 32; off > 0; off >>= 1) obj += __shfl_xor(obj, off);
    if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = obj;
    __syncthreads();
    if (threadIdx.x == 0) atomicAdd(a.inertia, a.sq[l] + (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]));
}

hipError_t launch_kmeans_update(const KmeansArgs &a, hipStream_t s)
{
    if (a.n <= 0 || a.nlist <= 0 || a.d <= 0 || a.d > PK_MAX_DIM) return hipErrorInvalidValue;
    hipError_t e = launch_fill_u32(a.cnt, 0u, (size_t)a.nlist, s);
    if (e != hipSuccess) return e;
    e = launch_fill_u32(a.fill, 0u, (size_t)a.nlist, s);
    if (e != hipSuccess) return e;
    e = launch_fill_u32(reinterpret_cast<uint32_t *>(a.inertia), 0u, 2, s);
    if (e != hipSuccess) return e;
    const int grid = (int)((a.n + 255) / 256 < 4096 ? (a.n + 255) / 256 : 4096);
    hipLaunchKernelGGL(km_hist_kernel, dim3(grid), dim3(256), 0, s, a);
    hipLaunchKernelGGL(km_offsets_kernel, dim3(1), dim3(1024), 0, s, a);
    hipLaunchKernelGGL(km_scatter_kernel, dim3(grid), dim3(256), 0, s, a);
    e = launch_fill_u32(reinterpret_cast<uint32_t *>(a.sums), 0u, (size_t)a.nlist * a.d * 2, s);
    if (e != hipSuccess) return e;
    e = launch_fill_u32(reinterpret_cast<uint32_t *>(a.sq), 0u, (size_t)a.nlist * 2, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(km_accumulate_kernel, dim3((uint32_t)((a.n + kKmChunk - 1) / kKmChunk)), dim3(256), 0, s, a);
    hipLaunchKernelGGL(km_finalize_kernel, dim3(a.nlist), dim3(256), 0, s, a);
    return hipGetLastError();
}

} // namespace pk
