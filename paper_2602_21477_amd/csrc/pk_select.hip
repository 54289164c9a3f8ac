// Top-k selection for gfx950: best `nprobe` centroids per query (Section 2.2, coarse
// search) and best `k` vectors per query
// over the scored candidates of all probed lists, i.e. the merge of the per-list partial
// results (Section 4.4: partial results are merged into the final result).
//
// A candidate is one 64-bit key: the value mapped to an unsigned integer whose ascending
// order is best-first (high word) and the candidate's position inside the query's
// candidate range (low word).  Keys are unique, so "smaller key" is a strict total order
// and the selection is deterministic.  A workgroup streams candidates, keeps those that
// beat the current K-th key in an LDS buffer, and re-sorts the buffer (bitonic network)
// only when it runs full, so almost all candidates cost one compare.
#include <algorithm>
#include <type_traits>

#include "pk_internal.h"
PK_DEV_MARKS(sel)
#define PK_WL_MARK(i) PK_MARK(sel, i)
#include "pk_worklist_dev.h"
#include "pk_select_dev.h"

namespace pk {

typedef unsigned long long u64;
typedef unsigned long long u64x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t next_pow2(uint32_t n)
{
    uint32_t p = 2;
    while (p < n) p <<= 1;
    return p;
}

// ascending bitonic sort of keys[0, np2), np2 a power of two; all threads of the block call it
__device__ void bitonic_sort(u64 *keys, uint32_t np2)
{
    for (uint32_t size = 2; size <= np2; size <<= 1) {
        for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
            for (uint32_t i = threadIdx.x; i < (np2 >> 1); i += blockDim.x) {
                const uint32_t lo = 2 * i - (i & (stride - 1));
                const uint32_t hi = lo + stride;
                const bool up = (lo & size) == 0;
                const u64 x = keys[lo], y = keys[hi];
                if ((x > y) == up) {
                    keys[lo] = y;
                    keys[hi] = x;
                }
            }
            __syncthreads();
        }
    }
}

// Streaming selector state.  keys: LDS [cap]; cnt: LDS counter.
struct Selector {
    u64 *keys;
    uint32_t *cnt;
    int K;
    uint32_t cap; // entries of keys (a power of two >= 512)
    u64 thr;

    __device__ void init(u64 *k, uint32_t *c, int kk, uint32_t capacity = (uint32_t)kSelCap)
    {
        keys = k;
        cnt = c;
        K = kk;
        cap = capacity;
        thr = kMaxKey;
        if (threadIdx.x == 0) *cnt = 0;
        __syncthreads();
    }
    // sort what is buffered, keep the best K, tighten the threshold (block-wide)
    __device__ void flush()
    {
        __syncthreads();
        const uint32_t n = *cnt;
        const uint32_t np2 = next_pow2(n);
        for (uint32_t i = n + threadIdx.x; i < np2; i += blockDim.x) keys[i] = kMaxKey;
        __syncthreads();
        bitonic_sort(keys, np2);
        const uint32_t kept = n < (uint32_t)K ? n : (uint32_t)K;
        thr = kept == (uint32_t)K ? keys[K - 1] : kMaxKey;
        __syncthreads();
        if (threadIdx.x == 0) *cnt = kept;
        __syncthreads();
    }
    // make room for one round of at most `room` pushes (block-wide)
    __device__ void reserve(uint32_t room)
    {
        __syncthreads();
        const uint32_t n = *cnt; // read by everyone before anyone pushes again
        __syncthreads();
        // flush threshold: the smallest power of two that holds the kept keys plus one round
        // (small rounds and small K sort small buffers)
        uint32_t limit = next_pow2((uint32_t)K + room);
        limit = limit < 512u ? 512u : (limit > cap ? cap : limit);
        if (n + room > limit) flush();
    }
    __device__ __forceinline__ void push(u64 key)
    {
        if (key < thr) keys[atomicAdd(cnt, 1u)] = key;
    }
};

__global__ __launch_bounds__(kSelThreads) void select_partial_kernel(SelectArgs a)
{
    __shared__ u64 keys[kSelCap];
    __shared__ uint32_t s_cnt;
    const uint32_t q = blockIdx.y, c = blockIdx.x;
    const uint32_t base = a.qoff[q];
    const uint32_t total = a.qcnt[q];
    const uint32_t beg = c * (uint32_t)a.chunk;
    const uint32_t end = min(beg + (uint32_t)a.chunk, total);
    // nothing in this chunk; and a query whose emitted keys fit one chunk is merged directly
    // by the final kernel
    if (beg >= total || (!a.vals && total <= (uint32_t)a.chunk)) return;
    u64 *out = a.partial + ((size_t)q * a.nchunks + c) * a.K;

    Selector sel;
    sel.init(keys, &s_cnt, a.K);
    constexpr uint32_t kRound = kSelThreads * kSelVec;
    if (a.vals) {
        const float *v = a.vals + base;
        for (uint32_t r = beg; r < end; r += kRound) {
            sel.reserve(kRound);
            const uint32_t p = r + threadIdx.x * kSelVec;
            if (p < end) {
                const f32x4 x = *reinterpret_cast<const f32x4 *>(v + p);
#pragma unroll
                for (int j = 0; j < kSelVec; ++j)
                    if (p + j < end) sel.push(((u64)order_bits(x[j], a.metric) << 32) | (p + j));
            }
        }
    } else {
        // keys were emitted under a threshold that tightened over time, so the latest are
        // the best: reading the range backwards sets a tight selection threshold at once
        const u64 *v = a.keys + base;
        for (uint32_t r = end; r > beg;) {
            const uint32_t lo = r - beg > kRound ? r - kRound : beg;
            sel.reserve(kRound);
            const uint32_t p = lo + threadIdx.x * kSelVec;
#pragma unroll
            for (int j = 0; j < kSelVec; ++j)
                if (p + j < r) sel.push(v[p + j]);
            r = lo;
        }
    }
    sel.flush();
    const uint32_t n = s_cnt;
    for (uint32_t i = threadIdx.x; i < (uint32_t)a.K; i += blockDim.x) out[i] = i < n ? keys[i] : kMaxKey;
}

// merge `nchunks` sorted partial lists of one query; leaves the best K sorted in keys[], returns count
__device__ uint32_t merge_partials(Selector &sel, const u64 *part, int nchunks, int K)
{
    const uint32_t total = (uint32_t)nchunks * (uint32_t)K;
    for (uint32_t r = 0; r < total; r += kSelThreads) {
        sel.reserve(kSelThreads);
        const uint32_t p = r + threadIdx.x;
        if (p < total) {
            const u64 key = part[p];
            if (key != kMaxKey) sel.push(key);
        }
    }
    sel.flush();
    return *sel.cnt;
}

__global__ __launch_bounds__(kSelThreads) void select_probes_kernel(const u64 *partial, int nchunks, int K, int nprobe,
                                                                    int32_t *probes)
{
    __shared__ u64 keys[kSelCap];
    __shared__ uint32_t s_cnt;
    const uint32_t q = blockIdx.x;
    Selector sel;
    sel.init(keys, &s_cnt, K);
    merge_partials(sel, partial + (size_t)q * nchunks * K, nchunks, K);
    for (int r = threadIdx.x; r < nprobe; r += blockDim.x) probes[(size_t)q * nprobe + r] = (int32_t)(uint32_t)keys[r];
}


// ---------------------------------------------------------------- dense rows (coarse search)

// Best K of a row of n <= 256 * VPT scores (Section 2.2: the top-nprobe clusters), for the
// coarse step and for the top-1 assignment of inserts and the build.  Every thread keeps
// VPT keys in registers; the exact K-th smallest key is found digit by digit (four 8-bit
// radix passes over a 256-bin LDS histogram), then the keys below it and as many of the keys
// equal to it as are needed, lowest positions first, are collected and sorted.  Positions
// are list numbers, so ties go to the lower list number.
// COUNT: the workgroup goes on to do its query's share of the work-list construction (pairs per list,
// candidate layout, sample tiles), which saves the launch that would otherwise follow the selection.
template <int VPT, bool COUNT>
__global__ __launch_bounds__(256) void select_dense_kernel(const float *vals, const uint32_t *qoff, const uint32_t *qcnt,
                                                           int metric, int K, int32_t *probes, WorklistArgs wa,
                                                           SampleArgs sm, MultiArgs ma)
{
    __shared__ __align__(16) uint32_t hist[4][256]; // one histogram per radix pass: zeroed once
    __shared__ uint32_t s_w[4];
    __shared__ uint32_t s_n;
    __shared__ __align__(16) u64 sel[PK_MAX_NPROBE + 2];
    __shared__ int32_t s_probe[COUNT ? PK_MAX_NPROBE : 1];
    __shared__ std::conditional_t<COUNT, WlCountLds, uint32_t> s_wl;
    PK_MARK(sel, 0);
    const uint32_t q = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t n = qcnt[q];
    const float *v = vals + qoff[q];
    WlIndexView view{};
    if constexpr (COUNT) view = wl_index_view(wa, ma, q); // these loads are over by the time the count needs them
    uint32_t key[VPT];
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
        const uint32_t p = tid + 256u * j;
        key[j] = p < n ? order_bits(v[p], metric) : 0xffffffffu;
    }
    if (tid == 0) s_n = 0;
    bool live[VPT];
#pragma unroll
    for (int j = 0; j < VPT; ++j) live[j] = tid + 256u * j < n;
    PK_MARK(sel, 1);
    uint32_t krem, ties;
    const uint32_t prefix = radix_kth<VPT>(key, live, (uint32_t)K, hist, krem, ties);
    PK_MARK(sel, 2);
    // prefix is the K-th smallest key; krem of the `ties` keys equal to it are needed
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
        const uint32_t p = tid + 256u * j;
        if (p < n && (key[j] < prefix || (key[j] == prefix && ties == krem)))
            sel[atomicAdd(&s_n, 1u)] = ((u64)key[j] << 32) | p;
    }
    if (ties != krem) { // more equal keys than needed: take them in position order
        uint32_t taken = 0;
        for (int j = 0; j < VPT && taken < krem; ++j) { // position = tid + 256 j: ascending in j, then tid
            const uint32_t p = tid + 256u * j;
            const bool tie = p < n && key[j] == prefix;
            const unsigned long long m = __ballot(tie);
            if (lane == 0) s_w[wave] = (uint32_t)__popcll(m);
            __syncthreads();
            uint32_t rank = taken + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            for (uint32_t w = 0; w < wave; ++w) rank += s_w[w];
            const uint32_t total = s_w[0] + s_w[1] + s_w[2] + s_w[3];
            if (tie && rank < krem) sel[atomicAdd(&s_n, 1u)] = ((u64)prefix << 32) | p;
            taken += total;
            __syncthreads();
        }
    }
    if (tid < 2) sel[K + tid] = kMaxKey; // padding: the rank count reads pairs
    __syncthreads();
    PK_MARK(sel, 3);
    if (K <= 256) {
        // rank of each selected key among the K of them (keys are unique): its place in the probe list
        if (tid < (uint32_t)K) {
            const u64 mine = sel[tid];
            uint32_t rank = 0;
            for (int o = 0; o < K; o += 2) {
                const u64x2 w = *reinterpret_cast<const u64x2 *>(sel + o);
                rank += (w[0] < mine ? 1u : 0u) + (w[1] < mine ? 1u : 0u);
            }
            if constexpr (COUNT) s_probe[rank] = (int32_t)(uint32_t)mine; // the count stores the list, after its loads
            else probes[(size_t)q * K + rank] = (int32_t)(uint32_t)mine;
        }
    } else {
        const uint32_t np2 = next_pow2((uint32_t)K);
        for (uint32_t i = (uint32_t)K + tid; i < np2; i += 256) sel[i] = kMaxKey;
        __syncthreads();
        bitonic_sort(sel, np2);
        for (uint32_t r = tid; r < (uint32_t)K; r += 256) {
            if constexpr (COUNT) s_probe[r] = (int32_t)(uint32_t)sel[r];
            else probes[(size_t)q * K + r] = (int32_t)(uint32_t)sel[r];
        }
    }
    PK_MARK(sel, 4);
    if constexpr (COUNT) {
        __syncthreads(); // the probe list is in s_probe
        wl_count_query(wa, sm, ma, q, s_wl, s_probe, probes + (size_t)q * K, view);
        PK_MARK(sel, 7);
    }
}

hipError_t launch_select_dense(const float *vals, const uint32_t *qoff, const uint32_t *qcnt, uint32_t max_cnt, int metric,
                               int K, int64_t nq, int32_t *probes, hipStream_t s, const WorklistArgs *wa, const SampleArgs *sm,
                               const MultiArgs *ma)
{
    if (nq <= 0) return hipSuccess;
    if (max_cnt > (uint32_t)kDenseSelectMax || K > PK_MAX_NPROBE) return hipErrorInvalidValue;
    const dim3 g((uint32_t)nq), b(256);
    if (wa) {
        if (!sm || !ma || wa->nprobe != K) return hipErrorInvalidValue;
        if (max_cnt <= 1024)
            hipLaunchKernelGGL((select_dense_kernel<4, true>), g, b, 0, s, vals, qoff, qcnt, metric, K, probes, *wa, *sm, *ma);
        else if (max_cnt <= 4096)
            hipLaunchKernelGGL((select_dense_kernel<16, true>), g, b, 0, s, vals, qoff, qcnt, metric, K, probes, *wa, *sm, *ma);
        else
            hipLaunchKernelGGL((select_dense_kernel<32, true>), g, b, 0, s, vals, qoff, qcnt, metric, K, probes, *wa, *sm, *ma);
        return hipGetLastError();
    }
    const WorklistArgs w0{};
    const SampleArgs s0{};
    MultiArgs m0;
    m0.n = 0;
    if (max_cnt <= 1024)
        hipLaunchKernelGGL((select_dense_kernel<4, false>), g, b, 0, s, vals, qoff, qcnt, metric, K, probes, w0, s0, m0);
    else if (max_cnt <= 4096)
        hipLaunchKernelGGL((select_dense_kernel<16, false>), g, b, 0, s, vals, qoff, qcnt, metric, K, probes, w0, s0, m0);
    else
        hipLaunchKernelGGL((select_dense_kernel<32, false>), g, b, 0, s, vals, qoff, qcnt, metric, K, probes, w0, s0, m0);
    return hipGetLastError();
}

// position inside the query's candidate range -> id stored in the list page
__device__ int64_t resolve_id(const FinalArgs &a, const MultiArgs &h, uint32_t q, uint32_t pos)
{
    const uint32_t *po = a.pair_off + (size_t)q * (a.nprobe + 1);
    int lo = 0, hi = a.nprobe - 1;
    while (lo < hi) { // largest r with po[r] <= pos
        const int mid = (lo + hi + 1) >> 1;
        if (po[mid] <= pos) lo = mid;
        else hi = mid - 1;
    }
    const uint32_t row = pos - po[lo];
    const uint32_t list = (uint32_t)a.probes[(size_t)q * a.nprobe + lo];
    const DevIndex &ix = *h.ix[a.qagent[q]];
    const uint32_t lp = row / (uint32_t)ix.P;
    const uint32_t pg = phys_page(ix, list, lp);
    const Arena &ar = arena_of(ix, pg);
    return ar.ids[(size_t)(pg - ar.first_page) * ix.P + (row - lp * ix.P)];
}


// the same with the query's rows of pair_off and probes in LDS
__device__ int64_t resolve_id_lds(const FinalArgs &a, const DevIndex &ix, uint32_t pos, const uint32_t *po, const uint32_t *pr)
{
    int lo = 0, hi = a.nprobe - 1;
    while (lo < hi) { // largest r with po[r] <= pos
        const int mid = (lo + hi + 1) >> 1;
        if (po[mid] <= pos) lo = mid;
        else hi = mid - 1;
    }
    const uint32_t row = pos - po[lo];
    const uint32_t list = pr[lo];
    const uint32_t lp = row / (uint32_t)ix.P;
    const uint32_t pg = phys_page(ix, list, lp);
    const Arena &ar = arena_of(ix, pg);
    return ar.ids[(size_t)(pg - ar.first_page) * ix.P + (row - lp * ix.P)];
}

// buffer of the final selection: K kept keys plus the largest round pushed at once, as a power of two
static uint32_t final_cap(int K)
{
    uint32_t c = 512;
    while (c < (uint32_t)K + (uint32_t)(kSelThreads * kSelVec) && c < (uint32_t)kSelCap) c <<= 1;
    return c;
}

// Exact pass over every row the query probes, for a query whose emission region overflowed
// (more candidates passed the gate than the region holds: no usable threshold, or a tie group
// larger than the region).  One workgroup walks the probed lists page by page; each wave
// scores 32 rows against the one query with the MFMA sequence of the scan kernels (the query
// in MFMA row 0, zeros in the other rows), so the values are bit-identical to the scan's.
//   by_id false: every value goes to the selector as (value key, position)  -> best K
//   by_id true:  the ids of the rows whose value key equals `tau` go to the selector
//                (lowest ids of a tie group; several rows may carry one id)
// s_q: LDS, the query row then a row of zeros, qstride bytes apart.
template <int STORAGE>
__device__ void rescore_query(const FinalArgs &a, const MultiArgs &h, uint32_t q, const char *s_q, int qstride,
                              Selector &sel, bool by_id, uint32_t tau)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ln = lane & 15, lg = lane >> 4;
    const DevIndex &ix = *h.ix[a.qagent[q]];
    const int row_bytes = a.row_bytes, nit = row_bytes / kIterBytes;
    const uint32_t P = (uint32_t)ix.P;
    const float qn = a.qnorm[q];
    const uint32_t *po = a.pair_off + (size_t)q * (a.nprobe + 1);
    const char *qbase = s_q + (size_t)(ln == 0 ? 0 : 1) * qstride + lg * 16;
    for (int r = 0; r < a.nprobe; ++r) {
        const uint32_t l = (uint32_t)a.probes[(size_t)q * a.nprobe + r];
        if (l >= (uint32_t)ix.nlist) continue;
        const uint32_t len = ix.list_len[l];
        for (uint32_t lp = 0; lp * P < len; ++lp) {
            const uint32_t pg = phys_page(ix, l, lp);
            const Arena &ar = arena_of(ix, pg);
            const size_t local = (size_t)(pg - ar.first_page) * P;
            const gbytes px = in_global(ar.vec + local * (size_t)row_bytes);
            const uint32_t nrows = len - lp * P < P ? len - lp * P : P;
            for (uint32_t rb0 = 0; rb0 < nrows; rb0 += 4 * kRowBlock) {
                sel.reserve(4 * kRowBlock);
                const uint32_t rb = rb0 + (uint32_t)wave * kRowBlock;
                if (rb >= nrows) continue; // the next reserve() is a barrier every wave reaches
                // rows rb .. rb + 31 lie inside the page (its size is a multiple of 32); those past
                // nrows hold stale bytes and their values are not used
                const gbytes p0 = px + (size_t)(rb + ln) * row_bytes + lg * 16;
                const gbytes p1 = p0 + (size_t)16 * row_bytes;
                f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
                for (int it = 0; it < nit; ++it) {
#pragma unroll
                    for (int s4 = 0; s4 < 4; ++s4) {
                        const u32x4 qa = *reinterpret_cast<const u32x4 *>(qbase + (size_t)it * kIterBytes + s4 * 64);
                        const u32x4 x0 = *reinterpret_cast<gvec4>(p0 + (size_t)it * kIterBytes + s4 * 64);
                        const u32x4 x1 = *reinterpret_cast<gvec4>(p1 + (size_t)it * kIterBytes + s4 * 64);
                        mfma_step<STORAGE>(acc0, qa, x0);
                        mfma_step<STORAGE>(acc1, qa, x1);
                    }
                }
                if (lg == 0) { // accumulator element 0 of lanes 0..15: MFMA row 0 (the query) x column ln (the row)
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt) {
                        const uint32_t row = rb + (uint32_t)nt * 16u + (uint32_t)ln;
                        if (row >= nrows) continue;
                        float v = nt == 0 ? acc0[0] : acc1[0];
                        if (a.metric == PK_METRIC_L2) v = l2_from_dot(ar.norm[local + row], v, qn);
                        const uint32_t bits = order_bits(v, a.metric);
                        if (!by_id) {
                            sel.push(((u64)bits << 32) | (po[r] + lp * P + row));
                        } else if (bits == tau) {
                            sel.push((u64)ar.ids[local + row] ^ 0x8000000000000000ull); // order of signed ids
                        }
                    }
                }
            }
        }
    }
}

// Best K of the cnt_q <= 256 * VPT keys of a query's region, held in registers: the K-th smallest value by
// radix selection; among the keys with that value, if not all of them are needed, the lowest positions by a
// second selection over the low words.  The kept keys end up sorted in keys[0, min(K, cnt_q)); *s_cnt is
// their number.  early: key number threadIdx.x of the region, already loaded.  hist: LDS [4][256].
template <int VPT>
__device__ __forceinline__ void final_by_radix(const u64 *v, uint32_t cnt_q, uint32_t K, u64 early, uint32_t (*hist)[256],
                                               u64 *keys, uint32_t *s_cnt)
{
    const uint32_t tid = threadIdx.x;
    u64 k64[VPT];
    uint32_t hi[VPT];
    bool live[VPT];
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
        const uint32_t p = tid + (uint32_t)kSelThreads * j;
        live[j] = p < cnt_q;
        k64[j] = live[j] ? (j == 0 ? early : v[p]) : kMaxKey;
        hi[j] = (uint32_t)(k64[j] >> 32);
    }
    if (tid == 0) *s_cnt = 0;
    uint32_t prefix = 0xffffffffu, lo_max = 0xffffffffu; // everything is kept
    if (cnt_q > K) {
        uint32_t left, ties;
        prefix = radix_kth<VPT>(hi, live, K, hist, left, ties);
        if (ties != left) { // block-uniform: only the `left` lowest positions of the boundary value are kept
            uint32_t lo[VPT];
            bool tl[VPT];
#pragma unroll
            for (int j = 0; j < VPT; ++j) {
                lo[j] = (uint32_t)k64[j];
                tl[j] = live[j] && hi[j] == prefix;
            }
            __syncthreads(); // the histograms are read no more
            uint32_t l2, t2;
            lo_max = radix_kth<VPT>(lo, tl, left, hist, l2, t2);
        }
    } else {
        __syncthreads();
    }
#pragma unroll
    for (int j = 0; j < VPT; ++j)
        if (live[j] && (hi[j] < prefix || (hi[j] == prefix && (uint32_t)k64[j] <= lo_max))) keys[atomicAdd(s_cnt, 1u)] = k64[j];
    __syncthreads();
    const uint32_t n = *s_cnt;
    if (n <= (uint32_t)kSelThreads) {
        // order by counting: the rank of a key is the number of smaller ones (keys are unique)
        if (tid < 2) keys[n + tid] = kMaxKey; // padding: the keys are read in pairs
        __syncthreads();
        const u64 mine = tid < n ? keys[tid] : kMaxKey;
        uint32_t rank = 0;
        if (tid < n)
            for (uint32_t o = 0; o < n; o += 2) {
                const u64x2 w = *reinterpret_cast<const u64x2 *>(keys + o);
                rank += (w[0] < mine ? 1u : 0u) + (w[1] < mine ? 1u : 0u);
            }
        __syncthreads();
        if (tid < n) keys[rank] = mine;
        __syncthreads();
    } else {
        const uint32_t np2 = next_pow2(n);
        for (uint32_t i = n + tid; i < np2; i += blockDim.x) keys[i] = kMaxKey;
        __syncthreads();
        bitonic_sort(keys, np2);
    }
}

__global__ __launch_bounds__(kSelThreads) void select_final_kernel(FinalArgs a, MultiArgs h, uint32_t cap, uint32_t qbytes)
{
    // LDS sized by K, not by the largest K the library takes: small k leaves room for every
    // query's workgroup to be resident at once
    extern __shared__ __align__(16) unsigned char s_dyn[];
    u64 *keys = reinterpret_cast<u64 *>(s_dyn);                  // [cap]
    int64_t *s_id = reinterpret_cast<int64_t *>(keys + cap);     // [k]
    // [2][row_bytes + kQPadBytes] when rescoring; the histograms of the radix selection otherwise
    char *s_q = reinterpret_cast<char *>(s_id + ((a.k + 1) & ~1));
    uint32_t *s_po = reinterpret_cast<uint32_t *>(s_q + qbytes); // [nprobe + 1] the query's row of pair_off
    uint32_t *s_pr = s_po + a.nprobe + 1;                        // [nprobe] its probe list
    __shared__ uint32_t s_cnt;
    __shared__ long long s_red[kSelThreads / 64];
    __shared__ uint32_t s_redpos[kSelThreads / 64];
    __shared__ long long s_pick;
    __shared__ uint32_t s_pickpos;
    const uint32_t q = blockIdx.x;
    const int k = a.k;
    const int qstride = a.row_bytes + kQPadBytes;
    PK_MARK(sel, 32);
    const size_t region = (size_t)q * a.ecap;
    // everything the usual path reads from global memory is requested at once: the count, the thread's key
    // of a short region (the entry exists whatever the count; it is used only if it is below it), the
    // query's rows of the candidate layout, its index
    const uint32_t cnt_q = a.qcnt[q];
    const u64 early = threadIdx.x < a.ecap ? a.keys[region + threadIdx.x] : kMaxKey;
    for (int r = threadIdx.x; r <= a.nprobe; r += blockDim.x) {
        s_po[r] = a.pair_off[(size_t)q * (a.nprobe + 1) + r];
        if (r < a.nprobe) s_pr[r] = (uint32_t)a.probes[(size_t)q * a.nprobe + r];
    }
    const DevIndex &qix = *h.ix[a.qagent[q]];
    // Running sums of the call (candidates met, candidates emitted, most emitted by one query, queries whose
    // region overflowed): workgroup 0 adds up every query's numbers, so that they cost four atomics per call
    // and not several per query on the same words.
    unsigned long long st_cand = 0, st_emit = 0;
    uint32_t st_max = 0, st_over = 0;
    if (blockIdx.x == 0) {
        for (uint32_t t = threadIdx.x; t < gridDim.x; t += blockDim.x) {
            const uint32_t c = a.qcnt[t];
            st_cand += a.pair_off[(size_t)t * (a.nprobe + 1) + a.nprobe];
            st_emit += c;
            st_max = c > st_max ? c : st_max;
            st_over += c > a.ecap ? 1u : 0u;
        }
    }
    Selector sel;
    sel.init(keys, &s_cnt, a.K, cap);
    const bool overflow = cnt_q > a.ecap; // the region lost candidates: select by rescoring the query's rows
    const bool in_registers = cnt_q <= 16u * kSelThreads && !overflow;
    if (in_registers) {
        uint32_t(*hist)[256] = reinterpret_cast<uint32_t(*)[256]>(s_q);
        const u64 *v = a.keys + region;
        if (cnt_q <= (uint32_t)kSelThreads) final_by_radix<1>(v, cnt_q, (uint32_t)a.K, early, hist, keys, &s_cnt);
        else if (cnt_q <= 4u * kSelThreads) final_by_radix<4>(v, cnt_q, (uint32_t)a.K, early, hist, keys, &s_cnt);
        else final_by_radix<16>(v, cnt_q, (uint32_t)a.K, early, hist, keys, &s_cnt);
    } else if (!overflow) {
        const u64 *v = a.keys + region;
        // short ranges go one key per thread and round, so the buffer that gets sorted stays small
        const uint32_t per = cnt_q <= 8192u ? 1u : (uint32_t)kSelVec;
        const uint32_t round = kSelThreads * per;
        // keys were emitted under a gate that tightened over time, so the latest are the best:
        // reading the region backwards sets a tight selection threshold at once
        for (uint32_t r = cnt_q; r > 0;) {
            const uint32_t lo = r > round ? r - round : 0u;
            sel.reserve(round);
            const uint32_t p = lo + threadIdx.x * per;
            for (uint32_t j = 0; j < per; ++j)
                if (p + j < r) sel.push(v[p + j]);
            r = lo;
        }
    } else {
        // the query row (its padding zeroed), then a row of zeros
        for (int i = threadIdx.x; i < 2 * qstride / 16; i += blockDim.x) {
            u32x4 w = {0u, 0u, 0u, 0u};
            if (i < a.row_bytes / 16) w = *reinterpret_cast<const u32x4 *>(a.qs + (size_t)q * a.row_bytes + (size_t)i * 16);
            *reinterpret_cast<u32x4 *>(s_q + (size_t)i * 16) = w;
        }
        __syncthreads();
        if (a.storage == PK_F16) rescore_query<PK_F16>(a, h, q, s_q, qstride, sel, false, 0u);
        else rescore_query<PK_F32>(a, h, q, s_q, qstride, sel, false, 0u);
    }
    PK_MARK(sel, 33);
    if (!in_registers) sel.flush();
    const uint32_t n = s_cnt;

    // entries carrying the padding value are not candidates
    const uint32_t worst = kWorstBits;
    uint32_t n_valid = 0;
    for (uint32_t i = 0; i < n; ++i) { // n <= K, uniform loop
        if ((uint32_t)(keys[i] >> 32) >= worst) break;
        ++n_valid;
    }
    const uint32_t kk = n_valid < (uint32_t)k ? n_valid : (uint32_t)k;
    for (uint32_t i = threadIdx.x; i < kk; i += blockDim.x) s_id[i] = resolve_id_lds(a, qix, (uint32_t)keys[i], s_po, s_pr);
    __syncthreads();
    PK_MARK(sel, 34);

    // Equal values must come in ascending id order.  If the tie group of the k-th value
    // reaches past position k, its members inside the top k are the lowest ids of the
    // whole group, which may include candidates the selection above did not keep: look again.
    if (n_valid > (uint32_t)k && (uint32_t)(keys[k - 1] >> 32) == (uint32_t)(keys[k] >> 32)) {
        const uint32_t tau = (uint32_t)(keys[k - 1] >> 32);
        uint32_t nb = 0;
        while (nb < (uint32_t)k && (uint32_t)(keys[nb] >> 32) < tau) ++nb;
        if (overflow) {
            // the kept keys better than the tie value wait in the query's (unusable) region while
            // the selector collects the lowest ids of the tie group
            u64 *spill = a.spill + region;
            __syncthreads();
            for (uint32_t i = threadIdx.x; i < nb; i += blockDim.x) spill[i] = keys[i];
            __syncthreads();
            sel.init(keys, &s_cnt, (int)((uint32_t)k - nb), cap);
            if (a.storage == PK_F16) rescore_query<PK_F16>(a, h, q, s_q, qstride, sel, true, tau);
            else rescore_query<PK_F32>(a, h, q, s_q, qstride, sel, true, tau);
            sel.flush();
            for (uint32_t t = nb + threadIdx.x; t < (uint32_t)k; t += blockDim.x)
                s_id[t] = (int64_t)(keys[t - nb] ^ 0x8000000000000000ull);
            __syncthreads();
            for (uint32_t t = threadIdx.x; t < (uint32_t)k; t += blockDim.x)
                keys[t] = t < nb ? spill[t] : (((u64)tau << 32) | t); // the low word is no longer used
            __syncthreads();
        } else {
        const uint32_t total = cnt_q;
        const u64 *rk = a.keys + region;
        // Members are taken in (id, position) order: several rows may carry one id, and each
        // of them is a candidate of its own.
        long long last_id = 0;
        uint32_t last_pos = 0;
        bool have_last = false;
        for (uint32_t t = nb; t < (uint32_t)k; ++t) {
            long long best = INT64_MAX;
            uint32_t best_pos = 0xffffffffu;
            for (uint32_t p = threadIdx.x; p < total; p += blockDim.x) {
                const u64 key = rk[p];
                if ((uint32_t)(key >> 32) == tau) {
                    const uint32_t pos = (uint32_t)key;
                    const long long id = resolve_id(a, h, q, pos);
                    const bool after = !have_last || id > last_id || (id == last_id && pos > last_pos);
                    if (after && (id < best || (id == best && pos < best_pos))) {
                        best = id;
                        best_pos = pos;
                    }
                }
            }
            for (int off = 32; off > 0; off >>= 1) {
                const long long o = __shfl_xor(best, off);
                const uint32_t op = __shfl_xor(best_pos, off);
                if (o < best || (o == best && op < best_pos)) {
                    best = o;
                    best_pos = op;
                }
            }
            if ((threadIdx.x & 63) == 0) {
                s_red[threadIdx.x >> 6] = best;
                s_redpos[threadIdx.x >> 6] = best_pos;
            }
            __syncthreads();
            if (threadIdx.x == 0) {
                long long b = s_red[0];
                uint32_t bp = s_redpos[0];
                for (int w = 1; w < kSelThreads / 64; ++w)
                    if (s_red[w] < b || (s_red[w] == b && s_redpos[w] < bp)) {
                        b = s_red[w];
                        bp = s_redpos[w];
                    }
                s_pick = b;
                s_pickpos = bp;
                s_id[t] = b;
                keys[t] = ((u64)tau << 32) | (uint32_t)t; // keeps the value; the low word is no longer used
            }
            __syncthreads();
            last_id = s_pick;
            last_pos = s_pickpos;
            have_last = true;
            __syncthreads();
        }
        }
    }

    PK_MARK(sel, 35);
    // final order: (value key, id) ascending; rows that carry the same id with the same value
    // keep their order in keys[], so ranks are unique
    for (uint32_t i = threadIdx.x; i < (uint32_t)k; i += blockDim.x) {
        if (i < kk) {
            const uint32_t ki = (uint32_t)(keys[i] >> 32);
            const int64_t idi = s_id[i];
            uint32_t rank = 0;
            for (uint32_t j = 0; j < kk; ++j) {
                const uint32_t kj = (uint32_t)(keys[j] >> 32);
                rank += (kj < ki || (kj == ki && (s_id[j] < idi || (s_id[j] == idi && j < i)))) ? 1u : 0u;
            }
            a.out_ids[(size_t)q * k + rank] = idi;
            a.out_dist[(size_t)q * k + rank] = value_of(ki, a.metric);
        } else {
            a.out_ids[(size_t)q * k + i] = -1;
            a.out_dist[(size_t)q * k + i] = a.metric == PK_METRIC_IP ? -INFINITY : INFINITY;
        }
    }
    if (blockIdx.x == 0) { // last: no load above queues behind these atomics
        for (int off = 32; off > 0; off >>= 1) {
            st_cand += __shfl_xor(st_cand, off);
            st_emit += __shfl_xor(st_emit, off);
            const uint32_t o = __shfl_xor(st_max, off);
            st_max = o > st_max ? o : st_max;
            st_over += __shfl_xor(st_over, off);
        }
        __syncthreads(); // keys[] is no longer read
        if ((threadIdx.x & 63) == 0) {
            u64 *w = keys + 4 * (threadIdx.x >> 6);
            w[0] = st_cand;
            w[1] = st_emit;
            w[2] = st_max;
            w[3] = st_over;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            u64 cand = 0, emit = 0, mx = 0, over = 0;
            for (int w = 0; w < kSelThreads / 64; ++w) {
                cand += keys[4 * w];
                emit += keys[4 * w + 1];
                mx = keys[4 * w + 2] > mx ? keys[4 * w + 2] : mx;
                over += keys[4 * w + 3];
            }
            unsigned long long *st = h.ix[0]->stats;
            atomicAdd(&st[1], cand);
            atomicAdd(&st[3], emit);
            if (over) atomicAdd(&st[4], over);
            atomicMax(&st[5], mx);
        }
    }
}

// k-th best of each query's sample -> threshold key; fewer than k real samples: no threshold.  For samples
// scored by a launch of their own (large batches; small ones usually take sample_tau_kernel instead).
// WL: the workgroups then lay out the second half of the work list between them (offsets, slots, tiles:
// small batches whose samples are too long for the one-launch form), so that no launch of its own is
// needed for it.
template <bool WL>
__global__ __launch_bounds__(kSelThreads) void tau_kernel(SampleArgs a, WorklistArgs wa, MultiArgs ma)
{
    __shared__ __align__(16) u64 keys[kSelCap];
    __shared__ uint32_t s_cnt;
    __shared__ uint32_t s_wave[17];
    const uint32_t q = blockIdx.x;
    PK_MARK(sel, 16);
    WlPrefetch pre;
    auto read_ahead = [&]() {
        if constexpr (WL) wl_spread_prefetch(wa, ma, q, pre); // in flight while the threshold is worked out
    };
    const float *v = a.vals + (size_t)q * a.span;
    uint32_t cnt = 0;                      // real samples (or k, if there are more)
    uint32_t first = 0, kth = 0, last = 0; // value keys: best, k-th best, worst real sample
    uint32_t(*hist)[256] = reinterpret_cast<uint32_t(*)[256]>(keys);
    if (a.span <= 4u * kSelThreads) {
        tau_by_radix<4>(a, v, hist, s_wave, cnt, first, kth, last, read_ahead);
    } else if (a.span <= 16u * kSelThreads) {
        tau_by_radix<16>(a, v, hist, s_wave, cnt, first, kth, last, read_ahead);
    } else {
        read_ahead();
        Selector sel;
        sel.init(keys, &s_cnt, a.k);
        constexpr uint32_t kRound = kSelThreads * kSelVec;
        for (uint32_t r = 0; r < a.span; r += kRound) {
            sel.reserve(kRound);
            const uint32_t p = r + threadIdx.x * kSelVec;
            if (p < a.span) {
                const f32x4 x = *reinterpret_cast<const f32x4 *>(v + p);
#pragma unroll
                for (int j = 0; j < kSelVec; ++j) {
                    const uint32_t b = order_bits(x[j], a.metric);
                    if (b < kWorstBits) sel.push(((u64)b << 32) | (p + j));
                }
            }
        }
        sel.flush();
        cnt = s_cnt; // at most k are kept
        if (cnt > 0) {
            first = (uint32_t)(keys[0] >> 32);
            last = (uint32_t)(keys[cnt - 1] >> 32);
            kth = last;
        }
    }
    PK_MARK(sel, 18);
    if constexpr (WL) {
        __syncthreads(); // the key buffer is free
        wl_spread(wa, ma, reinterpret_cast<uint32_t *>(keys), s_wave, q, pre);
        PK_MARK(sel, 24);
    }
    // the kernel's own results last: no load above queues behind these stores
    tau_publish(a, q, cnt, first, kth, last);
}

hipError_t launch_tau(const SampleArgs &a, hipStream_t s, const WorklistArgs *wa, const MultiArgs *ma)
{
    if (a.nq <= 0) return hipSuccess;
    if (a.span % 4 != 0) return hipErrorInvalidValue;
    if (wa) {
        static_assert(2 * kSelCap >= 3 * ((int)kWlSmallLists + 1), "the work-list layout borrows the key buffer");
        static_assert(kSelThreads * 8 >= (int)kWlSmallLists, "one round of the list scan covers every list");
        if (!ma || (uint64_t)wa->n_handles * (uint64_t)wa->nlist_max > kWlSmallLists) return hipErrorInvalidValue;
        hipLaunchKernelGGL(tau_kernel<true>, dim3((uint32_t)a.nq), dim3(kSelThreads), 0, s, a, *wa, *ma);
        return hipGetLastError();
    }
    MultiArgs m0;
    m0.n = 0;
    hipLaunchKernelGGL(tau_kernel<false>, dim3((uint32_t)a.nq), dim3(kSelThreads), 0, s, a, WorklistArgs{}, m0);
    return hipGetLastError();
}

hipError_t launch_select_partial(const SelectArgs &a, int64_t nq, hipStream_t s)
{
    if (nq <= 0) return hipSuccess;
    hipLaunchKernelGGL(select_partial_kernel, dim3(a.nchunks, (uint32_t)nq), dim3(kSelThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_select_probes(const unsigned long long *partial, int nchunks, int K, int nprobe, int64_t nq,
                                int32_t *probes, hipStream_t s)
{
    if (nq <= 0) return hipSuccess;
    hipLaunchKernelGGL(select_probes_kernel, dim3((uint32_t)nq), dim3(kSelThreads), 0, s, partial, nchunks, K, nprobe,
                       probes);
    return hipGetLastError();
}

hipError_t launch_select_final(const FinalArgs &a, const MultiArgs &h, int64_t nq, hipStream_t s)
{
    if (nq <= 0) return hipSuccess;
    if (a.row_bytes <= 0 || a.row_bytes % kIterBytes != 0 || a.ecap < (uint32_t)a.K) return hipErrorInvalidValue;
    const uint32_t cap = final_cap(a.K);
    // keys, ids, and the query row + a row of zeros for a query that has to be rescored
    const size_t qbytes = std::max((size_t)2 * (a.row_bytes + kQPadBytes), (size_t)4 * 256 * sizeof(uint32_t));
    // ..., and the query's rows of the candidate layout
    const size_t lds = (size_t)cap * sizeof(u64) + (size_t)((a.k + 1) & ~1) * sizeof(int64_t) + qbytes +
                       (size_t)(2 * a.nprobe + 1) * sizeof(uint32_t);
    hipLaunchKernelGGL(select_final_kernel, dim3((uint32_t)nq), dim3(kSelThreads), lds, s, a, h, cap, (uint32_t)qbytes);
    return hipGetLastError();
}

// ------------------------------------------------------------------ scope union

// Merge of the per-handle results of one query (Section 3.2: a request searches the memories
// of a set of agents and merges what each returns).  Every handle's row is already sorted
// (value, id); a candidate's key is (value key, position of the handle in the scope, rank
// inside that handle's row), so equal values come out by handle, then by id.
__global__ __launch_bounds__(kSelThreads) void union_merge_kernel(UnionArgs a)
{
    __shared__ u64 keys[kSelCap];
    __shared__ uint32_t s_cnt;
    const size_t q = blockIdx.x;
    const uint32_t k = (uint32_t)a.k, total = (uint32_t)a.n_handles * k;
    Selector sel;
    sel.init(keys, &s_cnt, a.k);
    for (uint32_t base = 0; base < total; base += kSelThreads) {
        sel.reserve(kSelThreads);
        const uint32_t i = base + threadIdx.x;
        if (i < total) {
            const uint32_t h = i / k, j = i - h * k;
            const size_t at = ((size_t)h * a.nq + q) * k + j;
            if (a.ids[at] >= 0) sel.push(((u64)order_bits(a.dist[at], a.metric) << 32) | (u64)(h << 10 | j));
        }
    }
    sel.flush();
    const uint32_t n = s_cnt;
    for (uint32_t j = threadIdx.x; j < k; j += kSelThreads) {
        const size_t o = q * k + j;
        if (j < n) {
            const uint32_t lo = (uint32_t)keys[j];
            const uint32_t h = (lo >> 10) & 0x7fu, r = lo & 0x3ffu;
            const size_t at = ((size_t)h * a.nq + q) * k + r;
            a.out_src[o] = (int32_t)h;
            a.out_ids[o] = a.ids[at];
            a.out_dist[o] = a.dist[at];
        } else {
            a.out_src[o] = -1;
            a.out_ids[o] = -1;
            a.out_dist[o] = a.metric == PK_METRIC_IP ? -INFINITY : INFINITY;
        }
    }
}

hipError_t launch_union_merge(const UnionArgs &a, hipStream_t s)
{
    if (a.nq <= 0) return hipSuccess;
    if (a.k < 1 || a.k > PK_MAX_K || a.n_handles < 1 || a.n_handles > PK_MAX_HANDLES) return hipErrorInvalidValue;
    hipLaunchKernelGGL(union_merge_kernel, dim3((uint32_t)a.nq), dim3(kSelThreads), 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------ level cascade

// Section 4.2, early termination: one wave per query.  An open query takes this level's row;
// it ends here if the row holds k candidates and the k-th (the farthest of a row sorted best
// first) beats the query's threshold, or if this is the last level.
__global__ __launch_bounds__(256) void level_accept_kernel(LevelArgs a)
{
    const int64_t q = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (q >= a.nq) return;
    if (!a.first && a.open[q] == 0u) return;
    const size_t row = (size_t)q * a.k;
    if (a.row_ids) {
        for (int j = lane; j < a.k; j += 64) {
            a.out_ids[row + j] = a.row_ids[row + j];
            a.out_dist[row + j] = a.row_dist[row + j];
        }
    }
    if (lane == 0) {
        const int64_t *ids = a.row_ids ? a.row_ids : a.out_ids;
        const float *dist = a.row_ids ? a.row_dist : a.out_dist;
        const bool full = ids[row + a.k - 1] >= 0;
        const float kth = dist[row + a.k - 1], t = a.stop[q];
        const bool beats = a.metric == PK_METRIC_IP ? kth > t : kth < t;
        const bool done = a.last || (full && beats);
        a.open[q] = done ? 0u : 1u;
        if (a.level_out && (done || a.first)) a.level_out[q] = a.level;
    }
}

hipError_t launch_level_accept(const LevelArgs &a, hipStream_t s)
{
    if (a.nq <= 0) return hipSuccess;
    hipLaunchKernelGGL(level_accept_kernel, dim3((uint32_t)((a.nq + 3) / 4)), dim3(256), 0, s, a);
    return hipGetLastError();
}

__global__ void level_mask_kernel(int32_t *probes, int nprobe, const uint32_t *open, int64_t nq)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nq * nprobe) return;
    if (open[i / nprobe] == 0u) probes[i] = -1;
}

hipError_t launch_level_mask(int32_t *probes, int nprobe, const uint32_t *open, int64_t nq, hipStream_t s)
{
    if (nq <= 0) return hipSuccess;
    const int64_t n = nq * nprobe;
    hipLaunchKernelGGL(level_mask_kernel, dim3((uint32_t)((n + 255) / 256)), dim3(256), 0, s, probes, nprobe, open, nq);
    return hipGetLastError();
}

} // namespace pk
