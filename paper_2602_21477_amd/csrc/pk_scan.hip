// List scan (fine search) and centroid scoring (coarse search) for gfx950.
//
// Section 2.2 of the paper: the coarse step scores a query against every centroid, the
// fine step against every vector of the probed clusters.  Both are "rows streamed from
// HBM once, scored against a small group of queries", so one kernel serves both: a tile
// is one page of rows (list page or a slice of the centroid table) plus a group of up to
// MQ query slots.  Inserted vectors (Section 4.4's buffer) live in ordinary pages of the
// list and are scored by the same tiles.
//
// Mapping to CDNA4.  The rows are the streaming operand and go HBM -> registers directly
// in MFMA operand layout; the query group is staged once in LDS and re-read per pass.
// With A = queries (M = 16 slots) and B = rows (N = 16 rows) the 16x16 accumulator puts
// rows along lanes, so each store instruction writes 64 contiguous bytes per 16 lanes.
// The contraction index may be permuted freely as long as A and B use the same
// permutation, which lets every lane fetch 16 contiguous bytes per load (4 lanes cover a
// 64-byte segment of one row, 16 rows per instruction) and feed them straight into
// v_mfma_f32_16x16x32_f16 (fp16 storage) or four v_mfma_f32_16x16x4_f32 (fp32 storage),
// always with fp32 accumulation.
#include "pk_internal.h"

namespace pk {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// per-slot LDS arrays of the scan kernel: out, qn, thr, q, base, lo, inv, bmax
constexpr int kScanSlotWords = 8;

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

// MT = query tiles of 16 slots held in LDS (MQ = 16*MT); WAVES = waves per workgroup;
// GATED = emit only values that pass the per-query threshold (fine search) instead of
// writing every value (coarse search, threshold sampling).
template <int STORAGE, int MT, int WAVES, bool GATED>
__global__ __launch_bounds__(WAVES * 64) void scan_kernel(ScanArgs a)
{
    extern __shared__ __align__(16) char smem[];
    constexpr int MQ = MT * 16;
    const int row_bytes = a.row_bytes;
    const int qstride = row_bytes + kQPadBytes;
    char *qtile = smem;
    uint32_t *s_out = reinterpret_cast<uint32_t *>(smem + (size_t)MQ * qstride);
    float *s_qn = reinterpret_cast<float *>(s_out + MQ);
    uint32_t *s_thr = reinterpret_cast<uint32_t *>(s_qn + MQ); // gated: threshold key per slot
    uint32_t *s_q = s_thr + MQ;                                 // gated: query of the slot
    uint32_t *s_base = s_q + MQ;                                // gated: start of the query's region
    float *s_lo = reinterpret_cast<float *>(s_base + MQ);       // gated: origin of the bucket scale
    float *s_inv = s_lo + MQ;                                   // gated: bucket scale
    uint32_t *s_bmax = reinterpret_cast<uint32_t *>(s_inv + MQ);// gated: buckets above this are cut
    uint32_t *s_misc = s_bmax + MQ; // kScanSlotWords per-slot arrays precede this: keep scan_lds_bytes in step

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 15, lg = lane >> 4;
    const uint32_t ntiles = *a.ntiles;
    const uint32_t grab = *a.batch;
    const int nit = row_bytes / kIterBytes;
    const int chunks_per_row = row_bytes / 16;
    const float worst = a.metric == PK_METRIC_IP ? -INFINITY : INFINITY;
    uint32_t cur_qbeg = 0xffffffffu, cur_qcnt = 0;

    // Schedule: the first batch of every workgroup is fixed (tile b for workgroup b), later
    // batches of `grab` tiles are handed out by a counter, so uneven tiles (hot lists scored
    // against many query groups) still balance while the launch does not start with a burst
    // of atomics.  The first batch is a single tile so that the emission thresholds get
    // their first refresh early.  Every workgroup leaves the loop the first time it is handed
    // a batch past the end.
    uint32_t t0 = blockIdx.x, t1 = min(t0 + 1u, ntiles);
    for (;;) {
        if (t0 >= ntiles) break;
        for (uint32_t t = t0; t < t1; ++t) {
            const Tile *tp = a.tiles + t;
            const char *tx = tp->x;
            const float *txn = tp->xn;
            const uint32_t row0 = tp->row0;
            const uint32_t qbeg = __builtin_amdgcn_readfirstlane(tp->qbeg);
            const uint32_t qcnt = __builtin_amdgcn_readfirstlane((uint32_t)tp->qcnt);
            const int nrows = __builtin_amdgcn_readfirstlane((int)tp->nrows);
            if (qbeg != cur_qbeg || qcnt != cur_qcnt) {
                __syncthreads(); // everyone is done with the previous query group
                const int mrows = (int)((qcnt + 15u) & ~15u);
                for (int idx = tid; idx < mrows * chunks_per_row; idx += WAVES * 64) {
                    const int m = idx / chunks_per_row, c = idx - m * chunks_per_row;
                    u32x4 v = {0u, 0u, 0u, 0u};
                    if ((uint32_t)m < qcnt)
                        v = *reinterpret_cast<const u32x4 *>(a.qs + (size_t)a.slot_query[qbeg + m] * row_bytes +
                                                             (size_t)c * 16);
                    *reinterpret_cast<u32x4 *>(qtile + (size_t)m * qstride + (size_t)c * 16) = v;
                }
                if (tid < MQ) {
                    const bool on = (uint32_t)tid < qcnt;
                    const uint32_t q = on ? a.slot_query[qbeg + tid] : 0u;
                    s_out[tid] = on ? a.slot_out[qbeg + tid] : 0u;
                    s_qn[tid] = on ? a.qnorm[q] : 0.f;
                    if constexpr (GATED) {
                        const uint32_t base = on ? a.qoff[q] : 0u;
                        s_q[tid] = q;
                        s_base[tid] = base;
                        s_out[tid] -= base; // position inside the query's candidate range
                        // Emission gate of the slot: a fixed key threshold from the query's
                        // sample, and a bucket limit that tightens while the scan runs: the
                        // histogram counts the emitted candidates per bucket, and the first
                        // bucket at which the running count reaches k bounds the k-th best.
                        uint32_t bmax = (uint32_t)kHistBins - 1u;
                        if (on && a.use_hist) {
                            const uint32_t *hp = a.hist + (size_t)q * kHistBins;
                            uint32_t h[kHistBins];
#pragma unroll
                            for (int j = 0; j < kHistBins; ++j) // device-scope loads: counts other CUs just added
                                h[j] = __hip_atomic_load(hp + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            uint32_t cum = 0;
                            bool found = false;
#pragma unroll
                            for (int j = 0; j < kHistBins; ++j) {
                                cum += h[j];
                                if (!found && cum >= (uint32_t)a.k) {
                                    found = true;
                                    bmax = (uint32_t)j;
                                }
                            }
                            // share the limit with every workgroup scoring this query
                            const uint32_t seen = atomicMin(a.tcur + q, bmax);
                            bmax = seen < bmax ? seen : bmax;
                        }
                        s_thr[tid] = on ? a.tau[q] : 0u;
                        s_lo[tid] = on ? a.tlo[q] : 0.f;
                        s_inv[tid] = on ? a.tinv[q] : 0.f;
                        s_bmax[tid] = bmax;
                    }
                }
                __syncthreads();
                cur_qbeg = qbeg;
                cur_qcnt = qcnt;
            }
            else if (GATED && a.use_hist == 1) {
                // same query group as the previous tile: pick up thresholds others have tightened
                if ((uint32_t)tid < qcnt) {
                    const uint32_t seen = __hip_atomic_load(a.tcur + s_q[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (seen < s_bmax[tid]) s_bmax[tid] = seen;
                }
                __syncthreads();
            }
            const int mt_used = (int)((qcnt + 15u) >> 4);
            const int nrows_pad = (nrows + 15) & ~15;

            for (int rb = wave; rb * kRowBlock < nrows; rb += WAVES) {
                const int row_a = rb * kRowBlock + ln;
                const char *p0 = tx + (size_t)row_a * row_bytes + lg * 16;
                const char *p1 = p0 + (size_t)16 * row_bytes;
                f32x4 acc[MT][2];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    acc[mt][0] = f32x4{0.f, 0.f, 0.f, 0.f};
                    acc[mt][1] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
                u32x4 xa[2][4], xb[2][4]; // two register buffers of one iteration each
                const char *qbase = qtile + (size_t)ln * qstride + lg * 16;

#define PK_LOAD(buf, it)                                                                          \
    _Pragma("unroll") for (int s = 0; s < 4; ++s)                                                 \
    {                                                                                             \
        buf[0][s] = *reinterpret_cast<const u32x4 *>(p0 + (size_t)(it) * kIterBytes + s * 64);    \
        buf[1][s] = *reinterpret_cast<const u32x4 *>(p1 + (size_t)(it) * kIterBytes + s * 64);    \
    }
#define PK_COMPUTE(buf, it)                                                                       \
    _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)                                             \
    {                                                                                             \
        if (mt < mt_used) {                                                                       \
            const char *qrow = qbase + (size_t)mt * 16 * qstride + (size_t)(it) * kIterBytes;     \
            _Pragma("unroll") for (int s = 0; s < 4; ++s)                                         \
            {                                                                                     \
                const u32x4 qa = *reinterpret_cast<const u32x4 *>(qrow + s * 64);                 \
                mfma_step<STORAGE>(acc[mt][0], qa, buf[0][s]);                                    \
                mfma_step<STORAGE>(acc[mt][1], qa, buf[1][s]);                                    \
            }                                                                                     \
        }                                                                                         \
    }
                PK_LOAD(xa, 0)
                for (int it = 0; it < nit; it += 2) {
                    if (it + 1 < nit) { PK_LOAD(xb, it + 1) }
                    PK_COMPUTE(xa, it)
                    if (it + 2 < nit) { PK_LOAD(xa, it + 2) }
                    if (it + 1 < nit) { PK_COMPUTE(xb, it + 1) }
                }
#undef PK_LOAD
#undef PK_COMPUTE

                // epilogue: lane holds row (rb*32 + nt*16 + ln) for slots mt*16 + lg*4 + i
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) {
                    const int row = rb * kRowBlock + nt * 16 + ln;
                    const bool live = row < nrows;
                    float xn = 0.f;
                    if (a.metric == PK_METRIC_L2 && live) xn = txn[row];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int m = mt * 16 + lg * 4 + i;
                            float v = acc[mt][nt][i];
                            if (a.metric == PK_METRIC_L2) v = fmaxf(xn - 2.f * v + s_qn[m & (MQ - 1)], 0.f);
                            if constexpr (!GATED) {
                                if ((uint32_t)m < qcnt && row < nrows_pad)
                                    a.out[(size_t)s_out[m] + row0 + row] = live ? v : worst;
                            } else {
                                // The 16 lanes of a group share slot m.  Values that pass the
                                // query's threshold are rare: one ballot, and only then one
                                // aggregated atomic per group to reserve room in the query's region.
                                const uint32_t bits = order_bits(v, a.metric);
                                bool pass = live && (uint32_t)m < qcnt && bits <= s_thr[m];
                                if (__ballot(pass) == 0ull) continue; // the usual case: nothing survives
                                uint32_t b = 0;
                                if (pass) {
                                    b = bucket_of(v, s_lo[m], s_inv[m], a.metric);
                                    pass = b <= s_bmax[m];
                                }
                                const unsigned long long mask = __ballot(pass);
                                const uint32_t gmask = (uint32_t)(mask >> (lg * 16)) & 0xffffu;
                                if (gmask) {
                                    const int leader = __ffs(gmask) - 1;
                                    uint32_t base = 0;
                                    if (ln == leader) base = atomicAdd(&a.ccnt[s_q[m]], (uint32_t)__popc(gmask));
                                    base = __shfl(base, lg * 16 + leader);
                                    if (pass) {
                                        const uint32_t rank = __popc(gmask & ((1u << ln) - 1u));
                                        a.cbuf[(size_t)s_base[m] + base + rank] =
                                            ((unsigned long long)bits << 32) | (s_out[m] + row0 + (uint32_t)row);
                                    }
                                    if (a.use_hist) {
                                        // count the emitted candidates per bucket; one atomic for the
                                        // group when its candidates share a bucket (the usual case)
                                        const uint32_t b0 = __shfl(b, lg * 16 + leader);
                                        const uint32_t odd =
                                            (uint32_t)(__ballot(pass && b != b0) >> (lg * 16)) & 0xffffu;
                                        uint32_t *hq = a.hist + (size_t)s_q[m] * kHistBins;
                                        if (odd == 0u) {
                                            if (ln == leader) atomicAdd(hq + b0, (uint32_t)__popc(gmask));
                                        } else if (pass) {
                                            atomicAdd(hq + b, 1u);
                                        }
                                    }
                                }
                            }
                        }
                    }
                }
            }
        }
        __syncthreads();
        if (tid == 0) s_misc[0] = gridDim.x + atomicAdd(a.tile_ctr, 1u) * grab;
        __syncthreads();
        t0 = s_misc[0];
        t1 = min(t0 + grab, ntiles);
    }
}

int scan_lds_bytes(int row_bytes, int mq)
{
    return mq * (row_bytes + kQPadBytes) + mq * kScanSlotWords * 4 + 16; // query tile + per-slot arrays + scratch
}

// Largest query group (16, 32 or 64 slots) whose LDS tile fits.  fp32 storage is held to
// 32 slots: beyond that the fp32 MFMA rate, not HBM, would bound the scan.  Returns 0 when
// even 16 slots do not fit.
int scan_max_mq(int row_bytes, int storage, int lds_limit)
{
    const int budget = lds_limit < 100 * 1024 ? lds_limit : 100 * 1024;
    const int cap = storage == PK_F16 ? 64 : 32;
    int best = 0;
    for (int mq = 16; mq <= cap; mq *= 2)
        if (scan_lds_bytes(row_bytes, mq) <= budget) best = mq;
    return best;
}

template <int STORAGE, int MT, int WAVES, bool GATED>
static hipError_t launch_one(const ScanArgs &a, int grid, hipStream_t s)
{
    const int lds = scan_lds_bytes(a.row_bytes, MT * 16);
    static int attr_bytes = 0; // per instantiation: dynamic LDS size the kernel is cleared for
    if (lds > attr_bytes) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&scan_kernel<STORAGE, MT, WAVES, GATED>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        attr_bytes = lds;
    }
    hipLaunchKernelGGL((scan_kernel<STORAGE, MT, WAVES, GATED>), dim3(grid), dim3(WAVES * 64), lds, s, a);
    return hipGetLastError();
}

template <int STORAGE, int WAVES, bool GATED>
static hipError_t launch_mt(const ScanArgs &a, int grid, hipStream_t s)
{
    switch (a.mq) {
    case 16: return launch_one<STORAGE, 1, WAVES, GATED>(a, grid, s);
    case 32: return launch_one<STORAGE, 2, WAVES, GATED>(a, grid, s);
    case 64: return launch_one<STORAGE, 4, WAVES, GATED>(a, grid, s);
    default: return hipErrorInvalidValue;
    }
}

// waves_per_wg: 4 for list pages, 1 for the narrow tiles of the coarse and sampling passes
hipError_t launch_scan(const ScanArgs &a, int waves_per_wg, int grid, hipStream_t s)
{
    if (a.row_bytes <= 0 || a.row_bytes % kIterBytes != 0) return hipErrorInvalidValue;
    const bool gated = a.tau != nullptr;
    if (gated && waves_per_wg != 4) return hipErrorInvalidValue;
    if (a.storage == PK_F16) {
        if (gated) return launch_mt<PK_F16, 4, true>(a, grid, s);
        return waves_per_wg == 1 ? launch_mt<PK_F16, 1, false>(a, grid, s) : launch_mt<PK_F16, 4, false>(a, grid, s);
    }
    if (gated) return launch_mt<PK_F32, 4, true>(a, grid, s);
    return waves_per_wg == 1 ? launch_mt<PK_F32, 1, false>(a, grid, s) : launch_mt<PK_F32, 4, false>(a, grid, s);
}

} // namespace pk
