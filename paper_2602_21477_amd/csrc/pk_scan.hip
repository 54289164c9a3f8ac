// List scan (fine search) and small-batch centroid scoring (coarse search) for gfx950.
//
// Section 2.2 of the paper: the coarse step scores a query against every centroid, the
// fine step against every vector of the probed clusters.  The fine step is "rows streamed
// from HBM once, scored against a small group of queries": a tile is one page of a list
// plus a group of query slots.  Inserted vectors (Section 4.4's buffer) live in ordinary
// pages of the list and are scored by the same tiles.
//
// Mapping to CDNA4.  The rows are the streaming operand and go HBM -> registers directly
// in MFMA operand layout; the queries come from LDS.  With A = queries (M = 16 slots) and
// B = rows (N = 16 rows) the 16x16 accumulator puts rows along lanes, so each store
// instruction writes 64 contiguous bytes per 16 lanes.  The contraction index may be
// permuted freely as long as A and B use the same permutation, which lets every lane fetch
// 16 contiguous bytes per load (4 lanes cover a 64-byte segment of one row, 16 rows per
// instruction) and feed them straight into v_mfma_f32_16x16x32_f16 (fp16 storage) or four
// v_mfma_f32_16x16x4_f32 (fp32 storage), always with fp32 accumulation.
//
// Two list-scan kernels differ in how the queries reach LDS:
//   scan_kernel     the whole query group (up to 64 slots x full rows) sits in LDS and is
//                   reused over a batch of tiles: least traffic when groups are small;
//   scan_ks_kernel  the queries are staged 256 bytes of every row at a time (double
//                   buffered), so LDS use is independent of the row length and up to 128
//                   slots fit: for lists probed by many queries of the batch and for rows
//                   too wide for the first kernel to keep several workgroups per CU.
// sample_tau_kernel is scan_kernel's one-query form for the threshold sample of a small batch,
// with the thresholds and the work-list layout in the same launch (Section 3.3: small
// batches are bound by launches).
// centroid_scores_kernel is the coarse step for small query segments (the same operand
// layout, no LDS staging); large segments go through the GEMM in pk_gemm.hip.
#include <algorithm>

#include "pk_internal.h"
PK_DEV_MARKS(scan)
#define PK_WL_MARK(i) PK_MARK(scan, i)
#include "pk_select_dev.h"
#include "pk_worklist_dev.h"

namespace pk {

// per-slot LDS arrays of the scan kernels: out, qn, thr, q, base, lo, inv, bmax
constexpr int kScanSlotWords = 8;
constexpr int kKsStride = kIterBytes + kQPadBytes; // LDS bytes per slot and staged slice

// What a workgroup knows about the query slots of the group it is scoring (all in LDS).
struct Slots {
    uint32_t *out;  // dense: first output element of the (slot, list) pair; gated: its position in the query's range
    float *qn;      // squared norm of the query
    uint32_t *thr;  // gated: key threshold from the query's sample
    uint32_t *q;    // gated: query of the slot
    uint32_t *base; // gated: start of the query's emission region
    float *lo;      // gated: origin of the bucket scale
    float *inv;     // gated: bucket scale
    uint32_t *bmax; // gated: buckets above this are cut
    __device__ __forceinline__ void carve(char *p, int mq)
    {
        out = reinterpret_cast<uint32_t *>(p);
        qn = reinterpret_cast<float *>(out + mq);
        thr = reinterpret_cast<uint32_t *>(qn + mq);
        q = thr + mq;
        base = q + mq;
        lo = reinterpret_cast<float *>(base + mq);
        inv = lo + mq;
        bmax = reinterpret_cast<uint32_t *>(inv + mq);
    }
};

// Fills the per-slot arrays of the group [qbeg, qbeg + qcnt); every thread of the workgroup
// calls it.  Dense kernels: thread m fills slot m.  Gated kernels (256 threads): 256 / MQ
// neighbouring lanes share a slot and split its 64 histogram counters between them.
template <int MQ, bool GATED>
__device__ __forceinline__ void load_slots(const ScanArgs &a, const Slots &s, int tid, uint32_t qbeg, uint32_t qcnt)
{
    if constexpr (!GATED) {
        if (tid < MQ) {
            const bool on = (uint32_t)tid < qcnt;
            s.out[tid] = on ? a.slot_out[qbeg + tid] : 0u;
            s.qn[tid] = on ? a.qnorm[a.slot_query[qbeg + tid]] : 0.f;
        }
    } else {
        constexpr int TPS = 256 / MQ;       // threads per slot
        constexpr int NB = kHistBins / TPS; // counters per thread
        const int m = tid / TPS, sub = tid % TPS;
        const bool on = (uint32_t)m < qcnt;
        const uint32_t q = on ? a.slot_query[qbeg + m] : 0u;
        // Emission gate of the slot: a fixed key threshold from the query's sample, and a
        // bucket limit that tightens while the scan runs: the histogram counts the emitted
        // candidates per bucket, and the first bucket at which the running count reaches k
        // bounds the k-th best.
        uint32_t bmax = (uint32_t)kHistBins - 1u;
        if (a.use_hist) {
            uint32_t h[NB], sum = 0;
#pragma unroll
            for (int j = 0; j < NB; ++j) { // device-scope loads: counts other CUs just added
                h[j] = on ? __hip_atomic_load(a.hist + (size_t)q * kHistBins + sub * NB + j, __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT)
                          : 0u;
                sum += h[j];
            }
            uint32_t incl = sum;
#pragma unroll
            for (int off = 1; off < TPS; off <<= 1) {
                const uint32_t y = __shfl_up(incl, off);
                if (sub >= off) incl += y;
            }
            uint32_t run = incl - sum; // emitted in the buckets before this thread's
            bool found = false;
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                run += h[j];
                if (!found && run >= (uint32_t)a.k) {
                    found = true;
                    bmax = (uint32_t)(sub * NB + j);
                }
            }
#pragma unroll
            for (int off = 1; off < TPS; off <<= 1) {
                const uint32_t y = __shfl_xor(bmax, off);
                bmax = y < bmax ? y : bmax;
            }
        }
        if (sub == 0) {
            if (on && a.use_hist) { // share the limit with every workgroup scoring this query
                const uint32_t seen = atomicMin(a.tcur + q, bmax);
                bmax = seen < bmax ? seen : bmax;
            }
            const uint32_t base = on ? q * a.ecap : 0u;
            s.out[m] = on ? a.slot_out[qbeg + m] : 0u; // position of the pair inside the query's candidate range
            s.qn[m] = on ? a.qnorm[q] : 0.f;
            s.q[m] = q;
            s.base[m] = base;
            s.thr[m] = on ? a.tau[q] : 0u;
            s.lo[m] = on ? a.tlo[q] : 0.f;
            s.inv[m] = on ? a.tinv[q] : 0.f;
            s.bmax[m] = bmax;
        }
    }
}

// same query group as the previous tile: pick up bucket limits other workgroups have tightened
__device__ __forceinline__ void refresh_slot(const ScanArgs &a, const Slots &s, int tid, uint32_t qcnt)
{
    if ((uint32_t)tid < qcnt) {
        const uint32_t seen = __hip_atomic_load(a.tcur + s.q[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (seen < s.bmax[tid]) s.bmax[tid] = seen;
    }
}

// Gated emission of one 32-row block.  The lane holds, for each of its 4 * MT slots m, the values of
// rows r0 (nt = 0) and r0 + 16 (nt = 1); the 16 lanes of a group share slot m.  Room in the query's
// region is reserved with one atomic per slot and group; the reservations of sixteen slots are issued
// before the first answer is used, so they cost one round trip to the counters, not one per slot.
template <int MT>
__device__ __forceinline__ void emit_block(const ScanArgs &a, const Slots &s, f32x4 (&acc)[MT][2], int rb, int ln, int lg,
                                           int nrows, uint32_t qcnt, uint32_t row0, gfloats txn)
{
    constexpr int MQ = MT * 16;
    const int r0 = rb * kRowBlock + ln, r1 = r0 + 16;
    const bool live0 = r0 < nrows, live1 = r1 < nrows;
    float xn0 = 0.f, xn1 = 0.f;
    if (a.metric == PK_METRIC_L2) {
        if (live0) xn0 = txn[r0];
        if (live1) xn1 = txn[r1];
    }
    auto value = [&](int mt, int nt, int i) {
        float v = acc[mt][nt][i];
        if (a.metric == PK_METRIC_L2) v = l2_from_dot(nt ? xn1 : xn0, v, s.qn[(mt * 16 + lg * 4 + i) & (MQ - 1)]);
        return v;
    };
    // survivors are rare: one ballot decides whether the wave goes on to emit
    uint32_t cand = 0; // bit 2 * (mt * 4 + i) + nt
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        if ((uint32_t)(mt * 16) >= qcnt) break; // wave-uniform
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = mt * 16 + lg * 4 + i;
            const bool on = (uint32_t)m < qcnt;
            const uint32_t thr = s.thr[m];
            const bool p0 = live0 && on && order_bits(value(mt, 0, i), a.metric) <= thr;
            const bool p1 = live1 && on && order_bits(value(mt, 1, i), a.metric) <= thr;
            cand |= ((uint32_t)p0 | ((uint32_t)p1 << 1)) << (2 * (mt * 4 + i));
        }
    }
    if (__ballot(cand != 0u) == 0ull) return; // the usual case: nothing survives

#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        if (__ballot(((cand >> (8 * mt)) & 0xffu) != 0u) == 0ull) continue; // wave-uniform
        uint32_t base[4], groups[4]; // answer of the reservation; the group's survivors (nt = 0 in the low half)
        uint32_t any = 0;            // wave-uniform: slots i with a survivor somewhere in the wave
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int j = mt * 4 + i, m = mt * 16 + lg * 4 + i;
            base[i] = 0;
            groups[i] = 0;
            if (__ballot(((cand >> (2 * j)) & 3u) != 0u) == 0ull) continue;
            bool p[2];
            uint32_t b[2] = {0u, 0u};
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                p[nt] = ((cand >> (2 * j + nt)) & 1u) != 0u;
                if (p[nt]) { // the bucket limit tightens while the scan runs
                    b[nt] = bucket_of(value(mt, nt, i), s.lo[m], s.inv[m], a.metric);
                    p[nt] = b[nt] <= s.bmax[m];
                }
            }
            const uint32_t g0 = (uint32_t)(__ballot(p[0]) >> (lg * 16)) & 0xffffu;
            const uint32_t g1 = (uint32_t)(__ballot(p[1]) >> (lg * 16)) & 0xffffu;
            groups[i] = g0 | (g1 << 16);
            if (__ballot(groups[i] != 0u) == 0ull) continue;
            any |= 1u << i;
            if (groups[i] != 0u) {
                if (ln == 0) base[i] = atomicAdd(&a.ccnt[s.q[m]], (uint32_t)__popc(groups[i]));
                if (a.use_hist) {
                    // count the emitted candidates per bucket; one atomic for the group's rows of one
                    // half when they share a bucket (the usual case)
                    uint32_t *hq = a.hist + (size_t)s.q[m] * kHistBins;
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt) {
                        const uint32_t g = nt ? g1 : g0;
                        if (g == 0u) continue; // uniform over the group
                        const int leader = __ffs(g) - 1;
                        const uint32_t b0 = __shfl(b[nt], lg * 16 + leader);
                        const uint32_t odd = (uint32_t)(__ballot(p[nt] && b[nt] != b0) >> (lg * 16)) & 0xffffu;
                        if (odd == 0u) {
                            if (ln == leader) atomicAdd(hq + b0, (uint32_t)__popc(g));
                        } else if (p[nt]) {
                            atomicAdd(hq + b[nt], 1u);
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = mt * 16 + lg * 4 + i;
            if (((any >> i) & 1u) == 0u) continue; // wave-uniform
            const uint32_t first = __shfl(base[i], lg * 16);
            const uint32_t g0 = groups[i] & 0xffffu, g1 = groups[i] >> 16;
            const uint32_t below = (1u << ln) - 1u;
            // a region that is full keeps counting (the selection then rescores the query) but stores nothing
            if ((g0 >> ln) & 1u) {
                const uint32_t at = first + __popc(g0 & below);
                if (at < a.ecap)
                    a.cbuf[(size_t)s.base[m] + at] = ((unsigned long long)order_bits(value(mt, 0, i), a.metric) << 32) |
                                                     (s.out[m] + row0 + (uint32_t)r0);
            }
            if ((g1 >> ln) & 1u) {
                const uint32_t at = first + __popc(g0) + __popc(g1 & below);
                if (at < a.ecap)
                    a.cbuf[(size_t)s.base[m] + at] = ((unsigned long long)order_bits(value(mt, 1, i), a.metric) << 32) |
                                                     (s.out[m] + row0 + (uint32_t)r1);
            }
        }
    }
}

// Epilogue of one 32-row block: the lane holds rows (rb*32 + nt*16 + ln) for slots
// mt*16 + lg*4 + i.  Dense mode writes every value; gated mode emits the survivors.
// COHERENT (dense mode): the values are written through to where every CU of the device reads them
// (another workgroup of the same launch goes on to read them).
template <int MT, bool GATED, bool COHERENT = false>
__device__ __forceinline__ void finish_block(const ScanArgs &a, const Slots &s, f32x4 (&acc)[MT][2], int rb, int ln, int lg,
                                             int nrows, uint32_t qcnt, uint32_t row0, gfloats txn, float *lds_vals = nullptr)
{
    if constexpr (GATED) {
        emit_block<MT>(a, s, acc, rb, ln, lg, nrows, qcnt, row0, txn);
    } else {
        constexpr int MQ = MT * 16;
        const float worst = a.metric == PK_METRIC_IP ? -INFINITY : INFINITY;
        const int nrows_pad = (nrows + 15) & ~15;
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const int row = rb * kRowBlock + nt * 16 + ln;
            const bool live = row < nrows;
            float xn = 0.f;
            if (a.metric == PK_METRIC_L2 && live) xn = txn[row];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                if ((uint32_t)(mt * 16) >= qcnt) break; // wave-uniform
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int m = mt * 16 + lg * 4 + i;
                    float v = acc[mt][nt][i];
                    if (a.metric == PK_METRIC_L2) v = l2_from_dot(xn, v, s.qn[m & (MQ - 1)]);
                    if ((uint32_t)m < qcnt && row < nrows_pad) {
                        float *dst = a.out + (size_t)s.out[m] + row0 + row;
                        if constexpr (COHERENT) {
                            if (lds_vals) lds_vals[row0 + row] = live ? v : worst; // (one slot, one tile: the values' only reader is this workgroup)
                            else __hip_atomic_store(dst, live ? v : worst, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        } else {
                            *dst = live ? v : worst;
                        }
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------------------ whole-group kernel

// MT = query tiles of 16 slots held in LDS (MQ = 16*MT); WAVES = waves per workgroup;
// GATED = emit only values that pass the per-query gate (fine search) instead of writing
// every value (coarse search, threshold sampling).
// FUSED (threshold sample of a small batch; sm, extra_off given): the workgroup that scores the last of a
// query's sample tiles goes on to work out that query's threshold, so that no launch of its own is needed
// for it.  bid / nblk: this workgroup's number among those of the launch that take tiles.
template <int STORAGE, int MT, int WAVES, bool GATED, bool FUSED>
__device__ __forceinline__ void scan_body(const ScanArgs &a, char *smem, uint32_t bid, uint32_t nblk, const SampleArgs *sm,
                                          uint32_t extra_off)
{
    constexpr int MQ = MT * 16;
    const int row_bytes = a.row_bytes;
    const int qstride = row_bytes + kQPadBytes;
    char *qtile = smem;
    // Groups of fewer than 16 slots (a.mq of 1 to 15, MT = 1): only that many query rows are
    // held, plus one row of zeros that the MFMA columns without a slot read.  The threshold
    // sample, one query per tile, runs this way: its LDS use stays small for any row length.
    const int qrows = a.mq < MQ ? a.mq : MQ;
    const int qheld = qrows < MQ ? qrows + 1 : MQ;
    Slots s;
    s.carve(smem + (size_t)qheld * qstride, MQ);
    uint32_t *s_misc = s.bmax + MQ; // kScanSlotWords per-slot arrays precede this: keep scan_lds_bytes in step

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 15, lg = lane >> 4;
    const int nit = row_bytes / kIterBytes;
    const int chunks_per_row = row_bytes / 16;
    uint32_t cur_qbeg = 0xffffffffu, cur_qcnt = 0;
    const char *qbase = qtile + (size_t)(ln < qrows ? ln : qrows) * qstride + lg * 16;

    PK_MARK_IF(scan, GATED ? 0 : 8, bid == 0);
    Sched sc;
    if constexpr (FUSED) {
        // the sample has sp tiles for every query (the scalars in memory say the same: no need to wait for them)
        const uint32_t nt = (uint32_t)sm->nq * (uint32_t)sm->sp;
        const uint32_t g = nt / (uint32_t)(sm->scan_grid * 4);
        sc.start(nt, g < 1 ? 1 : (g > 8 ? 8 : g), bid, nblk);
    } else {
        sc.start(*a.ntiles, *a.batch, bid, nblk);
    }
    if (sc.t >= sc.ntiles) return;
    // FUSED with one tile per query: the tile's values go to the threshold through LDS, not through memory
    [[maybe_unused]] const bool one = FUSED && sm->sp == 1;
    [[maybe_unused]] uint32_t *const fx = reinterpret_cast<uint32_t *>(smem + extra_off); // [4][256] histograms, [12] reduction, [4] flag
    [[maybe_unused]] float *const sv = reinterpret_cast<float *>(fx + 4 * 256 + 16);      // [span] values (one tile per query)
    Tile cur = a.tiles[sc.t];
    while (sc.t < sc.ntiles) {
        const gbytes tx = in_global(cur.x);
        const gfloats txn = in_global(cur.xn);
        const uint32_t row0 = cur.row0;
        PK_MARK_IF(scan, GATED ? 1 : 9, bid == 0);
        const uint32_t qbeg = __builtin_amdgcn_readfirstlane(cur.qbeg);
        const uint32_t qcnt = __builtin_amdgcn_readfirstlane((uint32_t)cur.qcnt);
        const int nrows = __builtin_amdgcn_readfirstlane((int)cur.nrows);

        u32x4 xa[2][4], xb[2][4]; // two register buffers of one 256-byte slice of 32 rows each
        gbytes p0, p1;
#define PK_ROWS(rb)                                                                               \
    p0 = tx + (size_t)((rb) * kRowBlock + ln) * row_bytes + lg * 16;                              \
    p1 = p0 + (size_t)16 * row_bytes;
#define PK_LOAD(buf, it)                                                                          \
    _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4)                                              \
    {                                                                                             \
        buf[0][s4] = *reinterpret_cast<gvec4>(p0 + (size_t)(it) * kIterBytes + s4 * 64);  \
        buf[1][s4] = *reinterpret_cast<gvec4>(p1 + (size_t)(it) * kIterBytes + s4 * 64);  \
    }
#define PK_COMPUTE(buf, it)                                                                       \
    _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)                                             \
    {                                                                                             \
        if (mt < mt_used) {                                                                       \
            const char *qrow = qbase + (size_t)mt * 16 * qstride + (size_t)(it) * kIterBytes;     \
            _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4)                                      \
            {                                                                                     \
                const u32x4 qa = *reinterpret_cast<const u32x4 *>(qrow + s4 * 64);                \
                mfma_step<STORAGE>(acc[mt][0], qa, buf[0][s4]);                                   \
                mfma_step<STORAGE>(acc[mt][1], qa, buf[1][s4]);                                   \
            }                                                                                     \
        }                                                                                         \
    }
        // The wave's first slice of rows is requested first of all: the batch bookkeeping, the
        // fetch of the next tile's descriptor and a reload of the query group then overlap with
        // the memory latency.
        int rb = wave;
        bool preloaded = false;
        if (rb * kRowBlock < nrows) {
            PK_ROWS(rb)
            PK_LOAD(xa, 0)
            preloaded = true;
        }
        if (sc.fresh) sc.request(a, s_misc);
        uint32_t next_end;
        bool next_fresh;
        const uint32_t tn = sc.peek(s_misc, next_end, next_fresh);
        const Tile nxt = a.tiles[tn < sc.ntiles ? tn : sc.ntiles - 1]; // in flight while this tile is scored
        if (qbeg != cur_qbeg || qcnt != cur_qcnt) {
            __syncthreads(); // everyone is done with the previous query group
            const int mrows = qrows < MQ ? qheld : (int)((qcnt + 15u) & ~15u); // rows past the group's last: zeros
            // two pieces per thread at a time: their slot numbers first, then the row pieces, so that a
            // round costs two trips to memory, not four
            const int total = mrows * chunks_per_row;
            for (int idx0 = tid; idx0 < total; idx0 += 2 * WAVES * 64) {
                const int idx1 = idx0 + WAVES * 64;
                const int m0 = idx0 / chunks_per_row, m1 = idx1 / chunks_per_row;
                // (the sample's slot numbers are its query numbers)
                const uint32_t sq0 = (uint32_t)m0 < qcnt ? (FUSED ? qbeg + m0 : a.slot_query[qbeg + m0]) : 0xffffffffu;
                const uint32_t sq1 =
                    idx1 < total && (uint32_t)m1 < qcnt ? (FUSED ? qbeg + m1 : a.slot_query[qbeg + m1]) : 0xffffffffu;
                u32x4 v0 = {0u, 0u, 0u, 0u}, v1 = {0u, 0u, 0u, 0u};
                if (sq0 != 0xffffffffu)
                    v0 = *reinterpret_cast<const u32x4 *>(a.qs + (size_t)sq0 * row_bytes + (size_t)(idx0 - m0 * chunks_per_row) * 16);
                if (sq1 != 0xffffffffu)
                    v1 = *reinterpret_cast<const u32x4 *>(a.qs + (size_t)sq1 * row_bytes + (size_t)(idx1 - m1 * chunks_per_row) * 16);
                *reinterpret_cast<u32x4 *>(qtile + (size_t)m0 * qstride + (size_t)(idx0 - m0 * chunks_per_row) * 16) = v0;
                if (idx1 < total)
                    *reinterpret_cast<u32x4 *>(qtile + (size_t)m1 * qstride + (size_t)(idx1 - m1 * chunks_per_row) * 16) = v1;
            }
            if constexpr (FUSED) {
                if (tid < MQ) {
                    const bool on = (uint32_t)tid < qcnt;
                    s.out[tid] = on ? (qbeg + (uint32_t)tid) * sm->span : 0u;
                    s.qn[tid] = on ? a.qnorm[qbeg + tid] : 0.f;
                }
            } else {
                load_slots<MQ, GATED>(a, s, tid, qbeg, qcnt);
            }
            __syncthreads();
            cur_qbeg = qbeg;
            cur_qcnt = qcnt;
        } else if (GATED && a.use_hist == 1) {
            if (tid < MQ) refresh_slot(a, s, tid, qcnt);
            __syncthreads();
        }
        const int mt_used = (int)((qcnt + 15u) >> 4);
        if constexpr (FUSED) {
            if (one) {
                const float worst = a.metric == PK_METRIC_IP ? -INFINITY : INFINITY;
                for (uint32_t i = tid; i < sm->span; i += WAVES * 64) sv[i] = worst;
                __syncthreads();
            }
        }
        PK_MARK_IF(scan, GATED ? 2 : 10, bid == 0);

        for (; rb * kRowBlock < nrows; rb += WAVES) {
            f32x4 acc[MT][2];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                acc[mt][0] = f32x4{0.f, 0.f, 0.f, 0.f};
                acc[mt][1] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            if (!preloaded) {
                PK_ROWS(rb)
                PK_LOAD(xa, 0)
            }
            preloaded = false;
            bool scored = false;
            if constexpr (!GATED && MT == 1) {
                // The threshold sample: one query per tile, one 32-row block per wave, so a wave's time is its
                // chain of slices.  Long rows keep three slices in flight ahead of the one being multiplied
                // (four register buffers; the multiplication order is unchanged, so the values are too).
                if ((nit & 3) == 0 && nit >= 8) { // wave-uniform
                    u32x4 xc[2][4], xd[2][4];
                    PK_LOAD(xb, 1)
                    PK_LOAD(xc, 2)
                    int it = 0;
                    for (; it + 4 < nit; it += 4) {
                        PK_LOAD(xd, it + 3)
                        PK_COMPUTE(xa, it)
                        PK_LOAD(xa, it + 4)
                        PK_COMPUTE(xb, it + 1)
                        PK_LOAD(xb, it + 5)
                        PK_COMPUTE(xc, it + 2)
                        PK_LOAD(xc, it + 6)
                        PK_COMPUTE(xd, it + 3)
                    }
                    PK_LOAD(xd, it + 3)
                    PK_COMPUTE(xa, it)
                    PK_COMPUTE(xb, it + 1)
                    PK_COMPUTE(xc, it + 2)
                    PK_COMPUTE(xd, it + 3)
                    scored = true;
                }
            }
            if (!scored) {
                for (int it = 0; it < nit; it += 2) {
                    if (it + 1 < nit) { PK_LOAD(xb, it + 1) }
                    PK_COMPUTE(xa, it)
                    if (it + 2 < nit) { PK_LOAD(xa, it + 2) }
                    if (it + 1 < nit) { PK_COMPUTE(xb, it + 1) }
                }
            }
            PK_MARK_IF(scan, GATED ? 3 : 11, bid == 0);
            finish_block<MT, GATED, FUSED>(a, s, acc, rb, ln, lg, nrows, qcnt, row0, txn, FUSED && one ? sv : nullptr);
            PK_MARK_IF(scan, GATED ? 4 : 12, bid == 0);
        }
#undef PK_ROWS
#undef PK_LOAD
#undef PK_COMPUTE
        if constexpr (FUSED) {
            // A sample tile is one page against one query (slot number = query number), and every query has
            // sm->sp of them (pages it lacks are empty tiles).  The query's running limit word, unused until its
            // threshold exists, counts the tiles that are done: each thread makes its values of the tile
            // visible to the device, the workgroup meets, one thread counts.  Whoever counts the last one
            // finds every value of the query's sample in place.
            bool mine = true; // this workgroup works out the query's threshold
            if (one) {
                __syncthreads(); // the tile's values are in LDS
            } else {
                __builtin_amdgcn_s_waitcnt(0x0f70); // vmcnt(0): this thread's written-through values have arrived
                __syncthreads();
                if (tid == 0)
                    fx[4 * 256 + 12] =
                        __hip_atomic_fetch_add(sm->tcur + qbeg, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u ==
                                (uint32_t)sm->sp
                            ? 1u
                            : 0u;
                __syncthreads();
                mine = fx[4 * 256 + 12] != 0u;
            }
            PK_MARK_IF(scan, 13, bid == 0);
            if (mine) {
                PK_MARK_IF(scan, 14, qbeg == 0);
                uint32_t cnt = 0, first = 0, kth = 0, last = 0;
                uint32_t(*hist)[256] = reinterpret_cast<uint32_t(*)[256]>(fx);
                if (one) {
                    tau_by_radix<4, false>(*sm, sv, hist, fx + 4 * 256, cnt, first, kth, last, [] {});
                } else {
                    // (the sample is read past the CU's and the XCD's caches)
                    const float *v = sm->vals + (size_t)qbeg * sm->span;
                    if (sm->span <= 4u * kSelThreads)
                        tau_by_radix<4, true>(*sm, v, hist, fx + 4 * 256, cnt, first, kth, last, [] {});
                    else
                        tau_by_radix<16, true>(*sm, v, hist, fx + 4 * 256, cnt, first, kth, last, [] {});
                }
                tau_publish(*sm, qbeg, cnt, first, kth, last);
                PK_MARK_IF(scan, 15, qbeg == 0);
            }
        }
        sc.t = tn;
        sc.end = next_end;
        if (next_fresh) sc.parity ^= 1;
        sc.fresh = next_fresh;
        cur = nxt;
    }
}

template <int STORAGE, int MT, int WAVES, bool GATED>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu((!GATED && MT == 1) ? 2 : 3, 8))) void scan_kernel(ScanArgs a)
{
    extern __shared__ __align__(16) char smem[];
    scan_body<STORAGE, MT, WAVES, GATED, false>(a, smem, blockIdx.x, gridDim.x, nullptr, 0u);
}

// The threshold sample of a small batch with everything that hangs on it, in one launch.  The first sm.nq
// workgroups lay out the second half of the work list (slots and tiles of the fine scan: it needs the
// pair counts only, which the coarse selection left); the others score the sample tiles, and the one that
// finishes a query's last tile works out its threshold (scan_body, FUSED).  extra_off: where, in the
// dynamic LDS, the threshold's histograms lie (behind the scan's own part).
template <int STORAGE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 8))) void sample_tau_kernel(ScanArgs a, SampleArgs sm,
                                                                                                     WorklistArgs wa,
                                                                                                     MultiArgs ma,
                                                                                                     uint32_t extra_off)
{
    extern __shared__ __align__(16) char smem[]; // (all of the kernel's LDS: the limit set for it counts static LDS in)
    const uint32_t nq = (uint32_t)sm.nq;
    if (blockIdx.x < nq) {
        PK_MARK(scan, 19);
        uint32_t *s_pref = reinterpret_cast<uint32_t *>(smem); // [3][kWlSmallLists + 1], then [12] for the waves' sums
        WlPrefetch pre;
        wl_spread_prefetch(wa, ma, blockIdx.x, pre);
        wl_spread(wa, ma, s_pref, s_pref + 3 * (kWlSmallLists + 1), blockIdx.x, pre);
        PK_MARK(scan, 23);
        return;
    }
    scan_body<STORAGE, 1, 4, false, true>(a, smem, blockIdx.x - nq, gridDim.x - nq, &sm, extra_off);
}

// ------------------------------------------------------------------ sliced-query kernel

// The query group is staged through LDS one 256-byte slice of every row at a time, double
// buffered: while the waves multiply slice c, the next slice of the rows (registers) and of
// the queries (registers, then LDS) is already on its way.  One barrier per slice keeps the
// four waves of the workgroup in step.  MT up to 4 (64 slots).  Always 4 waves, one 32-row
// block each per pass over the page.
template <int STORAGE, int MT, bool GATED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 8))) void scan_ks_kernel(ScanArgs a)
{
    extern __shared__ __align__(16) char smem[];
    constexpr int MQ = MT * 16;
    constexpr int QLOADS = MQ / 16; // 16-byte pieces of a slice each thread moves: MQ slots x 16 pieces / 256 threads
    char *qbuf = smem;              // [2][MQ][kKsStride]
    Slots s;
    s.carve(smem + (size_t)2 * MQ * kKsStride, MQ);
    uint32_t *s_slotq = reinterpret_cast<uint32_t *>(s.bmax + MQ); // query row of each slot (all modes)
    uint32_t *s_misc = s_slotq + MQ;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 15, lg = lane >> 4;
    const int row_bytes = a.row_bytes;
    const int nit = row_bytes / kIterBytes;
    uint32_t cur_qbeg = 0xffffffffu, cur_qcnt = 0;
    const int qm = tid >> 4, qpiece = (tid & 15) * 16; // this thread's slot (mod 16) and piece of a slice

    Sched sc;
    sc.start(*a.ntiles, *a.batch, blockIdx.x, gridDim.x);
    if (sc.t >= sc.ntiles) return;
    Tile cur = a.tiles[sc.t];
    while (sc.t < sc.ntiles) {
        if (sc.fresh) sc.request(a, s_misc);
        uint32_t next_end;
        bool next_fresh;
        const uint32_t tn = sc.peek(s_misc, next_end, next_fresh);
        const Tile nxt = a.tiles[tn < sc.ntiles ? tn : sc.ntiles - 1]; // in flight while this tile is scored
        {
            const gbytes tx = in_global(cur.x);
            const gfloats txn = in_global(cur.xn);
            const uint32_t row0 = cur.row0;
            const uint32_t qbeg = __builtin_amdgcn_readfirstlane(cur.qbeg);
            const uint32_t qcnt = __builtin_amdgcn_readfirstlane((uint32_t)cur.qcnt);
            const int nrows = __builtin_amdgcn_readfirstlane((int)cur.nrows);
            if (qbeg != cur_qbeg || qcnt != cur_qcnt) {
                __syncthreads();
                load_slots<MQ, GATED>(a, s, tid, qbeg, qcnt);
                if (tid < MQ) s_slotq[tid] = (uint32_t)tid < qcnt ? a.slot_query[qbeg + tid] : 0xffffffffu;
                __syncthreads();
                cur_qbeg = qbeg;
                cur_qcnt = qcnt;
            } else if (GATED && a.use_hist == 1) {
                if (tid < MQ) refresh_slot(a, s, tid, qcnt);
                __syncthreads();
            }
            const int mt_used = (int)((qcnt + 15u) >> 4);
            // global addresses of this thread's pieces of the query slices
            const char *qsrc[QLOADS];
#pragma unroll
            for (int j = 0; j < QLOADS; ++j) {
                const uint32_t q = s_slotq[j * 16 + qm];
                qsrc[j] = q == 0xffffffffu ? nullptr : a.qs + (size_t)q * row_bytes + qpiece;
            }

            const int npass = (nrows + 4 * kRowBlock - 1) / (4 * kRowBlock);
            for (int pass = 0; pass < npass; ++pass) {
                const int rb = pass * 4 + wave;
                // a wave past the end of the page keeps in step (barriers) on the page's first rows
                const bool active = rb * kRowBlock < nrows;
                const int row_a = (active ? rb * kRowBlock : 0) + ln;
                const gbytes p0 = tx + (size_t)row_a * row_bytes + lg * 16;
                const gbytes p1 = p0 + (size_t)16 * row_bytes;
                f32x4 acc[MT][2];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    acc[mt][0] = f32x4{0.f, 0.f, 0.f, 0.f};
                    acc[mt][1] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
                u32x4 xa[2][4], xb[2][4], qr[QLOADS];
                const char *qrd = qbuf + (size_t)ln * kKsStride + lg * 16;

#define PK_LOAD(buf, it)                                                                          \
    _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4)                                              \
    {                                                                                             \
        buf[0][s4] = *reinterpret_cast<gvec4>(p0 + (size_t)(it) * kIterBytes + s4 * 64);  \
        buf[1][s4] = *reinterpret_cast<gvec4>(p1 + (size_t)(it) * kIterBytes + s4 * 64);  \
    }
#define PK_QLOAD(it)                                                                              \
    _Pragma("unroll") for (int j = 0; j < QLOADS; ++j)                                            \
    {                                                                                             \
        qr[j] = u32x4{0u, 0u, 0u, 0u};                                                            \
        if (j < mt_used && qsrc[j])                                                               \
            qr[j] = *reinterpret_cast<const u32x4 *>(qsrc[j] + (size_t)(it) * kIterBytes);        \
    }
#define PK_QSTORE(b)                                                                              \
    _Pragma("unroll") for (int j = 0; j < QLOADS; ++j)                                            \
    {                                                                                             \
        if (j < mt_used)                                                                          \
            *reinterpret_cast<u32x4 *>(qbuf + ((size_t)(b) * MQ + j * 16 + qm) * kKsStride + qpiece) = qr[j]; \
    }
#define PK_COMPUTE(buf, b)                                                                        \
    _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)                                             \
    {                                                                                             \
        if (mt < mt_used) {                                                                       \
            const char *qrow = qrd + ((size_t)(b) * MQ + mt * 16) * kKsStride;                    \
            _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4)                                      \
            {                                                                                     \
                const u32x4 qa = *reinterpret_cast<const u32x4 *>(qrow + s4 * 64);                \
                mfma_step<STORAGE>(acc[mt][0], qa, buf[0][s4]);                                   \
                mfma_step<STORAGE>(acc[mt][1], qa, buf[1][s4]);                                   \
            }                                                                                     \
        }                                                                                         \
    }
                // slice 0 of the queries into LDS buffer 0, slice 0 of the rows into xa
                __syncthreads(); // the previous pass / tile no longer reads the query buffers
                PK_LOAD(xa, 0)
                PK_QLOAD(0)
                PK_QSTORE(0)
                __syncthreads();
                for (int it = 0; it < nit; it += 2) {
                    if (it + 1 < nit) {
                        PK_LOAD(xb, it + 1)
                        PK_QLOAD(it + 1)
                    }
                    PK_COMPUTE(xa, 0)
                    if (it + 1 < nit) { PK_QSTORE(1) }
                    __syncthreads();
                    if (it + 1 < nit) {
                        if (it + 2 < nit) {
                            PK_LOAD(xa, it + 2)
                            PK_QLOAD(it + 2)
                        }
                        PK_COMPUTE(xb, 1)
                        if (it + 2 < nit) { PK_QSTORE(0) }
                        __syncthreads();
                    }
                }
#undef PK_LOAD
#undef PK_QLOAD
#undef PK_QSTORE
#undef PK_COMPUTE
                if (active) finish_block<MT, GATED>(a, s, acc, rb, ln, lg, nrows, qcnt, row0, txn);
            }
        }
        sc.t = tn;
        sc.end = next_end;
        if (next_fresh) sc.parity ^= 1;
        sc.fresh = next_fresh;
        cur = nxt;
    }
}

// ------------------------------------------------------------------ centroid scoring, small batches

// Coarse step (Section 2.2) for query segments too small to fill the GEMM's 128 x 128
// tiles: inserts of a few vectors, search batches of tens of queries.  The whole centroid
// table is a few MB, so latency, not bandwidth, sets the time: the work is cut fine.  A
// workgroup scores 16 centroids against up to 16*MT queries; its 4 waves split the
// contraction index, so each wave streams a quarter of every row (centroids and queries
// alike come straight from global memory / L2 in MFMA operand layout, no LDS staging), and
// the four partial accumulators meet in LDS.  Output: out[query * stride + centroid].
template <int MT, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void centroid_scores_kernel(CentroidArgs a, MultiArgs m)
{
    __shared__ float s_red[WAVES][MT][4][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 15, lg = lane >> 4;
    int h = 0;
    while (h + 1 < m.n && blockIdx.x >= a.blk[h + 1]) ++h;
    const DevIndex &ix = *m.ix[h];
    const uint32_t nblk = (uint32_t)ix.nlist_pad / 16u;
    const uint32_t local = blockIdx.x - a.blk[h];
    const uint32_t qc = local / nblk, cb = local - qc * nblk;
    const uint32_t q0 = m.qlo[h] + qc * (uint32_t)(MT * 16);
    const uint32_t left = m.qlo[h + 1] - q0;
    const uint32_t qcnt = left < (uint32_t)(MT * 16) ? left : (uint32_t)(MT * 16);
    const int mt_used = (int)((qcnt + 15u) >> 4);
    const int row_bytes = a.row_bytes;
    const int nit = row_bytes / kIterBytes;
    const int per = (nit + WAVES - 1) / WAVES;
    const int it0 = wave * per, it1 = it0 + per < nit ? it0 + per : nit;
    const char *xp = reinterpret_cast<const char *>(ix.cent) + (size_t)(cb * 16u + ln) * row_bytes + lg * 16;
    const char *qp[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const uint32_t slot = (uint32_t)(mt * 16 + ln);
        qp[mt] = slot < qcnt ? a.qs + (size_t)(q0 + slot) * row_bytes + lg * 16 : nullptr;
    }
    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    u32x4 xa[4], xb[4], qa[MT][4], qb[MT][4];
#define PK_CLOAD(xbuf, qbuf, it)                                                                  \
    _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4)                                              \
    {                                                                                             \
        xbuf[s4] = *reinterpret_cast<const u32x4 *>(xp + (size_t)(it) * kIterBytes + s4 * 64);    \
        _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)                                         \
        {                                                                                         \
            qbuf[mt][s4] = u32x4{0u, 0u, 0u, 0u};                                                 \
            if (mt < mt_used && qp[mt])                                                           \
                qbuf[mt][s4] = *reinterpret_cast<const u32x4 *>(qp[mt] + (size_t)(it) * kIterBytes + s4 * 64); \
        }                                                                                         \
    }
#define PK_CCOMPUTE(xbuf, qbuf)                                                                   \
    _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)                                             \
    {                                                                                             \
        if (mt < mt_used) {                                                                       \
            _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4) mfma_step<PK_F32>(acc[mt], qbuf[mt][s4], xbuf[s4]); \
        }                                                                                         \
    }
    if (it0 < it1) { PK_CLOAD(xa, qa, it0) }
    for (int it = it0; it < it1; it += 2) {
        if (it + 1 < it1) { PK_CLOAD(xb, qb, it + 1) }
        PK_CCOMPUTE(xa, qa)
        if (it + 2 < it1) { PK_CLOAD(xa, qa, it + 2) }
        if (it + 1 < it1) { PK_CCOMPUTE(xb, qb) }
    }
#undef PK_CLOAD
#undef PK_CCOMPUTE
    // lane (ln, lg) of a wave holds centroid cb*16 + ln against slots mt*16 + lg*4 + i
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int i = 0; i < 4; ++i) s_red[wave][mt][i][lane] = acc[mt][i];
    __syncthreads();
    const int i = wave & 3; // after the barrier wave w < 4 adds up element i = w of every lane
    auto partial_sum = [&](int mt) {
        float v = (s_red[0][mt][i][lane] + s_red[1][mt][i][lane]) + (s_red[2][mt][i][lane] + s_red[3][mt][i][lane]);
        if constexpr (WAVES == 8)
            v += (s_red[4][mt][i][lane] + s_red[5][mt][i][lane]) + (s_red[6][mt][i][lane] + s_red[7][mt][i][lane]);
        return v;
    };
    if (wave < 4) {
    const uint32_t c = cb * 16u + (uint32_t)ln;
    float cn = 0.f;
    if (a.metric == PK_METRIC_L2 && c < (uint32_t)ix.nlist) cn = ix.cnorm[c];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const uint32_t slot = (uint32_t)(mt * 16 + lg * 4 + i);
        if (slot >= qcnt || c >= (uint32_t)ix.nlist) continue;
        float v = partial_sum(mt);
        if (a.metric == PK_METRIC_L2) v = fmaxf(cn - 2.f * v + a.qnorm[q0 + slot], 0.f);
        if (!a.best) a.out[(size_t)(q0 + slot) * a.stride + c] = v;
    }
    if (a.best) {
        // top-1: the 16 lanes of a group hold 16 centroids of one query; the best of them goes to the
        // query's word (ties to the lower list number: the key's low word)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const uint32_t slot = (uint32_t)(mt * 16 + lg * 4 + i);
            unsigned long long key = ~0ull;
            if (slot < qcnt && c < (uint32_t)ix.nlist) {
                float v = partial_sum(mt);
                if (a.metric == PK_METRIC_L2) v = fmaxf(cn - 2.f * v + a.qnorm[q0 + slot], 0.f);
                key = ((unsigned long long)order_bits(v, a.metric) << 32) | c;
            }
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) {
                const unsigned long long o = __shfl_xor(key, off);
                key = o < key ? o : key;
            }
            if (ln == 0 && slot < qcnt && key != ~0ull) atomicMin(a.best + q0 + slot, key);
        }
    }
    } // wave < 4
    if (a.meta.cand_off) {
        // bookkeeping of the coarse step (otherwise done while the queries are prepared); last, so that no
        // load of this kernel queues behind these stores
        for (uint32_t i = blockIdx.x * blockDim.x + tid; i < a.meta.nclear; i += gridDim.x * blockDim.x) a.meta.clear[i] = 0u;
        if (cb == 0 && (uint32_t)tid < qcnt) {
            const uint32_t t = q0 + (uint32_t)tid;
            a.meta.cand_off[t] = t * a.meta.stride;
            a.meta.cand_cnt[t] = (uint32_t)ix.nlist;
            a.meta.qagent[t] = (uint16_t)h;
        }
    }
}

// ------------------------------------------------------------------------ host side

template <int MT>
static hipError_t launch_centroid_mt(const CentroidArgs &a, const MultiArgs &m, hipStream_t s)
{
    static_assert(MT >= 1, "");
    if (MT == 1 && a.row_bytes / kIterBytes >= 16) {
        // one group of queries over long rows: eight waves share the row, so that each has few slices in a row to wait for
        hipLaunchKernelGGL((centroid_scores_kernel<1, 8>), dim3(a.blk[m.n]), dim3(512), 0, s, a, m);
        return hipGetLastError();
    }
    hipLaunchKernelGGL((centroid_scores_kernel<MT, 4>), dim3(a.blk[m.n]), dim3(256), 0, s, a, m);
    return hipGetLastError();
}

hipError_t launch_centroid_scores(const CentroidArgs &a, const MultiArgs &m, hipStream_t s)
{
    if (a.row_bytes <= 0 || a.row_bytes % kIterBytes != 0) return hipErrorInvalidValue;
    if (a.blk[m.n] == 0) return hipSuccess;
    switch (a.chunk) {
    case 16: return launch_centroid_mt<1>(a, m, s);
    case 32: return launch_centroid_mt<2>(a, m, s);
    case 48: return launch_centroid_mt<3>(a, m, s);
    case 64: return launch_centroid_mt<4>(a, m, s);
    default: return hipErrorInvalidValue;
    }
}

int scan_lds_bytes(int row_bytes, int mq)
{
    const int rows = mq < 16 ? mq + 1 : mq; // small groups: their query rows and one row of zeros
    const int cols = mq < 16 ? 16 : mq;     // MFMA columns = length of the per-slot arrays
    return rows * (row_bytes + kQPadBytes) + cols * kScanSlotWords * 4 + 16; // query tile + per-slot arrays + scratch
}

int scan_ks_lds_bytes(int mq)
{
    return 2 * mq * kKsStride + mq * (kScanSlotWords + 1) * 4 + 16; // two slices + per-slot arrays + scratch
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
    static LdsCleared cleared;
    return launch_with_lds(&scan_kernel<STORAGE, MT, WAVES, GATED>, cleared, scan_lds_bytes(a.row_bytes, a.mq), a, grid,
                           WAVES * 64, s);
}

template <int STORAGE, int MT, bool GATED>
static hipError_t launch_ks_one(const ScanArgs &a, int grid, hipStream_t s)
{
    static LdsCleared cleared;
    return launch_with_lds(&scan_ks_kernel<STORAGE, MT, GATED>, cleared, scan_ks_lds_bytes(MT * 16), a, grid, 256, s);
}

template <int STORAGE, int WAVES, bool GATED>
static hipError_t launch_mt(const ScanArgs &a, int grid, hipStream_t s)
{
    if (a.mq >= 1 && a.mq < 16) return launch_one<STORAGE, 1, WAVES, GATED>(a, grid, s);
    switch (a.mq) {
    case 16: return launch_one<STORAGE, 1, WAVES, GATED>(a, grid, s);
    case 32: return launch_one<STORAGE, 2, WAVES, GATED>(a, grid, s);
    case 64: return launch_one<STORAGE, 4, WAVES, GATED>(a, grid, s);
    default: return hipErrorInvalidValue;
    }
}

template <int STORAGE, bool GATED>
static hipError_t launch_ks_mt(const ScanArgs &a, int grid, hipStream_t s)
{
    switch (a.mq) {
    case 16: return launch_ks_one<STORAGE, 1, GATED>(a, grid, s);
    case 32: return launch_ks_one<STORAGE, 2, GATED>(a, grid, s);
    case 64: return launch_ks_one<STORAGE, 4, GATED>(a, grid, s);
    default: return hipErrorInvalidValue;
    }
}

// Threshold sample of a small batch: the sample's tiles (a.mq < 16: one query each), every query's threshold and
// the second half of the work list in one launch.  grid: workgroups for the tiles; sm.nq more are added.
hipError_t launch_sample_tau(const ScanArgs &a, const SampleArgs &sm, const WorklistArgs &wa, const MultiArgs &ma, int grid,
                             hipStream_t s)
{
    if (a.row_bytes <= 0 || a.row_bytes % kIterBytes != 0 || a.tau != nullptr || a.mq < 1 || a.mq >= 16)
        return hipErrorInvalidValue;
    if (sm.nq <= 0 || sm.span % 4 != 0 || sm.span > 16u * kSelThreads) return hipErrorInvalidValue;
    if ((uint64_t)wa.n_handles * (uint64_t)wa.nlist_max > kWlSmallLists) return hipErrorInvalidValue;
    const int scan_part = (scan_lds_bytes(a.row_bytes, a.mq) + 15) & ~15;
    const int tau_part = (4 * 256 + 16) * 4 + (sm.sp == 1 ? (int)sm.span * 4 : 0); // histograms, reduction, flag; one tile's values
    const int spread_part = (3 * ((int)kWlSmallLists + 1) + 12) * 4; // the three prefix sums over the lists, the waves' sums
    const int lds = std::max(scan_part + tau_part, spread_part);
    const void *fn = a.storage == PK_F16 ? reinterpret_cast<const void *>(&sample_tau_kernel<PK_F16>)
                                         : reinterpret_cast<const void *>(&sample_tau_kernel<PK_F32>);
    static LdsCleared cleared[2];
    LdsCleared &c = cleared[a.storage == PK_F16 ? 1 : 0];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < kMaxDevices;
    if (!tracked || c.on[dev].load(std::memory_order_acquire) == 0) {
        int most = 0;
        e = hipDeviceGetAttribute(&most, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, most);
        if (e != hipSuccess) return e;
        if (tracked) c.on[dev].store(1, std::memory_order_release);
    }
    const dim3 g((uint32_t)grid + (uint32_t)sm.nq), b(256);
    if (a.storage == PK_F16)
        hipLaunchKernelGGL(sample_tau_kernel<PK_F16>, g, b, lds, s, a, sm, wa, ma, (uint32_t)scan_part);
    else
        hipLaunchKernelGGL(sample_tau_kernel<PK_F32>, g, b, lds, s, a, sm, wa, ma, (uint32_t)scan_part);
    return hipGetLastError();
}

// whole-group kernel: gated (fine search) when a.tau is set, else every value is written (threshold sampling)
hipError_t launch_scan(const ScanArgs &a, int grid, hipStream_t s)
{
    if (a.row_bytes <= 0 || a.row_bytes % kIterBytes != 0) return hipErrorInvalidValue;
    const bool gated = a.tau != nullptr;
    if (a.storage == PK_F16) return gated ? launch_mt<PK_F16, 4, true>(a, grid, s) : launch_mt<PK_F16, 4, false>(a, grid, s);
    return gated ? launch_mt<PK_F32, 4, true>(a, grid, s) : launch_mt<PK_F32, 4, false>(a, grid, s);
}

// the sliced-query kernel (gated fine search only; fp32 rows are held to 32 slots)
hipError_t launch_scan_ks(const ScanArgs &a, int grid, hipStream_t s)
{
    if (a.row_bytes <= 0 || a.row_bytes % kIterBytes != 0 || a.tau == nullptr) return hipErrorInvalidValue;
    if (a.storage == PK_F16) return launch_ks_mt<PK_F16, true>(a, grid, s);
    if (a.mq > 32) return hipErrorInvalidValue;
    return launch_ks_mt<PK_F32, true>(a, grid, s);
}

} // namespace pk
