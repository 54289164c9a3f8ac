// List scan (fine search, Section 2.2) for lists probed by more queries of the batch than one
// query group of scan_kernel holds: rows stationary in registers, queries streamed through LDS.
//
// Scored group by group with scan_kernel, such a list is read once per group.  Here a tile is
// kRrTileRows (128) rows of one page against up to kRrSlots slots of the list, and the rows are
// held in REGISTERS: four waves, one per SIMD with the whole register file to itself, each
// keeping 32 rows of the tile in MFMA operand layout for the whole tile (loaded straight from
// HBM, 16 rows x 64 bytes per instruction, as scan_kernel loads them).  Only the queries go
// through LDS: blocks of kRqBlock slots in slices of 256 bytes of every query row, double
// buffered, fetched by coalesced loads that are held two slices ahead in registers.  Every
// wave scores its rows against all slots of the block (8 x 2 MFMA tiles per 64 bytes: eight
// 16-byte LDS reads feed sixteen MFMAs), so a 32 KB slice in LDS is good for 128 x 128 x 128
// multiply-adds between two barriers, and the list's queries are streamed once per 128 rows.
//
// Per (row, query) the same MFMAs run in the same order as in scan_kernel, so the values are
// bit-identical and the thresholds of the sample apply.  The launch runs after the regular
// lists' scan or beside it: it reads the bucket limits that scan has published by then (a
// limit only ever tightens, so an early reading emits more, never less) and does not maintain
// the histogram itself.
//
// The row length is a template parameter (NIT = row bytes / 256): every inner loop has a
// compile-time trip count and the steady state is straight-line code, which is what lets the
// loads of one slice stay in flight across the barriers of the two slices before it.
#include "pk_internal.h"

namespace pk {

constexpr int kRqBlock = 128;                     // slots per block
constexpr int kRrSlice = 256;                     // bytes of a row per staged slice
constexpr int kRrAStride = kRrSlice + kQPadBytes; // LDS bytes per slot of a staged slice

// A candidate some lane holds passed its query's sample threshold: bucket test, reservation in
// the query's region, store.  The 16 lanes of a group share query q; wave-uniform call.
__device__ __forceinline__ void emit_direct(const ScanArgs &a, uint32_t q, uint32_t out, float v, uint32_t bits, bool pass,
                                            uint32_t position, int ln, int lg)
{
    uint32_t b = 0;
    if (pass) {
        b = bucket_of(v, a.tlo[q], a.tinv[q], a.metric);
        pass = b <= __hip_atomic_load(a.tcur + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const unsigned long long mask = __ballot(pass);
    const uint32_t gmask = (uint32_t)(mask >> (lg * 16)) & 0xffffu;
    if (gmask) {
        const int leader = __ffs(gmask) - 1;
        uint32_t base = 0;
        if (ln == leader) base = atomicAdd(&a.ccnt[q], (uint32_t)__popc(gmask));
        base = __shfl(base, lg * 16 + leader);
        if (pass) {
            const uint32_t at = base + __popc(gmask & ((1u << ln) - 1u));
            if (at < a.ecap) a.cbuf[(size_t)q * a.ecap + at] = ((unsigned long long)bits << 32) | (out + position);
        }
    }
}

template <int STORAGE, int NIT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void scan_rr_kernel(ScanArgs a)
{
    extern __shared__ __align__(16) char smem[];
    constexpr int ROW_BYTES = NIT * kIterBytes;
    constexpr int NCH = ROW_BYTES / 64; // 64-byte MFMA steps per row
    char *abuf = smem;                                                     // [2][kRqBlock][kRrAStride]
    uint32_t *s_slotq = reinterpret_cast<uint32_t *>(abuf + 2 * kRqBlock * kRrAStride); // [kRrSlots] query of each slot
    float *s_c = reinterpret_cast<float *>(s_slotq + kRrSlots);            // [kRrSlots] gate constant of each slot
    uint32_t *s_misc = reinterpret_cast<uint32_t *>(s_c + kRrSlots);       // keep scan_rr_lds_bytes in step

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 15, lg = lane >> 4;
    const gbytes qs = in_global(a.qs);
    const bool l2 = a.metric == PK_METRIC_L2;
    uint32_t cur_qbeg = 0xffffffffu, cur_qcnt = 0;
    // query-slice staging: piece j of a thread = slot (tid >> 4) + 16 j of the block, bytes (tid & 15) * 16 .. of the slice
    const int scol = (tid & 15) * 16, srow = tid >> 4;
    char *const adst = abuf + (size_t)srow * kRrAStride + scol;
    const char *const apb = abuf + (size_t)ln * kRrAStride + lg * 16;

    // Tiles are handed out in pairs of neighbours (the tiles of a list and slot group follow one another, so the
    // second of a pair nearly always finds the per-slot arrays of the first in LDS): workgroup b starts with
    // pair b; every later pair is claimed from one counter (tiles are long and differ tenfold in length, so
    // no more than two per claim), a pair ahead: the claim made while the last tile of pair i - 1 runs names
    // pair i + 1, and the descriptor of the next tile is fetched while the current one runs.
    const uint32_t ntiles = *a.ntiles;
    const uint32_t npairs = (ntiles + 1u) >> 1;
    if (blockIdx.x >= npairs) return;
    if (tid == 0) s_misc[0] = gridDim.x + atomicAdd(a.tile_ctr, 1u);
    uint32_t pair = blockIdx.x;
    int half = 0;
    Tile cur = a.tiles[2u * pair];
    while (true) {
        const uint32_t row0 = cur.row0;
        const uint32_t qbeg = __builtin_amdgcn_readfirstlane(cur.qbeg);
        const uint32_t qcnt = __builtin_amdgcn_readfirstlane((uint32_t)cur.qcnt);
        const int nrows = __builtin_amdgcn_readfirstlane((int)cur.nrows);

        __syncthreads(); // every wave is done with the previous tile's slices and slot arrays
        const uint32_t p_next = __builtin_amdgcn_readfirstlane(s_misc[0]);
        const bool last_of_pair = half == 1 || 2u * pair + 1u >= ntiles;
        const bool more = !last_of_pair || p_next < npairs;
        const uint32_t t_next = last_of_pair ? 2u * p_next : 2u * pair + 1u;
        const Tile nxt = a.tiles[t_next < ntiles ? t_next : ntiles - 1]; // on its way while this tile is scored
        uint32_t claim = npairs;
        if (tid == 0 && last_of_pair && p_next < npairs) claim = gridDim.x + atomicAdd(a.tile_ctr, 1u); // read when the pair ends
        // ---- this wave's 32 rows, whole, into registers, requested first of all: they come from HBM, and the
        // per-slot arrays and the first query slices (L2) are fetched while they are on their way (rows past
        // the tile's last lie inside the page and hold stale bytes: h = +inf keeps them out)
        u32x4 xb[NCH][2];
        float xn[2], h[2];
        {
            const gbytes p0 = in_global(cur.x) + (size_t)(wave * 32 + ln) * ROW_BYTES + lg * 16;
            const gbytes p1 = p0 + (size_t)16 * ROW_BYTES;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                xb[c][0] = *reinterpret_cast<gvec4>(p0 + c * 64);
                xb[c][1] = *reinterpret_cast<gvec4>(p1 + c * 64);
            }
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                const int row = wave * 32 + nt * 16 + ln;
                xn[nt] = l2 && row < nrows ? in_global(cur.xn)[row] : 0.f;
            }
        }
        asm volatile("" ::: "memory");
        if (qbeg != cur_qbeg || qcnt != cur_qcnt) {
            // Gate: a value passes iff dot >= h(row) + c(slot), up to rounding, for which both constants
            // are lowered a little so that the test passes a superset (what passes is tested again exactly):
            //   inner product  value = dot,              passes iff dot >= tv      h = 0,      c = tv
            //   squared L2     value = xn - 2 dot + qn,  passes iff value <= tv    h = xn / 2, c = (qn - tv) / 2
            // tv = the sample threshold, or the far edge of the last bucket the published limit lets through.
            // Slots past the list's last, up to the end of their block, never pass (c = +inf); their slices
            // are those of the batch's first query (any valid row will do).
            const uint32_t padded = (qcnt + (uint32_t)kRqBlock - 1u) & ~((uint32_t)kRqBlock - 1u);
            for (uint32_t m = tid; m < padded; m += 256) {
                uint32_t q = 0xffffffffu;
                float c = INFINITY;
                if (m < qcnt) {
                    q = a.slot_query[qbeg + m];
                    const uint32_t tau = a.tau[q];
                    const uint32_t bmax = __hip_atomic_load(a.tcur + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const float inv = a.tinv[q], lo = a.tlo[q];
                    const float reach = bmax < (uint32_t)kHistBins - 1u && inv > 0.f
                                            ? (float)(bmax + 1u) / inv * (1.f + 0x1p-18f) : INFINITY;
                    if (l2) {
                        float tv = tau == 0xffffffffu ? INFINITY : value_of(tau, a.metric);
                        tv = fminf(tv, lo + reach + 0x1p-20f * fabsf(lo));
                        const float qn = a.qnorm[q];
                        c = 0.5f * (qn - tv) - 0x1p-21f * (qn + tv);
                    } else {
                        float tv = tau == 0xffffffffu ? -INFINITY : value_of(tau, a.metric);
                        tv = fmaxf(tv, lo - reach - 0x1p-20f * fabsf(lo));
                        c = tv - 0x1p-21f * fabsf(tv);
                    }
                }
                s_slotq[m] = q;
                s_c[m] = c;
            }
            cur_qbeg = qbeg;
            cur_qcnt = qcnt;
        }
        __syncthreads();

        const int nblocks = (int)((qcnt + (uint32_t)kRqBlock - 1u) / (uint32_t)kRqBlock);
        // ---- the query-slice stream: slices of block 0, then of block 1, ...; past the last slice of
        // the tile it repeats that slice, so that the steady state needs no conditions
        int lblk = 0, lsl = 0;
        gbytes ap[8];
        u32x4 R0[8], R1[8];
#define PK_SETPTR(blk)                                                                            \
    _Pragma("unroll") for (int j = 0; j < 8; ++j)                                                 \
    {                                                                                             \
        const uint32_t q = s_slotq[(blk) * kRqBlock + srow + 16 * j];                             \
        ap[j] = qs + (size_t)(q == 0xffffffffu ? 0u : q) * ROW_BYTES + scol;                      \
    }
#define PK_LOADA(R)                                                                               \
    {                                                                                             \
        _Pragma("unroll") for (int j = 0; j < 8; ++j)                                             \
            R[j] = *reinterpret_cast<gvec4>(ap[j] + (size_t)lsl * kRrSlice);                      \
        if (lsl + 1 < NIT) {                                                                      \
            ++lsl;                                                                                \
        } else if (lblk + 1 < nblocks) {                                                          \
            lsl = 0;                                                                              \
            ++lblk;                                                                               \
            PK_SETPTR(lblk)                                                                       \
        }                                                                                         \
    }
#define PK_STOREA(R, buf)                                                                         \
    _Pragma("unroll") for (int j = 0; j < 8; ++j)                                                 \
        *reinterpret_cast<u32x4 *>(adst + ((size_t)(buf) * kRqBlock + 16 * j) * kRrAStride) = R[j];
        // the first two query slices
        PK_SETPTR(0)
        PK_LOADA(R0)
        PK_LOADA(R1)
        asm volatile("" ::: "memory");
        PK_STOREA(R0, 0)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) h[nt] = wave * 32 + nt * 16 + ln < nrows ? xn[nt] * (0.5f - 0x1p-21f) : INFINITY;
        __syncthreads();

        int g = 0; // slices scored so far in this tile: slice g sits in buffer g & 1 (a constant per slice when NIT is even)
        for (int blk = 0; blk < nblocks; ++blk) {
            const int left = (int)qcnt - blk * kRqBlock;
            const bool wide = left > 64; // more than four slot tiles of this block hold slots
            f32x4 acc[8][2];             // [slot tile][row tile]
#pragma unroll
            for (int f = 0; f < 8; ++f) {
                acc[f][0] = f32x4{0.f, 0.f, 0.f, 0.f};
                acc[f][1] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            // One wave per SIMD has nobody to hide an LDS round trip, so the operand reads run one
            // 64-byte step ahead of the MFMAs that use them: a slot tile's operand of the next step is
            // read right after its two MFMAs of this step have issued (the register is free then), which
            // gives every read the other seven tiles' MFMAs to arrive in.  The scheduling hints pin that
            // interleave (two MFMAs, one LDS read); the pipeline drains once per slice, at the barrier
            // that switches the LDS buffers.
#define PK_COMPUTE(buf, slice, NF)                                                                \
    {                                                                                             \
        const char *ab = apb + (size_t)(buf) * kRqBlock * kRrAStride;                             \
        u32x4 qa[NF];                                                                             \
        _Pragma("unroll") for (int f = 0; f < NF; ++f)                                            \
            qa[f] = *reinterpret_cast<const u32x4 *>(ab + (size_t)f * 16 * kRrAStride);           \
        __builtin_amdgcn_sched_barrier(0);                                                        \
        _Pragma("unroll") for (int jj = 0; jj < 4; ++jj)                                          \
        {                                                                                         \
            _Pragma("unroll") for (int f = 0; f < NF; ++f)                                        \
            {                                                                                     \
                mfma_step<STORAGE>(acc[f][0], qa[f], xb[(slice) * 4 + jj][0]);                    \
                mfma_step<STORAGE>(acc[f][1], qa[f], xb[(slice) * 4 + jj][1]);                    \
                if (jj < 3)                                                                       \
                    qa[f] = *reinterpret_cast<const u32x4 *>(ab + (size_t)f * 16 * kRrAStride + (jj + 1) * 64); \
            }                                                                                     \
            _Pragma("unroll") for (int f = 0; f < NF; ++f)                                        \
            {                                                                                     \
                __builtin_amdgcn_sched_group_barrier(0x008, STORAGE == PK_F16 ? 2 : 8, 0);        \
                if (jj < 3) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                    \
            }                                                                                     \
        }                                                                                         \
        __builtin_amdgcn_sched_barrier(0);                                                        \
    }
            // (the empty asm statements keep the compiler from sinking the loads below the MFMAs, which
            // would leave them one slice of lead instead of two)
#define PK_SLICE(sl)                                                                              \
    {                                                                                             \
        if ((NIT % 2 == 0 ? ((sl) & 1) : (g & 1)) == 0) {                                         \
            PK_LOADA(R0)                                                                          \
            asm volatile("" ::: "memory");                                                        \
            if (wide) PK_COMPUTE(0, sl, 8) else PK_COMPUTE(0, sl, 4)                              \
            asm volatile("" ::: "memory");                                                        \
            PK_STOREA(R1, 1)                                                                      \
        } else {                                                                                  \
            PK_LOADA(R1)                                                                          \
            asm volatile("" ::: "memory");                                                        \
            if (wide) PK_COMPUTE(1, sl, 8) else PK_COMPUTE(1, sl, 4)                              \
            asm volatile("" ::: "memory");                                                        \
            PK_STOREA(R0, 0)                                                                      \
        }                                                                                         \
        __syncthreads();                                                                          \
        ++g;                                                                                      \
    }
#pragma unroll
            for (int sl = 0; sl < NIT; ++sl) PK_SLICE(sl)
#undef PK_SLICE
#undef PK_COMPUTE
            // ---- the block is scored.  The lane holds rows wave*32 + nt*16 + ln against slots
            // blk*128 + f*16 + lg*4 + i.  First the largest margin by which a value of each slot tile
            // passes; only tiles where some lane's margin is not negative are looked at value by value.
            const int s0 = blk * kRqBlock + lg * 4;
            float best[8];
#pragma unroll
            for (int f = 0; f < 8; ++f) {
                best[f] = -INFINITY;
                if (f >= 4 && !wide) continue; // wave-uniform
                const f32x4 c = *reinterpret_cast<const f32x4 *>(s_c + s0 + f * 16);
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                    for (int i = 0; i < 4; ++i) best[f] = fmaxf(best[f], acc[f][nt][i] - (h[nt] + c[i]));
            }
            float any = best[0];
#pragma unroll
            for (int f = 1; f < 8; ++f) any = fmaxf(any, best[f]);
            if (__ballot(any >= 0.f) != 0ull) {
#pragma unroll
                for (int f = 0; f < 8; ++f) {
                    if (__ballot(best[f] >= 0.f) == 0ull) continue;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int m = s0 + f * 16 + i;
                        const uint32_t q = s_slotq[m];
                        const bool on = q != 0xffffffffu;
                        const float c = s_c[m];
                        if (__ballot(on && (acc[f][0][i] >= h[0] + c || acc[f][1][i] >= h[1] + c)) == 0ull) continue;
                        const uint32_t thr = on ? a.tau[q] : 0u;
                        const float qn = on && l2 ? a.qnorm[q] : 0.f;
#pragma unroll
                        for (int nt = 0; nt < 2; ++nt) {
                            float v = acc[f][nt][i];
                            if (l2) v = l2_from_dot(xn[nt], v, qn);
                            const uint32_t bits = order_bits(v, a.metric);
                            const bool pass = wave * 32 + nt * 16 + ln < nrows && on && bits <= thr;
                            if (__ballot(pass) == 0ull) continue;
                            const uint32_t out = on ? a.slot_out[qbeg + (uint32_t)m] : 0u;
                            emit_direct(a, on ? q : 0u, out, v, bits, pass, row0 + (uint32_t)(wave * 32 + nt * 16 + ln), ln, lg);
                        }
                    }
                }
            }
        }
#undef PK_SETPTR
#undef PK_LOADA
#undef PK_STOREA
        if (!more) break;
        if (last_of_pair) {
            // every wave has read s_misc[0] long ago (barriers since); the next tile's first barrier publishes this
            if (tid == 0) s_misc[0] = claim;
            pair = p_next;
            half = 0;
        } else {
            half = 1;
        }
        cur = nxt;
    }
}

int scan_rr_lds_bytes()
{
    return 2 * kRqBlock * kRrAStride + kRrSlots * 8 + 16; // two query slices + per-slot arrays (query, gate constant) + scratch
}

template <int STORAGE, int NIT>
static hipError_t launch_rr_one(const ScanArgs &a, int grid, hipStream_t s)
{
    static LdsCleared cleared;
    return launch_with_lds(&scan_rr_kernel<STORAGE, NIT>, cleared, scan_rr_lds_bytes(), a, grid, 256, s);
}

template <int STORAGE>
static hipError_t launch_rr_nit(const ScanArgs &a, int grid, hipStream_t s)
{
    switch (a.row_bytes / kIterBytes) {
    case 1: return launch_rr_one<STORAGE, 1>(a, grid, s);
    case 2: return launch_rr_one<STORAGE, 2>(a, grid, s);
    case 3: return launch_rr_one<STORAGE, 3>(a, grid, s);
    case 4: return launch_rr_one<STORAGE, 4>(a, grid, s);
    case 5: return launch_rr_one<STORAGE, 5>(a, grid, s);
    case 6: return launch_rr_one<STORAGE, 6>(a, grid, s);
    default: return hipErrorInvalidValue;
    }
}

// gated fine search; tiles of kRrTileRows rows x up to kRrSlots slots; rows of at most 1536 bytes
hipError_t launch_scan_rr(const ScanArgs &a, int grid, hipStream_t s)
{
    if (a.row_bytes <= 0 || a.row_bytes % kIterBytes != 0 || a.row_bytes > 1536 || a.tau == nullptr || a.mq != kRrSlots ||
        a.use_hist != 0)
        return hipErrorInvalidValue;
    return a.storage == PK_F16 ? launch_rr_nit<PK_F16>(a, grid, s) : launch_rr_nit<PK_F32>(a, grid, s);
}

} // namespace pk
