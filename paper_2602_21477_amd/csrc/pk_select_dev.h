// Device-side pieces of the selection kernels that other kernels take along: the radix
// selection over keys held in registers, and the threshold of one query from its sample
// (Section 2.2 fine search: the k-th best of a sample of the probed rows bounds the k-th best
// of all of them, so no row beyond it needs to be kept).
#pragma once

#include "pk_internal.h"

namespace pk {

// The K-th smallest (K counts from 1) of the keys that the 256 threads of a workgroup hold in registers
// (key[j] takes part if live[j]; K is at most the number of live keys), found digit by digit: four
// 8-bit passes over LDS histograms with one barrier each; every wave works out each digit for itself.
// hist: LDS [4][256], need not be initialised.  Returns that key; of the `ties` keys equal to it, `left`
// belong to the K smallest.
template <int VPT>
__device__ __forceinline__ uint32_t radix_kth(const uint32_t (&key)[VPT], const bool (&live)[VPT], uint32_t K,
                                              uint32_t (*hist)[256], uint32_t &left, uint32_t &ties)
{
    const uint32_t tid = threadIdx.x, lane = tid & 63;
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) hist[pass][tid] = 0;
    __syncthreads();
    uint32_t prefix = 0, krem = K, tie = 0;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        const uint32_t himask = pass == 0 ? 0u : 0xffffffffu << (shift + 8);
#pragma unroll
        for (int j = 0; j < VPT; ++j)
            if (live[j] && (key[j] & himask) == prefix) atomicAdd(&hist[pass][(key[j] >> shift) & 255u], 1u);
        __syncthreads();
        // which digit holds the krem-th smallest of the keys that share the prefix (a lane takes four
        // neighbouring digits)
        const u32x4 c4 = *reinterpret_cast<const u32x4 *>(&hist[pass][lane * 4]);
        const uint32_t t = c4[0] + c4[1] + c4[2] + c4[3];
        uint32_t incl = t;
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t y = __shfl_up(incl, off);
            if (lane >= (uint32_t)off) incl += y;
        }
        uint32_t run = incl - t, digit = 0, rem = 0, cnt = 0;
        const bool here = run < krem && krem <= incl;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (run < krem && krem <= run + c4[e]) {
                digit = lane * 4 + e;
                rem = krem - run;
                cnt = c4[e];
            }
            run += c4[e];
        }
        const int src = __ffsll((unsigned long long)__ballot(here)) - 1; // K <= live keys: some lane has it
        prefix |= (uint32_t)__shfl(digit, src) << shift;
        krem = __shfl(rem, src);
        tie = __shfl(cnt, src);
    }
    left = krem;
    ties = tie;
    return prefix;
}

// Threshold of one query from a sample held in registers (up to 256 * VPT values): the k-th best by radix
// selection, the best and the worst real value and their number by reduction.  s_red: LDS [12].
// after_loads: called once the sample's loads are on their way (the caller's own read-ahead goes there).
// COHERENT: the sample was written by other workgroups of the same launch (device-scope loads).
template <int VPT, bool COHERENT = false, typename F>
__device__ __forceinline__ void tau_by_radix(const SampleArgs &a, const float *v, uint32_t (*hist)[256], uint32_t *s_red,
                                             uint32_t &cnt, uint32_t &first, uint32_t &kth, uint32_t &last, F after_loads)
{
    const uint32_t tid = threadIdx.x;
    uint32_t key[VPT];
    bool live[VPT];
    float raw[VPT];
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
        const uint32_t p = tid + (uint32_t)kSelThreads * j;
        live[j] = p < a.span;
        raw[j] = 0.f;
        if (live[j]) {
            if constexpr (COHERENT) raw[j] = __hip_atomic_load(v + p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            else raw[j] = v[p];
        }
    }
    after_loads();
    uint32_t mn = 0xffffffffu, mx = 0u, real = 0u;
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
        key[j] = live[j] ? order_bits(raw[j], a.metric) : 0xffffffffu;
        if (live[j] && key[j] < kWorstBits) { // padding of the sample takes part in the ranking (last) but is no value
            mn = key[j] < mn ? key[j] : mn;
            mx = key[j] > mx ? key[j] : mx;
            ++real;
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t a0 = __shfl_xor(mn, off), a1 = __shfl_xor(mx, off);
        mn = a0 < mn ? a0 : mn;
        mx = a1 > mx ? a1 : mx;
        real += __shfl_xor(real, off);
    }
    if ((tid & 63) == 0) {
        s_red[tid >> 6] = mn;
        s_red[4 + (tid >> 6)] = mx;
        s_red[8 + (tid >> 6)] = real;
    }
    uint32_t left, ties;
    kth = radix_kth<VPT>(key, live, (uint32_t)a.k, hist, left, ties); // its barriers publish s_red
    first = min(min(s_red[0], s_red[1]), min(s_red[2], s_red[3]));
    last = max(max(s_red[4], s_red[5]), max(s_red[6], s_red[7]));
    cnt = s_red[8] + s_red[9] + s_red[10] + s_red[11];
}

// The threshold's outputs for query q (one workgroup; cnt = real samples, at most k are counted when the
// selector keeps only k): threshold key, origin and scale of the bucket histogram, and the histogram and
// its running limit in their starting state.
__device__ __forceinline__ void tau_publish(const SampleArgs &a, uint32_t q, uint32_t cnt, uint32_t first, uint32_t kth,
                                            uint32_t last)
{
    if (threadIdx.x == 0) {
        const bool full = cnt >= (uint32_t)a.k;
        a.tau[q] = full ? kth : 0xffffffffu;
        a.tcur[q] = (uint32_t)kHistBins - 1u;
        float lo = 0.f, inv = 0.f;
        if (cnt > 0) {
            lo = value_of(first, a.metric);
            const float far = value_of(full ? kth : last, a.metric);
            const float range = fabsf(far - lo);
            if (range > 0.f && range < INFINITY) inv = ((float)kHistBins - 1.001f) / range;
        }
        a.tlo[q] = lo;
        a.tinv[q] = inv;
    }
    if (threadIdx.x < kHistBins) a.hist[(size_t)q * kHistBins + threadIdx.x] = 0u;
}

} // namespace pk
