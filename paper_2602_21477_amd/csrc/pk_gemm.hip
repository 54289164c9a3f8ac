// Coarse scoring for large query batches (and for the build, where every base vector is a
// "query"): S[m][n] = <Q_m, C_n> (inner product) or |C_n|^2 - 2 <Q_m, C_n> + |Q_m|^2
// (squared L2), Section 2.2's ranking of clusters by centroid distance, for all m, n.
//
// This is a dense contraction, so it runs on the matrix cores with fp32 inputs and fp32
// accumulation (v_mfma_f32_32x32x2_f32): no down-conversion of queries or centroids, so
// the probe ranking tracks the fp64 oracle to fp32 rounding.  128 x 128 output tile per
// workgroup (4 waves, 64 x 64 each as 2 x 2 MFMA blocks), K consumed 32 floats at a time
// through double-buffered LDS; both operands are row-major with the padded row stride of
// the scan layout, so K needs no tail handling.  As in the scan kernel the contraction
// index is permuted identically on both operands so that a lane's four consecutive floats
// (one ds_read_b128) feed four MFMAs.
#include "pk_internal.h"

namespace pk {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kGemmTile = 128;
constexpr int kGemmBK = 32;               // floats per K step
constexpr int kGemmLdsStride = kGemmBK + 4; // floats; +4 keeps the b128 reads conflict free

__global__ __launch_bounds__(256) void gemm_scores_kernel(GemmArgs a)
{
    __shared__ __align__(16) float sA[2][kGemmTile * kGemmLdsStride];
    __shared__ __align__(16) float sB[2][kGemmTile * kGemmLdsStride];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;        // wave's 64 x 64 quadrant
    const int l32 = lane & 31, kg = lane >> 5;      // MFMA row / column and k group
    const int m0 = blockIdx.y * kGemmTile, n0 = blockIdx.x * kGemmTile;
    const int ld = a.ld;                            // floats per row, multiple of 64
    const int ksteps = ld / kGemmBK;

    // global -> register staging: each thread moves 4 x 16 B of A and of B per K step
    // row = (tid >> 3) + 32 * i, 16-byte column = tid & 7
    const int srow = tid >> 3, scol = (tid & 7) * 4;
    const float *ga[4], *gb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int ra = m0 + srow + 32 * i, rb = n0 + srow + 32 * i;
        ra = ra < a.m ? ra : a.m - 1; // clamp: rows past the end are computed and dropped
        rb = rb < a.n_pad ? rb : a.n_pad - 1;
        ga[i] = a.q + (size_t)ra * ld + scol;
        gb[i] = a.c + (size_t)rb * ld + scol;
    }
    f32x4 ra4[4], rb4[4];
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

#define PK_GLOAD(ks)                                                                     \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                        \
    {                                                                                    \
        ra4[i] = *reinterpret_cast<const f32x4 *>(ga[i] + (size_t)(ks) * kGemmBK);       \
        rb4[i] = *reinterpret_cast<const f32x4 *>(gb[i] + (size_t)(ks) * kGemmBK);       \
    }
#define PK_LSTORE(buf)                                                                                   \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                        \
    {                                                                                                    \
        *reinterpret_cast<f32x4 *>(&sA[buf][(srow + 32 * i) * kGemmLdsStride + scol]) = ra4[i];          \
        *reinterpret_cast<f32x4 *>(&sB[buf][(srow + 32 * i) * kGemmLdsStride + scol]) = rb4[i];          \
    }

    PK_GLOAD(0)
    PK_LSTORE(0)
    __syncthreads();
    for (int ks = 0; ks < ksteps; ++ks) {
        const int buf = ks & 1;
        if (ks + 1 < ksteps) { PK_GLOAD(ks + 1) }
        const float *pa = &sA[buf][(wm * 64 + l32) * kGemmLdsStride + kg * 4];
        const float *pb = &sB[buf][(wn * 64 + l32) * kGemmLdsStride + kg * 4];
#pragma unroll
        for (int kc = 0; kc < kGemmBK / 8; ++kc) {
            f32x4 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                fa[i] = *reinterpret_cast<const f32x4 *>(pa + i * 32 * kGemmLdsStride + kc * 8);
                fb[i] = *reinterpret_cast<const f32x4 *>(pb + i * 32 * kGemmLdsStride + kc * 8);
            }
#pragma unroll
            for (int j4 = 0; j4 < 4; ++j4)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][j4], fb[j][j4], acc[i][j], 0, 0, 0);
        }
        if (ks + 1 < ksteps) {
            PK_LSTORE(buf ^ 1) // the other buffer was last read before the previous barrier
        }
        __syncthreads();
    }
#undef PK_GLOAD
#undef PK_LSTORE

    // epilogue: lane holds column n = l32 of rows (kg*4 + 8*(r/4) + r%4) of each 32 x 32 block
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int n = n0 + wn * 64 + j * 32 + l32;
        if (n >= a.n_store) continue;
        const bool live = n < a.n;
        const float cn = (a.metric == PK_METRIC_L2 && live) ? a.cnorm[n] : 0.f;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 64 + i * 32 + kg * 4 + 8 * (r >> 2) + (r & 3);
                if (m < a.m) {
                    float v = acc[i][j][r];
                    if (a.metric == PK_METRIC_L2) v = fmaxf(cn - 2.f * v + a.qnorm[m], 0.f);
                    if (!live) v = a.metric == PK_METRIC_IP ? -INFINITY : INFINITY;
                    a.out[(size_t)m * a.stride + n] = v;
                }
            }
        }
    }
}

hipError_t launch_gemm_scores(const GemmArgs &a, hipStream_t s)
{
    if (a.m <= 0) return hipSuccess;
    if (a.ld % 64 != 0) return hipErrorInvalidValue;
    dim3 grid((a.n_pad + kGemmTile - 1) / kGemmTile, (a.m + kGemmTile - 1) / kGemmTile);
    hipLaunchKernelGGL(gemm_scores_kernel, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

} // namespace pk
