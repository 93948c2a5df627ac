// Coarse assignment: scores of query rows against an index's centroids as a dense contraction
// on the matrix cores (IVF replacement for "select the parents to expand" in the paper's
// Sec. 3.2 step loop; also the assignment pass of index construction).
//
//   C[m][n] = L2:  |b_n|^2 - 2 a_m.b_n      (the per-query constant |a_m|^2 does not change a ranking)
//             IP:  a_m.b_n
//
// A: m rows (queries), B: n rows (centroids), both K-contiguous with a row length that is a
// multiple of 128 bytes.  Workgroup = 4 wavefronts, output tile 128 x 128, K advanced 128 bytes
// at a time through LDS; each wavefront owns a 64 x 64 sub-tile = 2 x 2 MFMA 32x32 blocks.
#include "tri_common.h"
#include "tri_mfma.h"

#define CG_BM 128
#define CG_BN 128
#define CG_KB 128                 // K bytes per stage
#define CG_PITCH (CG_KB + 16)     // LDS row pitch: odd multiple of 16 B past 128 -> conflict-free 16 B reads

template <int DT>
__global__ __launch_bounds__(256) void coarse_gemm_kernel(
    const uint8_t *__restrict__ A, uint32_t a_pitch, uint32_t M,
    const uint8_t *__restrict__ B, uint32_t b_pitch, const float *__restrict__ bnorm, uint32_t N,
    uint32_t k_bytes, const uint32_t *__restrict__ row_metric, uint32_t metric_stride, uint32_t fixed_metric,
    float *__restrict__ C, uint32_t ldc)
{
    __shared__ __attribute__((aligned(16))) uint8_t As[CG_BM * CG_PITCH];
    __shared__ __attribute__((aligned(16))) uint8_t Bs[CG_BN * CG_PITCH];

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63, wave = tid >> 6;
    const uint32_t wm = wave >> 1, wn = wave & 1;
    const uint32_t bm = blockIdx.y * CG_BM, bn = blockIdx.x * CG_BN;

    // global -> register staging: thread owns 16-byte column (tid % 8) of rows tid/8 + 32*i
    const uint32_t ld_col = (tid & 7) * 16, ld_row = tid >> 3;
    const uint8_t *a_src[4];
    const uint8_t *b_src[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint32_t ra = bm + ld_row + 32 * i;
        uint32_t rb = bn + ld_row + 32 * i;
        ra = ra < M ? ra : M - 1;        // rows past the edge re-read the last row; never stored
        rb = rb < N ? rb : N - 1;
        a_src[i] = A + (size_t)ra * a_pitch + ld_col;
        b_src[i] = B + (size_t)rb * b_pitch + ld_col;
    }
    uint4 ra4[4], rb4[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        ra4[i] = *(const uint4 *)(a_src[i]);
        rb4[i] = *(const uint4 *)(b_src[i]);
    }

    tri_f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const uint32_t fr = lane & 31, fk = (lane >> 5) * 16;
    for (uint32_t k0 = 0; k0 < k_bytes; k0 += CG_KB) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            *(uint4 *)(As + (ld_row + 32 * i) * CG_PITCH + ld_col) = ra4[i];
            *(uint4 *)(Bs + (ld_row + 32 * i) * CG_PITCH + ld_col) = rb4[i];
        }
        __syncthreads();
        if (k0 + CG_KB < k_bytes) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ra4[i] = *(const uint4 *)(a_src[i] + k0 + CG_KB);
                rb4[i] = *(const uint4 *)(b_src[i] + k0 + CG_KB);
            }
        }
#pragma unroll
        for (int c = 0; c < CG_KB / 32; ++c) {
            uint4 af[2], bf[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                af[i] = *(const uint4 *)(As + (wm * 64 + i * 32 + fr) * CG_PITCH + c * 32 + fk);
                bf[i] = *(const uint4 *)(Bs + (wn * 64 + i * 32 + fr) * CG_PITCH + c * 32 + fk);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) tri_mma32<DT>(acc[i][j], af[i], bf[j]);
        }
        __syncthreads();
    }

    // epilogue: accumulator r of lane l is (row 8*(r/4) + 4*(l/32) + r%4, col l%32) of its 32x32 block
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const uint32_t n = bn + wn * 64 + j * 32 + fr;
        if (n >= N) continue;
        const float bn2 = bnorm[n];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const uint32_t m = bm + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (m >= M) continue;
                const uint32_t metric = row_metric ? row_metric[(size_t)m * metric_stride] : fixed_metric;
                const float dot = acc[i][j][r];
                C[(size_t)m * ldc + n] = metric == 0 ? (bn2 - 2.0f * dot) : dot;
            }
        }
    }
}

hipError_t tri_launch_coarse_gemm(hipStream_t s, int dtype, const void *a_rows, uint32_t a_pitch_bytes, uint32_t m,
                                  const void *b_rows, const float *b_norm, uint32_t n, uint32_t row_bytes,
                                  const uint32_t *row_metric, uint32_t metric_stride_u32, uint32_t fixed_metric,
                                  float *scores, uint32_t ldc)
{
    if (m == 0 || n == 0) return hipSuccess;
    if (row_bytes == 0 || row_bytes % CG_KB != 0 || a_pitch_bytes % 16 != 0) return hipErrorInvalidValue;
    dim3 grid((n + CG_BN - 1) / CG_BN, (m + CG_BM - 1) / CG_BM);
    if (dtype == TRI_DT_F16)
        hipLaunchKernelGGL(coarse_gemm_kernel<TRI_DT_F16>, grid, dim3(256), 0, s, (const uint8_t *)a_rows,
                           a_pitch_bytes, m, (const uint8_t *)b_rows, row_bytes, b_norm, n, row_bytes, row_metric,
                           metric_stride_u32, fixed_metric, scores, ldc);
    else
        hipLaunchKernelGGL(coarse_gemm_kernel<TRI_DT_F32>, grid, dim3(256), 0, s, (const uint8_t *)a_rows,
                           a_pitch_bytes, m, (const uint8_t *)b_rows, row_bytes, b_norm, n, row_bytes, row_metric,
                           metric_stride_u32, fixed_metric, scores, ldc);
    return hipGetLastError();
}
