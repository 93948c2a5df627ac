// Coarse assignment: scores of query rows against an index's centroids as a dense contraction
// on the matrix cores (the IVF counterpart of choosing which parents to expand in the paper's
// Sec. 3.2 step loop; also the assignment pass of index construction).
//
//   C[m][n] = L2:  |b_n|^2 - 2 a_m.b_n      (the per-query constant |a_m|^2 does not change a ranking)
//             IP:  a_m.b_n
//
// A: m rows (queries), B: n rows (centroids), both K-contiguous with a row length that is a
// multiple of 128 bytes.  Workgroup = 4 wavefronts, output tile 256 x 128; each wavefront owns a
// 128 x 64 sub-tile = 4 x 2 MFMA 32x32 blocks (128 accumulators per lane), so one 32-byte K chunk
// costs 6 operand reads from LDS for 8 MFMAs.  Two workgroups share a compute unit (two wavefronts per
// SIMD, 256 registers each): one multiplies while the other waits at its barrier.
// K advances 64 bytes per stage through a two-stage LDS ring: while stage s is multiplied, the
// registers holding stage s+1 are written to the other half of the ring and the global loads of
// stage s+3 are issued, so a load has two compute phases to arrive and a stage costs one barrier.
#include "tri_common.h"
#include "tri_mfma.h"

#define CG_BM 256
#define CG_BN 128
#define CG_KB 64                  // K bytes per stage
#define CG_PITCH (CG_KB + 16)     // LDS row pitch 80 B: 8 consecutive rows start in 8 different 16-byte columns
#define CG_STAGE ((CG_BM + CG_BN) * CG_PITCH)
#define CG_LDS (2 * CG_STAGE)          // + CG_BM * 4 bytes of row metrics behind it
#define CG_PIECES ((CG_BM + CG_BN) * (CG_KB / 16) / 256)   // 16-byte pieces per thread and stage (6)
#define CG_PIECES_A (CG_BM * (CG_KB / 16) / 256)             // of which A rows (4)

extern __shared__ __attribute__((aligned(16))) uint8_t cg_lds[];

template <int DT>
__device__ __forceinline__ void coarse_gemm_tile(
    const uint8_t *__restrict__ A, uint32_t a_pitch, uint32_t M,
    const uint8_t *__restrict__ B, uint32_t b_pitch, const float *__restrict__ bnorm, uint32_t N,
    uint32_t k_bytes, const uint32_t *__restrict__ row_metric, uint32_t metric_stride, uint32_t fixed_metric,
    float *__restrict__ C, uint32_t ldc)
{

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63, wave = tid >> 6;
    const uint32_t wm = wave >> 1, wn = wave & 1;
    const uint32_t bm = blockIdx.y * CG_BM, bn = blockIdx.x * CG_BN;

    // global -> register staging: piece p = tid + 256 * i is 16-byte column p % 4 of tile row p / 4;
    // tile rows 0..255 are A rows, 256..383 B rows.  Loads go through buffer descriptors that end with
    // the matrices: rows past the edge read zeros (their products are never stored) and the addresses
    // need one register per operand, the piece and stage offsets being uniform.
    const uint32_t a_rows = M - bm < CG_BM ? M - bm : CG_BM, b_rows = N - bn < CG_BN ? N - bn : CG_BN;
    const __amdgpu_buffer_rsrc_t ars = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(A + (size_t)bm * a_pitch), 0, (a_rows - 1) * a_pitch + k_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t brs = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(B + (size_t)bn * b_pitch), 0, (b_rows - 1) * b_pitch + k_bytes, 0x00020000);
    const uint32_t a_off = (tid >> 2) * a_pitch + (tid & 3) * 16, b_off = (tid >> 2) * b_pitch + (tid & 3) * 16;
    const uint32_t dst0 = (tid >> 2) * CG_PITCH + (tid & 3) * 16;
    typedef unsigned int cg_u32x4 __attribute__((ext_vector_type(4)));
    auto fetch = [&](uint4 (&r)[CG_PIECES], uint32_t s) {
#pragma unroll
        for (int i = 0; i < CG_PIECES; ++i) {
            const cg_u32x4 v = i < CG_PIECES_A
                ? __builtin_amdgcn_raw_buffer_load_b128(ars, a_off, s * CG_KB + i * 64 * a_pitch, 0)
                : __builtin_amdgcn_raw_buffer_load_b128(brs, b_off, s * CG_KB + (i - CG_PIECES_A) * 64 * b_pitch, 0);
            r[i] = make_uint4(v.x, v.y, v.z, v.w);
        }
    };
    auto deposit = [&](const uint4 (&r)[CG_PIECES], uint32_t s) {
        uint8_t *to = cg_lds + (s & 1u) * CG_STAGE + dst0;
#pragma unroll
        for (int i = 0; i < CG_PIECES; ++i) *(uint4 *)(to + i * 64 * CG_PITCH) = r[i];
    };
    const uint32_t nsteps = k_bytes / CG_KB;
    uint4 r0[CG_PIECES], r1[CG_PIECES];
    // (fetches past the last stage are harmless: inside the matrix they read bytes that are never
    // multiplied, past its end zeros -- and being unconditional they keep the count of loads in flight
    // known at every wait, so depositing one stage never waits for the loads of the next)
    // metric of the tile's rows, for the epilogue.  Asked for before the first fetch and stored with the first stage:
    // waiting for it later would wait for every fetch issued before it, and the loop would be entered with no load
    // outstanding -- from which the compiler concludes (the loop's waits must hold on every path into it) that the
    // deposits inside the loop have to wait for ALL outstanding loads, the set fetched one stage ago included, which
    // halves the distance the fetches run ahead.
    uint32_t *row_is_ip = (uint32_t *)(cg_lds + CG_LDS);
    const uint32_t ml0 = tid < a_rows ? tid : a_rows - 1;
    const uint32_t my_metric = row_metric ? row_metric[(size_t)(bm + ml0) * metric_stride] : fixed_metric;
    asm volatile("" ::: "memory");
    fetch(r0, 0);
    deposit(r0, 0);
    row_is_ip[tid] = my_metric;
    asm volatile("" ::: "memory");          // (the issue order of the two sets must be the loop's: older set first)
    fetch(r1, 1);
    asm volatile("" ::: "memory");
    fetch(r0, 2);
    asm volatile("" ::: "memory");
    __syncthreads();

    tri_f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const uint32_t fr = lane & 31, fk = (lane >> 5) * 16;
    const uint32_t a_frag = (wm * 128 + fr) * CG_PITCH + fk;
    const uint32_t b_frag = (CG_BM + wn * 64 + fr) * CG_PITCH + fk;

    // One stage: multiply LDS stage `cur`, then move `ready` (stage s+1, loaded two stages ago) into the
    // other half and refill it with stage s+3.
    auto stage = [&](uint32_t s, uint4 (&ready)[CG_PIECES]) {
        const uint8_t *cur = cg_lds + (s & 1u) * CG_STAGE;
#pragma unroll
        for (int c = 0; c < CG_KB / 32; ++c) {
            uint4 af[4], bf[2];
#pragma unroll
            for (int i = 0; i < 4; ++i) af[i] = *(const uint4 *)(cur + a_frag + i * 32 * CG_PITCH + c * 32);
#pragma unroll
            for (int j = 0; j < 2; ++j) bf[j] = *(const uint4 *)(cur + b_frag + j * 32 * CG_PITCH + c * 32);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) tri_mma32<DT>(acc[i][j], af[i], bf[j]);
        }
        deposit(ready, s + 1);
        fetch(ready, s + 3);
        __syncthreads();
    };
    // (rows are multiples of 128 bytes: an even number of stages.  No "if there is a second one" here: a path through
    // the loop that skips the second stage would have the compiler make the first stage's deposits wait for every load
    // in flight, the set fetched one stage ago included)
    for (uint32_t s = 0; s < nsteps; s += 2) {
        stage(s, r1);
        stage(s + 1, r0);
    }

    // epilogue: accumulator r of lane l is (row 8*(r/4) + 4*(l/32) + r%4, col l%32) of its 32x32 block.
    // Stores go through a descriptor of the tile's rows of C; elements past an edge aim outside it.
    const uint32_t c_rows = a_rows;
    const __amdgpu_buffer_rsrc_t crs = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(C + (size_t)bm * ldc), 0, ((c_rows - 1) * ldc + N) * 4u, 0x00020000);
    float bn2[2];
    uint32_t ncol[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const uint32_t n = bn + wn * 64 + j * 32 + fr;
        bn2[j] = bnorm[n < N ? n : N - 1];
        ncol[j] = n < N ? n * 4u : 0xFFFFFFFCu;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const uint32_t ml = wm * 128 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);   // row inside the tile
            const uint32_t metric = row_is_ip[ml];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const float dot = acc[i][j][r];
                const float v = metric == 0 ? (bn2[j] - 2.0f * dot) : dot;
                const uint32_t off = (ml < c_rows && ncol[j] != 0xFFFFFFFCu) ? ml * ldc * 4u + ncol[j] : 0xFFFFFFFCu;
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), crs, off, 0, 0);
            }
        }
    }
}

template <int DT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void coarse_gemm_kernel(
    const uint8_t *__restrict__ A, uint32_t a_pitch, uint32_t M,
    const uint8_t *__restrict__ B, uint32_t b_pitch, const float *__restrict__ bnorm, uint32_t N,
    uint32_t k_bytes, const uint32_t *__restrict__ row_metric, uint32_t metric_stride, uint32_t fixed_metric,
    float *__restrict__ C, uint32_t ldc)
{
    coarse_gemm_tile<DT>(A, a_pitch, M, B, b_pitch, bnorm, N, k_bytes, row_metric, metric_stride, fixed_metric, C, ldc);
}

// The same contraction for group `gi` of a step's newly admitted queries: rows, index and count come
// from the step's header, so the launch is the same whatever the step admits.  Workgroups beyond the
// group's rows or the index's centroids, and launches whose storage type is not the index's, leave at once.
template <int DT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void coarse_gemm_step_kernel(
    const uint8_t *__restrict__ upload, uint32_t gi, const TriIndexDev *__restrict__ indexes, float *__restrict__ C)
{
    const TriStepHdr *hdr = (const TriStepHdr *)upload;
    if (gi >= hdr->n_groups) return;
    const TriCoarseGroup g = hdr->group[gi];
    const TriIndexDev &ix = indexes[g.index];
    if (ix.dtype != (uint32_t)DT || blockIdx.y * CG_BM >= g.m || blockIdx.x * CG_BN >= ix.nlist) return;
    const TriNewDesc *desc = (const TriNewDesc *)(upload + hdr->desc_off);
    coarse_gemm_tile<DT>(upload + hdr->rows_off + g.row_off, ix.row_bytes, g.m, (const uint8_t *)ix.centroids,
                         ix.row_bytes, ix.cnorm, ix.nlist, ix.row_bytes, &desc[g.first_new].metric,
                         (uint32_t)(sizeof(TriNewDesc) / 4), 0u, C, tri_coarse_ldc(ix.nlist));
}

static hipError_t cg_raise_lds(const void *fn, bool *done)
{
    if (*done) return hipSuccess;                  // (more LDS than a kernel gets by default)
    const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, CG_LDS + CG_BM * 4);
    if (e == hipSuccess) *done = true;
    return e;
}

static bool g_cg_step_lds_set[2] = {false, false};

// What the first step launch of each variant would set up, done ahead.
hipError_t tri_coarse_prepare()
{
    hipError_t e = cg_raise_lds((const void *)coarse_gemm_step_kernel<TRI_DT_F32>, &g_cg_step_lds_set[0]);
    if (e == hipSuccess) e = cg_raise_lds((const void *)coarse_gemm_step_kernel<TRI_DT_F16>, &g_cg_step_lds_set[1]);
    return e;
}

hipError_t tri_launch_coarse_gemm_step(const TriLaunchCtx &c, const TriDevWs &ws, int dtype, uint32_t group,
                                       uint32_t grid_m, uint32_t grid_n)
{
    if (grid_m == 0 || grid_n == 0) return hipSuccess;
    const int v = dtype == TRI_DT_F16 ? 1 : 0;
    const void *fn = v ? (const void *)coarse_gemm_step_kernel<TRI_DT_F16> : (const void *)coarse_gemm_step_kernel<TRI_DT_F32>;
    const hipError_t e = cg_raise_lds(fn, &g_cg_step_lds_set[v]);
    if (e != hipSuccess) return e;
    const dim3 grid((grid_n + CG_BN - 1) / CG_BN, (grid_m + CG_BM - 1) / CG_BM);
    if (v)
        hipLaunchKernelGGL(coarse_gemm_step_kernel<TRI_DT_F16>, grid, dim3(256), CG_LDS + CG_BM * 4, c.stream, ws.upload,
                           group, ws.indexes, ws.coarse_scores);
    else
        hipLaunchKernelGGL(coarse_gemm_step_kernel<TRI_DT_F32>, grid, dim3(256), CG_LDS + CG_BM * 4, c.stream, ws.upload,
                           group, ws.indexes, ws.coarse_scores);
    return hipGetLastError();
}

hipError_t tri_launch_coarse_gemm(hipStream_t s, int dtype, const void *a_rows, uint32_t a_pitch_bytes, uint32_t m,
                                  const void *b_rows, const float *b_norm, uint32_t n, uint32_t row_bytes,
                                  const uint32_t *row_metric, uint32_t metric_stride_u32, uint32_t fixed_metric,
                                  float *scores, uint32_t ldc)
{
    if (m == 0 || n == 0) return hipSuccess;
    if (row_bytes == 0 || row_bytes % (2 * CG_KB) != 0 || a_pitch_bytes % 16 != 0) return hipErrorInvalidValue;
    dim3 grid((n + CG_BN - 1) / CG_BN, (m + CG_BM - 1) / CG_BM);
    static bool lds_set[2] = {false, false};       // (more LDS than a kernel gets by default)
    const int v = dtype == TRI_DT_F16 ? 1 : 0;
    if (!lds_set[v]) {
        const void *fn = v ? (const void *)coarse_gemm_kernel<TRI_DT_F16> : (const void *)coarse_gemm_kernel<TRI_DT_F32>;
        const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, CG_LDS + CG_BM * 4);
        if (e != hipSuccess) return e;
        lds_set[v] = true;
    }
    if (dtype == TRI_DT_F16)
        hipLaunchKernelGGL(coarse_gemm_kernel<TRI_DT_F16>, grid, dim3(256), CG_LDS + CG_BM * 4, s, (const uint8_t *)a_rows,
                           a_pitch_bytes, m, (const uint8_t *)b_rows, row_bytes, b_norm, n, row_bytes, row_metric,
                           metric_stride_u32, fixed_metric, scores, ldc);
    else
        hipLaunchKernelGGL(coarse_gemm_kernel<TRI_DT_F32>, grid, dim3(256), CG_LDS + CG_BM * 4, s, (const uint8_t *)a_rows,
                           a_pitch_bytes, m, (const uint8_t *)b_rows, row_bytes, b_norm, n, row_bytes, row_metric,
                           metric_stride_u32, fixed_metric, scores, ldc);
    return hipGetLastError();
}
