// Kernels of index construction (not on the timed path): row padding / gathering, row norms,
// best-centroid reduction, stable partition of rows by list, cluster means.
#include "tri_common.h"

// ------------------------------------------------------------------------------ padded row copy
// dst row i (row_bytes, zero padded past dim) = src row sel(i), where
//   sel(i) = row_sel ? row_sel[i] : (row_mul * i + row_add) % row_mod.
template <typename T>
__global__ void pad_rows_kernel(const T *__restrict__ src, uint32_t dim, uint64_t src_pitch_elems,
                                const uint32_t *__restrict__ row_sel, uint64_t row_mul, uint64_t row_add,
                                uint64_t row_mod, uint64_t nrows, T *__restrict__ dst, uint32_t dpad)
{
    const uint64_t i = blockIdx.x;
    if (i >= nrows) return;
    const uint64_t r = row_sel ? (uint64_t)row_sel[i] : (row_mul * i + row_add) % row_mod;
    const T *s = src + r * src_pitch_elems;
    T *d = dst + i * (uint64_t)dpad;
    for (uint32_t e = threadIdx.x; e < dpad; e += blockDim.x) d[e] = e < dim ? s[e] : (T)0;
}

hipError_t tri_build_pad_rows(hipStream_t s, int dtype, const void *src, uint32_t dim, uint64_t src_pitch_elems,
                              const uint32_t *row_sel, uint64_t row_mul, uint64_t row_add, uint64_t row_mod,
                              uint64_t nrows, void *dst, uint32_t dpad)
{
    if (nrows == 0) return hipSuccess;
    if (nrows > 0x7FFFFFFFull) return hipErrorInvalidValue;
    if (dtype == 1)
        hipLaunchKernelGGL(pad_rows_kernel<_Float16>, dim3((unsigned)nrows), dim3(128), 0, s, (const _Float16 *)src,
                           dim, src_pitch_elems, row_sel, row_mul, row_add, row_mod, nrows, (_Float16 *)dst, dpad);
    else
        hipLaunchKernelGGL(pad_rows_kernel<float>, dim3((unsigned)nrows), dim3(128), 0, s, (const float *)src, dim,
                           src_pitch_elems, row_sel, row_mul, row_add, row_mod, nrows, (float *)dst, dpad);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------ widen / narrow
template <typename T>
__global__ void widen_rows_kernel(const T *__restrict__ src, uint64_t n_elems, float *__restrict__ dst)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_elems) dst[i] = (float)src[i];
}

hipError_t tri_build_widen_rows(hipStream_t s, int dtype, const void *src, uint64_t n_elems, float *dst)
{
    if (n_elems == 0) return hipSuccess;
    const unsigned grid = (unsigned)((n_elems + 255) / 256);
    if (dtype == 1)
        hipLaunchKernelGGL(widen_rows_kernel<_Float16>, dim3(grid), dim3(256), 0, s, (const _Float16 *)src, n_elems, dst);
    else
        hipLaunchKernelGGL(widen_rows_kernel<float>, dim3(grid), dim3(256), 0, s, (const float *)src, n_elems, dst);
    return hipGetLastError();
}

template <typename T>
__global__ void narrow_rows_kernel(const float *__restrict__ src, uint64_t n_elems, T *__restrict__ dst)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_elems) dst[i] = (T)src[i];
}

hipError_t tri_build_convert_centroids(hipStream_t s, int dtype, const float *cent_f32, uint32_t nlist, uint32_t dpad,
                                       void *dst)
{
    const uint64_t n_elems = (uint64_t)nlist * dpad;
    if (n_elems == 0) return hipSuccess;
    const unsigned grid = (unsigned)((n_elems + 255) / 256);
    if (dtype == 1)
        hipLaunchKernelGGL(narrow_rows_kernel<_Float16>, dim3(grid), dim3(256), 0, s, cent_f32, n_elems, (_Float16 *)dst);
    else
        hipLaunchKernelGGL(narrow_rows_kernel<float>, dim3(grid), dim3(256), 0, s, cent_f32, n_elems, (float *)dst);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------ row norms
// |row|^2 in fp32, one wavefront per row: lane-strided partial sums, then a butterfly.
template <typename T>
__global__ __launch_bounds__(256) void row_norms_kernel(const T *__restrict__ rows, uint32_t dpad, uint64_t nrows,
                                                        float *__restrict__ out)
{
    const uint64_t row = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= nrows) return;
    const uint32_t lane = threadIdx.x & 63;
    const T *p = rows + row * dpad;
    float acc = 0.f;
    for (uint32_t e = lane; e < dpad; e += 64) {
        const float f = (float)p[e];
        acc += f * f;
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) acc += __shfl_xor(acc, d, 64);
    if (lane == 0) out[row] = acc;
}

hipError_t tri_build_row_norms(hipStream_t s, int dtype, const void *rows, uint32_t dpad, uint64_t nrows, float *out)
{
    if (nrows == 0) return hipSuccess;
    const unsigned grid = (unsigned)((nrows + 3) / 4);
    if (dtype == 1)
        hipLaunchKernelGGL(row_norms_kernel<_Float16>, dim3(grid), dim3(256), 0, s, (const _Float16 *)rows, dpad, nrows, out);
    else
        hipLaunchKernelGGL(row_norms_kernel<float>, dim3(grid), dim3(256), 0, s, (const float *)rows, dpad, nrows, out);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------ best centroid
// One wavefront per row of the score matrix: best column (L2 smallest / IP largest score as
// written by the coarse contraction), ties -> smaller column.
__global__ __launch_bounds__(256) void argbest_kernel(const float *__restrict__ scores, uint32_t ldc, uint32_t nrows,
                                                      uint32_t ncols, int metric, uint32_t *__restrict__ out)
{
    const uint32_t row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= nrows) return;
    const uint32_t lane = threadIdx.x & 63;
    const float *p = scores + (size_t)row * ldc;
    float best = 0.f;
    uint32_t bj = 0xFFFFFFFFu;
    for (uint32_t j = lane; j < ncols; j += 64) {
        const float v = metric == 0 ? p[j] : -p[j];
        if (bj == 0xFFFFFFFFu || v < best) { best = v; bj = j; }   // strided ascending j: first hit is the smallest j
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) {
        const float ob = __shfl_xor(best, d, 64);
        const uint32_t oj = __shfl_xor(bj, d, 64);
        if (oj != 0xFFFFFFFFu && (bj == 0xFFFFFFFFu || ob < best || (ob == best && oj < bj))) { best = ob; bj = oj; }
    }
    if (lane == 0) out[row] = bj;
}

hipError_t tri_build_argbest(hipStream_t s, const float *scores, uint32_t ldc, uint32_t nrows, uint32_t ncols,
                             int metric, uint32_t *out)
{
    if (nrows == 0) return hipSuccess;
    hipLaunchKernelGGL(argbest_kernel, dim3((nrows + 3) / 4), dim3(256), 0, s, scores, ldc, nrows, ncols, metric, out);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------ stable partition
// Counting sort of the rows by list that keeps ascending row order inside every list.
//   (a) every block counts the labels of its contiguous chunk of rows
//   (b) per list: exclusive prefix of the counts over blocks, list length
//   (c) exclusive prefix of the list lengths (single workgroup)
//   (d) every block places its rows, 256 at a time in row order; inside such a group the rank of a
//       row among the rows with the same label is found by comparing with the labels before it.
__global__ void part_count_kernel(const uint32_t *__restrict__ assign, uint64_t nrows, uint64_t chunk, uint32_t nlist,
                                  uint32_t *__restrict__ block_hist)
{
    const uint64_t b = blockIdx.x;
    const uint64_t r0 = b * chunk, r1 = min(r0 + chunk, nrows);
    uint32_t *h = block_hist + b * nlist;
    for (uint64_t r = r0 + threadIdx.x; r < r1; r += blockDim.x) atomicAdd(&h[assign[r]], 1u);
}

__global__ void part_block_prefix_kernel(uint32_t *__restrict__ block_hist, uint32_t nblocks, uint32_t nlist,
                                         uint32_t *__restrict__ list_len)
{
    const uint32_t l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= nlist) return;
    uint32_t run = 0;
    for (uint32_t b = 0; b < nblocks; ++b) {
        const uint32_t c = block_hist[(size_t)b * nlist + l];
        block_hist[(size_t)b * nlist + l] = run;
        run += c;
    }
    list_len[l] = run;
}

// exclusive prefix over n values by one workgroup of 1024 threads; out has n+1 entries
__global__ __launch_bounds__(1024) void excl_scan_kernel(const uint32_t *__restrict__ in, uint32_t n,
                                                         uint32_t *__restrict__ out)
{
    __shared__ uint32_t s[1024];
    const uint32_t t = threadIdx.x;
    const uint32_t per = (n + 1023) / 1024;
    const uint32_t i0 = min(t * per, n), i1 = min(i0 + per, n);
    uint32_t mine = 0;
    for (uint32_t i = i0; i < i1; ++i) mine += in[i];
    s[t] = mine;
    __syncthreads();
    for (uint32_t d = 1; d < 1024; d <<= 1) {
        const uint32_t a = t >= d ? s[t - d] : 0u;
        __syncthreads();
        s[t] += a;
        __syncthreads();
    }
    uint32_t run = s[t] - mine;
    for (uint32_t i = i0; i < i1; ++i) {
        const uint32_t v = in[i];
        out[i] = run;
        run += v;
    }
    if (t == 1023) out[n] = s[1023];
}

__global__ __launch_bounds__(256) void part_place_kernel(const uint32_t *__restrict__ assign, uint64_t nrows,
                                                         uint64_t chunk, uint32_t nlist,
                                                         uint32_t *__restrict__ block_hist,
                                                         const uint32_t *__restrict__ list_off,
                                                         uint32_t *__restrict__ perm)
{
    __shared__ uint32_t lab[256];
    const uint64_t b = blockIdx.x;
    const uint64_t r0 = b * chunk, r1 = min(r0 + chunk, nrows);
    uint32_t *cur = block_hist + b * nlist;      // running count of this block's rows already placed, per list
    const uint32_t t = threadIdx.x;
    for (uint64_t base = r0; base < r1; base += 256) {
        const uint64_t r = base + t;
        const bool live = r < r1;
        const uint32_t mine = live ? assign[r] : 0xFFFFFFFFu;
        lab[t] = mine;
        __syncthreads();
        uint32_t rank = 0;
        bool last = true;
        if (live) {
            for (uint32_t u = 0; u < t; ++u) rank += lab[u] == mine;
            for (uint32_t u = t + 1; u < 256; ++u)
                if (lab[u] == mine) { last = false; break; }
            perm[list_off[mine] + cur[mine] + rank] = (uint32_t)r;
        }
        __syncthreads();                        // every read of cur[] above precedes the updates below
        if (live && last) cur[mine] += rank + 1;
        __threadfence_block();
        __syncthreads();
    }
}

hipError_t tri_build_partition(hipStream_t s, const uint32_t *assign, uint64_t nrows, uint32_t nlist,
                               uint32_t *block_hist, uint32_t nblocks, uint32_t *list_len_tmp, uint32_t *list_off,
                               uint32_t *perm)
{
    if (nrows == 0 || nblocks == 0) return hipErrorInvalidValue;
    const uint64_t chunk = (nrows + nblocks - 1) / nblocks;
    hipError_t e = tri_launch_fill_u32(s, block_hist, 0u, (size_t)nblocks * nlist);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(part_count_kernel, dim3(nblocks), dim3(256), 0, s, assign, nrows, chunk, nlist, block_hist);
    hipLaunchKernelGGL(part_block_prefix_kernel, dim3((nlist + 255) / 256), dim3(256), 0, s, block_hist, nblocks,
                       nlist, list_len_tmp);
    hipLaunchKernelGGL(excl_scan_kernel, dim3(1), dim3(1024), 0, s, list_len_tmp, nlist, list_off);
    hipLaunchKernelGGL(part_place_kernel, dim3(nblocks), dim3(256), 0, s, assign, nrows, chunk, nlist, block_hist,
                       list_off, perm);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------ cluster means
// One workgroup per list: mean of its member rows (fixed member order, fp32), optionally
// normalised to unit length (spherical k-means).  An empty list keeps its centroid.
template <typename T>
__global__ __launch_bounds__(256) void cluster_means_kernel(const T *__restrict__ rows, uint32_t dpad,
                                                            const uint32_t *__restrict__ list_off,
                                                            const uint32_t *__restrict__ perm, int normalise,
                                                            float *__restrict__ cent)
{
    __shared__ float red[256];
    const uint32_t l = blockIdx.x;
    const uint32_t p0 = list_off[l], p1 = list_off[l + 1];
    if (p0 == p1) return;
    const float inv = 1.0f / (float)(p1 - p0);
    float sq = 0.f;
    for (uint32_t e = threadIdx.x; e < dpad; e += 256) {
        float acc = 0.f;
        for (uint32_t p = p0; p < p1; ++p) acc += (float)rows[(size_t)perm[p] * dpad + e];
        acc *= inv;
        cent[(size_t)l * dpad + e] = acc;
        sq += acc * acc;
    }
    if (!normalise) return;
    red[threadIdx.x] = sq;
    __syncthreads();
    for (uint32_t s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    const float nrm = sqrtf(red[0]);
    if (nrm > 0.f) {
        const float sc = 1.0f / nrm;
        for (uint32_t e = threadIdx.x; e < dpad; e += 256) cent[(size_t)l * dpad + e] *= sc;
    }
}

hipError_t tri_build_cluster_means(hipStream_t s, int dtype, const void *rows, uint32_t dpad, const uint32_t *list_off,
                                   const uint32_t *perm, uint32_t nlist, int normalise, float *cent_f32)
{
    if (nlist == 0) return hipSuccess;
    if (dtype == 1)
        hipLaunchKernelGGL(cluster_means_kernel<_Float16>, dim3(nlist), dim3(256), 0, s, (const _Float16 *)rows, dpad,
                           list_off, perm, normalise, cent_f32);
    else
        hipLaunchKernelGGL(cluster_means_kernel<float>, dim3(nlist), dim3(256), 0, s, (const float *)rows, dpad,
                           list_off, perm, normalise, cent_f32);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------ where every base row is stored
// Storage slot of the vector at stored position p: list l (the one with list_off[l] <= p < list_off[l + 1]) starts at
// block blk_off[l]; slot = 32 * blk_off[l] + (p - list_off[l]).
__device__ __forceinline__ uint32_t build_slot_of(uint32_t p, const uint32_t *__restrict__ list_off,
                                                  const uint32_t *__restrict__ blk_off, uint32_t nlist)
{
    uint32_t lo = 0, hi = nlist;                 // last l with list_off[l] <= p (empty lists share their start: take the last)
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (list_off[mid] <= p) lo = mid; else hi = mid;
    }
    return blk_off[lo] * 32u + (p - list_off[lo]);
}

// inv[ids[p]] = slot of p (ids is a permutation of 0..n-1).
__global__ void slot_map_kernel(const uint32_t *__restrict__ ids, const uint32_t *__restrict__ list_off,
                                const uint32_t *__restrict__ blk_off, uint32_t nlist, uint64_t n, uint32_t *__restrict__ inv)
{
    const uint64_t p = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < n) inv[ids[p]] = build_slot_of((uint32_t)p, list_off, blk_off, nlist);
}

hipError_t tri_build_slot_map(hipStream_t s, const uint32_t *ids, const uint32_t *list_off, const uint32_t *blk_off,
                              uint32_t nlist, uint64_t n, uint32_t *inv)
{
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(slot_map_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, ids, list_off, blk_off, nlist, n, inv);
    return hipGetLastError();
}

// Rows p0 .. p0 + nrows - 1 (stored positions; row-major, pitch row_bytes, in `rows`) into their storage slots: one
// thread per 16-byte piece, consecutive threads take the same piece of consecutive rows (contiguous in the block).
__global__ void interleave_rows_kernel(const uint8_t *__restrict__ rows, uint32_t row_bytes, uint64_t p0, uint32_t nrows,
                                       const uint32_t *__restrict__ ids, const uint32_t *__restrict__ inv,
                                       uint8_t *__restrict__ vecs)
{
    const uint32_t pieces = row_bytes / 16;
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (uint64_t)nrows * pieces) return;
    const uint32_t i = (uint32_t)(t % nrows), j = (uint32_t)(t / nrows);
    const uint32_t slot = inv[ids[p0 + i]];
    const uint4 v = *(const uint4 *)(rows + (size_t)i * row_bytes + j * 16);
    *(uint4 *)(vecs + (size_t)(slot >> 5) * tri_block_stride(row_bytes) + (size_t)j * TRI_PIECE_PITCH + (slot & 31u) * 16u) = v;
}

hipError_t tri_build_interleave_rows(hipStream_t s, const void *rows, uint32_t row_bytes, uint64_t p0, uint32_t nrows,
                                     const uint32_t *ids, const uint32_t *inv, void *vecs)
{
    if (nrows == 0) return hipSuccess;
    const uint64_t total = (uint64_t)nrows * (row_bytes / 16);
    hipLaunchKernelGGL(interleave_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const uint8_t *)rows,
                       row_bytes, p0, nrows, ids, inv, (uint8_t *)vecs);
    return hipGetLastError();
}
