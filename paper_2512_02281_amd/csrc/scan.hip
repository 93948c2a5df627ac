// List scan: the "global distance stage" of the paper's Sec. 3.2 -- one fixed-shape kernel that
// evaluates every accumulated distance task of the step.  A task here is (query slot, inverted
// list); tasks on the same list were packed next to each other, so a tile = (list, up to TRI_QT
// of its queries) streams the list's vectors from HBM ONCE and scores them against all of the
// tile's queries: a [vectors x dim] x [dim x queries] contraction per 32-vector block on the
// matrix cores, fp32 accumulation.
//
//   L2:  score = |x|^2 + |q|^2 - 2 x.q   (|x|^2 stored at build time, |q|^2 at admission)
//   IP:  score = x.q
//
// Launch shape is fixed (a persistent grid that pulls tiles from a device-side queue); the number
// of real tiles of the step is read from device memory, the rest of the capacity is padding.
//
// Memory behaviour: each lane loads 16-byte pieces straight from the list into MFMA operand
// registers; the four loads a wavefront issues for one 128-byte group cover one full 128-byte line
// of each of its 32 vectors, and up to SCAN_RING groups (SCAN_RING KiB per wavefront) are in
// flight.  Queries sit in LDS (row pitch = row bytes + 16, which makes the 16-byte operand reads of
// 32 rows conflict-free) and are re-read for every block.  Scores leave as 16-byte stores.
#include "tri_common.h"
#include "tri_mfma.h"

#define SCAN_RING 4   // 128-byte groups in flight per wavefront

struct __attribute__((packed, aligned(4))) ScanF4 {
    float x, y, z, w;
};

struct ScanShared {
    uint32_t slot[TRI_QT];
    float qnorm[TRI_QT];
    uint32_t metric[TRI_QT];
    uint32_t tile;
};

template <int DT>
__device__ __forceinline__ void scan_tile(const TriTile &tl, const TriIndexDev &ix, uint32_t voff, uint32_t len,
                                          const uint8_t *__restrict__ qlds, uint32_t pitch, const ScanShared &sh,
                                          float *__restrict__ scores)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t r = lane & 31, kg = lane >> 5;
    const uint32_t row_bytes = ix.row_bytes;
    const uint32_t ngroups = row_bytes / 128;
    const uint32_t nblocks = (len + TRI_VB - 1) / TRI_VB;
    const uint32_t npad = nblocks * TRI_VB;
    const uint8_t *vbase = (const uint8_t *)ix.vecs + (size_t)voff * row_bytes;
    const float *vnorm = ix.vnorm + voff;
    const uint8_t *qrow = qlds + r * pitch + kg * 16;
    const bool is_l2 = sh.metric[r] == 0u;
    const float qn = sh.qnorm[r];
    float *out_row = scores + tl.score_off + (size_t)r * npad;

    for (uint32_t b = wave; b < nblocks; b += TRI_SCAN_THREADS / 64) {
        uint32_t row = b * TRI_VB + r;
        row = row < len ? row : len - 1;                 // tail rows re-read the last vector
        const uint8_t *p = vbase + (size_t)row * row_bytes + kg * 16;
        tri_f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;

        uint4 buf[SCAN_RING][4];
#pragma unroll
        for (int s = 0; s < SCAN_RING; ++s) {
            if ((uint32_t)s < ngroups) {
#pragma unroll
                for (int c = 0; c < 4; ++c) buf[s][c] = *(const uint4 *)(p + s * 128 + c * 32);
            }
        }
        for (uint32_t g0 = 0; g0 < ngroups; g0 += SCAN_RING) {
#pragma unroll
            for (int s = 0; s < SCAN_RING; ++s) {
                const uint32_t g = g0 + s;
                if (g < ngroups) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const uint4 q = *(const uint4 *)(qrow + g * 128 + c * 32);
                        tri_mma32<DT>(acc, buf[s][c], q);
                    }
                    if (g + SCAN_RING < ngroups) {
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            buf[s][c] = *(const uint4 *)(p + (size_t)(g + SCAN_RING) * 128 + c * 32);
                    }
                }
            }
        }
        // accumulator i of lane l: vector 8*(i/4) + 4*(l/32) + i%4 of the block, query l%32
        if (r < tl.nq) {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const uint32_t v0 = b * TRI_VB + 8 * q4 + 4 * kg;
                float4 o;
                if (is_l2) {
                    const ScanF4 vn = *(const ScanF4 *)(vnorm + v0);   // only 4-byte aligned: lists start anywhere
                    o.x = (vn.x + qn) - 2.0f * acc[4 * q4 + 0];
                    o.y = (vn.y + qn) - 2.0f * acc[4 * q4 + 1];
                    o.z = (vn.z + qn) - 2.0f * acc[4 * q4 + 2];
                    o.w = (vn.w + qn) - 2.0f * acc[4 * q4 + 3];
                } else {
                    o.x = acc[4 * q4 + 0];
                    o.y = acc[4 * q4 + 1];
                    o.z = acc[4 * q4 + 2];
                    o.w = acc[4 * q4 + 3];
                }
                *(float4 *)(out_row + v0) = o;
            }
        }
    }
}

__global__ __launch_bounds__(TRI_SCAN_THREADS) void scan_kernel(
    const TriTile *__restrict__ tiles, const TriStepDev *__restrict__ step_dev, uint32_t *__restrict__ tile_counter,
    const TriIndexDev *__restrict__ indexes, const uint32_t *__restrict__ glist_len,
    const uint32_t *__restrict__ glist_voff, const uint32_t *__restrict__ glist_index,
    const uint32_t *__restrict__ sorted_slot, const uint8_t *__restrict__ slot_query, uint32_t slot_row_bytes,
    const TriSlotMeta *__restrict__ slot_meta, const float *__restrict__ slot_qnorm, float *__restrict__ scores)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t qlds[];
    __shared__ ScanShared sh;
    const uint32_t n_tiles = step_dev->n_tiles;
    for (;;) {
        __syncthreads();                        // previous tile's LDS reads are done
        if (threadIdx.x == 0) sh.tile = atomicAdd(tile_counter, 1u);
        __syncthreads();
        const uint32_t t = sh.tile;
        if (t >= n_tiles) break;                // uniform: every thread of the workgroup leaves here
        const TriTile tl = tiles[t];
        const TriIndexDev &ix = indexes[glist_index[tl.glist]];
        const uint32_t len = glist_len[tl.glist], voff = glist_voff[tl.glist];
        if (len == 0) continue;
        const uint32_t row_bytes = ix.row_bytes, pitch = row_bytes + 16;
        if (threadIdx.x < TRI_QT) {
            const uint32_t j = threadIdx.x;
            const uint32_t slot = j < tl.nq ? sorted_slot[tl.item_pos + j] : 0xFFFFFFFFu;
            sh.slot[j] = slot;
            sh.qnorm[j] = slot != 0xFFFFFFFFu ? slot_qnorm[slot] : 0.f;
            sh.metric[j] = slot != 0xFFFFFFFFu ? slot_meta[slot].metric : 1u;
        }
        __syncthreads();
        // stage the tile's query rows; rows past nq are zero (masked padding)
        const uint32_t n16 = row_bytes / 16;
        for (uint32_t idx = threadIdx.x; idx < TRI_QT * n16; idx += TRI_SCAN_THREADS) {
            const uint32_t j = idx / n16, c = idx - j * n16;
            const uint32_t slot = sh.slot[j];
            uint4 v = make_uint4(0, 0, 0, 0);
            if (slot != 0xFFFFFFFFu) v = *(const uint4 *)(slot_query + (size_t)slot * slot_row_bytes + c * 16);
            *(uint4 *)(qlds + j * pitch + c * 16) = v;
        }
        __syncthreads();
        if (ix.dtype == TRI_DT_F16)
            scan_tile<TRI_DT_F16>(tl, ix, voff, len, qlds, pitch, sh, scores);
        else
            scan_tile<TRI_DT_F32>(tl, ix, voff, len, qlds, pitch, sh, scores);
    }
}

static uint32_t g_scan_lds_limit = 0;

hipError_t tri_scan_configure(uint32_t max_row_bytes)
{
    const uint32_t need = TRI_QT * (max_row_bytes + 16);
    if (need > g_scan_lds_limit) {
        hipError_t e = hipFuncSetAttribute((const void *)scan_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)need);
        if (e != hipSuccess) return e;
        g_scan_lds_limit = need;
    }
    return hipSuccess;
}

hipError_t tri_launch_scan(const TriLaunchCtx &c, const TriDevWs &ws, uint32_t max_row_bytes)
{
    const uint32_t lds = TRI_QT * (max_row_bytes + 16);
    hipError_t e = tri_scan_configure(max_row_bytes);
    if (e != hipSuccess) return e;
    // persistent grid: as many workgroups as fit at once (LDS-limited), each loops over the tile queue
    uint32_t per_cu = (160u * 1024u - 1024u) / (lds + 1024u);
    per_cu = per_cu < 1 ? 1 : (per_cu > 4 ? 4 : per_cu);
    const uint32_t grid = c.n_cu * per_cu;
    hipLaunchKernelGGL(scan_kernel, dim3(grid), dim3(TRI_SCAN_THREADS), lds, c.stream, ws.tiles, ws.step_dev,
                       ws.tile_counter, ws.indexes, ws.glist_len, ws.glist_voff, ws.glist_index, ws.sorted_slot,
                       ws.slot_query, c.slot_row_bytes, ws.slot_meta, ws.slot_qnorm, ws.scores);
    return hipGetLastError();
}
