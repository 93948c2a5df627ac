// Admission and packing of one step (paper Sec. 3.2: every running request emits its next units of
// work into one global, cross-request task array; the array has a fixed capacity and unused
// entries are masked).  The work items (slot, list) of all running slots are grouped by inverted
// list, so that the queries probing the same list share one read of it, and cut into scan tiles of
// up to TRI_QT queries.
#include "tri_common.h"

#include <algorithm>

// ---------------------------------------------------------------------------------------- fill
__global__ void fill_u32_kernel(uint32_t *p, uint32_t v, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// The step's upload block (admission records, plan), pulled from pinned host memory by a
// kernel of the pool's own stream: it starts the moment the previous kernel ends, where a runtime copy
// first spends tens of microseconds being set up.  16 bytes per thread and load; how much there is to
// pull stands in the block's own header (first word), so the launch does not depend on it.
__global__ void pull_block_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src_host)
{
    const size_t n16 = ((const TriStepHdr *)src_host)->n16;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src_host[i];
}

hipError_t tri_launch_pull_block(hipStream_t s, void *dst_dev, const void *src_host_as_device, size_t grid_bytes)
{
    const size_t n16 = (grid_bytes + 15) / 16;          // (both buffers are padded to 256 bytes)
    if (n16 == 0) return hipSuccess;
    const unsigned blocks = (unsigned)std::min<size_t>((n16 + 255) / 256, 64);
    hipLaunchKernelGGL(pull_block_kernel, dim3(blocks), dim3(256), 0, s, (uint4 *)dst_dev, (const uint4 *)src_host_as_device);
    return hipGetLastError();
}

hipError_t tri_launch_fill_u32(hipStream_t s, uint32_t *p, uint32_t v, size_t n)
{
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, v, n);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------- stage
// Rows of a caller's device array -> rows of the pool's own store (queries submitted with device-resident
// vectors: from here on the caller's array is no longer needed).  One workgroup per row; the run a row
// belongs to is found by walking the (short) run table, which arrives as a kernel argument.
__global__ __launch_bounds__(256) void stage_rows_kernel(const TriStageRuns runs)
{
    uint32_t row = blockIdx.x, i = 0;
    if (row >= runs.n_rows) return;
    while (i + 1 < runs.n_runs && row >= runs.run[i].count) row -= runs.run[i++].count;
    const uint16_t *src = (const uint16_t *)(runs.src + (uint64_t)(runs.run[i].src_first + row) * runs.src_pitch);
    uint16_t *dst = (uint16_t *)(runs.dst + (uint64_t)(runs.run[i].dst_first + row) * runs.dst_pitch);
    for (uint32_t e = threadIdx.x; e < runs.row_bytes / 2; e += 256) dst[e] = src[e];
}

hipError_t tri_launch_stage_rows(hipStream_t s, const TriStageRuns &runs)
{
    if (runs.n_rows == 0) return hipSuccess;
    hipLaunchKernelGGL(stage_rows_kernel, dim3(runs.n_rows), dim3(256), 0, s, runs);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------- admit
// One workgroup per admitted query: bring its zero-padded row into the slot -- from the pool's pinned
// query store (host-submitted queries) or from the caller's device vector; either is also written to
// the step's row area for the coarse contraction --, compute |q|^2 in fp32 (fixed order: thread-strided partial sums, then a
// tree), write the slot's static description.
template <typename T>
__device__ __forceinline__ float admit_row(const TriNewDesc &d, uint32_t dim, uint32_t dpad, uint8_t *rows,
                                           uint8_t *slot_row)
{
    T *up = (T *)(rows + d.row_off);
    T *dst = (T *)slot_row;
    const T *dev = (const T *)d.src_dev;
    float part = 0.f;
    for (uint32_t e = threadIdx.x; e < dpad; e += 256) {
        const T v = e < dim ? dev[e] : (T)0;
        up[e] = v;
        dst[e] = v;
        const float f = (float)v;
        part += f * f;
    }
    return part;
}

__global__ __launch_bounds__(256) void admit_kernel(uint8_t *__restrict__ upload,
                                                    const TriIndexDev *__restrict__ indexes,
                                                    uint8_t *__restrict__ slot_query, uint32_t slot_row_bytes,
                                                    TriSlotMeta *__restrict__ slot_meta,
                                                    float *__restrict__ slot_qnorm, uint32_t *__restrict__ topk_count)
{
    __shared__ float red[256];
    const TriStepHdr *hdr = (const TriStepHdr *)upload;
    if (blockIdx.x >= hdr->n_new) return;
    const TriNewDesc d = ((const TriNewDesc *)(upload + hdr->desc_off))[blockIdx.x];
    uint8_t *rows = upload + hdr->rows_off;
    const TriIndexDev &ix = indexes[d.index];
    uint8_t *dst = slot_query + (size_t)d.slot * slot_row_bytes;
    const float part = ix.dtype == 1u ? admit_row<_Float16>(d, ix.dim, ix.dpad, rows, dst)
                                      : admit_row<float>(d, ix.dim, ix.dpad, rows, dst);
    red[threadIdx.x] = part;
    __syncthreads();
    for (uint32_t s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        slot_meta[d.slot] = TriSlotMeta{d.index, d.metric, d.k, d.nprobe};
        slot_qnorm[d.slot] = red[0];
        topk_count[d.slot] = 0;
    }
}

hipError_t tri_launch_admit(const TriLaunchCtx &c, const TriDevWs &ws, uint32_t grid_new)
{
    if (grid_new == 0) return hipSuccess;
    hipLaunchKernelGGL(admit_kernel, dim3(grid_new), dim3(256), 0, c.stream, ws.upload, ws.indexes,
                       ws.slot_query, c.slot_row_bytes, ws.slot_meta, ws.slot_qnorm, ws.topk_count);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------- pack
// (1) emit: one thread per work item.  Item i of plan entry e (found by binary search over the
//     entries' item_base) is list probe[slot][cursor + j]; its rank inside the list's group is
//     taken from an atomic counter.  The rank decides only which tile row a query occupies; every
//     score is computed independently of its neighbours, so results do not depend on it.
__global__ void pack_emit_kernel(const uint8_t *__restrict__ upload,
                                 const TriSlotMeta *__restrict__ slot_meta, const TriIndexDev *__restrict__ indexes,
                                 const uint32_t *__restrict__ probe, uint32_t nprobe_max,
                                 uint32_t *__restrict__ item_glist, uint32_t *__restrict__ item_slot,
                                 uint32_t *__restrict__ item_rank, uint32_t *__restrict__ hist)
{
    const TriStepHdr *hdr = (const TriStepHdr *)upload;
    const TriPlanEntry *plan = (const TriPlanEntry *)(upload + hdr->plan_off);
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= hdr->n_items) return;
    uint32_t lo = 0, hi = hdr->n_plan;     // last entry with item_base <= i
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (plan[mid].item_base <= i) lo = mid; else hi = mid;
    }
    const TriPlanEntry e = plan[lo];
    const uint32_t j = i - e.item_base;
    const uint32_t list = probe[(size_t)e.slot * nprobe_max + e.cursor + j];
    const uint32_t g = indexes[slot_meta[e.slot].index].list_base + list;
    item_glist[i] = g;
    item_slot[i] = e.slot;
    item_rank[i] = atomicAdd(&hist[g], 1u);
}

// (2) scan.  Exclusive prefix sums, taken over the attached lists in the order of descending byte
//     length (so the longest tiles are dealt out first and the step ends on the shortest), of: items
//     per list (-> list_start) and tiles per list (-> tile_base, stile_base).
//     Also the step totals and the reset of the work-queue heads.  Up to PACK_SCAN_BLOCKS workgroups,
//     each over a contiguous span of the order, in two launches: FINAL = false leaves every span's
//     totals in block_tot, FINAL = true adds the totals of the spans before its own and writes.
#define PACK_SCAN_BLOCKS 16
#define PACK_SCAN_SUMS 9      // values per span in block_tot (8 used)

template <bool FINAL>
__global__ __launch_bounds__(1024) void pack_scan_kernel(const uint32_t *__restrict__ hist, uint32_t n_order,
                                                         const uint4 *__restrict__ order,
                                                         uint32_t *__restrict__ list_start,
                                                         uint32_t *__restrict__ tile_base,
                                                         uint32_t *__restrict__ stile_base,
                                                         TriStepDev *__restrict__ step_dev,
                                                         uint32_t *__restrict__ tile_counter,
                                                         const TriStepHdr *__restrict__ hdr,
                                                         uint64_t *__restrict__ block_tot,
                                                         TriStepDev *__restrict__ step_host)
{
    __shared__ uint32_t s_items[1024], s_tiles[1024], s_lists[1024], s_stiles[1024];
    __shared__ uint64_t s_scores[1024], s_tbytes[1024], s_ubytes[1024], s_lbytes[1024];
    const uint32_t t = threadIdx.x;
    const uint32_t min_chunk = hdr->min_chunk;
    const uint32_t span = (n_order + gridDim.x - 1) / gridDim.x;
    const uint32_t s0 = min(blockIdx.x * span, n_order), s1 = min(s0 + span, n_order);
    const uint32_t per = (span + 1023) / 1024;
    const uint32_t i0 = min(s0 + t * per, s1), i1 = min(i0 + per, s1);
    uint32_t items = 0, tiles = 0, lists = 0, stiles = 0;
    uint64_t sc = 0, tb = 0, ub = 0, lb = 0;
    // (entries {list, length, row bytes, chunks} are static; only the item counts are gathered, several at once)
    for (uint32_t ib = i0; ib < i1; ib += 8) {
        uint4 o[8];
        uint32_t cnt[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) o[u] = ib + u < i1 ? order[ib + u] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int u = 0; u < 8; ++u) cnt[u] = ib + u < i1 ? hist[o[u].x] : 0u;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t c = cnt[u];
            if (c) {
                const uint32_t len = o[u].y;
                const uint32_t nt = (c + TRI_QT - 1) / TRI_QT;
                // (bytes the MAIN scan launch has to read: the list without its first block, which the sample launch scores)
                const uint64_t bytes = (uint64_t)(len > TRI_SAMPLE_VECS ? len - TRI_SAMPLE_VECS : 0u) * o[u].z;
                items += c;
                tiles += nt * ((len + tri_chunk_vecs(len, min_chunk) - 1) / tri_chunk_vecs(len, min_chunk));
                stiles += len ? nt : 0;
                lists += 1;
                sc += (uint64_t)c * 2u * ((len + TRI_VB - 1) / TRI_VB * TRI_VB);
                tb += bytes * nt;
                ub += bytes;
                lb += (uint64_t)len * o[u].z;
            }
        }
    }
    s_items[t] = items; s_tiles[t] = tiles; s_lists[t] = lists; s_stiles[t] = stiles;
    s_scores[t] = sc; s_tbytes[t] = tb; s_ubytes[t] = ub; s_lbytes[t] = lb;
    __syncthreads();
    // Hillis-Steele inclusive scan over the 1024 thread totals
    for (uint32_t d = 1; d < 1024; d <<= 1) {
        uint32_t a = 0, b = 0, l = 0, e = 0;
        uint64_t x = 0, y = 0, z = 0, w8 = 0;
        if (t >= d) {
            a = s_items[t - d]; b = s_tiles[t - d]; l = s_lists[t - d]; e = s_stiles[t - d];
            x = s_scores[t - d]; y = s_tbytes[t - d]; z = s_ubytes[t - d]; w8 = s_lbytes[t - d];
        }
        __syncthreads();
        s_items[t] += a; s_tiles[t] += b; s_lists[t] += l; s_stiles[t] += e;
        s_scores[t] += x; s_tbytes[t] += y; s_ubytes[t] += z; s_lbytes[t] += w8;
        __syncthreads();
    }
    if (!FINAL) {
        if (t == 1023) {
            uint64_t *o = block_tot + blockIdx.x * PACK_SCAN_SUMS;
            o[0] = s_items[t]; o[1] = s_tiles[t]; o[2] = s_lists[t]; o[3] = s_stiles[t];
            o[4] = s_scores[t]; o[5] = s_tbytes[t]; o[6] = s_ubytes[t]; o[7] = s_lbytes[t];
        }
        return;
    }
    uint64_t base[PACK_SCAN_SUMS - 1] = {};      // totals of the spans before this one
    for (uint32_t b = 0; b < blockIdx.x; ++b)
#pragma unroll
        for (int v = 0; v < PACK_SCAN_SUMS - 1; ++v) base[v] += block_tot[b * PACK_SCAN_SUMS + v];
    uint32_t it = (uint32_t)base[0] + s_items[t] - items, ti = (uint32_t)base[1] + s_tiles[t] - tiles,
             sti = (uint32_t)base[3] + s_stiles[t] - stiles;
    for (uint32_t ib = i0; ib < i1; ib += 8) {
        uint4 o[8];
        uint32_t cnt[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) o[u] = ib + u < i1 ? order[ib + u] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int u = 0; u < 8; ++u) cnt[u] = ib + u < i1 ? hist[o[u].x] : 0u;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (ib + u >= i1) break;
            const uint32_t g = o[u].x, c = cnt[u], len = o[u].y;
            list_start[g] = it;
            tile_base[g] = ti;
            stile_base[g] = sti;
            if (c) {
                it += c;
                ti += (c + TRI_QT - 1) / TRI_QT * ((len + tri_chunk_vecs(len, min_chunk) - 1) / tri_chunk_vecs(len, min_chunk));
                sti += len ? (c + TRI_QT - 1) / TRI_QT : 0;
            }
        }
    }
    if (t == 1023 && blockIdx.x == gridDim.x - 1) {
        step_dev->n_tiles = (uint32_t)base[1] + s_tiles[t];
        step_dev->n_sample_tiles = (uint32_t)base[3] + s_stiles[t];
        step_dev->n_lists_touched = (uint32_t)base[2] + s_lists[t];
        step_dev->total_scores = base[4] + s_scores[t];
        step_dev->tile_vec_bytes = base[5] + s_tbytes[t];
        step_dev->unique_vec_bytes = base[6] + s_ubytes[t];
        step_dev->list_bytes = base[7] + s_lbytes[t];
        if (step_host) *step_host = *step_dev;       // a copy for the host's statistics (pinned host memory)
        for (uint32_t k = 0; k < 2 * TRI_SCAN_CLASSES; ++k) tile_counter[k] = 0;
    }
}

// (3) scatter: one thread per item -> list-sorted slot array.
__device__ __forceinline__ void pack_scatter(uint32_t i, const TriStepHdr *__restrict__ hdr, const uint32_t *__restrict__ item_glist,
                                             const uint32_t *__restrict__ item_slot, const uint32_t *__restrict__ item_rank,
                                             const uint32_t *__restrict__ list_start, uint32_t *__restrict__ sorted_slot,
                                             uint32_t *__restrict__ item_sorted_pos)
{
    if (i >= hdr->n_items) return;
    const uint32_t g = item_glist[i], r = item_rank[i];
    sorted_slot[list_start[g] + r] = item_slot[i];
    item_sorted_pos[i] = list_start[g] + r;
}

// (4) tiles: one thread per list of the pool-wide table.  A list longer than its chunk length is cut into
//     chunks; the tiles of one chunk (one per group of TRI_QT queries) are adjacent in the queue.  Every
//     list also gets its sample tiles (first TRI_SAMPLE_VECS vectors, one per group of queries).  This is the
//     last reader of the histogram: it puts the list's count back to zero, which is how the next step finds it.
__device__ __forceinline__ void pack_tiles(uint32_t g, uint32_t total_lists, uint32_t *__restrict__ hist,
                                           const uint32_t *__restrict__ list_start, const uint32_t *__restrict__ tile_base,
                                           const uint32_t *__restrict__ stile_base,
                                           const uint32_t *__restrict__ glist_len, const uint32_t *__restrict__ glist_voff,
                                           const uint32_t *__restrict__ glist_index, const TriIndexDev *__restrict__ indexes,
                                           const TriStepHdr *__restrict__ hdr, TriTile *__restrict__ tiles,
                                           TriTile *__restrict__ stiles)
{
    if (g >= total_lists) return;
    const uint32_t min_chunk = hdr->min_chunk;
    const uint32_t c = hist[g];
    const uint32_t len = glist_len[g];
    if (c) hist[g] = 0;
    if (!c || !len) return;
    const TriIndexDev &ix = indexes[glist_index[g]];
    const uint32_t nt = (c + TRI_QT - 1) / TRI_QT;
    const uint32_t chunk_vecs = tri_chunk_vecs(len, min_chunk);
    const uint32_t nchunks = (len + chunk_vecs - 1) / chunk_vecs;
    const uint32_t voff = glist_voff[g];
    // the list's blocks of 32 interleaved vectors (a chunk is a whole number of blocks)
    const uint64_t list_addr = (uint64_t)(uintptr_t)ix.vecs + (uint64_t)ix.blk_off[g - ix.list_base] * tri_block_stride(ix.row_bytes);
    TriTile tl;
    tl.klass = tri_scan_class(ix.dtype, ix.row_bytes);
    tl.row_bytes = ix.row_bytes;
    uint32_t w = tile_base[g];
    for (uint32_t ch = 0; ch < nchunks; ++ch) {
        const uint32_t v0 = ch * chunk_vecs;
        tl.vec_addr = list_addr + (uint64_t)(v0 / TRI_VB) * tri_block_stride(ix.row_bytes);
        tl.vnorm_addr = (uint64_t)(uintptr_t)(ix.vnorm + voff + v0);
        tl.vec_count = min(chunk_vecs, len - v0);
        tl.pitch = 0;
        tl.vec_begin = v0;
        tl.chunk = ch;
        tl.out_off = (uint64_t)voff + v0;            // (candidates carry the stored position of their vector)
        for (uint32_t q = 0; q < nt; ++q) {
            tl.item_pos = list_start[g] + q * TRI_QT;
            tl.nq = min((uint32_t)TRI_QT, c - q * TRI_QT);
            tiles[w++] = tl;
        }
    }
    tl.vec_addr = list_addr;
    tl.vnorm_addr = (uint64_t)(uintptr_t)(ix.vnorm + voff);
    tl.vec_count = min((uint32_t)TRI_SAMPLE_VECS, len);
    tl.pitch = TRI_SAMPLE_VECS;
    tl.vec_begin = 0;
    tl.chunk = 0;
    w = stile_base[g];
    for (uint32_t q = 0; q < nt; ++q) {
        tl.item_pos = list_start[g] + q * TRI_QT;
        tl.out_off = (uint64_t)tl.item_pos * TRI_SAMPLE_VECS;
        tl.nq = min((uint32_t)TRI_QT, c - q * TRI_QT);
        stiles[w++] = tl;
    }
}

// (3) + (4) in one launch: the first item_blocks workgroups scatter, the others make tiles (neither reads what
//     the other writes).
__global__ void pack_place_kernel(uint32_t item_blocks, uint32_t total_lists, uint32_t *__restrict__ hist,
                                  const uint32_t *__restrict__ item_glist, const uint32_t *__restrict__ item_slot,
                                  const uint32_t *__restrict__ item_rank, const uint32_t *__restrict__ list_start,
                                  uint32_t *__restrict__ sorted_slot, uint32_t *__restrict__ item_sorted_pos,
                                  const uint32_t *__restrict__ tile_base, const uint32_t *__restrict__ stile_base,
                                  const uint32_t *__restrict__ glist_len, const uint32_t *__restrict__ glist_voff,
                                  const uint32_t *__restrict__ glist_index, const TriIndexDev *__restrict__ indexes,
                                  const TriStepHdr *__restrict__ hdr, TriTile *__restrict__ tiles, TriTile *__restrict__ stiles)
{
    if (blockIdx.x < item_blocks)
        pack_scatter(blockIdx.x * blockDim.x + threadIdx.x, hdr, item_glist, item_slot, item_rank, list_start, sorted_slot,
                     item_sorted_pos);
    else
        pack_tiles((blockIdx.x - item_blocks) * blockDim.x + threadIdx.x, total_lists, hist, list_start, tile_base, stile_base,
                   glist_len, glist_voff, glist_index, indexes, hdr, tiles, stiles);
}

hipError_t tri_launch_pack(const TriLaunchCtx &c, const TriDevWs &ws, uint32_t grid_items, uint32_t total_lists,
                           uint32_t n_order)
{
    if (total_lists == 0) return hipSuccess;
    const TriStepHdr *hdr = (const TriStepHdr *)ws.upload;
    // (the histogram of items per list is all zero here: so the pool starts, and so every step leaves it)
    if (grid_items)
        hipLaunchKernelGGL(pack_emit_kernel, dim3((grid_items + 255) / 256), dim3(256), 0, c.stream, ws.upload,
                           ws.slot_meta, ws.indexes, ws.probe, c.nprobe_max, ws.item_glist, ws.item_slot,
                           ws.item_rank, ws.hist);
    const uint32_t nb = std::min<uint32_t>(PACK_SCAN_BLOCKS, (n_order + 1023) / 1024);
    if (nb > 1)
        hipLaunchKernelGGL(pack_scan_kernel<false>, dim3(nb), dim3(1024), 0, c.stream, ws.hist, n_order, ws.glist_order,
                           ws.list_start, ws.tile_base, ws.stile_base, ws.step_dev, ws.tile_counter,
                           hdr, ws.pack_tot, (TriStepDev *)nullptr);
    hipLaunchKernelGGL(pack_scan_kernel<true>, dim3(nb ? nb : 1), dim3(1024), 0, c.stream, ws.hist, n_order, ws.glist_order,
                       ws.list_start, ws.tile_base, ws.stile_base, ws.step_dev, ws.tile_counter, hdr,
                       ws.pack_tot, ws.step_host);
    const uint32_t item_blocks = (grid_items + 255) / 256;
    hipLaunchKernelGGL(pack_place_kernel, dim3(item_blocks + (total_lists + 255) / 256), dim3(256), 0, c.stream, item_blocks,
                       total_lists, ws.hist, ws.item_glist, ws.item_slot, ws.item_rank, ws.list_start, ws.sorted_slot,
                       ws.item_sorted_pos, ws.tile_base, ws.stile_base, ws.glist_len, ws.glist_voff, ws.glist_index,
                       ws.indexes, hdr, ws.tiles, ws.stiles);
    return hipGetLastError();
}
