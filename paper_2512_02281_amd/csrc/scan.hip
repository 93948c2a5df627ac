// List scan: the "global distance stage" of the paper's Sec. 3.2 -- fixed-shape kernels that
// evaluate every accumulated distance task of the step.  A task here is (query slot, inverted
// list); tasks on the same list were packed next to each other, so a tile = (list chunk, up to
// TRI_QT of its queries) streams the chunk's vectors from HBM ONCE and scores them against all of
// the tile's queries: a [vectors x dim] x [dim x queries] contraction per 32-vector block on the
// matrix cores, fp32 accumulation.
//
//   L2:  score = |x|^2 + |q|^2 - 2 x.q   (|x|^2 stored at build time, |q|^2 at admission)
//   IP:  score = x.q
//
// Launch shape is fixed (a persistent grid that pulls tiles from a device-side queue); the number
// of real tiles of the step is read from device memory, the rest of the capacity is padding.
//
// Two kernels:
//  * scan_wave_kernel (rows of 512 / 1024 / 1536 bytes): ONE WAVEFRONT PER TILE, no LDS and no
//    barriers.  The wavefront keeps the tile's 32 query rows in registers as MFMA operands (one
//    wavefront per SIMD, so it owns all 512 vector registers) and streams the list through a
//    register ring that holds one to three whole 32-vector blocks: while block b is multiplied,
//    the 16-byte loads of block b + RB are in flight (about 48 KiB per wavefront).  Wavefronts are
//    independent workers on the tile queue, so nothing waits at a barrier for a slower neighbour.
//  * scan_lds_kernel (any other row length): a workgroup of four wavefronts shares the tile's
//    queries through LDS (row pitch = row bytes + 16: conflict-free 16-byte operand reads).
//
// Memory behaviour of both: each lane loads 16-byte pieces straight from the list into MFMA operand
// registers; the four loads a wavefront issues for one 128-byte group cover one full 128-byte line
// of each of its 32 vectors.  Loads go through buffer descriptors sized to the chunk, so rows past
// the end of a list and prefetches past its last block return zeros without touching memory and
// the stream needs no branches.  The issue order is pinned with scheduling barriers, which lets the
// compiler count outstanding loads exactly and wait only for the oldest ones.  Scores leave as
// complete 128-byte lines (32 consecutive vectors of one query per half-wavefront store).
#include "tri_common.h"
#include "tri_mfma.h"

#define SCAN_RING 4   // 128-byte groups in flight per wavefront in the LDS kernel
#define SCAN_BUF_FLAGS 0x00020000

typedef unsigned int scan_u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint4 scan_ld16(__amdgpu_buffer_rsrc_t rs, uint32_t off)
{
    const scan_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Scores of one 32-vector block.  The MFMA takes the query pieces as its first operand, so
// accumulator i of lane l is (query 8*(i/4) + 4*(l/32) + i%4, vector l%32): for a fixed i the 32
// lanes of a half-wavefront hold 32 consecutive vectors of ONE query, and each 4-byte store
// instruction writes two complete 128-byte lines.  Stores go through a buffer descriptor that ends
// after the tile's last query row: lanes whose query does not exist (masked padding) fall outside
// it and are dropped by the hardware, so the epilogue has no branches -- and, being straight-line,
// never makes the stream wait for a store to be acknowledged.
//   qn[i], l2mask: |q|^2 and metric of this lane's 16 queries; vn: |x|^2 of this lane's vector.
//   block_valid = false drops the whole block (a ring slot past the chunk's last block).
__device__ __forceinline__ void scan_store_block(const tri_f32x16 &acc, float vn, const float (&qn)[16],
                                                 uint32_t l2mask, __amdgpu_buffer_rsrc_t ors, uint32_t lane_off,
                                                 uint32_t npad_bytes, bool block_valid)
{
    // The 16 values are first all computed into registers of their own (pinned to accumulation
    // registers by the empty asm statements) and only then stored: a store reads its data register
    // when it reaches the head of the memory pipeline, behind the prefetches already queued, and
    // re-using one register for the next value would stall the wavefront until then, 16 times a block.
    float v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = (l2mask >> i) & 1u ? (vn + qn[i]) - 2.0f * acc[i] : acc[i];
#pragma unroll
    for (int i = 0; i < 16; ++i) asm volatile("" : "+a"(v[i]));
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t jrel = 8 * (i / 4) + (i % 4);             // + 4*(l/32), folded into lane_off
        const uint32_t o = block_valid ? lane_off + jrel * npad_bytes : 0xFFFFFFFCu;   // (no wrap-around: see sizes)
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v[i]), ors, o, 0, 0);
    }
}

// ================================================================================ wavefront kernel
// NG = 128-byte groups per row, RB = 32-vector blocks held in the register ring.
template <int DT, int NG, int RB>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(1, 1))) void scan_wave_kernel(
    const TriTile *__restrict__ tiles, const TriStepDev *__restrict__ step_dev, uint32_t *__restrict__ tile_counter,
    uint32_t my_class, const uint32_t *__restrict__ sorted_slot, const uint8_t *__restrict__ slot_query,
    uint32_t slot_row_bytes, uint32_t n_slots, const TriSlotMeta *__restrict__ slot_meta,
    const float *__restrict__ slot_qnorm, float *__restrict__ scores)
{
    constexpr uint32_t row_bytes = NG * 128;
    constexpr uint32_t blk_bytes = TRI_VB * row_bytes;
    const uint32_t lane = threadIdx.x;
    const uint32_t r = lane & 31, kg = lane >> 5;
    const uint32_t n_tiles = step_dev->n_tiles;
    const __amdgpu_buffer_rsrc_t qrs =
        __builtin_amdgcn_make_buffer_rsrc((void *)slot_query, 0, n_slots * slot_row_bytes, SCAN_BUF_FLAGS);

    uint32_t t = 0;
    if (lane == 0) t = atomicAdd(tile_counter, 1u);
    t = __builtin_amdgcn_readfirstlane(t);
    while (t < n_tiles) {
        const TriTile tl = tiles[t];
        uint32_t t_next = 0;                    // claimed now, needed only when this tile is done
        if (lane == 0) t_next = atomicAdd(tile_counter, 1u);
        if (tl.klass == my_class) {
            const uint32_t len = tl.vec_count;
            const uint32_t nblocks = (len + TRI_VB - 1) / TRI_VB;
            const __amdgpu_buffer_rsrc_t vrs =
                __builtin_amdgcn_make_buffer_rsrc((void *)tl.vec_addr, 0, len * row_bytes, SCAN_BUF_FLAGS);
            // (sized to whole blocks: a 16-byte load never straddles its end; the norm array has a block of slack)
            const __amdgpu_buffer_rsrc_t nrs =
                __builtin_amdgcn_make_buffer_rsrc((void *)tl.vnorm_addr, 0, nblocks * TRI_VB * 4u, SCAN_BUF_FLAGS);
            // the stream's first RB blocks go out before anything else
            const uint32_t off0 = r * row_bytes + kg * 16;
            uint4 buf[RB][NG][4];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int g = 0; g < NG; ++g) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) buf[rb][g][c] = scan_ld16(vrs, off0 + rb * blk_bytes + g * 128 + c * 32);
                    __builtin_amdgcn_sched_barrier(0);
                }
            // this lane's query (row l%32 of the first MFMA operand): its vector as operand pieces; a
            // lane past nq reads out of range, i.e. zeros (masked padding).  All loads are issued
            // first; the empty asm statements then pin the pieces to accumulation registers, which
            // leaves the architectural ones to the stream ring and avoids copies.
            const uint32_t slot = r < tl.nq ? sorted_slot[tl.item_pos + r] : 0xFFFFFFFFu;
            const bool live = slot != 0xFFFFFFFFu;
            const uint32_t qoff = live ? slot * slot_row_bytes + kg * 16 : 0xFFFF0000u;
            scan_u32x4 qf[NG][4];
#pragma unroll
            for (int g = 0; g < NG; ++g)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    qf[g][c] = __builtin_amdgcn_raw_buffer_load_b128(qrs, qoff + g * 128 + c * 32, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int g = 0; g < NG; ++g)
#pragma unroll
                for (int c = 0; c < 4; ++c) asm volatile("" : "+a"(qf[g][c]));
            // |q|^2 and metric of the 16 queries whose scores this lane will hold
            const float qn_own = live ? slot_qnorm[slot] : 0.f;
            const bool l2_own = live ? slot_meta[slot].metric == 0u : false;
            const uint32_t l2_all = (uint32_t)__ballot(l2_own && lane < 32);
            float qn[16];
            uint32_t l2mask = 0;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const uint32_t j = 8 * (i / 4) + 4 * kg + (i % 4);
                qn[i] = __shfl(qn_own, (int)j, 64);
                l2mask |= ((l2_all >> j) & 1u) << i;
            }
            const uint32_t npad_bytes = tl.npad * 4u;
            const __amdgpu_buffer_rsrc_t ors = __builtin_amdgcn_make_buffer_rsrc(
                (void *)(scores + tl.score_off), 0, ((tl.nq - 1) * tl.npad + nblocks * TRI_VB) * 4u, SCAN_BUF_FLAGS);
            const uint32_t lane_off = 4 * kg * npad_bytes + r * 4;
            __builtin_amdgcn_sched_barrier(0);

            uint32_t off = off0;
            for (uint32_t b = 0; b < nblocks; b += RB) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    // |x|^2 of this lane's vector, issued before the prefetches below so that waiting
                    // for it never waits for them (vector-memory operations complete in order)
                    const float vn = __uint_as_float(
                        __builtin_amdgcn_raw_buffer_load_b32(nrs, ((b + rb) * TRI_VB + r) * 4u, 0, 0));
                    __builtin_amdgcn_sched_barrier(0);
                    tri_f32x16 acc;
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
                    for (int g = 0; g < NG; ++g) {
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            tri_mma32<DT>(acc, make_uint4(qf[g][c].x, qf[g][c].y, qf[g][c].z, qf[g][c].w), buf[rb][g][c]);
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            buf[rb][g][c] = scan_ld16(vrs, off + (RB + rb) * blk_bytes + g * 128 + c * 32);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    scan_store_block(acc, vn, qn, l2mask, ors, lane_off + (b + rb) * (TRI_VB * 4u), npad_bytes,
                                     b + rb < nblocks);
                    __builtin_amdgcn_sched_barrier(0);
                }
                off += RB * blk_bytes;
            }
        }
        t = __builtin_amdgcn_readfirstlane(t_next);
    }
}

// ================================================================================ LDS kernel
struct ScanShared {
    uint32_t slot[TRI_QT];
    float qnorm[TRI_QT];
    uint32_t metric[TRI_QT];
    uint32_t tile;
};

// One tile with a compile-time number NG of 128-byte groups per row (NG % SCAN_RING == 0).  The
// wavefront's blocks b = wave, wave+4, ... form ONE stream of (block, group) steps: while group g is
// multiplied, the loads of the group SCAN_RING steps ahead -- in this block or the wavefront's next
// one -- are already in flight, so the stream does not drain at block boundaries.
template <int DT, int NG>
__device__ __forceinline__ void scan_tile_pipelined(const TriTile &tl, const uint8_t *__restrict__ qlds,
                                                    uint32_t pitch, const ScanShared &sh, float *__restrict__ scores)
{
    static_assert(NG % SCAN_RING == 0, "ring slots must line up across blocks");
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t r = lane & 31, kg = lane >> 5;
    constexpr uint32_t row_bytes = NG * 128;
    const uint32_t len = tl.vec_count;
    const uint32_t nblocks = (len + TRI_VB - 1) / TRI_VB;
    const __amdgpu_buffer_rsrc_t vrs =
        __builtin_amdgcn_make_buffer_rsrc((void *)tl.vec_addr, 0, len * row_bytes, SCAN_BUF_FLAGS);
    const __amdgpu_buffer_rsrc_t nrs =      // whole blocks: a 16-byte load never straddles its end
        __builtin_amdgcn_make_buffer_rsrc((void *)tl.vnorm_addr, 0, nblocks * TRI_VB * 4u, SCAN_BUF_FLAGS);
    const uint8_t *qrow = qlds + r * pitch + kg * 16;
    float qn[16];
    uint32_t l2mask = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t j = 8 * (i / 4) + 4 * kg + (i % 4);
        qn[i] = sh.qnorm[j];
        l2mask |= (sh.metric[j] == 0u ? 1u : 0u) << i;
    }
    const uint32_t npad_bytes = tl.npad * 4u;
    const __amdgpu_buffer_rsrc_t ors = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(scores + tl.score_off), 0, ((tl.nq - 1) * tl.npad + nblocks * TRI_VB) * 4u, SCAN_BUF_FLAGS);
    const uint32_t lane_off = 4 * kg * npad_bytes + r * 4;
    constexpr uint32_t bstride = (TRI_SCAN_THREADS / 64) * TRI_VB * row_bytes;   // to the wavefront's next block

    uint32_t off = (wave * TRI_VB + r) * row_bytes + kg * 16;
    uint4 buf[SCAN_RING][4];
#pragma unroll
    for (int s = 0; s < SCAN_RING; ++s) {
#pragma unroll
        for (int c = 0; c < 4; ++c) buf[s][c] = scan_ld16(vrs, off + s * 128 + c * 32);
        __builtin_amdgcn_sched_barrier(0);
    }
    for (uint32_t b = wave; b < nblocks; b += TRI_SCAN_THREADS / 64, off += bstride) {
        const float vn = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(nrs, (b * TRI_VB + r) * 4u, 0, 0));
        __builtin_amdgcn_sched_barrier(0);
        tri_f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const int s = g % SCAN_RING;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint4 q = *(const uint4 *)(qrow + g * 128 + c * 32);
                tri_mma32<DT>(acc, q, buf[s][c]);
            }
            __builtin_amdgcn_sched_barrier(0);
            const uint32_t nxt = g + SCAN_RING < NG ? off + (g + SCAN_RING) * 128
                                                    : off + bstride + (g + SCAN_RING - NG) * 128;
#pragma unroll
            for (int c = 0; c < 4; ++c) buf[s][c] = scan_ld16(vrs, nxt + c * 32);
            __builtin_amdgcn_sched_barrier(0);
        }
        scan_store_block(acc, vn, qn, l2mask, ors, lane_off + b * (TRI_VB * 4u), npad_bytes, true);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Any row length: same arithmetic, the groups of a block are loaded SCAN_RING at a time without
// overlap across blocks.
template <int DT>
__device__ __forceinline__ void scan_tile_generic(const TriTile &tl, const uint8_t *__restrict__ qlds, uint32_t pitch,
                                                  const ScanShared &sh, float *__restrict__ scores)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t r = lane & 31, kg = lane >> 5;
    const uint32_t row_bytes = tl.row_bytes;
    const uint32_t ngroups = row_bytes / 128;
    const uint32_t len = tl.vec_count;
    const uint32_t nblocks = (len + TRI_VB - 1) / TRI_VB;
    const __amdgpu_buffer_rsrc_t vrs =
        __builtin_amdgcn_make_buffer_rsrc((void *)tl.vec_addr, 0, len * row_bytes, SCAN_BUF_FLAGS);
    const __amdgpu_buffer_rsrc_t nrs =      // whole blocks: a 16-byte load never straddles its end
        __builtin_amdgcn_make_buffer_rsrc((void *)tl.vnorm_addr, 0, nblocks * TRI_VB * 4u, SCAN_BUF_FLAGS);
    const uint8_t *qrow = qlds + r * pitch + kg * 16;
    float qn[16];
    uint32_t l2mask = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t j = 8 * (i / 4) + 4 * kg + (i % 4);
        qn[i] = sh.qnorm[j];
        l2mask |= (sh.metric[j] == 0u ? 1u : 0u) << i;
    }
    const uint32_t npad_bytes = tl.npad * 4u;
    const __amdgpu_buffer_rsrc_t ors = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(scores + tl.score_off), 0, ((tl.nq - 1) * tl.npad + nblocks * TRI_VB) * 4u, SCAN_BUF_FLAGS);
    const uint32_t lane_off = 4 * kg * npad_bytes + r * 4;

    for (uint32_t b = wave; b < nblocks; b += TRI_SCAN_THREADS / 64) {
        const uint32_t off = (b * TRI_VB + r) * row_bytes + kg * 16;
        const float vn = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(nrs, (b * TRI_VB + r) * 4u, 0, 0));
        tri_f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
        for (uint32_t g0 = 0; g0 < ngroups; g0 += SCAN_RING) {
            uint4 buf[SCAN_RING][4];
#pragma unroll
            for (int s = 0; s < SCAN_RING; ++s)
#pragma unroll
                for (int c = 0; c < 4; ++c)     // groups past the row end: offset forced out of range -> zeros
                    buf[s][c] = scan_ld16(vrs, g0 + s < ngroups ? off + (g0 + s) * 128 + c * 32 : 0xFFFFFFF0u);
#pragma unroll
            for (int s = 0; s < SCAN_RING; ++s) {
                const uint32_t g = g0 + s < ngroups ? g0 + s : 0u;   // (zeros times any valid query piece)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint4 q = *(const uint4 *)(qrow + g * 128 + c * 32);
                    tri_mma32<DT>(acc, q, buf[s][c]);
                }
            }
        }
        scan_store_block(acc, vn, qn, l2mask, ors, lane_off + b * (TRI_VB * 4u), npad_bytes, true);
    }
}

template <int DT, int NG>
__global__ __launch_bounds__(TRI_SCAN_THREADS) __attribute__((amdgpu_waves_per_eu(2, 3))) void scan_lds_kernel(
    const TriTile *__restrict__ tiles, const TriStepDev *__restrict__ step_dev, uint32_t *__restrict__ tile_counter,
    uint32_t my_class, const uint32_t *__restrict__ sorted_slot, const uint8_t *__restrict__ slot_query,
    uint32_t slot_row_bytes, uint32_t n_slots, const TriSlotMeta *__restrict__ slot_meta,
    const float *__restrict__ slot_qnorm, float *__restrict__ scores)
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
        if (tl.klass != my_class) continue;
        const uint32_t row_bytes = tl.row_bytes, pitch = row_bytes + 16;
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
        if constexpr (NG != 0)
            scan_tile_pipelined<DT, NG>(tl, qlds, pitch, sh, scores);
        else
            scan_tile_generic<DT>(tl, qlds, pitch, sh, scores);
    }
}

// ================================================================================ launch
typedef void (*scan_fn)(const TriTile *, const TriStepDev *, uint32_t *, uint32_t, const uint32_t *, const uint8_t *,
                        uint32_t, uint32_t, const TriSlotMeta *, const float *, float *);

struct ScanVariant {
    scan_fn fn;
    bool wave;      // scan_wave_kernel (64 threads, no LDS) or scan_lds_kernel
};

// class = storage type * 5 + (0: other row length, 1..4: 512, 1024, 1536, 2048 bytes per row)
static ScanVariant scan_variant(uint32_t klass)
{
    switch (klass) {
    case 0: return {scan_lds_kernel<TRI_DT_F32, 0>, false};
    case 1: return {scan_wave_kernel<TRI_DT_F32, 4, 3>, true};
    case 2: return {scan_wave_kernel<TRI_DT_F32, 8, 1>, true};
    case 3: return {scan_lds_kernel<TRI_DT_F32, 12>, false};   // (the register-resident form would spill)
    case 4: return {scan_lds_kernel<TRI_DT_F32, 16>, false};
    case 5: return {scan_lds_kernel<TRI_DT_F16, 0>, false};
    case 6: return {scan_wave_kernel<TRI_DT_F16, 4, 3>, true};
    case 7: return {scan_wave_kernel<TRI_DT_F16, 8, 1>, true};
    case 8: return {scan_wave_kernel<TRI_DT_F16, 12, 1>, true};
    default: return {scan_lds_kernel<TRI_DT_F16, 16>, false};
    }
}

static uint32_t g_scan_lds_limit[TRI_SCAN_CLASSES] = {};

// Launch the scan kernels of one step: one per class present in class_mask, each a persistent grid
// sized to what the chip holds at once.
hipError_t tri_launch_scan(const TriLaunchCtx &c, const TriDevWs &ws, uint32_t max_row_bytes, uint32_t class_mask)
{
    for (uint32_t k = 0; k < TRI_SCAN_CLASSES; ++k) {
        if (!(class_mask & (1u << k))) continue;
        const ScanVariant v = scan_variant(k);
        if (v.wave) {
            // one wavefront per SIMD: 4 per compute unit
            hipLaunchKernelGGL(v.fn, dim3(c.n_cu * 4), dim3(64), 0, c.stream, ws.tiles, ws.step_dev,
                               ws.tile_counter + k, k, ws.sorted_slot, ws.slot_query, c.slot_row_bytes, c.S,
                               ws.slot_meta, ws.slot_qnorm, ws.scores);
        } else {
            const uint32_t lds = TRI_QT * (max_row_bytes + 16);
            uint32_t per_cu = (160u * 1024u - 1024u) / (lds + 1024u);
            per_cu = per_cu < 1 ? 1 : (per_cu > 3 ? 3 : per_cu);
            if (lds > g_scan_lds_limit[k]) {
                hipError_t e = hipFuncSetAttribute((const void *)v.fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
                if (e != hipSuccess) return e;
                g_scan_lds_limit[k] = lds;
            }
            hipLaunchKernelGGL(v.fn, dim3(c.n_cu * per_cu), dim3(TRI_SCAN_THREADS), lds, c.stream, ws.tiles,
                               ws.step_dev, ws.tile_counter + k, k, ws.sorted_slot, ws.slot_query, c.slot_row_bytes,
                               c.S, ws.slot_meta, ws.slot_qnorm, ws.scores);
        }
    }
    return hipGetLastError();
}
