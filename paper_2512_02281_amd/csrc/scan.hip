// List scan: the batched distance stage of the paper's Sec. 3.2 -- fixed-shape kernels that
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
// Output.  Writing every score would cost far more than its share of bytes (0.7 GB of stores beside
// 15 GB of loads slowed the scan by a quarter), and almost all scores are useless: a query keeps k
// of tens of thousands.  So each step runs the kernels twice:
//  * sample launch (FILTER = false): the first TRI_SAMPLE_VECS vectors of every probed list, all
//    scores written densely; a small kernel then sets each query's threshold to the k-th best of
//    its sample (and running top-k).  A k-th best of a SUBSET of the candidates can only be worse
//    than the k-th best of all of them, so nothing that belongs to the top-k is beyond it.
//  * main launch (FILTER = true): every other vector is scored (the sample was the first two blocks of
//    each list; what passed of it already heads the candidate regions, put there by the threshold
//    kernel), and only the scores not worse than the query's threshold are appended, as (score bits,
//    stored position of the vector) pairs, to the query's region of the candidate buffer: one region per
//    running query and step, sized by the step's plan from what the filter is expected to let through, with
//    a counter that keeps counting when the region is full -- the merge kernel then sees that pairs are
//    missing and scores that query's lists again itself.  The result is exact either way; the threshold
//    only decides how much is written (about k / sample size of the scores).
//
// Two kernels:
//  * scan_wave_kernel (rows of 512 / 1024 bytes, fp16 rows of 1536 / 2048 bytes): ONE WAVEFRONT PER TILE, no barriers.  The wavefront keeps the tile's 32 query rows in registers as MFMA operands (one
//    wavefront per SIMD, so it owns all 512 vector registers) and streams the list through a
//    register ring of RG 128-byte groups: while group g is multiplied, the 16-byte loads of the
//    group RG steps ahead are in flight (16-24 KiB per wavefront, never drained at block or -- apart
//    from the query load -- tile boundaries).  Wavefronts are independent workers on the tile queue,
//    so nothing waits at a barrier for a slower neighbour.  The wavefront's own 33 KiB of LDS only
//    stage the candidates that pass the filter.
//  * scan_lds_kernel (any other row length): a workgroup of four wavefronts shares the tile's
//    queries through LDS (row pitch = row bytes + 16: conflict-free 16-byte operand reads).
//
// Memory behaviour of both: each lane loads 16-byte pieces straight from the list into MFMA operand
// registers.  The index stores a list in blocks of 32 vectors interleaved by 16-byte pieces (piece j of the
// block's vector i at j * 512 + i * 16), which is the order in which a wavefront's lanes want them: lane
// (kg, r) holds piece 8g + 2c + kg of vector r for load (g, c), so every load instruction reads ONE CONTIGUOUS
// KiB -- eight full 128-byte lines, 16 cache accesses per instruction instead of the 64 that 32 rows a row
// length apart cost (the vector cache's tag pipeline was busy or stalled 98 % of the time with row-major lists).
// Loads go through buffer descriptors sized to the chunk's blocks; a lane whose storage slot lies behind the
// chunk's last vector, and prefetches past the last block, ask out of range and get zeros without touching
// memory, so the stream needs no branches.  The issue order is pinned with scheduling barriers, which lets the
// compiler count outstanding loads exactly and wait only for the oldest ones.  Dense scores (sample
// launch) leave as complete 128-byte lines (32 consecutive vectors of one query per half-wavefront
// store); filtered candidates leave in bursts (see scan_stage_block).
#include "tri_common.h"
#include "tri_mfma.h"

#define SCAN_RING 4   // 128-byte groups in flight per wavefront in the LDS kernel
#define SCAN_BUF_FLAGS 0x00020000

typedef unsigned int scan_u32x4 __attribute__((ext_vector_type(4)));

// 16 bytes of a list.  NT: the load is marked non-temporal -- for an index far larger than the last-level cache the
// lists only pass through, and keeping them out of the caches leaves those to the query rows (configuration 4's
// main launch: 5.74 -> 6.36 TB/s).  It costs what the caches would have served: the part of a small index that stays
// resident from step to step, and the second and later reads of a list that more than TRI_QT queries probe in one
// step (one tile per TRI_QT queries: 16384 queries per step on the same index, 64 per list: 4.47 -> 5.41 ms).  Hence a
// choice per launch (tri_scan_streams_lists).
template <bool NT = false>
__device__ __forceinline__ uint4 scan_ld16(__amdgpu_buffer_rsrc_t rs, uint32_t off)
{
    const scan_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, NT ? 2 : 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Where lane (kg, r) starts in block b of a chunk of len vectors: its slot's 16 bytes of piece kg; out of range
// (zeros, no read) when the slot lies behind the chunk's last vector.  (Offsets stay below 2^31: see the index build.)
__device__ __forceinline__ uint32_t scan_lane_off(uint32_t b, uint32_t r, uint32_t kg, uint32_t len, uint32_t blk_bytes)
{
    return b * TRI_VB + r < len ? b * blk_bytes + kg * TRI_PIECE_PITCH + r * 16u : 0x80000000u;
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

// Candidates of a tile are first staged in LDS -- a store instruction that really writes is costly in the
// middle of the stream (vector-memory operations of a wavefront retire in order, so every later wait for a
// prefetched group also waits for the store's acknowledgement from memory), while a block yields only a few
// dozen candidates -- and leave for the queries' regions in a burst when the array could not take another full
// block, or when the tile ends.
//   entry = (score bits, query row in the tile << 27 | position in the tile's chunk); positions are below
//   2^24 (a list is shorter than 2^31 bytes, a row at least 128).
// A burst: count the staged entries per query (LDS), reserve that many pairs in each query's region with ONE
// global atomic per query -- the counter keeps counting past the region's capacity, which is how the merge kernel
// learns that pairs were dropped --, then write the pairs that fit.  The order inside a region carries no meaning.
#define SCAN_STAGE_CAP 4096u            // entries (8 bytes each) of a wavefront's array; a block adds at most TRI_QT * TRI_VB = 1024
#define SCAN_LSTAGE_CAP 3072u           // entries of the array the four wavefronts of the LDS kernel share

// One-wavefront-per-tile kernel: no branches, no vector-memory traffic while staging -- a ballot gives each passing
// lane its place, lanes that did not pass write to a per-lane dump entry behind the array.
__device__ __forceinline__ void scan_stage_block(const tri_f32x16 &acc, float vn, const float (&qn)[16],
                                                 uint32_t l2mask, const uint32_t (&thr)[16], uint32_t kg, uint32_t lane,
                                                 uint32_t nq, bool vec_ok, uint32_t chunk_pos, uint2 *stage,
                                                 uint32_t &stage_n)
{
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t j = 8 * (i / 4) + 4 * kg + (i % 4);
        const bool is_l2 = (l2mask >> i) & 1u;
        const float v = is_l2 ? (vn + qn[i]) - 2.0f * acc[i] : acc[i];
        const uint32_t key = tri_score_key(v, is_l2 ? 0u : 1u);
        const bool pass = vec_ok && j < nq && key <= thr[i];
        const uint64_t m = __ballot(pass);
        const uint32_t before = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
        stage[pass ? stage_n + before : SCAN_STAGE_CAP + lane] = make_uint2(__float_as_uint(v), (j << 27) | chunk_pos);
        stage_n += (uint32_t)__popcll(m);
    }
}

// Burst of a wavefront's staged candidates.  qloc / qbase: LDS scratch per query row; qoff / qcap: the queries'
// regions; slot: this lane's query (lanes below nq); pos_base: stored position of the chunk's first vector.
__device__ __forceinline__ void scan_stage_flush(const uint2 *stage, uint32_t &stage_n, uint32_t *qloc, uint32_t *qbase,
                                                 const uint32_t *qoff, const uint32_t *qcap, uint32_t lane, uint32_t nq,
                                                 uint32_t slot, uint32_t *__restrict__ slot_cand_cnt,
                                                 uint2 *__restrict__ cand, uint32_t pos_base)
{
    __builtin_amdgcn_wave_barrier();
    if (lane < TRI_QT) qloc[lane] = 0;
    __builtin_amdgcn_wave_barrier();
    for (uint32_t e = lane; e < stage_n; e += 64) atomicAdd(&qloc[stage[e].y >> 27], 1u);
    __builtin_amdgcn_wave_barrier();
    if (lane < nq) {
        const uint32_t c = qloc[lane];
        qbase[lane] = c ? atomicAdd(&slot_cand_cnt[slot], c) : 0u;
        qloc[lane] = 0;
    }
    __builtin_amdgcn_wave_barrier();
    for (uint32_t e = lane; e < stage_n; e += 64) {
        const uint2 en = stage[e];
        const uint32_t j = en.y >> 27;
        const uint32_t pos = qbase[j] + atomicAdd(&qloc[j], 1u);
        if (pos < qcap[j]) cand[(size_t)qoff[j] + pos] = make_uint2(en.x, pos_base + (en.y & 0x07FFFFFFu));
    }
    __builtin_amdgcn_wave_barrier();
    stage_n = 0;
}

// ================================================================================ wavefront kernel
// NG = 128-byte groups per row, RG = groups held in the register ring (NG % RG == 0): while group g
// of a block is multiplied, the loads of the group RG steps ahead -- in this block or the next --
// are in flight.
template <int DT, int NG, int RG, bool FILTER, bool NT>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(1, 1))) void scan_wave_kernel(
    const TriTile *__restrict__ tiles, const uint32_t *__restrict__ n_tiles_ptr, uint32_t *__restrict__ tile_counter,
    uint32_t my_class, const uint32_t *__restrict__ sorted_slot, const uint8_t *__restrict__ slot_query,
    uint32_t slot_row_bytes, uint32_t n_slots, const TriSlotMeta *__restrict__ slot_meta,
    const float *__restrict__ slot_qnorm, const uint32_t *__restrict__ thr_key,
    const uint32_t *__restrict__ slot_cand_off, const uint32_t *__restrict__ slot_cand_cap,
    uint32_t *__restrict__ slot_cand_cnt, void *__restrict__ out_buf)
{
    static_assert(NG % RG == 0, "ring slots must line up across blocks");
    constexpr uint32_t row_bytes = NG * 128;
    constexpr uint32_t blk_bytes = TRI_VB * row_bytes;
    const uint32_t lane = threadIdx.x;
    const uint32_t r = lane & 31, kg = lane >> 5;
    const uint32_t n_tiles = *n_tiles_ptr;
    const __amdgpu_buffer_rsrc_t qrs =
        __builtin_amdgcn_make_buffer_rsrc((void *)slot_query, 0, n_slots * slot_row_bytes, SCAN_BUF_FLAGS);
    // candidate staging of this wavefront (the workgroup IS one wavefront) + 64 dump entries
    __shared__ uint2 stage[FILTER ? SCAN_STAGE_CAP + 64 : 1];
    __shared__ uint32_t rg_loc[TRI_QT], rg_base[TRI_QT], rg_off[TRI_QT], rg_cap[TRI_QT];   // the queries' candidate regions

    uint32_t t = 0;
    if (lane == 0) t = atomicAdd(tile_counter, 1u);
    t = __builtin_amdgcn_readfirstlane(t);
    TriTile tl_ahead = tiles[t < n_tiles ? t : 0u];        // (the queue's capacity is never zero)
    while (t < n_tiles) {
        const TriTile tl = tl_ahead;
        uint32_t t_next = 0;                    // claimed now, needed only when this tile is done
        if (lane == 0) t_next = atomicAdd(tile_counter, 1u);
        bool ahead = false;                     // the next tile's descriptor has been asked for
        if (tl.klass == my_class) {
            const uint32_t len = tl.vec_count;
            const uint32_t nblocks = (len + TRI_VB - 1) / TRI_VB;
            const __amdgpu_buffer_rsrc_t vrs =         // (whole blocks: that is how the chunk is stored)
                __builtin_amdgcn_make_buffer_rsrc((void *)tl.vec_addr, 0, nblocks * blk_bytes, SCAN_BUF_FLAGS);
            // (sized to whole blocks: the norm array has a block of slack)
            const __amdgpu_buffer_rsrc_t nrs =
                __builtin_amdgcn_make_buffer_rsrc((void *)tl.vnorm_addr, 0, nblocks * TRI_VB * 4u, SCAN_BUF_FLAGS);
            // (main launch: the first TRI_SAMPLE_VECS vectors of a list were scored by the sample launch, and what
            // passed of them already heads the candidate regions; the scan of a list's first chunk starts behind them)
            const uint32_t b0 = FILTER && tl.vec_begin == 0 ? TRI_SAMPLE_VECS / TRI_VB : 0u;
            // the stream's first RG groups go out before anything else
            // (lane l = (kg, r) holds pieces 8g + 2c + kg of vector r: its 16 bytes of load (g, c) lie at
            // (8g + 2c + kg) * 512 + r * 16 of the block, so one load instruction reads one contiguous KiB; a lane
            // whose slot lies behind the chunk's last vector asks out of range and gets zeros without a read)
            uint32_t off = scan_lane_off(b0, r, kg, len, blk_bytes);
            uint4 buf[RG][4];
#pragma unroll
            for (int g = 0; g < RG; ++g) {
#pragma unroll
                for (int c = 0; c < 4; ++c) buf[g][c] = scan_ld16<NT>(vrs, off + g * 4096 + c * 1024);
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
            // |q|^2, metric and threshold of the 16 queries whose scores this lane will hold
            const float qn_own = live ? slot_qnorm[slot] : 0.f;
            const bool l2_own = live ? slot_meta[slot].metric == 0u : false;
            const uint32_t thr_own = FILTER && live ? thr_key[slot] : 0u;
            if constexpr (FILTER) {
                if (lane < TRI_QT) {
                    rg_off[lane] = live ? slot_cand_off[slot] : 0u;
                    rg_cap[lane] = live ? slot_cand_cap[slot] : 0u;
                }
            }
            const uint32_t l2_all = (uint32_t)__ballot(l2_own && lane < 32);
            float qn[16];
            uint32_t thr[16];
            uint32_t l2mask = 0;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const uint32_t j = 8 * (i / 4) + 4 * kg + (i % 4);
                qn[i] = __shfl(qn_own, (int)j, 64);
                thr[i] = (uint32_t)__shfl((int)thr_own, (int)j, 64);
                l2mask |= ((l2_all >> j) & 1u) << i;
            }
            uint32_t stage_n = 0;
            const uint32_t pitch_bytes = tl.pitch * 4u;
            // sample launch: the tile's dense rows of nblocks*32 scores
            const __amdgpu_buffer_rsrc_t ors = __builtin_amdgcn_make_buffer_rsrc(
                (void *)((float *)out_buf + (FILTER ? 0 : tl.out_off)), 0,
                FILTER ? 0u : ((tl.nq - 1) * tl.pitch + nblocks * TRI_VB) * 4u, SCAN_BUF_FLAGS);
            const uint32_t lane_off = 4 * kg * pitch_bytes + r * 4;
            const uint32_t pos_base = (uint32_t)tl.out_off;     // (main launch: stored position of the chunk's first vector)
            __builtin_amdgcn_sched_barrier(0);

            for (uint32_t b = b0; b < nblocks; ++b) {
                const uint32_t off_next = scan_lane_off(b + 1, r, kg, len, blk_bytes);
                // |x|^2 of this lane's vector, issued before the prefetches below so that waiting
                // for it never waits for them (vector-memory operations complete in order)
                const float vn = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(nrs, (b * TRI_VB + r) * 4u, 0, 0));
                __builtin_amdgcn_sched_barrier(0);
                tri_f32x16 acc;
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    const int sl = g % RG;
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        tri_mma32<DT>(acc, make_uint4(qf[g][c].x, qf[g][c].y, qf[g][c].z, qf[g][c].w), buf[sl][c]);
                    __builtin_amdgcn_sched_barrier(0);
                    const uint32_t nxt = g + RG < NG ? off + (g + RG) * 4096 : off_next + (g + RG - NG) * 4096;
#pragma unroll
                    for (int c = 0; c < 4; ++c) buf[sl][c] = scan_ld16<NT>(vrs, nxt + c * 1024);
                    __builtin_amdgcn_sched_barrier(0);
                }
                off = off_next;
                if (!ahead) {
                    // The claim of the next tile has come back by now (it was issued before this tile's first
                    // loads, and loads return in order): its descriptor is fetched while the rest of this tile
                    // streams, through the scalar path, which the vector loads' bookkeeping does not see.
                    const uint32_t tn = __builtin_amdgcn_readfirstlane(t_next);
                    tl_ahead = tiles[tn < n_tiles ? tn : 0u];
                    ahead = true;
                }
                if constexpr (FILTER) {
                    const uint32_t vpos = b * TRI_VB + r;
                    if (stage_n > SCAN_STAGE_CAP - TRI_QT * TRI_VB)     // (uniform, and rare: a few dozen pass per block)
                        scan_stage_flush(stage, stage_n, rg_loc, rg_base, rg_off, rg_cap, lane, tl.nq, slot, slot_cand_cnt,
                                         (uint2 *)out_buf, pos_base);
                    scan_stage_block(acc, vn, qn, l2mask, thr, kg, lane, tl.nq, vpos < len, vpos, stage, stage_n);
                } else {
                    scan_store_block(acc, vn, qn, l2mask, ors, lane_off + b * (TRI_VB * 4u), pitch_bytes, true);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (FILTER)
                scan_stage_flush(stage, stage_n, rg_loc, rg_base, rg_off, rg_cap, lane, tl.nq, slot, slot_cand_cnt,
                                 (uint2 *)out_buf, pos_base);
        }
        t = __builtin_amdgcn_readfirstlane(t_next);
        if (!ahead) tl_ahead = tiles[t < n_tiles ? t : 0u];   // (a tile of another class, or one without a block to score)
    }
}

// ================================================================================ LDS kernel
struct ScanShared {
    uint32_t slot[TRI_QT];
    float qnorm[TRI_QT];
    uint32_t metric[TRI_QT];
    uint32_t thr[TRI_QT];
    uint32_t cnt[TRI_QT], base[TRI_QT];     // scratch of the candidate burst
    uint32_t off[TRI_QT], cap[TRI_QT];      // the queries' regions of the candidate buffer
    uint32_t tile;
    uint32_t stage_n;                       // entries asked for in the workgroup's staging array
};

// What the scan kernels get besides the tile: where the candidates go.
struct ScanOut {
    uint32_t *slot_cand_cnt;
    uint2 *cand;
    uint2 *lstage;          // the LDS kernel's staging array
    uint32_t pos_base;      // stored position of the chunk's first vector
};

// Filtering epilogue of one 32-vector block in the LDS kernel: passing scores are appended to the staging array
// the workgroup's four wavefronts share (one LDS atomic per wavefront and accumulator); should it be full, a
// candidate goes straight to its query's region, one global atomic each.
__device__ __forceinline__ void scan_filter_block(const tri_f32x16 &acc, float vn, const float (&qn)[16],
                                                  uint32_t l2mask, ScanShared &sh, const ScanOut &out, uint32_t kg,
                                                  uint32_t nq, bool vec_ok, uint32_t chunk_pos)
{
    const uint32_t lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t j = 8 * (i / 4) + 4 * kg + (i % 4);
        const bool is_l2 = (l2mask >> i) & 1u;
        const float v = is_l2 ? (vn + qn[i]) - 2.0f * acc[i] : acc[i];
        const uint32_t key = tri_score_key(v, is_l2 ? 0u : 1u);
        const bool pass = vec_ok && j < nq && key <= sh.thr[j];
        const uint64_t m = __ballot(pass);
        if (m) {                                               // (uniform across the wavefront)
            const int leader = __ffsll((unsigned long long)m) - 1;
            uint32_t first = 0;
            if ((int)lane == leader) first = atomicAdd(&sh.stage_n, (uint32_t)__popcll(m));
            first = (uint32_t)__shfl((int)first, leader, 64);
            const uint32_t idx = first + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            if (pass) {
                if (idx < SCAN_LSTAGE_CAP) {
                    out.lstage[idx] = make_uint2(__float_as_uint(v), (j << 27) | chunk_pos);
                } else {
                    const uint32_t pos = atomicAdd(&out.slot_cand_cnt[sh.slot[j]], 1u);
                    if (pos < sh.cap[j]) out.cand[(size_t)sh.off[j] + pos] = make_uint2(__float_as_uint(v), out.pos_base + chunk_pos);
                }
            }
        }
    }
}

// Burst of the workgroup's staged candidates at the end of a tile (all threads; barriers inside).
__device__ __forceinline__ void scan_lds_flush(ScanShared &sh, const ScanOut &out, uint32_t nq)
{
    __syncthreads();                        // every wavefront has staged its candidates
    const uint32_t n = sh.stage_n < SCAN_LSTAGE_CAP ? sh.stage_n : SCAN_LSTAGE_CAP;
    if (threadIdx.x < TRI_QT) sh.cnt[threadIdx.x] = 0;
    __syncthreads();
    for (uint32_t e = threadIdx.x; e < n; e += TRI_SCAN_THREADS) atomicAdd(&sh.cnt[out.lstage[e].y >> 27], 1u);
    __syncthreads();
    if (threadIdx.x < nq) {
        const uint32_t c = sh.cnt[threadIdx.x];
        sh.base[threadIdx.x] = c ? atomicAdd(&out.slot_cand_cnt[sh.slot[threadIdx.x]], c) : 0u;
        sh.cnt[threadIdx.x] = 0;
    }
    __syncthreads();
    for (uint32_t e = threadIdx.x; e < n; e += TRI_SCAN_THREADS) {
        const uint2 en = out.lstage[e];
        const uint32_t j = en.y >> 27;
        const uint32_t pos = sh.base[j] + atomicAdd(&sh.cnt[j], 1u);
        if (pos < sh.cap[j]) out.cand[(size_t)sh.off[j] + pos] = make_uint2(en.x, out.pos_base + (en.y & 0x07FFFFFFu));
    }
}

// One tile with a compile-time number NG of 128-byte groups per row (NG % SCAN_RING == 0).  The
// wavefront's blocks b = wave, wave+4, ... form ONE stream of (block, group) steps: while group g is
// multiplied, the loads of the group SCAN_RING steps ahead -- in this block or the wavefront's next
// one -- are already in flight, so the stream does not drain at block boundaries.
template <int DT, int NG, bool FILTER, bool NT>
__device__ __forceinline__ void scan_tile_pipelined(const TriTile &tl, const uint8_t *__restrict__ qlds,
                                                    uint32_t pitch, ScanShared &sh, float *__restrict__ out_buf,
                                                    const ScanOut &out)
{
    static_assert(NG % SCAN_RING == 0, "ring slots must line up across blocks");
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t r = lane & 31, kg = lane >> 5;
    constexpr uint32_t row_bytes = NG * 128;
    const uint32_t len = tl.vec_count;
    const uint32_t nblocks = (len + TRI_VB - 1) / TRI_VB;
    constexpr uint32_t blk_bytes = TRI_VB * row_bytes;
    const __amdgpu_buffer_rsrc_t vrs =
        __builtin_amdgcn_make_buffer_rsrc((void *)tl.vec_addr, 0, nblocks * blk_bytes, SCAN_BUF_FLAGS);
    const __amdgpu_buffer_rsrc_t nrs =
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
    const uint32_t pitch_bytes = tl.pitch * 4u;
    const __amdgpu_buffer_rsrc_t ors = __builtin_amdgcn_make_buffer_rsrc(       // (sample launch: the tile's dense rows)
        (void *)(out_buf + (FILTER ? 0 : tl.out_off)), 0, FILTER ? 0u : ((tl.nq - 1) * tl.pitch + nblocks * TRI_VB) * 4u,
        SCAN_BUF_FLAGS);
    const uint32_t lane_off = 4 * kg * pitch_bytes + r * 4;
    constexpr uint32_t NWV = TRI_SCAN_THREADS / 64;                              // blocks from one of the wavefront's to its next

    const uint32_t b0 = FILTER && tl.vec_begin == 0 ? TRI_SAMPLE_VECS / TRI_VB : 0u;    // (the sample launch scored the list's first blocks)
    uint32_t off = scan_lane_off(b0 + wave, r, kg, len, blk_bytes);
    uint4 buf[SCAN_RING][4];
#pragma unroll
    for (int s = 0; s < SCAN_RING; ++s) {
#pragma unroll
        for (int c = 0; c < 4; ++c) buf[s][c] = scan_ld16<NT>(vrs, off + s * 4096 + c * 1024);
        __builtin_amdgcn_sched_barrier(0);
    }
    for (uint32_t b = b0 + wave; b < nblocks; b += NWV) {
        const uint32_t off_next = scan_lane_off(b + NWV, r, kg, len, blk_bytes);
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
            const uint32_t nxt = g + SCAN_RING < NG ? off + (g + SCAN_RING) * 4096
                                                    : off_next + (g + SCAN_RING - NG) * 4096;
#pragma unroll
            for (int c = 0; c < 4; ++c) buf[s][c] = scan_ld16<NT>(vrs, nxt + c * 1024);
            __builtin_amdgcn_sched_barrier(0);
        }
        off = off_next;
        if constexpr (FILTER)
            scan_filter_block(acc, vn, qn, l2mask, sh, out, kg, tl.nq, b * TRI_VB + r < len, b * TRI_VB + r);
        else
            scan_store_block(acc, vn, qn, l2mask, ors, lane_off + b * (TRI_VB * 4u), pitch_bytes, true);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Any row length: same arithmetic, the groups of a block are loaded SCAN_RING at a time without
// overlap across blocks.
template <int DT, bool FILTER, bool NT>
__device__ __forceinline__ void scan_tile_generic(const TriTile &tl, const uint8_t *__restrict__ qlds, uint32_t pitch,
                                                  ScanShared &sh, float *__restrict__ out_buf, const ScanOut &out)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t r = lane & 31, kg = lane >> 5;
    const uint32_t row_bytes = tl.row_bytes;
    const uint32_t ngroups = row_bytes / 128;
    const uint32_t len = tl.vec_count;
    const uint32_t nblocks = (len + TRI_VB - 1) / TRI_VB;
    const uint32_t blk_bytes = tri_block_stride(row_bytes);
    const __amdgpu_buffer_rsrc_t vrs =
        __builtin_amdgcn_make_buffer_rsrc((void *)tl.vec_addr, 0, nblocks * blk_bytes, SCAN_BUF_FLAGS);
    const __amdgpu_buffer_rsrc_t nrs =
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
    const uint32_t pitch_bytes = tl.pitch * 4u;
    const __amdgpu_buffer_rsrc_t ors = __builtin_amdgcn_make_buffer_rsrc(       // (sample launch: the tile's dense rows)
        (void *)(out_buf + (FILTER ? 0 : tl.out_off)), 0, FILTER ? 0u : ((tl.nq - 1) * tl.pitch + nblocks * TRI_VB) * 4u,
        SCAN_BUF_FLAGS);
    const uint32_t lane_off = 4 * kg * pitch_bytes + r * 4;

    const uint32_t b0 = FILTER && tl.vec_begin == 0 ? TRI_SAMPLE_VECS / TRI_VB : 0u;    // (the sample launch scored the list's first blocks)
    for (uint32_t b = b0 + wave; b < nblocks; b += TRI_SCAN_THREADS / 64) {
        const uint32_t off = scan_lane_off(b, r, kg, len, blk_bytes);
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
                    buf[s][c] = scan_ld16<NT>(vrs, g0 + s < ngroups ? off + (g0 + s) * 4096 + c * 1024 : 0xFFFFFFF0u);
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
        if constexpr (FILTER)
            scan_filter_block(acc, vn, qn, l2mask, sh, out, kg, tl.nq, b * TRI_VB + r < len, b * TRI_VB + r);
        else
            scan_store_block(acc, vn, qn, l2mask, ors, lane_off + b * (TRI_VB * 4u), pitch_bytes, true);
    }
}

template <int DT, int NG, bool FILTER, bool NT>
__global__ __launch_bounds__(TRI_SCAN_THREADS) __attribute__((amdgpu_waves_per_eu(2, 3))) void scan_lds_kernel(
    const TriTile *__restrict__ tiles, const uint32_t *__restrict__ n_tiles_ptr, uint32_t *__restrict__ tile_counter,
    uint32_t my_class, const uint32_t *__restrict__ sorted_slot, const uint8_t *__restrict__ slot_query,
    uint32_t slot_row_bytes, uint32_t n_slots, const TriSlotMeta *__restrict__ slot_meta,
    const float *__restrict__ slot_qnorm, const uint32_t *__restrict__ thr_key,
    const uint32_t *__restrict__ slot_cand_off, const uint32_t *__restrict__ slot_cand_cap,
    uint32_t *__restrict__ slot_cand_cnt, void *__restrict__ out_buf)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t qlds[];
    __shared__ ScanShared sh;
    __shared__ uint2 lstage[FILTER ? SCAN_LSTAGE_CAP : 1];
    const uint32_t n_tiles = *n_tiles_ptr;
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
            sh.thr[j] = FILTER && slot != 0xFFFFFFFFu ? thr_key[slot] : 0u;
            sh.off[j] = FILTER && slot != 0xFFFFFFFFu ? slot_cand_off[slot] : 0u;
            sh.cap[j] = FILTER && slot != 0xFFFFFFFFu ? slot_cand_cap[slot] : 0u;
            if (j == 0) sh.stage_n = 0;
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
        const ScanOut out = {slot_cand_cnt, (uint2 *)out_buf, lstage, (uint32_t)tl.out_off};
        if constexpr (NG != 0)
            scan_tile_pipelined<DT, NG, FILTER, NT>(tl, qlds, pitch, sh, (float *)out_buf, out);
        else
            scan_tile_generic<DT, FILTER, NT>(tl, qlds, pitch, sh, (float *)out_buf, out);
        if constexpr (FILTER) scan_lds_flush(sh, out, tl.nq);
    }
}

// ================================================================================ launch
typedef void (*scan_fn)(const TriTile *, const uint32_t *, uint32_t *, uint32_t, const uint32_t *, const uint8_t *,
                        uint32_t, uint32_t, const TriSlotMeta *, const float *, const uint32_t *, const uint32_t *,
                        const uint32_t *, uint32_t *, void *);

struct ScanVariant {
    scan_fn fn;
    bool wave;      // scan_wave_kernel (64 threads, no query tile in LDS) or scan_lds_kernel
};

// class = storage type * 5 + (0: other row length, 1..4: 512, 1024, 1536, 2048 bytes per row)
template <bool FILTER, bool NT>
static ScanVariant scan_variant_nt(uint32_t klass)
{
    switch (klass) {
    case 0: return {scan_lds_kernel<TRI_DT_F32, 0, FILTER, NT>, false};
    case 1: return {scan_wave_kernel<TRI_DT_F32, 4, 4, FILTER, NT>, true};
    case 2: return {scan_wave_kernel<TRI_DT_F32, 8, 4, FILTER, NT>, true};
    case 3: return {scan_lds_kernel<TRI_DT_F32, 12, FILTER, NT>, false};   // (the register-resident form spills for fp32 rows this
                                                                        //  wide, whatever the ring length: 150-350 bytes per lane)
    case 4: return {scan_lds_kernel<TRI_DT_F32, 16, FILTER, NT>, false};
    case 5: return {scan_lds_kernel<TRI_DT_F16, 0, FILTER, NT>, false};
    case 6: return {scan_wave_kernel<TRI_DT_F16, 4, 4, FILTER, NT>, true};
    case 7: return {scan_wave_kernel<TRI_DT_F16, 8, 4, FILTER, NT>, true};
    case 8: return {scan_wave_kernel<TRI_DT_F16, 12, 6, FILTER, NT>, true};
    default: return {scan_wave_kernel<TRI_DT_F16, 16, 4, FILTER, NT>, true};   // (2048-byte fp16 rows: 256 query registers + a 4-group ring still fit)
    }
}

template <bool FILTER>
static ScanVariant scan_variant(uint32_t klass, bool nt = false)
{
    return nt ? scan_variant_nt<FILTER, true>(klass) : scan_variant_nt<FILTER, false>(klass);
}

static uint32_t g_scan_lds_limit[4 * TRI_SCAN_CLASSES] = {};     // [non-temporal][sample][class]

// LDS of the workgroup kernels: the query tile at the widest attached row length; a kernel's limit is
// raised (once per growth) before it is first launched with that much.
static uint32_t scan_lds_bytes(uint32_t max_row_bytes) { return TRI_QT * (max_row_bytes + 16); }

static hipError_t scan_raise_lds(const ScanVariant &v, uint32_t slot, uint32_t lds)
{
    uint32_t &limit = g_scan_lds_limit[slot];
    if (lds <= limit) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute((const void *)v.fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) limit = lds;
    return e;
}

// Everything tri_launch_scan would set up on first use, done ahead (so that a recording of the launches
// holds nothing but launches).
hipError_t tri_scan_prepare(uint32_t max_row_bytes, uint32_t class_mask)
{
    for (uint32_t k = 0; k < TRI_SCAN_CLASSES; ++k) {
        if (!(class_mask & (1u << k))) continue;
        for (int var = 0; var < 4; ++var) {
            const bool sample = var & 1, nt = var & 2;
            const ScanVariant v = sample ? scan_variant<false>(k, nt) : scan_variant<true>(k, nt);
            if (v.wave) continue;
            const hipError_t e = scan_raise_lds(v, (nt ? 2 * TRI_SCAN_CLASSES : 0) + (sample ? TRI_SCAN_CLASSES : 0) + k,
                                                scan_lds_bytes(max_row_bytes));
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

// Launch the scan kernels of one step -- the sample launch or the main launch -- one kernel per class
// present in class_mask, each a persistent grid sized to what the chip holds at once.
hipError_t tri_launch_scan(const TriLaunchCtx &c, const TriDevWs &ws, uint32_t max_row_bytes, uint32_t class_mask,
                           bool sample, bool nt)
{
    const TriTile *tiles = sample ? ws.stiles : ws.tiles;
    const uint32_t *n_ptr = sample ? &ws.step_dev->n_sample_tiles : &ws.step_dev->n_tiles;
    void *out = sample ? (void *)ws.sample_scores : (void *)ws.cand;
    for (uint32_t k = 0; k < TRI_SCAN_CLASSES; ++k) {
        if (!(class_mask & (1u << k))) continue;
        const ScanVariant v = sample ? scan_variant<false>(k, nt) : scan_variant<true>(k, nt);
        uint32_t *counter = ws.tile_counter + (sample ? TRI_SCAN_CLASSES : 0) + k;
        if (v.wave) {
            // one wavefront per SIMD: 4 per compute unit
            hipLaunchKernelGGL(v.fn, dim3(c.n_cu * 4), dim3(64), 0, c.stream, tiles, n_ptr, counter, k, ws.sorted_slot,
                               ws.slot_query, c.slot_row_bytes, c.S, ws.slot_meta, ws.slot_qnorm, ws.thr_key,
                               ws.slot_cand_off, ws.slot_cand_cap, ws.slot_cand_cnt, out);
        } else {
            const uint32_t lds = scan_lds_bytes(max_row_bytes);
            uint32_t per_cu = (160u * 1024u - 1024u) / (lds + 1024u + (sample ? 0u : SCAN_LSTAGE_CAP * 8u));
            per_cu = per_cu < 1 ? 1 : (per_cu > 3 ? 3 : per_cu);
            const hipError_t e = scan_raise_lds(v, (nt ? 2 * TRI_SCAN_CLASSES : 0) + (sample ? TRI_SCAN_CLASSES : 0) + k, lds);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(v.fn, dim3(c.n_cu * per_cu), dim3(TRI_SCAN_THREADS), lds, c.stream, tiles, n_ptr, counter,
                               k, ws.sorted_slot, ws.slot_query, c.slot_row_bytes, c.S, ws.slot_meta, ws.slot_qnorm,
                               ws.thr_key, ws.slot_cand_off, ws.slot_cand_cap, ws.slot_cand_cnt, out);
        }
    }
    return hipGetLastError();
}
