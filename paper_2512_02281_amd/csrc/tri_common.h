// Shared declarations of the HIP library's translation units (device-side layouts, launchers).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#define TRI_QT 32            // queries per scan tile (columns of one MFMA output block)
#define TRI_VB 32            // vectors per scan block (rows of one MFMA output block)
#define TRI_SEL_THREADS 256  // threads of a selection workgroup
#define TRI_SCAN_THREADS 256 // threads of a scan workgroup (4 wavefronts)
#define TRI_SCAN_CLASSES 10  // scan kernel variants: 2 storage types x (generic + 4 row lengths)
#define TRI_KMAX_POW2 1024   // largest k (and nprobe) a selection can return

// One attached index as the kernels see it.  All pointers are device pointers.
// Stored vectors.  A list occupies whole blocks of TRI_VB = 32 storage slots; inside a block the vectors are
// interleaved by 16-byte pieces: piece j of the vector in slot i of block b lies at
//     vecs + b * tri_block_stride(row_bytes) + j * 512 + i * 16,
// so the 32 pieces that one MFMA operand register of a half-wavefront holds (one piece of each of 32 vectors) are 512
// contiguous bytes and a wavefront's 16-byte load covers one contiguous KiB.  Slots behind a list's last vector hold
// zeros.  "Stored position" p numbers the vectors list-major without the padding (ids, vnorm, candidates);
// "storage slot" = 32 * block + i.  List l starts at block blk_off[l]: the vector at position p of list l is in slot
// 32 * blk_off[l] + (p - list_off[l]).
struct TriIndexDev {
    const void *vecs;        // blocks of 32 interleaved vectors (see above), 256-B aligned
    const float *vnorm;      // |x|^2 per stored vector (list-major order), fp32
    const uint32_t *ids;     // base-row number per stored vector (list-major order)
    const uint32_t *list_off;// [nlist+1] first stored position of each list
    const void *centroids;   // [nlist] rows of pitch row_bytes, index dtype
    const float *cnorm;      // |c|^2 per centroid, fp32
    const uint32_t *inv;     // storage slot of every base row
    const uint32_t *blk_off; // [nlist] first block of each list
    uint32_t dim, dpad, nlist, dtype;
    uint32_t row_bytes;      // dpad * element size, multiple of 128
    uint32_t list_base;      // number of this index's list 0 in the pool-wide list numbering
    uint32_t max_list_len;
    uint32_t pad_;
    uint64_t n;
};

#define TRI_PIECE_PITCH 512u    // bytes between consecutive 16-byte pieces of a stored vector
// Bytes of one block of 32 stored vectors.  (A pad of 256 bytes behind every block, so that lists do not all start at
// the same offset modulo a large power of two, made no measurable difference.)
__host__ __device__ inline uint32_t tri_block_stride(uint32_t row_bytes) { return 32u * row_bytes; }

// First 16-byte piece of the vector in a storage slot; piece j follows at + j * TRI_PIECE_PITCH.
__device__ __forceinline__ const uint8_t *tri_slot_ptr(const TriIndexDev &ix, uint32_t slot)
{
    return (const uint8_t *)ix.vecs + (size_t)(slot >> 5) * tri_block_stride(ix.row_bytes) + (slot & 31u) * 16u;
}
// Byte b of that vector.
__device__ __forceinline__ const uint8_t *tri_slot_byte(const TriIndexDev &ix, uint32_t slot, uint32_t b)
{
    return tri_slot_ptr(ix, slot) + (size_t)(b >> 4) * TRI_PIECE_PITCH + (b & 15u);
}

// Static description of the request in a slot (written at admission).
struct TriSlotMeta {
    uint32_t index;   // which attached index
    uint32_t metric;  // TRI_L2 / TRI_IP
    uint32_t k;
    uint32_t nprobe;
};

// One admitted query in the step's upload block.
struct TriNewDesc {
    uint32_t slot, index, metric, k, nprobe;
    uint32_t row_off;   // byte offset of its padded row inside the step's row area
    uint64_t src_dev;   // GPU address of the query's vector: a row of the pool's pinned query store, or the caller's device vector
};

// One running slot's share of this step.
struct TriPlanEntry {
    uint32_t slot;
    uint32_t cursor;     // probe-list rank of the first list scanned in this step
    uint32_t take;       // lists scanned in this step
    uint32_t item_base;  // first work item of this slot in the unsorted item array
    int32_t retire_idx;  // >= 0: the slot finishes in this step, result goes to this record
    uint32_t cand_cap;   // pairs its region of the candidate buffer holds in this step
    uint32_t cand_off;   // first pair of that region
    uint32_t pad_;
};

// What a step's kernels need to know about it, at the head of the step's upload block.  Every kernel of
// the step reads its counts from here, never from a launch argument, so that the launch sequence of a
// step is the same whatever the step holds (paper Sec. 3.2: a step of fixed shape that can be captured
// once and replayed); grids may be larger than the step needs, the surplus workgroups leave at once.
#define TRI_MAX_COARSE_GROUPS 60
struct TriCoarseGroup {      // newly admitted queries [first_new, first_new + m) target one index
    uint32_t first_new, m, index, row_off;   // row_off: byte offset of the group's first padded row in the row area
};
struct TriStepHdr {
    uint32_t n16;            // 16-byte pieces of the upload block (this header, admission records, plan)
    uint32_t n_new;          // admission records
    uint32_t n_plan;         // plan entries (running slots that take part in this step)
    uint32_t n_items;        // work items of the step
    uint32_t min_chunk;      // chunk length floor of the step (tri_chunk_vecs)
    uint32_t desc_off;       // byte offsets inside the upload block
    uint32_t plan_off;
    uint32_t rows_off;       // row area (filled on the device by the admit kernel)
    uint32_t n_groups;
    uint32_t merge_parity;   // which of the two queue heads of the merge kernels this step uses (alternates with every merge launch)
    uint32_t coarse_parity;  // which set of queue heads the coarse selection of this step uses (alternates with every step that admits queries)
    uint32_t pad_[5];
    TriCoarseGroup group[TRI_MAX_COARSE_GROUPS];
};
static_assert(sizeof(TriStepHdr) == 1024, "header is 1024 bytes");

// One scan tile: up to TRI_QT queries against one chunk (all of it, for short lists) of one inverted
// list.  Self-contained: the scan kernels read nothing else about the list.  Two kinds share the layout:
//  * main tiles: every vector of the chunk is scored; the scores that pass a query's threshold are appended
//    as (score bits, stored position of the vector in its index) pairs to THAT QUERY's region of the
//    candidate buffer (one region per running query and step, sized by the step's plan);
//  * sample tiles: only the first TRI_SAMPLE_VECS vectors of the list, all scores written densely.
struct TriTile {
    uint64_t vec_addr;    // device address of the first vector
    uint64_t vnorm_addr;  // device address of its |x|^2
    uint64_t out_off;     // sample tiles: 4-byte-word offset of query 0's row in the sample buffer (query j at
                          // + j * pitch); main tiles: stored position (in its index) of the tile's first vector
    uint32_t item_pos;    // first of the tile's queries in the list-sorted item array
    uint32_t nq;          // 1..TRI_QT real queries
    uint32_t vec_count;   // vectors to score
    uint32_t pitch;       // sample tiles: words between the rows of consecutive queries
    uint32_t klass;       // which scan kernel serves it (tri_scan_class)
    uint32_t row_bytes;
    uint32_t vec_begin;   // position of the first vector inside its list
    uint32_t chunk;       // chunk number inside the list (main tiles)
};

#define TRI_SAMPLE_VECS 64     // vectors per list scored ahead of the scan to find each query's threshold
#define TRI_THRESH_ITEMS 64    // at most this many items' samples enter one query's threshold (one register per item)

// Order-preserving image of an fp32 score: ascending key = better (bit-flipped for inner product).
__device__ __forceinline__ uint32_t tri_score_key(float f, uint32_t descending)
{
    uint32_t u = __float_as_uint(f);
    if (u == 0x80000000u) u = 0;                       // -0 and +0 are the same score
    u ^= (u >> 31) ? 0xFFFFFFFFu : 0x80000000u;        // ascending float order -> ascending unsigned
    return descending ? ~u : u;
}

__device__ __forceinline__ float tri_key_score(uint32_t key, uint32_t descending)
{
    uint32_t u = descending ? ~key : key;
    u ^= (u >> 31) ? 0x80000000u : 0xFFFFFFFFu;
    return __uint_as_float(u);
}

// Small per-step numbers the device produces for the host (copied back with the results).
struct TriStepDev {
    uint32_t n_tiles;
    uint32_t n_lists_touched;
    uint32_t n_sample_tiles;
    uint32_t pad_;
    uint64_t total_scores;
    uint64_t tile_vec_bytes;    // sum over tiles of list_len * row_bytes
    uint64_t unique_vec_bytes;  // sum over touched lists of (list_len - sample) * row_bytes: what the main launch must read
    uint64_t list_bytes;        // sum over touched lists of list_len * row_bytes: what the whole scan stage must read
};

// Device workspace of a pool, carved once at creation.
struct TriDevWs {
    // persistent per-slot state
    uint8_t *slot_query;      // [S][slot_row_bytes]
    uint8_t *dev_qstore;      // [max_outstanding][slot_row_bytes] rows of device-submitted queries, by ticket number
    TriSlotMeta *slot_meta;   // [S]
    float *slot_qnorm;        // [S]
    uint32_t *probe;          // [S][nprobe_max]
    float *topk_score;        // [S][kmax]
    uint32_t *topk_id;        // [S][kmax]
    uint32_t *topk_count;     // [S]
    // attached indexes and the pool-wide list table
    TriIndexDev *indexes;     // [max_indexes]
    uint32_t *glist_len;      // [max_total_lists]
    uint32_t *glist_voff;     // [max_total_lists] first stored position inside its index
    uint32_t *glist_index;    // [max_total_lists]
    TriStepDev *step_host;    // NULL, or where the step totals are mirrored for the host (pinned host memory)
    uint64_t *pack_tot;       // [16][9] per-span totals of the pack prefix sums
    uint4 *glist_order;       // [max_total_lists] attached lists by descending byte length (scan order):
                              //   {pool-wide list number, length, row bytes, 0}
    // per-step upload block (device copy)
    uint8_t *upload;          // upload_bytes
    // coarse ranking
    float *coarse_scores;     // [coarse_rows][max_nlist]
    // packing
    uint32_t *item_glist;     // [W]
    uint32_t *item_slot;      // [W]
    uint32_t *item_rank;      // [W]
    uint32_t *item_sorted_pos;// [W] position of the item in the list-sorted order
    uint32_t *sorted_slot;    // [W]
    uint32_t *hist;           // [max_total_lists+1]
    uint32_t *list_start;     // [max_total_lists+1]
    uint32_t *tile_base;      // [max_total_lists+1]
    uint32_t *stile_base;     // [max_total_lists+1] first sample tile of each list
    TriTile *tiles;           // [TRI_TILES_PER_ITEM * W]
    TriTile *stiles;          // [W] sample tiles
    uint32_t *tile_counter;   // [2 * TRI_SCAN_CLASSES] work-queue heads of the scan kernels (main, sample)
    float *sample_scores;     // [W * TRI_SAMPLE_VECS]
    uint32_t *thr_key;        // [S] per slot: keys above this cannot reach its top-k
    uint32_t *slot_cand_off;  // [S] this step's region of the slot in the candidate buffer: first pair,
    uint32_t *slot_cand_cap;  // [S]   pairs it holds,
    uint32_t *slot_cand_cnt;  // [S]   pairs asked for so far (beyond cap: not stored, the merge then re-scans)
    uint32_t *rescans;        // [0] slots whose region overflowed and whose lists the merge kernel scored again (since creation);
                              // [1], [2]: entries in merge_queue, one head for each parity of the merge launches (a launch
                              // fills and reads its own and clears the other)
    uint32_t *merge_queue;    // [S] plan entries of the step that the one-wavefront merge did not settle
    uint32_t *coarse_queue;   // [S] rows of the step's coarse groups that the one-wavefront selection did not settle (group g from g.first_new on);
                              // their counts: words 4 + 64 * parity + group of `rescans`
    TriStepDev *step_dev;     // [1]
    uint2 *cand;              // [score_capacity / 2] candidate buffer: (score bits, stored position) pairs
    // results of retiring slots, compact, per step
    uint32_t *res_block;      // [S][1 + 2*kmax]  n, ids[kmax], score bits[kmax]   (pinned host memory of the step
    uint32_t *res_probes;     // [S][nprobe_max]                                    in flight, as the GPU addresses it)
};

struct TriLaunchCtx {
    hipStream_t stream;
    uint32_t S, W, kmax, nprobe_max, max_total_lists, slot_row_bytes, n_cu;
    uint32_t scan_nt;         // 0: the scan kernels may not read the lists with non-temporal loads; 1: they may (the attached
                              // indexes are large, TRI_NT_INDEX_BYTES); 2: they must (TRI_FLAG_STREAM_LISTS)
};

// From this many bytes of attached vectors on (several times the 256 MB last-level cache), the lists may be streamed
// past the caches (non-temporal loads) ...
#define TRI_NT_INDEX_BYTES (1ull << 30)
// ... and only in a step whose lists are mostly read once: a list probed by more than TRI_QT queries is read once per
// tile of TRI_QT queries, the second time from the caches -- unless the first read went past them.  Measured on the
// 15 GB index: 16 queries per list on average +9 %, 64 per list -21 %; on a 3 GB index with 32 per list -10 %; on a
// 1.5 GB index with 24 per list +5 %, and +3.5 % on the two-index stream of configuration 3 (8 lists per query and step).
inline bool tri_scan_streams_lists(uint32_t scan_nt, uint32_t n_items, uint32_t total_lists)
{
    return scan_nt == 2u || (scan_nt == 1u && (uint64_t)n_items <= 24ull * total_lists);
}

// What another engine of the library needs to know of a resident index (tri_api.hip owns the object).
struct tri_index;
struct TriIndexView {
    TriIndexDev dev;
    hipStream_t stream;       // of the pool the index is attached to
    int device;
    uint64_t n;
};
void tri_index_view(const tri_index *ix, TriIndexView *out);

// Record the thread's last error text (what tri_last_error() returns) and hand back `code`.
int tri_fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

// ---- launchers (each returns hipGetLastError() of its launches) -----------------------------
// The kernels of a step read what the step holds from the TriStepHdr at the head of ws.upload; the
// grid_* arguments only size the launches: at least what the step needs (its exact counts, or the
// pool's maxima when the sequence is recorded once for replay).
hipError_t tri_launch_fill_u32(hipStream_t s, uint32_t *p, uint32_t v, size_t n);
hipError_t tri_launch_pull_block(hipStream_t s, void *dst_dev, const void *src_host_as_device, size_t grid_bytes);
hipError_t tri_launch_admit(const TriLaunchCtx &c, const TriDevWs &ws, uint32_t grid_new);
// Copy rows of a caller's device array into rows of the pool's store: run i moves `count` consecutive source
// rows starting at src_first to consecutive store rows starting at dst_first (row_bytes bytes each, a multiple of 2).
#define TRI_STAGE_RUNS 120
struct TriStageRuns {
    uint64_t src, src_pitch, dst, dst_pitch;
    uint32_t row_bytes, n_runs, n_rows, pad_;
    struct { uint32_t src_first, dst_first, count; } run[TRI_STAGE_RUNS];
};
hipError_t tri_launch_stage_rows(hipStream_t s, const TriStageRuns &runs);
// scores[m][ldc] for m rows (pitch a_pitch_bytes) against n rows of b (pitch row_bytes); the metric
// is per row (row_metric[m * metric_stride_u32]) or, with row_metric == NULL, fixed_metric.
hipError_t tri_launch_coarse_gemm(hipStream_t s, int dtype, const void *a_rows, uint32_t a_pitch_bytes,
                                  uint32_t m, const void *b_rows, const float *b_norm, uint32_t n,
                                  uint32_t row_bytes, const uint32_t *row_metric, uint32_t metric_stride_u32,
                                  uint32_t fixed_metric, float *scores, uint32_t ldc);
// the same for group `group` of the step's header (rows of the step's row area against the group's index),
// into ws.coarse_scores with a row pitch of nlist rounded up to 32; dtype = the kernel variant to launch
hipError_t tri_launch_coarse_gemm_step(const TriLaunchCtx &c, const TriDevWs &ws, int dtype, uint32_t group,
                                       uint32_t grid_m, uint32_t grid_n);
hipError_t tri_launch_coarse_select(const TriLaunchCtx &c, const TriDevWs &ws, uint32_t group, uint32_t grid_m, uint32_t nlist);
hipError_t tri_launch_pack(const TriLaunchCtx &c, const TriDevWs &ws, uint32_t grid_items, uint32_t total_lists,
                           uint32_t n_order);
hipError_t tri_launch_scan(const TriLaunchCtx &c, const TriDevWs &ws, uint32_t max_row_bytes, uint32_t class_mask,
                           bool sample, bool nt);
hipError_t tri_launch_threshold(const TriLaunchCtx &c, const TriDevWs &ws, uint32_t grid_plan);
// one-time set-up the launchers above would otherwise do at their first launch (LDS limits)
hipError_t tri_scan_prepare(uint32_t max_row_bytes, uint32_t class_mask);
hipError_t tri_coarse_prepare();
#define TRI_TILES_PER_ITEM 4   // tile capacity = 4 W: a list is cut into at most 4 chunks

// Chunking of a list for the scan: at most TRI_TILES_PER_ITEM chunks of equal length (a multiple of 32
// vectors), none shorter than min_chunk.  min_chunk is chosen per step: large when the step has far more
// tiles than wavefronts anyway (fewer tiles, fewer query loads), small when tiles are few, so that one
// long list does not keep a single wavefront busy for the whole launch.
__host__ __device__ inline uint32_t tri_chunk_vecs(uint32_t len, uint32_t min_chunk)
{
    uint32_t c = (len + TRI_TILES_PER_ITEM - 1) / TRI_TILES_PER_ITEM;
    c = (c + TRI_VB - 1) / TRI_VB * TRI_VB;
    return c > min_chunk ? c : min_chunk;
}

// Row pitch (in scores) of a coarse score block over nlist centroids: whole 128-byte lines.  (256 bytes more per row,
// so that rows do not all start at the same offset modulo 64 KiB, made no measurable difference.)
__host__ __device__ inline uint32_t tri_coarse_ldc(uint32_t nlist) { return (nlist + 31u) / 32u * 32u; }

// Which scan kernel serves an index: 5 classes per storage type (other, 512, 1024, 1536, 2048 bytes per row).
__host__ __device__ inline uint32_t tri_scan_class(uint32_t dtype, uint32_t row_bytes)
{
    const bool special = row_bytes == 512 || row_bytes == 1024 || row_bytes == 1536 || row_bytes == 2048;
    return dtype * 5 + (special ? row_bytes / 512 : 0);
}
hipError_t tri_launch_merge(const TriLaunchCtx &c, const TriDevWs &ws, uint32_t grid_plan, bool keep_probes);

// ---- index construction helpers ------------------------------------------------------------
hipError_t tri_build_pad_rows(hipStream_t s, int dtype, const void *src, uint32_t dim, uint64_t src_pitch_elems,
                              const uint32_t *row_sel, uint64_t row_mul, uint64_t row_add, uint64_t row_mod,
                              uint64_t nrows, void *dst, uint32_t dpad);
hipError_t tri_build_widen_rows(hipStream_t s, int dtype, const void *src, uint64_t n_elems, float *dst);
hipError_t tri_build_convert_centroids(hipStream_t s, int dtype, const float *cent_f32, uint32_t nlist,
                                       uint32_t dpad, void *dst);
hipError_t tri_build_row_norms(hipStream_t s, int dtype, const void *rows, uint32_t dpad, uint64_t nrows,
                               float *out);
hipError_t tri_build_argbest(hipStream_t s, const float *scores, uint32_t ldc, uint32_t nrows, uint32_t ncols,
                             int metric, uint32_t *out);
hipError_t tri_build_partition(hipStream_t s, const uint32_t *assign, uint64_t nrows, uint32_t nlist,
                               uint32_t *block_hist /*[nblocks][nlist]*/, uint32_t nblocks,
                               uint32_t *list_len_tmp /*[nlist]*/, uint32_t *list_off /*[nlist+1]*/,
                               uint32_t *perm /*[nrows]*/);
hipError_t tri_build_slot_map(hipStream_t s, const uint32_t *ids, const uint32_t *list_off, const uint32_t *blk_off,
                              uint32_t nlist, uint64_t n, uint32_t *inv /*[n] storage slot of every base row*/);
hipError_t tri_build_interleave_rows(hipStream_t s, const void *rows /*row-major, pitch row_bytes*/, uint32_t row_bytes,
                                     uint64_t p0, uint32_t nrows, const uint32_t *ids, const uint32_t *inv, void *vecs);
hipError_t tri_build_cluster_means(hipStream_t s, int dtype, const void *rows, uint32_t dpad,
                                   const uint32_t *list_off, const uint32_t *perm, uint32_t nlist, int normalise,
                                   float *cent_f32 /*[nlist][dpad] in/out*/);
