// IVF search over product-quantised lists (the compressed variant of the inverted-file index named in the
// paper's Sec. 1), on top of a resident IVF index: that index's centroids and lists choose a query's candidates,
// what is scored are m-byte codes, by summing one table entry per sub-space.
//
// Build: codebooks (given, or Lloyd per sub-space on a sample of the stored vectors), then every stored vector is
// encoded, list-major.  Search, per batch of queries with one k, nprobe and metric:
//   1. the query rows are copied into zero-padded rows of the index's row length;
//   2. coarse scores against the centroids: the same matrix-core contraction the IVF-Flat pool uses;
//   3. the nprobe best lists per query (one workgroup per query, streaming selection, see PqCollector);
//   4. the query's tables, m x 256 fp32 partial scores (values where smaller is better: the negative partial
//      products for the inner product);
//   5. one workgroup per query: tables into LDS, the codes of its probed lists streamed once (m bytes per vector,
//      one vector per thread and round), m LDS look-ups summed in sub-space order, the k best by (score, id) kept
//      by the same streaming selection.
// Bound of step 5: LDS look-ups (m per vector and query, 4 bytes each, random banks); the codes themselves are
// 1/16 of the fp16 rows and mostly cache-resident.
#include "../../include/trinity_pq.h"
#include "tri_common.h"

#include <algorithm>
#include <new>
#include <vector>

namespace {

#define PQ_TRY(expr)                                                                           \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess) return tri_fail(TRI_EHIP, "%s -> %s", #expr, hipGetErrorString(e_)); \
    } while (0)

constexpr uint32_t PQ_THREADS = 1024;     // a workgroup: 16 wavefronts, so that the LDS look-ups of a compute unit have enough in flight
constexpr uint32_t PQ_GROUPS_MAX = 8;     // 16-byte groups of a code: m <= 128
typedef _Float16 pq_half8 __attribute__((ext_vector_type(8)));
typedef float pq_float4 __attribute__((ext_vector_type(4)));
#ifndef PQ_RANK_SORT_MAX
#define PQ_RANK_SORT_MAX 128u            // composites up to which a sort counts ranks instead of running the network
#endif
constexpr uint32_t PQ_RERANK_ROWS = 4;   // stored rows a half-wavefront re-scores at a time
constexpr uint32_t PQ_BUF = 4096;         // composites the streaming selection holds in LDS (32 KB)

size_t up256(size_t x) { return (x + 255) / 256 * 256; }

// Where byte mm of the code of the vector at stored position v lies.  Codes are kept in blocks of 64 consecutive
// stored positions, transposed: 16-byte group g (sub-spaces 16 g .. 16 g + 15) of the 64 codes side by side (1 KiB),
// group after group -- so that the 64 lanes of a wavefront, which score 64 consecutive positions, read one contiguous
// KiB per load instruction instead of 64 pieces m bytes apart, and a code is a handful of 16-byte loads that are all
// in flight together.  m is padded to a multiple of 16 in this layout (the padding bytes are never looked up).
__host__ __device__ __forceinline__ uint32_t pq_mpad(uint32_t m) { return (m + 15u) / 16u * 16u; }
__host__ __device__ __forceinline__ size_t pq_code_at(uint64_t v, uint32_t mm, uint32_t m)
{
    return (size_t)(v / 64) * ((size_t)pq_mpad(m) * 64) + (size_t)(mm / 16) * 1024 + (size_t)(v % 64) * 16 + mm % 16;
}

// Codebooks are kept with the entry number fastest -- cb[(mm * dsub + e) * 256 + c] is coordinate e of entry c of
// sub-space mm -- so that threads that work on consecutive entries read consecutive words.
__host__ __device__ __forceinline__ size_t pq_cb_at(uint32_t mm, uint32_t c, uint32_t e, uint32_t dsub)
{
    return ((size_t)mm * dsub + e) * TRI_PQ_KSUB + c;
}

// Element i of the index's stored vector at stored position pos (the index keeps its vectors in blocks of 32,
// interleaved by 16-byte pieces; a vector's storage slot is found through its id).
__device__ __forceinline__ uint32_t pq_slot_of(const TriIndexDev &ix, uint64_t pos) { return ix.inv[ix.ids[pos]]; }
__device__ __forceinline__ float pq_elem(const TriIndexDev &ix, uint32_t slot, uint32_t i)
{
    return ix.dtype == 1u ? (float)*(const _Float16 *)tri_slot_byte(ix, slot, i * 2u) : *(const float *)tri_slot_byte(ix, slot, i * 4u);
}

// ---------------------------------------------------------------------------------------- build
// The index's vectors once more, row-major by vector id: one thread per 16-byte piece.
__global__ void pq_refine_copy_kernel(const TriIndexDev ix, uint64_t n, uint8_t *__restrict__ refine)
{
    const uint32_t pieces = ix.row_bytes / 16;
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n * pieces) return;
    const uint32_t id = (uint32_t)(t / pieces), j = (uint32_t)(t % pieces);
    *(uint4 *)(refine + (size_t)id * ix.row_bytes + j * 16) = *(const uint4 *)(tri_slot_ptr(ix, ix.inv[id]) + (size_t)j * TRI_PIECE_PITCH);
}

// Stored position of training row r: every stride-th stored vector.
__global__ void pq_init_kernel(const TriIndexDev ix, uint64_t n,
                               uint32_t m, uint32_t dsub, uint64_t seed, float *__restrict__ cb)
{
    // entry c of every sub-space starts as the sub-vector of one stored vector: 256 positions spread over the
    // index, shifted by the seed
    const uint32_t c = blockIdx.x;
    const uint64_t step = n / TRI_PQ_KSUB;               // (n >= 256: at least 1)
    const uint64_t pos = ((uint64_t)c * step + seed % step) % n;
    const uint32_t slot = pq_slot_of(ix, pos);
    for (uint32_t j = threadIdx.x; j < m * dsub; j += blockDim.x) {      // j over the dim values
        const uint32_t mm = j / dsub, e = j % dsub;
        cb[pq_cb_at(mm, c, e, dsub)] = pq_elem(ix, slot, j);
    }
}

// Nearest entry of sub-space mm's codebook (in LDS) to the sub-vector x: squared L2 accumulated in coordinate
// order, ties to the smaller number.
template <int DSUB_MAX>
__device__ __forceinline__ uint32_t pq_nearest(const float *cb_lds, const float (&x)[DSUB_MAX], uint32_t dsub)
{
    float best = INFINITY;
    uint32_t arg = 0;
    for (uint32_t c = 0; c < TRI_PQ_KSUB; ++c) {
        float d2 = 0.f;
        for (uint32_t e = 0; e < dsub; ++e) {
            const float d = x[e] - cb_lds[c * dsub + e];
            d2 = __builtin_fmaf(d, d, d2);
        }
        if (d2 < best) {
            best = d2;
            arg = c;
        }
    }
    return arg;
}

// Encoding, grid (n / 1024, m): one thread per (stored vector, sub-space); the sub-space's codebook sits in LDS.
__global__ __launch_bounds__(PQ_THREADS) void pq_assign_kernel(const TriIndexDev ix, uint64_t rows, uint32_t m,
                                                               uint32_t dsub, const float *__restrict__ cb,
                                                               uint8_t *__restrict__ codes)
{
    extern __shared__ float cb_lds[];
    const uint32_t mm = blockIdx.y;
    for (uint32_t i = threadIdx.x; i < TRI_PQ_KSUB * dsub; i += PQ_THREADS)       // i = e * 256 + c in memory -> [c][e] in LDS
        cb_lds[(i % TRI_PQ_KSUB) * dsub + i / TRI_PQ_KSUB] = cb[(size_t)mm * TRI_PQ_KSUB * dsub + i];
    __syncthreads();
    const uint64_t r = (uint64_t)blockIdx.x * PQ_THREADS + threadIdx.x;
    if (r >= rows) return;
    const uint64_t pos = r;
    float x[TRI_PQ_DSUB_MAX];
    const uint32_t slot = pq_slot_of(ix, pos);
    for (uint32_t e = 0; e < dsub; ++e) x[e] = pq_elem(ix, slot, mm * dsub + e);
    codes[pq_code_at(pos, mm, m)] = (uint8_t)pq_nearest<TRI_PQ_DSUB_MAX>(cb_lds, x, dsub);
}

// One Lloyd iteration's sums, grid (PQ_TRAIN_BLOCKS, m), 256 threads: the training sample (every stride-th stored
// vector) is dealt out in PQ_TRAIN_BLOCKS runs of consecutive rows; a workgroup takes its run 256 rows at a time --
// thread t finds the cell of row t's sub-vector and leaves both in LDS, then thread c adds the sub-vectors of cell c
// to its own sums in row order.  No atomics: the partial sums of the runs, added in run order by pq_update_kernel,
// make the trained codebooks the same bit for bit on every run.
constexpr uint32_t PQ_TRAIN_BLOCKS = 16;
__global__ __launch_bounds__(TRI_PQ_KSUB) void pq_train_kernel(const TriIndexDev ix, uint64_t rows, uint64_t stride, uint32_t m,
                                                               uint32_t dsub, const float *__restrict__ cb,
                                                               float *__restrict__ part_sums, uint32_t *__restrict__ part_counts)
{
    extern __shared__ float cb_lds[];                                  // [256][dsub] entries, then [256][dsub] sub-vectors of the rows at hand
    __shared__ uint32_t cell_of[TRI_PQ_KSUB];
    float *xs = cb_lds + TRI_PQ_KSUB * dsub;
    const uint32_t mm = blockIdx.y, t = threadIdx.x;
    for (uint32_t i = t; i < TRI_PQ_KSUB * dsub; i += TRI_PQ_KSUB)       // i = e * 256 + c in memory -> [c][e] in LDS
        cb_lds[(i % TRI_PQ_KSUB) * dsub + i / TRI_PQ_KSUB] = cb[(size_t)mm * TRI_PQ_KSUB * dsub + i];
    const uint64_t per = (rows + gridDim.x - 1) / gridDim.x;
    const uint64_t r_begin = blockIdx.x * per < rows ? blockIdx.x * per : rows, r_end = r_begin + per < rows ? r_begin + per : rows;
    float acc[TRI_PQ_DSUB_MAX];
#pragma unroll
    for (uint32_t e = 0; e < TRI_PQ_DSUB_MAX; ++e) acc[e] = 0.f;
    uint32_t cnt = 0;
    for (uint64_t base = r_begin; base < r_end; base += TRI_PQ_KSUB) {
        __syncthreads();                                               // (the codebook is in LDS; the last turn's rows have been read)
        const uint64_t r = base + t;
        uint32_t c = 0xFFFFFFFFu;
        if (r < r_end) {
            float x[TRI_PQ_DSUB_MAX];
            const uint32_t slot = pq_slot_of(ix, r * stride);
            for (uint32_t e = 0; e < dsub; ++e) x[e] = pq_elem(ix, slot, mm * dsub + e);
            c = pq_nearest<TRI_PQ_DSUB_MAX>(cb_lds, x, dsub);
            for (uint32_t e = 0; e < dsub; ++e) xs[t * dsub + e] = x[e];
        }
        cell_of[t] = c;
        __syncthreads();
        const uint32_t here = r_end - base < TRI_PQ_KSUB ? (uint32_t)(r_end - base) : TRI_PQ_KSUB;
        for (uint32_t j = 0; j < here; ++j) {
            if (cell_of[j] == t) {
#pragma unroll
                for (uint32_t e = 0; e < TRI_PQ_DSUB_MAX; ++e)
                    if (e < dsub) acc[e] += xs[j * dsub + e];
                ++cnt;
            }
        }
    }
    const size_t cell = ((size_t)blockIdx.x * m + mm) * TRI_PQ_KSUB + t;
#pragma unroll
    for (uint32_t e = 0; e < TRI_PQ_DSUB_MAX; ++e)
        if (e < dsub) part_sums[cell * dsub + e] = acc[e];
    part_counts[cell] = cnt;
}

// New entries from the runs' partial sums (added in run order); a cell nothing is nearest to keeps its entry.
__global__ void pq_update_kernel(uint32_t total, uint32_t dsub, uint32_t runs, const float *__restrict__ part_sums,
                                 const uint32_t *__restrict__ part_counts, float *__restrict__ cb)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const uint32_t cell = i / dsub;                              // (sums: [run][sub-space][entry][coordinate])
    float sum = 0.f;
    uint32_t cnt = 0;
    for (uint32_t b = 0; b < runs; ++b) {
        sum += part_sums[(size_t)b * total + i];
        cnt += part_counts[(size_t)b * (total / dsub) + cell];
    }
    if (cnt) cb[pq_cb_at(cell / TRI_PQ_KSUB, cell % TRI_PQ_KSUB, i % dsub, dsub)] = sum / (float)cnt;
}

// ---------------------------------------------------------------------------------------- search
__global__ void pq_pad_queries_kernel(const uint8_t *__restrict__ q, size_t pitch, uint32_t nq, uint32_t dim_bytes,
                                      uint32_t row_bytes, uint8_t *__restrict__ rows)
{
    const uint32_t r = blockIdx.x;
    for (uint32_t b = threadIdx.x; b < row_bytes; b += blockDim.x) rows[(size_t)r * row_bytes + b] = b < dim_bytes ? q[r * pitch + b] : 0;
}

// Streaming selection of the k smallest 64-bit composites (score key << 32 | id) offered to a workgroup: the
// current best (at most k, sorted) head an LDS array, offers that beat the k-th are appended behind them, and when
// the array could not take another round of offers it is sorted and cut back to k.  Exact: an offer is dropped only
// when k composites smaller than it are known.
struct PqCollector {
    uint64_t buf[PQ_BUF];
    uint32_t count;        // composites in buf
    uint32_t have;         // of which sorted best (the first `have`)
    uint64_t bound;        // the k-th best when have == k, else all-ones
    uint64_t wave_kth[PQ_THREADS / 64];   // first round: per wavefront, the last of its smallest offers that are kept
};

// One compare-exchange step of a bitonic network among the 64 lanes of a wavefront: lanes l and l ^ s.
__device__ __forceinline__ uint64_t pq_cx(uint64_t x, uint32_t lane, uint32_t s, bool up)
{
    const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)x, (int)s, 64), hi = (uint32_t)__shfl_xor((int)(uint32_t)(x >> 32), (int)s, 64);
    const uint64_t o = ((uint64_t)hi << 32) | lo;
    const bool take_min = ((lane & s) == 0) == up;            // the lower lane of an ascending pair keeps the smaller one
    return take_min ? (o < x ? o : x) : (o > x ? o : x);
}

// Sort of a[0..n) ascending (n <= PQ_BUF); all NT threads.
// Up to NT / 4 composites (what a selection of a few hundred holds at most times): by rank counting -- four threads
// per composite, each of which reads a quarter of all composites (the same addresses for all lanes that work on the
// same quarter: few LDS accesses per wavefront, none waiting for another), counts those that come before its own,
// the four counts are added across the lanes and, after a barrier, the composite is put at that position.
// More: a bitonic network on a[] padded with all-ones to a power of two >= 64.  The steps whose partners lie less than
// 64 apart -- most of them -- are done in registers, a wavefront per chunk of 64 with lane exchanges and no barrier;
// only the steps with farther partners go through LDS, one barrier each.
template <uint32_t NT = PQ_THREADS>
__device__ void pq_sort(uint64_t *a, uint32_t n)
{
    if (n <= PQ_RANK_SORT_MAX && n <= NT / 4) {                           // (uniform)
        const uint32_t i = threadIdx.x >> 2, part = threadIdx.x & 3u;
        uint64_t x = 0;
        uint32_t rank = 0;
        if (i < n) {
            x = a[i];
            for (uint32_t o = part; o < n; o += 4) {
                const uint64_t y = a[o];
                rank += (y < x || (y == x && o < i)) ? 1u : 0u;           // (equal composites keep their order)
            }
        }
        rank += (uint32_t)__shfl_xor((int)rank, 1, 64);
        rank += (uint32_t)__shfl_xor((int)rank, 2, 64);
        __syncthreads();
        if (i < n && part == 0) a[rank] = x;
        __syncthreads();
        return;
    }
    constexpr uint32_t NW = NT / 64;
    uint32_t np2 = 64;
    while (np2 < n) np2 <<= 1;
    for (uint32_t i = n + threadIdx.x; i < np2; i += NT) a[i] = ~0ull;
    __syncthreads();
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (uint32_t i = wave * 64 + lane; i < np2; i += NW * 64) {             // sizes 2 .. 64
        uint64_t x = a[i];
#pragma unroll
        for (uint32_t size = 2; size <= 64; size <<= 1) {
            const bool up = (i & size) == 0;
#pragma unroll
            for (uint32_t s = size >> 1; s > 0; s >>= 1) x = pq_cx(x, lane, s, up);
        }
        a[i] = x;
    }
    __syncthreads();
    for (uint32_t size = 128; size <= np2; size <<= 1) {
        for (uint32_t stride = size >> 1; stride >= 64; stride >>= 1) {
            for (uint32_t i = threadIdx.x; i < np2 / 2; i += NT) {
                const uint32_t lo = 2 * i - (i & (stride - 1)), hi = lo + stride;
                const bool up = (lo & size) == 0;
                const uint64_t x = a[lo], y = a[hi];
                if ((x > y) == up) {
                    a[lo] = y;
                    a[hi] = x;
                }
            }
            __syncthreads();
        }
        for (uint32_t i = wave * 64 + lane; i < np2; i += NW * 64) {
            uint64_t x = a[i];
            const bool up = (i & size) == 0;
#pragma unroll
            for (uint32_t s = 32; s > 0; s >>= 1) x = pq_cx(x, lane, s, up);
            a[i] = x;
        }
        __syncthreads();
    }
}

__device__ __forceinline__ void pq_collect_init(PqCollector &c)
{
    if (threadIdx.x == 0) {
        c.count = 0;
        c.have = 0;
        c.bound = ~0ull;
    }
    __syncthreads();
}

// Sort what was collected and keep the k best.  All threads; ends with a barrier.
template <uint32_t NT = PQ_THREADS>
__device__ void pq_collect_settle(PqCollector &c, uint32_t k)
{
    __syncthreads();
    const uint32_t n = c.count;
    pq_sort<NT>(c.buf, n);
    if (threadIdx.x == 0) {
        c.have = n < k ? n : k;
        c.count = c.have;
        c.bound = c.have == k ? c.buf[k - 1] : ~0ull;
    }
    __syncthreads();
}

// A round of offers: every thread offers composites (pq_collect_offer: valid = it has one; no barrier), then all
// threads call pq_collect_close together, `room` = the offers the next round may bring at most.  Whether the array
// could take that round is decided by all threads as one: the barrier that ends the round also combines what each
// thread saw of the counter after its own appends (the thread that appended last saw them all).
__device__ __forceinline__ void pq_collect_offer(PqCollector &c, bool valid, uint64_t comp)
{
    // one counter update per wavefront, not per lane: before the first bound exists every lane appends
    const bool push = valid && comp < c.bound;
    const uint64_t mask = __ballot(push);
    if (mask) {
        const uint32_t lane = threadIdx.x & 63;
        const int leader = __ffsll((unsigned long long)mask) - 1;
        uint32_t base = 0;
        if ((int)lane == leader) base = atomicAdd(&c.count, (uint32_t)__popcll(mask));
        base = (uint32_t)__shfl((int)base, leader, 64);
        if (push) c.buf[base + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull))] = comp;
    }
}
template <uint32_t NT = PQ_THREADS>
__device__ __forceinline__ void pq_collect_close(PqCollector &c, uint32_t k, uint32_t room)
{
    // settle when the array could not take another round -- or as soon as k composites are there and no bound yet:
    // from then on only offers that beat the k-th best are appended
    if (__syncthreads_or(c.count + room > PQ_BUF || (c.have < k && c.count >= k))) pq_collect_settle<NT>(c, k);
}
template <uint32_t NT = PQ_THREADS>
__device__ __forceinline__ void pq_collect_round(PqCollector &c, uint32_t k, bool valid, uint64_t comp)
{
    pq_collect_offer(c, valid, comp);
    pq_collect_close<NT>(c, k, NT);
}

// The first round of a selection, when no bound exists yet and every offer would be appended (and the first settle
// would sort them all): whether this thread's offer has to be kept.  Every wavefront finds the j-th smallest of its 64
// offers, j = ceil(k / wavefronts), by rank counting across its lanes; the largest of these over the wavefronts has at
// least k offers of this round at or below it, so an offer above it is dropped exactly.  A wavefront with fewer than
// j offers makes every offer kept.  All threads call it together (one barrier).
template <uint32_t NT = PQ_THREADS>
__device__ __forceinline__ bool pq_first_round_keeps(PqCollector &c, uint32_t k, bool valid, uint64_t comp)
{
    constexpr uint32_t NW = NT / 64;
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t j = (k + NW - 1) / NW;                          // (1 <= j <= 64: k <= 64 NW)
    const uint64_t mine = valid ? comp : ~0ull;
    const uint32_t lo = (uint32_t)mine, hi = (uint32_t)(mine >> 32);
    uint32_t rank = 0;
#pragma unroll
    for (int i = 0; i < 64; ++i) {
        const uint64_t o = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)hi, i) << 32) | (uint32_t)__builtin_amdgcn_readlane((int)lo, i);
        rank += o < mine ? 1u : 0u;
    }
    const uint64_t hit = __ballot(valid && rank == j - 1);
    uint64_t kth = ~0ull;
    if (hit) {
        const int src = __ffsll((unsigned long long)hit) - 1;
        kth = ((uint64_t)(uint32_t)__shfl((int)hi, src, 64) << 32) | (uint32_t)__shfl((int)lo, src, 64);
    }
    if (lane == 0) c.wave_kth[wave] = kth;
    __syncthreads();
    uint64_t pre = 0;
#pragma unroll
    for (uint32_t w = 0; w < NW; ++w) pre = c.wave_kth[w] > pre ? c.wave_kth[w] : pre;
    return valid && mine <= pre;
}

// (3) the nprobe best lists of each query: best first, ties to the smaller list number.  (Small workgroups: the first
// settle, which gives the bound that turns most later offers away, then sorts 256 composites instead of 1024, and
// several workgroups share a compute unit.)
constexpr uint32_t PQ_PROBE_THREADS = 256, PQ_PROBE_R = 8;
// `todo` (may be null): one word per query, the kernel leaves the queries alone whose word is zero.
__global__ __launch_bounds__(PQ_PROBE_THREADS) void pq_probe_kernel(const float *__restrict__ scores, uint32_t ldc, uint32_t nlist,
                                                              uint32_t nprobe, uint32_t metric, uint32_t *__restrict__ probes,
                                                              const uint32_t *__restrict__ todo)
{
    __shared__ PqCollector col;
    if (todo && !todo[blockIdx.x]) return;
    const float *row = scores + (size_t)blockIdx.x * ldc;
    const uint32_t kind = metric == 1u ? 1u : 0u;
    pq_collect_init(col);
    // after the first round, PQ_PROBE_R scores per thread and round (one barrier for all of them), loaded one round ahead
    auto load = [&](uint32_t i0, float (&v)[PQ_PROBE_R]) {
#pragma unroll
        for (uint32_t r = 0; r < PQ_PROBE_R; ++r) {
            const uint32_t i = i0 + r * PQ_PROBE_THREADS + threadIdx.x;
            v[r] = i < nlist ? row[i] : 0.f;
        }
    };
    float v[PQ_PROBE_R], nv[PQ_PROBE_R];
    load(PQ_PROBE_THREADS, v);
    {   // the first 256 scores: they give the bound
        const bool valid = threadIdx.x < nlist;
        const uint64_t comp = valid ? ((uint64_t)tri_score_key(row[threadIdx.x], kind) << 32) | threadIdx.x : ~0ull;
        pq_collect_offer(col, pq_first_round_keeps<PQ_PROBE_THREADS>(col, nprobe, valid, comp), comp);
        pq_collect_close<PQ_PROBE_THREADS>(col, nprobe, PQ_PROBE_R * PQ_PROBE_THREADS);
    }
    for (uint32_t i0 = PQ_PROBE_THREADS; i0 < nlist; i0 += PQ_PROBE_R * PQ_PROBE_THREADS) {
        load(i0 + PQ_PROBE_R * PQ_PROBE_THREADS, nv);
#pragma unroll
        for (uint32_t r = 0; r < PQ_PROBE_R; ++r) {
            const uint32_t i = i0 + r * PQ_PROBE_THREADS + threadIdx.x;
            pq_collect_offer(col, i < nlist, ((uint64_t)tri_score_key(v[r], kind) << 32) | i);
        }
        pq_collect_close<PQ_PROBE_THREADS>(col, nprobe, PQ_PROBE_R * PQ_PROBE_THREADS);
#pragma unroll
        for (uint32_t r = 0; r < PQ_PROBE_R; ++r) v[r] = nv[r];
    }
    pq_collect_settle<PQ_PROBE_THREADS>(col, nprobe);
    for (uint32_t i = threadIdx.x; i < nprobe; i += PQ_PROBE_THREADS)
        probes[(size_t)blockIdx.x * nprobe + i] = i < col.have ? (uint32_t)(col.buf[i] & 0xFFFFFFFFu) : 0xFFFFFFFFu;
}

// (3a) the same selection for rows of at most PQ_PW_NLIST scores and at most PQ_PW_NPROBE probes, one wavefront per
// row with no barrier at all: the row sits in registers (64 keys per lane, read as 16 loads of 16 bytes); the
// nprobe-th smallest of the 1024 minima of the four keys of a load and lane is found by bisection on its 32 bits with
// ballots -- at least nprobe keys lie at or below it, so the nprobe best do; the keys at or below it (nprobe or a
// few more) are compacted into LDS as composites by a prefix count across the lanes, ranked by counting and written
// in rank order.  A row this does not settle (fewer than nprobe non-empty minima, or more than PQ_PW_CAP candidates:
// masses of equal scores) gets its word of `todo` set and is left to pq_probe_kernel.
constexpr uint32_t PQ_PW_NLIST = 4096, PQ_PW_NPROBE = 128, PQ_PW_CAP = 256, PQ_PW_ROWS = 4;
__global__ __launch_bounds__(64 * PQ_PW_ROWS) void pq_probe_wave_kernel(const float *__restrict__ scores, uint32_t ldc, uint32_t nlist,
                                                                        uint32_t nprobe, uint32_t metric, uint32_t nq,
                                                                        uint32_t *__restrict__ probes, uint32_t *__restrict__ todo)
{
    __shared__ uint64_t cand[PQ_PW_ROWS][PQ_PW_CAP];
    const uint32_t lane = threadIdx.x & 63, wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint32_t r = blockIdx.x * PQ_PW_ROWS + wave;
    if (r >= nq) return;
    const float *row = scores + (size_t)r * ldc;
    const uint32_t kind = metric == 1u ? 1u : 0u;
    // load j of lane l: scores 256 j + 4 l .. + 3 (rows are ldc >= nlist scores long, ldc a multiple of 4)
    uint32_t key[16][4], mn[16];
    float4 v[16];
#pragma unroll
    for (uint32_t j = 0; j < 16; ++j) {
        const uint32_t e0 = j * 256 + lane * 4;
        v[j] = e0 < ldc ? *(const float4 *)(row + e0) : float4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (uint32_t j = 0; j < 16; ++j) {
        const uint32_t e0 = j * 256 + lane * 4;
        const float x[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
        for (uint32_t c = 0; c < 4; ++c) key[j][c] = e0 + c < nlist ? tri_score_key(x[c], kind) : 0xFFFFFFFFu;
        const uint32_t a = key[j][0] < key[j][1] ? key[j][0] : key[j][1], b = key[j][2] < key[j][3] ? key[j][2] : key[j][3];
        mn[j] = a < b ? a : b;
    }
    uint32_t T = 0;
    for (int b = 31; b >= 0; --b) {
        const uint32_t trial = T | ((1u << b) - 1u);                  // (bit b clear, every lower bit set)
        uint32_t cnt = 0;
#pragma unroll
        for (uint32_t j = 0; j < 16; ++j) cnt += (uint32_t)__popcll(__ballot(mn[j] <= trial));
        if (cnt < nprobe) T |= 1u << b;
    }
    uint32_t mine = 0;
#pragma unroll
    for (uint32_t j = 0; j < 16; ++j)
#pragma unroll
        for (uint32_t c = 0; c < 4; ++c) mine += key[j][c] <= T ? 1u : 0u;
    uint32_t incl = mine;
#pragma unroll
    for (int dd = 1; dd < 64; dd <<= 1) {
        const uint32_t o = (uint32_t)__shfl_up((int)incl, dd, 64);
        if ((int)lane >= dd) incl += o;
    }
    const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    const bool settled = T != 0xFFFFFFFFu && total <= PQ_PW_CAP;      // (uniform)
    if (lane == 0) todo[r] = settled ? 0u : 1u;
    if (!settled) return;
    uint64_t *a = cand[wave];
    uint32_t pos = incl - mine;
#pragma unroll
    for (uint32_t j = 0; j < 16; ++j)
#pragma unroll
        for (uint32_t c = 0; c < 4; ++c)
            if (key[j][c] <= T) a[pos++] = ((uint64_t)key[j][c] << 32) | (j * 256 + lane * 4 + c);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (uint32_t i = lane; i < total; i += 64) {
        const uint64_t x = a[i];
        uint32_t rank = 0;
        for (uint32_t o = 0; o < total; ++o) rank += a[o] < x ? 1u : 0u;
        if (rank < nprobe) probes[(size_t)r * nprobe + rank] = (uint32_t)(x & 0xFFFFFFFFu);
    }
}

// (4) tables: lut[q][mm][c] = sum over the sub-space of (q - entry)^2, or of -q * entry, in coordinate order.  A
// workgroup makes the tables of PQ_LUT_Q queries for PQ_LUT_M sub-spaces (grid: query groups x m / PQ_LUT_M; m is a
// multiple of 4), one wavefront per sub-space, four entries per lane: a codebook word read from the cache serves all
// the queries, a query value read from LDS four entries, and the kernel is left with writing the tables.
constexpr uint32_t PQ_LUT_Q = 16, PQ_LUT_M = 4;
__global__ __launch_bounds__(64 * PQ_LUT_M) void pq_lut_kernel(const uint8_t *__restrict__ qrows, uint32_t row_bytes, uint32_t dtype,
                                                               uint32_t nq, uint32_t m, uint32_t dsub, uint32_t metric,
                                                               const float *__restrict__ cb, float *__restrict__ lut)
{
    __shared__ __attribute__((aligned(16))) float qv[PQ_LUT_Q][PQ_LUT_M * TRI_PQ_DSUB_MAX];
    const uint32_t q0 = blockIdx.x * PQ_LUT_Q, m0 = blockIdx.y * PQ_LUT_M, span = PQ_LUT_M * dsub;
    for (uint32_t i = threadIdx.x; i < PQ_LUT_Q * span; i += 64 * PQ_LUT_M) {
        const uint32_t j = i / span, e = i % span;
        const uint8_t *row = qrows + (size_t)(q0 + j < nq ? q0 + j : q0) * row_bytes;
        qv[j][e] = dtype == 1u ? (float)((const _Float16 *)row)[m0 * dsub + e] : ((const float *)row)[m0 * dsub + e];
    }
    __syncthreads();
    auto term = [&](float x, float y, float a) {
        const float d = x - y;
        return metric == 0u ? __builtin_fmaf(d, d, a) : __builtin_fmaf(-x, y, a);
    };
    const uint32_t u = threadIdx.x >> 6, lane = threadIdx.x & 63, mm = m0 + u;      // entries lane, lane + 64, + 128, + 192
    float acc[PQ_LUT_Q][4];
#pragma unroll
    for (uint32_t j = 0; j < PQ_LUT_Q; ++j)
#pragma unroll
        for (uint32_t i = 0; i < 4; ++i) acc[j][i] = 0.f;
    if (dsub % 4 == 0) {
        for (uint32_t e = 0; e < dsub; e += 4) {
            float y[4][4];
#pragma unroll
            for (uint32_t i = 0; i < 4; ++i)
#pragma unroll
                for (uint32_t f = 0; f < 4; ++f) y[i][f] = cb[pq_cb_at(mm, lane + 64 * i, e + f, dsub)];
#pragma unroll
            for (uint32_t j = 0; j < PQ_LUT_Q; ++j) {
                const float4 x = *(const float4 *)&qv[j][u * dsub + e];
#pragma unroll
                for (uint32_t i = 0; i < 4; ++i)
                    acc[j][i] = term(x.w, y[i][3], term(x.z, y[i][2], term(x.y, y[i][1], term(x.x, y[i][0], acc[j][i]))));
            }
        }
    } else {
        for (uint32_t e = 0; e < dsub; ++e) {
            float y[4];
#pragma unroll
            for (uint32_t i = 0; i < 4; ++i) y[i] = cb[pq_cb_at(mm, lane + 64 * i, e, dsub)];
#pragma unroll
            for (uint32_t j = 0; j < PQ_LUT_Q; ++j) {
                const float x = qv[j][u * dsub + e];
#pragma unroll
                for (uint32_t i = 0; i < 4; ++i) acc[j][i] = term(x, y[i], acc[j][i]);
            }
        }
    }
#pragma unroll
    for (uint32_t j = 0; j < PQ_LUT_Q; ++j)
        if (q0 + j < nq) {
#pragma unroll
            for (uint32_t i = 0; i < 4; ++i) lut[((size_t)(q0 + j) * m + mm) * TRI_PQ_KSUB + lane + 64 * i] = acc[j][i];
        }
}

// (5) one workgroup per query.  G: the 16-byte groups of a code when m is a multiple of 16 (the look-ups of a code are
// then one straight run of instructions), 0 for any other m.
template <uint32_t G>
__global__ __launch_bounds__(PQ_THREADS) void pq_scan_kernel(const float *__restrict__ lut, uint32_t m,
                                                             const uint32_t *__restrict__ probes, uint32_t nprobe,
                                                             const uint32_t *__restrict__ list_off, const uint32_t *__restrict__ ids,
                                                             const uint8_t *__restrict__ codes, uint32_t k, uint32_t metric,
                                                             uint32_t k_adc, const uint8_t *__restrict__ qrows,
                                                             const uint8_t *__restrict__ vecs, const uint32_t *__restrict__ inv,
                                                             const uint8_t *__restrict__ refine,
                                                             uint32_t row_bytes, uint32_t dtype,
                                                             uint32_t *__restrict__ ids_out, float *__restrict__ dist_out,
                                                             uint32_t *__restrict__ n_out)
{
    extern __shared__ float lut_lds[];
    __shared__ PqCollector col;
    __shared__ uint32_t first[TRI_PQ_NPROBE_MAX], start[TRI_PQ_NPROBE_MAX + 1];   // per probed list: first stored position; running sum of lengths
    const uint32_t q = blockIdx.x;
    // A query's tables on their way from memory into LDS: 16 bytes per thread and turn, held in registers between.
    constexpr uint32_t LUT_TURNS = G ? G : PQ_GROUPS_MAX;
    const uint32_t lut16 = m * (TRI_PQ_KSUB / 4);
    typedef uint32_t pq_u32x4 __attribute__((ext_vector_type(4)));
    pq_u32x4 lreg[LUT_TURNS];
    auto lut_load = [&](uint32_t qn) {
        const pq_u32x4 *src = (const pq_u32x4 *)(lut + (size_t)qn * m * TRI_PQ_KSUB);
#pragma unroll
        for (uint32_t i = 0; i < LUT_TURNS; ++i) {
            const uint32_t t = threadIdx.x + i * PQ_THREADS;
            if (G || t < lut16) lreg[i] = src[t];
        }
    };
    auto lut_store = [&]() {
#pragma unroll
        for (uint32_t i = 0; i < LUT_TURNS; ++i) {
            const uint32_t t = threadIdx.x + i * PQ_THREADS;
            if (G || t < lut16) ((pq_u32x4 *)lut_lds)[t] = lreg[i];
        }
    };
    // A query's list table, made by the first wavefront in three steps that can lie apart (each step's loads are on
    // their way until the next one needs them): lane l takes probes 4 l .. 4 l + 3, the running sums come from a scan
    // across the lanes.
    constexpr uint32_t PER = TRI_PQ_NPROBE_MAX / 64;
    uint32_t pl[PER], plo[PER], phi[PER];
    auto lists_probes = [&](uint32_t qn) {
#pragma unroll
        for (uint32_t j = 0; j < PER; ++j) {
            const uint32_t p = threadIdx.x * PER + j;
            pl[j] = p < nprobe ? probes[(size_t)qn * nprobe + p] : 0xFFFFFFFFu;
        }
    };
    auto lists_offsets = [&]() {
#pragma unroll
        for (uint32_t j = 0; j < PER; ++j) {
            plo[j] = pl[j] == 0xFFFFFFFFu ? 0u : list_off[pl[j]];
            phi[j] = pl[j] == 0xFFFFFFFFu ? 0u : list_off[pl[j] + 1];
        }
    };
    auto lists_table = [&]() {
        uint32_t mine = 0;
#pragma unroll
        for (uint32_t j = 0; j < PER; ++j) mine += phi[j] - plo[j];
        uint32_t incl = mine;
#pragma unroll
        for (int dd = 1; dd < 64; dd <<= 1) {
            const uint32_t o = (uint32_t)__shfl_up((int)incl, dd, 64);
            if ((int)threadIdx.x >= dd) incl += o;
        }
        uint32_t run = incl - mine;
#pragma unroll
        for (uint32_t j = 0; j < PER; ++j) {
            const uint32_t p = threadIdx.x * PER + j;
            if (p < nprobe) {
                first[p] = plo[j];
                start[p] = run;
            }
            run += phi[j] - plo[j];
        }
        if (threadIdx.x == 63) start[nprobe] = run;             // (the total: probes past nprobe count nothing)
    };
    // (in this order the list table's two rounds of loads and the tables' loads are in flight together)
    if (threadIdx.x < 64) lists_probes(q);
    lut_load(q);
    if (threadIdx.x < 64) lists_offsets();
    lut_store();
    if (threadIdx.x < 64) lists_table();
    pq_collect_init(col);
    // the vectors of all probed lists as ONE sequence (short lists would otherwise leave most of a round's threads
    // idle): thread t of a round takes element r0 + t and finds its list by bisection in the running sums
    const uint32_t groups = G ? G : pq_mpad(m) / 16, total = start[nprobe];
    const uint32_t ksel = k_adc ? k_adc : k;              // how many the table scores select
    // The codes (and the id) of a round's element are fetched one round ahead: the loads of round r + 1 are in flight
    // while round r does its look-ups and its offer, which ends in a barrier.
    auto locate = [&](uint32_t e) -> uint32_t {
        uint32_t lo = 0, hi = nprobe;                                      // start[lo] <= e < start[hi]
        while (hi - lo > 1) {
            const uint32_t mid = (lo + hi) / 2;
            if (start[mid] <= e) lo = mid; else hi = mid;
        }
        return first[lo] + (e - start[lo]);
    };
    uint4 cw_next[PQ_GROUPS_MAX];
    uint32_t id_next = 0;
    auto fetch = [&](uint32_t e) {
        if (e < total) {
            const uint32_t v = locate(e);
            const uint4 *code = (const uint4 *)(codes + pq_code_at(v, 0, m));
#pragma unroll
            for (uint32_t g = 0; g < PQ_GROUPS_MAX; ++g)
                if (g < groups) cw_next[g] = code[g * 64];                     // (uniform)
            id_next = ids[v];
        }
    };
    fetch(threadIdx.x);
    for (uint32_t r0 = 0; r0 < total; r0 += PQ_THREADS) {
        const bool valid = r0 + threadIdx.x < total;
        uint4 cw[PQ_GROUPS_MAX];
#pragma unroll
        for (uint32_t g = 0; g < PQ_GROUPS_MAX; ++g) cw[g] = cw_next[g];
        const uint32_t id = id_next;
        fetch(r0 + PQ_THREADS + threadIdx.x);
        float sum = 0.f;
        if (valid) {
            // four look-ups for the four code bytes of a word (sub-spaces mm .. mm + 3), added in sub-space order
            auto look4 = [&](uint32_t word, uint32_t mm) {
                const float *t = lut_lds + (size_t)mm * TRI_PQ_KSUB;
                const float a = t[word & 0xFFu], b = t[TRI_PQ_KSUB + ((word >> 8) & 0xFFu)];
                const float c = t[2 * TRI_PQ_KSUB + ((word >> 16) & 0xFFu)], d = t[3 * TRI_PQ_KSUB + (word >> 24)];
                sum = (((sum + a) + b) + c) + d;
            };
#pragma unroll
            for (uint32_t g = 0; g < PQ_GROUPS_MAX; ++g) {
                if (g < groups) {                                                  // (uniform, as is all of m)
                    if (G || g * 16 + 16 <= m) {                                        // a whole group: 16 look-ups with nothing between them
                        look4(cw[g].x, g * 16);
                        look4(cw[g].y, g * 16 + 4);
                        look4(cw[g].z, g * 16 + 8);
                        look4(cw[g].w, g * 16 + 12);
                    } else {                                                       // the last one of an m that is no multiple of 16
                        look4(cw[g].x, g * 16);
                        if (g * 16 + 4 < m) look4(cw[g].y, g * 16 + 4);
                        if (g * 16 + 8 < m) look4(cw[g].z, g * 16 + 8);
                    }
                }
            }
        }
        const uint32_t key = tri_score_key(sum, 0u);
        const uint64_t comp = ((uint64_t)key << 32) | id;
        const bool maybe = r0 == 0 ? pq_first_round_keeps(col, ksel, valid, comp) : valid && ((uint64_t)key << 32) <= col.bound;
        pq_collect_round(col, ksel, maybe, comp);
    }
    pq_collect_settle(col, ksel);
    if (k_adc) {
        // Re-ranking: the k_adc best by table scores are scored again exactly against the stored rows (the tri_pq's own
        // row-major copy when it keeps one, else the index's blocks found through its slot map) -- squared L2 in the difference form, or the inner product, fp32, one row per
        // half-wavefront with a fixed reduction order -- and put in the order of those scores.
        const uint32_t have = col.have, l32 = threadIdx.x & 31;
        const uint8_t *qrow = qrows + (size_t)q * row_bytes;
        // (a half-wavefront works on PQ_RERANK_ROWS rows at a time, so that as many row loads are in flight per lane)
        constexpr uint32_t HW = PQ_THREADS / 32;
        const uint32_t piece_pitch = refine ? 16u : TRI_PIECE_PITCH;              // distance between a row's 16-byte pieces
        const uint8_t *rows = refine ? refine : vecs;
        for (uint32_t i0 = threadIdx.x >> 5; i0 < have; i0 += PQ_RERANK_ROWS * HW) {
            uint32_t id[PQ_RERANK_ROWS];
            size_t x[PQ_RERANK_ROWS];                                              // where the row starts in `rows`
            float acc[PQ_RERANK_ROWS];
#pragma unroll
            for (uint32_t r = 0; r < PQ_RERANK_ROWS; ++r) {
                const uint32_t i = i0 + r * HW;
                id[r] = i < have ? (uint32_t)(col.buf[i] & 0xFFFFFFFFu) : 0u;
                acc[r] = 0.f;
            }
#pragma unroll
            for (uint32_t r = 0; r < PQ_RERANK_ROWS; ++r) {
                if (refine) {
                    x[r] = (size_t)id[r] * row_bytes;
                } else {
                    const uint32_t slot = i0 + r * HW < have ? inv[id[r]] : 0u;
                    x[r] = (size_t)(slot >> 5) * tri_block_stride(row_bytes) + (slot & 31u) * 16u;
                }
            }
            for (uint32_t o = l32 * 16; o < row_bytes; o += 32 * 16) {
                const uint4 qv = *(const uint4 *)(qrow + o);
                uint4 xv[PQ_RERANK_ROWS];
#pragma unroll
                for (uint32_t r = 0; r < PQ_RERANK_ROWS; ++r)
                    xv[r] = i0 + r * HW < have ? *(const uint4 *)(rows + x[r] + (size_t)(o / 16) * piece_pitch) : uint4{0u, 0u, 0u, 0u};
#pragma unroll
                for (uint32_t r = 0; r < PQ_RERANK_ROWS; ++r) {
                    if (dtype == 1u) {
                        const pq_half8 xe = __builtin_bit_cast(pq_half8, xv[r]), qe = __builtin_bit_cast(pq_half8, qv);
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const float a = (float)xe[j], b = (float)qe[j];
                            acc[r] = metric == 0u ? __builtin_fmaf(a - b, a - b, acc[r]) : __builtin_fmaf(-a, b, acc[r]);
                        }
                    } else {
                        const pq_float4 xe = __builtin_bit_cast(pq_float4, xv[r]), qe = __builtin_bit_cast(pq_float4, qv);
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            acc[r] = metric == 0u ? __builtin_fmaf(xe[j] - qe[j], xe[j] - qe[j], acc[r]) : __builtin_fmaf(-xe[j], qe[j], acc[r]);
                    }
                }
            }
#pragma unroll
            for (uint32_t r = 0; r < PQ_RERANK_ROWS; ++r) {
                float t = acc[r];
#pragma unroll
                for (int dd = 16; dd > 0; dd >>= 1) t += __shfl_xor(t, dd, 32);
                if (l32 == 0 && i0 + r * HW < have) col.buf[i0 + r * HW] = ((uint64_t)tri_score_key(t, 0u) << 32) | id[r];
            }
        }
        __syncthreads();
        pq_sort(col.buf, have);
        if (threadIdx.x == 0) col.have = have < k ? have : k;
        __syncthreads();
    }
    const uint32_t n = col.have;
    for (uint32_t i = threadIdx.x; i < k; i += PQ_THREADS) {
        const bool real = i < n;
        const float val = real ? tri_key_score((uint32_t)(col.buf[i] >> 32), 0u) : INFINITY;
        ids_out[(size_t)q * k + i] = real ? (uint32_t)(col.buf[i] & 0xFFFFFFFFu) : 0xFFFFFFFFu;
        dist_out[(size_t)q * k + i] = metric == 1u ? (real && val == 0.f ? 0.f : -val) : val;
    }
    if (threadIdx.x == 0) n_out[q] = n;
}

// Measurement: the scan's inner loop alone -- byte-indexed look-ups into m tables in LDS, on random bytes.
__global__ __launch_bounds__(PQ_THREADS) void pq_gather_rate_kernel(uint32_t m, uint32_t rounds, uint32_t *__restrict__ sink)
{
    extern __shared__ float lut_lds[];
    for (uint32_t i = threadIdx.x; i < m * TRI_PQ_KSUB; i += PQ_THREADS) lut_lds[i] = (float)(i & 1023u);
    __syncthreads();
    uint32_t word = (blockIdx.x * PQ_THREADS + threadIdx.x) * 2654435761u + 12345u;
    float sum = 0.f;
    for (uint32_t r = 0; r < rounds; ++r) {
#pragma unroll 4
        for (uint32_t mm = 0; mm < m; mm += 4) {
            word = word * 1664525u + 1013904223u;
            const uint32_t x = word ^ (word >> 15);               // (the low bits of such a sequence repeat early)
            const float *t = lut_lds + (size_t)mm * TRI_PQ_KSUB;
            sum += t[x & 0xFFu];
            sum += t[TRI_PQ_KSUB + ((x >> 8) & 0xFFu)];
            sum += t[2 * TRI_PQ_KSUB + ((x >> 16) & 0xFFu)];
            sum += t[3 * TRI_PQ_KSUB + (x >> 24)];
        }
    }
    if (sum == -1.f) *sink = 1u;                                  // (never: the entries are not negative)
}

}  // namespace

extern "C" int pq_lds_gather_rate(uint32_t m, uint32_t rounds, void *dev_sink, void *hip_stream, double *lookups_per_s)
{
    if (!dev_sink || !lookups_per_s || m == 0 || m % 4 || m > 124 || rounds == 0 || rounds > (1u << 20))
        return tri_fail(TRI_EINVAL, "need m = 4..124, a multiple of 4, 1 <= rounds <= 2^20, a 4-byte device sink");
    hipStream_t s = (hipStream_t)hip_stream;
    int dev = 0, cus = 0;
    PQ_TRY(hipGetDevice(&dev));
    PQ_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const uint32_t lds = m * TRI_PQ_KSUB * 4;
    PQ_TRY(hipFuncSetAttribute((const void *)pq_gather_rate_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipEvent_t a = nullptr, b = nullptr;
    hipError_t e = hipEventCreate(&a);
    if (e == hipSuccess) e = hipEventCreate(&b);
    float ms = 0.f;
    for (int pass = 0; pass < 2 && e == hipSuccess; ++pass) {     // (the first pass warms up)
        e = hipEventRecord(a, s);
        if (e == hipSuccess) {
            hipLaunchKernelGGL(pq_gather_rate_kernel, dim3((unsigned)cus), dim3(PQ_THREADS), lds, s, m, rounds, (uint32_t *)dev_sink);
            e = hipGetLastError();
        }
        if (e == hipSuccess) e = hipEventRecord(b, s);
        if (e == hipSuccess) e = hipEventSynchronize(b);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
    }
    if (a) (void)hipEventDestroy(a);
    if (b) (void)hipEventDestroy(b);
    if (e != hipSuccess) return tri_fail(TRI_EHIP, "look-up rate probe -> %s", hipGetErrorString(e));
    *lookups_per_s = ms > 0.f ? (double)cus * PQ_THREADS * rounds * m / (ms * 1e-3) : 0.0;
    return TRI_OK;
}

struct tri_pq {
    const tri_index *index = nullptr;
    TriIndexView view{};
    pq_params p{};
    uint32_t dsub = 0;
    float *cb = nullptr;        // [m][dsub][256] (pq_cb_at)
    uint8_t *codes = nullptr;   // codes of the stored positions, in transposed blocks of 64 (pq_code_at)
    uint8_t *refine = nullptr;  // pq_params.refine_rows: the vectors row-major by id (pitch row_bytes), else null
};

namespace {

int pq_check(const TriIndexView &v, const pq_params *p, uint32_t *dsub)
{
    if (!p) return tri_fail(TRI_EINVAL, "params is NULL");
    const uint32_t dim = v.dev.dim;
    if (p->m == 0 || p->m % 4 != 0 || dim % p->m != 0)
        return tri_fail(TRI_EINVAL, "m = %u must be a multiple of 4 that divides dim = %u", p->m, dim);
    if (dim / p->m > TRI_PQ_DSUB_MAX) return tri_fail(TRI_EINVAL, "dim / m = %u exceeds %u", dim / p->m, TRI_PQ_DSUB_MAX);
    if ((size_t)p->m * TRI_PQ_KSUB * 4 + sizeof(PqCollector) + (2 * TRI_PQ_NPROBE_MAX + 1) * 4 + 64 > 160u * 1024u)   // (+ the list table)
        return tri_fail(TRI_EINVAL, "m = %u: the tables of a query (%u KiB) do not fit the LDS beside the selection buffer",
                        p->m, p->m * TRI_PQ_KSUB * 4 / 1024);
    if (v.n < TRI_PQ_KSUB) return tri_fail(TRI_EINVAL, "the index holds %llu vectors, fewer than a codebook has entries", (unsigned long long)v.n);
    *dsub = dim / p->m;
    return TRI_OK;
}

}  // namespace

extern "C" int pq_build_bytes(const tri_index *index, const pq_params *p, size_t *dev_bytes, size_t *tmp_bytes)
{
    if (!index || !dev_bytes || !tmp_bytes) return tri_fail(TRI_EINVAL, "NULL argument");
    TriIndexView v;
    tri_index_view(index, &v);
    uint32_t dsub = 0;
    const int rc = pq_check(v, p, &dsub);
    if (rc) return rc;
    *dev_bytes = up256((size_t)p->m * TRI_PQ_KSUB * dsub * 4) + up256((size_t)(v.n + 63) / 64 * 64 * pq_mpad(p->m)) +
                 (p->refine_rows ? up256((size_t)v.n * v.dev.row_bytes) : 0);
    *tmp_bytes = up256((size_t)PQ_TRAIN_BLOCKS * p->m * TRI_PQ_KSUB * dsub * 4) + up256((size_t)PQ_TRAIN_BLOCKS * p->m * TRI_PQ_KSUB * 4);
    return TRI_OK;
}

extern "C" int pq_build(const tri_index *index, const pq_params *p, const float *codebooks, void *dev_mem, size_t dev_mem_bytes,
                        void *tmp_dev, size_t tmp_bytes, tri_pq **out)
{
    if (!index || !dev_mem || !out) return tri_fail(TRI_EINVAL, "NULL argument");
    size_t need = 0, tmp_need = 0;
    int rc = pq_build_bytes(index, p, &need, &tmp_need);
    if (rc) return rc;
    if ((uintptr_t)dev_mem % 256 || (tmp_dev && (uintptr_t)tmp_dev % 256)) return tri_fail(TRI_EINVAL, "dev_mem and tmp_dev must be 256-byte aligned");
    if (dev_mem_bytes < need) return tri_fail(TRI_ENOMEM, "dev_mem has %zu bytes, %zu needed", dev_mem_bytes, need);
    if (!codebooks && (!tmp_dev || tmp_bytes < tmp_need)) return tri_fail(TRI_ENOMEM, "tmp_dev has %zu bytes, %zu needed to train the codebooks", tmp_bytes, tmp_need);
    tri_pq *Q = new (std::nothrow) tri_pq();
    if (!Q) return tri_fail(TRI_ENOMEM, "out of host memory");
    Q->index = index;
    tri_index_view(index, &Q->view);
    Q->p = *p;
    Q->dsub = Q->view.dev.dim / p->m;
    const TriIndexView &v = Q->view;
    const uint32_t m = p->m, dsub = Q->dsub;
    const size_t cb_bytes = (size_t)m * TRI_PQ_KSUB * dsub * 4;
    Q->cb = (float *)dev_mem;
    Q->codes = (uint8_t *)dev_mem + up256(cb_bytes);
    if (p->refine_rows) Q->refine = Q->codes + up256((size_t)(Q->view.n + 63) / 64 * 64 * pq_mpad(p->m));
    hipStream_t s = v.stream;
    auto fail = [&](int code) { delete Q; return code; };
#define PQ_TRY_B(expr)                                                                                         \
    do {                                                                                                       \
        hipError_t e_ = (expr);                                                                                \
        if (e_ != hipSuccess) return fail(tri_fail(TRI_EHIP, "%s -> %s", #expr, hipGetErrorString(e_)));       \
    } while (0)
    PQ_TRY_B(hipSetDevice(v.device));
    PQ_TRY_B(hipStreamSynchronize(s));
    const uint32_t lds = TRI_PQ_KSUB * dsub * 4;
    if (codebooks) {
        std::vector<float> t((size_t)m * TRI_PQ_KSUB * dsub);
        for (uint32_t mm = 0; mm < m; ++mm)
            for (uint32_t c = 0; c < TRI_PQ_KSUB; ++c)
                for (uint32_t e = 0; e < dsub; ++e) t[pq_cb_at(mm, c, e, dsub)] = codebooks[((size_t)mm * TRI_PQ_KSUB + c) * dsub + e];
        PQ_TRY_B(hipMemcpy(Q->cb, t.data(), cb_bytes, hipMemcpyHostToDevice));
    } else {
        float *sums = (float *)tmp_dev;                       // [run][sub-space][entry][coordinate]
        uint32_t *counts = (uint32_t *)((uint8_t *)tmp_dev + up256((size_t)PQ_TRAIN_BLOCKS * cb_bytes));
        uint64_t rows = p->train_rows ? p->train_rows : 65536;
        rows = std::min<uint64_t>(rows, v.n);
        const uint64_t stride = v.n / rows;
        hipLaunchKernelGGL(pq_init_kernel, dim3(TRI_PQ_KSUB), dim3(1024), 0, s, v.dev,
                           v.n, m, dsub, p->seed, Q->cb);
        PQ_TRY_B(hipGetLastError());
        PQ_TRY_B(hipFuncSetAttribute((const void *)pq_train_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(2 * lds)));
        for (uint32_t it = 0; it < p->train_iters; ++it) {
            hipLaunchKernelGGL(pq_train_kernel, dim3(PQ_TRAIN_BLOCKS, m), dim3(TRI_PQ_KSUB), 2 * lds, s, v.dev, rows, stride, m, dsub, Q->cb, sums, counts);
            PQ_TRY_B(hipGetLastError());
            const uint32_t total = m * TRI_PQ_KSUB * dsub;
            hipLaunchKernelGGL(pq_update_kernel, dim3((total + 255) / 256), dim3(256), 0, s, total, dsub, PQ_TRAIN_BLOCKS, sums, counts, Q->cb);
            PQ_TRY_B(hipGetLastError());
        }
    }
    hipLaunchKernelGGL(pq_assign_kernel, dim3((unsigned)((v.n + PQ_THREADS - 1) / PQ_THREADS), m), dim3(PQ_THREADS), lds, s, v.dev, v.n, m, dsub,
                       Q->cb, Q->codes);
    PQ_TRY_B(hipGetLastError());
    if (Q->refine) {
        const uint64_t pieces = (uint64_t)v.n * (v.dev.row_bytes / 16);
        hipLaunchKernelGGL(pq_refine_copy_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, s, v.dev, v.n, Q->refine);
        PQ_TRY_B(hipGetLastError());
    }
    PQ_TRY_B(hipStreamSynchronize(s));
#undef PQ_TRY_B
    *out = Q;
    return TRI_OK;
}

extern "C" int pq_destroy(tri_pq *pq)
{
    if (!pq) return TRI_OK;
    (void)hipSetDevice(pq->view.device);
    (void)hipStreamSynchronize(pq->view.stream);
    delete pq;
    return TRI_OK;
}

extern "C" int pq_export(const tri_pq *pq, float *codebooks, uint8_t *codes)
{
    if (!pq) return tri_fail(TRI_EINVAL, "pq is NULL");
    PQ_TRY(hipSetDevice(pq->view.device));
    PQ_TRY(hipStreamSynchronize(pq->view.stream));
    if (codebooks) {
        const uint32_t m = pq->p.m, dsub = pq->dsub;
        std::vector<float> raw((size_t)m * TRI_PQ_KSUB * dsub);
        PQ_TRY(hipMemcpy(raw.data(), pq->cb, raw.size() * 4, hipMemcpyDeviceToHost));
        for (uint32_t mm = 0; mm < m; ++mm)
            for (uint32_t c = 0; c < TRI_PQ_KSUB; ++c)
                for (uint32_t e = 0; e < dsub; ++e) codebooks[((size_t)mm * TRI_PQ_KSUB + c) * dsub + e] = raw[pq_cb_at(mm, c, e, dsub)];
    }
    if (codes) {
        const uint32_t m = pq->p.m;
        std::vector<uint8_t> raw((size_t)(pq->view.n + 63) / 64 * 64 * pq_mpad(m));
        PQ_TRY(hipMemcpy(raw.data(), pq->codes, raw.size(), hipMemcpyDeviceToHost));
        for (uint64_t v = 0; v < pq->view.n; ++v)
            for (uint32_t mm = 0; mm < m; ++mm) codes[v * m + mm] = raw[pq_code_at(v, mm, m)];
    }
    return TRI_OK;
}

namespace {

struct PqWs {
    uint8_t *qrows;
    float *scores;
    uint32_t *probes;
    float *lut;
    uint32_t *todo;             // per query: its probes are still to be selected by the workgroup kernel
    size_t total;
};

PqWs pq_carve(const tri_pq *pq, uint32_t nq, uint8_t *base)
{
    const TriIndexDev &d = pq->view.dev;
    const uint32_t ldc = tri_coarse_ldc(d.nlist);
    size_t off = 0;
    auto take = [&](size_t bytes) { uint8_t *p = base ? base + off : nullptr; off += up256(bytes); return p; };
    PqWs w;
    w.qrows = take((size_t)nq * d.row_bytes);
    w.scores = (float *)take((size_t)nq * ldc * 4);
    w.probes = (uint32_t *)take((size_t)nq * TRI_PQ_NPROBE_MAX * 4);
    w.lut = (float *)take((size_t)nq * pq->p.m * TRI_PQ_KSUB * 4);
    w.todo = (uint32_t *)take((size_t)nq * 4);
    w.total = off;
    return w;
}

}  // namespace

extern "C" int pq_search_bytes(const tri_pq *pq, uint32_t nq, size_t *ws_bytes)
{
    if (!pq || !ws_bytes) return tri_fail(TRI_EINVAL, "NULL argument");
    if (nq == 0) return tri_fail(TRI_EINVAL, "nq must be at least 1");
    *ws_bytes = pq_carve(pq, nq, nullptr).total;
    return TRI_OK;
}

extern "C" int pq_search_batch(tri_pq *pq, const void *queries, size_t pitch_bytes, uint32_t nq, uint32_t k, uint32_t k_adc,
                               uint32_t nprobe, uint32_t metric, void *ws, size_t ws_bytes, uint32_t *ids_out, float *dist_out, uint32_t *n_out,
                               uint32_t *probes_out)
{
    if (!pq || !queries || !ws || !ids_out || !dist_out || !n_out) return tri_fail(TRI_EINVAL, "NULL argument");
    const TriIndexDev &d = pq->view.dev;
    const uint32_t es = d.dtype == 1u ? 2u : 4u;
    if (nq == 0) return TRI_OK;
    if (k == 0 || k > TRI_PQ_KMAX) return tri_fail(TRI_EINVAL, "k must be 1..%u", TRI_PQ_KMAX);
    if (k_adc && (k_adc < k || k_adc > TRI_PQ_KMAX)) return tri_fail(TRI_EINVAL, "k_adc must be 0 or k..%u", TRI_PQ_KMAX);
    if (nprobe == 0 || nprobe > TRI_PQ_NPROBE_MAX || nprobe > d.nlist) return tri_fail(TRI_EINVAL, "nprobe must be 1..min(nlist, %u)", TRI_PQ_NPROBE_MAX);
    if (metric != TRI_L2 && metric != TRI_IP) return tri_fail(TRI_EINVAL, "metric must be TRI_L2 or TRI_IP");
    if (pitch_bytes < (size_t)d.dim * es) return tri_fail(TRI_EINVAL, "pitch_bytes %zu is shorter than a query row (%u bytes)", pitch_bytes, d.dim * es);
    if ((uintptr_t)ws % 256) return tri_fail(TRI_EINVAL, "ws must be 256-byte aligned");
    const PqWs w = pq_carve(pq, nq, (uint8_t *)ws);
    if (ws_bytes < w.total) return tri_fail(TRI_ENOMEM, "ws has %zu bytes, %zu needed", ws_bytes, w.total);
    PQ_TRY(hipSetDevice(pq->view.device));
    hipStream_t s = pq->view.stream;
    const uint32_t m = pq->p.m, ldc = tri_coarse_ldc(d.nlist);
    const uint32_t lut_bytes = m * TRI_PQ_KSUB * 4;
    typedef void (*scan_fn)(const float *, uint32_t, const uint32_t *, uint32_t, const uint32_t *, const uint32_t *, const uint8_t *,
                            uint32_t, uint32_t, uint32_t, const uint8_t *, const uint8_t *, const uint32_t *, const uint8_t *, uint32_t,
                            uint32_t, uint32_t *, float *, uint32_t *);
    static const scan_fn scans[PQ_GROUPS_MAX + 1] = {pq_scan_kernel<0>, pq_scan_kernel<1>, pq_scan_kernel<2>, pq_scan_kernel<3>, pq_scan_kernel<4>,
                                                     pq_scan_kernel<5>, pq_scan_kernel<6>, pq_scan_kernel<7>, pq_scan_kernel<8>};
    const uint32_t variant = m % 16 == 0 ? m / 16 : 0;
    static uint32_t lds_limit[PQ_GROUPS_MAX + 1] = {};          // (more LDS than a kernel gets by default: raised once per growth)
    if (lut_bytes > lds_limit[variant]) {
        PQ_TRY(hipFuncSetAttribute((const void *)scans[variant], hipFuncAttributeMaxDynamicSharedMemorySize, (int)lut_bytes));
        lds_limit[variant] = lut_bytes;
    }
    hipLaunchKernelGGL(pq_pad_queries_kernel, dim3(nq), dim3(256), 0, s, (const uint8_t *)queries, pitch_bytes, nq, d.dim * es,
                       d.row_bytes, w.qrows);
    PQ_TRY(hipGetLastError());
    PQ_TRY(tri_launch_coarse_gemm(s, d.dtype == 1u ? 1 : 0, w.qrows, d.row_bytes, nq, d.centroids, d.cnorm, d.nlist, d.row_bytes,
                                  nullptr, 0u, metric, w.scores, ldc));
    uint32_t *probes = probes_out ? probes_out : w.probes;
    const bool by_wave = d.nlist <= PQ_PW_NLIST && nprobe <= PQ_PW_NPROBE;
    if (by_wave) {
        hipLaunchKernelGGL(pq_probe_wave_kernel, dim3((nq + PQ_PW_ROWS - 1) / PQ_PW_ROWS), dim3(64 * PQ_PW_ROWS), 0, s, w.scores, ldc, d.nlist, nprobe,
                           metric, nq, probes, w.todo);
        PQ_TRY(hipGetLastError());
    }
    hipLaunchKernelGGL(pq_probe_kernel, dim3(nq), dim3(PQ_PROBE_THREADS), 0, s, w.scores, ldc, d.nlist, nprobe, metric, probes,
                       by_wave ? (const uint32_t *)w.todo : (const uint32_t *)nullptr);
    PQ_TRY(hipGetLastError());
    hipLaunchKernelGGL(pq_lut_kernel, dim3((nq + PQ_LUT_Q - 1) / PQ_LUT_Q, m / PQ_LUT_M), dim3(64 * PQ_LUT_M), 0, s, w.qrows, d.row_bytes, d.dtype, nq, m,
                       pq->dsub, metric, pq->cb, w.lut);
    PQ_TRY(hipGetLastError());
    hipLaunchKernelGGL(scans[variant], dim3(nq), dim3(PQ_THREADS), lut_bytes, s, w.lut, m, probes, nprobe, d.list_off, d.ids, pq->codes,
                       k, metric, k_adc, w.qrows, (const uint8_t *)d.vecs, d.inv, (const uint8_t *)pq->refine, d.row_bytes, d.dtype, ids_out, dist_out, n_out);
    PQ_TRY(hipGetLastError());
    return TRI_OK;
}

extern "C" int pq_sync(tri_pq *pq)
{
    if (!pq) return tri_fail(TRI_EINVAL, "pq is NULL");
    PQ_TRY(hipSetDevice(pq->view.device));
    PQ_TRY(hipStreamSynchronize(pq->view.stream));
    return TRI_OK;
}
