// Per-query top-k (Sec. 3.2 of the paper: the step that returns each distance to the request it
// belongs to and merges it into that request's candidate list; here the request's candidates of one step are the (score, position) pairs the
// scan kept for its work items plus its running top-k).
//
// Order: ascending 64-bit composite (key << 32 | id), key = order-preserving image of the fp32
// score (bit-flipped for inner product, so "smaller key" always means "better").  Equal scores are
// therefore ordered by ascending id, which makes the result independent of how the candidates
// were batched.
//
// One workgroup selects for one query, in LDS.  Sorting networks over thousands of elements cost a
// hundred barriers; here sorting is kept for the few elements that survive a bucket cut:
//  * k best of n <= SEL_CAP composites in LDS (sel_pool_topk): 2048 buckets, linear in the key between
//    the smallest and largest key present; a prefix sum finds the bucket B that holds rank k; the
//    elements of buckets <= B (k plus a handful) are compacted and sorted -- by counting ranks when
//    they are at most 256 (one element per thread, no barriers inside), else by a bitonic network.
//    Degenerate inputs (everything in one bucket) fall back to the network over all n.
//  * a bound for rank m among n keys in LDS (sel_keys_threshold): same buckets; the result is the
//    largest key of bucket B, so at least m keys are not above it, and only a few more.
//  * candidate sets larger than SEL_CAP: a sample of about SEL_SAMPLE keys gives, through the bound
//    above, a threshold that almost surely admits at least k and far fewer than SEL_CAP candidates; ONE
//    pass collects those not worse than it.  Whatever the sample says, the result is exact whenever the
//    pass collected between k and SEL_CAP candidates: the k best of the collected set are then the k
//    best of all.
//  * a query whose region of the candidate buffer was too small for what the scan's filter let through (the
//    region is sized by expectation, the counter says how much was asked for): its candidates are then ALL
//    vectors of the lists it scanned in this step, scored again here, by the same contraction in the same order
//    as in the scan kernels (so every score has the same bits), and enumerated as often as the selection needs.
//  * otherwise (heavy ties, adversarial order): three histogram passes (11 + 11 + 10 bits) find
//    the key T of the k-th best element; if more elements equal T than are still needed, three more
//    passes over the ids of those elements find the largest id to keep; one pass gathers exactly k.
#include "tri_common.h"
#include "tri_mfma.h"

#define SEL_BINS 2048
#define SEL_SEGCACHE 544   // pair-segment descriptors cached in LDS (128 lists x 4 chunks, and some)
#define SEL_CAP 2816       // composites held in LDS; chosen so that a workgroup stays under 40 KB of LDS and four of
                           // them share a compute unit (with 4096 three did, and the three selection kernels ran slower)
#define SEL_SMALL 1024     // composites in the second array (which shares its storage with the histogram)
#define SEL_RANK_MAX 256   // sorted by rank counting up to here (one element per thread)
#define SEL_SAMPLE 1024    // target size of the key sample
#define SEL_UNROLL 8

__device__ __forceinline__ uint32_t sel_key(float f, uint32_t desc) { return tri_score_key(f, desc); }
__device__ __forceinline__ float sel_unkey(uint32_t key, uint32_t desc) { return tri_key_score(key, desc); }

// Candidate source of one query: pair segments [0, nps) inside the candidate buffer -- (score bits,
// position) pairs, id = ids[id_off + position] -- and at most one dense array (scores, with ids or, if
// dense_ids is null, id = element number).
struct SelSeg {
    uint32_t off;      // first pair of the segment (pair index into cand)
    uint32_t len;      // pairs
    uint32_t id_off;   // index of the list's first id in ids
    uint32_t pfx;      // len summed over this and all earlier segments (cached descriptors only)
};

// Candidates that are not stored but scored on demand: every vector of `take` inverted lists of one index
// against one query row.
struct SelRescan {
    const uint32_t *item_glist;   // the lists: item_glist[item_base .. item_base + take)
    const uint32_t *glist_len, *glist_voff;
    const TriIndexDev *ix;
    const uint8_t *qrow;          // the query's padded row
    float qnorm;
    uint32_t is_l2;
    uint32_t item_base, take;
    uint32_t total;               // vectors in those lists
};

struct SelSrc {
    const uint2 *cand;
    const uint32_t *ids;
    const float *dense;
    const uint32_t *dense_ids;
    uint32_t nps;
    uint32_t dense_len;
    const SelRescan *rescan;      // or NULL
};

struct SelShared {
    uint64_t pool[SEL_CAP];        // candidates (the key sample uses it as uint32_t[2 * SEL_CAP])
    union {
        uint32_t hist[SEL_BINS];
        uint64_t small[SEL_SMALL];
    };
    SelSeg seg[SEL_SEGCACHE];
    uint32_t wave_tot[8];
    uint32_t wmin[TRI_SEL_THREADS / 64], wmax[TRI_SEL_THREADS / 64];
    uint32_t digit, need, count, cnt, tmax, tmin, total_pairs;
};

__device__ __forceinline__ uint32_t sel_id(const SelSrc &src, uint32_t idx, bool pair)
{
    return pair ? src.ids[idx] : (src.dense_ids ? src.dense_ids[idx] : idx);
}

// Inclusive scan of one value per thread across the workgroup (TRI_SEL_THREADS threads).
__device__ __forceinline__ uint32_t sel_block_scan_incl(uint32_t v, uint32_t *wave_tot)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t x = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t y = __shfl_up(x, d, 64);
        if (lane >= (uint32_t)d) x += y;
    }
    if (lane == 63) wave_tot[wave] = x;
    __syncthreads();
    uint32_t add = 0;
    for (uint32_t w = 0; w < wave; ++w) add += wave_tot[w];
    __syncthreads();
    return x + add;
}

// After a histogram pass: find the smallest digit D with cumulative count >= need.
// Writes sh.digit = D, sh.need = need - (count of digits < D), sh.count = hist[D].
__device__ __forceinline__ void sel_find_digit(SelShared &sh, uint32_t nbins, uint32_t need)
{
    const uint32_t per = nbins / TRI_SEL_THREADS;   // 8 or 4
    const uint32_t b0 = threadIdx.x * per;
    uint32_t mine = 0;
    for (uint32_t i = 0; i < per; ++i) mine += sh.hist[b0 + i];
    const uint32_t incl = sel_block_scan_incl(mine, sh.wave_tot);
    const uint32_t excl = incl - mine;
    if (excl < need && need <= incl) {
        uint32_t run = excl;
        for (uint32_t i = 0; i < per; ++i) {
            const uint32_t h = sh.hist[b0 + i];
            if (run + h >= need) {
                sh.digit = b0 + i;
                sh.need = need - run;
                sh.count = h;
                break;
            }
            run += h;
        }
    }
    __syncthreads();
}

// Descriptors of the first SEL_SEGCACHE pair segments -> LDS, with running sums of their lengths;
// sh.total_pairs = pairs in ALL pair segments.  Ends with a barrier.
template <class SegFn>
__device__ __forceinline__ void sel_cache_segments(SelShared &sh, uint32_t nps, SegFn seg_of)
{
    const uint32_t ncache = nps < SEL_SEGCACHE ? nps : SEL_SEGCACHE;
    const uint32_t per = (ncache + TRI_SEL_THREADS - 1) / TRI_SEL_THREADS;      // <= 3
    const uint32_t s0 = threadIdx.x * per;
    SelSeg mine[(SEL_SEGCACHE + TRI_SEL_THREADS - 1) / TRI_SEL_THREADS];
    uint32_t sum = 0;
#pragma unroll
    for (uint32_t i = 0; i < (SEL_SEGCACHE + TRI_SEL_THREADS - 1) / TRI_SEL_THREADS; ++i)
        if (i < per && s0 + i < ncache) {
            mine[i] = seg_of(s0 + i);
            sum += mine[i].len;
        }
    const uint32_t incl = sel_block_scan_incl(sum, sh.wave_tot);
    uint32_t rest_incl = 0;                      // segments beyond the cache (very large probe counts only)
    if (nps > SEL_SEGCACHE) {
        uint32_t rest = 0;
        for (uint32_t s = SEL_SEGCACHE + threadIdx.x; s < nps; s += TRI_SEL_THREADS) rest += seg_of(s).len;
        rest_incl = sel_block_scan_incl(rest, sh.wave_tot);
    }
    uint32_t run = incl - sum;
#pragma unroll
    for (uint32_t i = 0; i < (SEL_SEGCACHE + TRI_SEL_THREADS - 1) / TRI_SEL_THREADS; ++i)
        if (i < per && s0 + i < ncache) {
            run += mine[i].len;
            mine[i].pfx = run;
            sh.seg[s0 + i] = mine[i];
        }
    if (threadIdx.x == TRI_SEL_THREADS - 1) sh.total_pairs = incl + rest_incl;
    __syncthreads();
}

// Scores of the 32 stored vectors of one block (at `block`: 32 vectors interleaved by 16-byte pieces, zeros behind
// the list's last vector) against the query, by one wavefront:
// the query's pieces as the first operand of every product (all 32 rows of that operand are the query), the
// vectors' as the second, 128-byte group after group and 32-byte chunk after chunk -- the order in which the scan
// kernels accumulate, so the sums come out bit for bit the same.  Lane l returns the score of vector v0 + l % 32.
template <int DT>
__device__ __forceinline__ float sel_rescan_block(const SelRescan &rs, const uint8_t *__restrict__ block, uint32_t lane)
{
    const uint32_t r = lane & 31, kg = lane >> 5;
    const uint32_t row_bytes = rs.ix->row_bytes;
    const uint8_t *x = block + kg * TRI_PIECE_PITCH + r * 16;            // piece 8g + 2c + kg of vector r: + g * 4096 + c * 1024
    const uint8_t *q = rs.qrow + kg * 16;
    tri_f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    for (uint32_t g = 0; g < row_bytes; g += 128)
#pragma unroll
        for (int c = 0; c < 4; ++c)
            tri_mma32<DT>(acc, *(const uint4 *)(q + g + c * 32), *(const uint4 *)(x + (size_t)g * 32 + c * 1024));
    return acc[0];
}

// f(valid, key, stored position, true) for every stride-th 32-vector block of the lists of rs, uniformly by all
// 64 lanes; the blocks are dealt round-robin to the workgroup's wavefronts.
template <class Fn>
__device__ __forceinline__ void sel_rescan_for_each(const SelRescan &rs, uint32_t desc, uint32_t stride, Fn f)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr uint32_t NW = TRI_SEL_THREADS / 64;
    const uint32_t row_bytes = rs.ix->row_bytes;
    uint32_t gblock = 0;
    for (uint32_t it = 0; it < rs.take; ++it) {
        const uint32_t g = rs.item_glist[rs.item_base + it];
        const uint32_t len = rs.glist_len[g], voff = rs.glist_voff[g];
        const uint8_t *list = (const uint8_t *)rs.ix->vecs + (size_t)rs.ix->blk_off[g - rs.ix->list_base] * tri_block_stride(row_bytes);
        for (uint32_t v0 = 0; v0 < len; v0 += 32, ++gblock) {
            if (gblock % stride != 0 || (gblock / stride) % NW != wave) continue;
            const uint8_t *block = list + (size_t)(v0 / 32u) * tri_block_stride(row_bytes);
            const float dot = rs.ix->dtype == 1u ? sel_rescan_block<TRI_DT_F16>(rs, block, lane)
                                                 : sel_rescan_block<TRI_DT_F32>(rs, block, lane);
            const uint32_t v = v0 + (lane & 31);
            const bool valid = lane < 32 && v < len;
            const float vn = rs.ix->vnorm[voff + (valid ? v : v0)];
            const float score = rs.is_l2 ? (vn + rs.qnorm) - 2.0f * dot : dot;
            f(valid, valid ? sel_key(score, desc) : 0xFFFFFFFFu, voff + v, true);
        }
    }
}

// Enumerate candidates with wavefront-uniform control flow: f(valid, key, idx, pair) is called by all
// 64 lanes together (valid = this lane has an element; idx, pair: what sel_id needs).  Work is cut into
// chunks of 64 * SEL_UNROLL elements that the wavefronts take round-robin, and the loads of a chunk are
// issued together.
//  * pair segments, all cached: ONE flat index space over all of them (a lane finds its segment by
//    binary search in the running sums), so hundreds of segments of a dozen pairs cost no more than one
//    long one.  stride > 1 visits every stride-th flat index.
//  * pair segments beyond the cache: segment by segment (stride > 1: the first len/stride of each).
//  * the dense array: stride > 1 visits its first ceil(len / stride) elements.
// (The order of candidates inside the candidate buffer and of the centroids carries no information
// about scores, which is what makes such subsets usable as samples.)
template <bool RESCAN, class SegFn, class Fn>
__device__ __forceinline__ void sel_for_each(const SelShared &sh, const SelSrc &src, SegFn seg_of, uint32_t desc,
                                             uint32_t stride, Fn f)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr uint32_t CH = 64 * SEL_UNROLL;
    constexpr uint32_t NW = TRI_SEL_THREADS / 64;
    if (src.nps && src.nps <= SEL_SEGCACHE) {
        const uint32_t nps = src.nps;
        const uint32_t nvis = (sh.total_pairs + stride - 1) / stride;
        uint32_t top = 1;
        while (top * 2 <= nps) top *= 2;
        for (uint32_t i0 = wave * CH; i0 < nvis; i0 += NW * CH) {
            uint2 v[SEL_UNROLL];
            uint32_t idx[SEL_UNROLL];
#pragma unroll
            for (int u = 0; u < SEL_UNROLL; ++u) {
                const uint32_t i = i0 + u * 64 + lane;
                const uint32_t e = i < nvis ? i * stride : 0u;
                uint32_t lo = 0;                                 // segments whose running sum is <= e
                for (uint32_t step = top; step > 0; step >>= 1) {
                    const uint32_t m = lo + step;
                    if (m <= nps && sh.seg[m - 1].pfx <= e) lo = m;
                }
                const SelSeg sg = sh.seg[lo < nps ? lo : nps - 1];
                const uint32_t within = e - (sg.pfx - sg.len);
                v[u] = i < nvis ? src.cand[(size_t)sg.off + within] : make_uint2(0u, 0u);
                idx[u] = sg.id_off;
            }
#pragma unroll
            for (int u = 0; u < SEL_UNROLL; ++u) {
                const bool valid = i0 + u * 64 + lane < nvis;
                f(valid, valid ? sel_key(__uint_as_float(v[u].x), desc) : 0xFFFFFFFFu, idx[u] + v[u].y, true);
            }
        }
    } else if (src.nps) {
        uint32_t next = wave, base = 0;
        for (uint32_t s = 0; s < src.nps; ++s) {
            const SelSeg sg = s < SEL_SEGCACHE ? sh.seg[s] : seg_of(s);
            const uint32_t n = stride > 1 ? (sg.len + stride - 1) / stride : sg.len;
            const uint32_t nch = (n + CH - 1) / CH;
            while (next < base + nch) {
                const uint32_t i0 = (next - base) * CH + lane;
                uint2 v[SEL_UNROLL];
#pragma unroll
                for (int u = 0; u < SEL_UNROLL; ++u)
                    v[u] = i0 + u * 64 < n ? src.cand[(size_t)sg.off + i0 + u * 64] : make_uint2(0u, 0u);
#pragma unroll
                for (int u = 0; u < SEL_UNROLL; ++u) {
                    const bool valid = i0 + u * 64 < n;
                    f(valid, valid ? sel_key(__uint_as_float(v[u].x), desc) : 0xFFFFFFFFu, sg.id_off + v[u].y, true);
                }
                next += NW;
            }
            base += nch;
        }
    }
    if (src.dense_len) {
        const uint32_t n = stride > 1 ? (src.dense_len + stride - 1) / stride : src.dense_len;
        for (uint32_t i0 = wave * CH; i0 < n; i0 += NW * CH) {
            float v[SEL_UNROLL];
#pragma unroll
            for (int u = 0; u < SEL_UNROLL; ++u) v[u] = i0 + u * 64 + lane < n ? src.dense[i0 + u * 64 + lane] : 0.f;
#pragma unroll
            for (int u = 0; u < SEL_UNROLL; ++u) {
                const bool valid = i0 + u * 64 + lane < n;
                f(valid, valid ? sel_key(v[u], desc) : 0xFFFFFFFFu, i0 + u * 64 + lane, false);
            }
        }
    }
    if constexpr (RESCAN) {
        if (src.rescan) sel_rescan_for_each(*src.rescan, desc, stride, f);
    }
}

// Append slot for every lane with pred set: one LDS atomic per wavefront call, not per lane.
__device__ __forceinline__ uint32_t sel_append_pos(bool pred, uint32_t *counter)
{
    const uint64_t m = __ballot(pred);
    if (m == 0) return 0;
    const uint32_t lane = threadIdx.x & 63;
    const int leader = __ffsll((unsigned long long)m) - 1;
    uint32_t base = 0;
    if ((int)lane == leader) base = atomicAdd(counter, (uint32_t)__popcll(m));
    base = __shfl(base, leader, 64);
    return base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
}

// Bitonic sort (ascending) of n elements of LDS array a, padded with all-ones up to a power of two.
template <typename T>
__device__ __forceinline__ void sel_bitonic(T *a, uint32_t n)
{
    const uint32_t tid = threadIdx.x;
    uint32_t np2 = 1;
    while (np2 < n) np2 <<= 1;
    for (uint32_t i = n + tid; i < np2; i += TRI_SEL_THREADS) a[i] = (T)~(T)0;
    __syncthreads();
    for (uint32_t size = 2; size <= np2; size <<= 1) {
        for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
            for (uint32_t i = tid; i < np2 / 2; i += TRI_SEL_THREADS) {
                const uint32_t lo = 2 * i - (i & (stride - 1));   // index with the `stride` bit clear
                const uint32_t hi = lo + stride;
                const bool up = (lo & size) == 0;
                const T x = a[lo], y = a[hi];
                if ((x > y) == up) {
                    a[lo] = y;
                    a[hi] = x;
                }
            }
            __syncthreads();
        }
    }
}

// ---- buckets ------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t sel_key_of(uint32_t x) { return x; }
__device__ __forceinline__ uint32_t sel_key_of(uint64_t x) { return (uint32_t)(x >> 32); }

// Bucket of a key: monotone in the key (conversions, the product with a positive factor and the
// truncation all preserve order), 0 at or below kmin, SEL_BINS - 1 at or above the largest key.
__device__ __forceinline__ uint32_t sel_bucket(uint32_t key, uint32_t kmin, float scale)
{
    if (key <= kmin) return 0u;
    return (uint32_t)fminf((float)(key - kmin) * scale, (float)(SEL_BINS - 1));
}

// Bucket range from the smallest and largest key (every thread passes those of its own keys; all-ones,
// the padding value, must be left out).  Also zeroes the histogram.  Ends with a barrier.  Returns the
// scale of sel_bucket.
__device__ __forceinline__ float sel_range(SelShared &sh, uint32_t lo, uint32_t hi, uint32_t &kmin, uint32_t *kmax = nullptr)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) {
        const uint32_t l2 = (uint32_t)__shfl_xor((int)lo, d, 64), h2 = (uint32_t)__shfl_xor((int)hi, d, 64);
        lo = l2 < lo ? l2 : lo;
        hi = h2 > hi ? h2 : hi;
    }
    if (lane == 0) {
        sh.wmin[wave] = lo;
        sh.wmax[wave] = hi;
    }
    for (uint32_t i = threadIdx.x; i < SEL_BINS; i += TRI_SEL_THREADS) sh.hist[i] = 0;
    __syncthreads();
#pragma unroll
    for (uint32_t w = 0; w < TRI_SEL_THREADS / 64; ++w) {
        lo = sh.wmin[w] < lo ? sh.wmin[w] : lo;
        hi = sh.wmax[w] > hi ? sh.wmax[w] : hi;
    }
    kmin = lo;
    if (kmax) *kmax = hi;
    return hi > lo ? ((float)SEL_BINS - 0.01f) / (float)(hi - lo) : 0.f;
}

// A key T with at least m of the n keys a[0..n) not above it, and few more (a: LDS, n >= m >= 1 keys of
// which at least m are not the padding value all-ones).  Uses sh.hist.
// The buckets are linear in the KEY, and keys are bit patterns of floats: roughly logarithmic in the score, and
// around a score of zero immensely sparse (all the tiny values of either sign lie between -x and +x).  Scores that
// straddle zero therefore leave the best keys crowded into a handful of buckets, and the largest key of the
// bucket that holds rank m may admit several times m keys.  So the cut is refined: while the bucket of rank m holds
// more than a few keys, its own key range is cut into buckets again (each level narrows the range 2048-fold).
__device__ uint32_t sel_keys_threshold(SelShared &sh, const uint32_t *a, uint32_t n, uint32_t m)
{
    uint32_t range_lo = 0u, range_hi = 0xFFFFFFFEu;      // keys still in play
    uint32_t need = m, t = 0xFFFFFFFEu;
    for (int level = 0; level < 3; ++level) {
        uint32_t kmin, lo = 0xFFFFFFFFu, hi = 0u;
        for (uint32_t i = threadIdx.x; i < n; i += TRI_SEL_THREADS) {
            const uint32_t key = a[i];
            if (key >= range_lo && key <= range_hi) {
                lo = key < lo ? key : lo;
                hi = key > hi ? key : hi;
            }
        }
        uint32_t kmax;
        float scale = sel_range(sh, lo, hi, kmin, &kmax);
        // (first level: buckets linear in the SCORE -- the float a key stands for, negated for descending order --,
        // which spreads the keys evenly where scores straddle zero; deeper levels, inside one such bucket: linear in the key)
        float fmin = 0.f;
        bool by_value = false;
        if (level == 0 && kmax > kmin) {
            fmin = tri_key_score(kmin, 0u);
            const float span = tri_key_score(kmax, 0u) - fmin;
            if (span > 0.f && span < 3.0e38f) {
                by_value = true;
                scale = ((float)SEL_BINS - 0.01f) / span;
            }
        }
        auto bucket_of = [&](uint32_t key) {
            return by_value ? (uint32_t)fminf(fmaxf((tri_key_score(key, 0u) - fmin) * scale, 0.f), (float)(SEL_BINS - 1))
                            : sel_bucket(key, kmin, scale);
        };
        for (uint32_t i = threadIdx.x; i < n; i += TRI_SEL_THREADS) {
            const uint32_t key = a[i];
            if (key >= range_lo && key <= range_hi) atomicAdd(&sh.hist[bucket_of(key)], 1u);
        }
        if (threadIdx.x == 0) {
            sh.tmax = 0u;
            sh.tmin = 0xFFFFFFFFu;
        }
        __syncthreads();
        sel_find_digit(sh, SEL_BINS, need);
        const uint32_t B = sh.digit, in_bucket = sh.count, need_in = sh.need;
        uint32_t best = 0u, least = 0xFFFFFFFFu;
        for (uint32_t i = threadIdx.x; i < n; i += TRI_SEL_THREADS) {
            const uint32_t key = a[i];
            if (key >= range_lo && key <= range_hi && bucket_of(key) == B) {
                best = key > best ? key : best;
                least = key < least ? key : least;
            }
        }
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) {
            const uint32_t b2 = (uint32_t)__shfl_xor((int)best, d, 64), l2 = (uint32_t)__shfl_xor((int)least, d, 64);
            best = b2 > best ? b2 : best;
            least = l2 < least ? l2 : least;
        }
        if ((threadIdx.x & 63) == 0) {
            atomicMax(&sh.tmax, best);
            atomicMin(&sh.tmin, least);
        }
        __syncthreads();
        t = sh.tmax;
        const uint32_t t_lo = sh.tmin;
        __syncthreads();                 // (sh.tmax, sh.tmin and the histogram may be reused right away)
        if (in_bucket <= need_in + 4u || t_lo == t) break;      // the bucket admits at most a few keys beyond rank m, or holds equal keys only
        range_lo = t_lo;
        range_hi = t;
        need = need_in;
    }
    return t;
}

// Sort m <= SEL_RANK_MAX composites by counting, src -> dst (both LDS, distinct): the thread that owns an
// element counts the elements ordered before it and writes it to that place.  Every thread of a
// wavefront reads the same address in each round (a broadcast).  Ends with a barrier.
__device__ __forceinline__ void sel_rank_sort(const uint64_t *src, uint32_t m, uint64_t *dst)
{
    const uint32_t t = threadIdx.x;
    const uint64_t x = t < m ? src[t] : ~0ull;
    uint32_t rank = 0;
    uint32_t u = 0;
    for (; u + 4 <= m; u += 4) {
        const uint64_t y0 = src[u], y1 = src[u + 1], y2 = src[u + 2], y3 = src[u + 3];
        rank += (y0 < x || (y0 == x && u < t)) + (y1 < x || (y1 == x && u + 1 < t)) +
                (y2 < x || (y2 == x && u + 2 < t)) + (y3 < x || (y3 == x && u + 3 < t));
    }
    for (; u < m; ++u) {
        const uint64_t y = src[u];
        rank += (y < x || (y == x && u < t));
    }
    if (t < m) dst[rank] = x;
    __syncthreads();
}

// The k best of the n <= SEL_CAP composites in sh.pool[0..n), sorted ascending; returns where they are
// (sh.pool or sh.small).  All threads must call it with everything in sh.pool visible (after a barrier);
// it ends with a barrier.
__device__ const uint64_t *sel_pool_topk(SelShared &sh, uint32_t n, uint32_t k)
{
    if (n <= SEL_RANK_MAX) {
        sel_rank_sort(sh.pool, n, sh.small);
        return sh.small;
    }
    if (k < n && k < SEL_SMALL) {
        uint32_t kmin, lo = 0xFFFFFFFFu, hi = 0u;
        for (uint32_t i = threadIdx.x; i < n; i += TRI_SEL_THREADS) {
            const uint32_t key = sel_key_of(sh.pool[i]);
            lo = key < lo ? key : lo;
            hi = key > hi ? key : hi;
        }
        const float scale = sel_range(sh, lo, hi, kmin);
        for (uint32_t i = threadIdx.x; i < n; i += TRI_SEL_THREADS)
            atomicAdd(&sh.hist[sel_bucket(sel_key_of(sh.pool[i]), kmin, scale)], 1u);
        if (threadIdx.x == 0) sh.cnt = 0;
        __syncthreads();
        sel_find_digit(sh, SEL_BINS, k);
        const uint32_t B = sh.digit;
        const uint32_t c_le = k - sh.need + sh.count;        // elements in buckets <= B
        __syncthreads();                                      // the histogram is dead from here: sh.small reuses it
        if (c_le <= SEL_SMALL) {
            for (uint32_t i0 = 0; i0 < n; i0 += TRI_SEL_THREADS) {
                const uint32_t i = i0 + threadIdx.x;
                const uint64_t x = i < n ? sh.pool[i] : ~0ull;
                const bool take = i < n && sel_bucket(sel_key_of(x), kmin, scale) <= B;
                const uint32_t pos = sel_append_pos(take, &sh.cnt);
                if (take) sh.small[pos] = x;
            }
            __syncthreads();
            if (c_le <= SEL_RANK_MAX) {
                sel_rank_sort(sh.small, c_le, sh.pool);
                return sh.pool;
            }
            sel_bitonic(sh.small, c_le);
            return sh.small;
        }
    }
    sel_bitonic(sh.pool, n);
    return sh.pool;
}

// Exact radix select of the k best into sh.pool[0..k), unsorted.  total > k.
template <bool RESCAN, class SegFn>
__device__ void sel_radix(SelShared &sh, const SelSrc &src, SegFn seg_of, uint32_t k, uint32_t desc)
{
    const uint32_t tid = threadIdx.x;
    uint32_t T = 0, Tid = 0xFFFFFFFFu;
    uint32_t need = k, prefix = 0, count_eq = 0;
    const uint32_t shifts[3] = {21, 10, 0}, widths[3] = {11, 11, 10};
    for (int pass = 0; pass < 3; ++pass) {
        const uint32_t shift = shifts[pass], width = widths[pass], nb = 1u << width;
        for (uint32_t i = tid; i < SEL_BINS; i += TRI_SEL_THREADS) sh.hist[i] = 0;
        __syncthreads();
        const uint32_t hi_shift = shift + width;
        sel_for_each<RESCAN>(sh, src, seg_of, desc, 1u, [&](bool valid, uint32_t key, uint32_t, bool) {
            if (valid && (pass == 0 || (key >> hi_shift) == prefix)) atomicAdd(&sh.hist[(key >> shift) & (nb - 1)], 1u);
        });
        __syncthreads();
        sel_find_digit(sh, nb, need);
        prefix = (prefix << width) | sh.digit;
        need = sh.need;
        count_eq = sh.count;
        __syncthreads();
    }
    T = prefix;
    // ties at T: keep the `need` smallest ids among the count_eq elements equal to T
    if (need < count_eq) {
        uint32_t idprefix = 0, need_id = need;
        for (int pass = 0; pass < 3; ++pass) {
            const uint32_t shift = shifts[pass], width = widths[pass], nb = 1u << width;
            for (uint32_t i = tid; i < SEL_BINS; i += TRI_SEL_THREADS) sh.hist[i] = 0;
            __syncthreads();
            const uint32_t hi_shift = shift + width;
            sel_for_each<RESCAN>(sh, src, seg_of, desc, 1u, [&](bool valid, uint32_t key, uint32_t idx, bool pair) {
                if (!valid || key != T) return;
                const uint32_t id = sel_id(src, idx, pair);
                if (pass == 0 || (id >> hi_shift) == idprefix) atomicAdd(&sh.hist[(id >> shift) & (nb - 1)], 1u);
            });
            __syncthreads();
            sel_find_digit(sh, nb, need_id);
            idprefix = (idprefix << width) | sh.digit;
            need_id = sh.need;
            __syncthreads();
        }
        Tid = idprefix;
    }
    if (tid == 0) sh.cnt = 0;
    __syncthreads();
    sel_for_each<RESCAN>(sh, src, seg_of, desc, 1u, [&](bool valid, uint32_t key, uint32_t idx, bool pair) {
        bool take = valid && key <= T;
        uint32_t id = 0;
        if (take) {
            id = sel_id(src, idx, pair);
            take = key < T || id <= Tid;
        }
        const uint32_t pos = sel_append_pos(take, &sh.cnt);
        if (take && pos < SEL_CAP) sh.pool[pos] = ((uint64_t)key << 32) | id;
    });
    __syncthreads();
}

// Select the k best candidates of src, sorted ascending by (key, id); *n_out = min(k, total).  Returns
// where they are in LDS.  All threads of the workgroup must call it; it ends with a barrier.
template <bool RESCAN, class SegFn>
__device__ const uint64_t *sel_block_topk(SelShared &sh, const SelSrc &src, SegFn seg_of, uint32_t k, uint32_t desc,
                                          uint32_t *n_out)
{
    const uint32_t tid = threadIdx.x;
    sel_cache_segments(sh, src.nps, seg_of);
    const uint32_t total = sh.total_pairs + src.dense_len + (RESCAN && src.rescan ? src.rescan->total : 0u);
    *n_out = total < k ? total : k;
    if (tid == 0) sh.cnt = 0;
    __syncthreads();
    if (total <= SEL_CAP) {
        // ---- everything fits
        sel_for_each<RESCAN>(sh, src, seg_of, desc, 1u, [&](bool valid, uint32_t key, uint32_t idx, bool pair) {
            const uint32_t pos = sel_append_pos(valid, &sh.cnt);
            if (valid) sh.pool[pos] = ((uint64_t)key << 32) | sel_id(src, idx, pair);
        });
        __syncthreads();
        return sel_pool_topk(sh, total, k);
    }
    // ---- threshold from a sample
    uint32_t *skeys = (uint32_t *)sh.pool;
    const uint32_t stride = (total + SEL_SAMPLE - 1) / SEL_SAMPLE;
    sel_for_each<RESCAN>(sh, src, seg_of, desc, stride, [&](bool valid, uint32_t key, uint32_t, bool) {
        const uint32_t pos = sel_append_pos(valid, &sh.cnt);
        if (valid && pos < 2 * SEL_CAP) skeys[pos] = key;      // (a few sample keys too many are simply dropped)
    });
    __syncthreads();
    const uint32_t ns = sh.cnt < 2 * SEL_CAP ? sh.cnt : 2 * SEL_CAP;
    // expected rank of the k-th best inside the sample, plus five standard deviations and a floor
    const float mu = (float)k * (float)ns / (float)total;
    const uint32_t m = (uint32_t)(mu + 5.0f * sqrtf(mu) + 4.0f);
    bool done = false;
    const uint64_t *res = sh.pool;
    if (m < ns) {
        const uint32_t t0 = sel_keys_threshold(sh, skeys, ns, m + 1);
        if (tid == 0) sh.cnt = 0;
        __syncthreads();
        sel_for_each<RESCAN>(sh, src, seg_of, desc, 1u, [&](bool valid, uint32_t key, uint32_t idx, bool pair) {
            const bool take = valid && key <= t0;
            const uint32_t pos = sel_append_pos(take, &sh.cnt);
            if (take && pos < SEL_CAP) sh.pool[pos] = ((uint64_t)key << 32) | sel_id(src, idx, pair);
        });
        __syncthreads();
        const uint32_t c = sh.cnt;
        if (c >= k && c <= SEL_CAP) {
            res = sel_pool_topk(sh, c, k);
            done = true;
        }
    }
    __syncthreads();
    if (!done) {
        // ---- exact radix select, then sort the k survivors
        sel_radix<RESCAN>(sh, src, seg_of, k, desc);
        res = sel_pool_topk(sh, k, k);
    }
    return res;
}

// ------------------------------------------------------------------------------------------------
// Coarse selection: probe list of each newly admitted query = the nprobe best centroids, best
// first, ties -> smaller centroid number.  Rows of up to CSEL_PER * 256 scores take a one-pass path
// (the row sits in registers while the bucket cut is made); longer rows, and rows in which the cut
// fails to isolate a small set (masses of equal scores), go through the general selection.
#define CSEL_PER 64        // scores per thread the fast path holds in registers: rows of up to 16384 centroids

// Row `r` of group g by the whole workgroup, any shape (all threads; every return is taken by all of them).
__device__ void coarse_select_row(SelShared &sh, const float *__restrict__ scores, const uint8_t *__restrict__ upload,
                                  const TriStepHdr *hdr, const TriCoarseGroup &g, uint32_t r,
                                  const TriIndexDev *__restrict__ indexes, uint32_t *__restrict__ probe, uint32_t nprobe_max)
{
    const uint32_t nlist = indexes[g.index].nlist, ldc = tri_coarse_ldc(nlist);
    const TriNewDesc d = ((const TriNewDesc *)(upload + hdr->desc_off))[g.first_new + r];
    const float *row = scores + (size_t)r * ldc;
    uint32_t *dst = probe + (size_t)d.slot * nprobe_max;
    const uint32_t tid = threadIdx.x;
    if (nlist <= CSEL_PER * TRI_SEL_THREADS && d.nprobe < nlist) {
        // ---- fast path: the whole row is read once, into registers, and cut by buckets from there
        // (loads through a descriptor that ends with the row: all 64 are in flight together, no branches)
        const __amdgpu_buffer_rsrc_t rrs = __builtin_amdgcn_make_buffer_rsrc((void *)row, 0, nlist * 4u, 0x00020000);
        uint32_t key[CSEL_PER];
#pragma unroll
        for (int u = 0; u < CSEL_PER; ++u)
            key[u] = __builtin_amdgcn_raw_buffer_load_b32(rrs, (u * TRI_SEL_THREADS + tid) * 4u, 0, 0);
#pragma unroll
        for (int u = 0; u < CSEL_PER; ++u)                         // (all-ones: padding, ignored below)
            key[u] = u * TRI_SEL_THREADS + tid < nlist ? sel_key(__uint_as_float(key[u]), d.metric) : 0xFFFFFFFFu;
        if (tid == 0) sh.cnt = 0;
        if (d.nprobe <= TRI_SEL_THREADS) {
            // A bound without a histogram: every thread's best key is one of 256 distinct elements, so the
            // nprobe-th smallest of those 256 is not better than the nprobe-th best of the whole row.  With 64
            // keys per thread it admits nprobe and a few dozen more; those are compacted and sorted exactly.
            uint32_t best = 0xFFFFFFFFu;
#pragma unroll
            for (int u = 0; u < CSEL_PER; ++u) best = key[u] < best ? key[u] : best;
            uint32_t *mins = (uint32_t *)sh.pool;
            mins[tid] = best;
            __syncthreads();
            // (the nprobe-th smallest VALUE is the largest one with fewer than nprobe strictly smaller ones:
            // one comparison per pair, no tie-break needed)
            if (tid == 0) sh.tmax = 0u;
            uint32_t below = 0;
            for (uint32_t j = 0; j < TRI_SEL_THREADS; j += 4) {
                const uint4 y = *(const uint4 *)(mins + j);
                below += (y.x < best) + (y.y < best) + (y.z < best) + (y.w < best);
            }
            __syncthreads();                                          // (the bound starts at zero)
            if (below < d.nprobe) atomicMax(&sh.tmax, best);
            __syncthreads();
            const uint32_t bound = sh.tmax;
            __syncthreads();                                          // (mins is read: the pool may be written)
            if (bound != 0xFFFFFFFFu) {
                uint32_t mine = 0;
#pragma unroll
                for (int u = 0; u < CSEL_PER; ++u) mine += key[u] <= bound;
                const uint32_t c_le = sel_block_scan_incl(mine, sh.wave_tot);
                if (tid == TRI_SEL_THREADS - 1) sh.count = c_le;
                __syncthreads();
                const uint32_t total = sh.count;
                if (total <= SEL_SMALL) {
                    uint32_t pos = c_le - mine;                       // (this thread's place among the admitted)
#pragma unroll
                    for (int u = 0; u < CSEL_PER; ++u)
                        if (key[u] <= bound) sh.small[pos++] = ((uint64_t)key[u] << 32) | (uint32_t)(u * TRI_SEL_THREADS + tid);
                    __syncthreads();
                    const uint64_t *best_of;
                    if (total <= SEL_RANK_MAX) {
                        sel_rank_sort(sh.small, total, sh.pool);
                        best_of = sh.pool;
                    } else {
                        sel_bitonic(sh.small, total);
                        best_of = sh.small;
                    }
                    for (uint32_t i = tid; i < d.nprobe; i += TRI_SEL_THREADS) dst[i] = (uint32_t)(best_of[i] & 0xFFFFFFFFu);
                    return;                                           // (uniform: total comes from shared memory)
                }
            }
            __syncthreads();
        }
        uint32_t kmin, lo = 0xFFFFFFFFu, hi = 0u;
#pragma unroll
        for (int u = 0; u < CSEL_PER; ++u)
            if (key[u] != 0xFFFFFFFFu) {
                lo = key[u] < lo ? key[u] : lo;
                hi = key[u] > hi ? key[u] : hi;
            }
        const float scale = sel_range(sh, lo, hi, kmin);
#pragma unroll
        for (int u = 0; u < CSEL_PER; ++u)
            if (u * TRI_SEL_THREADS + tid < nlist) atomicAdd(&sh.hist[sel_bucket(key[u], kmin, scale)], 1u);
        __syncthreads();
        sel_find_digit(sh, SEL_BINS, d.nprobe);
        const uint32_t B = sh.digit;
        const uint32_t c_le = d.nprobe - sh.need + sh.count;     // centroids in buckets <= B
        __syncthreads();                                          // the histogram is dead: sh.small reuses it
        if (c_le <= SEL_SMALL) {
#pragma unroll
            for (int u = 0; u < CSEL_PER; ++u) {
                const uint32_t e = u * TRI_SEL_THREADS + tid;
                const bool take = e < nlist && sel_bucket(key[u], kmin, scale) <= B;
                const uint32_t pos = sel_append_pos(take, &sh.cnt);
                if (take) sh.small[pos] = ((uint64_t)key[u] << 32) | e;
            }
            __syncthreads();
            const uint64_t *best;
            if (c_le <= SEL_RANK_MAX) {
                sel_rank_sort(sh.small, c_le, sh.pool);
                best = sh.pool;
            } else {
                sel_bitonic(sh.small, c_le);
                best = sh.small;
            }
            for (uint32_t i = tid; i < d.nprobe; i += TRI_SEL_THREADS) dst[i] = (uint32_t)(best[i] & 0xFFFFFFFFu);
            return;                                               // (uniform: c_le comes from shared memory)
        }
    }
    const SelSrc src = {nullptr, nullptr, row, nullptr, 0u, nlist, nullptr};
    auto seg_of = [&](uint32_t) { return SelSeg{0u, 0u, 0u, 0u}; };
    uint32_t n;
    const uint64_t *best = sel_block_topk<false>(sh, src, seg_of, d.nprobe, d.metric, &n);
    for (uint32_t i = tid; i < n; i += TRI_SEL_THREADS) dst[i] = (uint32_t)(best[i] & 0xFFFFFFFFu);
}

// ------------------------------------------------------------------------------------------------
// Threshold of each running slot for this step's scan: a bound for the k-th best key among the slot's
// sample scores (the first TRI_SAMPLE_VECS vectors of up to TRI_THRESH_ITEMS of its lists) and its
// running top-k -- a subset of its candidates, so nothing of its final top-k lies beyond it.  Fewer
// than k such keys: no filtering (all-ones).
//
// ONE WAVEFRONT PER SLOT, four slots per workgroup, no workgroup barriers: the keys sit in registers (lane l
// holds sample l of every item, and every 64th entry of the running top-k), the histogram of the bucket cut is
// the wavefront's own 8 KB of LDS, and whatever the lanes have to agree on goes through cross-lane operations.
// A wavefront's LDS operations execute in program order, so its histogram needs no more than compiler fences.
#define THR_TOPK_PER 4        // entries of the running top-k per lane in registers (256); a longer one: the slow cut

__device__ __forceinline__ void thr_wave_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Inclusive scan of one value per lane across the wavefront with data-parallel-primitive moves instead of trips
// through the LDS crossbar: four shifts inside each row of 16 lanes (a lane that has no source keeps `ident`), then
// lane 15 of rows 0 and 2 is broadcast into rows 1 and 3, then lane 31 into rows 2 and 3.  op(a, ident) == a.
__device__ __forceinline__ uint32_t thr_bits(uint32_t x) { return x; }
__device__ __forceinline__ uint32_t thr_bits(float x) { return __float_as_uint(x); }
__device__ __forceinline__ void thr_unbits(uint32_t b, uint32_t &x) { x = b; }
__device__ __forceinline__ void thr_unbits(uint32_t b, float &x) { x = __uint_as_float(b); }

template <int CTRL, int ROW_MASK, class T>
__device__ __forceinline__ T thr_dpp(T v, T ident)
{
    T r;
    thr_unbits((uint32_t)__builtin_amdgcn_update_dpp((int)thr_bits(ident), (int)thr_bits(v), CTRL, ROW_MASK, 0xF, false), r);
    return r;
}

template <class T, class Op>
__device__ __forceinline__ T thr_wave_scan(T v, T ident, Op op)
{
    v = op(v, thr_dpp<0x111, 0xF>(v, ident));      // row_shr:1
    v = op(v, thr_dpp<0x112, 0xF>(v, ident));      // row_shr:2
    v = op(v, thr_dpp<0x114, 0xF>(v, ident));      // row_shr:4
    v = op(v, thr_dpp<0x118, 0xF>(v, ident));      // row_shr:8
    v = op(v, thr_dpp<0x142, 0xA>(v, ident));      // row_bcast:15 into rows 1 and 3
    v = op(v, thr_dpp<0x143, 0xC>(v, ident));      // row_bcast:31 into rows 2 and 3
    return v;
}

template <class T, class Op>
__device__ __forceinline__ T thr_wave_reduce(T v, T ident, Op op)
{
    T r;
    thr_unbits((uint32_t)__builtin_amdgcn_readlane((int)thr_bits(thr_wave_scan(v, ident, op)), 63), r);
    return r;
}

template <uint32_t BINS = SEL_BINS>
__device__ __forceinline__ void thr_hist_zero(uint32_t *hist, uint32_t lane)
{
#pragma unroll
    for (uint32_t i = 0; i < BINS / 256; ++i) ((uint4 *)hist)[i * 64 + lane] = make_uint4(0u, 0u, 0u, 0u);
    thr_wave_fence();
}

// Smallest bucket B of the wavefront's histogram whose cumulative count reaches need (256 bins a round, four
// consecutive ones per lane, a prefix sum across the lanes).  in_bucket = hist[B], need_in = need - (count below B).
template <uint32_t BINS = SEL_BINS>
__device__ __forceinline__ void thr_hist_find(const uint32_t *hist, uint32_t need, uint32_t lane, uint32_t &B,
                                              uint32_t &in_bucket, uint32_t &need_in)
{
    thr_wave_fence();
    B = BINS - 1;
    in_bucket = 0;
    need_in = need;
    uint32_t run = 0;
    for (uint32_t j = 0; j < BINS / 256; ++j) {
        const uint4 h = ((const uint4 *)hist)[j * 64 + lane];
        const uint32_t mine = h.x + h.y + h.z + h.w;
        const uint32_t incl = thr_wave_scan(mine, 0u, [](uint32_t a, uint32_t b) { return a + b; });
        const uint32_t excl = run + incl - mine;
        const bool here = excl < need && need <= excl + mine;
        const uint64_t who = __ballot(here);
        if (who) {
            uint32_t b = 0, cnt = 0, left = 0;
            if (here) {
                const uint32_t hh[4] = {h.x, h.y, h.z, h.w};
                uint32_t r2 = excl;
                bool found = false;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    if (!found && r2 + hh[c] >= need) {
                        b = j * 256 + lane * 4 + c;
                        cnt = hh[c];
                        left = need - r2;
                        found = true;
                    }
                    r2 += hh[c];
                }
            }
            const int src = __ffsll((unsigned long long)who) - 1;
            B = (uint32_t)__builtin_amdgcn_readlane((int)b, src);
            in_bucket = (uint32_t)__builtin_amdgcn_readlane((int)cnt, src);
            need_in = (uint32_t)__builtin_amdgcn_readlane((int)left, src);
            return;
        }
        run += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    }
}

// The values a wavefront selects from: val = the score where smaller is better, its negative where larger is
// (so smaller is always better); +infinity = absent.  tri_score_key(val, 0) is the key of the score.
struct ThrVals {
    float item[TRI_THRESH_ITEMS];     // lane l: sample l of item s
    float topk[THR_TOPK_PER];         // lane l: entry 64 s + l of the running top-k
};

template <class Fn>
__device__ __forceinline__ void thr_for_each(const ThrVals &v, Fn f)
{
#pragma unroll
    for (int s = 0; s < TRI_THRESH_ITEMS; ++s) f(v.item[s]);
#pragma unroll
    for (int s = 0; s < THR_TOPK_PER; ++s) f(v.topk[s]);
}

// Exact-to-the-key cut, for the cases the one-pass cut below does not settle: a key T with at least m of the
// wavefront's keys not above it and few more.  Buckets linear in the key, the bucket of rank m cut again (each level
// narrows the key range 2048-fold) until it holds at most a few keys beyond rank m or equal keys only.  Rare;
// for_each_key(f) reads the keys again from memory (all-ones for absent ones), f(key) called by all lanes together,
// so that it needs none of the registers of the common path.
template <class ForEachKey>
__device__ __forceinline__ uint32_t thr_wave_refine(ForEachKey for_each_key, uint32_t m, uint32_t *hist, uint32_t lane)
{
    uint32_t range_lo = 0u, range_hi = 0xFFFFFFFEu;
    uint32_t need = m, t = 0xFFFFFFFEu;
    for (int level = 0; level < 4; ++level) {
        uint32_t lo = 0xFFFFFFFFu, hi = 0u;
        for_each_key([&](uint32_t k) {
            if (k >= range_lo && k <= range_hi) {
                lo = k < lo ? k : lo;
                hi = k > hi ? k : hi;
            }
        });
        const uint32_t kmin = thr_wave_reduce(lo, 0xFFFFFFFFu, [](uint32_t a, uint32_t b) { return a < b ? a : b; });
        const uint32_t kmax = thr_wave_reduce(hi, 0u, [](uint32_t a, uint32_t b) { return a > b ? a : b; });
        const float scale = kmax > kmin ? ((float)SEL_BINS - 0.01f) / (float)(kmax - kmin) : 0.f;
        thr_hist_zero(hist, lane);
        for_each_key([&](uint32_t k) {
            if (k >= range_lo && k <= range_hi) atomicAdd(&hist[sel_bucket(k, kmin, scale)], 1u);
        });
        uint32_t B, in_bucket, need_in;
        thr_hist_find(hist, need, lane, B, in_bucket, need_in);
        uint32_t best = 0u, least = 0xFFFFFFFFu;
        for_each_key([&](uint32_t k) {
            if (k >= range_lo && k <= range_hi && sel_bucket(k, kmin, scale) == B) {
                best = k > best ? k : best;
                least = k < least ? k : least;
            }
        });
        t = thr_wave_reduce(best, 0u, [](uint32_t a, uint32_t b) { return a > b ? a : b; });
        const uint32_t t_lo = thr_wave_reduce(least, 0xFFFFFFFFu, [](uint32_t a, uint32_t b) { return a < b ? a : b; });
        if (in_bucket <= need_in + 4u || t_lo == t) break;
        range_lo = t_lo;
        range_hi = t;
        need = need_in;
    }
    return t;
}

// A value E with at least m of the wavefront's values not above it, and few more (at least m values are present;
// for_each(f) calls f(x) for every value the wavefront holds in registers, +infinity = absent).
// One pass: buckets linear in the VALUE between the smallest and the largest one (keys are bit patterns of floats:
// linear in the key, the best scores of a set that straddles zero crowd into a handful of buckets), E = the upper
// edge of the bucket that holds rank m.  The edge is computed in floating point, so the count of values not above
// it is checked; false for a crowded bucket (more than `slack` values beyond rank m) or a failed check.
template <uint32_t BINS = SEL_BINS, class ForEach>
__device__ __forceinline__ bool sel_wave_cut(ForEach for_each, uint32_t m, uint32_t slack, uint32_t *hist, uint32_t lane,
                                             float &edge)
{
    float lo = INFINITY, hi = -INFINITY;
    for_each([&](float x) {
        if (x < INFINITY) {
            lo = fminf(lo, x);
            hi = fmaxf(hi, x);
        }
    });
    lo = thr_wave_reduce(lo, INFINITY, [](float a, float b) { return fminf(a, b); });
    hi = thr_wave_reduce(hi, -INFINITY, [](float a, float b) { return fmaxf(a, b); });
    const float span = hi - lo;
    if (!(span > 0.f && span < 3.0e38f)) return false;
    const float scale = ((float)BINS - 0.01f) / span;
    thr_hist_zero<BINS>(hist, lane);
    for_each([&](float x) {
        if (x < INFINITY) atomicAdd(&hist[(uint32_t)fminf((x - lo) * scale, (float)(BINS - 1))], 1u);
    });
    uint32_t B, in_bucket, need_in;
    thr_hist_find<BINS>(hist, m, lane, B, in_bucket, need_in);
    if (in_bucket > need_in + slack) return false;
    edge = B >= BINS - 1 ? hi : fminf(lo + (float)(B + 1) / scale, hi);
    uint32_t c = 0;
    for_each([&](float x) { c += x <= edge; });
    c = thr_wave_reduce(c, 0u, [](uint32_t a, uint32_t b) { return a + b; });
    return c >= m;
}

__global__ __launch_bounds__(TRI_SEL_THREADS) __attribute__((amdgpu_waves_per_eu(4, 4))) void slot_threshold_kernel(
    const uint8_t *__restrict__ upload, const TriSlotMeta *__restrict__ slot_meta,
    const uint32_t *__restrict__ item_glist, const uint32_t *__restrict__ item_sorted_pos,
    const uint32_t *__restrict__ glist_len, const uint32_t *__restrict__ glist_voff,
    const float *__restrict__ sample_scores, const float *__restrict__ topk_score,
    const uint32_t *__restrict__ topk_count, uint32_t kmax, uint32_t *__restrict__ thr_key, uint2 *__restrict__ cand,
    uint32_t *__restrict__ slot_cand_off, uint32_t *__restrict__ slot_cand_cap, uint32_t *__restrict__ slot_cand_cnt)
{
    static_assert(TRI_SAMPLE_VECS == 64 && TRI_THRESH_ITEMS == 64, "lane l holds sample l of item s in register s");
    __shared__ __attribute__((aligned(16))) uint32_t hist_all[TRI_SEL_THREADS / 64][SEL_BINS];
    __shared__ uint32_t item_all[TRI_SEL_THREADS / 64][3][TRI_THRESH_ITEMS];
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t *hist = hist_all[wave], *voffs = item_all[wave][0], *rows = item_all[wave][1], *lens = item_all[wave][2];
    const TriStepHdr *hdr = (const TriStepHdr *)upload;
    const uint32_t pe = blockIdx.x * (TRI_SEL_THREADS / 64) + wave;
    if (pe >= hdr->n_plan) return;                           // (per wavefront; the kernel has no workgroup barrier)
    const TriPlanEntry e = ((const TriPlanEntry *)(upload + hdr->plan_off))[pe];
    const TriSlotMeta meta = slot_meta[e.slot];
    const bool desc = meta.metric == 1u;
    const uint32_t have = e.cursor > 0 ? min(topk_count[e.slot], (uint32_t)TRI_KMAX_POW2) : 0u;
    const uint32_t nitems = e.take < TRI_THRESH_ITEMS ? e.take : TRI_THRESH_ITEMS;
    // lane s: sample row and sample count of item s; first stored position of its list -> LDS
    uint32_t it_row = 0, it_len = 0;
    if (lane < nitems) {
        const uint32_t it = e.item_base + lane, g = item_glist[it];
        it_row = item_sorted_pos[it];
        it_len = min(glist_len[g], (uint32_t)TRI_SAMPLE_VECS);
        voffs[lane] = glist_voff[g];
        rows[lane] = it_row;
        lens[lane] = it_len;
    }
    // All loads first (every address valid: absent items read item 0's row, and a row always has TRI_SAMPLE_VECS
    // entries); what is absent -- a list shorter than the sample, fewer items, a shorter running top-k -- then
    // becomes +infinity.  Row starts travel as scalar offsets of a buffer load, so no address is kept per item.
    const __amdgpu_buffer_rsrc_t srs = __builtin_amdgcn_make_buffer_rsrc((void *)sample_scores, 0, 0xFFFFFFFFu, 0x00020000);
    const float pad = desc ? -INFINITY : INFINITY;           // (before the sign is settled)
    ThrVals v;
#pragma unroll
    for (int s = 0; s < TRI_THRESH_ITEMS; ++s) {
        const uint32_t row = __builtin_amdgcn_readlane(it_row, s);
        v.item[s] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(srs, lane * 4u, row * (TRI_SAMPLE_VECS * 4u), 0));
    }
#pragma unroll
    for (int s = 0; s < THR_TOPK_PER; ++s) {
        const uint32_t i = s * 64 + lane;
        v.topk[s] = i < have ? topk_score[(size_t)e.slot * kmax + i] : pad;
    }
    uint64_t there = 0;                                      // bit s: this lane's sample of item s exists
#pragma unroll
    for (int s = 0; s < TRI_THRESH_ITEMS; ++s)
        there |= (uint64_t)(lane < __builtin_amdgcn_readlane(it_len, s) ? 1u : 0u) << s;
    uint32_t present = 0;
#pragma unroll
    for (int s = 0; s < TRI_THRESH_ITEMS; ++s) v.item[s] = (there >> s) & 1u ? (desc ? -v.item[s] : v.item[s]) : INFINITY;
#pragma unroll
    for (int s = 0; s < THR_TOPK_PER; ++s) v.topk[s] = desc ? -v.topk[s] : v.topk[s];
#pragma unroll
    for (int s = 0; s < TRI_THRESH_ITEMS; ++s) present += v.item[s] < INFINITY;
    present = thr_wave_reduce(present, 0u, [](uint32_t a, uint32_t b) { return a + b; }) + have;
    uint32_t thr = 0xFFFFFFFFu;
    // (beyond rank k the cut may admit a few keys, or an eighth of k: that many more candidates pass the scan's filter)
    float cut = 0.f;
    const bool enough = present >= meta.k;
    const bool settled = enough && have <= 64u * THR_TOPK_PER &&
                         sel_wave_cut([&](auto f) { thr_for_each(v, f); }, meta.k, max(8u, meta.k >> 3), hist, lane, cut);
    // The sample IS the first block(s) of every list: its scores that pass the threshold become the first
    // candidates of the query's region here, and the scan starts every list behind them.  (score bits, stored
    // position) pairs; the main launch counts on from what this leaves in the slot's counter.
    uint32_t count = 0;
    auto emit = [&](bool pass, float val, uint32_t pos0) {
        const uint64_t m = __ballot(pass);
        const uint32_t pos = count + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
        const float score = desc ? -val : val;
        if (pass && pos < e.cand_cap)
            cand[(size_t)e.cand_off + pos] = make_uint2(score == 0.f ? 0u : __float_as_uint(score), pos0 + lane);
        count += (uint32_t)__popcll(m);
    };
    thr_wave_fence();                                        // (voffs, rows, lens)
    uint32_t from_memory = 0;                                // first item whose samples are read again below
    if (settled) {
        thr = tri_score_key(cut, 0u);
        const float edge = tri_key_score(thr, 0u);           // (value <= edge: its key is not above thr)
#pragma unroll
        for (int s = 0; s < TRI_THRESH_ITEMS; ++s)
            if (__ballot(v.item[s] <= edge)) emit(v.item[s] <= edge, v.item[s], voffs[s]);    // (uniform; most rows pass nothing)
        from_memory = TRI_THRESH_ITEMS;
    } else if (enough) {
        thr = thr_wave_refine([&](auto f) {
            for (uint32_t s = 0; s < nitems; ++s) {
                float x = lane < lens[s] ? sample_scores[(size_t)rows[s] * TRI_SAMPLE_VECS + lane] : pad;
                x = desc ? -x : x;
                f(x < INFINITY ? tri_score_key(x, 0u) : 0xFFFFFFFFu);
            }
            for (uint32_t i0 = 0; i0 < have; i0 += 64) {
                float x = i0 + lane < have ? topk_score[(size_t)e.slot * kmax + i0 + lane] : pad;
                x = desc ? -x : x;
                f(x < INFINITY ? tri_score_key(x, 0u) : 0xFFFFFFFFu);
            }
        }, meta.k, hist, lane);
    }
    // From memory: items beyond those the threshold was made of; every item where the one-pass cut did not settle the
    // threshold (the registers of the common path are not kept for that), or where there is none (the value that
    // stands for "absent" cannot tell an absent sample from a score of infinity, the lists' lengths can).
    {
        const bool all = thr == 0xFFFFFFFFu;
        const float edge = tri_key_score(thr, 0u);
        // (64 items a round: every lane fetches what describes one of them, then the items' sample rows are read four at
        // a time -- one dependent load per item instead of three, and four of those in flight)
        for (uint32_t s0 = from_memory; s0 < e.take; s0 += 64) {
            const bool mine = s0 + lane < e.take;
            const uint32_t it = e.item_base + s0 + lane, g = mine ? item_glist[it] : 0u;
            const uint32_t len_l = mine ? min(glist_len[g], (uint32_t)TRI_SAMPLE_VECS) : 0u;
            const uint32_t voff_l = mine ? glist_voff[g] : 0u, row_l = mine ? item_sorted_pos[it] : 0u;
            const uint32_t n = min(64u, e.take - s0);
            for (uint32_t j = 0; j < n; j += 4) {
                float val[4];
                uint32_t len4[4], voff4[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t jj = j + u < n ? j + u : n - 1;                     // (uniform)
                    len4[u] = (uint32_t)__builtin_amdgcn_readlane((int)len_l, (int)jj);
                    voff4[u] = (uint32_t)__builtin_amdgcn_readlane((int)voff_l, (int)jj);
                    const uint32_t row = (uint32_t)__builtin_amdgcn_readlane((int)row_l, (int)jj);
                    val[u] = lane < len4[u] ? sample_scores[(size_t)row * TRI_SAMPLE_VECS + lane] : pad;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (j + u >= n) break;                                              // (uniform)
                    const float x = desc ? -val[u] : val[u];
                    emit(lane < len4[u] && (all || x <= edge), x, voff4[u]);
                }
            }
        }
    }
    if (lane == 0) {
        thr_key[e.slot] = thr;
        slot_cand_off[e.slot] = e.cand_off;
        slot_cand_cap[e.slot] = e.cand_cap;
        slot_cand_cnt[e.slot] = count;
    }
}

hipError_t tri_launch_threshold(const TriLaunchCtx &c, const TriDevWs &ws, uint32_t grid_plan)
{
    if (grid_plan == 0) return hipSuccess;
    hipLaunchKernelGGL(slot_threshold_kernel, dim3((grid_plan + TRI_SEL_THREADS / 64 - 1) / (TRI_SEL_THREADS / 64)),
                       dim3(TRI_SEL_THREADS), 0, c.stream, ws.upload, ws.slot_meta,
                       ws.item_glist, ws.item_sorted_pos, ws.glist_len, ws.glist_voff, ws.sample_scores, ws.topk_score,
                       ws.topk_count, c.kmax, ws.thr_key, ws.cand, ws.slot_cand_off, ws.slot_cand_cap, ws.slot_cand_cnt);
    return hipGetLastError();
}

// Squared L2 distance of a stored vector (x: its first 16-byte piece; the pieces lie TRI_PIECE_PITCH apart) to a
// query row in the difference form, sum of (x_i - q_i)^2, by the 32
// lanes of a half-wavefront: lane l takes the 16-byte pieces l, l + 32, ... of both, the partial sums are
// combined by a butterfly (a fixed order, the same in every lane).  fp32 arithmetic; fp16 inputs widen exactly.
template <typename T>
__device__ __forceinline__ float sel_l2_diff_form(const uint8_t *__restrict__ x, const uint8_t *__restrict__ q, uint32_t row_bytes,
                                                  uint32_t l32)
{
    constexpr int PER = 16 / sizeof(T);
    float acc = 0.f;
    for (uint32_t o = l32 * 16; o < row_bytes; o += 32 * 16) {
        const uint4 xv = *(const uint4 *)(x + (size_t)o * (TRI_PIECE_PITCH / 16)), qv = *(const uint4 *)(q + o);
        const T *xe = (const T *)&xv, *qe = (const T *)&qv;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const float d = (float)xe[i] - (float)qe[i];
            acc = __builtin_fmaf(d, d, acc);
        }
    }
#pragma unroll
    for (int d = 16; d > 0; d >>= 1) acc += __shfl_xor(acc, d, 32);
    return acc;
}

// ------------------------------------------------------------------------------------------------
// Slot merge.  Candidates of a running slot = the (score, stored position) pairs the scan kept in the slot's
// region of the candidate buffer in this step + its running top-k.  Output = the new running top-k, or -- when
// the slot retires in this step -- its final result.
//
// Two kernels.  In the first every slot is tried by one wavefront on its own (merge_wave: candidates in
// registers, one-pass cut, survivors sorted by rank counting in the wavefront's LDS; no workgroup barrier).  Slots
// that do not settle there -- too many candidates or survivors, masses of equal scores, a candidate region that
// was too small -- are queued and taken by the second, one workgroup per slot with the general selection
// (merge_block).  Should a region have been too small (the slot's counter ran past its capacity), the pairs in it are
// ignored and the slot's lists of this step are scored again right here (SelRescan): slow, exact, and rare.
struct MergeArgs {
    const uint8_t *upload;
    const TriSlotMeta *slot_meta;
    const TriIndexDev *indexes;
    const uint32_t *item_glist, *slot_cand_cnt, *glist_len, *glist_voff;
    const uint2 *cand;
    float *topk_score;
    uint32_t *topk_id, *topk_count;
    uint32_t kmax;
    uint32_t *res_block;
    const uint32_t *probe;
    uint32_t nprobe_max;
    uint32_t *res_probes;
    const uint8_t *slot_query;
    uint32_t slot_row_bytes;
    const float *slot_qnorm;
    uint32_t *rescans;               // [0] counter of rescans, [1], [2] entries in merge_queue (one head per parity of the launch)
    uint32_t *merge_queue;
};

#define MRG_PER 24           // candidates per lane the wavefront path holds in registers (1536 per slot)
#define MRG_BINS 1024
#define MRG_TOPK_PER 4       // entries of the running top-k per lane (256)
#define MRG_CAP 256          // survivors it sorts

struct MergeWaveLds {
    uint32_t hist[MRG_BINS];
    uint64_t a[MRG_CAP], b[MRG_CAP];
};

// Sort c <= MRG_CAP composites by rank counting within one wavefront, src -> dst (LDS, distinct): a lane owns the
// elements lane, lane + 64, ... and counts, for each, the elements ordered before it (every lane reads the same
// element at a time, a broadcast; four reads are in flight together).
__device__ __forceinline__ void mrg_rank_sort(const uint64_t *src, uint32_t c, uint64_t *dst, uint32_t lane)
{
    thr_wave_fence();
    constexpr int OWN = MRG_CAP / 64;
    uint64_t x[OWN];
    uint32_t rank[OWN];
#pragma unroll
    for (int j = 0; j < OWN; ++j) {
        x[j] = j * 64 + lane < c ? src[j * 64 + lane] : ~0ull;
        rank[j] = 0;
    }
    const uint32_t own = (c + 63) / 64;                                 // (uniform)
    auto count = [&](uint64_t y, uint32_t u) {
#pragma unroll
        for (int j = 0; j < OWN; ++j)
            if ((uint32_t)j < own) rank[j] += (y < x[j] || (y == x[j] && u < j * 64 + lane)) ? 1u : 0u;
    };
    uint32_t u = 0;
    for (; u + 4 <= c; u += 4) {
        const uint64_t y0 = src[u], y1 = src[u + 1], y2 = src[u + 2], y3 = src[u + 3];
        count(y0, u);
        count(y1, u + 1);
        count(y2, u + 2);
        count(y3, u + 3);
    }
    for (; u < c; ++u) count(src[u], u);
    thr_wave_fence();
#pragma unroll
    for (int j = 0; j < OWN; ++j)
        if (j * 64 + lane < c) dst[rank[j]] = x[j];
    thr_wave_fence();
}

// Results of a slot: to the record of a retiring query (pinned host memory), else to its running top-k.
// best[0..n): sorted composites (LDS); called by `nthreads` threads with index `tid`.
__device__ __forceinline__ void mrg_write_out(const MergeArgs &A, const TriPlanEntry &e, const TriSlotMeta &meta, uint32_t desc,
                                              const uint64_t *best, uint32_t n, uint32_t tid, uint32_t nthreads)
{
    if (e.retire_idx >= 0) {
        uint32_t *rec = A.res_block + (size_t)e.retire_idx * (1u + 2u * A.kmax);
        if (tid == 0) rec[0] = n;
        for (uint32_t i = tid; i < n; i += nthreads) {
            const uint64_t c = best[i];
            rec[1 + i] = (uint32_t)(c & 0xFFFFFFFFu);
            rec[1 + A.kmax + i] = __float_as_uint(sel_unkey((uint32_t)(c >> 32), desc));
        }
        if (A.res_probes) {
            const uint32_t *srcp = A.probe + (size_t)e.slot * A.nprobe_max;
            uint32_t *dst = A.res_probes + (size_t)e.retire_idx * A.nprobe_max;
            for (uint32_t i = tid; i < meta.nprobe; i += nthreads) dst[i] = srcp[i];
        }
    } else {
        float *run_score = A.topk_score + (size_t)e.slot * A.kmax;
        uint32_t *run_id = A.topk_id + (size_t)e.slot * A.kmax;
        for (uint32_t i = tid; i < n; i += nthreads) {
            const uint64_t c = best[i];
            run_id[i] = (uint32_t)(c & 0xFFFFFFFFu);
            run_score[i] = sel_unkey((uint32_t)(c >> 32), desc);
        }
        if (tid == 0) A.topk_count[e.slot] = n;
    }
}

// The k best of a slot's candidates, by one wavefront: for_each(f) calls f(value, payload, is_pair) for every
// candidate (value: smaller is better, +infinity = absent; payload: stored position of a pair, id of a running
// entry; all pairs before the running entries), all lanes together.  Leaves the c survivors of the cut in L.a as
// (key, id) composites -- those of the pairs first, from_pairs of them, with the stored position in the id's place.
// false: not settled.
template <class ForEach>
__device__ __forceinline__ bool mrg_wave_select(ForEach for_each, uint32_t total, uint32_t k, bool desc, MergeWaveLds &L,
                                                uint32_t lane, uint32_t &c, uint32_t &from_pairs)
{
    uint32_t present = 0;
    for_each([&](float x, uint32_t, bool) { present += x < INFINITY; });
    present = thr_wave_reduce(present, 0u, [](uint32_t a, uint32_t b) { return a + b; });
    if (present != total) return false;                                       // (scores that are infinite or not numbers)
    float edge = INFINITY;
    if (total > k &&
        !sel_wave_cut<MRG_BINS>([&](auto f) { for_each([&](float x, uint32_t, bool) { f(x); }); }, k, MRG_CAP - k, L.hist, lane, edge))
        return false;
    uint32_t cnt = 0, pairs = 0;
    for_each([&](float x, uint32_t payload, bool is_pair) {
        const bool pass = x <= edge && x < INFINITY;
        const uint64_t m = __ballot(pass);
        if (m == 0) return;                                                 // (uniform)
        const uint32_t at = cnt + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
        if (pass && at < MRG_CAP) L.a[at] = ((uint64_t)sel_key(desc ? -x : x, desc) << 32) | payload;
        cnt += (uint32_t)__popcll(m);
        if (is_pair) pairs = cnt;
    });
    c = cnt;
    from_pairs = pairs;
    return c <= MRG_CAP;
}

// One slot by one wavefront.  false: not settled, nothing written.
__device__ __forceinline__ bool merge_wave(const MergeArgs &A, const TriPlanEntry &e, MergeWaveLds &L, uint32_t lane)
{
    const TriSlotMeta meta = A.slot_meta[e.slot];
    const bool desc = meta.metric == 1u;
    const uint32_t k = meta.k;
    const uint32_t asked = A.slot_cand_cnt[e.slot];
    const uint32_t have = e.cursor > 0 ? A.topk_count[e.slot] : 0u;
    if (asked > e.cand_cap || k > MRG_CAP) return false;
    const TriIndexDev &ix = A.indexes[meta.index];
    const float *run_score = A.topk_score + (size_t)e.slot * A.kmax;
    const uint32_t *run_id = A.topk_id + (size_t)e.slot * A.kmax;
    const uint2 *mine = A.cand + e.cand_off;
    uint32_t c = 0, from_pairs = 0;
    bool settled;
    if (asked <= 64u * MRG_PER && have <= 64u * MRG_TOPK_PER) {
        // the usual size: everything in registers, read once (all loads are issued before the first value is
        // looked at: one round trip to memory, not one per 64 pairs)
        float val[MRG_PER], rv[MRG_TOPK_PER];
        uint32_t pos[MRG_PER], rid[MRG_TOPK_PER];
        uint2 raw[MRG_PER];
#pragma unroll
        for (int j = 0; j < MRG_PER; ++j) {
            raw[j] = make_uint2(0u, 0u);
            if ((uint32_t)j * 64 < asked) raw[j] = mine[j * 64 + lane < asked ? j * 64 + lane : 0u];    // (uniform)
        }
#pragma unroll
        for (int j = 0; j < MRG_TOPK_PER; ++j) {
            const uint32_t i = j * 64 + lane;
            rv[j] = i < have ? run_score[i] : 0.f;
            rid[j] = i < have ? run_id[i] : 0u;
        }
#pragma unroll
        for (int j = 0; j < MRG_PER; ++j) {
            const float sc = __uint_as_float(raw[j].x);
            val[j] = (uint32_t)j * 64 + lane < asked ? (desc ? -sc : sc) : INFINITY;
            pos[j] = raw[j].y;
        }
#pragma unroll
        for (int j = 0; j < MRG_TOPK_PER; ++j) rv[j] = (uint32_t)j * 64 + lane < have ? (desc ? -rv[j] : rv[j]) : INFINITY;
        settled = mrg_wave_select([&](auto f) {
#pragma unroll
            for (int j = 0; j < MRG_PER; ++j) f(val[j], pos[j], true);
#pragma unroll
            for (int j = 0; j < MRG_TOPK_PER; ++j) f(rv[j], rid[j], false);
        }, asked + have, k, desc, L, lane, c, from_pairs);
    } else {
        // more than the registers hold: every pass reads the candidates again, eight loads per lane in flight
        settled = mrg_wave_select([&](auto f) {
            constexpr int U = 8;
            for (uint32_t i0 = 0; i0 < asked; i0 += 64 * U) {
                uint2 raw[U];
#pragma unroll
                for (int u = 0; u < U; ++u) raw[u] = mine[i0 + u * 64 + lane < asked ? i0 + u * 64 + lane : 0u];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const float sc = __uint_as_float(raw[u].x);
                    f(i0 + u * 64 + lane < asked ? (desc ? -sc : sc) : INFINITY, raw[u].y, true);
                }
            }
            for (uint32_t i0 = 0; i0 < have; i0 += 64) {
                const float sc = i0 + lane < have ? run_score[i0 + lane] : 0.f;
                f(i0 + lane < have ? (desc ? -sc : sc) : INFINITY, i0 + lane < have ? run_id[i0 + lane] : 0u, false);
            }
        }, asked + have, k, desc, L, lane, c, from_pairs);
    }
    if (!settled) return false;
    // the ids of the survivors that came from pairs are fetched together (one round trip to memory for all of them)
    thr_wave_fence();
    {
        uint64_t x[MRG_CAP / 64];
#pragma unroll
        for (int j = 0; j < MRG_CAP / 64; ++j) x[j] = j * 64 + lane < from_pairs ? L.a[j * 64 + lane] : 0ull;
        uint32_t id[MRG_CAP / 64];
#pragma unroll
        for (int j = 0; j < MRG_CAP / 64; ++j) id[j] = j * 64 + lane < from_pairs ? ix.ids[(uint32_t)(x[j] & 0xFFFFFFFFu)] : 0u;
#pragma unroll
        for (int j = 0; j < MRG_CAP / 64; ++j)
            if (j * 64 + lane < from_pairs) L.a[j * 64 + lane] = (x[j] & 0xFFFFFFFF00000000ull) | id[j];
    }
    mrg_rank_sort(L.a, c, L.b, lane);
    uint32_t n = c < k ? c : k;
    const uint64_t *best = L.b;
    if (e.retire_idx >= 0 && !desc && n > 0) {
        // squared L2 handed back in the difference form (see merge_block): the n survivors are scored again, one row
        // per half-wavefront at a time, and put in the order of those scores
        const uint8_t *qrow = A.slot_query + (size_t)e.slot * A.slot_row_bytes;
        const uint32_t l32 = lane & 31;
        uint32_t *stored = L.hist;                                              // (where each survivor's row is: fetched together; n <= MRG_CAP <= MRG_BINS)
        for (uint32_t i = lane; i < n; i += 64) stored[i] = ix.inv[(uint32_t)(L.b[i] & 0xFFFFFFFFu)];
        thr_wave_fence();
        for (uint32_t i = lane >> 5; i < n; i += 2) {
            const uint32_t id = (uint32_t)(L.b[i] & 0xFFFFFFFFu);
            const uint8_t *x = tri_slot_ptr(ix, stored[i]);
            const float d2 = ix.dtype == 1u ? sel_l2_diff_form<_Float16>(x, qrow, ix.row_bytes, l32)
                                            : sel_l2_diff_form<float>(x, qrow, ix.row_bytes, l32);
            if (l32 == 0) L.a[i] = ((uint64_t)sel_key(d2, 0u) << 32) | id;
        }
        mrg_rank_sort(L.a, n, L.b, lane);
    }
    mrg_write_out(A, e, meta, desc ? 1u : 0u, best, n, lane, 64u);
    return true;
}

// One slot by the whole workgroup, any size.
__device__ void merge_block(const MergeArgs &A, const TriPlanEntry &e, SelShared &sh)
{
    const TriSlotMeta meta = A.slot_meta[e.slot];
    const uint32_t desc = meta.metric == 1u;
    const uint32_t have = e.cursor > 0 ? A.topk_count[e.slot] : 0u;
    float *run_score = A.topk_score + (size_t)e.slot * A.kmax;
    uint32_t *run_id = A.topk_id + (size_t)e.slot * A.kmax;
    const uint32_t asked = A.slot_cand_cnt[e.slot];
    const bool overflow = asked > e.cand_cap;                 // (the same for every thread of the workgroup)
    SelRescan rs = {A.item_glist, A.glist_len, A.glist_voff, &A.indexes[meta.index],
                    A.slot_query + (size_t)e.slot * A.slot_row_bytes, A.slot_qnorm[e.slot], meta.metric == 0u, e.item_base,
                    e.take, 0u};
    if (overflow) {
        uint32_t part = 0;
        for (uint32_t it = threadIdx.x; it < e.take; it += TRI_SEL_THREADS) part += A.glist_len[A.item_glist[e.item_base + it]];
        const uint32_t incl = sel_block_scan_incl(part, sh.wave_tot);
        if (threadIdx.x == TRI_SEL_THREADS - 1) {
            sh.tmax = incl;
            atomicAdd(A.rescans, 1u);
        }
        __syncthreads();
        rs.total = sh.tmax;
        __syncthreads();
    }
    const SelSrc src = {A.cand, A.indexes[meta.index].ids, run_score, run_id, overflow ? 0u : 1u, have, overflow ? &rs : nullptr};
    auto seg_of = [&](uint32_t) { return SelSeg{e.cand_off, asked, 0u, 0u}; };
    uint32_t n;
    const uint64_t *best = sel_block_topk<true>(sh, src, seg_of, meta.k, desc, &n);
    // (all reads of the running buffer are done: sel_block_topk ends with a barrier)
    if (e.retire_idx >= 0 && !desc && n > 0) {
        // The scan scores squared L2 in the expanded form |x|^2 + |q|^2 - 2 x.q, whose fp32 error grows with
        // the norms, not with the distance: fine for choosing the k best, too coarse for the distance that is
        // handed back when a query nearly coincides with a stored vector.  The k survivors of a retiring
        // query are scored again in the difference form (k rows re-read: nothing beside the scan) and put in
        // the order of those scores (equal scores by ascending id, as everywhere).
        const TriIndexDev &ix = A.indexes[meta.index];
        const uint8_t *qrow = A.slot_query + (size_t)e.slot * A.slot_row_bytes;
        uint64_t *fresh = best == sh.pool ? sh.small : sh.pool;             // (n <= kmax <= SEL_SMALL)
        const uint32_t l32 = threadIdx.x & 31;
        for (uint32_t i = threadIdx.x >> 5; i < n; i += TRI_SEL_THREADS / 32) {
            const uint32_t id = (uint32_t)(best[i] & 0xFFFFFFFFu);
            const uint8_t *x = tri_slot_ptr(ix, ix.inv[id]);
            const float d2 = ix.dtype == 1u ? sel_l2_diff_form<_Float16>(x, qrow, ix.row_bytes, l32)
                                            : sel_l2_diff_form<float>(x, qrow, ix.row_bytes, l32);
            if (l32 == 0) fresh[i] = ((uint64_t)sel_key(d2, 0u) << 32) | id;
        }
        __syncthreads();
        if (fresh != sh.pool) {
            for (uint32_t i = threadIdx.x; i < n; i += TRI_SEL_THREADS) sh.pool[i] = fresh[i];
            __syncthreads();
        }
        best = sel_pool_topk(sh, n, n);
    }
    mrg_write_out(A, e, meta, desc, best, n, threadIdx.x, TRI_SEL_THREADS);
    __syncthreads();                                          // (the workgroup's next slot reuses sh)
}

__global__ __launch_bounds__(TRI_SEL_THREADS) __attribute__((amdgpu_waves_per_eu(4, 4))) void slot_merge_wave_kernel(const MergeArgs A)
{
    constexpr uint32_t NW = TRI_SEL_THREADS / 64;
    __shared__ MergeWaveLds wv[NW];
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const TriStepHdr *hdr = (const TriStepHdr *)A.upload;
    const uint32_t pe = blockIdx.x * NW + wave;
    if (pe >= hdr->n_plan) return;                           // (per wavefront; the kernel has no workgroup barrier)
    const TriPlanEntry *plan = (const TriPlanEntry *)(A.upload + hdr->plan_off);
    if (!merge_wave(A, plan[pe], wv[wave], lane) && lane == 0) A.merge_queue[atomicAdd(A.rescans + 1 + hdr->merge_parity, 1u)] = pe;
}

// The slots the kernel above left, dealt out among a fixed number of workgroups.  There are two queue heads, used in
// turn by successive launches: this launch reads its own and clears the other one, for the next launch.
__global__ __launch_bounds__(TRI_SEL_THREADS) void slot_merge_block_kernel(const MergeArgs A)
{
    __shared__ SelShared sh;
    const TriStepHdr *hdr = (const TriStepHdr *)A.upload;
    const TriPlanEntry *plan = (const TriPlanEntry *)(A.upload + hdr->plan_off);
    if (hdr->n_plan == 0) return;                            // (a replayed launch of a step without a plan: not a turn)
    const uint32_t parity = hdr->merge_parity & 1u;
    if (blockIdx.x == 0 && threadIdx.x == 0) A.rescans[1 + (parity ^ 1u)] = 0;
    const uint32_t queued = A.rescans[1 + parity];
    for (uint32_t i = blockIdx.x; i < queued; i += gridDim.x) merge_block(A, plan[A.merge_queue[i]], sh);   // (uniform)
}

// ------------------------------------------------------------------------------------------------
// Coarse selection by one wavefront per newly admitted query (no workgroup barrier anywhere).
//  pass 1: the row of scores streams through registers, 2048 at a time: load q of chunk c gives lane l the four
//          scores from c * 2048 + q * 256 + l * 4 on (a wavefront's load reads one contiguous KiB), so the 32 scores
//          of every 128-byte line sit in eight neighbouring lanes.  The minimum key of each line is taken inside
//          those eight lanes (three DPP steps) and kept by one of them: up to 512 line minima, each a distinct element
//          of the row.  The nprobe-th smallest of them, T, is not better than the nprobe-th best of the row (the
//          nprobe-th best of a subset never is); it is found by bisection on its 32 bits, every count a ballot.
//  pass 2: only lines whose minimum is not beyond T can hold a key that is not -- nprobe lines or a few more.  They are
//          listed, each is read again by one lane, and their keys not beyond T (a few dozen) are compacted into LDS by
//          a prefix count across the lanes, sorted exactly by rank counting and the nprobe best written.
// The row is read from memory once and an eighth of it twice.  (Reading all of it twice made the kernel wait for
// HBM: 536 MB per launch at configuration 4, as long as the workgroup kernel before it took.)
// Rows it cannot settle -- more than CW_CHUNKS * 2048 centroids, more than CW_NPROBE_MAX probes, masses of equal
// scores -- are queued for coarse_select_kernel.  Word 4 + 64 * parity + group of the counter block holds the number
// of queued rows of that group; the rows of group g are queued from g.first_new on.
#define CW_CHUNKS 8
#define CW_LINES (CW_CHUNKS * 64)       // 128-byte lines of a row the kernel can hold minima of
#define CW_NPROBE_MAX 128
#define CSEL_QHEAD(parity, gi) (4u + 64u * (parity) + (gi))

struct CoarseWaveLds {
    uint64_t a[MRG_CAP], b[MRG_CAP];
    uint16_t line[CW_LINES];            // lines to read again
};

// Minimum over the eight lanes 8 * (l / 8) .. + 7: quad butterfly, then the mirror image inside the half row.
__device__ __forceinline__ uint32_t cw_min8(uint32_t v)
{
    uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0xB1, 0xF, 0xF, false);    // quad_perm [1,0,3,2]
    v = o < v ? o : v;
    o = (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x4E, 0xF, 0xF, false);             // quad_perm [2,3,0,1]
    v = o < v ? o : v;
    o = (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x141, 0xF, 0xF, false);            // row_half_mirror
    return o < v ? o : v;
}

// SHORT: the instantiation for rows of at most 4096 scores (kept in registers); the other one serves the longer rows.
// A launch of the wrong one for a group's index leaves at once.
template <bool SHORT>
__global__ __launch_bounds__(TRI_SEL_THREADS) __attribute__((amdgpu_waves_per_eu(SHORT ? 3 : 4, SHORT ? 3 : 4))) void coarse_select_wave_kernel(
    const float *__restrict__ scores, const uint8_t *__restrict__ upload, uint32_t gi,
    const TriIndexDev *__restrict__ indexes, uint32_t *__restrict__ probe, uint32_t nprobe_max,
    uint32_t *__restrict__ counters, uint32_t *__restrict__ queue)
{
    constexpr uint32_t NW = TRI_SEL_THREADS / 64;
    __shared__ CoarseWaveLds wv[NW];
    // (the wavefront's number as a scalar: everything that depends on the row -- the descriptor of its scores first of
    // all -- is then uniform for the compiler too)
    const uint32_t lane = threadIdx.x & 63, wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    // (group gi of the step's header: which admission records, which index; surplus wavefronts leave)
    const TriStepHdr *hdr = (const TriStepHdr *)upload;
    if (gi >= hdr->n_groups) return;
    const TriCoarseGroup g = hdr->group[gi];
    const uint32_t r = blockIdx.x * NW + wave;
    if (r >= g.m) return;
    const uint32_t nlist = indexes[g.index].nlist, ldc = tri_coarse_ldc(nlist);
    if ((nlist <= 4096u) != SHORT) return;
    const TriNewDesc d = ((const TriNewDesc *)(upload + hdr->desc_off))[g.first_new + r];
    uint32_t *dst = probe + (size_t)d.slot * nprobe_max;
    CoarseWaveLds &L = wv[wave];
    auto defer = [&]() {                                              // (all lanes of the wavefront take the same way)
        if (lane == 0) queue[g.first_new + atomicAdd(&counters[CSEL_QHEAD(hdr->coarse_parity, gi)], 1u)] = r;
    };
    if (nlist > CW_LINES * 32u || d.nprobe >= nlist || d.nprobe > CW_NPROBE_MAX) { defer(); return; }
    // (loads through a descriptor that ends with the row: past its end they return zeros, which the padding mask covers)
    const __amdgpu_buffer_rsrc_t rrs =
        __builtin_amdgcn_make_buffer_rsrc((void *)(scores + (size_t)r * ldc), 0, nlist * 4u, 0x00020000);
    typedef unsigned int cw_u32x4 __attribute__((ext_vector_type(4)));
    // keys of the four scores from element e0 on (all-ones: padding past the row's end)
    auto keys_of = [&](const cw_u32x4 &v, uint32_t e0, uint32_t (&k)[4]) {
        const uint32_t raw[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) k[j] = sel_key(__uint_as_float(raw[j]), d.metric) | (e0 + j < nlist ? 0u : 0xFFFFFFFFu);
    };
    const uint32_t nchunks = (nlist + 2047u) / 2048u;                 // (uniform)
    // A row of at most 4096 scores is one or two chunks, which stay in registers: the minima are then taken over the
    // four scores of every load and lane (up to 1024 of them -- the lines of so short a row would be too few to bound
    // anything), and pass 2 needs no second read.
    constexpr bool short_row = SHORT;                                 // (nchunks <= 2)
    constexpr int CW_MINIMA = SHORT ? 16 : CW_CHUNKS;
    uint32_t m[CW_MINIMA];        // long rows: m[c] = minimum of line c * 64 + (l % 8) * 8 + l / 8; short rows: m[8 c + q] = of this lane's load q of chunk c
    if constexpr (SHORT) {
#pragma unroll
        for (int i = 0; i < CW_MINIMA; ++i) m[i] = 0xFFFFFFFFu;
    }
    cw_u32x4 v[2][8];
#pragma unroll
    for (int q = 0; q < 8; ++q) v[0][q] = __builtin_amdgcn_raw_buffer_load_b128(rrs, lane * 16u, q * 1024u, 2);   // (read once: non-temporal)
    if constexpr (short_row) {
#pragma unroll
        for (int q = 0; q < 8; ++q) v[1][q] = __builtin_amdgcn_raw_buffer_load_b128(rrs, lane * 16u, 8192u + q * 1024u, 2);
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                uint32_t k[4];
                keys_of(v[c][q], c * 2048u + q * 256u + lane * 4u, k);
                const uint32_t mn = k[0] < k[1] ? k[0] : k[1], mn2 = k[2] < k[3] ? k[2] : k[3];
                m[c * 8 + q] = mn < mn2 ? mn : mn2;
            }
    } else {
        // (the loads of chunk c + 1 are issued before chunk c is worked on; a chunk past the row's end costs no memory
        // access and is skipped)
#pragma unroll
        for (int c = 0; c < CW_CHUNKS; ++c) {
            if (c + 1 < CW_CHUNKS) {
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    v[(c + 1) & 1][q] = __builtin_amdgcn_raw_buffer_load_b128(rrs, lane * 16u, (c + 1) * 8192u + q * 1024u, 2);
            }
            m[c] = 0xFFFFFFFFu;
            if ((uint32_t)c < nchunks) {
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    uint32_t k[4];
                    keys_of(v[c & 1][q], c * 2048u + q * 256u + lane * 4u, k);
                    uint32_t mn = k[0] < k[1] ? k[0] : k[1];
                    const uint32_t mn2 = k[2] < k[3] ? k[2] : k[3];
                    mn = cw_min8(mn < mn2 ? mn : mn2);
                    m[c] = (lane & 7u) == (uint32_t)q ? mn : m[c];
                }
            }
        }
    }
    uint32_t T = 0;
    for (int b = 31; b >= 0; --b) {
        const uint32_t trial = T | ((1u << b) - 1u);                  // (bit b clear, every lower bit set)
        uint32_t cnt = 0;
#pragma unroll
        for (int c = 0; c < CW_MINIMA; ++c)
            cnt += (uint32_t)__popcll(__ballot(m[c] <= trial));
        if (cnt < d.nprobe) T |= 1u << b;
    }
    if (T == 0xFFFFFFFFu) { defer(); return; }                        // (fewer than nprobe minima that are not padding)
    if constexpr (short_row) {
        uint32_t cnt = 0;                                             // (the keys are made twice rather than kept: registers)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                uint32_t k[4];
                keys_of(v[c][q], c * 2048u + q * 256u + lane * 4u, k);
#pragma unroll
                for (int j = 0; j < 4; ++j) cnt += k[j] <= T ? 1u : 0u;
            }
        const uint32_t inc2 = thr_wave_scan(cnt, 0u, [](uint32_t a, uint32_t b2) { return a + b2; });
        const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)inc2, 63);
        if (total > MRG_CAP) { defer(); return; }
        uint32_t pos = inc2 - cnt;
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                uint32_t k[4];
                keys_of(v[c][q], c * 2048u + q * 256u + lane * 4u, k);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (k[j] <= T) L.a[pos++] = ((uint64_t)k[j] << 32) | (c * 2048u + q * 256u + lane * 4u + j);
            }
        mrg_rank_sort(L.a, total, L.b, lane);
        for (uint32_t i = lane; i < d.nprobe; i += 64) dst[i] = (uint32_t)(L.b[i] & 0xFFFFFFFFu);
        return;
    }
    // the lines to read again
    uint32_t mine = 0;
#pragma unroll
    for (int c = 0; c < CW_CHUNKS; ++c) mine += m[c] <= T ? 1u : 0u;
    const uint32_t incl = thr_wave_scan(mine, 0u, [](uint32_t a, uint32_t b2) { return a + b2; });
    const uint32_t nlines = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    {
        uint32_t pos = incl - mine;
#pragma unroll
        for (int c = 0; c < CW_CHUNKS; ++c)
            if (m[c] <= T) L.line[pos++] = (uint16_t)(c * 64u + (lane & 7u) * 8u + (lane >> 3));
    }
    thr_wave_fence();
    uint32_t total = 0;
    for (uint32_t l0 = 0; l0 < nlines; l0 += 64) {                    // (nlines >= nprobe; one round unless scores tie in masses)
        const bool have = l0 + lane < nlines;
        const uint32_t e0 = have ? (uint32_t)L.line[l0 + lane] * 32u : 0xFFFFFFE0u;    // (no line: out of range, padding keys)
        cw_u32x4 v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = __builtin_amdgcn_raw_buffer_load_b128(rrs, e0 * 4u, q * 16u, 0);
        uint32_t k[8][4];
        uint32_t cnt = 0;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            keys_of(v[q], e0 + q * 4u, k[q]);
#pragma unroll
            for (int j = 0; j < 4; ++j) cnt += have && k[q][j] <= T ? 1u : 0u;
        }
        const uint32_t inc2 = thr_wave_scan(cnt, 0u, [](uint32_t a, uint32_t b2) { return a + b2; });
        uint32_t pos = total + inc2 - cnt;
        total += (uint32_t)__builtin_amdgcn_readlane((int)inc2, 63);
        if (total > MRG_CAP) break;                                   // (uniform)
#pragma unroll
        for (int q = 0; q < 8; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (have && k[q][j] <= T) L.a[pos++] = ((uint64_t)k[q][j] << 32) | (e0 + q * 4u + j);
    }
    if (total > MRG_CAP) { defer(); return; }
    mrg_rank_sort(L.a, total, L.b, lane);
    for (uint32_t i = lane; i < d.nprobe; i += 64) dst[i] = (uint32_t)(L.b[i] & 0xFFFFFFFFu);
}

// The rows the kernel above queued, dealt out among a fixed number of workgroups.  The queue heads come in two sets,
// used in turn by the steps that admit queries: the first group's launch of a step puts the other set back to zero
// (its last readers, the launches of the previous such step, have finished).
__global__ __launch_bounds__(TRI_SEL_THREADS) void coarse_select_kernel(
    const float *__restrict__ scores, const uint8_t *__restrict__ upload, uint32_t gi,
    const TriIndexDev *__restrict__ indexes, uint32_t *__restrict__ probe, uint32_t nprobe_max,
    uint32_t *__restrict__ counters, const uint32_t *__restrict__ queue)
{
    __shared__ SelShared sh;
    const TriStepHdr *hdr = (const TriStepHdr *)upload;
    if (gi >= hdr->n_groups) return;
    if (gi == 0 && blockIdx.x == 0 && threadIdx.x < TRI_MAX_COARSE_GROUPS)
        counters[CSEL_QHEAD(hdr->coarse_parity ^ 1u, threadIdx.x)] = 0u;
    const TriCoarseGroup g = hdr->group[gi];
    const uint32_t nq = counters[CSEL_QHEAD(hdr->coarse_parity, gi)];
    for (uint32_t qi = blockIdx.x; qi < nq; qi += gridDim.x) {
        coarse_select_row(sh, scores, upload, hdr, g, queue[g.first_new + qi], indexes, probe, nprobe_max);
        __syncthreads();                                              // (the workgroup's next row reuses sh)
    }
}

// nlist: the number of centroids of the group's index when the caller knows it (only the kernel for that row length is
// launched), 0 when it does not (a recorded step serves whatever index a group turns out to have: both are).
hipError_t tri_launch_coarse_select(const TriLaunchCtx &c, const TriDevWs &ws, uint32_t group, uint32_t grid_m, uint32_t nlist)
{
    if (grid_m == 0) return hipSuccess;
    constexpr uint32_t NW = TRI_SEL_THREADS / 64;
    if (nlist == 0 || nlist <= 4096u)
        hipLaunchKernelGGL(coarse_select_wave_kernel<true>, dim3((grid_m + NW - 1) / NW), dim3(TRI_SEL_THREADS), 0, c.stream,
                           ws.coarse_scores, ws.upload, group, ws.indexes, ws.probe, c.nprobe_max, ws.rescans, ws.coarse_queue);
    if (nlist == 0 || nlist > 4096u)
        hipLaunchKernelGGL(coarse_select_wave_kernel<false>, dim3((grid_m + NW - 1) / NW), dim3(TRI_SEL_THREADS), 0, c.stream,
                           ws.coarse_scores, ws.upload, group, ws.indexes, ws.probe, c.nprobe_max, ws.rescans, ws.coarse_queue);
    hipLaunchKernelGGL(coarse_select_kernel, dim3(grid_m < 256u ? grid_m : 256u), dim3(TRI_SEL_THREADS), 0, c.stream,
                       ws.coarse_scores, ws.upload, group, ws.indexes, ws.probe, c.nprobe_max, ws.rescans, ws.coarse_queue);
    return hipGetLastError();
}

hipError_t tri_launch_merge(const TriLaunchCtx &c, const TriDevWs &ws, uint32_t grid_plan, bool keep_probes)
{
    if (grid_plan == 0) return hipSuccess;
    const MergeArgs A = {ws.upload, ws.slot_meta, ws.indexes, ws.item_glist, ws.slot_cand_cnt, ws.glist_len, ws.glist_voff, ws.cand,
                         ws.topk_score, ws.topk_id, ws.topk_count, c.kmax, ws.res_block, ws.probe, c.nprobe_max,
                         keep_probes ? ws.res_probes : (uint32_t *)nullptr, ws.slot_query, c.slot_row_bytes, ws.slot_qnorm,
                         ws.rescans, ws.merge_queue};
    constexpr uint32_t NW = TRI_SEL_THREADS / 64;
    hipLaunchKernelGGL(slot_merge_wave_kernel, dim3((grid_plan + NW - 1) / NW), dim3(TRI_SEL_THREADS), 0, c.stream, A);
    const uint32_t general = grid_plan < c.n_cu * 4 ? grid_plan : c.n_cu * 4;
    hipLaunchKernelGGL(slot_merge_block_kernel, dim3(general), dim3(TRI_SEL_THREADS), 0, c.stream, A);
    return hipGetLastError();
}
