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

// Scores of 32 stored vectors (v0 .. v0 + 31 of a list that starts at `list`) against the query, by one wavefront:
// the query's pieces as the first operand of every product (all 32 rows of that operand are the query), the
// vectors' as the second, 128-byte group after group and 32-byte chunk after chunk -- the order in which the scan
// kernels accumulate, so the sums come out bit for bit the same.  Lane l returns the score of vector v0 + l % 32.
template <int DT>
__device__ __forceinline__ float sel_rescan_block(const SelRescan &rs, const uint8_t *__restrict__ list, uint32_t v0, uint32_t len,
                                                  uint32_t lane)
{
    const uint32_t r = lane & 31, kg = lane >> 5;
    const uint32_t row_bytes = rs.ix->row_bytes;
    const uint32_t v = v0 + r < len ? v0 + r : len - 1;                  // (rows past the end: any valid row, never used)
    const uint8_t *x = list + (size_t)v * row_bytes + kg * 16;
    const uint8_t *q = rs.qrow + kg * 16;
    tri_f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    for (uint32_t g = 0; g < row_bytes; g += 128)
#pragma unroll
        for (int c = 0; c < 4; ++c) tri_mma32<DT>(acc, *(const uint4 *)(q + g + c * 32), *(const uint4 *)(x + g + c * 32));
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
        const uint8_t *list = (const uint8_t *)rs.ix->vecs + (size_t)voff * row_bytes;
        for (uint32_t v0 = 0; v0 < len; v0 += 32, ++gblock) {
            if (gblock % stride != 0 || (gblock / stride) % NW != wave) continue;
            const float dot = rs.ix->dtype == 1u ? sel_rescan_block<TRI_DT_F16>(rs, list, v0, len, lane)
                                                 : sel_rescan_block<TRI_DT_F32>(rs, list, v0, len, lane);
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

__global__ __launch_bounds__(TRI_SEL_THREADS) void coarse_select_kernel(
    const float *__restrict__ scores, const uint8_t *__restrict__ upload, uint32_t gi,
    const TriIndexDev *__restrict__ indexes, uint32_t *__restrict__ probe, uint32_t nprobe_max)
{
    __shared__ SelShared sh;
    // (group gi of the step's header: which admission records, which index; surplus workgroups leave)
    const TriStepHdr *hdr = (const TriStepHdr *)upload;
    if (gi >= hdr->n_groups) return;
    const TriCoarseGroup g = hdr->group[gi];
    if (blockIdx.x >= g.m) return;
    const uint32_t nlist = indexes[g.index].nlist, ldc = (nlist + 31u) / 32u * 32u;
    const TriNewDesc d = ((const TriNewDesc *)(upload + hdr->desc_off))[g.first_new + blockIdx.x];
    const float *row = scores + (size_t)blockIdx.x * ldc;
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

hipError_t tri_launch_coarse_select(const TriLaunchCtx &c, const TriDevWs &ws, uint32_t group, uint32_t grid_m)
{
    if (grid_m == 0) return hipSuccess;
    hipLaunchKernelGGL(coarse_select_kernel, dim3(grid_m), dim3(TRI_SEL_THREADS), 0, c.stream, ws.coarse_scores,
                       ws.upload, group, ws.indexes, ws.probe, c.nprobe_max);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Threshold of each running slot for this step's scan: a bound for the k-th best key among the slot's
// sample scores (the first TRI_SAMPLE_VECS vectors of up to TRI_THRESH_ITEMS of its lists) and its
// running top-k -- a subset of its candidates, so nothing of its final top-k lies beyond it.  Fewer
// than k such keys: no filtering (all-ones).
__global__ __launch_bounds__(TRI_SEL_THREADS) void slot_threshold_kernel(
    const uint8_t *__restrict__ upload, const TriSlotMeta *__restrict__ slot_meta,
    const uint32_t *__restrict__ item_glist, const uint32_t *__restrict__ item_sorted_pos,
    const uint32_t *__restrict__ glist_len, const uint32_t *__restrict__ glist_voff,
    const float *__restrict__ sample_scores, const float *__restrict__ topk_score,
    const uint32_t *__restrict__ topk_count, uint32_t kmax, uint32_t *__restrict__ thr_key, uint2 *__restrict__ cand,
    uint32_t *__restrict__ slot_cand_off, uint32_t *__restrict__ slot_cand_cap, uint32_t *__restrict__ slot_cand_cnt)
{
    static_assert(TRI_SAMPLE_VECS % TRI_VB == 0 && TRI_VB == 32, "the sample is the first blocks of a list");
    static_assert(TRI_THRESH_ITEMS * TRI_SAMPLE_VECS + TRI_KMAX_POW2 <= 2 * SEL_CAP, "the sample keys must fit the LDS array");
    __shared__ SelShared sh;
    const TriStepHdr *hdr = (const TriStepHdr *)upload;
    if (blockIdx.x >= hdr->n_plan) return;
    const TriPlanEntry e = ((const TriPlanEntry *)(upload + hdr->plan_off))[blockIdx.x];
    const TriSlotMeta meta = slot_meta[e.slot];
    const uint32_t desc = meta.metric == 1u;
    const uint32_t have = e.cursor > 0 ? topk_count[e.slot] : 0u;
    const uint32_t nitems = e.take < TRI_THRESH_ITEMS ? e.take : TRI_THRESH_ITEMS;
    uint32_t *keys = (uint32_t *)sh.pool;                  // room for 2 * SEL_CAP keys
    // per item (kept in the segment cache, which this kernel does not use otherwise): .off = its sample
    // row, .len = how many of its TRI_SAMPLE_VECS scores exist, .id_off = stored position of its list's first vector
    const uint32_t ncached = e.take < SEL_SEGCACHE ? e.take : SEL_SEGCACHE;
    if (threadIdx.x == 0) sh.cnt = 0;
    for (uint32_t s = threadIdx.x; s < ncached; s += TRI_SEL_THREADS) {
        const uint32_t it = e.item_base + s, g = item_glist[it];
        sh.seg[s] = SelSeg{item_sorted_pos[it], min(glist_len[g], (uint32_t)TRI_SAMPLE_VECS), glist_voff[g], 0u};
    }
    __syncthreads();
    // keys[s * TRI_SAMPLE_VECS + l] = key of sample l of item s (all-ones where the list is shorter), then the running top-k
    const uint32_t nsample = nitems * TRI_SAMPLE_VECS, n = nsample + have;
    uint32_t valid_here = 0;
    for (uint32_t i = threadIdx.x; i < n; i += TRI_SEL_THREADS) {
        uint32_t key = 0xFFFFFFFFu;
        if (i < nsample) {
            const uint32_t s = i / TRI_SAMPLE_VECS, l = i % TRI_SAMPLE_VECS;
            if (l < sh.seg[s].len) key = sel_key(sample_scores[(size_t)sh.seg[s].off * TRI_SAMPLE_VECS + l], desc);
        } else {
            key = sel_key(topk_score[(size_t)e.slot * kmax + (i - nsample)], desc);
        }
        keys[i] = key;
        valid_here += key != 0xFFFFFFFFu;
    }
    if (valid_here) atomicAdd(&sh.cnt, valid_here);
    __syncthreads();
    const uint32_t nvalid = sh.cnt;
    __syncthreads();
    uint32_t thr = 0xFFFFFFFFu;
    if (nvalid >= meta.k) thr = sel_keys_threshold(sh, keys, n, meta.k);
    if (threadIdx.x == 0) {
        thr_key[e.slot] = thr;
        sh.count = 0;                     // (the selection above used it; from here on: pairs emitted)
    }
    __syncthreads();
    // The sample IS the first block(s) of every list: its scores that pass the threshold become the first
    // candidates of the query's region here, and the scan starts every list behind them.  One item per
    // half-wavefront; (score bits, stored position) pairs, placed through one LDS counter; the main launch counts
    // on from what this leaves in the slot's counter.
    // (The first TRI_THRESH_ITEMS items' keys are still in LDS -- a key gives back its score bit for bit --;
    // items beyond them, and beyond the cached descriptors, are read again.)
    const uint32_t l32 = threadIdx.x & 31;
    for (uint32_t s = threadIdx.x >> 5; s < e.take; s += TRI_SEL_THREADS / 32) {
        uint32_t row, n_l, voff;
        if (s < ncached) {
            row = sh.seg[s].off; n_l = sh.seg[s].len; voff = sh.seg[s].id_off;
        } else {
            const uint32_t it = e.item_base + s, g = item_glist[it];
            row = item_sorted_pos[it];
            n_l = min(glist_len[g], (uint32_t)TRI_SAMPLE_VECS);
            voff = glist_voff[g];
        }
#pragma unroll
        for (uint32_t sb = 0; sb < TRI_SAMPLE_VECS / 32; ++sb) {      // 32 samples at a time
            const uint32_t l = sb * 32 + l32;
            uint32_t key = 0xFFFFFFFFu;
            if (l < n_l) key = s < nitems ? keys[s * TRI_SAMPLE_VECS + l] : sel_key(sample_scores[(size_t)row * TRI_SAMPLE_VECS + l], desc);
            const bool pass = l < n_l && key <= thr;
            const uint64_t m = __ballot(pass);
            const uint32_t half = (threadIdx.x & 32) ? (uint32_t)(m >> 32) : (uint32_t)m;
            uint32_t first = 0;
            if (l32 == 0 && half) first = atomicAdd(&sh.count, (uint32_t)__popc(half));
            first = (uint32_t)__shfl((int)first, (int)(threadIdx.x & 32), 64);
            const uint32_t pos = first + __popc(half & ((1u << l32) - 1u));
            if (pass && pos < e.cand_cap) cand[(size_t)e.cand_off + pos] = make_uint2(__float_as_uint(sel_unkey(key, desc)), voff + l);
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        slot_cand_off[e.slot] = e.cand_off;
        slot_cand_cap[e.slot] = e.cand_cap;
        slot_cand_cnt[e.slot] = sh.count;
    }
}

hipError_t tri_launch_threshold(const TriLaunchCtx &c, const TriDevWs &ws, uint32_t grid_plan)
{
    if (grid_plan == 0) return hipSuccess;
    hipLaunchKernelGGL(slot_threshold_kernel, dim3(grid_plan), dim3(TRI_SEL_THREADS), 0, c.stream, ws.upload, ws.slot_meta,
                       ws.item_glist, ws.item_sorted_pos, ws.glist_len, ws.glist_voff, ws.sample_scores, ws.topk_score,
                       ws.topk_count, c.kmax, ws.thr_key, ws.cand, ws.slot_cand_off, ws.slot_cand_cap, ws.slot_cand_cnt);
    return hipGetLastError();
}

// Squared L2 distance of a stored row to a query row in the difference form, sum of (x_i - q_i)^2, by the 32
// lanes of a half-wavefront: lane l takes the 16-byte pieces l, l + 32, ... of both rows, the partial sums are
// combined by a butterfly (a fixed order, the same in every lane).  fp32 arithmetic; fp16 inputs widen exactly.
template <typename T>
__device__ __forceinline__ float sel_l2_diff_form(const uint8_t *__restrict__ x, const uint8_t *__restrict__ q, uint32_t row_bytes,
                                                  uint32_t l32)
{
    constexpr int PER = 16 / sizeof(T);
    float acc = 0.f;
    for (uint32_t o = l32 * 16; o < row_bytes; o += 32 * 16) {
        const uint4 xv = *(const uint4 *)(x + o), qv = *(const uint4 *)(q + o);
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
// Slot merge: one workgroup per running slot of the step.  Candidates = the (score, stored position) pairs
// the scan kept in the slot's region of the candidate buffer in this step + its running top-k.  Should the
// region have been too small (the slot's counter ran past its capacity), the pairs in it are ignored and the
// slot's lists of this step are scored again right here (SelRescan): slow, exact, and rare.
// Output = new running top-k, or -- when the slot retires in this step -- its final result.
__global__ __launch_bounds__(TRI_SEL_THREADS) void slot_merge_kernel(
    const uint8_t *__restrict__ upload, const TriSlotMeta *__restrict__ slot_meta,
    const TriIndexDev *__restrict__ indexes, const uint32_t *__restrict__ item_glist,
    const uint32_t *__restrict__ slot_cand_cnt, const uint32_t *__restrict__ glist_len,
    const uint32_t *__restrict__ glist_voff, const uint2 *__restrict__ cand, float *__restrict__ topk_score,
    uint32_t *__restrict__ topk_id, uint32_t *__restrict__ topk_count, uint32_t kmax,
    uint32_t *__restrict__ res_block, const uint32_t *__restrict__ probe, uint32_t nprobe_max,
    uint32_t *__restrict__ res_probes, const uint8_t *__restrict__ slot_query, uint32_t slot_row_bytes,
    const float *__restrict__ slot_qnorm, uint32_t *__restrict__ rescans)
{
    __shared__ SelShared sh;
    const TriStepHdr *hdr = (const TriStepHdr *)upload;
    if (blockIdx.x >= hdr->n_plan) return;
    const TriPlanEntry e = ((const TriPlanEntry *)(upload + hdr->plan_off))[blockIdx.x];
    const TriSlotMeta meta = slot_meta[e.slot];
    const uint32_t desc = meta.metric == 1u;
    const uint32_t have = e.cursor > 0 ? topk_count[e.slot] : 0u;
    float *run_score = topk_score + (size_t)e.slot * kmax;
    uint32_t *run_id = topk_id + (size_t)e.slot * kmax;
    const uint32_t asked = slot_cand_cnt[e.slot];
    const bool overflow = asked > e.cand_cap;                 // (the same for every thread of the workgroup)
    SelRescan rs = {item_glist, glist_len, glist_voff, &indexes[meta.index], slot_query + (size_t)e.slot * slot_row_bytes,
                    slot_qnorm[e.slot], meta.metric == 0u, e.item_base, e.take, 0u};
    if (overflow) {
        uint32_t part = 0;
        for (uint32_t it = threadIdx.x; it < e.take; it += TRI_SEL_THREADS) part += glist_len[item_glist[e.item_base + it]];
        const uint32_t incl = sel_block_scan_incl(part, sh.wave_tot);
        if (threadIdx.x == TRI_SEL_THREADS - 1) {
            sh.tmax = incl;
            atomicAdd(rescans, 1u);
        }
        __syncthreads();
        rs.total = sh.tmax;
        __syncthreads();
    }
    const SelSrc src = {cand, indexes[meta.index].ids, run_score, run_id, overflow ? 0u : 1u, have, overflow ? &rs : nullptr};
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
        const TriIndexDev &ix = indexes[meta.index];
        const uint8_t *qrow = slot_query + (size_t)e.slot * slot_row_bytes;
        uint64_t *fresh = best == sh.pool ? sh.small : sh.pool;             // (n <= kmax <= SEL_SMALL)
        const uint32_t l32 = threadIdx.x & 31;
        for (uint32_t i = threadIdx.x >> 5; i < n; i += TRI_SEL_THREADS / 32) {
            const uint32_t id = (uint32_t)(best[i] & 0xFFFFFFFFu);
            const uint8_t *x = (const uint8_t *)ix.vecs + (size_t)ix.inv[id] * ix.row_bytes;
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
    if (e.retire_idx >= 0) {
        uint32_t *rec = res_block + (size_t)e.retire_idx * (1u + 2u * kmax);
        if (threadIdx.x == 0) rec[0] = n;
        for (uint32_t i = threadIdx.x; i < n; i += TRI_SEL_THREADS) {
            const uint64_t c = best[i];
            rec[1 + i] = (uint32_t)(c & 0xFFFFFFFFu);
            rec[1 + kmax + i] = __float_as_uint(sel_unkey((uint32_t)(c >> 32), desc));
        }
        if (res_probes) {
            const uint32_t *srcp = probe + (size_t)e.slot * nprobe_max;
            uint32_t *dst = res_probes + (size_t)e.retire_idx * nprobe_max;
            for (uint32_t i = threadIdx.x; i < meta.nprobe; i += TRI_SEL_THREADS) dst[i] = srcp[i];
        }
    } else {
        for (uint32_t i = threadIdx.x; i < n; i += TRI_SEL_THREADS) {
            const uint64_t c = best[i];
            run_id[i] = (uint32_t)(c & 0xFFFFFFFFu);
            run_score[i] = sel_unkey((uint32_t)(c >> 32), desc);
        }
        if (threadIdx.x == 0) topk_count[e.slot] = n;
    }
}

hipError_t tri_launch_merge(const TriLaunchCtx &c, const TriDevWs &ws, uint32_t grid_plan, bool keep_probes)
{
    if (grid_plan == 0) return hipSuccess;
    hipLaunchKernelGGL(slot_merge_kernel, dim3(grid_plan), dim3(TRI_SEL_THREADS), 0, c.stream, ws.upload, ws.slot_meta,
                       ws.indexes, ws.item_glist, ws.slot_cand_cnt, ws.glist_len, ws.glist_voff, ws.cand, ws.topk_score,
                       ws.topk_id, ws.topk_count, c.kmax, ws.res_block, ws.probe, c.nprobe_max,
                       keep_probes ? ws.res_probes : (uint32_t *)nullptr, ws.slot_query, c.slot_row_bytes, ws.slot_qnorm,
                       ws.rescans);
    return hipGetLastError();
}
