// Per-query top-k (the paper's Sec. 3.2 step "scatter (id, dist) back to the owning request and
// merge into its topM"; here the request's candidates of one step are the score segments of its
// work items plus its running top-k).
//
// Order: ascending 64-bit composite (key << 32 | id), key = order-preserving image of the fp32
// score (bit-flipped for inner product, so "smaller key" always means "better").  Equal scores are
// therefore ordered by ascending id, which makes the result independent of how the candidates
// were batched.
//
// One workgroup selects for one query, in LDS:
//  (1) at most SEL_CAP candidates: all (key, id) pairs are loaded and sorted (bitonic network).
//  (2) more: a strided sample of about SEL_SAMPLE keys is sorted; the sample's m-th key, with m
//      five standard deviations above the expected rank of the k-th best, is a threshold that almost
//      surely admits at least k and far fewer than SEL_CAP candidates; ONE pass over the candidates
//      collects those not worse than it, and they are sorted as in (1).  Whatever the sample says,
//      the result is exact whenever the pass collected between k and SEL_CAP candidates: the k best
//      of the collected set are then the k best of all.
//  (3) otherwise (heavy ties, adversarial order): three histogram passes (11 + 11 + 10 bits) find
//      the key T of the k-th best element; if more elements equal T than are still needed, three more
//      passes over the ids of those elements find the largest id to keep; one pass gathers exactly k.
#include "tri_common.h"

#define SEL_BINS 2048
#define SEL_SEGCACHE 256   // segment descriptors cached in LDS
#define SEL_CAP 4096      // (key, id) pairs sorted in LDS
#define SEL_SAMPLE 1024   // target size of the key sample (at most SEL_CAP keys are kept)

__device__ __forceinline__ uint32_t sel_key(float f, uint32_t desc) { return tri_score_key(f, desc); }
__device__ __forceinline__ float sel_unkey(uint32_t key, uint32_t desc) { return tri_key_score(key, desc); }

// A candidate source: segments.  Dense segment: scores[i], id = ids ? ids[i] : id_base + i.
// Pair segment (pairs != 0): scores points at (score bits, position) pairs, id = ids[position].
struct SelSeg {
    const float *scores;
    const uint32_t *ids;
    uint32_t len;
    uint32_t id_base;
    uint32_t pairs;
    uint32_t pad_;
};

struct SelShared {
    uint64_t pool[SEL_CAP];        // candidates / result (the sample's keys use its first half as uint32_t[SEL_CAP])
    uint32_t hist[SEL_BINS];
    SelSeg seg[SEL_SEGCACHE];      // descriptors of the first segments
    uint32_t wave_tot[8];
    uint32_t digit, need, count, cnt;
};

// `where` is what sel_for_each hands to its callback: the element's index (dense) or stored position (pairs)
__device__ __forceinline__ uint32_t sel_id(const SelSeg &sg, uint32_t where) { return sg.ids ? sg.ids[where] : sg.id_base + where; }

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

// Enumerate candidates with wavefront-uniform control flow: f(valid, key, seg, pos) is called by all
// 64 lanes together (valid = this lane has an element).  The segments are cut into chunks of
// 64 * SEL_UNROLL elements and the workgroup's wavefronts take chunks round-robin across ALL
// segments, so one long segment keeps every wavefront busy and many short ones are spread evenly;
// the SEL_UNROLL loads of a chunk are issued together.  `stride` > 1 visits only the first
// ceil(len / stride) elements of every segment (the sample: list order is id order, which carries no
// information about the scores).  Segment descriptors come from the LDS cache filled by
// sel_cache_segments, beyond it from seg_of.
#define SEL_UNROLL 8

template <class SegFn, class Fn>
__device__ __forceinline__ void sel_for_each(const SelSeg *cache, uint32_t nseg, SegFn seg_of, uint32_t desc,
                                             uint32_t stride, Fn f)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr uint32_t CH = 64 * SEL_UNROLL;
    uint32_t next = wave, base = 0;
    for (uint32_t s = 0; s < nseg; ++s) {
        const SelSeg sg = s < SEL_SEGCACHE ? cache[s] : seg_of(s);
        const uint32_t n = stride > 1 ? (sg.len + stride - 1) / stride : sg.len;
        const uint32_t nch = (n + CH - 1) / CH;
        while (next < base + nch) {
            const uint32_t i0 = (next - base) * CH + lane;
            if (sg.pairs) {
                const uint2 *pp = (const uint2 *)sg.scores;
                uint2 v[SEL_UNROLL];
#pragma unroll
                for (int u = 0; u < SEL_UNROLL; ++u) v[u] = i0 + u * 64 < n ? pp[i0 + u * 64] : make_uint2(0u, 0u);
#pragma unroll
                for (int u = 0; u < SEL_UNROLL; ++u) {
                    const bool valid = i0 + u * 64 < n;
                    f(valid, valid ? sel_key(__uint_as_float(v[u].x), desc) : 0xFFFFFFFFu, sg, v[u].y);
                }
            } else {
                float v[SEL_UNROLL];
#pragma unroll
                for (int u = 0; u < SEL_UNROLL; ++u) v[u] = i0 + u * 64 < n ? sg.scores[i0 + u * 64] : 0.f;
#pragma unroll
                for (int u = 0; u < SEL_UNROLL; ++u) {
                    const bool valid = i0 + u * 64 < n;
                    f(valid, valid ? sel_key(v[u], desc) : 0xFFFFFFFFu, sg, i0 + u * 64);
                }
            }
            next += TRI_SEL_THREADS / 64;
        }
        base += nch;
    }
}

template <class SegFn>
__device__ __forceinline__ void sel_cache_segments(SelSeg *cache, uint32_t nseg, SegFn seg_of)
{
    for (uint32_t s = threadIdx.x; s < nseg && s < SEL_SEGCACHE; s += TRI_SEL_THREADS) cache[s] = seg_of(s);
    __syncthreads();
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

// Path (3): exact radix select of the k best into sh.pool[0..k), unsorted.  total > k.
template <class SegFn>
__device__ void sel_radix(SelShared &sh, uint32_t nseg, SegFn seg_of, uint32_t k, uint32_t desc)
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
        sel_for_each(sh.seg, nseg, seg_of, desc, 1u, [&](bool valid, uint32_t key, const SelSeg &, uint32_t) {
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
            sel_for_each(sh.seg, nseg, seg_of, desc, 1u, [&](bool valid, uint32_t key, const SelSeg &sg, uint32_t i) {
                if (!valid || key != T) return;
                const uint32_t id = sel_id(sg, i);
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
    sel_for_each(sh.seg, nseg, seg_of, desc, 1u, [&](bool valid, uint32_t key, const SelSeg &sg, uint32_t i) {
        bool take = valid && key <= T;
        uint32_t id = 0;
        if (take) {
            id = sel_id(sg, i);
            take = key < T || id <= Tid;
        }
        const uint32_t pos = sel_append_pos(take, &sh.cnt);
        if (take && pos < SEL_CAP) sh.pool[pos] = ((uint64_t)key << 32) | id;
    });
    __syncthreads();
}

// Select the k best of `total` candidates into sh.pool[0..n) sorted ascending by (key, id).
// Returns n = min(k, total).  All threads of the workgroup must call it; it ends with a barrier.
template <class SegFn>
__device__ uint32_t sel_block_topk(SelShared &sh, uint32_t nseg, SegFn seg_of, uint32_t total, uint32_t k,
                                   uint32_t desc)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t n = total < k ? total : k;
    sel_cache_segments(sh.seg, nseg, seg_of);
    if (total <= SEL_CAP) {
        // ---- (1) everything fits
        if (tid == 0) sh.cnt = 0;
        __syncthreads();
        sel_for_each(sh.seg, nseg, seg_of, desc, 1u, [&](bool valid, uint32_t key, const SelSeg &sg, uint32_t i) {
            const uint32_t pos = sel_append_pos(valid, &sh.cnt);
            if (valid) sh.pool[pos] = ((uint64_t)key << 32) | sel_id(sg, i);
        });
        __syncthreads();
        sel_bitonic(sh.pool, total);
        return n;
    }
    // ---- (2) threshold from a sorted sample
    uint32_t *skeys = (uint32_t *)sh.pool;
    const uint32_t stride = (total + SEL_SAMPLE - 1) / SEL_SAMPLE;
    if (tid == 0) sh.cnt = 0;
    __syncthreads();
    sel_for_each(sh.seg, nseg, seg_of, desc, stride, [&](bool valid, uint32_t key, const SelSeg &, uint32_t) {
        const uint32_t pos = sel_append_pos(valid, &sh.cnt);
        if (valid && pos < SEL_CAP) skeys[pos] = key;      // (a few sample keys too many are simply dropped)
    });
    __syncthreads();
    const uint32_t ns = sh.cnt < SEL_CAP ? sh.cnt : SEL_CAP;
    sel_bitonic(skeys, ns);
    // expected rank of the k-th best inside the sample, plus five standard deviations and a floor
    const float mu = (float)k * (float)ns / (float)total;
    const uint32_t m = (uint32_t)(mu + 5.0f * sqrtf(mu) + 4.0f);
    bool done = false;
    if (m < ns) {
        const uint32_t t0 = skeys[m];
        __syncthreads();                       // everyone has read the threshold before the pool is reused
        if (tid == 0) sh.cnt = 0;
        __syncthreads();
        sel_for_each(sh.seg, nseg, seg_of, desc, 1u, [&](bool valid, uint32_t key, const SelSeg &sg, uint32_t i) {
            const bool take = valid && key <= t0;
            const uint32_t pos = sel_append_pos(take, &sh.cnt);
            if (take && pos < SEL_CAP) sh.pool[pos] = ((uint64_t)key << 32) | sel_id(sg, i);
        });
        __syncthreads();
        const uint32_t c = sh.cnt;
        if (c >= k && c <= SEL_CAP) {
            sel_bitonic(sh.pool, c);
            done = true;
        }
    }
    __syncthreads();
    if (!done) {
        // ---- (3) exact radix select, then sort the k survivors
        sel_radix(sh, nseg, seg_of, k, desc);
        sel_bitonic(sh.pool, k);
    }
    return n;
}

// ------------------------------------------------------------------------------------------------
// Coarse selection: probe list of each newly admitted query = the nprobe best centroids, best
// first, ties -> smaller centroid number.
__global__ __launch_bounds__(TRI_SEL_THREADS) void coarse_select_kernel(
    const float *__restrict__ scores, uint32_t ldc, uint32_t nlist, const TriNewDesc *__restrict__ desc,
    uint32_t first_new, uint32_t *__restrict__ probe, uint32_t nprobe_max)
{
    __shared__ SelShared sh;
    const TriNewDesc d = desc[first_new + blockIdx.x];
    const float *row = scores + (size_t)blockIdx.x * ldc;
    auto seg_of = [&](uint32_t) { return SelSeg{row, nullptr, nlist, 0u, 0u, 0u}; };
    const uint32_t n = sel_block_topk(sh, 1u, seg_of, nlist, d.nprobe, d.metric);
    uint32_t *dst = probe + (size_t)d.slot * nprobe_max;
    for (uint32_t i = threadIdx.x; i < n; i += TRI_SEL_THREADS) dst[i] = (uint32_t)(sh.pool[i] & 0xFFFFFFFFu);
}

hipError_t tri_launch_coarse_select(const TriLaunchCtx &c, const TriDevWs &ws, const TriNewDesc *desc_dev,
                                    uint32_t first_new, uint32_t m, uint32_t nlist, uint32_t ldc)
{
    if (m == 0) return hipSuccess;
    hipLaunchKernelGGL(coarse_select_kernel, dim3(m), dim3(TRI_SEL_THREADS), 0, c.stream, ws.coarse_scores, ldc,
                       nlist, desc_dev, first_new, ws.probe, c.nprobe_max);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Threshold of each running slot for this step's scan: the k-th best key among the slot's sample
// scores (the first TRI_SAMPLE_VECS vectors of up to TRI_THRESH_ITEMS of its lists) and its running
// top-k -- a subset of its candidates, so nothing of its final top-k lies beyond it.  Fewer than k
// such keys: no filtering (all-ones).
__global__ __launch_bounds__(TRI_SEL_THREADS) void slot_threshold_kernel(
    const TriPlanEntry *__restrict__ plan, const TriSlotMeta *__restrict__ slot_meta,
    const uint32_t *__restrict__ item_glist, const uint32_t *__restrict__ item_sorted_pos,
    const uint32_t *__restrict__ glist_len, const float *__restrict__ sample_scores,
    const float *__restrict__ topk_score, const uint32_t *__restrict__ topk_count, uint32_t kmax,
    uint32_t *__restrict__ thr_key)
{
    __shared__ SelShared sh;
    const TriPlanEntry e = plan[blockIdx.x];
    const TriSlotMeta meta = slot_meta[e.slot];
    const uint32_t desc = meta.metric == 1u;
    const uint32_t have = e.cursor > 0 ? topk_count[e.slot] : 0u;
    const uint32_t nitems = e.take < TRI_THRESH_ITEMS ? e.take : TRI_THRESH_ITEMS;
    uint32_t *keys = (uint32_t *)sh.pool;                  // room for 2 * SEL_CAP keys
    if (threadIdx.x == 0) sh.cnt = 0;
    __syncthreads();
    // wavefronts take items round-robin; lanes 0..31 the item's sample row
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (uint32_t s = wave; s < nitems; s += TRI_SEL_THREADS / 64) {
        const uint32_t it = e.item_base + s;
        const uint32_t n = min(glist_len[item_glist[it]], (uint32_t)TRI_SAMPLE_VECS);
        const bool valid = lane < n;
        const float v = valid ? sample_scores[(size_t)item_sorted_pos[it] * TRI_SAMPLE_VECS + lane] : 0.f;
        const uint32_t pos = sel_append_pos(valid, &sh.cnt);
        if (valid) keys[pos] = sel_key(v, desc);
    }
    for (uint32_t i0 = wave * 64; i0 < have; i0 += TRI_SEL_THREADS) {
        const bool valid = i0 + lane < have;
        const float v = valid ? topk_score[(size_t)e.slot * kmax + i0 + lane] : 0.f;
        const uint32_t pos = sel_append_pos(valid, &sh.cnt);
        if (valid) keys[pos] = sel_key(v, desc);
    }
    __syncthreads();
    const uint32_t n = sh.cnt;                             // <= 96 * 32 + 1024 = SEL_CAP
    uint32_t thr = 0xFFFFFFFFu;
    if (n >= meta.k) {
        sel_bitonic(keys, n);
        thr = keys[meta.k - 1];
    }
    if (threadIdx.x == 0) thr_key[e.slot] = thr;
}

hipError_t tri_launch_threshold(const TriLaunchCtx &c, const TriDevWs &ws, const TriPlanEntry *plan_dev, uint32_t n_plan)
{
    if (n_plan == 0) return hipSuccess;
    hipLaunchKernelGGL(slot_threshold_kernel, dim3(n_plan), dim3(TRI_SEL_THREADS), 0, c.stream, plan_dev, ws.slot_meta,
                       ws.item_glist, ws.item_sorted_pos, ws.glist_len, ws.sample_scores, ws.topk_score, ws.topk_count,
                       c.kmax, ws.thr_key);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Slot merge: one workgroup per running slot of the step.  Candidates = the (score, position) pairs
// the scan kept for the slot's work items of this step, one segment per (item, chunk), + its running
// top-k.  Output = new running top-k, or -- when the slot retires in this step -- its final result.
__global__ __launch_bounds__(TRI_SEL_THREADS) void slot_merge_kernel(
    const TriPlanEntry *__restrict__ plan, const TriSlotMeta *__restrict__ slot_meta,
    const TriIndexDev *__restrict__ indexes, const uint32_t *__restrict__ item_glist,
    const uint64_t *__restrict__ item_score_off, const uint32_t *__restrict__ item_sorted_pos,
    const uint32_t *__restrict__ surv_count, uint32_t chunk_vecs, const uint32_t *__restrict__ glist_len,
    const uint32_t *__restrict__ glist_voff, const uint32_t *__restrict__ glist_index,
    const float *__restrict__ cand, float *__restrict__ topk_score, uint32_t *__restrict__ topk_id,
    uint32_t *__restrict__ topk_count, uint32_t kmax, uint32_t *__restrict__ res_block,
    const uint32_t *__restrict__ probe, uint32_t nprobe_max, uint32_t *__restrict__ res_probes)
{
    __shared__ SelShared sh;
    __shared__ uint32_t sh_total;
    const TriPlanEntry e = plan[blockIdx.x];
    const TriSlotMeta meta = slot_meta[e.slot];
    const uint32_t desc = meta.metric == 1u;
    const uint32_t have = e.cursor > 0 ? topk_count[e.slot] : 0u;
    float *run_score = topk_score + (size_t)e.slot * kmax;
    uint32_t *run_id = topk_id + (size_t)e.slot * kmax;
    const uint32_t nlist_seg = e.take * TRI_TILES_PER_ITEM;
    const uint32_t nseg = nlist_seg + (have ? 1u : 0u);

    // segment s < nlist_seg: chunk s % 4 of item s / 4 (empty when the list has fewer chunks)
    auto seg_of = [&](uint32_t s) {
        if (s < nlist_seg) {
            const uint32_t it = e.item_base + s / TRI_TILES_PER_ITEM, ch = s % TRI_TILES_PER_ITEM;
            const uint32_t g = item_glist[it];
            const uint32_t nch = (glist_len[g] + chunk_vecs - 1) / chunk_vecs;
            if (ch >= nch) return SelSeg{cand, nullptr, 0u, 0u, 1u, 0u};
            const TriIndexDev &ix = indexes[glist_index[g]];
            return SelSeg{cand + item_score_off[it] + 2u * (size_t)ch * chunk_vecs, ix.ids + glist_voff[g],
                          surv_count[item_sorted_pos[it] * TRI_TILES_PER_ITEM + ch], 0u, 1u, 0u};
        }
        return SelSeg{run_score, run_id, have, 0u, 0u, 0u};
    };
    // total number of candidates
    if (threadIdx.x == 0) sh_total = have;
    __syncthreads();
    uint32_t part = 0;
    for (uint32_t s = threadIdx.x; s < nlist_seg; s += TRI_SEL_THREADS) part += seg_of(s).len;
    if (part) atomicAdd(&sh_total, part);
    __syncthreads();
    const uint32_t total = sh_total;

    const uint32_t n = sel_block_topk(sh, nseg, seg_of, total, meta.k, desc);
    // (all reads of the running buffer are done: sel_block_topk ends with a barrier)
    if (e.retire_idx >= 0) {
        uint32_t *rec = res_block + (size_t)e.retire_idx * (1u + 2u * kmax);
        if (threadIdx.x == 0) rec[0] = n;
        for (uint32_t i = threadIdx.x; i < n; i += TRI_SEL_THREADS) {
            const uint64_t c = sh.pool[i];
            rec[1 + i] = (uint32_t)(c & 0xFFFFFFFFu);
            rec[1 + kmax + i] = __float_as_uint(sel_unkey((uint32_t)(c >> 32), desc));
        }
        if (res_probes) {
            const uint32_t *src = probe + (size_t)e.slot * nprobe_max;
            uint32_t *dst = res_probes + (size_t)e.retire_idx * nprobe_max;
            for (uint32_t i = threadIdx.x; i < meta.nprobe; i += TRI_SEL_THREADS) dst[i] = src[i];
        }
    } else {
        for (uint32_t i = threadIdx.x; i < n; i += TRI_SEL_THREADS) {
            const uint64_t c = sh.pool[i];
            run_id[i] = (uint32_t)(c & 0xFFFFFFFFu);
            run_score[i] = sel_unkey((uint32_t)(c >> 32), desc);
        }
        if (threadIdx.x == 0) topk_count[e.slot] = n;
    }
}

hipError_t tri_launch_merge(const TriLaunchCtx &c, const TriDevWs &ws, const TriPlanEntry *plan_dev, uint32_t n_plan,
                            bool keep_probes, uint32_t chunk_vecs)
{
    if (n_plan == 0) return hipSuccess;
    hipLaunchKernelGGL(slot_merge_kernel, dim3(n_plan), dim3(TRI_SEL_THREADS), 0, c.stream, plan_dev, ws.slot_meta,
                       ws.indexes, ws.item_glist, ws.item_score_off, ws.item_sorted_pos, ws.surv_count, chunk_vecs,
                       ws.glist_len, ws.glist_voff, ws.glist_index, ws.scores, ws.topk_score, ws.topk_id, ws.topk_count,
                       c.kmax, ws.res_block, ws.probe, c.nprobe_max, keep_probes ? ws.res_probes : (uint32_t *)nullptr);
    return hipGetLastError();
}
