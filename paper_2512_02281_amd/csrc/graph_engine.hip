// The paper's own engine (Sec. 3.2): continuous batching of best-first searches over a fixed-degree
// neighbour graph, one "extend" of every running request per step.  Per request and on the device: a
// candidate list topM (sorted composites of score key, id and an "expanded" mark), a visited set that is
// exact -- so "first seen" is a property of the ids alone and a trajectory does not depend on timing --, its
// query row.  The visited set is a hash table of ids sized by what one request can ever see (entry points +
// max_iters * p * D), whatever the size of the database: a small table that takes the first few thousand ids
// (a handful of linear probes each), and a large one behind it for ids whose neighbourhood in the small table
// is taken.  The small tables of all slots together stay cache-resident; a bit per database row and slot, which
// is used instead where that is the smaller of the two, is a gigabyte at a million rows and 8192 slots.  A step is ONE fixed-shape launch
// over the slots of a group, a workgroup per slot -- idle slots leave at once, which is the masked padding
// of the paper's fixed-shape task array -- in three phases:
//   distance : every task of the slot = one gathered row against the slot's query, 16 lanes per task;
//   merge    : tasks' (score, id) + topM -> new topM; stop rule; a finished request writes its record
//              into the step's pinned result block;
//   extend   : a request that goes on selects up to p non-expanded parents of the new topM, reads their
//              D neighbours, filters by visited and leaves the survivors (at most p * D) as its distance
//              tasks of the next step.
// A newly admitted request enters with its entry points as tasks (admit kernel, before the step launch).
#include "../../include/trinity_graph.h"
#include "tri_common.h"

#include <algorithm>
#include <chrono>
#include <cstring>
#include <deque>
#include <mutex>
#include <new>
#include <vector>

namespace {

constexpr uint32_t GRING = 4;
constexpr uint32_t GX_THREADS = 256;
constexpr uint32_t GX_TEAM = 16;                 // lanes that share one distance task

struct GxMeta {          // per slot
    uint32_t k, metric;
    uint32_t state;      // 0 idle, 1 running
    uint32_t fresh;      // admitted in this step: its tasks are the entry points, no extend yet
    uint32_t iters, evals;
    uint32_t n_par;      // parents selected by this step's extend
    uint32_t n_tasks;    // distance tasks of this step
};

struct GxNewDesc {       // one admitted query in the step's upload block
    uint32_t slot, k, metric, pad_;
    uint64_t src_dev;    // GPU address of the query's vector
    uint64_t pad2_;
};

struct GxHdr {           // head of the upload block
    uint32_t n16;        // 16-byte pieces to pull (this header + the admission records)
    uint32_t n_new;
    uint32_t pad_[2];
};

// A step's result block (pinned host memory, written with plain stores only): done[S] -- set to 1 by a
// slot that finished in the step, cleared by the host before the step is enqueued -- then S records
// [n, iters, evals, 0, ids[M], score bits[M]], record s for slot s.

struct GxDev {           // everything the kernels need, by value
    const uint8_t *vecs;
    const float *vnorm;
    const uint32_t *graph;
    const uint32_t *seeds;
    uint8_t *slot_q;
    float *qnorm;
    GxMeta *meta;
    unsigned long long *topm;
    uint32_t *visited;
    uint32_t *tasks;
    uint8_t *upload;
    uint64_t n;
    uint32_t dim, dtype, row_pitch, degree, n_seeds;
    uint32_t S, M, p, T, max_iters;
    uint32_t vwords;              // visited set of a slot, in 4-byte words: one bit per row (vcap == 0), or vcap table entries
    uint32_t vcap, vprim;         // hash mode: entries of the whole table and of the small table at its head (a power of two)
    uint32_t vprim_shift;         // 32 - log2(vprim)
    uint32_t *vis_spill;          // [S] hash mode: the slot has ids in the large table (so that one must be cleared at the next admission)
    uint32_t group, ngroups;      // this launch serves the slots s with s % ngroups == group
};

__device__ __forceinline__ uint32_t gx_key(float f, uint32_t descending)
{
    uint32_t u = __float_as_uint(f);
    if (u == 0x80000000u) u = 0;
    u ^= (u >> 31) ? 0xFFFFFFFFu : 0x80000000u;
    return descending ? ~u : u;
}

__device__ __forceinline__ float gx_unkey(uint32_t key, uint32_t descending)
{
    uint32_t u = descending ? ~key : key;
    u ^= (u >> 31) ? 0x80000000u : 0xFFFFFFFFu;
    return __uint_as_float(u);
}

// Position of this thread's element among the elements of the workgroup (256 threads) whose flag is set,
// in thread order; *total = how many are set.  wave_cnt: 4 words of shared memory.  Two barriers.
__device__ __forceinline__ uint32_t gx_block_rank(bool flag, uint32_t *wave_cnt, uint32_t *total)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long m = __ballot(flag);
    __syncthreads();                          // (wave_cnt may still be read from a previous use)
    if (lane == 0) wave_cnt[wave] = (uint32_t)__popcll(m);
    __syncthreads();
    uint32_t base = 0;
    for (uint32_t w = 0; w < wave; ++w) base += wave_cnt[w];
    *total = wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
    return base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
}

__global__ void gx_pull_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src_host)
{
    const size_t n16 = ((const GxHdr *)src_host)->n16;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src_host[i];
}

// ------------------------------------------------------------------------------------------ visited
#define GX_EMPTY 0xFFFFFFFFu
#define GX_PRIMARY_PROBES 8

// True if id c enters slot s's visited set now, false if it was in it already.  Insert-only, so concurrent calls
// (also with the same id: exactly one of them gets `true`) need nothing beyond the compare-and-swap.
__device__ __forceinline__ bool gx_first_seen(const GxDev &D, uint32_t s, uint32_t c)
{
    uint32_t *tab = D.visited + (size_t)s * D.vwords;
    if (D.vcap == 0) {                                     // one bit per database row
        const uint32_t bit = 1u << (c & 31);
        return !(atomicOr(&tab[c >> 5], bit) & bit);
    }
    const uint32_t h = c * 0x9E3779B1u;
    uint32_t pos = h >> D.vprim_shift;
    for (int probe = 0; probe < GX_PRIMARY_PROBES; ++probe) {
        const uint32_t was = atomicCAS(&tab[pos], GX_EMPTY, c);
        if (was == GX_EMPTY) return true;
        if (was == c) return false;
        pos = (pos + 1) & (D.vprim - 1);
    }
    // its neighbourhood in the small table is taken (and stays taken: nothing is ever removed, so a later look-up
    // of c walks the same way): the large table, which alone has room for every id a request can see
    uint32_t *sec = tab + D.vprim;
    const uint32_t nsec = D.vcap - D.vprim;
    D.vis_spill[s] = 1u;
    uint32_t p2 = (uint32_t)(((uint64_t)((h ^ (h >> 15)) * 0x85EBCA6Bu) * nsec) >> 32);
    for (uint32_t probe = 0; probe < nsec; ++probe) {
        const uint32_t was = atomicCAS(&sec[p2], GX_EMPTY, c);
        if (was == GX_EMPTY) return true;
        if (was == c) return false;
        p2 = p2 + 1 == nsec ? 0u : p2 + 1;
    }
    return false;                                          // (not reached: nsec exceeds the ids of one request)
}

// ------------------------------------------------------------------------------------------ admit
// One workgroup per admitted query: its zero-padded row and |q|^2 into the slot, visited cleared, topM
// emptied, the entry points (first-seen only) as the slot's tasks of this step.
template <typename T>
__device__ __forceinline__ float gx_admit_row(const T *src, T *dst, uint32_t dim, uint32_t dpad)
{
    float part = 0.f;
    for (uint32_t e = threadIdx.x; e < dpad; e += GX_THREADS) {
        const T v = e < dim ? src[e] : (T)0;
        dst[e] = v;
        const float f = (float)v;
        part += f * f;
    }
    return part;
}

__global__ __launch_bounds__(GX_THREADS) void gx_admit_kernel(GxDev D)
{
    __shared__ float red[GX_THREADS];
    __shared__ uint32_t wave_cnt[4];
    const GxHdr *hdr = (const GxHdr *)D.upload;
    if (blockIdx.x >= hdr->n_new) return;
    const GxNewDesc d = ((const GxNewDesc *)(D.upload + sizeof(GxHdr)))[blockIdx.x];
    const uint32_t s = d.slot, tid = threadIdx.x;
    uint8_t *qrow = D.slot_q + (size_t)s * D.row_pitch;
    red[tid] = D.dtype == TRI_F16
                   ? gx_admit_row<_Float16>((const _Float16 *)d.src_dev, (_Float16 *)qrow, D.dim, D.row_pitch / 2)
                   : gx_admit_row<float>((const float *)d.src_dev, (float *)qrow, D.dim, D.row_pitch / 4);
    uint4 *vis = (uint4 *)(D.visited + (size_t)s * D.vwords);
    if (D.vcap == 0) {
        for (uint32_t i = tid; i < D.vwords / 4; i += GX_THREADS) vis[i] = make_uint4(0u, 0u, 0u, 0u);
    } else {
        // the small table always; the large one only if the slot's previous request reached it
        const uint32_t clear = D.vis_spill[s] ? D.vcap : D.vprim;
        for (uint32_t i = tid; i < clear / 4; i += GX_THREADS) vis[i] = make_uint4(GX_EMPTY, GX_EMPTY, GX_EMPTY, GX_EMPTY);
        __syncthreads();                                           // (every thread has read the mark)
        if (tid == 0) D.vis_spill[s] = 0u;
    }
    for (uint32_t i = tid; i < D.M; i += GX_THREADS) D.topm[(size_t)s * D.M + i] = ~0ull;
    __syncthreads();
    for (uint32_t w = GX_THREADS / 2; w > 0; w >>= 1) {
        if (tid < w) red[tid] += red[tid + w];
        __syncthreads();
    }
    // entry points: thread j takes seed j (n_seeds <= 256)
    uint32_t v = TRI_GRAPH_PAD;
    if (tid < D.n_seeds) {
        const uint32_t c = D.seeds[tid];
        if (c < D.n && gx_first_seen(D, s, c)) v = c;
    }
    uint32_t total;
    const uint32_t pos = gx_block_rank(v != TRI_GRAPH_PAD, wave_cnt, &total);
    if (v != TRI_GRAPH_PAD) D.tasks[(size_t)s * D.T + pos] = v;
    if (tid == 0) {
        D.qnorm[s] = red[0];
        D.meta[s] = GxMeta{d.k, d.metric, 1u, 1u, 0u, total, 0u, total};
    }
}

// ------------------------------------------------------------------------------------------ distance
// One workgroup per slot, the slot's query row in LDS; a team of 16 lanes per task reads the task's row
// in 256-byte pieces (16 bytes per lane, consecutive lanes consecutive addresses: two full 128-byte
// lines per piece) and reduces its dot product in a fixed order, so a score does not depend on which
// other tasks share the launch.  L2 = |x|^2 + |q|^2 - 2 x.q with the stored |x|^2.
// NCH = 256-byte pieces per row when known at compile time (all loads of a row in flight together), 0 = any.
template <int DT>
__device__ __forceinline__ float gx_dot16(const uint4 &x, const uint4 &q, float acc)
{
    if (DT == TRI_F16) {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        const h2 *a = (const h2 *)&x, *b = (const h2 *)&q;
#pragma unroll
        for (int i = 0; i < 4; ++i) acc = __builtin_amdgcn_fdot2(a[i], b[i], acc, false);
    } else {
        const float *a = (const float *)&x, *b = (const float *)&q;
#pragma unroll
        for (int i = 0; i < 4; ++i) acc = fmaf(a[i], b[i], acc);
    }
    return acc;
}

// acc + sum of (x - q)^2 over one 16-byte piece, in fp32
template <int DT>
__device__ __forceinline__ float gx_diff16(const uint4 &x, const uint4 &q, float acc)
{
    if (DT == TRI_F16) {
        const _Float16 *a = (const _Float16 *)&x, *b = (const _Float16 *)&q;
#pragma unroll
        for (int i = 0; i < 8; ++i) { const float d = (float)a[i] - (float)b[i]; acc = fmaf(d, d, acc); }
    } else {
        const float *a = (const float *)&x, *b = (const float *)&q;
#pragma unroll
        for (int i = 0; i < 4; ++i) { const float d = a[i] - b[i]; acc = fmaf(d, d, acc); }
    }
    return acc;
}

extern __shared__ __attribute__((aligned(16))) uint8_t gx_q[];   // the slot's query row

template <int DT, int NCH>
__device__ __forceinline__ void gx_distance_phase(const GxDev &D, uint32_t s, const GxMeta &m, float *__restrict__ sdist)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t pieces = D.row_pitch / 16;
    for (uint32_t i = tid; i < pieces; i += GX_THREADS)
        ((uint4 *)gx_q)[i] = ((const uint4 *)(D.slot_q + (size_t)s * D.row_pitch))[i];
    __syncthreads();
    const uint32_t team = tid / GX_TEAM, c = tid % GX_TEAM;
    const float qn = D.qnorm[s];
    const uint32_t nch = NCH ? (uint32_t)NCH : D.row_pitch / 256;
    for (uint32_t t = team; t < m.n_tasks; t += GX_THREADS / GX_TEAM) {
        const uint32_t id = D.tasks[(size_t)s * D.T + t];
        const uint4 *row = (const uint4 *)(D.vecs + (size_t)id * D.row_pitch);
        float acc = 0.f;
        if (NCH) {
            uint4 x[NCH ? NCH : 1];
#pragma unroll
            for (int i = 0; i < NCH; ++i) x[i] = row[c + i * GX_TEAM];
#pragma unroll
            for (int i = 0; i < NCH; ++i) acc = gx_dot16<DT>(x[i], ((const uint4 *)gx_q)[c + i * GX_TEAM], acc);
        } else {
            for (uint32_t i = 0; i < nch; ++i) acc = gx_dot16<DT>(row[c + i * GX_TEAM], ((const uint4 *)gx_q)[c + i * GX_TEAM], acc);
        }
#pragma unroll
        for (int d = GX_TEAM / 2; d > 0; d >>= 1) acc += __shfl_xor(acc, d, GX_TEAM);
        if (c == 0) sdist[t] = m.metric == TRI_L2 ? (D.vnorm[id] + qn) - 2.0f * acc : acc;
    }
}

// ------------------------------------------------------------------------------------------ merge + extend
// One workgroup per slot.
//  merge : the step's (score, id) pairs join topM.  Elements are composites (key << 32 | id << 1 | expanded;
//          ids are unique: a row is scored at most once per request).  topM is sorted already, so only the
//          new pairs are sorted (rank counting among themselves); the final rank of a new pair is its rank
//          among the new ones plus the number of topM entries below it (binary search), that of a topM
//          entry its index plus the number of new pairs below it.  The first M form the new topM; it
//          changed iff a new pair ranks among them.
//  stop  : by the paper's rule (topM unchanged), the extend budget, or no parent left.
//  extend: a request that goes on selects its next parents at once -- thread i looks at entry i of the new
//          topM: the first p non-expanded ones (in topM's order) become parents and are marked; thread t
//          takes neighbour t % D of parent t / D through the visited filter; the survivors, compacted, are
//          the slot's distance tasks of the next step.
//  result: the first k entries of topM.  The search ranks squared L2 in the expanded form |x|^2 + |q|^2 - 2 x.q
//          (one contraction per row); what is handed back is the difference form: the k rows of a finishing
//          L2 request are read once more, scored as sum (x - q)^2 and put in the order of (that, id), so a
//          stored copy of the query comes back with distance exactly zero.
__device__ __forceinline__ uint32_t gx_count_below(const unsigned long long *a, uint32_t n, unsigned long long x)
{
    uint32_t lo = 0, hi = n;                 // a ascending: number of entries < x
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (a[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo;
}

template <int DT>
__device__ __forceinline__ void gx_merge_extend_phase(const GxDev &D, uint32_t s, GxMeta *mp, const GxMeta &m,
                                                      const float *__restrict__ sdist, unsigned long long old_e,
                                                      uint32_t task_id, uint32_t *__restrict__ done,
                                                      uint32_t *__restrict__ rec_base, uint32_t rec_words)
{
    __shared__ unsigned long long old[TRI_GRAPH_TOPM_LIMIT];
    __shared__ unsigned long long nw[TRI_GRAPH_TASK_LIMIT];
    __shared__ unsigned long long snew[TRI_GRAPH_TASK_LIMIT];
    __shared__ unsigned long long out[TRI_GRAPH_TOPM_LIMIT];
    __shared__ uint32_t parent[TRI_GRAPH_TASK_LIMIT];
    __shared__ uint32_t wave_cnt[4];
    __shared__ uint32_t changed, n_sh;
    const uint32_t tid = threadIdx.x;
    const uint32_t desc = m.metric == TRI_IP;
    const uint32_t nt = m.n_tasks, M = D.M;
    if (tid == 0) { changed = 0; n_sh = 0; }
    unsigned long long mine = ~0ull;                              // this thread's new pair (T <= 256 = threads)
    if (tid < nt)
        mine = ((unsigned long long)gx_key(sdist[tid], desc) << 32) | ((unsigned long long)task_id << 1);
    nw[tid] = mine;
    if (tid < M) { old[tid] = old_e; out[tid] = ~0ull; }
    __syncthreads();
    uint32_t r_new = 0;
    if (tid < nt)
        for (uint32_t j = 0; j < nt; ++j) r_new += nw[j] < mine;
    if (tid < nt) snew[r_new] = mine;
    __syncthreads();
    if (tid < nt) {
        const uint32_t r = r_new + gx_count_below(old, M, mine);
        if (r < M) { out[r] = mine; changed = 1u; }               // (benign race: every writer stores 1)
    }
    if (tid < M) {
        const unsigned long long e = old[tid];
        if (e != ~0ull) {                                          // empty entries stay at the end
            const uint32_t r = tid + gx_count_below(snew, nt, e);
            if (r < M) out[r] = e;
        }
    }
    __syncthreads();
    // stop rule
    bool finish;
    uint32_t iters = m.iters;
    if (m.fresh) finish = D.max_iters == 0;
    else {
        iters += 1;                                                // (a running slot reaches this kernel only with parents)
        finish = !changed || iters >= D.max_iters;
    }
    uint32_t n_par = 0, n_tasks = 0;
    if (!finish) {
        const unsigned long long e = tid < M ? out[tid] : ~0ull;
        const bool unexp = e != ~0ull && !(e & 1ull);
        uint32_t total;
        const uint32_t rank = gx_block_rank(unexp, wave_cnt, &total);
        if (unexp && rank < D.p) {
            parent[rank] = (uint32_t)(e & 0xFFFFFFFFull) >> 1;
            out[tid] = e | 1ull;
        }
        n_par = total < D.p ? total : D.p;
        if (n_par == 0) finish = true;                             // nothing left to expand: not an extend
        __syncthreads();
    }
    if (!finish) {
        uint32_t v = TRI_GRAPH_PAD;
        const uint32_t par = tid / D.degree, j = tid % D.degree;
        if (par < n_par) {
            const uint32_t c = D.graph[(size_t)parent[par] * D.degree + j];
            if (c < D.n && gx_first_seen(D, s, c)) v = c;
        }
        const uint32_t pos = gx_block_rank(v != TRI_GRAPH_PAD, wave_cnt, &n_tasks);
        if (v != TRI_GRAPH_PAD) D.tasks[(size_t)s * D.T + pos] = v;
    }
    if (tid < M) D.topm[(size_t)s * M + tid] = out[tid];
    if (finish) {
        uint32_t *rec = rec_base + (size_t)s * rec_words;
        uint32_t n_valid = 0;
        if (m.metric == TRI_L2) {
            const uint32_t kk = m.k < M ? m.k : M;
            float *d2 = (float *)nw;                               // (nw and snew were last read before the barrier above)
            const uint32_t team = tid / GX_TEAM, c = tid % GX_TEAM, pieces = D.row_pitch / 16;
            const uint4 *q = (const uint4 *)(D.slot_q + (size_t)s * D.row_pitch);
            for (uint32_t i = team; i < kk; i += GX_THREADS / GX_TEAM) {
                const unsigned long long e = out[i];
                float acc = 0.f;
                if (e != ~0ull) {
                    const uint4 *row = (const uint4 *)(D.vecs + (size_t)((uint32_t)(e & 0xFFFFFFFFull) >> 1) * D.row_pitch);
                    for (uint32_t j = c; j < pieces; j += GX_TEAM) acc = gx_diff16<DT>(row[j], q[j], acc);
                }
#pragma unroll
                for (int d = GX_TEAM / 2; d > 0; d >>= 1) acc += __shfl_xor(acc, d, GX_TEAM);
                if (c == 0) d2[i] = acc;
            }
            __syncthreads();
            if (tid < M) {
                const unsigned long long e = out[tid];
                const bool ok = e != ~0ull && tid < kk;
                uint32_t at = tid;                                 // (empty entries stand behind the valid ones)
                if (ok) {
                    const uint32_t id = (uint32_t)(e & 0xFFFFFFFFull) >> 1;
                    const unsigned long long mine2 = ((unsigned long long)__float_as_uint(d2[tid]) << 32) | id;
                    at = 0;
                    for (uint32_t j = 0; j < kk; ++j) {
                        const unsigned long long o = out[j];
                        if (o == ~0ull) break;
                        at += (((unsigned long long)__float_as_uint(d2[j]) << 32) | ((uint32_t)(o & 0xFFFFFFFFull) >> 1)) < mine2;
                    }
                    rec[4 + at] = id;
                    rec[4 + M + at] = __float_as_uint(d2[tid]);
                } else {
                    rec[4 + at] = 0xFFFFFFFFu;
                    rec[4 + M + at] = 0u;
                }
                n_valid = ok;
            }
        } else if (tid < M) {
            const unsigned long long e = out[tid];
            const bool ok = e != ~0ull && tid < m.k;
            rec[4 + tid] = ok ? (uint32_t)(e & 0xFFFFFFFFull) >> 1 : 0xFFFFFFFFu;
            rec[4 + M + tid] = ok ? __float_as_uint(gx_unkey((uint32_t)(e >> 32), desc)) : 0u;
            n_valid = ok;
        }
        if (n_valid) atomicAdd(&n_sh, n_valid);                   // n = valid entries among the first k
        __syncthreads();
        if (tid == 0) {
            rec[0] = n_sh; rec[1] = iters; rec[2] = m.evals; rec[3] = 0u;
            mp->state = 0u;
            done[s] = 1u;                                          // (the host looks only after the step has completed)
        }
    } else if (tid == 0) {
        mp->iters = iters;
        mp->fresh = 0u;
        mp->n_par = n_par;
        mp->n_tasks = n_tasks;
        mp->evals = m.evals + n_tasks;
    }
}

// ------------------------------------------------------------------------------------------ the step
// One workgroup per slot runs the slot's whole step: distances of its tasks, merge, stop rule, next
// extend.  Slots are independent of each other, so while one workgroup is in its latency-bound merge and
// extend the others on the same compute unit keep the memory system busy with their row reads: the step
// costs about what its row traffic costs, not the sum of its phases.
template <int DT, int NCH>
__global__ __launch_bounds__(GX_THREADS) void gx_step_kernel(GxDev D, uint32_t *__restrict__ done,
                                                             uint32_t *__restrict__ rec_base, uint32_t rec_words)
{
    __shared__ float sdist[TRI_GRAPH_TASK_LIMIT];
    const uint32_t s = blockIdx.x * D.ngroups + D.group;
    if (s >= D.S) return;
    GxMeta *mp = D.meta + s;
    const GxMeta m = *mp;
    if (m.state != 1u) return;                                    // (idle slot: masked)
    // what the merge needs from memory is asked for now and arrives while the rows are being read
    const unsigned long long old_e = threadIdx.x < D.M ? D.topm[(size_t)s * D.M + threadIdx.x] : ~0ull;
    const uint32_t task_id = threadIdx.x < m.n_tasks ? D.tasks[(size_t)s * D.T + threadIdx.x] : TRI_GRAPH_PAD;
    if (m.n_tasks) gx_distance_phase<DT, NCH>(D, s, m, sdist);
    __syncthreads();
    gx_merge_extend_phase<DT>(D, s, mp, m, sdist, old_e, task_id, done, rec_base, rec_words);
}

// ================================================================================== host side
inline int64_t gnow_ns()
{
    return std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now().time_since_epoch()).count();
}
inline size_t gup(size_t v, size_t m) { return (v + m - 1) / m * m; }

enum GState : uint8_t { G_FREE = 0, G_PENDING, G_RUNNING, G_DONE };

struct GTicket {
    uint32_t gen = 0;
    GState state = G_FREE;
    uint32_t k = 0, metric = 0, klass = 0, slot = 0;
    const void *dev_vec = nullptr;
    uint32_t n_out = 0, iters = 0, evals = 0;
};

struct GStep {
    bool in_use = false;
    bool profiled = false;
    uint64_t seq = 0;
    hipEvent_t done = nullptr, ev0 = nullptr, ev1 = nullptr;
    uint8_t *up_host = nullptr, *up_dev = nullptr;
    uint8_t *down_host = nullptr, *down_dev = nullptr;
    hipStream_t stream = nullptr;     // the group's stream (group 0: the caller's)
    bool own_stream = false;
    uint8_t *upload = nullptr;        // the group's device copy of the upload block
    std::vector<uint32_t> free_slots;
    uint32_t n_running = 0;
};

#define GHIP(expr)                                                                                   \
    do {                                                                                             \
        hipError_t e_ = (expr);                                                                      \
        if (e_ != hipSuccess) return tri_fail(TRI_EHIP, "%s -> %s", #expr, hipGetErrorString(e_));   \
    } while (0)

}  // namespace

struct tri_gpool {
    tri_graph_cfg cfg{};
    int device = 0;
    hipStream_t stream = nullptr;
    std::mutex mu;
    GxDev D{};
    uint32_t ngroups = 2, rec_words = 0;
    size_t up_bytes = 0, down_bytes = 0;
    uint8_t *pinned = nullptr, *qstore = nullptr, *qstore_dev = nullptr;
    std::vector<GTicket> tickets;
    std::vector<uint32_t> free_tickets, slot_ticket;
    std::vector<uint32_t> res_ids;
    std::vector<float> res_score;
    std::deque<uint32_t> pending[2];
    uint32_t n_running = 0;
    uint64_t step_seq = 0;
    GStep ring[GRING];
    tri_graph_times times{};
    // graph_run_stream: finished results go straight to the caller's arrays
    struct Sink {
        std::vector<uint32_t> q_of_ticket;
        uint32_t *n_out; int64_t *ids; float *dist; double *done_s;
        uint32_t stride; int64_t t0_ns; uint32_t delivered;
    } *sink = nullptr;
    bool static_batches = false;      // admit into a group of slots only when the whole group is idle
};

namespace {

struct GLayout {
    size_t vecs, vnorm, graph, seeds, slot_q, qnorm, meta, topm, visited, vis_spill, tasks, upload, upload_one, total;
    uint32_t row_pitch, vwords, vcap, vprim, T;
};

int g_validate(const tri_graph_cfg *c, uint64_t n, uint32_t dim, uint32_t degree, uint32_t dtype)
{
    if (!c) return tri_fail(TRI_EINVAL, "cfg is NULL");
    if (c->slots == 0 || c->slots > (1u << 16)) return tri_fail(TRI_EINVAL, "slots must be 1..65536");
    if (c->topm == 0 || c->topm > TRI_GRAPH_TOPM_LIMIT) return tri_fail(TRI_EINVAL, "topm must be 1..%u", TRI_GRAPH_TOPM_LIMIT);
    if (degree == 0 || c->parents == 0 || (uint64_t)c->parents * degree > TRI_GRAPH_TASK_LIMIT)
        return tri_fail(TRI_EINVAL, "need parents >= 1, degree >= 1 and parents * degree <= %u", TRI_GRAPH_TASK_LIMIT);
    if (c->max_outstanding < c->slots) return tri_fail(TRI_EINVAL, "max_outstanding must be >= slots");
    if (c->groups > GRING) return tri_fail(TRI_EINVAL, "groups must be 0..%u", GRING);
    if ((c->flags & TRI_GRAPH_VISITED_HASH) && (c->flags & TRI_GRAPH_VISITED_BITS))
        return tri_fail(TRI_EINVAL, "TRI_GRAPH_VISITED_HASH and TRI_GRAPH_VISITED_BITS exclude each other");
    if ((uint64_t)c->max_iters * c->parents * degree >= (1ull << 29))
        return tri_fail(TRI_EINVAL, "max_iters * parents * degree must stay below 2^29");
    if (n == 0 || n >= (1ull << 31)) return tri_fail(TRI_EINVAL, "n must be 1..2^31-1");
    if (dtype != TRI_F32 && dtype != TRI_F16) return tri_fail(TRI_EINVAL, "dtype must be TRI_F32 or TRI_F16");
    if (dim == 0 || gup((size_t)dim * (dtype == TRI_F16 ? 2 : 4), 256) > TRI_MAX_ROW_BYTES)
        return tri_fail(TRI_EINVAL, "dim out of range: a padded row may have at most %u bytes", TRI_MAX_ROW_BYTES);
    return TRI_OK;
}

GLayout g_layout(const tri_graph_cfg &c, uint64_t n, uint32_t dim, uint32_t degree, uint32_t dtype)
{
    GLayout L{};
    L.row_pitch = (uint32_t)gup((size_t)dim * (dtype == TRI_F16 ? 2 : 4), 256);
    // visited set of a slot: a hash table in two parts -- a small one in front (a power of two of at least a quarter
    // of the ids one request can ever see: its entry points and max_iters extends of p * D neighbours, never more than
    // n), which takes what a typical request sees, and a large one behind it with room for ALL of those ids at a load
    // of 0.8 -- or one bit per row where that is smaller (or asked for)
    const uint32_t bit_words = (uint32_t)gup((n + 31) / 32, 4);
    const uint64_t ids_seen = std::min<uint64_t>(n, (uint64_t)TRI_GRAPH_TASK_LIMIT + (uint64_t)c.max_iters * c.parents * degree);
    uint64_t prim = 256;
    while (prim * 4 < ids_seen) prim <<= 1;
    const uint64_t cap = prim + gup(ids_seen + ids_seen / 4 + 4, 4);
    const bool hash = (c.flags & TRI_GRAPH_VISITED_HASH) || (!(c.flags & TRI_GRAPH_VISITED_BITS) && cap < bit_words);
    L.vcap = hash ? (uint32_t)cap : 0u;
    L.vprim = hash ? (uint32_t)prim : 0u;
    L.vwords = hash ? L.vcap : bit_words;
    L.T = TRI_GRAPH_TASK_LIMIT;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = gup(o + bytes, 256); return at; };
    const size_t S = c.slots;
    L.vecs = take(n * L.row_pitch);
    L.vnorm = take(n * 4);
    L.graph = take(n * degree * 4);
    L.seeds = take(TRI_GRAPH_TASK_LIMIT * 4);
    L.slot_q = take(S * L.row_pitch);
    L.qnorm = take(S * 4);
    L.meta = take(S * sizeof(GxMeta));
    L.topm = take(S * c.topm * 8);
    L.visited = take(S * (size_t)L.vwords * 4);
    L.vis_spill = take(S * 4);
    L.tasks = take(S * L.T * 4);
    L.upload_one = gup(sizeof(GxHdr) + S * sizeof(GxNewDesc), 256);
    L.upload = take(L.upload_one * GRING);
    L.total = o;
    return L;
}

// Collect the records of completed steps, oldest first.  block: wait for all of them.
int g_reap(tri_gpool *P, bool block, uint32_t *finished)
{
    for (uint32_t it = 0; it < GRING; ++it) {
        GStep *R = nullptr;
        for (uint32_t i = 0; i < GRING; ++i)
            if (P->ring[i].in_use && (!R || P->ring[i].seq < R->seq)) R = &P->ring[i];
        if (!R) break;
        if (block) {
            GHIP(hipEventSynchronize(R->done));
        } else {
            const hipError_t q = hipEventQuery(R->done);
            if (q == hipErrorNotReady) break;
            if (q != hipSuccess) return tri_fail(TRI_EHIP, "hipEventQuery -> %s", hipGetErrorString(q));
        }
        const uint32_t *done = (const uint32_t *)R->down_host;
        const uint32_t *recs = done + P->cfg.slots;
        const uint32_t M = P->cfg.topm;
        uint64_t tasks = 0;
        for (uint32_t slot = 0; slot < P->cfg.slots; ++slot) {
            if (!done[slot]) continue;
            const uint32_t *rec = recs + (size_t)slot * P->rec_words;
            const uint32_t ti = P->slot_ticket[slot];
            GTicket &t = P->tickets[ti];
            t.n_out = rec[0]; t.iters = rec[1]; t.evals = rec[2];
            tasks += t.evals;
            if (P->sink) {
                tri_gpool::Sink &K = *P->sink;
                const uint32_t qi = K.q_of_ticket[ti];
                int64_t *oi = K.ids + (size_t)qi * K.stride;
                float *od = K.dist + (size_t)qi * K.stride;
                for (uint32_t j = 0; j < t.n_out; ++j) { oi[j] = (int64_t)rec[4 + j]; od[j] = __builtin_bit_cast(float, rec[4 + M + j]); }
                const float pad = t.metric == TRI_L2 ? __builtin_inff() : -__builtin_inff();
                for (uint32_t j = t.n_out; j < t.k; ++j) { oi[j] = -1; od[j] = pad; }
                K.n_out[qi] = t.n_out;
                K.done_s[qi] = (double)(gnow_ns() - K.t0_ns) * 1e-9;
                ++K.delivered;
                t.state = G_FREE;
                ++t.gen;
                P->free_tickets.push_back(ti);
            } else {
                memcpy(&P->res_ids[(size_t)ti * M], rec + 4, (size_t)t.n_out * 4);
                memcpy(&P->res_score[(size_t)ti * M], rec + 4 + M, (size_t)t.n_out * 4);
                t.state = G_DONE;
            }
            R->free_slots.push_back(slot);
            --R->n_running;
            --P->n_running;
            if (finished) ++*finished;
        }
        if (R->profiled) {
            float ms = 0.f;
            GHIP(hipEventElapsedTime(&ms, R->ev0, R->ev1));
            P->times.steps += 1;
            P->times.step_kernel_ms += ms;
            P->times.tasks += tasks;        // (tasks of the requests that finished in the step: over a run from idle
                                            //  to idle this adds up to every task scored)
        }
        R->in_use = false;
    }
    return TRI_OK;
}

template <int DT>
hipError_t g_launch_step(const GxDev &D, uint32_t nblocks, hipStream_t stream, uint32_t *done, uint32_t *rec_base,
                         uint32_t rec_words)
{
    const dim3 grid(nblocks), block(GX_THREADS);
    const size_t lds = D.row_pitch;
    switch (D.row_pitch / 256) {
    case 2: hipLaunchKernelGGL((gx_step_kernel<DT, 2>), grid, block, lds, stream, D, done, rec_base, rec_words); break;
    case 6: hipLaunchKernelGGL((gx_step_kernel<DT, 6>), grid, block, lds, stream, D, done, rec_base, rec_words); break;
    default: hipLaunchKernelGGL((gx_step_kernel<DT, 0>), grid, block, lds, stream, D, done, rec_base, rec_words); break;
    }
    return hipGetLastError();
}

}  // namespace

extern "C" int graph_pool_bytes(const tri_graph_cfg *cfg, uint64_t n, uint32_t dim, uint32_t degree, uint32_t dtype,
                                size_t *dev_bytes)
{
    const int rc = g_validate(cfg, n, dim, degree, dtype);
    if (rc) return rc;
    if (!dev_bytes) return tri_fail(TRI_EINVAL, "dev_bytes is NULL");
    *dev_bytes = g_layout(*cfg, n, dim, degree, dtype).total;
    return TRI_OK;
}

// |x|^2 of every stored row (fixed order per row: lane-strided partial sums, then a tree).
__global__ void gx_row_norm_kernel(const uint8_t *__restrict__ vecs, uint32_t row_pitch, uint32_t dtype, uint64_t n,
                                   float *__restrict__ out)
{
    const uint64_t row = (uint64_t)blockIdx.x * (blockDim.x / 64) + threadIdx.x / 64;
    if (row >= n) return;
    const uint32_t lane = threadIdx.x & 63;
    float acc = 0.f;
    if (dtype == TRI_F16) {
        const _Float16 *r = (const _Float16 *)(vecs + row * row_pitch);
        for (uint32_t e = lane; e < row_pitch / 2; e += 64) { const float f = (float)r[e]; acc += f * f; }
    } else {
        const float *r = (const float *)(vecs + row * row_pitch);
        for (uint32_t e = lane; e < row_pitch / 4; e += 64) acc += r[e] * r[e];
    }
    for (int d = 32; d > 0; d >>= 1) acc += __shfl_xor(acc, d, 64);
    if (lane == 0) out[row] = acc;
}

extern "C" int graph_pool_create(const tri_graph_cfg *cfg, const void *vectors, const uint32_t *neighbors, uint64_t n,
                                 uint32_t dim, uint32_t degree, uint32_t dtype, const uint32_t *seeds, uint32_t n_seeds,
                                 void *dev_mem, size_t dev_bytes, tri_gpool **out)
{
    int rc = g_validate(cfg, n, dim, degree, dtype);
    if (rc) return rc;
    if (!vectors || !neighbors || !dev_mem || !out || (!seeds && n_seeds)) return tri_fail(TRI_EINVAL, "NULL argument");
    if (n_seeds == 0 || n_seeds > TRI_GRAPH_TASK_LIMIT) return tri_fail(TRI_EINVAL, "n_seeds must be 1..%u", TRI_GRAPH_TASK_LIMIT);
    if ((uintptr_t)dev_mem % 256) return tri_fail(TRI_EINVAL, "dev_mem must be 256-byte aligned");
    const GLayout L = g_layout(*cfg, n, dim, degree, dtype);
    if (dev_bytes < L.total) return tri_fail(TRI_ENOMEM, "dev_mem has %zu bytes, %zu needed", dev_bytes, L.total);
    tri_gpool *P = new (std::nothrow) tri_gpool();
    if (!P) return tri_fail(TRI_ENOMEM, "out of host memory");
    P->cfg = *cfg;
    P->ngroups = std::min<uint32_t>(cfg->groups ? cfg->groups : 2u, cfg->slots);
    P->stream = (hipStream_t)cfg->hip_stream;
    hipError_t e = hipGetDevice(&P->device);
    if (e != hipSuccess) { delete P; return tri_fail(TRI_EHIP, "hipGetDevice -> %s", hipGetErrorString(e)); }
    uint8_t *base = (uint8_t *)dev_mem;
    GxDev &D = P->D;
    D.vecs = base + L.vecs; D.vnorm = (float *)(base + L.vnorm); D.graph = (uint32_t *)(base + L.graph);
    D.seeds = (uint32_t *)(base + L.seeds); D.slot_q = base + L.slot_q; D.qnorm = (float *)(base + L.qnorm);
    D.meta = (GxMeta *)(base + L.meta); D.topm = (unsigned long long *)(base + L.topm);
    D.visited = (uint32_t *)(base + L.visited); D.tasks = (uint32_t *)(base + L.tasks);
    D.upload = base + L.upload;
    D.group = 0; D.ngroups = P->ngroups;
    D.n = n; D.dim = dim; D.dtype = dtype; D.row_pitch = L.row_pitch; D.degree = degree; D.n_seeds = n_seeds;
    D.S = cfg->slots; D.M = cfg->topm; D.p = cfg->parents; D.T = L.T; D.vwords = L.vwords; D.max_iters = cfg->max_iters;
    D.vcap = L.vcap; D.vprim = L.vprim; D.vis_spill = (uint32_t *)(base + L.vis_spill);
    D.vprim_shift = 32;
    for (uint32_t v = L.vprim; v > 1; v >>= 1) --D.vprim_shift;
    // index data: rows padded with zeros, neighbour list, entry points, row norms, idle slots
    const size_t es = dtype == TRI_F16 ? 2 : 4;
    hipStream_t s = P->stream;
    e = hipMemsetAsync(base + L.vecs, 0, n * L.row_pitch, s);
    if (e == hipSuccess) e = hipMemcpy2DAsync(base + L.vecs, L.row_pitch, vectors, (size_t)dim * es, (size_t)dim * es, n, hipMemcpyDefault, s);
    if (e == hipSuccess) e = hipMemcpyAsync(base + L.graph, neighbors, n * degree * 4, hipMemcpyDefault, s);
    if (e == hipSuccess) e = hipMemcpyAsync(base + L.seeds, seeds, (size_t)n_seeds * 4, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipMemsetAsync(base + L.meta, 0, (size_t)cfg->slots * sizeof(GxMeta), s);
    if (e == hipSuccess) e = hipMemsetAsync(base + L.vis_spill, 0, (size_t)cfg->slots * 4, s);
    if (e == hipSuccess && L.vcap)      // (hash tables start empty; an admission clears only what its slot's previous request used)
        e = hipMemsetAsync(base + L.visited, 0xFF, (size_t)cfg->slots * L.vwords * 4, s);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(gx_row_norm_kernel, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, s, D.vecs, D.row_pitch, dtype, n,
                           (float *)(base + L.vnorm));
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) { delete P; return tri_fail(TRI_EHIP, "index upload -> %s", hipGetErrorString(e)); }
    // pinned blocks
    P->rec_words = 4 + 2 * cfg->topm;
    P->up_bytes = gup(sizeof(GxHdr) + (size_t)cfg->slots * sizeof(GxNewDesc), 256);
    P->down_bytes = gup((size_t)cfg->slots * 4 + (size_t)cfg->slots * P->rec_words * 4, 256);
    const size_t per = P->up_bytes + P->down_bytes;
    e = hipHostMalloc((void **)&P->pinned, per * GRING, hipHostMallocDefault);
    if (e == hipSuccess) e = hipHostMalloc((void **)&P->qstore, (size_t)cfg->max_outstanding * L.row_pitch, hipHostMallocDefault);
    if (e == hipSuccess) e = hipHostGetDevicePointer((void **)&P->qstore_dev, P->qstore, 0);
    for (uint32_t i = 0; i < GRING && e == hipSuccess; ++i) {
        GStep &R = P->ring[i];
        R.up_host = P->pinned + i * per;
        R.down_host = R.up_host + P->up_bytes;
        e = hipHostGetDevicePointer((void **)&R.up_dev, R.up_host, 0);
        if (e == hipSuccess) e = hipHostGetDevicePointer((void **)&R.down_dev, R.down_host, 0);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&R.done, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&R.ev0, hipEventDisableSystemFence);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&R.ev1, hipEventDisableSystemFence);
        R.upload = base + L.upload + i * L.upload_one;
        R.stream = P->stream;
        if (i > 0 && i < P->ngroups && e == hipSuccess) {        // (default priority, like the caller's stream)
            e = hipStreamCreateWithFlags(&R.stream, hipStreamNonBlocking);
            R.own_stream = e == hipSuccess;
        }
    }
    if (e != hipSuccess) { graph_pool_destroy(P); return tri_fail(TRI_EHIP, "pinned memory / events -> %s", hipGetErrorString(e)); }
    try {
        P->tickets.resize(cfg->max_outstanding);
        for (uint32_t i = cfg->max_outstanding; i-- > 0;) P->free_tickets.push_back(i);
        for (uint32_t i = cfg->slots; i-- > 0;) P->ring[i % P->ngroups].free_slots.push_back(i);
        P->slot_ticket.assign(cfg->slots, 0);
        P->res_ids.resize((size_t)cfg->max_outstanding * cfg->topm);
        P->res_score.resize((size_t)cfg->max_outstanding * cfg->topm);
    } catch (const std::bad_alloc &) {
        graph_pool_destroy(P);
        return tri_fail(TRI_ENOMEM, "out of host memory");
    }
    P->times.row_bytes = L.row_pitch;
    *out = P;
    return TRI_OK;
}

extern "C" int graph_pool_destroy(tri_gpool *P)
{
    if (!P) return tri_fail(TRI_EINVAL, "pool is NULL");
    (void)hipStreamSynchronize(P->stream);
    for (uint32_t i = 0; i < GRING; ++i) {
        if (P->ring[i].own_stream) { (void)hipStreamSynchronize(P->ring[i].stream); (void)hipStreamDestroy(P->ring[i].stream); }
        if (P->ring[i].done) (void)hipEventDestroy(P->ring[i].done);
        if (P->ring[i].ev0) (void)hipEventDestroy(P->ring[i].ev0);
        if (P->ring[i].ev1) (void)hipEventDestroy(P->ring[i].ev1);
    }
    if (P->pinned) (void)hipHostFree(P->pinned);
    if (P->qstore) (void)hipHostFree(P->qstore);
    delete P;
    return TRI_OK;
}

extern "C" int graph_submit(tri_gpool *P, const void *vecs, int on_device, uint64_t pitch_bytes, uint32_t n,
                            const uint32_t *k, const uint32_t *metric, const uint32_t *klass, tri_ticket *out, uint32_t *n_done)
{
    if (n_done) *n_done = 0;
    if (!P || (n && (!vecs || !k || !metric || !out))) return tri_fail(TRI_EINVAL, "NULL argument");
    if (n == 0) return TRI_OK;
    const size_t es = P->D.dtype == TRI_F16 ? 2 : 4;
    if (pitch_bytes < (uint64_t)P->D.dim * es || pitch_bytes % es) return tri_fail(TRI_EINVAL, "pitch_bytes too small or not a multiple of the element size");
    for (uint32_t i = 0; i < n; ++i) {
        if (k[i] == 0 || k[i] > P->cfg.topm) return tri_fail(TRI_EINVAL, "k must be 1..topm (query %u has %u)", i, k[i]);
        if (metric[i] != TRI_L2 && metric[i] != TRI_IP) return tri_fail(TRI_EINVAL, "metric must be TRI_L2 or TRI_IP");
        if (klass && klass[i] != TRI_CLASS_HIGH && klass[i] != TRI_CLASS_LOW) return tri_fail(TRI_EINVAL, "klass must be TRI_CLASS_HIGH or TRI_CLASS_LOW");
    }
    std::lock_guard<std::mutex> lk(P->mu);
    for (uint32_t i = 0; i < n; ++i) {
        if (P->free_tickets.empty()) return tri_fail(TRI_EAGAIN, "max_outstanding=%u tickets alive", P->cfg.max_outstanding);
        const uint32_t ti = P->free_tickets.back();
        P->free_tickets.pop_back();
        GTicket &t = P->tickets[ti];
        t.state = G_PENDING;
        t.k = k[i]; t.metric = metric[i]; t.klass = klass ? klass[i] : (uint32_t)TRI_CLASS_LOW;
        const uint8_t *src = (const uint8_t *)vecs + (size_t)i * pitch_bytes;
        if (on_device) {
            t.dev_vec = src;
        } else {
            memcpy(P->qstore + (size_t)ti * P->D.row_pitch, src, (size_t)P->D.dim * es);
            t.dev_vec = P->qstore_dev + (size_t)ti * P->D.row_pitch;
        }
        P->pending[t.klass].push_back(ti);
        out[i] = ((uint64_t)t.gen << 32) | ti;
        if (n_done) *n_done = i + 1;
    }
    return TRI_OK;
}

namespace {
int g_step_locked(tri_gpool *P, tri_graph_step_stats *st);
}

extern "C" int graph_step(tri_gpool *P, tri_graph_step_stats *st)
{
    if (!P) return tri_fail(TRI_EINVAL, "pool is NULL");
    std::lock_guard<std::mutex> lk(P->mu);
    GHIP(hipSetDevice(P->device));
    return g_step_locked(P, st);
}

namespace {
int g_step_locked(tri_gpool *P, tri_graph_step_stats *st)
{
    tri_graph_step_stats stats{};
    int rc = g_reap(P, false, &stats.finished);
    if (rc) return rc;
    // this call serves one group of slots; its previous step must have completed (its slots are then known)
    const uint32_t g = (uint32_t)(P->step_seq % P->ngroups);
    GStep &R = P->ring[g];
    if (R.in_use) {
        GHIP(hipEventSynchronize(R.done));
        rc = g_reap(P, false, &stats.finished);
        if (rc) return rc;
        if (R.in_use) return tri_fail(TRI_EHIP, "internal: a completed step was not collected");
    }
    // admit: high class first, first-in first-out inside a class
    GxHdr *hdr = (GxHdr *)R.up_host;
    GxNewDesc *desc = (GxNewDesc *)(R.up_host + sizeof(GxHdr));
    uint32_t n_new = 0;
    const bool may_admit = !P->static_batches || R.n_running == 0;
    for (int klass = 0; klass < 2 && may_admit; ++klass) {
        std::deque<uint32_t> &Q = P->pending[klass];
        while (!Q.empty() && !R.free_slots.empty()) {
            const uint32_t ti = Q.front();
            Q.pop_front();
            const uint32_t slot = R.free_slots.back();
            R.free_slots.pop_back();
            GTicket &t = P->tickets[ti];
            t.state = G_RUNNING;
            t.slot = slot;
            P->slot_ticket[slot] = ti;
            desc[n_new++] = GxNewDesc{slot, t.k, t.metric, 0u, (uint64_t)(uintptr_t)t.dev_vec, 0ull};
            ++R.n_running;
            ++P->n_running;
        }
    }
    stats.step = P->step_seq;
    stats.admitted = n_new;
    stats.running = P->n_running;
    stats.pending = (uint32_t)(P->pending[0].size() + P->pending[1].size());
    ++P->step_seq;                                  // (the next call serves the next group)
    if (R.n_running == 0) {
        if (st) *st = stats;
        return TRI_OK;
    }
    hdr->n16 = (uint32_t)((sizeof(GxHdr) + (size_t)n_new * sizeof(GxNewDesc) + 15) / 16);
    hdr->n_new = n_new;
    memset(R.down_host, 0, (size_t)P->cfg.slots * 4);   // (this entry's previous step has been collected: the block is ours)
    hipStream_t s = R.stream;
    GxDev D = P->D;
    D.upload = R.upload;
    D.group = g;
    const uint32_t nblocks = (D.S - g + D.ngroups - 1) / D.ngroups;      // slots of this group
    const bool prof = (P->cfg.flags & TRI_FLAG_PROFILE) != 0;
    hipLaunchKernelGGL(gx_pull_kernel, dim3((hdr->n16 + 255) / 256), dim3(256), 0, s, (uint4 *)D.upload, (const uint4 *)R.up_dev);
    if (n_new) hipLaunchKernelGGL(gx_admit_kernel, dim3(n_new), dim3(GX_THREADS), 0, s, D);
    GHIP(hipGetLastError());
    if (prof) GHIP(hipEventRecord(R.ev0, s));
    uint32_t *done_d = (uint32_t *)R.down_dev;
    GHIP(D.dtype == TRI_F16 ? g_launch_step<TRI_F16>(D, nblocks, s, done_d, done_d + D.S, P->rec_words)
                            : g_launch_step<TRI_F32>(D, nblocks, s, done_d, done_d + D.S, P->rec_words));
    if (prof) GHIP(hipEventRecord(R.ev1, s));
    GHIP(hipEventRecord(R.done, s));
    R.in_use = true;
    R.profiled = prof;
    R.seq = stats.step;
    if (st) *st = stats;
    return TRI_OK;
}

}  // namespace

// The serving loop of Sec. 3.2 as one native call (arrivals join at the next step of a group with a free slot,
// finished requests leave at once), or -- static_batches -- the scheme it replaces: a group of slots takes new
// requests only when all of its requests have finished.
extern "C" int graph_run_stream(tri_gpool *P, const void *vecs, uint64_t pitch_bytes, const double *arrival_s, uint32_t n,
                                const uint32_t *k, const uint32_t *metric, const uint32_t *klass, int static_batches,
                                uint32_t stride, uint32_t *n_out, int64_t *ids, float *dist, double *done_s,
                                tri_graph_stream_stats *stats)
{
    if (!P || (n && (!vecs || !arrival_s || !k || !metric || !n_out || !ids || !dist || !done_s)))
        return tri_fail(TRI_EINVAL, "NULL argument");
    const size_t es = P->D.dtype == TRI_F16 ? 2 : 4;
    if (pitch_bytes < (uint64_t)P->D.dim * es || pitch_bytes % es) return tri_fail(TRI_EINVAL, "pitch_bytes too small or not a multiple of the element size");
    for (uint32_t i = 0; i < n; ++i) {
        if (k[i] == 0 || k[i] > P->cfg.topm || k[i] > stride) return tri_fail(TRI_EINVAL, "k must be 1..min(topm, stride) (query %u has %u)", i, k[i]);
        if (metric[i] != TRI_L2 && metric[i] != TRI_IP) return tri_fail(TRI_EINVAL, "metric must be TRI_L2 or TRI_IP");
        if (klass && klass[i] != TRI_CLASS_HIGH && klass[i] != TRI_CLASS_LOW) return tri_fail(TRI_EINVAL, "klass must be TRI_CLASS_HIGH or TRI_CLASS_LOW");
        if (i && arrival_s[i] < arrival_s[i - 1]) return tri_fail(TRI_EINVAL, "arrival times must not decrease");
    }
    std::lock_guard<std::mutex> lk(P->mu);
    GHIP(hipSetDevice(P->device));
    if (P->n_running || !P->pending[0].empty() || !P->pending[1].empty()) return tri_fail(TRI_EINVAL, "the pool must be idle");
    if (P->free_tickets.size() < n) return tri_fail(TRI_ENOMEM, "max_outstanding leaves %zu free tickets, the stream has %u queries", P->free_tickets.size(), n);
    tri_gpool::Sink K;
    try { K.q_of_ticket.assign(P->tickets.size(), 0); } catch (const std::bad_alloc &) { return tri_fail(TRI_ENOMEM, "out of host memory"); }
    K.n_out = n_out; K.ids = ids; K.dist = dist; K.done_s = done_s; K.stride = stride; K.delivered = 0;
    K.t0_ns = gnow_ns();
    P->sink = &K;
    P->static_batches = static_batches != 0;
    tri_graph_stream_stats S{};
    uint32_t next = 0;
    int rc = TRI_OK;
    while (K.delivered < n && rc == TRI_OK) {
        const double now = (double)(gnow_ns() - K.t0_ns) * 1e-9;
        while (next < n && arrival_s[next] <= now) {              // queue what has arrived
            const uint32_t ti = P->free_tickets.back();
            P->free_tickets.pop_back();
            GTicket &t = P->tickets[ti];
            t.state = G_PENDING;
            t.k = k[next]; t.metric = metric[next]; t.klass = klass ? klass[next] : (uint32_t)TRI_CLASS_LOW;
            memcpy(P->qstore + (size_t)ti * P->D.row_pitch, (const uint8_t *)vecs + (size_t)next * pitch_bytes, (size_t)P->D.dim * es);
            t.dev_vec = P->qstore_dev + (size_t)ti * P->D.row_pitch;
            K.q_of_ticket[ti] = next;
            P->pending[t.klass].push_back(ti);
            ++next;
        }
        const uint64_t waiting = P->pending[0].size() + P->pending[1].size();
        S.max_pending = std::max<uint64_t>(S.max_pending, waiting);
        if (P->n_running == 0 && waiting == 0) continue;          // nothing to do until the next arrival
        tri_graph_step_stats st{};
        rc = g_step_locked(P, &st);
        if (rc == TRI_OK && (st.running || st.admitted)) { S.steps += 1; S.running += st.running; }
    }
    if (rc == TRI_OK) rc = g_reap(P, true, nullptr);
    S.wall_s = (double)(gnow_ns() - K.t0_ns) * 1e-9;
    P->sink = nullptr;
    P->static_batches = false;
    if (stats) *stats = S;
    return rc;
}

extern "C" int graph_poll(tri_gpool *P, const tri_ticket *tk, uint32_t n, uint32_t stride, uint32_t *n_out, int64_t *ids,
                          float *dist, uint32_t *iters, uint32_t *evals, int *status)
{
    if (!P || (n && (!tk || !n_out || !ids || !dist || !status))) return tri_fail(TRI_EINVAL, "NULL argument");
    std::lock_guard<std::mutex> lk(P->mu);
    int rc = g_reap(P, false, nullptr);
    if (rc) return rc;
    int delivered = 0;
    const uint32_t M = P->cfg.topm;
    for (uint32_t i = 0; i < n; ++i) {
        const uint32_t ti = (uint32_t)(tk[i] & 0xFFFFFFFFu), gen = (uint32_t)(tk[i] >> 32);
        if (ti >= P->tickets.size() || P->tickets[ti].gen != gen || P->tickets[ti].state == G_FREE) { status[i] = TRI_ENOENT; continue; }
        GTicket &t = P->tickets[ti];
        if (t.state != G_DONE) { status[i] = TRI_EAGAIN; continue; }
        if (stride < t.k) return tri_fail(TRI_EINVAL, "stride %u is smaller than ticket %u's k = %u", stride, i, t.k);
        int64_t *oi = ids + (size_t)i * stride;
        float *od = dist + (size_t)i * stride;
        for (uint32_t j = 0; j < t.n_out; ++j) { oi[j] = (int64_t)P->res_ids[(size_t)ti * M + j]; od[j] = P->res_score[(size_t)ti * M + j]; }
        const float pad = t.metric == TRI_L2 ? __builtin_inff() : -__builtin_inff();
        for (uint32_t j = t.n_out; j < t.k; ++j) { oi[j] = -1; od[j] = pad; }
        n_out[i] = t.n_out;
        if (iters) iters[i] = t.iters;
        if (evals) evals[i] = t.evals;
        status[i] = TRI_OK;
        t.state = G_FREE;
        ++t.gen;
        P->free_tickets.push_back(ti);
        ++delivered;
    }
    return delivered;
}

extern "C" int graph_sync(tri_gpool *P)
{
    if (!P) return tri_fail(TRI_EINVAL, "pool is NULL");
    std::lock_guard<std::mutex> lk(P->mu);
    GHIP(hipSetDevice(P->device));
    return g_reap(P, true, nullptr);
}

extern "C" int graph_kernel_times(tri_gpool *P, tri_graph_times *out, int reset)
{
    if (!P || !out) return tri_fail(TRI_EINVAL, "NULL argument");
    std::lock_guard<std::mutex> lk(P->mu);
    *out = P->times;
    if (reset) { const uint32_t rb = P->times.row_bytes; P->times = tri_graph_times{}; P->times.row_bytes = rb; }
    return TRI_OK;
}
