// Host side of the pool worker: C ABI, slot table, class queues, step planner, result delivery.
// (Paper Sec. 3.2 for the step loop -- admit, emit tasks, one fixed-shape evaluation, merge,
// retire, recycle -- and Sec. 3.3 for the two priority classes served at step boundaries.)
#include "../../include/trinity_ivf.h"
#include "tri_common.h"

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <chrono>
#include <deque>
#include <thread>
#include <mutex>
#include <new>
#include <string>
#include <vector>

namespace {
thread_local std::string g_err;
}  // namespace

// Device workspace of the pools made by tri_pool_create_static: one array per GPU the library is loaded on,
// part of the library's image, so that such a pool needs no allocation.  In host code the name is only a handle
// for hipGetSymbolAddress; the address the kernels get is looked up once per device (g_static).
static __device__ __align__(256) unsigned char scratch[TRI_STATIC_WS_BYTES];

int tri_fail(int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

namespace {

#define HIP_TRY(expr)                                                                          \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess) return tri_fail(TRI_EHIP, "%s -> %s", #expr, hipGetErrorString(e_)); \
    } while (0)

constexpr uint32_t RING = 4;          // steps that may be in flight before search_step waits
constexpr uint32_t N_EV = 8;          // profile events per step
constexpr uint32_t N_SHAPES = 3;      // captured sizes of a step: 1/16, 1/4 and all of the pool's slots and items

inline int64_t now_ns()
{
    return std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now().time_since_epoch()).count();
}
inline uint32_t round_up(uint32_t v, uint32_t m) { return (v + m - 1) / m * m; }
inline size_t round_up_sz(size_t v, size_t m) { return (v + m - 1) / m * m; }
inline uint32_t esize(uint32_t dtype) { return dtype == TRI_F16 ? 2u : 4u; }
inline uint32_t dpad_of(uint32_t dim, uint32_t dtype) { return round_up(dim, 128u / esize(dtype)); }

enum TState : uint8_t { T_FREE = 0, T_PENDING, T_RUNNING, T_RETIRING, T_DONE };

struct Ticket {
    uint32_t gen = 0;
    TState state = T_FREE;
    bool cancelled = false;
    tri_index *index = nullptr;
    uint32_t k = 0, nprobe = 0, metric = 0, klass = 0;
    uint64_t tag = 0;
    int64_t deadline_ns = INT64_MAX;   // absolute, on the pool's clock; INT64_MAX = none
    int64_t submit_ns = 0;
    const void *dev_vec = nullptr;   // non-NULL: the vector is read from device memory at admission
    uint32_t slot = 0;
    uint64_t step_seq = 0;
    uint32_t retire_idx = 0;
    uint32_t n_out = 0;
};

struct SlotH {
    bool active = false;
    uint32_t ticket = 0;
    uint32_t nprobe = 0, cursor = 0, klass = 0;
    uint64_t admit_seq = 0;
    tri_index *index = nullptr;
};

// Where search_run_stream wants finished results delivered: straight from a step's pinned block into the
// caller's arrays (row = the query's position in the stream), without the stop in the ticket store.
struct StreamSink {
    const uint32_t *q_of_ticket;
    uint32_t *n_out;
    int64_t *ids;
    float *dist;
    uint32_t *probes;
    uint32_t stride;
};

struct StepRec {
    bool in_use = false;
    bool profiled = false;            // all stages bracketed by events
    bool profiled_scan = false;       // only the list scan bracketed
    uint64_t seq = 0;
    hipEvent_t done = nullptr;
    hipEvent_t ev[N_EV] = {};
    uint8_t *up_host = nullptr;       // pinned: upload block
    uint8_t *down_host = nullptr;     // pinned: result block, probes, step numbers
    uint8_t *down_dev = nullptr;      // the same memory as the GPU addresses it
    uint8_t *up_dev = nullptr;        // up_host as the GPU addresses it
    int64_t enqueue_ns = 0;           // when search_step enqueued it
    std::vector<uint32_t> retire;     // ticket index per retire_idx
    uint32_t n_items = 0;
    bool had_scan = false;
    // TRI_FLAG_GRAPH: the step's launch sequence with this entry's pinned blocks, recorded once per captured
    // size (and set of attached indexes) and replayed
    hipGraph_t graph[2 * N_SHAPES] = {};            // [lists streamed past the caches or not][captured size]
    hipGraphExec_t graph_exec[2 * N_SHAPES] = {};
};

}  // namespace

struct tri_index {
    tri_pool *pool = nullptr;
    uint32_t id = 0;
    ivf_params p{};
    uint64_t n = 0;
    uint32_t dpad = 0, row_bytes = 0, list_base = 0, max_list_len = 0;
    TriIndexDev dev{};
    uint32_t *ids_dev = nullptr;
    uint32_t *list_off_dev = nullptr;
    std::vector<uint32_t> list_len;   // host copy of the list lengths
};

void tri_index_view(const tri_index *ix, TriIndexView *out);

struct tri_pool {
    tri_pool_cfg cfg{};
    int device = 0;
    hipStream_t stream = nullptr;
    std::mutex mu;
    TriDevWs ws{};
    TriLaunchCtx ctx{};
    uint32_t max_row_bytes = 0, coarse_rows = 0, coarse_ldc = 0;
    uint32_t attached_row_bytes = 128;   // widest row among the attached indexes (sizes the scan kernel's LDS)
    uint32_t scan_class_mask = 0;        // scan kernel variants the attached indexes need
    uint32_t n_order = 0;                // attached lists (entries of the device-side scan order)
    uint64_t score_capacity = 0;
    size_t upload_bytes = 0, down_bytes = 0;
    size_t down_probe_off = 0, down_step_off = 0;
    // indexes
    std::vector<tri_index *> indexes;
    uint32_t total_lists = 0;
    // tickets
    std::vector<Ticket> tickets;
    std::vector<uint32_t> free_tickets;
    uint8_t *qstore = nullptr;         // pinned [max_outstanding][max_row_bytes]: padded rows of host-submitted queries,
    uint8_t *qstore_dev = nullptr;     //   read by the admitting step's kernel straight from there (same memory, GPU address)
    std::vector<uint32_t> res_ids;     // [max_outstanding][kmax]
    std::vector<float> res_score;      // [max_outstanding][kmax]
    std::vector<uint32_t> res_probe;   // [max_outstanding][nprobe_max] (only with KEEP_PROBES)
    std::deque<uint32_t> pending[2];
    // slots
    std::vector<SlotH> slots;
    std::vector<uint32_t> free_slots;
    uint32_t n_running = 0;
    uint64_t admit_seq = 0, step_seq = 0;
    uint32_t merge_launches = 0;      // parity of the merge kernels' queue heads
    uint32_t coarse_steps = 0;        // parity of the coarse selection's queue heads
    StepRec ring[RING];
    uint8_t *pinned = nullptr;         // upload / result blocks of the steps in flight, then the query store
    bool own_pinned = false;           // allocated here (hipHostMalloc) and freed in tri_pool_destroy
    uint32_t cand_reserve = 0;         // != 0: pairs reserved per query and step instead of the estimate (tri_pool_set_candidate_reserve)
    int static_dev = -1;               // >= 0: the workspace is that device's static array (tri_pool_create_static)
    // a step that failed half-way leaves the slot table out of step with the GPU: the pool is then failed for good
    bool failed = false, inject_failure = false;
    std::string fail_text;
    tri_kernel_times times{};
    // scratch vectors reused by search_step
    std::vector<uint32_t> order, newq;
    std::vector<uint8_t> index_seen;      // per attached index: has a query been admitted for it in this step
    std::vector<uint32_t> run_order[2];   // running slots per class, in admission order (with the admission number
    std::vector<uint64_t> run_seq[2];     //   each had then: a slot number alone could be a later occupant)
    // scheduling policy (Sec. 3.3) and the measured mean step duration its slack order uses
    tri_policy policy{1.0f, TRI_ORDER_FIFO, 0.0, 0.0, 0u, 0u};
    double mean_step_s = 0.0;
    int64_t last_done_ns = 0;
    // control loop of Sec. 3.3 (search_set_feedback)
    bool fb_on = false;
    tri_feedback_cfg fb{};
    tri_feedback_signals fb_last{};       // what the last period saw
    float fb_u_kv = __builtin_nanf(""), fb_stall = __builtin_nanf(""), fb_stall_prev = __builtin_nanf("");
    int64_t fb_last_ns = 0;
    uint64_t fb_periods = 0;
    std::vector<float> fb_waits;          // submission-to-admission waits (s) of the high class since the last period
    // search_run_stream: tickets in the order their results arrived
    std::vector<uint32_t> done_log;
    const StreamSink *sink = nullptr;
};

namespace {

void drop_graphs(tri_pool *P);
void feedback_tick(tri_pool *P);
int step_locked(tri_pool *P, tri_step_stats *st);

// Carve the device workspace.  Must match TriDevWs field for field.
size_t carve(const tri_pool_cfg &c, uint32_t max_row_bytes, uint32_t coarse_rows, uint32_t coarse_ldc,
             uint64_t score_capacity, size_t upload_bytes, uint8_t *base, TriDevWs *ws)
{
    size_t o = 0;
    auto take = [&](size_t bytes) {
        size_t at = o;
        o = round_up_sz(o + bytes, 256);
        return base ? base + at : (uint8_t *)nullptr;
    };
    const size_t S = c.slots, W = c.items_per_step, G = (size_t)c.max_total_lists + 1;
    uint8_t *p;
#define CARVE(field, type, bytes) p = take(bytes); if (ws) ws->field = (type)p;
    CARVE(slot_query, uint8_t *, S * max_row_bytes)
    CARVE(dev_qstore, uint8_t *, (size_t)c.max_outstanding * max_row_bytes)
    CARVE(slot_meta, TriSlotMeta *, S * sizeof(TriSlotMeta))
    CARVE(slot_qnorm, float *, S * 4)
    CARVE(probe, uint32_t *, S * c.nprobe_max * 4)
    CARVE(topk_score, float *, S * c.kmax * 4)
    CARVE(topk_id, uint32_t *, S * c.kmax * 4)
    CARVE(topk_count, uint32_t *, S * 4)
    CARVE(indexes, TriIndexDev *, (size_t)c.max_indexes * sizeof(TriIndexDev))
    CARVE(glist_len, uint32_t *, G * 4)
    CARVE(glist_voff, uint32_t *, G * 4)
    CARVE(glist_index, uint32_t *, G * 4)
    CARVE(glist_order, uint4 *, G * 16)
    CARVE(pack_tot, uint64_t *, 16 * 9 * 8)
    CARVE(upload, uint8_t *, upload_bytes)
    CARVE(coarse_scores, float *, (size_t)coarse_rows * coarse_ldc * 4)
    CARVE(item_glist, uint32_t *, W * 4)
    CARVE(item_slot, uint32_t *, W * 4)
    CARVE(item_rank, uint32_t *, W * 4)
    CARVE(item_sorted_pos, uint32_t *, W * 4)
    CARVE(sorted_slot, uint32_t *, W * 4)
    CARVE(hist, uint32_t *, G * 4)
    CARVE(list_start, uint32_t *, G * 4)
    CARVE(tile_base, uint32_t *, G * 4)
    CARVE(stile_base, uint32_t *, G * 4)
    CARVE(tiles, TriTile *, (size_t)TRI_TILES_PER_ITEM * W * sizeof(TriTile))
    CARVE(stiles, TriTile *, W * sizeof(TriTile))
    CARVE(tile_counter, uint32_t *, 256)
    CARVE(sample_scores, float *, W * (size_t)TRI_SAMPLE_VECS * 4)
    CARVE(thr_key, uint32_t *, S * 4)
    CARVE(slot_cand_off, uint32_t *, S * 4)
    CARVE(slot_cand_cap, uint32_t *, S * 4)
    CARVE(slot_cand_cnt, uint32_t *, S * 4)
    CARVE(rescans, uint32_t *, 1024)
    CARVE(merge_queue, uint32_t *, S * 4)
    CARVE(coarse_queue, uint32_t *, S * 4)
    CARVE(step_dev, TriStepDev *, 256)
    CARVE(cand, uint2 *, (size_t)score_capacity * 4)
    // (res_block / res_probes point into the pinned host block of the step in flight: set per step)
#undef CARVE
    return o;
}

int derive(const tri_pool_cfg *c, uint32_t *max_row_bytes, uint32_t *coarse_rows, uint32_t *coarse_ldc,
           uint64_t *score_capacity, size_t *upload_bytes)
{
    if (!c) return tri_fail(TRI_EINVAL, "cfg is NULL");
    if (c->slots == 0 || c->slots > (1u << 20)) return tri_fail(TRI_EINVAL, "slots must be 1..2^20");
    if (c->items_per_step == 0) return tri_fail(TRI_EINVAL, "items_per_step must be > 0");
    if (c->kmax == 0 || c->kmax > TRI_KMAX_LIMIT) return tri_fail(TRI_EINVAL, "kmax must be 1..%u", TRI_KMAX_LIMIT);
    if (c->nprobe_max == 0 || c->nprobe_max > TRI_NPROBE_LIMIT)
        return tri_fail(TRI_EINVAL, "nprobe_max must be 1..%u", TRI_NPROBE_LIMIT);
    if (c->max_indexes == 0 || c->max_indexes > 256) return tri_fail(TRI_EINVAL, "max_indexes must be 1..256");
    if (c->max_nlist == 0 || c->max_total_lists < c->max_nlist)
        return tri_fail(TRI_EINVAL, "need 0 < max_nlist <= max_total_lists");
    if (c->max_dim == 0) return tri_fail(TRI_EINVAL, "max_dim must be > 0");
    if (c->max_outstanding < c->slots) return tri_fail(TRI_EINVAL, "max_outstanding must be >= slots");
    const uint32_t rb = round_up(c->max_dim * 4u, 128u);   // fp32 rows are the widest
    const uint32_t rb16 = round_up(c->max_dim * 2u, 128u);
    if (rb16 > TRI_MAX_ROW_BYTES) return tri_fail(TRI_EINVAL, "max_dim too large: padded fp16 row exceeds %u bytes", TRI_MAX_ROW_BYTES);
    *max_row_bytes = rb > TRI_MAX_ROW_BYTES ? TRI_MAX_ROW_BYTES : rb;
    if ((uint64_t)c->slots * *max_row_bytes >= (1ull << 31))
        return tri_fail(TRI_EINVAL, "slots * padded row bytes must stay below 2^31");
    *coarse_rows = c->coarse_rows ? c->coarse_rows : 1024u;
    if (*coarse_rows > c->slots) *coarse_rows = c->slots;
    *coarse_ldc = tri_coarse_ldc(c->max_nlist);
    // default: room for 1024 kept candidates per slot and 32 per work item (2 words each)
    *score_capacity = c->score_capacity ? c->score_capacity : 2ull * ((uint64_t)c->slots * 1024u + (uint64_t)c->items_per_step * 32u);
    if (*score_capacity > (1ull << 32))      // candidate pairs are addressed with 32-bit pair numbers
        return tri_fail(TRI_EINVAL, "score_capacity must not exceed 2^32 words");
    if (*score_capacity < 2ull * c->kmax) return tri_fail(TRI_EINVAL, "score_capacity must hold at least kmax pairs");
    *upload_bytes = sizeof(TriStepHdr) + round_up_sz((size_t)c->slots * sizeof(TriNewDesc), 256) +
                    round_up_sz((size_t)c->slots * sizeof(TriPlanEntry), 256) + (size_t)c->slots * *max_row_bytes;
    return TRI_OK;
}

// Deliver the results of every completed step (oldest first).  block: wait for all of them.
int reap(tri_pool *P, bool block, uint32_t *finished)
{
    uint32_t fin = 0;
    // oldest in-use entry first
    for (uint32_t n = 0; n < RING; ++n) {
        StepRec *R = nullptr;
        for (uint32_t i = 0; i < RING; ++i)
            if (P->ring[i].in_use && (!R || P->ring[i].seq < R->seq)) R = &P->ring[i];
        if (!R) break;
        if (block) {
            HIP_TRY(hipEventSynchronize(R->done));
        } else {
            hipError_t q = hipEventQuery(R->done);
            if (q == hipErrorNotReady) break;
            if (q != hipSuccess) return tri_fail(TRI_EHIP, "hipEventQuery -> %s", hipGetErrorString(q));
        }
        if (R->had_scan) {
            // mean step duration: completion to completion while the GPU is kept busy, else enqueue to completion
            const int64_t t = now_ns();
            const double d = (double)(t - std::max(R->enqueue_ns, P->last_done_ns)) * 1e-9;
            P->mean_step_s = P->mean_step_s == 0.0 ? d : 0.8 * P->mean_step_s + 0.2 * d;
            P->last_done_ns = t;
        }
        const uint32_t kmax = P->cfg.kmax, pmax = P->cfg.nprobe_max;
        const uint32_t *blk = (const uint32_t *)R->down_host;
        const uint32_t *prb = (const uint32_t *)(R->down_host + P->down_probe_off);
        for (size_t i = 0; i < R->retire.size(); ++i) {
            const uint32_t ti = R->retire[i];
            Ticket &t = P->tickets[ti];
            if (t.cancelled) {
                t.state = T_FREE;
                t.cancelled = false;
                ++t.gen;
                P->free_tickets.push_back(ti);
                continue;
            }
            const uint32_t *rec = blk + i * (1 + 2 * (size_t)kmax);
            t.n_out = rec[0];
            if (P->sink) {
                const StreamSink &K = *P->sink;
                const uint32_t qi = K.q_of_ticket[ti];
                int64_t *oi = K.ids + (size_t)qi * K.stride;
                float *od = K.dist + (size_t)qi * K.stride;
                const float *sc = (const float *)(rec + 1 + kmax);
                for (uint32_t j = 0; j < t.n_out; ++j) { oi[j] = (int64_t)rec[1 + j]; od[j] = sc[j]; }
                const float pad = t.metric == TRI_L2 ? __builtin_inff() : -__builtin_inff();
                for (uint32_t j = t.n_out; j < t.k; ++j) { oi[j] = -1; od[j] = pad; }
                K.n_out[qi] = t.n_out;
                if (K.probes) memcpy(K.probes + (size_t)qi * pmax, prb + i * (size_t)pmax, (size_t)t.nprobe * 4);
                P->done_log.push_back(qi);
                t.state = T_FREE;
                ++t.gen;
                P->free_tickets.push_back(ti);
                ++fin;
                continue;
            }
            memcpy(&P->res_ids[(size_t)ti * kmax], rec + 1, (size_t)t.n_out * 4);
            memcpy(&P->res_score[(size_t)ti * kmax], rec + 1 + kmax, (size_t)t.n_out * 4);
            if (P->cfg.flags & TRI_FLAG_KEEP_PROBES)
                memcpy(&P->res_probe[(size_t)ti * pmax], prb + i * (size_t)pmax, (size_t)t.nprobe * 4);
            t.state = T_DONE;
            ++fin;
        }
        if (R->profiled || R->profiled_scan) {
            // events: 0 block pulled, 1 admitted, 2 ranked, 3 packed, 4 sample scanned, 5 thresholds set, 6 lists
            // scanned, 7 merged; with only the scan profiled, 3..6 exist
            float ms[N_EV - 1] = {};
            if (R->profiled)
                for (uint32_t i = 0; i + 1 < N_EV; ++i) HIP_TRY(hipEventElapsedTime(&ms[i], R->ev[i], R->ev[i + 1]));
            else if (R->had_scan)
                for (uint32_t i = 3; i < 6; ++i) HIP_TRY(hipEventElapsedTime(&ms[i], R->ev[i], R->ev[i + 1]));
            const TriStepDev *sd = (const TriStepDev *)(R->down_host + P->down_step_off);
            P->times.steps += 1;
            P->times.admit_ms += ms[0];
            P->times.coarse_ms += ms[1];
            P->times.pack_ms += ms[2];
            P->times.sample_ms += ms[3];
            P->times.threshold_ms += ms[4];
            P->times.scan_ms += ms[5];
            P->times.select_ms += ms[6];
            if (R->had_scan) {
                P->times.scan_launches += 1;
                P->times.scan_vector_bytes += sd->tile_vec_bytes;
                P->times.scan_unique_bytes += sd->unique_vec_bytes;
                P->times.scan_list_bytes += sd->list_bytes;
                P->times.scan_items += R->n_items;
            }
        }
        R->retire.clear();
        R->in_use = false;
    }
    if (finished) *finished += fin;
    return TRI_OK;
}

// Scan order of the pool-wide list table: every attached list, longest (in bytes) first.
int upload_scan_order(tri_pool *P)
{
    std::vector<std::pair<uint64_t, uint32_t>> v;
    for (tri_index *ix : P->indexes)
        if (ix)
            for (uint32_t l = 0; l < ix->p.nlist; ++l)
                v.emplace_back((uint64_t)ix->list_len[l] * ix->row_bytes, ix->list_base + l);
    std::stable_sort(v.begin(), v.end(), [](const std::pair<uint64_t, uint32_t> &a, const std::pair<uint64_t, uint32_t> &b) {
        return a.first > b.first;
    });
    // per entry everything the per-step prefix sums need, so that they read this array front to back
    std::vector<uint4> order(v.size());
    uint32_t extent = 0;
    for (tri_index *ix : P->indexes)
        if (ix) extent = std::max(extent, ix->list_base + ix->p.nlist);
    std::vector<const tri_index *> owner(extent, nullptr);
    for (tri_index *ix : P->indexes)
        if (ix)
            for (uint32_t l = 0; l < ix->p.nlist; ++l) owner[ix->list_base + l] = ix;
    for (size_t i = 0; i < v.size(); ++i) {
        const uint32_t g = v[i].second;
        const tri_index *ix = owner[g];
        const uint32_t len = ix->list_len[g - ix->list_base];
        order[i] = make_uint4(g, len, ix->row_bytes, 0u);
    }
    if (!order.empty())
        HIP_TRY(hipMemcpy(P->ws.glist_order, order.data(), order.size() * sizeof(uint4), hipMemcpyHostToDevice));
    P->n_order = (uint32_t)order.size();
    return TRI_OK;
}

bool ticket_lookup(tri_pool *P, tri_ticket t, uint32_t *idx)
{
    const uint32_t i = (uint32_t)(t & 0xFFFFFFFFull), gen = (uint32_t)(t >> 32);
    if (i >= P->tickets.size()) return false;
    if (P->tickets[i].gen != gen || P->tickets[i].state == T_FREE) return false;
    *idx = i;
    return true;
}

// (compared as a pointer against the pool's table first: a handle of a destroyed index is never read)
bool is_attached(const tri_pool *P, const tri_index *ix)
{
    if (!ix) return false;
    for (const tri_index *a : P->indexes)
        if (a == ix) return true;
    return false;
}

// *known: the index of the previous query that passed (a batch mostly names one index; NULL at first)
int validate_query(tri_pool *P, const tri_query *q, const tri_index **known)
{
    if (q->index != *known) {
        if (!is_attached(P, q->index)) return tri_fail(TRI_EINVAL, "query.index is not attached to this pool");
        *known = q->index;
    }
    if (!q->vec) return tri_fail(TRI_EINVAL, "query.vec is NULL");
    if (q->k == 0 || q->k > P->cfg.kmax) return tri_fail(TRI_EINVAL, "k=%u outside 1..%u", q->k, P->cfg.kmax);
    if (q->nprobe == 0 || q->nprobe > P->cfg.nprobe_max || q->nprobe > q->index->p.nlist)
        return tri_fail(TRI_EINVAL, "nprobe=%u outside 1..min(%u, nlist=%u)", q->nprobe, P->cfg.nprobe_max, q->index->p.nlist);
    if (q->metric != TRI_L2 && q->metric != TRI_IP) return tri_fail(TRI_EINVAL, "metric must be TRI_L2 or TRI_IP");
    if (q->klass != TRI_CLASS_HIGH && q->klass != TRI_CLASS_LOW) return tri_fail(TRI_EINVAL, "klass must be TRI_CLASS_HIGH or TRI_CLASS_LOW");
    return TRI_OK;
}

void enqueue_locked(tri_pool *P, const tri_query *q, tri_ticket *out)
{
    const uint32_t ti = P->free_tickets.back();
    P->free_tickets.pop_back();
    Ticket &t = P->tickets[ti];
    t.state = T_PENDING;
    t.cancelled = false;
    t.index = const_cast<tri_index *>(q->index);
    t.k = q->k; t.nprobe = q->nprobe; t.metric = q->metric; t.klass = q->klass;
    t.tag = q->user_tag;
    t.submit_ns = now_ns();
    t.deadline_ns = q->deadline_ns ? t.submit_ns + (int64_t)std::min<uint64_t>(q->deadline_ns, (uint64_t)INT64_MAX / 2) : INT64_MAX;
    t.dev_vec = P->qstore_dev + (size_t)ti * P->max_row_bytes;   // (set before the copy below; read only after admission)
    uint8_t *row = P->qstore + (size_t)ti * P->max_row_bytes;
    const uint32_t es = esize(t.index->p.dtype);
    memcpy(row, q->vec, (size_t)t.index->p.dim * es);
    memset(row + (size_t)t.index->p.dim * es, 0, t.index->row_bytes - (size_t)t.index->p.dim * es);
    P->pending[t.klass].push_back(ti);
    *out = ((uint64_t)t.gen << 32) | ti;
}

}  // namespace

// ================================================================================== pool
namespace {
// Pinned host memory of a pool: RING x (upload block, result block), then the query store.
struct PinnedLayout { size_t blk, prb, down_bytes, per_step, qstore_off, total; };

PinnedLayout pinned_layout(const tri_pool_cfg &c, uint32_t max_row_bytes, size_t upload_bytes)
{
    PinnedLayout L;
    const size_t S = c.slots;
    L.blk = round_up_sz(S * (1 + 2 * (size_t)c.kmax) * 4, 256);
    L.prb = round_up_sz(S * (size_t)c.nprobe_max * 4, 256);
    L.down_bytes = L.blk + L.prb + 256;
    L.per_step = round_up_sz(upload_bytes, 256) + L.down_bytes;
    L.qstore_off = L.per_step * RING;
    L.total = L.qstore_off + round_up_sz((size_t)c.max_outstanding * max_row_bytes, 256);
    return L;
}

#define POOL_LIVE(P)                                                                                  \
    do {                                                                                              \
        if ((P)->failed) return tri_fail(TRI_EHIP, "the pool failed earlier: %s", (P)->fail_text.c_str()); \
    } while (0)
}  // namespace

extern "C" int tri_pool_workspace_bytes(const tri_pool_cfg *cfg, size_t *dev_bytes, size_t *pinned_host_bytes)
{
    uint32_t mrb, cr, ldc;
    uint64_t sc;
    size_t up;
    int rc = derive(cfg, &mrb, &cr, &ldc, &sc, &up);
    if (rc) return rc;
    if (!dev_bytes) return tri_fail(TRI_EINVAL, "dev_bytes is NULL");
    *dev_bytes = carve(*cfg, mrb, cr, ldc, sc, up, nullptr, nullptr);
    if (pinned_host_bytes) *pinned_host_bytes = pinned_layout(*cfg, mrb, up).total;
    return TRI_OK;
}

extern "C" int tri_pool_create(const tri_pool_cfg *cfg, void *dev_ws, size_t dev_ws_bytes, void *pinned_ws,
                               size_t pinned_ws_bytes, tri_pool **out)
{
    uint32_t mrb, cr, ldc;
    uint64_t sc;
    size_t up;
    int rc = derive(cfg, &mrb, &cr, &ldc, &sc, &up);
    if (rc) return rc;
    if (!dev_ws || !out) return tri_fail(TRI_EINVAL, "dev_ws / out is NULL");
    if ((cfg->flags & TRI_FLAG_GRAPH) && !cfg->hip_stream)
        return tri_fail(TRI_EINVAL, "TRI_FLAG_GRAPH needs a stream of the pool's own: a step cannot be recorded on the default stream");
    if ((uintptr_t)dev_ws % 256) return tri_fail(TRI_EINVAL, "dev_ws must be 256-byte aligned");
    const size_t need = carve(*cfg, mrb, cr, ldc, sc, up, nullptr, nullptr);
    if (dev_ws_bytes < need) return tri_fail(TRI_ENOMEM, "dev_ws has %zu bytes, %zu needed", dev_ws_bytes, need);
    const PinnedLayout L = pinned_layout(*cfg, mrb, up);
    if (pinned_ws) {
        if ((uintptr_t)pinned_ws % 256) return tri_fail(TRI_EINVAL, "pinned_ws must be 256-byte aligned");
        if (pinned_ws_bytes < L.total) return tri_fail(TRI_ENOMEM, "pinned_ws has %zu bytes, %zu needed", pinned_ws_bytes, L.total);
    }
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev == 0) return tri_fail(TRI_EHIP, "no HIP device");
    if (pinned_ws) {
        void *as_dev = nullptr;                   // (page-locked and mapped, or not usable: the kernels read and write it)
        if (hipHostGetDevicePointer(&as_dev, pinned_ws, 0) != hipSuccess || !as_dev) {
            (void)hipGetLastError();
            return tri_fail(TRI_EINVAL, "pinned_ws is not page-locked host memory the device can address");
        }
    }
    tri_pool *P = new (std::nothrow) tri_pool();
    if (!P) return tri_fail(TRI_ENOMEM, "out of host memory");
    P->cfg = *cfg;
    hipError_t e = hipGetDevice(&P->device);
    hipDeviceProp_t prop;
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, P->device);
    if (e != hipSuccess) { delete P; return tri_fail(TRI_EHIP, "device query -> %s", hipGetErrorString(e)); }
    P->stream = (hipStream_t)cfg->hip_stream;
    P->max_row_bytes = mrb; P->coarse_rows = cr; P->coarse_ldc = ldc; P->score_capacity = sc; P->upload_bytes = up;
    carve(*cfg, mrb, cr, ldc, sc, up, (uint8_t *)dev_ws, &P->ws);
    P->ctx = TriLaunchCtx{P->stream, cfg->slots, cfg->items_per_step, cfg->kmax, cfg->nprobe_max,
                          cfg->max_total_lists, mrb, (uint32_t)prop.multiProcessorCount, 0u};
    // pinned staging for RING steps and the query store: the caller's, or allocated here
    const size_t S = cfg->slots;
    P->down_probe_off = L.blk;
    P->down_step_off = L.blk + L.prb;
    P->down_bytes = L.down_bytes;
    if (pinned_ws) {
        P->pinned = (uint8_t *)pinned_ws;
    } else {
        e = hipHostMalloc((void **)&P->pinned, L.total, hipHostMallocDefault);
        if (e != hipSuccess) { delete P; return tri_fail(TRI_EHIP, "hipHostMalloc(%zu) -> %s", L.total, hipGetErrorString(e)); }
        P->own_pinned = true;
    }
    // what must start at zero: the rescan counter and the merge kernels' queue heads; the items-per-list histogram
    e = tri_launch_fill_u32(P->stream, P->ws.rescans, 0u, 256);
    if (e == hipSuccess) e = tri_launch_fill_u32(P->stream, P->ws.hist, 0u, cfg->max_total_lists);
    if (e == hipSuccess) e = hipStreamSynchronize(P->stream);
    if (e != hipSuccess) { tri_pool_destroy(P); return tri_fail(TRI_EHIP, "workspace set-up -> %s", hipGetErrorString(e)); }
    P->qstore = P->pinned + L.qstore_off;
    e = hipHostGetDevicePointer((void **)&P->qstore_dev, P->qstore, 0);
    if (e != hipSuccess) { tri_pool_destroy(P); return tri_fail(TRI_EHIP, "hipHostGetDevicePointer(query store) -> %s", hipGetErrorString(e)); }
    for (uint32_t i = 0; i < RING; ++i) {
        StepRec &R = P->ring[i];
        R.up_host = P->pinned + i * L.per_step;
        R.down_host = R.up_host + round_up_sz(up, 256);
        e = hipHostGetDevicePointer((void **)&R.down_dev, R.down_host, 0);
        if (e == hipSuccess) e = hipHostGetDevicePointer((void **)&R.up_dev, R.up_host, 0);
        if (e != hipSuccess) { tri_pool_destroy(P); return tri_fail(TRI_EHIP, "hipHostGetDevicePointer -> %s", hipGetErrorString(e)); }
        e = hipEventCreateWithFlags(&R.done, hipEventDisableTiming);
        for (uint32_t j = 0; j < N_EV && e == hipSuccess; ++j) e = hipEventCreateWithFlags(&R.ev[j], hipEventDisableSystemFence);   // (timing only: nothing on the host reads what the kernels between them wrote)
        if (e != hipSuccess) { tri_pool_destroy(P); return tri_fail(TRI_EHIP, "hipEventCreate -> %s", hipGetErrorString(e)); }
    }
    try {
        P->tickets.resize(cfg->max_outstanding);
        P->free_tickets.reserve(cfg->max_outstanding);
        for (uint32_t i = cfg->max_outstanding; i-- > 0;) P->free_tickets.push_back(i);
        P->res_ids.resize((size_t)cfg->max_outstanding * cfg->kmax);
        P->res_score.resize((size_t)cfg->max_outstanding * cfg->kmax);
        if (cfg->flags & TRI_FLAG_KEEP_PROBES) P->res_probe.resize((size_t)cfg->max_outstanding * cfg->nprobe_max);
        P->slots.resize(S);
        P->free_slots.reserve(S);
        for (uint32_t i = (uint32_t)S; i-- > 0;) P->free_slots.push_back(i);
        P->indexes.assign(cfg->max_indexes, nullptr);
        P->order.reserve(S);
        P->newq.reserve(S);
    } catch (const std::bad_alloc &) {
        tri_pool_destroy(P);
        return tri_fail(TRI_ENOMEM, "out of host memory");
    }
    *out = P;
    return TRI_OK;
}

namespace {
// The static workspace as each device addresses it, and whether a pool lives in it.
constexpr int MAX_STATIC_DEVICES = 64;
struct StaticWs { void *ptr = nullptr; bool in_use = false; };
StaticWs g_static[MAX_STATIC_DEVICES];
std::mutex g_static_mu;
}  // namespace

extern "C" int tri_pool_create_static(const tri_pool_cfg *cfg, void *pinned_ws, size_t pinned_ws_bytes, tri_pool **out)
{
    uint32_t mrb, cr, ldc;
    uint64_t sc;
    size_t up;
    int rc = derive(cfg, &mrb, &cr, &ldc, &sc, &up);
    if (rc) return rc;
    if (!pinned_ws || !out) return tri_fail(TRI_EINVAL, "pinned_ws / out is NULL (this call allocates no pinned memory either)");
    const size_t need = carve(*cfg, mrb, cr, ldc, sc, up, nullptr, nullptr);
    if (need > TRI_STATIC_WS_BYTES)
        return tri_fail(TRI_ENOMEM, "this configuration needs %zu bytes of device workspace, the static workspace holds %u: "
                                    "make it smaller (score_capacity, items_per_step, max_outstanding) or use tri_pool_create",
                        need, (unsigned)TRI_STATIC_WS_BYTES);
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_STATIC_DEVICES) return tri_fail(TRI_EINVAL, "device %d: the static workspace is kept for devices 0..%d", dev, MAX_STATIC_DEVICES - 1);
    std::lock_guard<std::mutex> lk(g_static_mu);
    StaticWs &W = g_static[dev];
    if (!W.ptr) {                               // once per device, with that device current
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return tri_fail(TRI_EHIP, "hipGetSymbolAddress returned no address for the static workspace");
        W.ptr = p;
    }
    if (W.in_use) return tri_fail(TRI_EAGAIN, "the static workspace of device %d holds a living pool: destroy that one first", dev);
    // Whatever an earlier pool left is cleared, up to the candidate buffer (whose entries are always written
    // before they are read, under counts the step itself produces).  A fill kernel, not a memset.
    TriDevWs lay{};
    carve(*cfg, mrb, cr, ldc, sc, up, (uint8_t *)W.ptr, &lay);
    const size_t head = (size_t)((uint8_t *)lay.cand - (uint8_t *)W.ptr);
    hipStream_t s = (hipStream_t)cfg->hip_stream;
    HIP_TRY(tri_launch_fill_u32(s, (uint32_t *)W.ptr, 0u, head / 4));
    HIP_TRY(hipStreamSynchronize(s));
    rc = tri_pool_create(cfg, W.ptr, TRI_STATIC_WS_BYTES, pinned_ws, pinned_ws_bytes, out);
    if (rc) return rc;
    (*out)->static_dev = dev;
    W.in_use = true;
    return TRI_OK;
}

extern "C" int tri_pool_destroy(tri_pool *P)
{
    if (!P) return tri_fail(TRI_EINVAL, "pool is NULL");
    for (tri_index *ix : P->indexes)
        if (ix) return tri_fail(TRI_EINVAL, "destroy the pool's indexes first");
    drop_graphs(P);
    if (P->static_dev >= 0) {
        std::lock_guard<std::mutex> lk(g_static_mu);
        g_static[P->static_dev].in_use = false;
    }
    for (uint32_t i = 0; i < RING; ++i) {
        if (P->ring[i].done) (void)hipEventDestroy(P->ring[i].done);
        for (uint32_t j = 0; j < N_EV; ++j)
            if (P->ring[i].ev[j]) (void)hipEventDestroy(P->ring[i].ev[j]);
    }
    if (P->pinned && P->own_pinned) (void)hipHostFree(P->pinned);
    delete P;
    return TRI_OK;
}

// ================================================================================== index
// Most blocks of 32 storage slots that n vectors in nlist lists can occupy (every list ends in a partly filled block).
static size_t index_blocks_max(uint64_t n, uint32_t nlist) { return (size_t)((n + 31ull * nlist + 31ull) / 32ull); }

extern "C" int ivf_build_bytes(const ivf_params *p, uint64_t n, size_t *dev_bytes)
{
    if (!p || !dev_bytes) return tri_fail(TRI_EINVAL, "NULL argument");
    if (p->dtype != TRI_F32 && p->dtype != TRI_F16) return tri_fail(TRI_EINVAL, "dtype must be TRI_F32 or TRI_F16");
    if (p->dim == 0 || p->nlist == 0 || n == 0) return tri_fail(TRI_EINVAL, "dim, nlist and n must be > 0");
    if (n >= (1ull << 32)) return tri_fail(TRI_EINVAL, "n must be < 2^32");
    if (p->nlist > n) return tri_fail(TRI_EINVAL, "nlist > n");
    const uint32_t dpad = dpad_of(p->dim, p->dtype), rb = dpad * esize(p->dtype);
    if (rb > TRI_MAX_ROW_BYTES) return tri_fail(TRI_EINVAL, "padded row of %u bytes exceeds %u", rb, TRI_MAX_ROW_BYTES);
    size_t o = 0;
    o += round_up_sz(index_blocks_max(n, p->nlist) * tri_block_stride(rb), 256);   // vectors: whole blocks of 32 per list
    o += round_up_sz(((size_t)n + TRI_VB) * 4, 256);       // |x|^2 (+ one block of slack for tail reads)
    o += round_up_sz((size_t)n * 4, 256);                  // ids
    o += round_up_sz((size_t)n * 4, 256);                  // stored position of every base row
    o += round_up_sz(((size_t)p->nlist + 1) * 4, 256);     // list offsets
    o += round_up_sz(((size_t)p->nlist + 1) * 4, 256);     // first block of every list
    o += round_up_sz((size_t)p->nlist * rb, 256);          // centroids
    o += round_up_sz((size_t)p->nlist * 4, 256);           // |c|^2
    *dev_bytes = o;
    return TRI_OK;
}

namespace {
// Temporary device memory of a build: carved from the caller's scratch, or -- without one -- allocated
// piece by piece and freed on scope exit.
struct TmpMem {
    uint8_t *arena = nullptr;
    size_t arena_bytes = 0, used = 0;
    std::vector<void *> ptrs;
    ~TmpMem() { for (void *p : ptrs) (void)hipFree(p); }
    hipError_t alloc(void **p, size_t bytes)
    {
        bytes = round_up_sz(bytes ? bytes : 256, 256);
        if (arena) {
            if (used + bytes > arena_bytes) return hipErrorOutOfMemory;
            *p = arena + used;
            used += bytes;
            return hipSuccess;
        }
        hipError_t e = hipMalloc(p, bytes);
        if (e == hipSuccess) ptrs.push_back(*p);
        return e;
    }
};

// Sizes of a build's temporary buffers (what ivf_build asks TmpMem for, in that order).
struct BuildTmp {
    uint32_t ldc, chunk, nblocks;
    uint64_t ns;
    size_t base_copy, cent_f32, scores, chunk_rows, assign, block_hist, list_len, train, perm_s, loff_s, total;
};

BuildTmp build_tmp(const ivf_params &p, uint64_t n, bool base_on_host)
{
    BuildTmp t{};
    const uint32_t es = esize(p.dtype), dpad = dpad_of(p.dim, p.dtype), rb = dpad * es;
    t.ldc = tri_coarse_ldc(p.nlist);
    t.chunk = round_up((uint32_t)std::min<uint64_t>(n, std::max<uint64_t>(128, (256ull << 20) / t.ldc)), 128);
    t.nblocks = (uint32_t)std::min<uint64_t>(512, (n + 255) / 256);
    t.ns = p.train_iters ? (n <= 256ull * p.nlist ? n : 256ull * p.nlist) : 0;
    t.base_copy = base_on_host ? (size_t)n * p.dim * es : 0;
    t.cent_f32 = (size_t)p.nlist * dpad * 4;
    t.scores = (size_t)t.chunk * t.ldc * 4;
    t.chunk_rows = (size_t)t.chunk * rb;
    t.assign = (size_t)n * 4;
    t.block_hist = (size_t)t.nblocks * p.nlist * 4;
    t.list_len = (size_t)p.nlist * 4;
    t.train = (size_t)t.ns * rb;
    t.perm_s = (size_t)t.ns * 4;
    t.loff_s = t.ns ? ((size_t)p.nlist + 1) * 4 : 0;
    for (size_t b : {t.base_copy, t.cent_f32, t.scores, t.chunk_rows, t.assign, t.block_hist, t.list_len, t.train, t.perm_s, t.loff_s})
        if (b) t.total += round_up_sz(b, 256);
    return t;
}

uint64_t splitmix64(uint64_t &s)
{
    uint64_t z = (s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
uint64_t gcd64(uint64_t a, uint64_t b) { while (b) { uint64_t t = a % b; a = b; b = t; } return a; }

// Assign rows [0, nrows) of `rows_of(chunk)` to their best centroid, chunk by chunk.
int assign_all(hipStream_t s, int dtype, uint32_t dim, uint32_t dpad, uint32_t rb, const void *base, uint64_t base_pitch,
               const void *padded_or_null, uint64_t nrows, const void *cent, const float *cnorm, uint32_t nlist,
               int metric, void *chunk_rows, float *scores, uint32_t ldc, uint32_t chunk, uint32_t *assign)
{
    for (uint64_t r0 = 0; r0 < nrows; r0 += chunk) {
        const uint32_t m = (uint32_t)std::min<uint64_t>(chunk, nrows - r0);
        const void *a_rows;
        if (padded_or_null) {
            a_rows = (const uint8_t *)padded_or_null + r0 * rb;
        } else {
            HIP_TRY(tri_build_pad_rows(s, dtype, base, dim, base_pitch, nullptr, 1, r0, ~0ull, m, chunk_rows, dpad));
            a_rows = chunk_rows;
        }
        HIP_TRY(tri_launch_coarse_gemm(s, dtype, a_rows, rb, m, cent, cnorm, nlist, rb, nullptr, 0, (uint32_t)metric,
                                       scores, ldc));
        HIP_TRY(tri_build_argbest(s, scores, ldc, m, nlist, metric, assign + r0));
    }
    return TRI_OK;
}
}  // namespace

// Lists are streamed past the caches once the attached vectors are far more than the caches hold.
static void set_scan_nt(tri_pool *P)
{
    uint64_t bytes = 0;
    for (const tri_index *o : P->indexes)
        if (o) bytes += o->n * o->row_bytes;
    P->ctx.scan_nt = (P->cfg.flags & TRI_FLAG_STREAM_LISTS) ? 2u : bytes >= TRI_NT_INDEX_BYTES ? 1u : 0u;
}

extern "C" int ivf_build_tmp_bytes(const ivf_params *p, uint64_t n, int base_on_host, size_t *tmp_bytes)
{
    size_t unused = 0;
    int rc = ivf_build_bytes(p, n, &unused);        // (validates the parameters)
    if (rc) return rc;
    if (!tmp_bytes) return tri_fail(TRI_EINVAL, "tmp_bytes is NULL");
    *tmp_bytes = build_tmp(*p, n, base_on_host != 0).total;
    return TRI_OK;
}

extern "C" int ivf_build(tri_pool *P, const ivf_params *p, const void *base, uint64_t n, const float *centroids,
                         void *dev_mem, size_t dev_mem_bytes, void *tmp_dev, size_t tmp_bytes, tri_index **out)
{
    if (!P || !p || !base || !dev_mem || !out) return tri_fail(TRI_EINVAL, "NULL argument");
    size_t need = 0;
    int rc = ivf_build_bytes(p, n, &need);
    if (rc) return rc;
    if (tmp_dev && (uintptr_t)tmp_dev % 256) return tri_fail(TRI_EINVAL, "tmp_dev must be 256-byte aligned");
    if (p->build_metric != TRI_L2 && p->build_metric != TRI_IP) return tri_fail(TRI_EINVAL, "build_metric must be TRI_L2 or TRI_IP");
    if ((uintptr_t)dev_mem % 256) return tri_fail(TRI_EINVAL, "dev_mem must be 256-byte aligned");
    if (dev_mem_bytes < need) return tri_fail(TRI_ENOMEM, "dev_mem has %zu bytes, %zu needed", dev_mem_bytes, need);
    std::lock_guard<std::mutex> lk(P->mu);
    POOL_LIVE(P);
    if (p->dim > P->cfg.max_dim) return tri_fail(TRI_EINVAL, "dim %u > pool max_dim %u", p->dim, P->cfg.max_dim);
    if (p->nlist > P->cfg.max_nlist) return tri_fail(TRI_EINVAL, "nlist %u > pool max_nlist %u", p->nlist, P->cfg.max_nlist);
    if ((uint64_t)P->total_lists + p->nlist > P->cfg.max_total_lists)
        return tri_fail(TRI_ENOMEM, "pool list table full (%u + %u > %u)", P->total_lists, p->nlist, P->cfg.max_total_lists);
    if (P->n_running || !P->pending[0].empty() || !P->pending[1].empty())
        return tri_fail(TRI_EINVAL, "ivf_build while queries are queued or running");
    uint32_t id = 0;
    while (id < P->cfg.max_indexes && P->indexes[id]) ++id;
    if (id == P->cfg.max_indexes) return tri_fail(TRI_ENOMEM, "pool already holds max_indexes=%u indexes", P->cfg.max_indexes);
    rc = reap(P, true, nullptr);
    if (rc) return rc;
    HIP_TRY(hipSetDevice(P->device));
    hipStream_t s = P->stream;
    HIP_TRY(hipStreamSynchronize(s));

    const int dtype = (int)p->dtype, metric = (int)p->build_metric;
    const uint32_t es = esize(p->dtype), dim = p->dim, nlist = p->nlist;
    const uint32_t dpad = dpad_of(dim, p->dtype), rb = dpad * es;
    if (rb > P->max_row_bytes) return tri_fail(TRI_EINVAL, "padded row %u bytes > pool row %u bytes", rb, P->max_row_bytes);

    // carve dev_mem
    uint8_t *m = (uint8_t *)dev_mem;
    const size_t vec_bytes = index_blocks_max(n, nlist) * tri_block_stride(rb);
    uint8_t *vecs = m;              m += round_up_sz(vec_bytes, 256);
    float *vnorm = (float *)m;      m += round_up_sz(((size_t)n + TRI_VB) * 4, 256);
    uint32_t *ids = (uint32_t *)m;  m += round_up_sz((size_t)n * 4, 256);
    uint32_t *inv = (uint32_t *)m;  m += round_up_sz((size_t)n * 4, 256);
    uint32_t *loff = (uint32_t *)m; m += round_up_sz(((size_t)nlist + 1) * 4, 256);
    uint32_t *boff = (uint32_t *)m; m += round_up_sz(((size_t)nlist + 1) * 4, 256);
    uint8_t *cent = m;              m += round_up_sz((size_t)nlist * rb, 256);
    float *cnorm = (float *)m;

    // base on the device
    const void *dbase = base;
    hipPointerAttribute_t attr;
    bool on_device = false;
    if (hipPointerGetAttributes(&attr, base) == hipSuccess)
        on_device = attr.type == hipMemoryTypeDevice || attr.type == hipMemoryTypeManaged;
    else
        (void)hipGetLastError();     // plain host memory: the query itself reports an error
    const BuildTmp bt = build_tmp(*p, n, !on_device);
    TmpMem tmp;
    if (tmp_dev) {
        if (tmp_bytes < bt.total) return tri_fail(TRI_ENOMEM, "tmp_dev has %zu bytes, %zu needed", tmp_bytes, bt.total);
        tmp.arena = (uint8_t *)tmp_dev;
        tmp.arena_bytes = tmp_bytes;
    }
    if (!on_device) {
        void *d = nullptr;
        HIP_TRY(tmp.alloc(&d, bt.base_copy));
        HIP_TRY(hipMemcpy(d, base, (size_t)n * dim * es, hipMemcpyHostToDevice));
        dbase = d;
    }
    // working buffers
    float *cent_f32 = nullptr;
    HIP_TRY(tmp.alloc((void **)&cent_f32, bt.cent_f32));
    const uint32_t ldc = bt.ldc, chunk = bt.chunk, nblocks = bt.nblocks;
    float *scores = nullptr;
    void *chunk_rows = nullptr;
    uint32_t *assign = nullptr, *block_hist = nullptr, *list_len = nullptr;
    HIP_TRY(tmp.alloc((void **)&scores, bt.scores));
    HIP_TRY(tmp.alloc(&chunk_rows, bt.chunk_rows));
    HIP_TRY(tmp.alloc((void **)&assign, bt.assign));
    HIP_TRY(tmp.alloc((void **)&block_hist, bt.block_hist));
    HIP_TRY(tmp.alloc((void **)&list_len, bt.list_len));

    // ---- initial centroids
    if (centroids) {
        std::vector<float> padded((size_t)nlist * dpad, 0.f);
        for (uint32_t l = 0; l < nlist; ++l) memcpy(&padded[(size_t)l * dpad], centroids + (size_t)l * dim, (size_t)dim * 4);
        HIP_TRY(hipMemcpy(cent_f32, padded.data(), padded.size() * 4, hipMemcpyHostToDevice));
    } else {
        // nlist distinct rows: an affine map j -> (a*j + b) mod n with gcd(a, n) = 1 is a permutation
        uint64_t st = p->seed, a = splitmix64(st) % n, b = splitmix64(st) % n;
        if (a == 0) a = 1;
        while (gcd64(a, n) != 1) a = a % n + 1;
        HIP_TRY(tri_build_pad_rows(s, dtype, dbase, dim, dim, nullptr, a, b, n, nlist, cent, dpad));
        HIP_TRY(tri_build_widen_rows(s, dtype, cent, (uint64_t)nlist * dpad, cent_f32));
    }

    // ---- Lloyd iterations on the training rows
    if (p->train_iters) {
        const uint64_t ns = bt.ns;
        void *train = nullptr;
        uint32_t *perm_s = nullptr, *loff_s = nullptr;
        HIP_TRY(tmp.alloc(&train, bt.train));
        HIP_TRY(tmp.alloc((void **)&perm_s, bt.perm_s));
        HIP_TRY(tmp.alloc((void **)&loff_s, bt.loff_s));
        uint64_t a = 1, b = 0;
        if (ns < n) {
            uint64_t st = p->seed ^ 0x7472696e69747921ull;
            a = splitmix64(st) % n; b = splitmix64(st) % n;
            if (a == 0) a = 1;
            while (gcd64(a, n) != 1) a = a % n + 1;
        }
        for (uint64_t r0 = 0; r0 < ns; r0 += (1u << 20)) {   // (a*(r0+i) + b) mod n, a million rows per launch
            const uint64_t cnt = std::min<uint64_t>(1u << 20, ns - r0);
            HIP_TRY(tri_build_pad_rows(s, dtype, dbase, dim, dim, nullptr, a, (a * r0 + b) % n, n, cnt,
                                       (uint8_t *)train + r0 * rb, dpad));
        }
        const uint32_t nb_s = (uint32_t)std::min<uint64_t>(512, (ns + 255) / 256);
        for (uint32_t it = 0; it < p->train_iters; ++it) {
            HIP_TRY(tri_build_convert_centroids(s, dtype, cent_f32, nlist, dpad, cent));
            HIP_TRY(tri_build_row_norms(s, dtype, cent, dpad, nlist, cnorm));
            rc = assign_all(s, dtype, dim, dpad, rb, nullptr, 0, train, ns, cent, cnorm, nlist, metric, chunk_rows,
                            scores, ldc, chunk, assign);
            if (rc) return rc;
            HIP_TRY(tri_build_partition(s, assign, ns, nlist, block_hist, nb_s, list_len, loff_s, perm_s));
            HIP_TRY(tri_build_cluster_means(s, dtype, train, dpad, loff_s, perm_s, nlist, metric == TRI_IP, cent_f32));
        }
    }

    // ---- final centroids, assignment of every row, list-major store
    HIP_TRY(tri_build_convert_centroids(s, dtype, cent_f32, nlist, dpad, cent));
    HIP_TRY(tri_build_row_norms(s, dtype, cent, dpad, nlist, cnorm));
    rc = assign_all(s, dtype, dim, dpad, rb, dbase, dim, nullptr, n, cent, cnorm, nlist, metric, chunk_rows, scores,
                    ldc, chunk, assign);
    if (rc) return rc;
    HIP_TRY(tri_build_partition(s, assign, n, nlist, block_hist, nblocks, list_len, loff, ids));
    HIP_TRY(hipStreamSynchronize(s));
    std::vector<uint32_t> h_off((size_t)nlist + 1), h_boff((size_t)nlist + 1);
    HIP_TRY(hipMemcpy(h_off.data(), loff, h_off.size() * 4, hipMemcpyDeviceToHost));
    if (h_off[nlist] != n) return tri_fail(TRI_EHIP, "partition produced %u rows, expected %llu", h_off[nlist], (unsigned long long)n);
    // every list in whole blocks of 32 storage slots, the vectors of a block interleaved by 16-byte pieces; slots
    // behind a list's last vector stay zero
    h_boff[0] = 0;
    for (uint32_t l = 0; l < nlist; ++l) h_boff[l + 1] = h_boff[l] + (h_off[l + 1] - h_off[l] + TRI_VB - 1) / TRI_VB;
    HIP_TRY(hipMemcpy(boff, h_boff.data(), h_boff.size() * 4, hipMemcpyHostToDevice));
    HIP_TRY(tri_build_slot_map(s, ids, loff, boff, nlist, n, inv));
    HIP_TRY(hipMemsetAsync(vecs, 0, vec_bytes, s));
    for (uint64_t r0 = 0; r0 < n; r0 += chunk) {
        const uint32_t cnt = (uint32_t)std::min<uint64_t>(chunk, n - r0);
        HIP_TRY(tri_build_pad_rows(s, dtype, dbase, dim, dim, ids + r0, 0, 0, 1, cnt, chunk_rows, dpad));
        HIP_TRY(tri_build_row_norms(s, dtype, chunk_rows, dpad, cnt, vnorm + r0));
        HIP_TRY(tri_build_interleave_rows(s, chunk_rows, rb, r0, cnt, ids, inv, vecs));
    }
    HIP_TRY(tri_launch_fill_u32(s, (uint32_t *)(vnorm + n), 0u, TRI_VB));
    HIP_TRY(hipStreamSynchronize(s));

    // ---- attach
    uint32_t maxlen = 0;
    std::vector<uint32_t> h_len(nlist), h_idx(nlist, id);
    for (uint32_t l = 0; l < nlist; ++l) { h_len[l] = h_off[l + 1] - h_off[l]; maxlen = std::max(maxlen, h_len[l]); }
    if (((uint64_t)maxlen / TRI_VB + 1) * tri_block_stride(rb) >= (1ull << 31))
        return tri_fail(TRI_EINVAL, "longest list (%u vectors of %u bytes) exceeds 2^31 bytes", maxlen, rb);
    tri_index *ix = new (std::nothrow) tri_index();
    if (!ix) return tri_fail(TRI_ENOMEM, "out of host memory");
    ix->pool = P; ix->id = id; ix->p = *p; ix->n = n; ix->dpad = dpad; ix->row_bytes = rb;
    ix->list_base = P->total_lists; ix->max_list_len = maxlen; ix->ids_dev = ids; ix->list_off_dev = loff;
    ix->dev = TriIndexDev{vecs, vnorm, ids, loff, cent, cnorm, inv, boff, dim, dpad, nlist, p->dtype, rb, ix->list_base, maxlen, 0, n};
    hipError_t e = hipMemcpy(P->ws.indexes + id, &ix->dev, sizeof(TriIndexDev), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(P->ws.glist_len + ix->list_base, h_len.data(), (size_t)nlist * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(P->ws.glist_voff + ix->list_base, h_off.data(), (size_t)nlist * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(P->ws.glist_index + ix->list_base, h_idx.data(), (size_t)nlist * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) { delete ix; return tri_fail(TRI_EHIP, "attach copy -> %s", hipGetErrorString(e)); }
    ix->list_len = h_len;
    P->indexes[id] = ix;
    rc = upload_scan_order(P);
    if (rc) { P->indexes[id] = nullptr; delete ix; return rc; }
    P->total_lists += nlist;
    P->attached_row_bytes = std::max(P->attached_row_bytes, rb);
    P->scan_class_mask |= 1u << tri_scan_class(p->dtype, rb);
    set_scan_nt(P);
    drop_graphs(P);                    // (recorded steps cover the indexes attached when they were recorded)
    *out = ix;
    return TRI_OK;
}

void tri_index_view(const tri_index *ix, TriIndexView *out)
{
    out->dev = ix->dev;
    out->stream = ix->pool->stream;
    out->device = ix->pool->device;
    out->n = ix->n;
}

extern "C" int ivf_export(const tri_index *ix, float *centroids, uint64_t *list_off, int64_t *list_ids)
{
    if (!ix) return tri_fail(TRI_EINVAL, "index is NULL");
    HIP_TRY(hipSetDevice(ix->pool->device));
    HIP_TRY(hipStreamSynchronize(ix->pool->stream));
    const uint32_t nlist = ix->p.nlist, dim = ix->p.dim;
    if (centroids) {
        std::vector<uint8_t> raw((size_t)nlist * ix->row_bytes);
        HIP_TRY(hipMemcpy(raw.data(), ix->dev.centroids, raw.size(), hipMemcpyDeviceToHost));
        for (uint32_t l = 0; l < nlist; ++l) {
            const uint8_t *row = raw.data() + (size_t)l * ix->row_bytes;
            for (uint32_t i = 0; i < dim; ++i)
                centroids[(size_t)l * dim + i] = ix->p.dtype == TRI_F16 ? (float)((const _Float16 *)row)[i] : ((const float *)row)[i];
        }
    }
    if (list_off) {
        std::vector<uint32_t> h((size_t)nlist + 1);
        HIP_TRY(hipMemcpy(h.data(), ix->list_off_dev, h.size() * 4, hipMemcpyDeviceToHost));
        for (size_t i = 0; i < h.size(); ++i) list_off[i] = h[i];
    }
    if (list_ids) {
        std::vector<uint32_t> h((size_t)ix->n);
        HIP_TRY(hipMemcpy(h.data(), ix->ids_dev, h.size() * 4, hipMemcpyDeviceToHost));
        for (size_t i = 0; i < h.size(); ++i) list_ids[i] = (int64_t)h[i];
    }
    return TRI_OK;
}

extern "C" int ivf_info(const tri_index *ix, uint64_t *n, uint32_t *dim, uint32_t *nlist, uint32_t *dtype,
                        uint32_t *max_list_len)
{
    if (!ix) return tri_fail(TRI_EINVAL, "index is NULL");
    if (n) *n = ix->n;
    if (dim) *dim = ix->p.dim;
    if (nlist) *nlist = ix->p.nlist;
    if (dtype) *dtype = ix->p.dtype;
    if (max_list_len) *max_list_len = ix->max_list_len;
    return TRI_OK;
}

extern "C" int ivf_destroy(tri_index *ix)
{
    if (!ix) return tri_fail(TRI_EINVAL, "index is NULL");
    tri_pool *P = ix->pool;
    std::lock_guard<std::mutex> lk(P->mu);
    if (!P->failed) {
        if (P->n_running || !P->pending[0].empty() || !P->pending[1].empty())
            return tri_fail(TRI_EINVAL, "ivf_destroy while queries are queued or running");
        int rc = reap(P, true, nullptr);
        if (rc) return rc;
        HIP_TRY(hipStreamSynchronize(P->stream));
    } else {
        (void)hipStreamSynchronize(P->stream);      // (a failed pool is only torn down)
    }
    // finished, unpolled tickets of this index stay valid: their results are already on the host
    P->indexes[ix->id] = nullptr;
    P->attached_row_bytes = 128;
    P->scan_class_mask = 0;
    for (tri_index *o : P->indexes)
        if (o) {
            P->attached_row_bytes = std::max(P->attached_row_bytes, o->row_bytes);
            P->scan_class_mask |= 1u << tri_scan_class(o->p.dtype, o->row_bytes);
        }
    if (ix->list_base + ix->p.nlist == P->total_lists) P->total_lists = ix->list_base;   // last attached: give its list range back
    delete ix;
    set_scan_nt(P);
    drop_graphs(P);
    return P->failed ? TRI_OK : upload_scan_order(P);
}

// ================================================================================== search
extern "C" int search_submit_batch(tri_pool *P, const tri_query *q, uint32_t n, tri_ticket *out, uint32_t *n_done)
{
    if (n_done) *n_done = 0;
    if (!P || (!q && n) || (!out && n)) return tri_fail(TRI_EINVAL, "NULL argument");
    std::lock_guard<std::mutex> lk(P->mu);
    POOL_LIVE(P);
    const tri_index *known = nullptr;
    for (uint32_t i = 0; i < n; ++i) {
        int rc = validate_query(P, &q[i], &known);
        if (rc) return rc;          // (nothing of this call has been queued)
    }
    for (uint32_t i = 0; i < n; ++i) {
        if (P->free_tickets.empty()) {
            return tri_fail(TRI_EAGAIN, "max_outstanding=%u tickets alive", P->cfg.max_outstanding);
        }
        enqueue_locked(P, &q[i], &out[i]);
        if (n_done) *n_done = i + 1;
    }
    return TRI_OK;
}

extern "C" int search_submit_batch_dev(tri_pool *P, const tri_index *index, const void *vecs, uint64_t pitch_bytes,
                                       uint32_t n, const uint32_t *k, const uint32_t *nprobe, const uint32_t *metric,
                                       const uint32_t *klass, tri_ticket *out, uint32_t *n_done)
{
    if (n_done) *n_done = 0;
    if (!P || !index || (n && (!vecs || !k || !nprobe || !metric || !klass || !out))) return tri_fail(TRI_EINVAL, "NULL argument");
    std::lock_guard<std::mutex> lk(P->mu);
    POOL_LIVE(P);
    if (!is_attached(P, index)) return tri_fail(TRI_EINVAL, "index is not attached to this pool");
    const uint32_t es = esize(index->p.dtype);
    if (pitch_bytes % es || pitch_bytes < (uint64_t)index->p.dim * es || (uintptr_t)vecs % es)
        return tri_fail(TRI_EINVAL, "pitch_bytes / vecs must be multiples of the element size and cover dim elements");
    tri_query q{};
    q.index = index;
    q.vec = vecs;
    const tri_index *known = index;
    for (uint32_t i = 0; i < n; ++i) {
        q.k = k[i]; q.nprobe = nprobe[i]; q.metric = metric[i]; q.klass = klass[i];
        int rc = validate_query(P, &q, &known);
        if (rc) return rc;
    }
    // tickets for as many as there is room for, in ascending order: query i's row then goes to store row
    // ticket[i], and stretches of consecutive tickets are copied as runs by one kernel of the pool's stream
    const uint32_t m = (uint32_t)std::min<size_t>(n, P->free_tickets.size());
    std::vector<uint32_t> tk(P->free_tickets.end() - m, P->free_tickets.end());
    std::sort(tk.begin(), tk.end());
    if (m) {
        HIP_TRY(hipSetDevice(P->device));
        TriStageRuns runs{};
        runs.src = (uint64_t)(uintptr_t)vecs; runs.src_pitch = pitch_bytes;
        runs.dst = (uint64_t)(uintptr_t)P->ws.dev_qstore; runs.dst_pitch = P->max_row_bytes;
        runs.row_bytes = index->p.dim * es;
        for (uint32_t i = 0; i < m;) {
            uint32_t j = i + 1;
            while (j < m && tk[j] == tk[j - 1] + 1) ++j;
            runs.run[runs.n_runs].src_first = i; runs.run[runs.n_runs].dst_first = tk[i]; runs.run[runs.n_runs].count = j - i;
            ++runs.n_runs;
            runs.n_rows += j - i;
            if (runs.n_runs == TRI_STAGE_RUNS || j == m) {
                HIP_TRY(tri_launch_stage_rows(P->stream, runs));      // (nothing has been queued yet: the tickets are still free)
                runs.n_runs = runs.n_rows = 0;
            }
            i = j;
        }
    }
    P->free_tickets.resize(P->free_tickets.size() - m);
    for (uint32_t i = 0; i < m; ++i) {
        const uint32_t ti = tk[i];
        Ticket &t = P->tickets[ti];
        t.state = T_PENDING;
        t.cancelled = false;
        t.index = const_cast<tri_index *>(index);
        t.k = k[i]; t.nprobe = nprobe[i]; t.metric = metric[i]; t.klass = klass[i];
        t.tag = 0;
        t.submit_ns = now_ns();
        t.deadline_ns = INT64_MAX;
        t.dev_vec = P->ws.dev_qstore + (size_t)ti * P->max_row_bytes;
        P->pending[t.klass].push_back(ti);
        out[i] = ((uint64_t)t.gen << 32) | ti;
    }
    if (n_done) *n_done = m;
    if (m < n) return tri_fail(TRI_EAGAIN, "max_outstanding=%u tickets alive", P->cfg.max_outstanding);
    return TRI_OK;
}

extern "C" int search_submit(tri_pool *P, const tri_query *q, tri_ticket *out)
{
    if (!q || !out) return tri_fail(TRI_EINVAL, "NULL argument");
    return search_submit_batch(P, q, 1, out, nullptr);
}

namespace {

// Forget the recorded steps (the attached indexes changed, or the pool goes away).
void drop_graphs(tri_pool *P)
{
    (void)hipStreamSynchronize(P->stream);
    for (uint32_t i = 0; i < RING; ++i) {
        StepRec &R = P->ring[i];
        for (uint32_t b = 0; b < 2 * N_SHAPES; ++b) {
            if (R.graph_exec[b]) (void)hipGraphExecDestroy(R.graph_exec[b]);
            if (R.graph[b]) (void)hipGraphDestroy(R.graph[b]);
            R.graph_exec[b] = nullptr;
            R.graph[b] = nullptr;
        }
    }
}

// One period of the control loop, when it is due: the pool's own measurement (P95 of the high class's
// waits since the last period) and the reported signals go through tri_policy_feedback.
void feedback_tick(tri_pool *P)
{
    const int64_t t = now_ns();
    if (P->fb_last_ns && (double)(t - P->fb_last_ns) * 1e-9 < P->fb.period_s) return;
    if (!P->fb_last_ns) { P->fb_last_ns = t; return; }          // the first period starts now
    tri_feedback_signals sg{};
    sg.u_kv = P->fb_u_kv;
    sg.decode_stall = P->fb_stall;
    sg.decode_stall_prev = P->fb_stall_prev;
    sg.wait_p95_s = __builtin_nan("");
    if (!P->fb_waits.empty()) {
        const size_t i95 = (size_t)std::min<double>((double)P->fb_waits.size() - 1.0, std::ceil(0.95 * (double)P->fb_waits.size()) - 1.0);
        std::nth_element(P->fb_waits.begin(), P->fb_waits.begin() + (ptrdiff_t)i95, P->fb_waits.end());
        sg.wait_p95_s = P->fb_waits[i95];
    }
    (void)tri_policy_feedback(&P->fb, &sg, &P->policy, nullptr);
    P->fb_last = sg;
    P->fb_stall_prev = P->fb_stall;
    P->fb_waits.clear();
    P->fb_last_ns = t;
    ++P->fb_periods;
}

// Captured sizes (Sec. 3.2: a step is rounded up to the next captured size, the surplus masked): shape b
// holds up to slots >> shift and items >> shift, shift = 4, 2, 0.
struct StepShape { uint32_t slots, items, groups; };

StepShape step_shape(const tri_pool *P, uint32_t b)
{
    const uint32_t shift = 2u * (N_SHAPES - 1u - b);
    uint32_t n_attached = 0;
    for (const tri_index *ix : P->indexes) n_attached += ix != nullptr;
    StepShape sh;
    sh.slots = std::max(1u, P->cfg.slots >> shift);
    sh.items = std::max(1u, P->cfg.items_per_step >> shift);
    sh.groups = std::min<uint32_t>(TRI_MAX_COARSE_GROUPS, n_attached + sh.slots / P->coarse_rows);
    return sh;
}

// Record the launch sequence of a step that uses ring entry R (its pinned upload and result blocks) at
// captured size b: that many slots admitted and running, that many items, every coarse group they can
// form, every scan kernel variant the attached indexes need.  The kernels take what a step really holds
// from its header, so one recording serves every later step that fits, until the set of attached
// indexes changes.
int record_step(tri_pool *P, StepRec &R, const TriDevWs &W, bool keep_probes, uint32_t b, bool nt)
{
    hipStream_t s = P->stream;
    uint32_t nlist_of[2] = {0, 0};
    for (const tri_index *ix : P->indexes)
        if (ix) nlist_of[ix->p.dtype == TRI_F16] = std::max(nlist_of[ix->p.dtype == TRI_F16], ix->p.nlist);
    const StepShape sh = step_shape(P, b);
    const uint32_t group_rows = std::min(P->coarse_rows, sh.slots);
    hipError_t e = tri_scan_prepare(P->attached_row_bytes, P->scan_class_mask);
    if (e == hipSuccess) e = tri_coarse_prepare();
    if (e != hipSuccess) return tri_fail(TRI_EHIP, "kernel set-up -> %s", hipGetErrorString(e));
    e = hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal);
    if (e != hipSuccess) return tri_fail(TRI_EHIP, "hipStreamBeginCapture -> %s (a pool with TRI_FLAG_GRAPH needs a stream of its own, not the default stream)", hipGetErrorString(e));
    e = tri_launch_pull_block(s, P->ws.upload, R.up_dev,
                              sizeof(TriStepHdr) + (size_t)sh.slots * (sizeof(TriNewDesc) + sizeof(TriPlanEntry)) + 512);
    if (e == hipSuccess) e = tri_launch_admit(P->ctx, P->ws, sh.slots);
    for (uint32_t g = 0; g < sh.groups && e == hipSuccess; ++g) {
        for (int dt = 0; dt < 2 && e == hipSuccess; ++dt)
            if (nlist_of[dt]) e = tri_launch_coarse_gemm_step(P->ctx, P->ws, dt ? TRI_F16 : TRI_F32, g, group_rows, nlist_of[dt]);
        if (e == hipSuccess) e = tri_launch_coarse_select(P->ctx, P->ws, g, group_rows, 0u);
    }
    if (e == hipSuccess) e = tri_launch_pack(P->ctx, W, sh.items, P->total_lists, P->n_order);
    if (e == hipSuccess) e = tri_launch_scan(P->ctx, P->ws, P->attached_row_bytes, P->scan_class_mask, true, nt);
    if (e == hipSuccess) e = tri_launch_threshold(P->ctx, P->ws, sh.slots);
    if (e == hipSuccess) e = tri_launch_scan(P->ctx, P->ws, P->attached_row_bytes, P->scan_class_mask, false, nt);
    if (e == hipSuccess) e = tri_launch_merge(P->ctx, W, sh.slots, keep_probes);
    hipGraph_t g = nullptr;
    const hipError_t e2 = hipStreamEndCapture(s, &g);      // (always: a stream must not be left capturing)
    if (e != hipSuccess || e2 != hipSuccess) {
        if (g) (void)hipGraphDestroy(g);
        return tri_fail(TRI_EHIP, "recording the step -> %s", hipGetErrorString(e != hipSuccess ? e : e2));
    }
    hipGraphExec_t x = nullptr;
    e = hipGraphInstantiate(&x, g, nullptr, nullptr, 0);
    if (e != hipSuccess) {
        (void)hipGraphDestroy(g);
        return tri_fail(TRI_EHIP, "hipGraphInstantiate -> %s", hipGetErrorString(e));
    }
    R.graph[b + (nt ? N_SHAPES : 0)] = g;
    R.graph_exec[b + (nt ? N_SHAPES : 0)] = x;
    return TRI_OK;
}

}  // namespace

extern "C" int search_step(tri_pool *P, tri_step_stats *st)
{
    if (!P) return tri_fail(TRI_EINVAL, "pool is NULL");
    std::lock_guard<std::mutex> lk(P->mu);
    POOL_LIVE(P);
    const int rc_step = step_locked(P, st);
    if (rc_step == TRI_EHIP) {          // queries may have been admitted on the host that the GPU never saw
        P->failed = true;
        P->fail_text = g_err;
    }
    return rc_step;
}

namespace {
int step_locked(tri_pool *P, tri_step_stats *st)
{
    HIP_TRY(hipSetDevice(P->device));
    tri_step_stats stats{};
    int rc = reap(P, false, &stats.finished);
    if (rc) return rc;
    StepRec &R = P->ring[P->step_seq % RING];
    if (R.in_use) {                       // RING steps in flight: wait for the oldest
        HIP_TRY(hipEventSynchronize(R.done));
        rc = reap(P, false, &stats.finished);
        if (rc) return rc;
    }
    const tri_pool_cfg &cfg = P->cfg;
    if (P->fb_on) feedback_tick(P);

    // ---- admit (Sec. 3.3): the free slots are split between the classes by the reserved share, the
    //      high class is taken in arrival or least-slack order, the low class first-in first-out
    P->newq.clear();
    // (the admitted queries are ranked in groups of one index and at most coarse_rows rows; a step's
    // header has room for TRI_MAX_COARSE_GROUPS of them, so admission stops where more could be needed)
    P->index_seen.assign(cfg.max_indexes, 0);
    uint32_t n_distinct = 0;
    {
        uint32_t take[2] = {0, 0};
        const bool hold = P->policy.static_batches && P->n_running > 0;       // (a batch must drain before the next starts)
        tri_policy_split(hold ? 0u : (uint32_t)P->free_slots.size(), (uint32_t)P->pending[0].size(), (uint32_t)P->pending[1].size(),
                         P->policy.high_share, &take[0], &take[1]);
        std::deque<uint32_t> &H = P->pending[TRI_CLASS_HIGH];
        if (P->policy.order_high == TRI_ORDER_SLACK && take[0] && H.size() > 1) {
            const uint32_t n = (uint32_t)H.size();
            std::vector<int64_t> ddl(n);
            std::vector<uint32_t> left(n), ord(n);
            for (uint32_t i = 0; i < n; ++i) {
                const Ticket &t = P->tickets[H[i]];
                ddl[i] = t.deadline_ns;
                left[i] = cfg.lists_per_query_step ? (t.nprobe + cfg.lists_per_query_step - 1) / cfg.lists_per_query_step : 1u;
            }
            tri_policy_slack_order(n, ddl.data(), left.data(), now_ns(), (int64_t)(P->mean_step_s * 1e9), take[0], ord.data());
            std::deque<uint32_t> reordered;       // admitted now: most urgent first; the rest keep their arrival order
            for (uint32_t i = 0; i < n; ++i) reordered.push_back(H[ord[i]]);
            H.swap(reordered);
        }
        for (int klass = 0; klass < 2; ++klass) {
            std::deque<uint32_t> &Q = P->pending[klass];
            for (uint32_t a = 0; a < take[klass]; ++a) {
                const uint32_t ti = Q.front();
                {
                    const uint32_t ix_id = P->tickets[ti].index->id;
                    const uint32_t d = n_distinct + (P->index_seen[ix_id] ? 0u : 1u);
                    if (d + ((uint32_t)P->newq.size() + 1) / P->coarse_rows > TRI_MAX_COARSE_GROUPS) break;
                    P->index_seen[ix_id] = 1;
                    n_distinct = d;
                }
                Q.pop_front();
                const uint32_t slot = P->free_slots.back();
                P->free_slots.pop_back();
                Ticket &t = P->tickets[ti];
                t.state = T_RUNNING;
                t.slot = slot;
                if (P->fb_on && klass == TRI_CLASS_HIGH && P->fb_waits.size() < (1u << 16))
                    P->fb_waits.push_back((float)((double)(now_ns() - t.submit_ns) * 1e-9));
                SlotH &sl = P->slots[slot];
                sl = SlotH{true, ti, t.nprobe, 0u, t.klass, P->admit_seq++, t.index};
                P->run_order[t.klass].push_back(slot);
                P->run_seq[t.klass].push_back(sl.admit_seq);
                ++P->n_running;
                P->newq.push_back(ti);
            }
        }
    }
    const uint32_t n_new = (uint32_t)P->newq.size();
    // group the admitted queries by index (stable) so each index's rows are contiguous
    std::stable_sort(P->newq.begin(), P->newq.end(), [&](uint32_t a, uint32_t b) {
        return P->tickets[a].index->id < P->tickets[b].index->id;
    });
    TriStepHdr *hdr_h = (TriStepHdr *)R.up_host;
    TriNewDesc *desc_h = (TriNewDesc *)(R.up_host + sizeof(TriStepHdr));
    const size_t desc_bytes = round_up_sz((size_t)n_new * sizeof(TriNewDesc), 256);

    // ---- plan: every running slot, higher class first, then admission order
    // (the running slots of each class are kept in admission order; retired ones are dropped here)
    P->order.clear();
    for (int klass = 0; klass < 2; ++klass) {
        std::vector<uint32_t> &ro = P->run_order[klass];
        size_t w = 0;
        for (size_t i = 0; i < ro.size(); ++i) {
            const SlotH &sl = P->slots[ro[i] & 0xFFFFFFFFu];
            if (sl.active && sl.admit_seq == P->run_seq[klass][i]) {
                ro[w] = ro[i];
                P->run_seq[klass][w] = P->run_seq[klass][i];
                ++w;
                P->order.push_back(ro[i]);
            }
        }
        ro.resize(w);
        P->run_seq[klass].resize(w);
    }
    TriPlanEntry *plan_h = (TriPlanEntry *)(R.up_host + sizeof(TriStepHdr) + desc_bytes);
    uint32_t n_plan = 0, n_items = 0, n_retire = 0;
    // Every slot of the step gets a region of the candidate buffer for the pairs the scan's filter lets through.
    // The filter's bound is the k-th best of a sample of 64 vectors per list.  A list of length L is sampled at the
    // rate 64 / L, so each of the k sample scores under the bound stands for L / 64 vectors of its list: about
    // k L / 64 vectors pass, with a relative spread of 1 / sqrt(k), and at most that with L the longest list of the
    // index when all k come from it (long lists are sampled thinnest).  The region holds that with a wide margin,
    // and everything where the sample cannot give a bound (fewer than k sample scores).  A query that still asks
    // for more is not wrong, only slow: the merge kernel then scores its lists again itself.
    const uint64_t cand_pairs = P->score_capacity / 2;
    uint64_t cand_used = 0;
    R.retire.clear();
    for (uint32_t s : P->order) {
        if (n_items >= cfg.items_per_step) break;
        SlotH &sl = P->slots[s];
        const uint32_t remaining = sl.nprobe - sl.cursor;
        uint32_t take = cfg.lists_per_query_step ? std::min(cfg.lists_per_query_step, remaining) : remaining;
        take = std::min(take, cfg.items_per_step - n_items);
        if (take == 0) continue;
        const Ticket &tk = P->tickets[sl.ticket];
        const uint64_t everything = (uint64_t)take * round_up(sl.index->max_list_len, TRI_VB);
        uint64_t want;
        if (P->cand_reserve) {
            want = P->cand_reserve;
        } else if ((uint64_t)tk.k > (uint64_t)take * (TRI_SAMPLE_VECS / 2)) {
            want = everything;                                      // (no bound from so small a sample)
        } else {
            const double per_sample = std::max(1.0, (double)sl.index->max_list_len / TRI_SAMPLE_VECS);
            want = (uint64_t)(((double)tk.k + 6.0 * std::sqrt((double)tk.k) + 12.0) * per_sample) + 64;
        }
        want = std::min<uint64_t>(std::min(want, everything), 0xFFFFFFFFull);
        const uint64_t room = cand_pairs - cand_used;
        if (want > room) {
            if (n_plan > 0 && room < want / 2) continue;            // (it waits for the next step; the first slot of a step always runs)
            want = room;
        }
        TriPlanEntry &e = plan_h[n_plan++];
        e.slot = s; e.cursor = sl.cursor; e.take = take; e.item_base = n_items; e.pad_ = 0;
        e.cand_off = (uint32_t)cand_used; e.cand_cap = (uint32_t)want;
        e.retire_idx = sl.cursor + take == sl.nprobe ? (int32_t)n_retire++ : -1;
        if (e.retire_idx >= 0) R.retire.push_back(sl.ticket);
        n_items += take;
        cand_used += want;
    }
    stats.step = P->step_seq;
    stats.admitted = n_new;
    stats.retired = n_retire;
    stats.running = P->n_running;
    stats.items = n_items;
    stats.capacity = cfg.items_per_step;
    stats.pending_high = (uint32_t)P->pending[0].size();
    stats.pending_low = (uint32_t)P->pending[1].size();
    if (n_new == 0 && n_plan == 0) {
        if (st) *st = stats;
        return TRI_OK;
    }

    // ---- upload block: [header][admission records][plan]; behind it, on the device only, the row area
    const size_t plan_bytes = round_up_sz((size_t)n_plan * sizeof(TriPlanEntry), 256);
    uint32_t row_off = 0;
    for (uint32_t i = 0; i < n_new; ++i) {
        const Ticket &t = P->tickets[P->newq[i]];
        desc_h[i] = TriNewDesc{t.slot, t.index->id, t.metric, t.k, t.nprobe, row_off, (uint64_t)(uintptr_t)t.dev_vec};
        row_off += t.index->row_bytes;     // (its place in the device row area; the kernel fetches the vector itself)
    }
    const size_t up_bytes = sizeof(TriStepHdr) + desc_bytes + plan_bytes;
    // chunk length floor of this step: with fewer tiles than a few per wavefront, cut the lists finer.
    // Tiles are estimated from the item count: below one item per attached list every item is a tile of
    // its own, above it a list's items share tiles of TRI_QT queries.
    const uint64_t per_list = P->n_order ? (n_items + P->n_order - 1) / P->n_order : 1;
    const uint64_t tiles_est = n_items <= P->n_order ? n_items : (uint64_t)P->n_order * ((per_list + TRI_QT - 1) / TRI_QT);
    hdr_h->n16 = (uint32_t)(up_bytes / 16);
    hdr_h->n_new = n_new;
    hdr_h->n_plan = n_plan;
    hdr_h->n_items = n_items;
    hdr_h->min_chunk = tiles_est < 16u * P->ctx.n_cu ? 128u : 1024u;
    hdr_h->desc_off = (uint32_t)sizeof(TriStepHdr);
    hdr_h->plan_off = (uint32_t)(sizeof(TriStepHdr) + desc_bytes);
    hdr_h->rows_off = (uint32_t)up_bytes;
    // coarse ranking of the admitted queries: groups of one index and at most coarse_rows rows
    uint32_t n_groups = 0;
    for (uint32_t a = 0; a < n_new;) {
        tri_index *ix = P->tickets[P->newq[a]].index;
        uint32_t b = a;
        while (b < n_new && P->tickets[P->newq[b]].index == ix) ++b;
        for (uint32_t c = a; c < b; c += P->coarse_rows) {
            if (n_groups == TRI_MAX_COARSE_GROUPS) return tri_fail(TRI_EINVAL, "internal: more coarse groups than the step header holds");
            hdr_h->group[n_groups++] = TriCoarseGroup{c, std::min(P->coarse_rows, b - c), ix->id, desc_h[c].row_off};
        }
        a = b;
    }
    hdr_h->n_groups = n_groups;
    hdr_h->coarse_parity = n_groups ? (P->coarse_steps++ & 1u) : 0u;   // (the coarse kernels act when the step admits queries)
    hdr_h->merge_parity = n_plan ? (P->merge_launches++ & 1u) : 0u;   // (the merge kernels run when the step has a plan)

    if (P->inject_failure) {
        P->inject_failure = false;
        return tri_fail(TRI_EHIP, "injected failure (tri_pool_inject_failure)");
    }
    hipStream_t s = P->stream;
    const bool prof = (cfg.flags & TRI_FLAG_PROFILE) != 0;
    const bool prof_scan = !prof && (cfg.flags & TRI_FLAG_PROFILE_SCAN) != 0;
    const bool replay = (cfg.flags & TRI_FLAG_GRAPH) && !prof && !prof_scan;
    // Everything the host wants back lands in this step's pinned host block, written by the kernels
    // themselves (the stores cross the bus while the kernels work on): no copy after the step.
    // (A result copy on a second stream was tried instead; it ran beside the next step's scan and slowed
    // that by far more than the transfer takes.)
    TriDevWs W = P->ws;
    W.res_block = (uint32_t *)R.down_dev;
    W.res_probes = (uint32_t *)(R.down_dev + P->down_probe_off);
    const bool keep_probes = (cfg.flags & TRI_FLAG_KEEP_PROBES) != 0;
    const bool nt = tri_scan_streams_lists(P->ctx.scan_nt, n_items, P->total_lists);   // (lists read past the caches in this step?)
    if (replay) {
        // Sec. 3.2: the step's launch sequence, recorded once at its fixed, largest shape, is replayed; what
        // this step holds stands in the header the first kernel pulls.
        uint32_t b = 0;                       // the smallest captured size this step fits
        for (; b + 1 < N_SHAPES; ++b) {
            const StepShape sh = step_shape(P, b);
            if (n_new <= sh.slots && n_plan <= sh.slots && n_items <= sh.items && n_groups <= sh.groups) break;
        }
        const uint32_t gi = b + (nt ? N_SHAPES : 0);
        if (!R.graph_exec[gi]) {
            rc = record_step(P, R, W, keep_probes, b, nt);
            if (rc) return rc;
        }
        HIP_TRY(hipGraphLaunch(R.graph_exec[gi], s));
    } else {
        W.step_host = prof || prof_scan ? (TriStepDev *)(R.down_dev + P->down_step_off) : nullptr;
        HIP_TRY(tri_launch_pull_block(s, P->ws.upload, R.up_dev, up_bytes));
        if (prof) HIP_TRY(hipEventRecord(R.ev[0], s));
        HIP_TRY(tri_launch_admit(P->ctx, P->ws, n_new));
        if (prof) HIP_TRY(hipEventRecord(R.ev[1], s));
        for (uint32_t g = 0; g < n_groups; ++g) {
            const tri_index *ix = P->indexes[hdr_h->group[g].index];
            HIP_TRY(tri_launch_coarse_gemm_step(P->ctx, P->ws, (int)ix->p.dtype, g, hdr_h->group[g].m, ix->p.nlist));
            HIP_TRY(tri_launch_coarse_select(P->ctx, P->ws, g, hdr_h->group[g].m, ix->p.nlist));
        }
        if (prof) HIP_TRY(hipEventRecord(R.ev[2], s));
        HIP_TRY(tri_launch_pack(P->ctx, W, n_items, P->total_lists, P->n_order));
        if (prof || (prof_scan && n_items)) HIP_TRY(hipEventRecord(R.ev[3], s));
        // thresholds: score a sample of every probed list, k-th best of each slot's sample
        if (n_items) HIP_TRY(tri_launch_scan(P->ctx, P->ws, P->attached_row_bytes, P->scan_class_mask, true, nt));
        if (prof || (prof_scan && n_items)) HIP_TRY(hipEventRecord(R.ev[4], s));
        if (n_items) HIP_TRY(tri_launch_threshold(P->ctx, P->ws, n_plan));
        if (prof || (prof_scan && n_items)) HIP_TRY(hipEventRecord(R.ev[5], s));
        if (n_items) HIP_TRY(tri_launch_scan(P->ctx, P->ws, P->attached_row_bytes, P->scan_class_mask, false, nt));
        if (prof || (prof_scan && n_items)) HIP_TRY(hipEventRecord(R.ev[6], s));
        HIP_TRY(tri_launch_merge(P->ctx, W, n_plan, keep_probes));
        if (prof) HIP_TRY(hipEventRecord(R.ev[7], s));
    }
    HIP_TRY(hipEventRecord(R.done, s));
    R.in_use = true;
    R.enqueue_ns = now_ns();
    R.profiled = prof;
    R.profiled_scan = prof_scan;
    R.seq = P->step_seq;
    R.n_items = n_items;
    R.had_scan = n_items != 0;

    // ---- host mirror: advance cursors, retire, recycle slots
    for (uint32_t i = 0; i < n_plan; ++i) {
        const TriPlanEntry &e = plan_h[i];
        SlotH &sl = P->slots[e.slot];
        sl.cursor += e.take;
        if (e.retire_idx >= 0) {
            Ticket &t = P->tickets[sl.ticket];
            t.state = T_RETIRING;
            t.step_seq = P->step_seq;
            t.retire_idx = (uint32_t)e.retire_idx;
            sl.active = false;
            P->free_slots.push_back(e.slot);
            --P->n_running;
        }
    }
    ++P->step_seq;
    if (st) *st = stats;
    return TRI_OK;
}
}  // namespace

namespace {
// search_poll without the lock and without the reap; returns TRI_OK / TRI_EAGAIN / TRI_ENOENT / TRI_EINVAL
int poll_locked(tri_pool *P, tri_ticket tk, uint32_t *n_out, int64_t *ids, float *dist, uint32_t room)
{
    uint32_t ti;
    if (!ticket_lookup(P, tk, &ti)) return tri_fail(TRI_ENOENT, "unknown ticket");
    Ticket &t = P->tickets[ti];
    if (t.cancelled) return tri_fail(TRI_ENOENT, "ticket was cancelled");
    if (t.state != T_DONE) return TRI_EAGAIN;
    if (!ids || !dist) return tri_fail(TRI_EINVAL, "ids / dist is NULL");
    if (room < t.k) return tri_fail(TRI_EINVAL, "row of %u entries is too short for k=%u", room, t.k);
    const uint32_t kmax = P->cfg.kmax;
    for (uint32_t i = 0; i < t.n_out; ++i) {
        ids[i] = (int64_t)P->res_ids[(size_t)ti * kmax + i];
        dist[i] = P->res_score[(size_t)ti * kmax + i];
    }
    const float pad = t.metric == TRI_L2 ? __builtin_inff() : -__builtin_inff();
    for (uint32_t i = t.n_out; i < t.k; ++i) { ids[i] = -1; dist[i] = pad; }
    if (n_out) *n_out = t.n_out;
    t.state = T_FREE;
    ++t.gen;
    P->free_tickets.push_back(ti);
    return TRI_OK;
}
}  // namespace

extern "C" int search_poll(tri_pool *P, tri_ticket tk, uint32_t *n_out, int64_t *ids, float *dist)
{
    if (!P) return tri_fail(TRI_EINVAL, "pool is NULL");
    std::lock_guard<std::mutex> lk(P->mu);
    POOL_LIVE(P);
    HIP_TRY(hipSetDevice(P->device));
    int rc = reap(P, false, nullptr);
    if (rc) return rc;
    return poll_locked(P, tk, n_out, ids, dist, 0xFFFFFFFFu);
}

extern "C" int search_poll_batch(tri_pool *P, const tri_ticket *tk, uint32_t n, uint32_t stride, uint32_t *n_out,
                                 int64_t *ids, float *dist, int *status)
{
    if (!P || (n && (!tk || !ids || !dist || !status || !n_out))) return tri_fail(TRI_EINVAL, "NULL argument");
    std::lock_guard<std::mutex> lk(P->mu);
    POOL_LIVE(P);
    HIP_TRY(hipSetDevice(P->device));
    int rc = reap(P, false, nullptr);
    if (rc) return rc;
    int delivered = 0;
    for (uint32_t i = 0; i < n; ++i) {
        status[i] = poll_locked(P, tk[i], &n_out[i], ids + (size_t)i * stride, dist + (size_t)i * stride, stride);
        delivered += status[i] == TRI_OK;
    }
    return delivered;
}

extern "C" int search_probes(tri_pool *P, tri_ticket tk, uint32_t *lists, uint32_t *n_out)
{
    if (!P || !lists) return tri_fail(TRI_EINVAL, "NULL argument");
    std::lock_guard<std::mutex> lk(P->mu);
    if (!(P->cfg.flags & TRI_FLAG_KEEP_PROBES)) return tri_fail(TRI_EINVAL, "pool was created without TRI_FLAG_KEEP_PROBES");
    uint32_t ti;
    if (!ticket_lookup(P, tk, &ti)) return tri_fail(TRI_ENOENT, "unknown ticket");
    Ticket &t = P->tickets[ti];
    if (t.cancelled) return tri_fail(TRI_ENOENT, "ticket was cancelled");
    if (t.state == T_RETIRING) {
        HIP_TRY(hipSetDevice(P->device));
        int rc = reap(P, false, nullptr);
        if (rc) return rc;
    }
    if (t.state != T_DONE) return TRI_EAGAIN;
    memcpy(lists, &P->res_probe[(size_t)ti * P->cfg.nprobe_max], (size_t)t.nprobe * 4);
    if (n_out) *n_out = t.nprobe;
    return TRI_OK;
}

extern "C" int search_cancel(tri_pool *P, tri_ticket tk)
{
    if (!P) return tri_fail(TRI_EINVAL, "pool is NULL");
    std::lock_guard<std::mutex> lk(P->mu);
    uint32_t ti;
    if (!ticket_lookup(P, tk, &ti)) return tri_fail(TRI_ENOENT, "unknown ticket");
    Ticket &t = P->tickets[ti];
    if (t.cancelled) return tri_fail(TRI_ENOENT, "ticket was cancelled");
    if (t.state == T_PENDING) {
        std::deque<uint32_t> &Q = P->pending[t.klass];
        Q.erase(std::find(Q.begin(), Q.end(), ti));
        t.state = T_FREE;
        ++t.gen;
        P->free_tickets.push_back(ti);
    } else if (t.state == T_DONE) {
        t.state = T_FREE;
        ++t.gen;
        P->free_tickets.push_back(ti);
    } else {
        t.cancelled = true;       // running / retiring: freed when its step is reaped
    }
    return TRI_OK;
}

extern "C" int search_sync(tri_pool *P)
{
    if (!P) return tri_fail(TRI_EINVAL, "pool is NULL");
    std::lock_guard<std::mutex> lk(P->mu);
    POOL_LIVE(P);
    HIP_TRY(hipSetDevice(P->device));
    return reap(P, true, nullptr);
}

// ================================================================================== policy
extern "C" int tri_policy_split(uint32_t free_slots, uint32_t n_high, uint32_t n_low, float high_share,
                                uint32_t *take_high, uint32_t *take_low)
{
    if (!take_high || !take_low) return tri_fail(TRI_EINVAL, "NULL argument");
    if (!(high_share >= 0.0f && high_share <= 1.0f)) return tri_fail(TRI_EINVAL, "high_share must lie in [0, 1]");
    // the reserved part first, then the other class up to what is left, then the high class again for the rest
    // (a share given as a rounded float must not reserve a slot more than its decimal value says: 0.1 of 30 is 3)
    const uint32_t reserved = (uint32_t)std::min<double>(free_slots, std::ceil((double)high_share * free_slots - 1e-4));
    const uint32_t first_high = std::min(n_high, reserved);
    const uint32_t low = std::min(n_low, free_slots - first_high);
    *take_high = std::min(n_high, free_slots - low);
    *take_low = low;
    return TRI_OK;
}

extern "C" int tri_policy_slack_order(uint32_t n, const int64_t *deadline_ns, const uint32_t *steps_left, int64_t now_ns_,
                                      int64_t step_ns, uint32_t m, uint32_t *order)
{
    if (n && (!deadline_ns || !steps_left || !order)) return tri_fail(TRI_EINVAL, "NULL argument");
    if (m > n) m = n;
    std::vector<std::pair<int64_t, uint32_t>> v(n);      // (slack, index); no deadline = latest possible slack
    for (uint32_t i = 0; i < n; ++i) {
        const int64_t finish = now_ns_ + (int64_t)steps_left[i] * step_ns;
        v[i] = {deadline_ns[i] == INT64_MAX ? INT64_MAX : deadline_ns[i] - finish, i};
    }
    // only the m most urgent need their exact order: selection is linear in n, sorting costs m log m
    if (m < n) std::nth_element(v.begin(), v.begin() + m, v.end());
    std::sort(v.begin(), v.begin() + m);
    std::vector<uint8_t> chosen(n, 0);
    for (uint32_t i = 0; i < m; ++i) {
        order[i] = v[i].second;
        chosen[v[i].second] = 1;
    }
    uint32_t w = m;
    for (uint32_t i = 0; i < n; ++i)
        if (!chosen[i]) order[w++] = i;
    return TRI_OK;
}

extern "C" int search_set_policy(tri_pool *P, const tri_policy *pol)
{
    if (!P || !pol) return tri_fail(TRI_EINVAL, "NULL argument");
    if (!(pol->high_share >= 0.0f && pol->high_share <= 1.0f)) return tri_fail(TRI_EINVAL, "high_share must lie in [0, 1]");
    if (pol->order_high != TRI_ORDER_FIFO && pol->order_high != TRI_ORDER_SLACK)
        return tri_fail(TRI_EINVAL, "order_high must be TRI_ORDER_FIFO or TRI_ORDER_SLACK");
    if (!(pol->flush_timeout_s >= 0.0) || !(pol->flush_timeout_high_s >= 0.0))
        return tri_fail(TRI_EINVAL, "flush time-outs must not be negative");
    std::lock_guard<std::mutex> lk(P->mu);
    P->policy = *pol;
    return TRI_OK;
}

extern "C" int search_get_policy(tri_pool *P, tri_policy *pol, double *mean_step_s)
{
    if (!P) return tri_fail(TRI_EINVAL, "pool is NULL");
    std::lock_guard<std::mutex> lk(P->mu);
    if (pol) *pol = P->policy;
    if (mean_step_s) *mean_step_s = P->mean_step_s;
    return TRI_OK;
}

extern "C" int search_set_feedback(tri_pool *P, const tri_feedback_cfg *c)
{
    if (!P) return tri_fail(TRI_EINVAL, "pool is NULL");
    std::lock_guard<std::mutex> lk(P->mu);
    if (!c) { P->fb_on = false; return TRI_OK; }
    tri_policy probe = P->policy;
    tri_feedback_signals none{__builtin_nanf(""), __builtin_nanf(""), __builtin_nanf(""), 0.f, __builtin_nan("")};
    if (!(c->period_s >= 0.0) || !(c->wait_p95_budget_s >= 0.0) || !(c->u_kv_band >= 0.0f) ||
        tri_policy_feedback(c, &none, &probe, nullptr) != TRI_OK)
        return tri_fail(TRI_EINVAL, "feedback configuration out of range (0 <= r_min <= r_max <= 1, r_step > 0, tau_factor > 1, "
                                "0 <= tau_min_s <= tau_max_s, period_s, wait_p95_budget_s, u_kv_band >= 0)");
    P->fb = *c;
    P->fb_on = true;
    P->fb_last_ns = 0;
    P->fb_periods = 0;
    P->fb_waits.clear();
    P->fb_stall_prev = __builtin_nanf("");
    P->policy.high_share = std::min(std::max(P->policy.high_share, c->r_min), c->r_max);
    P->policy.flush_timeout_high_s = std::min(std::max(P->policy.flush_timeout_high_s, c->tau_min_s), c->tau_max_s);
    return TRI_OK;
}

extern "C" int search_report_signals(tri_pool *P, float u_kv, float decode_stall)
{
    if (!P) return tri_fail(TRI_EINVAL, "pool is NULL");
    if ((u_kv == u_kv && !(u_kv >= 0.0f && u_kv <= 1.0f)) || (decode_stall == decode_stall && !(decode_stall >= 0.0f && decode_stall <= 1.0f)))
        return tri_fail(TRI_EINVAL, "signals are fractions in [0, 1] (or NaN for unknown)");
    std::lock_guard<std::mutex> lk(P->mu);
    P->fb_u_kv = u_kv;
    P->fb_stall = decode_stall;
    return TRI_OK;
}

extern "C" int search_get_feedback(tri_pool *P, uint64_t *periods, tri_feedback_signals *last)
{
    if (!P) return tri_fail(TRI_EINVAL, "pool is NULL");
    std::lock_guard<std::mutex> lk(P->mu);
    if (periods) *periods = P->fb_periods;
    if (last) *last = P->fb_last;
    return TRI_OK;
}

// ================================================================================== stream driver
// The serving loop of Sec. 3.2 as one native call: arrivals are queued when their time has come, a
// step is enqueued whenever there is work and fewer than `depth` steps are in flight, results are
// collected as soon as their step completes.  No waiting to fill a batch: a step starts with whatever
// is there (the paper's time-out flush with time-out zero).
extern "C" int search_run_stream(tri_pool *P, const tri_query *q, const double *arrival_s, uint32_t n, uint32_t depth,
                                 uint32_t stride, uint32_t *n_out, int64_t *ids, float *dist, double *done_s,
                                 uint32_t *probes, tri_stream_stats *out)
{
    if (!P || !q || !arrival_s || !n_out || !ids || !dist || !done_s) return tri_fail(TRI_EINVAL, "NULL argument");
    if (n == 0) return tri_fail(TRI_EINVAL, "empty stream");
    if (probes && !(P->cfg.flags & TRI_FLAG_KEEP_PROBES))
        return tri_fail(TRI_EINVAL, "probe lists need a pool created with TRI_FLAG_KEEP_PROBES");
    {
        std::lock_guard<std::mutex> lk(P->mu);
        POOL_LIVE(P);
        if (P->free_tickets.size() != P->tickets.size()) return tri_fail(TRI_EINVAL, "the pool has queries in flight");
        const tri_index *known = nullptr;
        for (uint32_t i = 0; i < n; ++i) {
            int rc = validate_query(P, &q[i], &known);
            if (rc) return rc;
            if (q[i].k > stride) return tri_fail(TRI_EINVAL, "query %u: k=%u exceeds the row stride %u", i, q[i].k, stride);
            if (i && arrival_s[i] < arrival_s[i - 1]) return tri_fail(TRI_EINVAL, "arrival times must not decrease");
        }
        P->done_log.clear();
    }
    if (depth == 0) depth = 2;
    if (depth > RING) depth = RING;
    std::vector<uint32_t> q_of_ticket(P->tickets.size());
    const StreamSink sink{q_of_ticket.data(), n_out, ids, dist, probes, stride};
    {
        std::lock_guard<std::mutex> lk(P->mu);
        P->sink = &sink;
    }
    tri_stream_stats acc{};
    using clk = std::chrono::steady_clock;
    const clk::time_point t0 = clk::now();
    auto elapsed = [&]() { return std::chrono::duration<double>(clk::now() - t0).count(); };
    uint32_t next = 0, done = 0;
    int rc = TRI_OK;
    while (done < n && rc == TRI_OK) {
        bool have_work = false;
        uint32_t inflight = 0;
        {
            std::lock_guard<std::mutex> lk(P->mu);
            const double now = elapsed();
            const double t_sub = now;
            // (a burst is taken in in portions, so that the first step does not wait for the last copy)
            uint32_t portion = 2 * P->cfg.slots;
            while (next < n && arrival_s[next] <= now && !P->free_tickets.empty() && portion--) {
                tri_ticket tk;
                enqueue_locked(P, &q[next], &tk);
                q_of_ticket[(uint32_t)(tk & 0xFFFFFFFFull)] = next;
                ++next;
            }
            const double t_col = elapsed();
            acc.submit_s += t_col - t_sub;
            rc = hipSetDevice(P->device) == hipSuccess ? reap(P, false, nullptr) : tri_fail(TRI_EHIP, "hipSetDevice failed");
            if (rc) break;
            if (!P->done_log.empty()) {              // (reap delivered them into the caller's arrays; here: their time)
                const double t = elapsed();
                for (uint32_t qi : P->done_log) done_s[qi] = t;
                done += (uint32_t)P->done_log.size();
                P->done_log.clear();
            }
            acc.collect_s += elapsed() - t_col;
            for (uint32_t i = 0; i < RING; ++i) inflight += P->ring[i].in_use;
            const uint64_t waiting = P->pending[0].size() + P->pending[1].size();
            have_work = P->n_running > 0 || waiting > 0;
            if (waiting > acc.max_pending) acc.max_pending = waiting;
            // flush time-outs (Sec. 3.2 / 3.3): an idle pool whose slot table could not be filled yet waits for
            // more arrivals, but only until its oldest query -- or its oldest high-class query -- has waited long enough
            if (P->n_running == 0 && waiting > 0 && waiting < P->cfg.slots && next < n &&
                (P->policy.flush_timeout_s > 0.0 || P->policy.flush_timeout_high_s > 0.0)) {
                const int64_t t = now_ns();
                bool due = false;
                for (int klass = 0; klass < 2; ++klass)
                    if (!P->pending[klass].empty()) {
                        const double waited = (double)(t - P->tickets[P->pending[klass].front()].submit_ns) * 1e-9;
                        due = due || waited >= P->policy.flush_timeout_s ||
                              (klass == TRI_CLASS_HIGH && waited >= P->policy.flush_timeout_high_s);
                    }
                if (!due) have_work = false;
            }
        }
        if (have_work && inflight < depth) {
            tri_step_stats st;
            const double t_step = elapsed();
            rc = search_step(P, &st);
            acc.step_s += elapsed() - t_step;
            if (rc) break;
            if (st.items) {
                acc.steps += 1;
                acc.items += st.items;
                acc.capacity += st.capacity;
                acc.running += st.running;
            }
        } else if (!have_work && inflight == 0 && next < n) {
            double wait = arrival_s[next] - elapsed() - 100e-6;    // idle until the next arrival (or a flush time-out)
            if (P->policy.flush_timeout_s > 0.0 || P->policy.flush_timeout_high_s > 0.0) wait = std::min(wait, 50e-6);
            if (wait > 100e-6 || (wait > 0 && wait <= 50e-6)) std::this_thread::sleep_for(std::chrono::duration<double>(wait));
        } else {
            std::this_thread::yield();                              // steps in flight: their events are polled above
        }
    }
    acc.wall_s = elapsed();
    {
        std::lock_guard<std::mutex> lk(P->mu);
        P->sink = nullptr;
        P->done_log.clear();
    }
    if (out) *out = acc;
    return rc;
}

extern "C" int tri_pool_set_profiling(tri_pool *P, uint32_t flags)
{
    if (!P) return tri_fail(TRI_EINVAL, "pool is NULL");
    if (flags & ~(uint32_t)(TRI_FLAG_PROFILE | TRI_FLAG_PROFILE_SCAN)) return tri_fail(TRI_EINVAL, "only the profiling flags can be changed");
    std::lock_guard<std::mutex> lk(P->mu);
    P->cfg.flags = (P->cfg.flags & ~(uint32_t)(TRI_FLAG_PROFILE | TRI_FLAG_PROFILE_SCAN)) | flags;
    return TRI_OK;
}

extern "C" int tri_pool_set_replay(tri_pool *P, int on)
{
    if (!P) return tri_fail(TRI_EINVAL, "pool is NULL");
    if (on && !P->stream) return tri_fail(TRI_EINVAL, "a step cannot be recorded on the default stream: give the pool a stream of its own");
    std::lock_guard<std::mutex> lk(P->mu);
    P->cfg.flags = on ? (P->cfg.flags | TRI_FLAG_GRAPH) : (P->cfg.flags & ~(uint32_t)TRI_FLAG_GRAPH);
    return TRI_OK;
}

extern "C" int tri_pool_set_candidate_reserve(tri_pool *P, uint32_t pairs)
{
    if (!P) return tri_fail(TRI_EINVAL, "pool is NULL");
    std::lock_guard<std::mutex> lk(P->mu);
    P->cand_reserve = pairs;
    return TRI_OK;
}

extern "C" int tri_pool_candidate_rescans(tri_pool *P, uint64_t *rescans)
{
    if (!P || !rescans) return tri_fail(TRI_EINVAL, "NULL argument");
    std::lock_guard<std::mutex> lk(P->mu);
    HIP_TRY(hipSetDevice(P->device));
    HIP_TRY(hipStreamSynchronize(P->stream));
    uint32_t v = 0;
    HIP_TRY(hipMemcpy(&v, P->ws.rescans, 4, hipMemcpyDeviceToHost));
    *rescans = v;
    return TRI_OK;
}

extern "C" int tri_pool_inject_failure(tri_pool *P)
{
    if (!P) return tri_fail(TRI_EINVAL, "pool is NULL");
    std::lock_guard<std::mutex> lk(P->mu);
    P->inject_failure = true;
    return TRI_OK;
}

extern "C" int tri_pool_kernel_times(tri_pool *P, tri_kernel_times *out, int reset)
{
    if (!P || !out) return tri_fail(TRI_EINVAL, "NULL argument");
    std::lock_guard<std::mutex> lk(P->mu);
    *out = P->times;
    if (reset) P->times = tri_kernel_times{};
    return TRI_OK;
}

extern "C" const char *tri_last_error(void) { return g_err.c_str(); }
extern "C" const char *tri_version(void) { return "trinity-ivf-mi355x 0.1 (gfx950)"; }
