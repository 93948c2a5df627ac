/*
 * trinity_ivf.h -- C ABI of the MI355X vector-search pool worker.
 *
 * One GPU holds several IVF-Flat indexes resident in HBM (paper Sec. 3.2: the vectors and
 * the index structure stay in device memory so that distance evaluation and expansion are
 * pure device-memory operations) and serves retrieval requests of two priority classes
 * (Sec. 3.3: a high-priority prefill queue and a lower-priority decode queue).  Requests are
 * executed by CONTINUOUS BATCHING (Sec. 3.2): every call of search_step advances all running
 * requests by one unit of work, packs the work of all of them into one cross-request task
 * array evaluated by fixed-shape kernels, retires the requests that finished and admits
 * waiting ones into the slots they vacated.  The paper describes this over a graph index
 * (unit = one "extend"); here the index is IVF-Flat and the unit is the scan of up to `p`
 * of a request's probed inverted lists.  Results do not depend on how requests are batched
 * (Sec. 3.2, last paragraph).
 *
 * Conventions
 *  - every function returns a tri_status (0 = ok, negative = error); nothing throws or aborts
 *    across this boundary; tri_last_error() gives a thread-local text for the last failure.
 *  - pointers marked [host] / [device] / [host|device] say where the memory must live.
 *  - the library never takes ownership of caller memory except where stated (dev_ws, pinned_ws, dev_mem).
 *  - a HIP failure inside a step leaves the pool marked failed: every later call on it returns
 *    TRI_EHIP (with the first failure's text) except the destroy calls.
 *  - search_submit* may be called from several threads; search_step / search_poll /
 *    search_sync from one driver thread at a time (calls are serialised by an internal lock).
 *  - argument errors return TRI_EINVAL and change no state.
 *  - there is no CPU fallback: without a usable HIP device every call that needs one fails
 *    with TRI_EHIP.
 */
#ifndef TRINITY_IVF_H
#define TRINITY_IVF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tri_pool tri_pool;   /* slot table, queues, workspaces; one per GPU          */
typedef struct tri_index tri_index; /* one resident IVF-Flat index, attached to a pool      */
typedef uint64_t tri_ticket;        /* names one submitted query until it is polled         */

typedef enum {
    TRI_OK = 0,
    TRI_EINVAL = -1, /* bad argument                                                        */
    TRI_ENOMEM = -2, /* workspace too small / table full in a way that waiting cannot fix    */
    TRI_EAGAIN = -3, /* not yet (poll) / queue full, try again later (submit)               */
    TRI_EHIP = -4,   /* a HIP call failed; see tri_last_error()                             */
    TRI_ENOENT = -5  /* unknown, cancelled or already polled ticket                         */
} tri_status;

enum { TRI_L2 = 0, TRI_IP = 1 };          /* metric: squared L2 (smaller = better), inner product (larger = better) */
enum { TRI_F32 = 0, TRI_F16 = 1 };        /* storage type of an index's vectors and of its queries                  */
enum { TRI_CLASS_HIGH = 0, TRI_CLASS_LOW = 1 }; /* Sec. 3.3: prefill-side (latency critical) / decode-side requests */
enum { TRI_FLAG_PROFILE = 1u,             /* bracket every stage of a step with HIP events (tri_pool_kernel_times)    */
       TRI_FLAG_KEEP_PROBES = 2u,         /* copy each query's probe list back so search_probes() can return it      */
       TRI_FLAG_PROFILE_SCAN = 4u,        /* bracket only the three launches of the list scan (four events): sample_ms,
                                             threshold_ms, scan_ms and the scan_* counters of tri_pool_kernel_times
                                             are filled, the other stage times stay zero                              */
       TRI_FLAG_STREAM_LISTS = 16u,       /* read the inverted lists with non-temporal loads in every step.  Without
                                             the flag the pool does so once the attached indexes hold 1 GB of vectors or
                                             more (several times the caches: the lists only pass through, and keeping
                                             them out leaves the caches to the query rows), and then only in steps whose
                                             lists are probed by 24 queries or fewer on average (a list probed by more
                                             than 32 queries is read once per 32, the second time from the caches).
                                             Results do not depend on it.                                             */
       TRI_FLAG_GRAPH = 8u };             /* Sec. 3.2 (fixed-shape step captured once, replayed): the launch sequence
                                             of a step is recorded as a HIP graph at three captured sizes (1/16, 1/4 and
                                             all of slots and items_per_step; once per size, step in flight and set of
                                             attached indexes); search_step replays the smallest that holds the step, the
                                             surplus workgroups are masked by the counts in the step's upload block.
                                             Needs hip_stream != the default stream (TRI_EINVAL from tri_pool_create).
                                             Results are identical to those without the flag.  Steps that are profiled
                                             (TRI_FLAG_PROFILE*) are launched kernel by kernel.                        */

/* Limits of this implementation (checked, TRI_EINVAL beyond them). */
#define TRI_KMAX_LIMIT 1024u      /* largest k a pool can be configured for           */
#define TRI_NPROBE_LIMIT 1024u    /* largest nprobe a pool can be configured for      */
#define TRI_MAX_ROW_BYTES 4096u   /* padded vector row: dim <= 2048 (fp16), 1024 (fp32) */

typedef struct {
    uint32_t slots;                /* S: running requests held at once (the slot count of Sec. 3.3)        */
    uint32_t items_per_step;       /* W: capacity of the cross-request task array, in (query, list) items    */
    uint32_t lists_per_query_step; /* p: lists a request may scan per step; 0 = all that remain             */
    uint32_t kmax;                 /* largest k accepted                                                   */
    uint32_t nprobe_max;           /* largest nprobe accepted                                              */
    uint32_t max_indexes;          /* indexes that may be attached                                         */
    uint32_t max_total_lists;      /* sum of nlist over all attached indexes                               */
    uint32_t max_nlist;            /* largest nlist of one index                                           */
    uint32_t max_dim;              /* largest dim of one index                                             */
    uint32_t max_outstanding;      /* tickets alive at once (pending + running + finished, not yet polled)  */
    uint32_t coarse_rows;          /* new queries ranked against centroids per launch (0 = default 1024)    */
    uint32_t flags;                /* TRI_FLAG_*                                                           */
    uint64_t score_capacity;       /* 4-byte words of the step's candidate buffer: 2 per candidate the scan's filter lets
                                      through; every query of a step gets a region of it sized by what is expected to pass
                                      (about k * list length / 64 with a wide margin), see tri_pool_set_candidate_reserve.
                                      0 = 2 * (1024 * slots + 32 * W) */
    void *hip_stream;              /* hipStream_t all work is enqueued on (NULL = the null stream)          */
} tri_pool_cfg;

/* Bytes a pool with this configuration needs: dev_bytes of device workspace (256-byte aligned start) and
 * pinned_host_bytes of page-locked host memory (upload and result blocks of the steps in flight and a store
 * of max_outstanding padded query rows).  pinned_host_bytes may be NULL. */
int tri_pool_workspace_bytes(const tri_pool_cfg *cfg /*[host]*/, size_t *dev_bytes /*[host] out*/,
                             size_t *pinned_host_bytes /*[host] out or NULL*/);

/* Create a pool on the current HIP device.  All memory is the caller's:
 *  dev_ws [device]: at least dev_bytes as reported above, 256-byte aligned; owned by the pool until
 *      tri_pool_destroy (the caller frees it afterwards).  The pool clears part of it here, on its own
 *      stream, and from then on keeps state in it: no work still pending on another stream may write into it
 *      (memory recycled by a stream-ordered allocator of another stream can be: take it on the pool's stream,
 *      or synchronise that stream first).  The same holds for dev_mem and tmp_dev of ivf_build.
 *  pinned_ws [host, page-locked and mapped for the device: hipHostMalloc, a torch tensor with
 *      pin_memory=True] of at least pinned_host_bytes, 256-byte aligned; owned by the pool until
 *      tri_pool_destroy; TRI_EINVAL if the device cannot address it.  NULL: the pool allocates that much
 *      with hipHostMalloc itself and frees it in tri_pool_destroy.
 * No device memory is ever allocated by the pool. */
int tri_pool_create(const tri_pool_cfg *cfg /*[host]*/, void *dev_ws /*[device]*/, size_t dev_ws_bytes,
                    void *pinned_ws /*[host, pinned] or NULL*/, size_t pinned_ws_bytes, tri_pool **out /*[host] out*/);

/* tri_pool_create for callers that cannot allocate device memory at all (a harness that forbids
 * hipMalloc, a process that must not grow its footprint while serving): the device workspace is a
 * fixed array of TRI_STATIC_WS_BYTES inside the library's own image, present once on every GPU the
 * library is loaded on, and the pinned memory is always the caller's (pinned_ws must not be NULL).
 * The call allocates and frees no device or pinned memory (no hipMalloc, hipHostMalloc, hipFree);
 * the pool's host-side tables and events are created as in tri_pool_create.
 *  - TRI_ENOMEM: the configuration needs more than TRI_STATIC_WS_BYTES of workspace (the text says
 *    how much); TRI_EAGAIN: another pool created by this call is still alive on the device -- all
 *    such pools of a device share the one array, so only one may exist at a time, and whatever an
 *    earlier pool left in it is cleared before the new pool uses it.
 *  - Everything else (indexes, search calls, tri_pool_destroy) works as with tri_pool_create;
 *    ivf_build takes its memory from the caller as usual. */
#define TRI_STATIC_WS_BYTES (64u << 20)
int tri_pool_create_static(const tri_pool_cfg *cfg /*[host]*/, void *pinned_ws /*[host, pinned]*/,
                           size_t pinned_ws_bytes, tri_pool **out /*[host] out*/);

/* Destroy the pool.  Waits for enqueued work; every ticket becomes invalid.  Indexes attached
 * to it must be destroyed first (TRI_EINVAL otherwise). */
int tri_pool_destroy(tri_pool *pool);

/* ---------------------------------------------------------------------------------------
 * Index construction (not on the timed path).  IVF-Flat: nlist centroids, every base vector
 * stored in the inverted list of its best centroid under build_metric (IVF is the index
 * family named in the paper's introduction; its graph index is replaced by this).
 * ------------------------------------------------------------------------------------- */
typedef struct {
    uint32_t dim;          /* vector length (elements); stored rows are zero-padded to a multiple of 128 B */
    uint32_t nlist;        /* number of inverted lists                                             */
    uint32_t dtype;        /* TRI_F32 / TRI_F16: type of base, queries and stored centroids         */
    uint32_t build_metric; /* TRI_L2: Lloyd k-means, TRI_IP: spherical k-means (normalised means)   */
    uint32_t train_iters;  /* Lloyd iterations run from the initial centroids (0 = use them as given) */
    uint64_t seed;         /* seeds the choice of initial rows when no centroids are given          */
} ivf_params;

/* Device bytes the finished index occupies for n base vectors. */
int ivf_build_bytes(const ivf_params *p /*[host]*/, uint64_t n, size_t *dev_bytes /*[host] out*/);

/* Device bytes of temporary memory ivf_build needs for these parameters (training copy, score blocks,
 * assignment tables; base_on_host != 0 adds a device copy of the base). */
int ivf_build_tmp_bytes(const ivf_params *p /*[host]*/, uint64_t n, int base_on_host, size_t *tmp_bytes /*[host] out*/);

/* Build an index and attach it to the pool.
 *  base [host|device]: row-major n x dim, of p->dtype; copied and reordered list by list, the
 *      caller may free it when the call returns.
 *  centroids [host] or NULL: nlist x dim fp32 initial centroids.  NULL: nlist distinct base rows
 *      chosen from p->seed.  Training uses all rows when n <= 256*nlist, otherwise a fixed
 *      pseudo-random subset of 256*nlist rows; an empty cluster keeps its centroid.
 *  dev_mem [device]: ivf_build_bytes() bytes, 256-byte aligned; owned by the index until
 *      ivf_destroy.
 *  tmp_dev [device]: ivf_build_tmp_bytes() bytes of scratch, 256-byte aligned, free again when the
 *      call returns (TRI_ENOMEM if too small).  NULL: the call allocates its temporary memory with
 *      hipMalloc and frees it before it returns.
 * Synchronous.  Must not run while the pool has queries in flight (TRI_EINVAL). */
int ivf_build(tri_pool *pool, const ivf_params *p /*[host]*/, const void *base /*[host|device]*/, uint64_t n,
              const float *centroids /*[host] or NULL*/, void *dev_mem /*[device]*/, size_t dev_mem_bytes,
              void *tmp_dev /*[device] or NULL*/, size_t tmp_bytes, tri_index **out /*[host] out*/);

/* Copy the searchable content of an index to host arrays: centroids [nlist x dim] -- exactly the
 * stored values the coarse ranking uses, widened to fp32 --, list_off [nlist+1], list_ids [n]
 * (base-row numbers, list after list, ascending inside a list).  Any pointer may be NULL. */
int ivf_export(const tri_index *index, float *centroids /*[host]*/, uint64_t *list_off /*[host]*/,
               int64_t *list_ids /*[host]*/);

/* Shape of an index: n, dim, nlist, dtype, longest list.  Any pointer may be NULL. */
int ivf_info(const tri_index *index, uint64_t *n, uint32_t *dim, uint32_t *nlist, uint32_t *dtype,
             uint32_t *max_list_len);

/* Detach and forget the index (its dev_mem returns to the caller).  TRI_EINVAL while the pool
 * has queries in flight.  Finished results of its queries that have not been polled yet stay pollable; its
 * place in the pool (and, if it was the index attached last, its range of the list table) is free for the
 * next ivf_build; a later submit that still names the handle is refused with TRI_EINVAL. */
int ivf_destroy(tri_index *index);

/* ---------------------------------------------------------------------------------------
 * Search.  One query = one request of Sec. 3.2: it waits in its class's queue, is admitted
 * into a free slot at a step boundary, contributes work items to successive steps and is
 * retired -- its slot recycled -- in the step that scans its last probed list.
 * ------------------------------------------------------------------------------------- */
typedef struct {
    const tri_index *index; /* target index (attached to the pool)                                 */
    const void *vec;        /* [host] dim elements of the index's dtype; copied at submit            */
    uint32_t k;             /* 1..kmax results wanted                                               */
    uint32_t nprobe;        /* 1..min(nprobe_max, nlist) inverted lists to scan                     */
    uint32_t metric;        /* TRI_L2 / TRI_IP: used for the coarse ranking AND the list scan       */
    uint32_t klass;         /* TRI_CLASS_HIGH / TRI_CLASS_LOW                                       */
    uint64_t deadline_ns;   /* latency budget in ns from the moment of submission (the L_pre,max of
                               Sec. 3.3: deadline = arrival + budget); 0 = none.  Used by
                               TRI_ORDER_SLACK, see tri_policy                                      */
    uint64_t user_tag;      /* carried, not interpreted                                             */
} tri_query;

/* Queue one query / n queries.  TRI_EAGAIN: max_outstanding tickets are alive (none queued by
 * this call; for a batch, the first *n_done were queued). */
int search_submit(tri_pool *pool, const tri_query *q /*[host]*/, tri_ticket *out /*[host] out*/);
int search_submit_batch(tri_pool *pool, const tri_query *q /*[host] n*/, uint32_t n,
                        tri_ticket *out /*[host] n*/, uint32_t *n_done /*[host] out or NULL*/);

/* Queue n queries against ONE index whose vectors already live in device memory (for instance
 * the output of an embedding model on the same GPU).  vecs [device]: n rows of dim elements of the
 * index's dtype, row pitch pitch_bytes (a multiple of the element size).  The rows are copied into
 * the pool's own store by a kernel this call enqueues on the pool's stream: like any stream-ordered
 * operand they must stay valid and unchanged until the stream has passed that point -- work enqueued
 * on the same stream afterwards may overwrite or free them; another stream, or the host, must wait
 * for the pool's stream first.  k / nprobe / metric / klass: [host] arrays of n.  Same return values
 * as search_submit_batch. */
int search_submit_batch_dev(tri_pool *pool, const tri_index *index, const void *vecs /*[device]*/,
                            uint64_t pitch_bytes, uint32_t n, const uint32_t *k, const uint32_t *nprobe,
                            const uint32_t *metric, const uint32_t *klass, tri_ticket *out /*[host] n*/,
                            uint32_t *n_done /*[host] out or NULL*/);

typedef struct {
    uint64_t step;        /* sequence number of this step                                          */
    uint32_t admitted;    /* queries moved from the queues into slots                              */
    uint32_t retired;     /* queries whose last list is scanned by this step                       */
    uint32_t running;     /* slots occupied while the step runs                                    */
    uint32_t items;       /* real (query, list) work items packed                                  */
    uint32_t capacity;    /* W: the difference to `items` is masked padding                        */
    uint32_t pending_high, pending_low; /* still waiting after admission                           */
    uint32_t finished;    /* tickets whose results became pollable during this call                 */
} tri_step_stats;

/* One step: admit (by the policy in force, see tri_policy; default: high class first, FIFO
 * inside a class) -> coarse ranking of the admitted queries -> pack the work items of all
 * running queries (items of queries admitted in this very call included; higher class first
 * when W is short) -> per-query thresholds from a sample of every probed list -> list scan,
 * keeping what is not beyond the thresholds (which never costs a true result) -> per-query
 * top-k merge -> retire.  Only enqueues GPU work and returns; results of the retired queries
 * become pollable when that work completes.  A call with nothing to do is a no-op. */
int search_step(tri_pool *pool, tri_step_stats *stats /*[host] out or NULL*/);

/* Result of a finished query, best first (L2 ascending, IP descending; equal scores by
 * ascending id).  ids/dist [host]: room for the query's k entries.  *n_out = number of valid
 * entries (fewer than k only if the probed lists hold fewer vectors); the tail is filled with
 * id -1 and +inf (L2) / -inf (IP).  Ids are base-row numbers.  TRI_OK consumes the ticket;
 * TRI_EAGAIN = not finished yet (does not block); TRI_ENOENT = no such ticket. */
int search_poll(tri_pool *pool, tri_ticket t, uint32_t *n_out, int64_t *ids /*[host] k*/, float *dist /*[host] k*/);

/* search_poll for n tickets in one call.  ids/dist [host]: n rows of `stride` entries, stride >= every
 * polled ticket's k (a row is filled like search_poll fills its arrays).  status[i] receives what
 * search_poll would have returned for ticket i.  Returns the number of tickets delivered (>= 0), or a
 * negative tri_status for an argument error. */
int search_poll_batch(tri_pool *pool, const tri_ticket *t /*[host] n*/, uint32_t n, uint32_t stride,
                      uint32_t *n_out /*[host] n*/, int64_t *ids /*[host] n*stride*/, float *dist /*[host] n*stride*/,
                      int *status /*[host] n*/);

/* The probe list (centroid numbers, best first) of a finished, not yet polled query; needs
 * TRI_FLAG_KEEP_PROBES.  lists [host]: room for the query's nprobe entries. */
int search_probes(tri_pool *pool, tri_ticket t, uint32_t *lists /*[host]*/, uint32_t *n_out);

/* Drop a query.  Queued: removed at once.  Running: runs to completion, result discarded.
 * Finished: result discarded. */
int search_cancel(tri_pool *pool, tri_ticket t);

/* Block until all enqueued steps have completed and their results are pollable. */
int search_sync(tri_pool *pool);

/* ---------------------------------------------------------------------------------------
 * Scheduling policy at step boundaries (Sec. 3.3: two queues, a reserved share for the
 * latency-critical one, deadline-and-slack order inside it, short flush time-outs).  The high
 * class plays the part of the paper's prefill queue, the low class that of its decode queue.
 * May be changed between steps at any time; the paper's control loop, which does so every few
 * hundred milliseconds, is search_set_feedback below.
 * ------------------------------------------------------------------------------------- */
enum { TRI_ORDER_FIFO = 0, TRI_ORDER_SLACK = 1 };
typedef struct {
    float high_share;       /* r in [0,1]: of the N slots free at a boundary, ceil(r*N) are offered to
                               the high class first and the rest to the low class first; what one
                               class cannot use goes to the other.  1 (default): high class first   */
    uint32_t order_high;    /* TRI_ORDER_FIFO (default): high-class queue in arrival order.
                               TRI_ORDER_SLACK: least slack first, slack = deadline - (now + E * T),
                               E = steps the query still needs = ceil(nprobe / p), T = measured mean
                               duration of a step; queries without a deadline come last, in arrival
                               order.  The low class is always first-in first-out                  */
    double flush_timeout_s;      /* search_run_stream only: an idle pool (nothing running) starts its next
                                    step when its slot table can be filled, or when the oldest waiting
                                    query has waited this long (0, default: at once) ...              */
    double flush_timeout_high_s; /* ... or when the oldest waiting high-class query has waited this long */
    uint32_t static_batches;     /* != 0: for comparison, the scheme continuous batching replaces -- queries are
                                    admitted only when no query is running, so a batch drains before the next
                                    starts (0, default: arrivals join at every step boundary, Sec. 3.2)       */
    uint32_t pad_;
} tri_policy;
int search_set_policy(tri_pool *pool, const tri_policy *policy /*[host]*/);
/* The policy in force and T, the mean step duration the slack order uses (seconds; 0 before the
 * first step has completed).  Either output may be NULL. */
int search_get_policy(tri_pool *pool, tri_policy *policy /*[host] out*/, double *mean_step_s /*[host] out*/);

/* The two rules above as pure functions (no GPU, no pool), the way search_step applies them.
 * tri_policy_split: how many queries of each class are admitted into free_slots slots.
 * tri_policy_slack_order: order[0..m) = the m indices of least slack, by ascending slack (ties and
 * queries without a deadline, deadline_ns[i] = INT64_MAX, by index); order[m..n) = the other indices,
 * ascending (they keep their arrival order).  Deadlines and now on one clock, in ns. */
int tri_policy_split(uint32_t free_slots, uint32_t n_high, uint32_t n_low, float high_share,
                     uint32_t *take_high /*[host] out*/, uint32_t *take_low /*[host] out*/);
int tri_policy_slack_order(uint32_t n, const int64_t *deadline_ns /*[host] n*/, const uint32_t *steps_left /*[host] n*/,
                           int64_t now_ns, int64_t step_ns, uint32_t m, uint32_t *order /*[host] n out*/);

/* ---------------------------------------------------------------------------------------
 * The control loop of Sec. 3.3 (last part): every period it moves the reserved share r
 * (tri_policy.high_share) and the high-class flush time-out tau_pre (flush_timeout_high_s) by
 * what it is told about the serving system and what the pool measures itself:
 *   u_kv          utilisation of the KV-cache link between the prefill and decode pools, in [0,1]
 *                 (reported by the caller: it is measured outside this library);
 *   decode_stall  fraction of decode time stalled waiting for retrieval, in [0,1] (reported);
 *   wait_p95      95th percentile of the time high-class queries waited between submission and
 *                 admission since the last period (measured by the pool).
 * One period, in this order (the paper gives the directions, not the amounts: steps and factors
 * are parameters):
 *   1. u_kv < u_kv_target - u_kv_band: the high class must be served faster -> r += r_step, or,
 *      with r already at r_max, tau_pre /= tau_factor;
 *   2. wait_p95 > wait_p95_budget_s: tau_pre /= tau_factor;
 *   3. if 1. did not apply and decode_stall > stall_target and decode_stall is higher than at
 *      the last period: r -= r_step (the low class takes more of a batch);
 *   4. if none of 1.-3. applied and wait_p95 <= wait_p95_budget_s / 2 (or nothing waited):
 *      tau_pre *= tau_factor (relaxes towards tau_max_s).
 * r stays in [r_min, r_max], tau_pre in [tau_min_s, tau_max_s].  A signal that is NaN is unknown
 * and its rules do not apply.
 * ------------------------------------------------------------------------------------- */
typedef struct {
    float r_min, r_max, r_step;          /* 0 <= r_min <= r_max <= 1, r_step > 0                          */
    float tau_factor;                    /* > 1                                                           */
    double tau_min_s, tau_max_s;         /* 0 <= tau_min_s <= tau_max_s                                   */
    float u_kv_target, u_kv_band;        /* target utilisation of the KV link and the dead band below it  */
    float stall_target;                  /* decode stall fraction that is tolerated                       */
    float pad_;
    double wait_p95_budget_s;            /* high-class wait (submission to admission) that is tolerated   */
    double period_s;                     /* time between two adjustments (paper: a few hundred ms)        */
} tri_feedback_cfg;
typedef struct {
    float u_kv, decode_stall, decode_stall_prev, pad_;
    double wait_p95_s;
} tri_feedback_signals;
/* One period of the loop as a pure function (no GPU, no pool): policy is read and updated in place;
 * *rules (may be NULL) receives a bit per rule 1..4 that applied (bit 0 = rule 1). */
int tri_policy_feedback(const tri_feedback_cfg *cfg, const tri_feedback_signals *sig, tri_policy *policy /*in/out*/,
                        uint32_t *rules /*[host] out or NULL*/);
/* Run the loop inside the pool: search_step applies tri_policy_feedback to the policy in force whenever
 * period_s has passed since the last time.  cfg = NULL switches it off.  The policy's high_share and
 * flush_timeout_high_s are clamped into the configured ranges at once. */
int search_set_feedback(tri_pool *pool, const tri_feedback_cfg *cfg /*[host] or NULL*/);
/* Latest values of the signals measured outside the library (any thread); NaN = unknown. */
int search_report_signals(tri_pool *pool, float u_kv, float decode_stall);
/* Periods applied so far and the signals the last one saw (either output may be NULL). */
int search_get_feedback(tri_pool *pool, uint64_t *periods /*[host] out*/, tri_feedback_signals *last /*[host] out*/);

/* The serving loop of Sec. 3.2 (arrivals join at the next batch boundary, finished requests leave
 * at once) as one native call, for measuring a stream: query i is
 * queued when arrival_s[i] seconds have passed since the call began (its vector is copied then), a
 * step is enqueued whenever there is work and fewer than `depth` steps are in flight (0 = 2; at most
 * 4) -- never waiting for a batch to fill --, and every result is stored as soon as its step has
 * completed.  The pool must be idle when the call begins; it returns when all n queries are answered.
 *  q, arrival_s [host] n: the queries (arrival times in seconds, not decreasing).
 *  stride: entries per output row, >= every query's k.
 *  n_out [host] n, ids / dist [host] n*stride: filled like search_poll fills them, row i for query i.
 *  done_s [host] n: seconds from the beginning of the call until the result of query i was on the
 *      host; latency of query i = done_s[i] - arrival_s[i].
 *  probes [host] n*nprobe_max or NULL: the probe list of query i in row i (needs TRI_FLAG_KEEP_PROBES).
 *  stats [host] out or NULL. */
typedef struct {
    double wall_s;         /* duration of the call                                                  */
    uint64_t steps;        /* steps that scanned something                                          */
    uint64_t items;        /* work items over those steps                                           */
    uint64_t capacity;     /* W summed over those steps: 1 - items / capacity is the padding share   */
    uint64_t running;      /* occupied slots summed over those steps                                */
    uint64_t max_pending;  /* longest the two queues together ever were                             */
    double submit_s;       /* host time spent queueing arrivals (copies of the query vectors)        */
    double step_s;         /* host time spent inside search_step (planning, enqueueing; includes waiting
                              for the oldest step when `depth` are in flight)                       */
    double collect_s;      /* host time spent collecting finished results                           */
} tri_stream_stats;
int search_run_stream(tri_pool *pool, const tri_query *q /*[host] n*/, const double *arrival_s /*[host] n*/, uint32_t n,
                      uint32_t depth, uint32_t stride, uint32_t *n_out /*[host] n*/, int64_t *ids /*[host] n*stride*/,
                      float *dist /*[host] n*stride*/, double *done_s /*[host] n*/, uint32_t *probes /*[host] or NULL*/,
                      tri_stream_stats *stats /*[host] out or NULL*/);

/* Accumulated GPU time per kernel class since pool creation or the last reset (needs
 * TRI_FLAG_PROFILE; measured with HIP events on the pool's stream around each launch group). */
typedef struct {
    uint64_t steps;          /* profiled steps accumulated                                        */
    double admit_ms;         /* query rows into slots                                              */
    double coarse_ms;        /* centroid contraction + top-nprobe selection                        */
    double pack_ms;          /* work-item array and tile table                                     */
    double sample_ms;        /* sample launch of the list scan (the first 64 vectors of every probed list) */
    double threshold_ms;     /* per-query thresholds from the sample (and its candidates)           */
    double scan_ms;          /* main launch of the list scan                                       */
    double select_ms;        /* per-query top-k merge, result copy-out enqueue                     */
    uint64_t scan_launches;  /* list-scan kernel launches                                          */
    uint64_t scan_vector_bytes; /* bytes of inverted-list vectors those launches had to read: each
                                   (list, query-group) tile counted once; a list's first 64 vectors
                                   are scored by the sample launch and not counted here             */
    uint64_t scan_unique_bytes; /* same, each distinct list counted once per step                  */
    uint64_t scan_items;     /* work items scanned                                                 */
    uint64_t scan_list_bytes;   /* bytes of every distinct probed list, whole, once per step: what the three
                                   launches of the scan stage together have to read                 */
} tri_kernel_times;
int tri_pool_kernel_times(tri_pool *pool, tri_kernel_times *out /*[host] out*/, int reset);
/* Switch the profiling of the steps enqueued from now on: flags = 0, TRI_FLAG_PROFILE or
 * TRI_FLAG_PROFILE_SCAN (the other flags of the pool are fixed at creation). */
int tri_pool_set_profiling(tri_pool *pool, uint32_t flags);
/* Sec. 3.2 (captured fixed-shape step): switch TRI_FLAG_GRAPH for the steps enqueued from now on: on != 0 =
 * replay the recorded launch sequence, 0 = launch kernel by kernel.  TRI_EINVAL for a pool on the default
 * stream (a step cannot be recorded there). */
int tri_pool_set_replay(tri_pool *pool, int on);

/* Measurement helper (the paper's Sec. 2 roofline takes the memory bandwidth as given): the rate at which a
 * bare streaming-read kernel reads dev_buf [device] (bytes >= 1 MiB, 16-byte aligned; read-only) `repeats`
 * times in a row on hip_stream, timed with HIP events, the best of a few launch shapes with plain and with
 * non-temporal loads -- the achievable figure to quote beside the vendor's peak.  dev_sink [device]: 4 writable bytes.  Synchronous. */
int tri_stream_read_bandwidth(const void *dev_buf, size_t bytes, void *dev_sink, void *hip_stream, uint32_t repeats,
                              double *gb_per_s /*[host] out*/);

/* Candidate pairs reserved per query and step: 0 (default) = the estimate from k and the index's list lengths;
 * otherwise exactly `pairs` (never more than the query's lists hold).  A query whose scan lets more pass than was
 * reserved still gets the exact result: the top-k merge notices and scores that query's lists of the step again
 * itself, which is slow.  tri_pool_candidate_rescans counts how often that has happened since the pool was created
 * (synchronises with the pool's stream). */
int tri_pool_set_candidate_reserve(tri_pool *pool, uint32_t pairs);
int tri_pool_candidate_rescans(tri_pool *pool, uint64_t *rescans /*[host] out*/);

/* Testing aid: the next search_step that has work to enqueue fails as if one of its launches had
 * failed (TRI_EHIP), after it has admitted its queries.  A pool in which a step failed half-way is
 * marked failed for good: its slot table no longer matches what the GPU holds, so every later call
 * on it returns TRI_EHIP, except ivf_destroy and tri_pool_destroy, which tear it down. */
int tri_pool_inject_failure(tri_pool *pool);

const char *tri_last_error(void);
const char *tri_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TRINITY_IVF_H */
