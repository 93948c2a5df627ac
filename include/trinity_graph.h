/*
 * trinity_graph.h -- C ABI of the pool worker's second engine: the paper's own continuous-batching
 * search over a fixed-degree neighbour graph (Sec. 3.2).
 *
 * The database X (n x dim) and the neighbour list G (n x degree) stay resident in HBM.  Every running
 * request keeps its state on the device: a candidate list topM (ids and scores, best first, with an
 * "expanded" mark per entry) and a visited table that admits only first-seen ids to the distance
 * computation.  One call of graph_step advances ALL running requests by one EXTEND:
 *   1. each request selects up to `parents` non-expanded entries of its topM (best first), reads the
 *      `degree` neighbours of each, drops the ids its visited table has seen and emits the rest as
 *      distance tasks into one cross-request task array of fixed shape (slots x parents x degree; unused
 *      entries are masked);
 *   2. one fixed-shape kernel scores all tasks;
 *   3. the scores return to their requests and are merged into topM; the consumed parents are marked
 *      expanded.  A request whose topM holds the same candidates after the merge as before has finished
 *      (so has one with no parent left, or after max_iters extends): its result -- the first k entries
 *      of topM -- is delivered and its slot is free for the next arrival, which joins the very next step.
 * The paper leaves open how a request starts (here: from the entry points given with the index, which
 * are scored and form the first topM in the step that admits the request; that step is not counted as
 * an extend), the order of topM (here: by (score, id); squared L2 ascending, inner product descending)
 * and the parents chosen (here: the first `parents` non-expanded entries in that order).
 * Results do not depend on which requests share a step.
 *
 * Conventions as in trinity_ivf.h: tri_status return values, [host] / [device] markers, no ownership
 * taken except dev_mem, no CPU fallback; one driver thread calls graph_step / graph_poll / graph_sync,
 * graph_submit may be called from several.  tri_last_error() (trinity_ivf.h) has the text of a failure.
 */
#ifndef TRINITY_GRAPH_H
#define TRINITY_GRAPH_H

#include "trinity_ivf.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tri_gpool tri_gpool;   /* one graph index resident on one GPU + the slot table serving it */

#define TRI_GRAPH_TOPM_LIMIT 256u     /* largest topM                                                     */
#define TRI_GRAPH_TASK_LIMIT 256u     /* largest parents * degree, and largest number of entry points      */
#define TRI_GRAPH_VISITED_HASH 16u     /* tri_graph_cfg.flags                                              */
#define TRI_GRAPH_VISITED_BITS 32u
#define TRI_GRAPH_PAD 0xFFFFFFFFu     /* neighbour entries >= n are padding and are skipped                 */

typedef struct {
    uint32_t slots;            /* S: requests advanced per step                                        */
    uint32_t topm;             /* M: length of a request's candidate list, k <= M <= TRI_GRAPH_TOPM_LIMIT */
    uint32_t parents;          /* p: parents expanded per request and extend; p * degree <= TRI_GRAPH_TASK_LIMIT */
    uint32_t max_iters;        /* a request stops after this many extends at the latest                 */
    uint32_t max_outstanding;  /* tickets alive at once (pending + running + finished, unpolled), >= slots */
    uint32_t groups;           /* the slots are split into this many groups (slot s in group s mod groups); a
                                  call of graph_step advances ONE group, in turn, each on a stream of its
                                  own, with at most one step per group in flight -- so the latency-bound
                                  merge of one group runs beside the bandwidth-bound distance launch of
                                  another, and a step is enqueued knowing which of its group's slots the
                                  previous one freed: 1..4 (0 = 2)                                      */
    uint32_t flags;            /* TRI_FLAG_PROFILE: bracket the step kernel with HIP events;
                                  TRI_GRAPH_VISITED_HASH / TRI_GRAPH_VISITED_BITS: how a request's visited set is kept
                                  (default: whichever is smaller) -- a hash table of ids sized by what one request
                                  can see (entry points + max_iters * parents * degree, at most n), or one bit per
                                  database row; both are exact                                          */
    uint32_t pad_;
    void *hip_stream;          /* stream all work is enqueued on (hipStream_t); NULL = default stream    */
} tri_graph_cfg;

/* Device memory a pool needs for an index of this shape plus its slot state. */
int graph_pool_bytes(const tri_graph_cfg *cfg, uint64_t n, uint32_t dim, uint32_t degree, uint32_t dtype,
                     size_t *dev_bytes /*[host] out*/);

/* Create the pool: copy the vectors (n x dim, row-major, TRI_F32 / TRI_F16) and the neighbour list
 * (n x degree uint32, row-major) into dev_mem, rows padded to a multiple of 256 bytes, and compute
 * |x|^2 per row.  seeds [host]: n_seeds <= TRI_GRAPH_TASK_LIMIT entry points every request starts from
 * (duplicates and entries >= n are ignored).  The caller may free vectors / neighbors / seeds after the
 * call; dev_mem (256-byte aligned, dev_bytes >= graph_pool_bytes) belongs to the pool until it is
 * destroyed.  Synchronous. */
int graph_pool_create(const tri_graph_cfg *cfg, const void *vectors /*[host|device]*/,
                      const uint32_t *neighbors /*[host|device]*/, uint64_t n, uint32_t dim, uint32_t degree,
                      uint32_t dtype, const uint32_t *seeds /*[host]*/, uint32_t n_seeds,
                      void *dev_mem /*[device]*/, size_t dev_bytes, tri_gpool **out);
int graph_pool_destroy(tri_gpool *pool);

/* Queue n queries.  vecs: n rows of dim elements of the index's type, row pitch pitch_bytes; on_device
 * = 0: [host] memory, copied now; != 0: [device] memory, read by the step that admits each query (rows
 * must stay valid until then).  k, metric, klass: [host] arrays of n (klass NULL = all TRI_CLASS_LOW;
 * the high class is admitted first).  TRI_EAGAIN: max_outstanding tickets alive (the first *n_done
 * were queued). */
int graph_submit(tri_gpool *pool, const void *vecs, int on_device, uint64_t pitch_bytes, uint32_t n,
                 const uint32_t *k, const uint32_t *metric, const uint32_t *klass,
                 tri_ticket *out /*[host] n*/, uint32_t *n_done /*[host] out or NULL*/);

typedef struct {
    uint64_t step;
    uint32_t admitted;     /* queries that started in this step                                         */
    uint32_t running;      /* slots occupied while the step runs (as the host knows: a request that has
                              finished on the device still counts until its step has been collected)   */
    uint32_t finished;     /* tickets whose results became pollable during this call                    */
    uint32_t pending;      /* queries still waiting for a slot                                          */
} tri_graph_step_stats;

/* One step of the next group of slots (see tri_graph_cfg.groups): wait for that group's previous step and
 * collect its results (their slots become free), admit waiting queries into the group's free slots (high
 * class first, first-in first-out inside a class), enqueue one extend of every running request of the
 * group.  Only enqueues GPU work.  A call with nothing running in the group and nothing to admit is a no-op. */
int graph_step(tri_gpool *pool, tri_graph_step_stats *stats /*[host] out or NULL*/);

/* Results of n tickets, as search_poll_batch delivers them: row i = best first, padded with id -1 and
 * +inf / -inf; squared L2 is delivered in the difference form sum (x - q)^2 (fp32), recomputed for the k
 * rows handed back and ordered by (that, id), so a stored copy of the query has distance exactly 0 (the
 * search itself ranks by |x|^2 + |q|^2 - 2 x.q); iters[i] (may be NULL) = extends the request ran; evals[i] (may be NULL) = distances it
 * computed.  status[i] = TRI_OK (delivered, ticket consumed), TRI_EAGAIN or TRI_ENOENT.  Returns the
 * number delivered or a negative tri_status. */
int graph_poll(tri_gpool *pool, const tri_ticket *t /*[host] n*/, uint32_t n, uint32_t stride,
               uint32_t *n_out /*[host] n*/, int64_t *ids /*[host] n*stride*/, float *dist /*[host] n*stride*/,
               uint32_t *iters /*[host] n or NULL*/, uint32_t *evals /*[host] n or NULL*/, int *status /*[host] n*/);

/* The serving loop of Sec. 3.2 as one native call, for measuring a stream: query i (vecs [host]: n rows, row
 * pitch pitch_bytes) is queued when arrival_s[i] seconds have passed since the call began, graph_step is
 * called whenever something runs or waits, and every result is stored as soon as its step has been
 * collected: row i of ids / dist (stride entries, >= every k) and n_out[i] as graph_poll fills them,
 * done_s[i] = seconds from the beginning of the call until the result was on the host (latency of query i =
 * done_s[i] - arrival_s[i]).  static_batches != 0 runs the scheme continuous batching replaces: a group of
 * slots admits new requests only when every request of the group has finished.  The pool must be idle and
 * have n free tickets; arrival_s must not decrease. */
typedef struct {
    double wall_s;         /* duration of the call                                                      */
    uint64_t steps;        /* steps enqueued                                                            */
    uint64_t running;      /* occupied slots (as the host knows) summed over those steps                */
    uint64_t max_pending;  /* longest the waiting queue ever was                                        */
} tri_graph_stream_stats;
int graph_run_stream(tri_gpool *pool, const void *vecs /*[host]*/, uint64_t pitch_bytes, const double *arrival_s /*[host] n*/,
                     uint32_t n, const uint32_t *k, const uint32_t *metric, const uint32_t *klass /*[host] n or NULL*/,
                     int static_batches, uint32_t stride, uint32_t *n_out /*[host] n*/, int64_t *ids /*[host] n*stride*/,
                     float *dist /*[host] n*stride*/, double *done_s /*[host] n*/, tri_graph_stream_stats *stats /*[host] out or NULL*/);

/* Block until every enqueued step has completed and collect their results. */
int graph_sync(tri_gpool *pool);

/* Accumulated since the last reset (TRI_FLAG_PROFILE): launches of the step kernel (distances, merge
 * and next extend of every slot of a group), their summed duration (HIP events on the group's stream)
 * and the distance tasks they scored; a task reads one padded row (row_bytes) -- the kernel's
 * algorithmic bytes. */
typedef struct {
    uint64_t steps;
    uint64_t tasks;
    double step_kernel_ms;
    uint32_t row_bytes;
    uint32_t pad_;
} tri_graph_times;
int graph_kernel_times(tri_gpool *pool, tri_graph_times *out /*[host] out*/, int reset);

#ifdef __cplusplus
}
#endif
#endif
