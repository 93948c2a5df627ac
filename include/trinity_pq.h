/*
 * trinity_pq.h -- C ABI of IVF search over product-quantised lists, the compressed variant of the inverted-file
 * index that the paper's Sec. 1 names beside IVF-Flat as what a vector pool serves.
 *
 * Built on a resident IVF index (trinity_ivf.h: ivf_build): its centroids and lists decide which vectors are a
 * query's candidates, exactly as for IVF-Flat.  What is scored are not the stored vectors but their codes:
 *   - the dim coordinates are cut into m consecutive sub-vectors of dim/m coordinates; sub-space j has a codebook
 *     of TRI_PQ_KSUB = 256 entries (rows of dim/m fp32 values);
 *   - a stored vector's code is, per sub-space, the number of the entry nearest (squared L2) to its sub-vector,
 *     ties to the smaller number: m bytes per vector instead of a row;
 *   - a query's score against a stored vector is the metric between the query itself (not quantised) and the
 *     concatenation of the entries the code names: squared L2 ascending, inner product descending.  It is computed
 *     as a sum of m table entries: one table of 256 partial scores per sub-space and query.
 * The sub-vectors quantised are those of the stored vector itself, not of its residual to the list's centroid, so a
 * query's tables do not depend on the list.  One call scores a whole batch of queries with the same k, nprobe and
 * metric; the calls are asynchronous on the stream of the index's pool.
 *
 * Conventions as in trinity_ivf.h: tri_status return values, [host] / [device] markers, all device memory is the
 * caller's, no CPU fallback.  tri_last_error() has the text of a failure.
 */
#ifndef TRINITY_PQ_H
#define TRINITY_PQ_H

#include "trinity_ivf.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tri_pq tri_pq;        /* codebooks and codes of one IVF index, resident on its GPU */

#define TRI_PQ_KSUB 256u             /* entries per codebook: one byte per sub-space and vector              */
#define TRI_PQ_KMAX 256u             /* largest k of pq_search_batch                                        */
#define TRI_PQ_NPROBE_MAX 256u       /* largest nprobe                                                      */
#define TRI_PQ_DSUB_MAX 32u          /* largest dim / m                                                     */

typedef struct {
    uint32_t m;             /* sub-spaces: divides the index's dim, a multiple of 4, m * 1 KiB of tables must fit
                               the LDS beside the selection buffer (m <= 124)                                */
    uint32_t train_iters;   /* Lloyd iterations per sub-space when the codebooks are trained here            */
    uint32_t train_rows;    /* stored vectors the training uses (every n/train_rows-th one; 0 = min(n, 65536)) */
    uint32_t refine_rows;   /* != 0: the tri_pq keeps its own copy of the index's vectors, row-major by vector id
                               (n padded rows more of device memory), and re-ranking (k_adc > 0) reads those: one
                               contiguous row per candidate instead of pieces scattered over a block of the index's
                               interleaved lists (which are laid out for the list scan).  Same results.          */
    uint64_t seed;          /* picks the 256 vectors whose sub-vectors start the codebooks                   */
} pq_params;

/* Bytes pq_build needs: dev_bytes of device memory that the tri_pq keeps (codebooks, codes, with
 * refine_rows the vectors), tmp_bytes of device memory it needs only during the call (training: the partial sums of
 * the 16 runs the sample is dealt out in, 16 codebooks' worth; they are added in a fixed order, so the same
 * parameters train the same codebooks bit for bit).  TRI_EINVAL for an m the index's dim does not allow. */
int pq_build_bytes(const tri_index *index /*[host]*/, const pq_params *p /*[host]*/, size_t *dev_bytes /*[host] out*/,
                   size_t *tmp_bytes /*[host] out*/);

/* Codebooks and codes for a resident index.  codebooks [host] [m][256][dim/m] fp32: used as given; NULL: trained
 * here by Lloyd's algorithm per sub-space (an entry nothing is nearest to keeps its value) from the sub-vectors of
 * 256 stored vectors picked by the seed.  Then every stored vector is encoded (list-major, the order of the
 * index's lists).  dev_mem [device], 256-byte aligned, is owned by the tri_pq until pq_destroy; tmp_dev [device] is
 * free again when the call returns.  The index must outlive the tri_pq and must not be searched through its pool
 * while this runs.  Synchronous. */
int pq_build(const tri_index *index /*[host]*/, const pq_params *p /*[host]*/, const float *codebooks /*[host] or NULL*/,
             void *dev_mem /*[device]*/, size_t dev_mem_bytes, void *tmp_dev /*[device]*/, size_t tmp_bytes,
             tri_pq **out /*[host] out*/);

int pq_destroy(tri_pq *pq);

/* The codebooks [m][256][dim/m] fp32 and the codes [n][m], list-major (the vector at stored position p of the index,
 * whose id ivf_export's list_ids[p] gives), to host memory; either may be NULL.  Synchronous. */
int pq_export(const tri_pq *pq, float *codebooks /*[host] out or NULL*/, uint8_t *codes /*[host] out or NULL*/);

/* Device workspace of a search of nq queries: padded query rows, coarse scores, probe lists, the queries' tables. */
int pq_search_bytes(const tri_pq *pq, uint32_t nq, size_t *ws_bytes /*[host] out*/);

/* Score a batch: for each of the nq query rows (the index's storage type, dim values, pitch_bytes apart, [device])
 * the nprobe best lists by `metric` against the centroids, every code of those lists, the k best by (score, id).
 * k_adc = 0: the scores returned are the table sums.  k_adc >= k: re-ranking -- the k_adc best by table sums are
 * scored again exactly against the index's stored vectors (squared L2 as the sum of squared differences, or the
 * inner product, fp32) and the k best of those by (exact score, id) are returned with their exact scores.
 * Outputs [device]: ids_out [nq][k] (0xFFFFFFFF past n_out), dist_out [nq][k] (+inf / -inf past n_out),
 * n_out [nq], probes_out [nq][nprobe] or NULL (the probed lists, best first).  1 <= k <= k_adc <= TRI_PQ_KMAX,
 * 1 <= nprobe <= min(nlist, TRI_PQ_NPROBE_MAX).  Asynchronous on the stream of the index's pool: outputs and ws
 * are in use until that stream has passed the call (pq_sync waits for it). */
int pq_search_batch(tri_pq *pq, const void *queries /*[device]*/, size_t pitch_bytes, uint32_t nq, uint32_t k,
                    uint32_t k_adc, uint32_t nprobe, uint32_t metric, void *ws /*[device]*/, size_t ws_bytes,
                    uint32_t *ids_out /*[device]*/, float *dist_out /*[device]*/, uint32_t *n_out /*[device]*/,
                    uint32_t *probes_out /*[device] or NULL*/);

int pq_sync(tri_pq *pq);

/* Measurement helper: what the scan's look-ups can reach at most.  One workgroup of 1024 threads per compute unit
 * holds m tables of TRI_PQ_KSUB fp32 entries in LDS and does nothing but the scan's inner loop -- four byte-indexed
 * 4-byte look-ups per 32-bit word of random bytes, summed -- `rounds` times per thread over m / 4 words; the rate comes
 * from HIP events around the launch on hip_stream.  lookups_per_s [host] out: look-ups per second of the whole GPU
 * (random indices collide on LDS banks, so this lies well below the LDS's 128 bytes per clock).  m: multiple of 4,
 * 4..124.  dev_sink [device]: 4 writable bytes.  Synchronous. */
int pq_lds_gather_rate(uint32_t m, uint32_t rounds, void *dev_sink, void *hip_stream, double *lookups_per_s /*[host] out*/);

#ifdef __cplusplus
}
#endif
#endif
