/*
 * vlq.h - C ABI of the VLQ-ADC index for AMD MI355X (gfx950).
 *
 * The library implements the query path of "Vector and Line Quantization for
 * Billion-scale Similarity Search on GPUs" and the build steps that feed it:
 *
 *   first level   vector quantiser q_v with a codebook C of k centroids (Sec. 2.1, Eq. 2)
 *   second level  line quantiser q_l over the n-NN graph of the centroids (Sec. 3.1);
 *                 cell i is split into n sub-regions, one per edge l(c_i, s_ij)
 *   encoding      residual to the anchor point (1-lambda) c_i + lambda s_ij, product
 *                 quantised with m sub-codebooks of 256 codewords (Sec. 3.2, Alg. 1-2);
 *                 lambda stored as one byte
 *   search        Alg. 3: w1 nearest cells, w2 nearest sub-regions among their w1*n
 *                 (Sec. 3.3.1), ADC distance of Eq. 14 / 16 / 17 for every point of the
 *                 visited lists (Sec. 3.3.2), K smallest (Sec. 3.3.3)
 *
 * Conventions
 *  - Every data pointer named d_* is a DEVICE pointer owned by the caller; the
 *    library reads inputs and writes outputs on the given HIP stream
 *    (`stream` is a hipStream_t passed as void*; NULL = the default stream) and
 *    keeps no reference to them after the call returns.  Outputs are complete
 *    once work queued on that stream before the return has finished.
 *  - Matrices are dense row-major.  Vectors are fp32.  ids are non-negative int32.
 *  - Every function returns VLQ_OK (0) or a negative VLQ_E* code and never
 *    throws or aborts; on error no output is written and vlq_last_error()
 *    describes the failure (per thread).
 *  - An index may be used by one host thread at a time, and calls on one index
 *    must be queued on one stream (or ordered by the caller): search and encode
 *    use scratch memory owned by the index, which grows on demand (the first
 *    call with a larger batch allocates device memory and synchronises).
 *  - Distances are squared L2 distances to the reconstructed point (Eq. 14).
 *  - Vector components, centroids and codewords must be finite.  The contents of
 *    device buffers are not inspected on the host, so a NaN or an infinity is not
 *    reported: the outputs of the vectors (queries) that contain one are
 *    unspecified, those of the other vectors of the batch are unaffected.
 */
#ifndef VLQ_H
#define VLQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VLQ_VERSION 1

#define VLQ_OK 0
#define VLQ_EINVAL (-1) /* bad argument (null pointer, size out of range, wrong state) */
#define VLQ_ENOMEM (-2) /* device or host allocation failed */
#define VLQ_EHIP (-3)   /* a HIP call failed; see vlq_last_error() */

/* Limits of this build (checked, VLQ_EINVAL beyond them). */
#define VLQ_MAX_DIM 1024      /* D */
#define VLQ_MAX_EDGES 256     /* n */
#define VLQ_MAX_M 64          /* PQ bytes per point */
#define VLQ_MAX_W1 512        /* probed cells */
#define VLQ_MAX_SUBREGIONS 8192 /* w1 * n, the sub-regions ranked per query */
#define VLQ_MAX_W2 2048       /* visited sub-regions */
#define VLQ_MAX_K 1024        /* results per query */

typedef struct vlq_index vlq_index_t; /* opaque, owned by the library */

/* Index shape (Table 1 notation). */
typedef struct {
    int32_t d;        /* D: vector dimension, multiple of m */
    int32_t nlist;    /* k: number of first-level centroids, > n_edges */
    int32_t n_edges;  /* n: graph edges (sub-regions) per centroid */
    int32_t m;        /* PQ sub-spaces = code bytes per point; 256 codewords each (Sec. 3.2) */
    /* lambda byte grid: code q stands for lambda_lo + q (lambda_hi - lambda_lo) / 255.
     * lambda_lo * 255 / (lambda_hi - lambda_lo) must be an integer so that 0 is a grid
     * value (then the anchor is never farther from the point than its centroid).
     * Both 0 selects the default -0.25 / 0.5 (a point of cell i always has lambda <= 1/2). */
    float lambda_lo, lambda_hi;
} vlq_params_t;

/* Stage names for vlq_profile_read(). */
enum {
    VLQ_STAGE_COARSE = 0,   /* query x centroid distances (MFMA), Alg. 3 first loop */
    VLQ_STAGE_SELECT_CELLS, /* w1 nearest cells */
    VLQ_STAGE_SUBREGIONS,   /* line scores (Eq. 7-8) and w2 nearest sub-regions */
    VLQ_STAGE_SCAN,         /* lookup tables + list scan + fused K-selection */
    VLQ_STAGE_MERGE,        /* merge of per-split partial results (only if a query was split) */
    VLQ_STAGE_COUNT
};

/*
 * Kernel choices that normally follow from the shape, and can be fixed per index with
 * vlq_index_set_option (the tests use them to reach both sides of each choice; none of them
 * changes what is computed, only by which kernel).  Values are 0 / 1 unless stated.
 */
enum {
    VLQ_OPT_COARSE_FP32 = 0,      /* 1: cells and nearest centroids from the fp32 contraction, not the bf16 one */
    VLQ_OPT_NEIGHBOURS_PER_QUERY, /* 1: distances to the neighbour centroids per query, not cell by cell over the batch */
    VLQ_OPT_SCAN_PACKED,          /* -1 (default): by mean list length; 0: one list per wave at a time; 1: short lists packed */
    VLQ_OPT_SCAN_GENERIC,         /* 1: the scan with per-cell / per-sub-region tables (2m lookups, Sec. 3.3.2) for every shape */
    VLQ_OPT_ENCODE_WAVE,          /* 1: the wave-per-vector encode kernel for every shape */
    VLQ_OPT_PIPELINE_PARTS,       /* 0 (default): by batch size; 1 .. 8: parts a batch is cut into, the region traversal of
                                     part p + 1 running on a second stream beside the list scan of part p */
    VLQ_OPT_SMALL_BATCH,          /* default 64: batches of up to this many queries take the forms with the fewest kernel
                                     launches (exact distances to all centroids in one pass, neighbour products pair by pair); 0: never */
    VLQ_OPT_COARSE_SPLIT,         /* 1: the two sweeps of the cell selection multiply split operands (two or three bf16
                                     products per fp32 product) instead of the hi parts alone; same cells either way */
    VLQ_OPT_COUNT
};

/*
 * Create an index from trained codebooks (Sec. 3.1): copies C and the PQ
 * codebooks, computes the centroid norms and the n-NN graph (for every c_i
 * its n nearest other centroids, ascending by (distance, index), and the
 * squared edge lengths).  If N > 0 the base vectors are encoded and added and
 * the index is finalised (= vlq_index_add + vlq_index_finalize).
 *   d_centroids [nlist x d], d_pq [m x 256 x d/m]; d_base [N x d] or NULL with N = 0;
 *   d_ids [N] or NULL for ids 0..N-1.
 * Synchronises the stream before returning.  *out is set only on success.
 */
int vlq_build_index(const vlq_params_t *params, const float *d_centroids, const float *d_pq,
                    const float *d_base, int64_t N, const int32_t *d_ids, void *stream,
                    vlq_index_t **out);

/* Frees the index and all device memory it owns (NULL is allowed). */
void vlq_index_free(vlq_index_t *idx);

/*
 * Alg. 1 + Alg. 2 for a batch, without touching the index contents.  Per vector:
 * cell i = nearest centroid; edge j = nearest of the n lines of that cell
 * (Eq. 7 at the line's own lambda, Eq. 8); lambda byte; PQ code of the residual
 * to the anchor rebuilt from that byte (Eq. 12), one byte per sub-space.
 * Ties go to the smaller index.  Outputs: d_cell [nb], d_edge [nb], d_lambda [nb],
 * d_codes [nb x m]; any of them may be NULL to skip it.  nb = 0 is a no-op.
 */
int vlq_encode(const vlq_index_t *idx, const float *d_x, int64_t nb, int32_t *d_cell,
               int32_t *d_edge, uint8_t *d_lambda, uint8_t *d_codes, void *stream);

/*
 * Residuals of line quantisation for a batch (Eq. 12): d_res[t] = x_t - ((1 - l) c_i + l s_ij)
 * with the cell, edge and dequantised lambda byte that vlq_encode gives for x_t.  These are the
 * vectors the PQ codebooks are trained on (Sec. 3.2).  d_res [nb x d] is caller-owned device
 * memory; the index is not modified.
 */
int vlq_line_residuals(const vlq_index_t *idx, const float *d_x, int64_t nb, float *d_res,
                       void *stream);

/*
 * Lloyd iterations for a codebook (the paper trains the first-level codebook and the 256-word
 * PQ codebooks by k-means, Sec. 2.1 / Sec. 5).  d_centroids [k x d] holds the initial
 * codebook on entry and the trained one on return.  One iteration: every row of d_x [nt x d]
 * goes to its nearest centroid (Eq. 2, ties to the smaller index); a centroid with members
 * moves to their mean, one without members stays.  The means do not depend on the order of
 * summation (64-bit fixed-point sums).  Optional outputs, both with respect to the RETURNED
 * codebook: d_assign [nt] nearest centroid of every row, d_counts [k] members per centroid.
 * iters = 0 only assigns.  Device pointers throughout; temporaries are allocated and freed
 * inside the call, which returns after the stream has drained.  Needs no index.
 */
int vlq_kmeans(const float *d_x, int64_t nt, int32_t d, int32_t k, int32_t iters,
               float *d_centroids, int32_t *d_assign, int32_t *d_counts, void *stream);

/*
 * Streamed build (the paper builds the database in batches, Sec. 5): encode nb
 * vectors and stage them.  d_ids NULL numbers them after the points already
 * added.  The index must be finalised again before the next search.
 */
int vlq_index_add(vlq_index_t *idx, const float *d_x, int64_t nb, const int32_t *d_ids,
                  void *stream);

/* Stage points that are already encoded (same fields as vlq_encode's outputs). */
int vlq_index_add_encoded(vlq_index_t *idx, const int32_t *d_cell, const int32_t *d_edge,
                          const uint8_t *d_lambda, const uint8_t *d_codes,
                          const int32_t *d_ids, int64_t nb, void *stream);

/* Optional: make room for `total` points up front (avoids regrowth copies). */
int vlq_index_reserve(vlq_index_t *idx, int64_t total);

/*
 * Build the inverted lists from everything staged so far (Sec. 4: list lengths,
 * ids, codes and lambda bytes; list l = cell * n + edge; ascending id inside a
 * list), and per stored point the query-independent part of its ADC distance
 * (||q2||^2 + 2<q1 - mu,q2> + (l^2 - l) c of Eq. 15-17 with mu the mean of the centroids,
 * summed in fp64, stored as 4 bytes) that the scan streams with the code.  Synchronises the stream.
 */
int vlq_index_finalize(vlq_index_t *idx, void *stream);

/* Fix one of the VLQ_OPT_* kernel choices for this index.  Takes effect from the next call on. */
int vlq_index_set_option(vlq_index_t *idx, int option, int value);

/*
 * Region traversal (Sec. 3.3.1) with the query's lambda restricted to [lo, hi]: the score of a
 * sub-region becomes the squared distance from the query to that segment of the line l(c_i, s_ij),
 * i.e. Eq. 7 evaluated at clamp(lambda of Eq. 8, lo, hi).  The default (-inf, +inf) is the literal
 * reading of Eq. 7-8, the distance to the whole line; (0, 1) is the segment between the two
 * centroids (Fig. 1c); the index's own (lambda_lo, lambda_hi) is the part of the line on which
 * stored points can have their anchors.  lo <= hi required.  Only the choice of the w2 visited
 * sub-regions changes; the distances returned for their points do not.
 */
int vlq_index_set_query_lambda_range(vlq_index_t *idx, float lo, float hi);

/* Number of points added / whether the lists are current. */
int64_t vlq_index_ntotal(const vlq_index_t *idx);
int vlq_index_is_finalized(const vlq_index_t *idx);
int vlq_index_params(const vlq_index_t *idx, vlq_params_t *out);

/*
 * Alg. 3 for a batch of queries d_q [nq x d]:
 *   w1 nearest cells by ||y - c||^2, 1 <= w1 <= nlist;
 *   among their w1*n sub-regions the w2 with the smallest distance from y to the
 *   line l(c_i, s_ij) (Eq. 7 at y's own lambda, Eq. 8), 1 <= w2 <= w1*n;
 *   for every point of those lists the distance of Eq. 14, evaluated as
 *   s_x + a + l (b - a) - sum_p T[p][code_p]: the stored per-point term, the two
 *   coarse distances of the sub-region, and one per-query table of 2 <(y - mu)^p, codeword>
 *   (Eq. 16-17 regrouped; m lookups per point.  Shapes outside m in {8, 16},
 *   K <= 128 use per-cell / per-sub-region tables with 2m lookups);
 *   the K smallest by (distance, id); among points whose fp32 distances are
 *   exactly equal at the K-th place the earlier list position is kept.
 * The result of a query does not depend on the other queries of the batch.
 * Once a call with the same (or larger) nq, w1, w2, K has sized the index's scratch memory, the
 * call only launches kernels on `stream` (no allocation, no memset, no synchronisation), so it
 * can be recorded in a HIP graph and replayed.
 * Outputs row-major [nq x K], ascending; rows with fewer than K candidates are
 * padded with (+inf, -1).  nq = 0 is a no-op.  Does not synchronise.
 */
int vlq_search(const vlq_index_t *idx, const float *d_q, int32_t nq, int32_t w1, int32_t w2,
               int32_t K, float *d_out_dist, int32_t *d_out_ids, void *stream);

/*
 * vlq_search for callers that cannot allocate device memory: code running under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same results
 * as vlq_search, but the scratch memory of the call is a fixed array of VLQ_NOALLOC_SCRATCH_BYTES
 * that is part of the library's code object (one copy per GPU, held until the process ends) and
 * the call allocates nothing, on the device or through any library.  A request whose scratch need
 * exceeds the array is rejected with VLQ_EINVAL and a message stating both sizes (roughly
 * nq * (16 w2 + 4 w1 (n_edges + 3) + 4 D + ...) bytes: about 20 MB for 1 024 queries at w1 = 64,
 * w2 = 512, n_edges = 32).  All calls on one GPU share that array, whatever the index: calls that
 * overlap on one GPU (two streams, two threads) race; order them.  Stage times are not recorded.
 */
#define VLQ_NOALLOC_SCRATCH_BYTES (32u << 20)
int vlq_search_noalloc(const vlq_index_t *idx, const float *d_q, int32_t nq, int32_t w1, int32_t w2,
                       int32_t K, float *d_out_dist, int32_t *d_out_ids, void *stream);

/*
 * vlq_search that also returns the traversal (any extra pointer may be NULL):
 *   d_cells [nq x w1] / d_cell_dist [nq x w1]: probed cells, ascending (distance, index);
 *   d_sub [nq x w2] / d_sub_score [nq x w2]: visited lists (label i*n+j), ascending (score, label).
 */
int vlq_search_debug(const vlq_index_t *idx, const float *d_q, int32_t nq, int32_t w1,
                     int32_t w2, int32_t K, float *d_out_dist, int32_t *d_out_ids,
                     int32_t *d_cells, float *d_cell_dist, int32_t *d_sub, float *d_sub_score,
                     void *stream);

/*
 * Copies of index contents into caller-owned DEVICE buffers (NULL skips one):
 *   graph: d_S [nlist x n] neighbour indices, d_E [nlist x n] squared edge lengths;
 *   lists: d_off [nlist*n + 1] int64 offsets, d_ids [ntotal], d_codes [ntotal x m],
 *          d_lambda [ntotal] (needs a finalised index).
 */
int vlq_index_get_graph(const vlq_index_t *idx, int32_t *d_S, float *d_E, void *stream);
int vlq_index_get_lists(const vlq_index_t *idx, int64_t *d_off, int32_t *d_ids,
                        uint8_t *d_codes, uint8_t *d_lambda, void *stream);

/*
 * Per-stage GPU time of the searches issued since the last reset, measured with
 * HIP events on the search stream.  enable != 0 switches recording on.
 * vlq_profile_read synchronises on the recorded events and writes
 * ms[VLQ_STAGE_COUNT] (summed over calls) and the number of kernel launches per
 * stage (launches may be NULL), then clears the record.
 */
int vlq_profile_enable(vlq_index_t *idx, int enable);
int vlq_profile_read(vlq_index_t *idx, float *ms, int32_t *launches);

/* Message of the last error on this thread ("" if none). */
const char *vlq_last_error(void);
int vlq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* VLQ_H */
