// Shared device helpers and internal declarations of libvlq (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/vlq.h"

#define VLQ_WAVE 64

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#define KEY_MAX 0xFFFFFFFFFFFFFFFFull

// ---- order-preserving float <-> uint32 map (all finite floats, -0 < +0) ----
__device__ __forceinline__ uint32_t f2ord(float f)
{
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ord2f(uint32_t o)
{
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o);
}
__device__ __forceinline__ uint64_t make_key(float d, uint32_t lo) { return ((uint64_t)f2ord(d) << 32) | lo; }


// ---- sum over each row of 16 lanes, identical in all 16: lane-crossing operands of the adder
// (neighbour in the pair, other pair of the quad, other quad of the half, other half of the row),
// no LDS traffic.  The order of the additions is fixed. ----
__device__ __forceinline__ float row16_sum(float v)
{
#define VLQ_DPP_ADD(ctrl)                                                                                      \
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, 0xF, 0xF, true))
    VLQ_DPP_ADD(0xB1);  // quad_perm [1, 0, 3, 2]
    VLQ_DPP_ADD(0x4E);  // quad_perm [2, 3, 0, 1]
    VLQ_DPP_ADD(0x141); // row_half_mirror
    VLQ_DPP_ADD(0x140); // row_mirror
#undef VLQ_DPP_ADD
    return v;
}

// ---- wave-wide sum, identical in every lane: rows of 16 first, then the four rows ----
__device__ __forceinline__ float wave_sum(float v)
{
    v = row16_sum(v);
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    return v;
}

// wave-wide fp64 sum (butterfly, fixed order), identical in every lane
__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ uint64_t shfl_xor_u64(uint64_t v, int o)
{
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    lo = __shfl_xor(lo, o, 64);
    hi = __shfl_xor(hi, o, 64);
    return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ uint64_t wave_min_u64(uint64_t v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        uint64_t w = shfl_xor_u64(v, o);
        v = w < v ? w : v;
    }
    return v;
}

// ||x - c||^2 by one wave: x in LDS (or any memory), c a global row.  Lanes
// stride over the dimensions, partial sums are combined by a butterfly, so the
// result is the same in all lanes and independent of the launch shape.
__device__ __forceinline__ float wave_sqdist(const float *x, const float *__restrict__ c, int D, int lane)
{
    float s = 0.f;
    for (int d = lane; d < D; d += VLQ_WAVE) {
        float t = x[d] - c[d];
        s = fmaf(t, t, s);
    }
    return wave_sum(s);
}

// ---- block-wide bitonic sort of sz (power of two) u64 keys in LDS, ascending ----
template <int NT>
__device__ __forceinline__ void block_bitonic_sort(uint64_t *a, int sz, int tid)
{
    for (int k = 2; k <= sz; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = tid; i < (sz >> 1); i += NT) {
                int l = ((i & ~(j - 1)) << 1) | (i & (j - 1));
                int r = l | j;
                uint64_t x = a[l], y = a[r];
                bool asc = (l & k) == 0;
                if ((x > y) == asc) {
                    a[l] = y;
                    a[r] = x;
                }
            }
            __syncthreads();
        }
    }
}

// same, carrying a 16-bit payload
template <int NT>
__device__ __forceinline__ void block_bitonic_sort_kv(uint64_t *a, uint16_t *v, int sz, int tid)
{
    for (int k = 2; k <= sz; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = tid; i < (sz >> 1); i += NT) {
                int l = ((i & ~(j - 1)) << 1) | (i & (j - 1));
                int r = l | j;
                uint64_t x = a[l], y = a[r];
                bool asc = (l & k) == 0;
                if ((x > y) == asc) {
                    a[l] = y;
                    a[r] = x;
                    uint16_t t = v[l];
                    v[l] = v[r];
                    v[r] = t;
                }
            }
            __syncthreads();
        }
    }
}

__device__ __forceinline__ int next_pow2_dev(int v)
{
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

static inline int next_pow2(int v)
{
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

// ---------------------------------------------------------------------------
// Kernel launchers (one per .hip file).  All pointers are device pointers.
// ---------------------------------------------------------------------------

// Squared norms of the rows of X [rows x D]; with mu [D] given, of X - mu.
void launch_row_norms(const float *X, int64_t rows, int D, const float *mu, float *out, hipStream_t st);
// out = X - mu row by row (the fp32 contraction is handed centred operands: its rounding error is
// relative to the norms, and distances do not depend on the origin).
void launch_center_rows(const float *X, int64_t rows, int D, const float *mu, float *out, hipStream_t st);
// Column means of X [rows x D] (fp64 sums in row order): mu [D] the mean, mu_int [D] the mean rounded
// to the nearest integer (subtracting it keeps integer-valued data exactly representable in bf16).
void launch_col_means(const float *X, int64_t rows, int D, float *mu, float *mu_int, hipStream_t st);

// GEMM-form squared distances between rows of A [M x D] and rows of B [N x D]
// on the fp32 matrix cores: out[i*ldo + j] = max(an[i] + bn[j] - 2 <A_i, B_j>, 0).
void launch_coarse_gemm_full(const float *A, int M, const float *B, int N, int D, const float *an,
                             const float *bn, float *out, int64_t ldo, hipStream_t st);

// Same product, but only nearest-row candidates are kept: for every row of A
// up to VLQ_NN_CANDS keys (distance bits << 32 | column) per column split that lie
// within the rounding band of the row minimum.  cand [M x nsplit x VLQ_NN_CANDS].
#define VLQ_NN_CANDS 8
// A lane of the product kernels keeps the two smallest keys per row among the columns it sees (its
// "slot": columns (slot >> 5) * 64 + 32 j + (slot & 31), j = 0, 1, of every 128-column tile of the
// split).  When its second key lies inside the band a third one may have been dropped: the
// (row, split) then carries, after its kept keys, a marker key whose high word is VLQ_NN_MARK and
// whose low word names the slot, and the consumer re-evaluates that slot's columns exactly.  A
// low word of VLQ_NN_ALL (more in-band columns than room, or several such slots) asks for an
// exact ranking over all columns.
#define VLQ_NN_MARK 0xFFFFFFFEu
#define VLQ_NN_ALL 0xFFFFFFFFu
#define VLQ_NN_TILE 128
// Width of the band around the smallest distance d of a row a:
// band_norm * (3 ||a||^2 + 2 d) + band_dist * (||a||^2 + d); the fp32 product has band_dist = 0.
// fp32 product: each value ||a||^2 + ||b||^2 - 2 <a, b> is off by at most
// (D + 8) 2^-24 (||a||^2 + ||b||^2): fp32 accumulation of D products in any order, doubled by
// the factor -2 (2 D 2^-24 |a||b|), plus the rounding of the two norms and of the final sums.
// A comparison involves two values, and ||a||^2 + ||b||^2 <= 3 ||a||^2 + 2 d.
static inline float vlq_fp32_band_norm(int D) { return 2.f * (float)(D + 8) * 5.9604645e-8f; }
int coarse_gemm_nn_splits(int M, int N);
void launch_coarse_gemm_nn(const float *A, int M, const float *B, int N, int D, const float *an,
                           const float *bn, uint64_t *cand, int nsplit, hipStream_t st);

// The same shortlist on the bf16 matrix cores (coarse_bf16.hip).  Both operands are first
// rewritten by launch_split_bf16 into an image of coarse_bf16_image_bytes(rows, D) bytes
// (bf16 hi/lo pairs in the order the product kernel reads them).  Requires
// coarse_bf16_supported(D).  The band the consumer has to apply is returned in
// *band_norm / *band_dist; the return value is 0 or a hipError_t.
// mu (optional, [D]) is subtracted from every row before the split.
bool coarse_bf16_supported(int D);
size_t coarse_bf16_image_bytes(int64_t rows, int D);
void launch_split_bf16(const float *X, int64_t rows, int D, const float *mu, void *img, int *any_lo, hipStream_t st);
int launch_coarse_gemm_nn_bf16(const void *Aimg, const int *a_any_lo, int M, const void *Bimg, int N, int D,
                               const float *an, const float *bn, uint64_t *cand, int nsplit, float *band_norm,
                               float *band_dist, hipStream_t st);

// w1 nearest centroids of every query from two sweeps of the bf16 product, without the nq x k
// matrix (coarse_bf16.hip).  cells_bf16_plan says whether the shape allows it and fixes the
// split count and the candidate capacity per query; the workspace holds group minima,
// thresholds, candidate counts and candidate lists.  launch_cells_bf16_coarse runs both sweeps
// (return value 0 or a hipError_t), launch_cells_bf16_exact ranks the candidates exactly.
// hi_only: both sweeps multiply the hi parts alone (a third to a half of the products) and carry that product's
// error bound inside the values they compare.
bool cells_bf16_plan(int nq, int k, int D, int w1, bool hi_only, int *nsplit, int *cap);
size_t cells_bf16_workspace(int nq, int nsplit, int cap, size_t *gmin_off, size_t *thr_off, size_t *ccnt_off,
                            size_t *cidx_off);
int launch_cells_bf16_coarse(const void *Qimg, const int *q_any_lo, int nq, const void *Cimg, int k, int D,
                             const float *qn, const float *cn, bool hi_only, int w1, int nsplit, int cap, void *ws,
                             hipStream_t st);
void launch_cells_bf16_exact(const float *Q, int nq, int D, const float *C, int k, int w1, int cap, const void *ws,
                             int nsplit, int32_t *cells, float *cell_dist, int32_t *pair_cnt, int32_t *pair_rank,
                             hipStream_t st);

// A handful of queries: exact distances to all centroids in one pass over the codebook, then the w1 nearest of
// every query, ascending by (distance, index), from those values.  ws: cells_small_workspace_floats(nq, k) floats
// of scratch (the distances and, per query, the minima of groups of 64 centroids).
bool cells_small_supported(int nq, int k, int D, int w1);
size_t cells_small_workspace_floats(int nq, int k);
void launch_cells_small(const float *Q, int nq, int D, const float *C, int k, int w1, float *ws, int32_t *cells,
                        float *cell_dist, hipStream_t st);

// w smallest entries of each row of dist [rows x k] (GEMM-form values), re-evaluated
// as direct sums of squared differences and ordered by (distance, index).
// self0 >= 0: row r must not select column self0 + r (graph construction).
void launch_select_cells(const float *dist, int64_t ld, int rows, int k, const float *Q, int D,
                         const float *qn, const float *C, const float *cn, int w, int self0,
                         int32_t *cells, float *cell_dist, hipStream_t st);

// Line scores of the w1*n sub-regions of the probed cells and the w2 best of them; the query's
// lambda is restricted to [lam_min, lam_max] (-inf / +inf: the whole line).
// desc (optional): per visited sub-region {list begin, list length, a, b - a} for the streaming scan.
// ws (optional, neighbour_dists_workspace() bytes): the distances to the neighbour centroids are
// then computed cell by cell over the whole batch first; neighbour_dists_by_cell() says when
// that pays.
bool neighbour_dists_by_cell(int nq, int k, int n, int D, int w1);
bool neighbour_dists_grouped(int nq, int w1); // false: few pairs, each served on its own (no counting needed)
size_t neighbour_dists_workspace(int nq, int k, int n, int w1);
// The parts of that workspace.  A cell selection that can count the (query, cell) pairs per cell as
// it writes them (and note each pair's rank inside its cell) gets `cnt`, zeroed by
// launch_pair_counts_zero, and `rank`; launch_subregions is then told that the counting is done.
struct PairWs {
    int32_t *cnt;   // [k]
    int64_t *poff;  // [k + 1]
    int32_t *rank;  // [nq x w1]
    int32_t *pairs; // [nq x w1]
    int64_t *woff;  // [k + 1] work items (a cell's pairs in chunks) before each cell
    int4 *work;     // [nq x w1 / chunk + k] {cell, place of the chunk's first pair, pairs in the chunk, -}
    float *bq;      // [nq x w1 x n]
};
PairWs neighbour_dists_carve(void *ws, int nq, int k, int n, int w1);
void launch_pair_counts_zero(const PairWs &pw, int k, hipStream_t st);
void launch_subregions(const float *Q, int nq, int D, const float *C, const int32_t *S, const float *E,
                       int n, int k, const int32_t *cells, const float *cell_dist, int w1, int w2,
                       float lam_min, float lam_max, int32_t *sub, float *sub_score, int32_t *scan_label,
                       float *scan_g, const int64_t *off, uint4 *desc, void *ws, bool pairs_counted, hipStream_t st);

struct ScanArgs {
    const float *Q;
    int nq, D, n, m, w2, K, nsplit;
    const float *C;
    const int32_t *S;
    const float *E;
    const float *P;
    const int64_t *off;
    const int32_t *ids;
    const uint8_t *codes;
    const uint8_t *lam;
    const float *sx;   // per point: query-independent part of the distance (streaming scan)
    const float *mu;   // [D] the vector both s_x and the query's table are taken relative to
    float lam_step, lam_zero;
    const uint4 *desc; // [nq x w2] {begin, length, a, b - a} per visited sub-region (streaming scan)
    int packed;        // streaming scan: short lists, several per chunk of lanes
    bool force_generic; // the 2m-lookup kernel whatever the shape
    const int32_t *scan_label;
    const float *scan_g;
    uint64_t *partial; // [nq x nsplit x K] when nsplit > 1
    float *out_dist;
    int32_t *out_ids;
};
void launch_scan(const ScanArgs &a, hipStream_t st);
bool scan_stream_supported(const ScanArgs &a);
bool scan_will_stream(const ScanArgs &a); // the choice launch_scan is going to make
void launch_scan_stream(const ScanArgs &a, hipStream_t st);
void launch_merge(const uint64_t *partial, int nq, int nsplit, int K, float *out_dist, int32_t *out_ids,
                  hipStream_t st);
int scan_pick_nsplit(int nq, int w2, int K);

struct EncodeArgs {
    const float *X;
    int64_t nb;
    int D, k, n, m;
    const float *C;
    const int32_t *S;
    const float *E;
    const float *P;
    float lam_step, lam_zero;
    double lam_step_d;  // the grid step of the lambda byte in full precision
    const float *mu;    // what the product subtracted from every operand row (or null)
    bool wave_per_vector; // the wave-per-vector kernel for every shape
    const uint64_t *cand;
    int nsplit;
    float band_norm, band_dist; // error band of the shortlist's distances
    int32_t *cell, *edge;
    uint8_t *lamq, *codes;
    float *res; // optional [nb x D]: the residual x - ((1 - l) c_i + l s_ij) of Eq. 12
};
// S == nullptr: only the nearest centroid is determined (a.cell must be given)
void launch_encode_finish(const EncodeArgs &a, hipStream_t st);

// Lloyd iteration pieces (train.hip)
void launch_absmax(const float *X, int64_t count, uint32_t *out_bits, hipStream_t st);
void launch_kmeans_accumulate(const float *X, int64_t nb, int D, const int32_t *assign, const uint32_t *absmax_bits,
                              int shift, long long *sums, int32_t *cnt, hipStream_t st);
void launch_kmeans_update(float *C, int k, int D, const long long *sums, const int32_t *cnt,
                          const uint32_t *absmax_bits, int shift, hipStream_t st);

// inverted lists
void launch_iota_i32(int32_t *p, int64_t n, int32_t start, hipStream_t st);
void launch_pack_labels(const int32_t *cell, const int32_t *edge, int n, int k, int32_t *label, int64_t nb,
                        int32_t *bad, hipStream_t st);
void launch_list_histogram(const int32_t *label, int64_t N, int32_t *cnt, hipStream_t st);
void launch_exclusive_scan(const int32_t *cnt, int64_t nl, int64_t *off, hipStream_t st);
// the same, and beside it the exclusive scan of ceil(cnt / chunk) into off2 (chunk a power of two, cnt 16-byte
// aligned, counts adding up to less than 2^31)
void launch_exclusive_scan_chunks(const int32_t *cnt, int64_t nl, int64_t *off, int chunk, int64_t *off2, hipStream_t st);
void launch_list_scatter(const int32_t *label, const int32_t *st_ids, const uint8_t *st_codes,
                         const uint8_t *st_lam, int64_t N, int m, const int64_t *off, int32_t *cursor,
                         int32_t *ids, uint8_t *codes, uint8_t *lam, hipStream_t st);
// s_x of every stored point (see scan_stream.hip)
void launch_list_static(const int64_t *off, int64_t nl, int n, int D, int m, const float *C, const int32_t *S,
                        const float *P, const float *mu, const uint8_t *codes, const uint8_t *lam, double lam_step,
                        float lam_zero, float *sx, hipStream_t st);
void launch_list_sort(const int64_t *off, int64_t nl, int m, int32_t *ids, uint8_t *codes, uint8_t *lam,
                      int32_t *long_lists, int32_t *n_long, int max_long, hipStream_t st);
// second tier of the per-list sort: the reported lists of up to list_sort_mid_max(m) points (0: tier unavailable)
int list_sort_mid_max(int m);
void launch_list_sort_mid(const int64_t *off, int m, const int32_t *in_lists, int n_in, int32_t *ids, uint8_t *codes,
                          uint8_t *lam, int32_t *out_lists, int32_t *n_out, int max_out, hipStream_t st);
void launch_long_list_sort_at(int64_t beg, int64_t len, int m, int32_t *ids, uint8_t *codes, uint8_t *lam,
                              uint64_t *scratch_keys, uint8_t *scratch_payload, hipStream_t st);
