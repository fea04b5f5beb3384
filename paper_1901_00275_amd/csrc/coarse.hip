// First-level quantiser on the GPU: distances between vectors and centroids
// (Eq. 2; Alg. 3, first loop) as a dense contraction on the fp32 matrix cores,
// and the selection of the nearest centroids.
//
// The contraction uses ||a||^2 + ||b||^2 - 2<a,b>, whose fp32 rounding error is
// relative to the norms rather than to the distance.  Every decision taken from
// it is therefore re-taken from direct sums of squared differences over a
// shortlist that contains everything within the rounding band of the cut.
#include "common.h"

// ---------------------------------------------------------------------------
// row norms
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_row_norms(const float *__restrict__ X, int64_t rows, int D,
                                                   const float *__restrict__ mu, float *__restrict__ out)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const float *x = X + row * D;
    float s = 0.f;
    for (int d = lane; d < D; d += 64) {
        const float v = mu ? x[d] - mu[d] : x[d];
        s = fmaf(v, v, s);
    }
    s = wave_sum(s);
    if (lane == 0) out[row] = s;
}

void launch_row_norms(const float *X, int64_t rows, int D, const float *mu, float *out, hipStream_t st)
{
    if (rows <= 0) return;
    hipLaunchKernelGGL(k_row_norms, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, X, rows, D, mu, out);
}

__global__ __launch_bounds__(256) void k_center_rows(const float *__restrict__ X, int64_t count, int D,
                                                     const float *__restrict__ mu, float *__restrict__ out)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += stride) out[i] = X[i] - mu[i % D];
}

void launch_center_rows(const float *X, int64_t rows, int D, const float *mu, float *out, hipStream_t st)
{
    const int64_t count = rows * D;
    if (count <= 0) return;
    int64_t blocks = (count + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(k_center_rows, dim3((unsigned)blocks), dim3(256), 0, st, X, count, D, mu, out);
}

// One workgroup per column: threads stride over the rows with fp64 partial sums, combined in a
// fixed order (wave butterfly, then the four waves in turn).
__global__ __launch_bounds__(256) void k_col_means(const float *__restrict__ X, int64_t rows, int D,
                                                   float *__restrict__ mu, float *__restrict__ mu_int)
{
    __shared__ double part[4];
    const int d = blockIdx.x, tid = threadIdx.x;
    double s = 0.0;
    for (int64_t r = tid; r < rows; r += 256) s += (double)X[r * D + d];
    s = wave_sum_f64(s);
    if ((tid & 63) == 0) part[tid >> 6] = s;
    __syncthreads();
    if (tid == 0) {
        const double mean = (part[0] + part[1] + part[2] + part[3]) / (double)rows;
        mu[d] = (float)mean;
        mu_int[d] = (float)rint(mean);
    }
}

void launch_col_means(const float *X, int64_t rows, int D, float *mu, float *mu_int, hipStream_t st)
{
    if (rows <= 0 || D <= 0) return;
    hipLaunchKernelGGL(k_col_means, dim3((unsigned)D), dim3(256), 0, st, X, rows, D, mu, mu_int);
}

// ---------------------------------------------------------------------------
// GEMM-form distances on v_mfma_f32_32x32x2_f32
//
// Workgroup = 256 threads = 4 waves, tile 128 (rows of A) x 128 (rows of B),
// each wave owns a 64 x 64 quadrant = 2 x 2 MFMA blocks.  Both operands are
// "row-major with the contraction index contiguous", so they are staged the
// same way: a [128 x 32] slab in LDS with a row stride of 33 floats (the 32
// lanes that read one k of 32 consecutive rows hit 32 different banks).
// Operand layout of the instruction: lane l supplies A[i = l % 32][k = l / 32]
// and B[k = l / 32][j = l % 32]; accumulator register r of lane l is
// D[i = 8 (r / 4) + 4 (l / 32) + r % 4][j = l % 32].
// ---------------------------------------------------------------------------
#define GT 128
#define GK 32
#define GLD 33

__device__ __forceinline__ void load_slab(float (*dst)[GLD], const float *__restrict__ src, int64_t row0,
                                          int64_t nrows, int D, int k0, int tid, bool vec)
{
    const int c4 = (tid & 7) * 4;
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
        const int r = pass * 32 + (tid >> 3);
        const int64_t gr = row0 + r;
        float v0 = 0.f, v1 = 0.f, v2 = 0.f, v3 = 0.f;
        if (gr < nrows) {
            const float *p = src + gr * D + k0 + c4;
            if (vec) {
                if (k0 + c4 < D) {
                    f32x4 t = *(const f32x4 *)p;
                    v0 = t.x; v1 = t.y; v2 = t.z; v3 = t.w;
                }
            } else {
                if (k0 + c4 + 0 < D) v0 = p[0];
                if (k0 + c4 + 1 < D) v1 = p[1];
                if (k0 + c4 + 2 < D) v2 = p[2];
                if (k0 + c4 + 3 < D) v3 = p[3];
            }
        }
        dst[r][c4 + 0] = v0;
        dst[r][c4 + 1] = v1;
        dst[r][c4 + 2] = v2;
        dst[r][c4 + 3] = v3;
    }
}

__device__ __forceinline__ void tile_product(float (*As)[GLD], float (*Bs)[GLD], const float *__restrict__ A,
                                             int64_t m0, int M, const float *__restrict__ B, int64_t n0, int N,
                                             int D, bool vec, int tid, int wm, int wn, int lane,
                                             f32x16 (&acc)[2][2])
{
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    for (int k0 = 0; k0 < D; k0 += GK) {
        __syncthreads();
        load_slab(As, A, m0, M, D, k0, tid, vec);
        load_slab(Bs, B, n0, N, D, k0, tid, vec);
        __syncthreads();
        const int kl = lane >> 5, rl = lane & 31;
#pragma unroll
        for (int kk = 0; kk < GK; kk += 2) {
            float a0 = As[wm + rl][kk + kl], a1 = As[wm + 32 + rl][kk + kl];
            float b0 = Bs[wn + rl][kk + kl], b1 = Bs[wn + 32 + rl][kk + kl];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        }
    }
}

__global__ __launch_bounds__(256) void k_coarse_gemm_full(const float *__restrict__ A, int M,
                                                          const float *__restrict__ B, int N, int D,
                                                          const float *__restrict__ an,
                                                          const float *__restrict__ bn, float *__restrict__ out,
                                                          int64_t ldo, int vec)
{
    __shared__ float As[GT][GLD];
    __shared__ float Bs[GT][GLD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    // blockIdx.x walks the tiles of B (centroids) fastest so that concurrently
    // resident workgroups share the same slab of A.
    const int64_t n0 = (int64_t)blockIdx.x * GT, m0 = (int64_t)blockIdx.y * GT;
    f32x16 acc[2][2];
    tile_product(As, Bs, A, m0, M, B, n0, N, D, vec != 0, tid, wm, wn, lane, acc);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t row = m0 + wm + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (row >= M) continue;
            const float ra = an[row];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int64_t col = n0 + wn + 32 * j + (lane & 31);
                if (col < N) out[row * ldo + col] = fmaxf(ra + bn[col] - 2.f * acc[i][j][r], 0.f) + 0.f; // +0: never -0
            }
        }
}

void launch_coarse_gemm_full(const float *A, int M, const float *B, int N, int D, const float *an,
                             const float *bn, float *out, int64_t ldo, hipStream_t st)
{
    if (M <= 0 || N <= 0) return;
    const int vec = (D % 4 == 0) && (((uintptr_t)A | (uintptr_t)B) % 16 == 0);
    dim3 grid((unsigned)((N + GT - 1) / GT), (unsigned)((M + GT - 1) / GT));
    hipLaunchKernelGGL(k_coarse_gemm_full, grid, dim3(256), 0, st, A, M, B, N, D, an, bn, out, ldo, vec);
}

// Nearest-row variant: a workgroup owns 128 rows of A and a contiguous range of
// tiles of B; every lane keeps, for each of its 32 accumulator rows, the two
// smallest keys it has seen.  At the end the row minimum over the workgroup is
// formed in LDS and every kept key within the rounding band of it is emitted.
__global__ __launch_bounds__(256) void k_coarse_gemm_nn(const float *__restrict__ A, int M,
                                                        const float *__restrict__ B, int N, int D,
                                                        const float *__restrict__ an,
                                                        const float *__restrict__ bn,
                                                        uint64_t *__restrict__ cand, int nsplit,
                                                        int tiles_per_split, int vec, float band_norm)
{
    __shared__ float As[GT][GLD];
    __shared__ float Bs[GT][GLD];
    __shared__ unsigned long long rowmin[GT];
    __shared__ int rowcnt[GT];
    __shared__ unsigned long long rowcand[GT][VLQ_NN_CANDS];
    __shared__ int rowovf[GT];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int64_t m0 = (int64_t)blockIdx.x * GT;
    const int split = blockIdx.y;
    const int ntiles = (N + GT - 1) / GT;
    const int t0 = split * tiles_per_split;
    const int t1 = min(ntiles, t0 + tiles_per_split);

    uint64_t b1[2][16], b2[2][16];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) b1[i][r] = b2[i][r] = KEY_MAX;
    float ra[2][16];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t row = m0 + wm + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            ra[i][r] = row < M ? an[row] : 0.f;
        }

    for (int t = t0; t < t1; ++t) {
        const int64_t n0 = (int64_t)t * GT;
        f32x16 acc[2][2];
        tile_product(As, Bs, A, m0, M, B, n0, N, D, vec != 0, tid, wm, wn, lane, acc);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t col = n0 + wn + 32 * j + (lane & 31);
            if (col >= N) continue;
            const float cb = bn[col];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float d = fmaxf(ra[i][r] + cb - 2.f * acc[i][j][r], 0.f) + 0.f; // +0: never -0
                    const uint64_t key = ((uint64_t)__float_as_uint(d) << 32) | (uint32_t)col;
                    if (key < b1[i][r]) {
                        b2[i][r] = b1[i][r];
                        b1[i][r] = key;
                    } else if (key < b2[i][r]) {
                        b2[i][r] = key;
                    }
                }
        }
    }

    if (tid < GT) {
        rowmin[tid] = KEY_MAX;
        rowcnt[tid] = 1; // slot 0 is the minimum itself
        rowovf[tid] = -1;
#pragma unroll
        for (int s = 0; s < VLQ_NN_CANDS; ++s) rowcand[tid][s] = KEY_MAX;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int rl = wm + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (b1[i][r] != KEY_MAX) atomicMin(&rowmin[rl], (unsigned long long)b1[i][r]);
        }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int rl = wm + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            const uint64_t mn = rowmin[rl];
            if (mn == KEY_MAX) continue;
            const float dmin = __uint_as_float((uint32_t)(mn >> 32));
            // rounding band of the GEMM form: a few ulp of ||a||^2 + ||b||^2 <= 3||a||^2 + 2 d
            const float band = dmin + band_norm * (3.f * ra[i][r] + 2.f * dmin);
            uint64_t ks[2] = {b1[i][r], b2[i][r]};
            // a lane keeps two keys per row: when its second one lies inside the band a third may
            // have been dropped, so the row is handed on as incomplete
            if (ks[1] != KEY_MAX && __uint_as_float((uint32_t)(ks[1] >> 32)) <= band) {
                const int slot = (wn >> 6) * 32 + (lane & 31);
                const int old = atomicCAS(&rowovf[rl], -1, slot);
                if (old != -1 && old != slot) rowovf[rl] = 64; // several slots
            }
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                if (ks[s] == KEY_MAX || ks[s] == mn) continue;
                if (__uint_as_float((uint32_t)(ks[s] >> 32)) <= band) {
                    int pos = atomicAdd(&rowcnt[rl], 1);
                    if (pos < VLQ_NN_CANDS) rowcand[rl][pos] = ks[s];
                }
            }
        }
    __syncthreads();
    if (tid < GT && m0 + tid < M) {
        uint64_t *dst = cand + ((m0 + tid) * nsplit + split) * VLQ_NN_CANDS;
        const int cnt = rowcnt[tid], sl = rowovf[tid];
        const bool all = cnt > VLQ_NN_CANDS || sl == 64 || (sl >= 0 && cnt >= VLQ_NN_CANDS);
        dst[0] = all ? (((uint64_t)VLQ_NN_MARK << 32) | VLQ_NN_ALL) : rowmin[tid];
#pragma unroll
        for (int s = 1; s < VLQ_NN_CANDS; ++s)
            dst[s] = !all && sl >= 0 && s == cnt ? (((uint64_t)VLQ_NN_MARK << 32) | (uint32_t)sl) : rowcand[tid][s];
    }
}

int coarse_gemm_nn_splits(int M, int N)
{
    // enough workgroups to fill 256 CUs twice over, but never split B finer than 4 tiles
    const int strips = (M + GT - 1) / GT;
    const int ntiles = (N + GT - 1) / GT;
    int want = (512 + strips - 1) / strips;
    int maxs = ntiles / 4 > 1 ? ntiles / 4 : 1;
    if (want > maxs) want = maxs;
    if (want < 1) want = 1;
    if (want > 64) want = 64;
    // make the split count exact for the tile partition
    const int per = (ntiles + want - 1) / want;
    return (ntiles + per - 1) / per;
}

void launch_coarse_gemm_nn(const float *A, int M, const float *B, int N, int D, const float *an,
                           const float *bn, uint64_t *cand, int nsplit, hipStream_t st)
{
    if (M <= 0 || N <= 0) return;
    const int vec = (D % 4 == 0) && (((uintptr_t)A | (uintptr_t)B) % 16 == 0);
    const int ntiles = (N + GT - 1) / GT;
    const int per = (ntiles + nsplit - 1) / nsplit;
    dim3 grid((unsigned)((M + GT - 1) / GT), (unsigned)nsplit);
    hipLaunchKernelGGL(k_coarse_gemm_nn, grid, dim3(256), 0, st, A, M, B, N, D, an, bn, cand, nsplit, per, vec,
                       vlq_fp32_band_norm(D));
}

// ---------------------------------------------------------------------------
// w nearest centroids of a row (Alg. 3, "w1-argmin"; also the n-NN graph rows)
//
// 1. radix select (4 passes of 8 bits over the float bit patterns, all
//    non-negative) finds the value v of the w-th smallest GEMM-form distance;
// 2. every column within the rounding band of v is collected;
// 3. each collected column gets its distance again as a direct sum of squared
//    differences (one wave per column);
// 4. the collected set is sorted by (direct distance, index) and cut at w.
// If more columns fall into the band than the shortlist holds (only possible
// with many exactly or almost coinciding centroids) the band is dropped and
// ties at v are resolved by index.
// ---------------------------------------------------------------------------
#define SEL_CAP 1024

__global__ __launch_bounds__(256) void k_select_cells(const float *__restrict__ dist, int64_t ld, int k,
                                                      const float *__restrict__ Q, int D,
                                                      const float *__restrict__ qn,
                                                      const float *__restrict__ C,
                                                      const float *__restrict__ cn, int w, int self0,
                                                      int32_t *__restrict__ cells,
                                                      float *__restrict__ cell_dist)
{
    extern __shared__ float yv[]; // [D]
    __shared__ int hist[256];
    __shared__ uint64_t keys[SEL_CAP];
    __shared__ int sh_cnt, sh_prefix, sh_rank, sh_eq_taken;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = blockIdx.x;
    const float *drow = dist + (int64_t)row * ld;
    const int self = self0 >= 0 ? self0 + row : -1;
    const int want = w + (self >= 0 ? 1 : 0); // the row itself is among its own nearest
    const float bandn = 2.f * (float)(D + 8) * 5.9604645e-8f; // vlq_fp32_band_norm(D)

    for (int d = tid; d < D; d += 256) yv[d] = Q[(int64_t)row * D + d];

    // ---- 1. radix select ----
    uint32_t prefix = 0;
    int rank = want - 1; // 0-based rank inside the current prefix bucket
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < k; i += 256) {
            const uint32_t b = __float_as_uint(drow[i]);
            const bool match = pass == 0 || (b >> (shift + 8)) == (prefix >> (shift + 8));
            if (match) atomicAdd(&hist[(b >> shift) & 255], 1);
        }
        __syncthreads();
        if (tid == 0) {
            int acc = 0, bin = 0;
            for (; bin < 256; ++bin) {
                if (acc + hist[bin] > rank) break;
                acc += hist[bin];
            }
            sh_prefix = bin;
            sh_rank = rank - acc;
        }
        __syncthreads();
        prefix |= (uint32_t)sh_prefix << shift;
        rank = sh_rank;
        __syncthreads();
    }
    const float v = __uint_as_float(prefix);
    const float rq = qn[row];

    // ---- 2. collect the band ----
    if (tid == 0) sh_cnt = 0;
    __syncthreads();
    for (int i = tid; i < k; i += 256) {
        const float d = drow[i];
        if (d <= v + bandn * (rq + cn[i])) {
            int pos = atomicAdd(&sh_cnt, 1);
            if (pos < SEL_CAP) keys[pos] = (uint64_t)(uint32_t)i;
        }
    }
    __syncthreads();
    int cnt = sh_cnt;
    if (cnt > SEL_CAP) {
        // degenerate: redo without the band; ties at v go to the smallest indices
        __syncthreads();
        if (tid == 0) {
            sh_cnt = 0;
            sh_eq_taken = 0;
        }
        __syncthreads();
        for (int i = tid; i < k; i += 256) {
            if (__float_as_uint(drow[i]) < prefix) {
                int pos = atomicAdd(&sh_cnt, 1);
                keys[pos] = (uint64_t)(uint32_t)i; // fewer than `want` such entries
            }
        }
        __syncthreads();
        const int need_eq = want - sh_cnt;
        __syncthreads();
        for (int base = 0; base < k; base += 256) {
            const int i = base + tid;
            const bool eq = i < k && __float_as_uint(drow[i]) == prefix;
            // rank of this thread among the equal entries of the chunk, in index order
            hist[tid] = eq ? 1 : 0;
            __syncthreads();
            if (tid == 0) {
                int acc = sh_eq_taken;
                for (int t = 0; t < 256; ++t) {
                    int f = hist[t];
                    hist[t] = acc;
                    acc += f;
                }
                sh_eq_taken = acc;
            }
            __syncthreads();
            if (eq && hist[tid] < need_eq) keys[sh_cnt + hist[tid]] = (uint64_t)(uint32_t)i;
            __syncthreads();
            if (sh_eq_taken >= need_eq) break;
        }
        __syncthreads();
        cnt = want;
    }

    // ---- 3. direct distances ----
    for (int c = wave; c < cnt; c += 4) {
        const int i = (int)(uint32_t)keys[c];
        const float d = wave_sqdist(yv, C + (int64_t)i * D, D, lane);
        if (lane == 0) keys[c] = (i == self) ? KEY_MAX : make_key(d, (uint32_t)i);
    }
    const int sz = next_pow2_dev(cnt);
    for (int c = cnt + tid; c < sz; c += 256) keys[c] = KEY_MAX;
    __syncthreads();

    // ---- 4. order and cut ----
    block_bitonic_sort<256>(keys, sz, tid);
    for (int e = tid; e < w; e += 256) {
        const uint64_t key = keys[e];
        const bool ok = e < cnt && key != KEY_MAX;
        cells[(int64_t)row * w + e] = ok ? (int32_t)(uint32_t)key : -1;
        if (cell_dist) cell_dist[(int64_t)row * w + e] = ok ? ord2f((uint32_t)(key >> 32)) : INFINITY;
    }
}

// ---------------------------------------------------------------------------
// Register-resident variant for k <= 65536: one workgroup of 1024 threads holds
// the whole row in registers (one pass over memory) and narrows a value range
// [lo, hi] around the w-th smallest entry with 1024-bin linear histograms until
// at most SEL_CAP entries are selected.  Entries are tracked by two bit masks per
// thread (selected / undecided).  Exact ties at the cut go to the smaller index.
// The selected entries are then ordered by (GEMM-form distance, index); those
// within the rounding band of the w-th get direct distances and the final order.
// ---------------------------------------------------------------------------
#define SEL2_NT 1024
#define SEL2_NB 1024

__device__ __forceinline__ int wave_incl_scan_int(int v, int lane)
{
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(v, o, 64);
        if (lane >= o) v += t;
    }
    return v;
}

// inclusive scan over the 1024 threads of the block; *total receives the block sum
__device__ __forceinline__ int block_incl_scan_int(int v, int tid, int *sh16, int *total)
{
    const int lane = tid & 63, wave = tid >> 6;
    const int inc = wave_incl_scan_int(v, lane);
    __syncthreads();
    if (lane == 63) sh16[wave] = inc;
    __syncthreads();
    int before = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < SEL2_NT / 64; ++w) {
        const int t = sh16[w];
        before += w < wave ? t : 0;
        tot += t;
    }
    *total = tot;
    return inc + before;
}

__device__ __forceinline__ void block_minmax(float mn, float mx, int tid, float *shf, float *omn, float *omx)
{
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        mn = fminf(mn, __shfl_xor(mn, o, 64));
        mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    }
    __syncthreads();
    if (lane == 0) {
        shf[wave] = mn;
        shf[16 + wave] = mx;
    }
    __syncthreads();
    float a = shf[0], b = shf[16];
#pragma unroll
    for (int w = 1; w < SEL2_NT / 64; ++w) {
        a = fminf(a, shf[w]);
        b = fmaxf(b, shf[16 + w]);
    }
    *omn = a;
    *omx = b;
}

template <int VPT>
__global__ __launch_bounds__(SEL2_NT) void k_select_cells_reg(const float *__restrict__ dist, int64_t ld, int k,
                                                              const float *__restrict__ Q, int D,
                                                              const float *__restrict__ qn,
                                                              const float *__restrict__ C,
                                                              const float *__restrict__ cn, int w, int self0,
                                                              int32_t *__restrict__ cells,
                                                              float *__restrict__ cell_dist)
{
    extern __shared__ float yv[]; // [D]
    __shared__ int hist[SEL2_NB];
    __shared__ uint64_t keys[SEL_CAP];
    __shared__ int sh16[16];
    __shared__ float shf[32];
    __shared__ int sh_bin, sh_before, sh_inbin, sh_cnt, sh_taken;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = blockIdx.x;
    const float *drow = dist + (int64_t)row * ld;
    const int self = self0 >= 0 ? self0 + row : -1;
    const int want = w + (self >= 0 ? 1 : 0);
    const float bandn = 2.f * (float)(D + 8) * 5.9604645e-8f; // vlq_fp32_band_norm(D)

    for (int d = tid; d < D; d += SEL2_NT) yv[d] = Q[(int64_t)row * D + d];
    // raw buffer over the row: base, stride 0, size in bytes, dword data format
    const __amdgpu_buffer_rsrc_t rowbuf = __builtin_amdgcn_make_buffer_rsrc((void *)drow, 0, k * 4, 0x00020000);
    float v[VPT];
#pragma unroll
    for (int e = 0; e < VPT; ++e) // one lane offset for all loads; the row end is range-checked by the buffer
        v[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rowbuf, tid * 4, e * SEL2_NT * 4, 0));
#pragma unroll
    for (int e = 0; e < VPT; ++e)
        if (e * SEL2_NT + tid >= k) v[e] = INFINITY;
    uint64_t selm = 0, undm = 0; // bit e: entry e*1024 + tid is selected / still undecided
    float mn = INFINITY, mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < VPT; ++e)
        if (v[e] < INFINITY) {
            undm |= 1ull << e;
            mn = fminf(mn, v[e]);
            mx = fmaxf(mx, v[e]);
        }
    float lo, hi;
    block_minmax(mn, mx, tid, shf, &lo, &hi);
    int nsel = 0;      // entries selected so far (all below lo)
    bool ties = false; // the undecided entries are all equal to lo == hi
    // Short cut: the want-th smallest of the 1 024 per-thread minima bounds the want-th smallest entry
    // from above (that many entries lie at or below it), and tightly, because the nearest columns
    // rarely share a thread.  If no more than SEL_CAP entries lie at or below it they are the
    // selection, and the histogram levels below have nothing left to decide.
    bool decided = false; // uniform over the workgroup
    {
        keys[tid] = ((uint64_t)f2ord(mn) << 32) | (uint32_t)tid;
        __syncthreads();
        block_bitonic_sort<SEL2_NT>(keys, SEL2_NT, tid);
        const float tau = ord2f((uint32_t)(keys[want - 1 < SEL2_NT ? want - 1 : SEL2_NT - 1] >> 32));
        __syncthreads();
        int c = 0;
#pragma unroll
        for (int e = 0; e < VPT; ++e) c += (undm >> e & 1) && v[e] <= tau;
        int total;
        (void)block_incl_scan_int(c, tid, sh16, &total);
        if (want <= SEL2_NT && total >= want && total <= SEL_CAP) {
#pragma unroll
            for (int e = 0; e < VPT; ++e)
                if ((undm >> e & 1) && v[e] <= tau) selm |= 1ull << e;
            undm = 0;
            nsel = total;
            decided = true;
        }
        __syncthreads();
    }
    for (int level = 0; level < 8 && !decided; ++level) {
        if (!(hi > lo)) {
            ties = true;
            break;
        }
        const float scale = (float)SEL2_NB / (hi - lo);
        hist[tid] = 0;
        __syncthreads();
#pragma unroll
        for (int e = 0; e < VPT; ++e)
            if (undm >> e & 1) {
                int b = (int)((v[e] - lo) * scale);
                b = b > SEL2_NB - 1 ? SEL2_NB - 1 : b;
                atomicAdd(&hist[b], 1);
            }
        __syncthreads();
        const int need = want - nsel; // rank of the cut among the undecided entries (1-based)
        const int mine = hist[tid];
        int total;
        const int cum = block_incl_scan_int(mine, tid, sh16, &total);
        if (cum - mine < need && need <= cum) {
            sh_bin = tid;
            sh_before = cum - mine;
            sh_inbin = mine;
        }
        __syncthreads();
        const int B = sh_bin, before = sh_before, inbin = sh_inbin;
        // bins below B are in, bins above B are out
        float bmn = INFINITY, bmx = -INFINITY;
#pragma unroll
        for (int e = 0; e < VPT; ++e)
            if (undm >> e & 1) {
                int b = (int)((v[e] - lo) * scale);
                b = b > SEL2_NB - 1 ? SEL2_NB - 1 : b;
                if (b < B) {
                    selm |= 1ull << e;
                    undm &= ~(1ull << e);
                } else if (b > B) {
                    undm &= ~(1ull << e);
                } else {
                    bmn = fminf(bmn, v[e]);
                    bmx = fmaxf(bmx, v[e]);
                }
            }
        nsel += before;
        if (nsel + inbin <= SEL_CAP) { // take the whole bin
            selm |= undm;
            undm = 0;
            nsel += inbin;
            break;
        }
        block_minmax(bmn, bmx, tid, shf, &lo, &hi);
    }
    if (tid == 0) {
        sh_cnt = 0;
        sh_taken = 0;
    }
    __syncthreads();
    const bool undecided = __syncthreads_or(undm != 0) != 0; // the same answer in every thread: barriers follow
    if (!decided && (ties || undecided || nsel < want)) {
        // the undecided entries share one value (or the range could not be narrowed further):
        // the missing ones are taken in index order
        const int need = want - nsel;
        for (int e = 0; e < VPT; ++e) {
            const int flag = (int)(undm >> e & 1);
            int total;
            const int inc = block_incl_scan_int(flag, tid, sh16, &total);
            const int taken = sh_taken;
            if (flag && taken + inc <= need) selm |= 1ull << e;
            __syncthreads();
            if (tid == 0) sh_taken = taken + total;
            __syncthreads();
            if (sh_taken >= need) break;
        }
        undm = 0;
    }
    // ---- gather the selected entries: (GEMM-form distance, index) ----
#pragma unroll
    for (int e = 0; e < VPT; ++e)
        if (selm >> e & 1) {
            const int pos = atomicAdd(&sh_cnt, 1);
            if (pos < SEL_CAP) keys[pos] = ((uint64_t)__float_as_uint(v[e]) << 32) | (uint32_t)(e * SEL2_NT + tid);
        }
    __syncthreads();
    int cnt = min(sh_cnt, SEL_CAP);
    int sz = next_pow2_dev(cnt);
    for (int c = cnt + tid; c < sz; c += SEL2_NT) keys[c] = KEY_MAX;
    __syncthreads();
    block_bitonic_sort<SEL2_NT>(keys, sz, tid);
    // ---- rounding band above the w-th smallest: entries not selected that may still belong ----
    const float vw = __uint_as_float((uint32_t)(keys[want - 1] >> 32));
    const float rq = qn[row];
    __syncthreads();
    // ||c|| <= ||y|| + sqrt(d) bounds the centroid norm without touching memory; the exact
    // band (with the centroid's own norm) is applied to the few survivors below
    const float sq = sqrtf(rq) + sqrtf(vw);
    const float wide = vw * (1.f + 1e-5f) + bandn * (rq + sq * sq) * 1.5f;
#pragma unroll
    for (int e = 0; e < VPT; ++e) {
        if (!(selm >> e & 1) && v[e] <= wide) {
            const int i = e * SEL2_NT + tid;
            if (v[e] <= vw + bandn * (rq + cn[i])) {
                const int pos = atomicAdd(&sh_cnt, 1);
                if (pos < SEL_CAP) keys[pos] = ((uint64_t)__float_as_uint(v[e]) << 32) | (uint32_t)i;
            }
        }
    }
    __syncthreads();
    cnt = min(sh_cnt, SEL_CAP);
    // ---- direct distances for everything inside the band; the rest cannot make the cut ----
    const bool vec = (D % 4 == 0) && (((uintptr_t)C) % 16 == 0);
    const int sub16 = lane >> 4, l16 = lane & 15;
    for (int c0 = wave * 4; c0 < cnt; c0 += (SEL2_NT / 64) * 4) {
        const int c = c0 + sub16;
        uint64_t key = c < cnt ? keys[c] : KEY_MAX;
        const int i = (int)(uint32_t)key;
        bool inband = false;
        if (c < cnt) inband = __uint_as_float((uint32_t)(key >> 32)) <= vw + bandn * (rq + cn[i]);
        float acc = 0.f;
        if (inband) {
            const float *rowp = C + (int64_t)i * D;
            if (vec) {
                for (int d = l16 * 4; d < D; d += 64) {
                    const f32x4 cv = *(const f32x4 *)(rowp + d);
                    const float t0 = yv[d] - cv.x, t1 = yv[d + 1] - cv.y, t2 = yv[d + 2] - cv.z, t3 = yv[d + 3] - cv.w;
                    acc = fmaf(t0, t0, acc);
                    acc = fmaf(t1, t1, acc);
                    acc = fmaf(t2, t2, acc);
                    acc = fmaf(t3, t3, acc);
                }
            } else {
                for (int d = l16; d < D; d += 16) {
                    const float t = yv[d] - rowp[d];
                    acc = fmaf(t, t, acc);
                }
            }
        }
        acc = row16_sum(acc);
        if (l16 == 0 && c < cnt) keys[c] = (inband && i != self) ? make_key(acc, (uint32_t)i) : KEY_MAX;
    }
    sz = next_pow2_dev(cnt);
    for (int c = cnt + tid; c < sz; c += SEL2_NT) keys[c] = KEY_MAX;
    __syncthreads();
    block_bitonic_sort<SEL2_NT>(keys, sz, tid);
    for (int e = tid; e < w; e += SEL2_NT) {
        const uint64_t key = keys[e];
        const bool ok = e < cnt && key != KEY_MAX;
        cells[(int64_t)row * w + e] = ok ? (int32_t)(uint32_t)key : -1;
        if (cell_dist) cell_dist[(int64_t)row * w + e] = ok ? ord2f((uint32_t)(key >> 32)) : INFINITY;
    }
}

// ---------------------------------------------------------------------------
// A handful of queries (Alg. 3, first loop, when launches count more than flop): exact distances of
// all queries to all centroids in one pass over the codebook, then one workgroup per query that
// takes its w nearest straight from those values.
//
// k_small_dists: 16 lanes per centroid row (four components per lane and step, the adder's
// lane-crossing sum: the summation order of every exact distance in this library), four rows per
// wave and pass, the queries in LDS; a centroid row is read once for all queries.  Beside the
// distances every workgroup leaves, per query, the smallest distance of its SMALL_ROWS rows.
// ---------------------------------------------------------------------------
#define SMALL_NQ 64   // most queries of the form
#define SMALL_ROWS 64 // centroid rows per workgroup (one group of the selection below)

__global__ __launch_bounds__(256) void k_small_dists(const float *__restrict__ Q, int nq, int D,
                                                     const float *__restrict__ C, int k, float *__restrict__ dist,
                                                     float *__restrict__ gmin)
{
    extern __shared__ float yq[]; // [nq][D]
    __shared__ uint32_t smin[SMALL_NQ];
    __shared__ float tile[SMALL_NQ][SMALL_ROWS]; // the workgroup's distances, written out in full rows at the end
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub16 = lane >> 4, l16 = lane & 15;
    for (int i = tid; i < nq * D; i += 256) yq[i] = Q[i];
    if (tid < SMALL_NQ) smin[tid] = 0xFFFFFFFFu;
    __syncthreads();
    const bool vec = (D % 4 == 0) && (((uintptr_t)C) % 16 == 0);
    const int r0 = blockIdx.x * SMALL_ROWS;
    for (int rr = wave * 4; rr < SMALL_ROWS; rr += 16) {
        const int i = r0 + rr + sub16;
        const float *rowp = C + (int64_t)min(i, k - 1) * D;
        if (nq >= 8 && vec && D <= 128) {
            // sixteen queries at a time: the row's components stay in registers, the 16 x 16 partial sums of a
            // lane group are added across its lanes and transposed at once (register s of lane l belongs to query
            // s ^ g(l); every step of row16_sum finds the same query in the partner's register): 15 lane-crossing
            // adds instead of 64, the same additions in the same association, so the same sums to the bit
            const int gl = (l16 & 3) ^ ((l16 & 4) ? 7 : 0) ^ ((l16 & 8) ? 12 : 0);
            const int d0 = l16 * 4, d1 = 64 + l16 * 4;
            const bool has0 = d0 < D, has1 = d1 < D;
            const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
            const f32x4 c0 = has0 ? *(const f32x4 *)(rowp + d0) : zero4, c1 = has1 ? *(const f32x4 *)(rowp + d1) : zero4;
            for (int q0 = 0; q0 < nq; q0 += 16) {
                float r[16];
#pragma unroll
                for (int sreg = 0; sreg < 16; ++sreg) {
                    const float *yv = yq + min(q0 + (sreg ^ gl), nq - 1) * D; // (queries past the end: computed, not kept)
                    float acc = 0.f;
                    if (has0) {
                        const f32x4 y = *(const f32x4 *)(yv + d0);
                        const float t0 = y.x - c0.x, t1 = y.y - c0.y, t2 = y.z - c0.z, t3 = y.w - c0.w;
                        acc = fmaf(t0, t0, acc);
                        acc = fmaf(t1, t1, acc);
                        acc = fmaf(t2, t2, acc);
                        acc = fmaf(t3, t3, acc);
                    }
                    if (has1) {
                        const f32x4 y = *(const f32x4 *)(yv + d1);
                        const float t0 = y.x - c1.x, t1 = y.y - c1.y, t2 = y.z - c1.z, t3 = y.w - c1.w;
                        acc = fmaf(t0, t0, acc);
                        acc = fmaf(t1, t1, acc);
                        acc = fmaf(t2, t2, acc);
                        acc = fmaf(t3, t3, acc);
                    }
                    r[sreg] = acc;
                }
#define VLQ_DPP_GET(x, ctrl) __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), ctrl, 0xF, 0xF, true))
#pragma unroll
                for (int u = 0; u < 16; u += 2) r[u] += VLQ_DPP_GET(r[u + 1], 0xB1);  // quad_perm [1, 0, 3, 2]
#pragma unroll
                for (int u = 0; u < 16; u += 4) r[u] += VLQ_DPP_GET(r[u + 2], 0x4E);  // quad_perm [2, 3, 0, 1]
#pragma unroll
                for (int u = 0; u < 16; u += 8) r[u] += VLQ_DPP_GET(r[u + 4], 0x141); // row_half_mirror
                r[0] += VLQ_DPP_GET(r[8], 0x140);                                     // row_mirror
#undef VLQ_DPP_GET
                const int q = q0 + gl;
                if (q < nq && i < k) {
                    tile[q][rr + sub16] = r[0];
                    atomicMin(&smin[q], f2ord(r[0]));
                }
            }
            continue;
        }
        for (int q = 0; q < nq; ++q) {
            const float *yv = yq + q * D;
            float acc = 0.f;
            if (vec) {
                for (int d = l16 * 4; d < D; d += 64) {
                    const f32x4 cv = *(const f32x4 *)(rowp + d);
                    const float t0 = yv[d] - cv.x, t1 = yv[d + 1] - cv.y, t2 = yv[d + 2] - cv.z, t3 = yv[d + 3] - cv.w;
                    acc = fmaf(t0, t0, acc);
                    acc = fmaf(t1, t1, acc);
                    acc = fmaf(t2, t2, acc);
                    acc = fmaf(t3, t3, acc);
                }
            } else {
                for (int d = l16; d < D; d += 16) {
                    const float t = yv[d] - rowp[d];
                    acc = fmaf(t, t, acc);
                }
            }
            acc = row16_sum(acc);
            if (l16 == 0 && i < k) {
                tile[q][rr + sub16] = acc;
                atomicMin(&smin[q], f2ord(acc));
            }
        }
    }
    __syncthreads();
    for (int t = tid; t < nq * SMALL_ROWS; t += 256) {
        const int q = t / SMALL_ROWS, r = t % SMALL_ROWS;
        if (r0 + r < k) dist[(int64_t)q * k + r0 + r] = tile[q][r];
    }
    if (tid < nq) gmin[(int64_t)tid * gridDim.x + blockIdx.x] = ord2f(smin[tid]);
}

// One workgroup per query.  The w-th smallest of the group minima (a group = the SMALL_ROWS rows of one
// workgroup above; at most 1 024 groups) bounds the w-th smallest distance from above, tightly: the nearest
// columns rarely share a group.  Only the groups whose minimum is at or below it can hold a wanted column:
// their rows are read again (about w groups of the k / SMALL_ROWS), the columns at or below the bound are
// ranked by (distance, index) by counting.  A query with more than SMALL_CAP such columns (masses of
// coinciding distances) is ranked by repeated selection over its whole row instead.
#define SMALL_CAP 1024

__global__ __launch_bounds__(1024) void k_small_cells(const float *__restrict__ dist, const float *__restrict__ gmin,
                                                      int k, int w, int32_t *__restrict__ cells,
                                                      float *__restrict__ cell_dist)
{
    __shared__ uint32_t mins[1024];
    __shared__ uint64_t keys[2 * SMALL_CAP];
    __shared__ int glist[1024];
    __shared__ uint32_t sh_tau;
    __shared__ int sh_n, sh_g;
    __shared__ unsigned long long sh_cut;
    const int tid = threadIdx.x, lane = tid & 63, row = blockIdx.x;
    const int G = (k + SMALL_ROWS - 1) / SMALL_ROWS; // <= 1 024
    const float *drow = dist + (int64_t)row * k;
    const uint32_t mymin = tid < G ? f2ord(gmin[(int64_t)row * G + tid]) : 0xFFFFFFFFu;
    mins[tid] = mymin;
    if (tid == 0) {
        sh_n = 0;
        sh_g = 0;
    }
    __syncthreads();
    if (tid < 64) { // one wave: the w-th smallest of the minima, bit by bit from the top (ballot counts)
        uint32_t u[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) u[e] = mins[lane + 64 * e];
        uint32_t result = 0;
        if (w > G) result = 0xFFFFFFFEu; // fewer groups than cells wanted: every group is looked at
        else
            for (int bit = 31; bit >= 0; --bit) {
                const uint32_t trial = result | (1u << bit);
                int below = 0;
#pragma unroll
                for (int e = 0; e < 16; ++e) below += __popcll(__ballot(u[e] < trial));
                if (below < w) result = trial;
            }
        if (lane == 0) sh_tau = result;
    }
    __syncthreads();
    const uint32_t tau = sh_tau;
    if (tid < G && mymin <= tau) glist[atomicAdd(&sh_g, 1)] = tid;
    __syncthreads();
    const int ng = sh_g;
    for (int t = tid; t < ng * SMALL_ROWS; t += 1024) {
        const int i = glist[t / SMALL_ROWS] * SMALL_ROWS + (t % SMALL_ROWS);
        if (i < k) {
            const float v = drow[i];
            if (f2ord(v) <= tau) {
                const int pos = atomicAdd(&sh_n, 1);
                if (pos < SMALL_CAP) keys[pos] = make_key(v, (uint32_t)i);
            }
        }
    }
    __syncthreads();
    int cnt = sh_n;
    if (cnt <= SMALL_CAP) {
        // rank of every key among the (distinct) keys = its place in the output
        const uint64_t mine = tid < cnt ? keys[tid] : KEY_MAX;
        int rank = 0;
        for (int c = 0; c < cnt; ++c) rank += keys[c] < mine;
        __syncthreads();
        if (tid < cnt) keys[rank] = mine;
        __syncthreads();
    } else {
        // repeated selection: keys below the current w-th smallest are collected over the whole row, 1 024
        // columns a round; a full buffer is sorted and cut back to w
        unsigned long long cut = KEY_MAX;
        if (tid == 0) sh_n = 0;
        __syncthreads();
        for (int i0 = 0; i0 < k; i0 += 1024) {
            const int i = i0 + tid;
            if (i < k) {
                const uint64_t key = make_key(drow[i], (uint32_t)i);
                if (key < cut) keys[atomicAdd(&sh_n, 1)] = key; // at most w + 1 024 keys: w from the last cut
            }
            __syncthreads();
            const int n = sh_n;
            __syncthreads();
            if (n > SMALL_CAP || i0 + 1024 >= k) {
                const int sz = next_pow2_dev(n);
                for (int c = n + tid; c < sz; c += 1024) keys[c] = KEY_MAX;
                __syncthreads();
                block_bitonic_sort<1024>(keys, sz, tid);
                if (tid == 0) {
                    sh_cut = n >= w ? keys[w - 1] : KEY_MAX;
                    sh_n = min(n, w);
                }
                __syncthreads();
                cut = sh_cut;
            }
        }
        cnt = sh_n;
    }
    for (int e = tid; e < w; e += 1024) {
        const uint64_t key = keys[e];
        const bool ok = e < cnt && key != KEY_MAX;
        cells[(int64_t)row * w + e] = ok ? (int32_t)(uint32_t)key : -1;
        cell_dist[(int64_t)row * w + e] = ok ? ord2f((uint32_t)(key >> 32)) : INFINITY;
    }
}

bool cells_small_supported(int nq, int k, int D, int w1)
{
    return nq <= SMALL_NQ && k >= 4096 && k <= 65536 && w1 <= 128 && (size_t)nq * D * 4 <= 65536;
}

size_t cells_small_workspace_floats(int nq, int k) { return (size_t)nq * k + (size_t)nq * ((k + SMALL_ROWS - 1) / SMALL_ROWS); }

void launch_cells_small(const float *Q, int nq, int D, const float *C, int k, int w1, float *ws, int32_t *cells,
                        float *cell_dist, hipStream_t st)
{
    const size_t smem = (size_t)nq * D * 4;
    float *dist = ws, *gmin = ws + (size_t)nq * k;
    if (smem > 49152) // (48 KB of dynamic LDS beside the static part need no asking)
        (void)hipFuncSetAttribute((const void *)k_small_dists, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    hipLaunchKernelGGL(k_small_dists, dim3((unsigned)((k + SMALL_ROWS - 1) / SMALL_ROWS)), dim3(256), smem, st, Q, nq, D, C, k,
                       dist, gmin);
    hipLaunchKernelGGL(k_small_cells, dim3((unsigned)nq), dim3(1024), 0, st, dist, gmin, k, w1, cells, cell_dist);
}

void launch_select_cells(const float *dist, int64_t ld, int rows, int k, const float *Q, int D,
                         const float *qn, const float *C, const float *cn, int w, int self0,
                         int32_t *cells, float *cell_dist, hipStream_t st)
{
    if (rows <= 0) return;
    const size_t smem = (size_t)D * sizeof(float);
    if (k <= 4 * SEL2_NT) {
        hipLaunchKernelGGL(k_select_cells_reg<4>, dim3((unsigned)rows), dim3(SEL2_NT), smem, st, dist, ld, k, Q, D, qn,
                           C, cn, w, self0, cells, cell_dist);
    } else if (k <= 16 * SEL2_NT) {
        hipLaunchKernelGGL(k_select_cells_reg<16>, dim3((unsigned)rows), dim3(SEL2_NT), smem, st, dist, ld, k, Q, D, qn,
                           C, cn, w, self0, cells, cell_dist);
    } else if (k <= 64 * SEL2_NT) {
        hipLaunchKernelGGL(k_select_cells_reg<64>, dim3((unsigned)rows), dim3(SEL2_NT), smem, st, dist, ld, k, Q, D, qn,
                           C, cn, w, self0, cells, cell_dist);
    } else {
        hipLaunchKernelGGL(k_select_cells, dim3((unsigned)rows), dim3(256), smem, st, dist, ld, k, Q, D, qn, C, cn, w,
                           self0, cells, cell_dist);
    }
}
