// First-level quantiser on the bf16 matrix cores (Eq. 2; Alg. 1 "nearest centroid").
//
// An fp32 value v is split into two bf16 numbers, hi = rne(v) and lo = rne(v - hi); a bf16 number
// has 8 significant bits, so |v - hi| <= 2^-8 |v| and |v - hi - lo| <= 2^-16 |v|.  The inner product of
// two split vectors is taken as hi.hi + hi.lo + lo.hi with fp32 accumulation on
// v_mfma_f32_32x32x16_bf16; the dropped lo.lo term and the representation error
// together stay below 3 * 2^-16 |x| |c|.  The result only shortlists centroids: every
// column whose approximate distance lies within the error band of the row minimum
// is handed on and re-evaluated there as a direct fp32 sum of squared differences,
// so the decision itself is taken in fp32 exactly as by the fp32 path.  The two sweeps of the search's
// cell selection multiply the hi parts alone and carry the (much wider, still rigorous) error bound of
// that product per column inside the values they compare; see the kernel's HI parameter.
//
// Operand images.  Both operands are first rewritten (k_split_bf16) into the exact
// byte image the product kernel wants in LDS: rows in blocks of 128, the contraction
// index in steps of 16, and per (block, step) a 4 KB "hi" page followed by a 4 KB "lo"
// page.  A page holds 128 rows x 2 chunks of 16 bytes (8 bf16); chunk c of row r sits
// at position 2 r + (c ^ ((r >> 2) & 1)), which keeps the 32-rows-by-one-chunk
// fragment reads of the MFMA operands free of bank conflicts.  Pages of one block are
// contiguous, so every global access of the product kernel is a fully used 4 KB run.
//
// Product kernel.  Workgroup = 256 threads = 4 waves, 128 rows of A against all
// columns of its split; each wave owns a 64 x 64 quadrant (2 x 2 MFMA blocks).  The
// 128 rows of A are staged in LDS once (D <= 128: 64 KB) and every wave then keeps the hi
// fragments of its 64 rows in registers for the whole sweep (the lo fragments, needed only for
// real-valued rows, are read from LDS); the pages of B stream global -> registers (four steps
// ahead) -> a two-page-pair ring in LDS, one barrier per step.  Two workgroups share a CU (2 x 80 KB of LDS), so one's
// selection epilogue overlaps the other's MFMAs.
#include "common.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

#define BT 128          // rows per block (= VLQ_NN_TILE columns per tile)
#define BSTEP 16        // contraction indices per step
#define PAGE 256        // 16-byte chunks per page
#define BF16_MAX_D 128  // A block resident in LDS: D / 16 steps x 2 pages x 4 KB

__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// X [rows x D] fp32 (minus mu [D], if given) -> image [ceil(rows / 128)][D / 16][hi page, lo page]; rows past
// the end are written as zeros.  *any_lo is raised when some lo is non-zero.
// One thread per (row, chunk of 8 values).
__global__ __launch_bounds__(256) void k_split_bf16(const float *__restrict__ X, int64_t rows, int D,
                                                    const float *__restrict__ mu, int64_t padded_rows,
                                                    u32x4 *__restrict__ img, int *__restrict__ any_lo)
{
    const int cpr = D / 8; // chunks per row
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    bool nz = false;
    if (i < padded_rows * cpr) {
        const int64_t row = i / cpr;
        const int ch = (int)(i - row * cpr);
        u32x4 ph = {0, 0, 0, 0}, pl = {0, 0, 0, 0};
        if (row < rows) {
            f32x4 v0 = *(const f32x4 *)(X + row * D + ch * 8);
            f32x4 v1 = *(const f32x4 *)(X + row * D + ch * 8 + 4);
            if (mu) { // distances do not depend on the origin; the error of the product does
                v0 -= *(const f32x4 *)(mu + ch * 8);
                v1 -= *(const f32x4 *)(mu + ch * 8 + 4);
            }
            uint32_t h[8], l[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float v = e < 4 ? v0[e] : v1[e - 4];
                h[e] = bf16_rne(v);
                l[e] = bf16_rne(v - __uint_as_float(h[e] << 16));
                nz |= (l[e] & 0x7FFFu) != 0;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                ph[e] = h[2 * e] | (h[2 * e + 1] << 16);
                pl[e] = l[2 * e] | (l[2 * e + 1] << 16);
            }
        }
        const int64_t blk = row / BT;
        const int r = (int)(row - blk * BT);
        const int step = ch >> 1, c = ch & 1;
        const int64_t page = (blk * (D / BSTEP) + step) * 2;
        const int pos = 2 * r + (c ^ ((r >> 2) & 1));
        img[page * PAGE + pos] = ph;
        img[(page + 1) * PAGE + pos] = pl;
    }
    // one look at the flag per workgroup, and a write only while it is still down: with
    // non-integer data every workgroup has something to report, all to the same address
    if (__syncthreads_or(nz) && threadIdx.x == 0 && *(volatile int *)any_lo == 0) atomicOr(any_lo, 1);
}

__global__ void k_zero_flag(int *p) { *p = 0; }

bool coarse_bf16_supported(int D) { return D == 32 || D == 64 || D == 96 || D == 128; }

size_t coarse_bf16_image_bytes(int64_t rows, int D)
{
    const int64_t blocks = (rows + BT - 1) / BT;
    return (size_t)blocks * BT * D * 4;
}

void launch_split_bf16(const float *X, int64_t rows, int D, const float *mu, void *img, int *any_lo, hipStream_t st)
{
    hipLaunchKernelGGL(k_zero_flag, dim3(1), dim3(1), 0, st, any_lo);
    const int64_t padded = (rows + BT - 1) / BT * BT;
    const int64_t n = padded * (D / 8);
    if (n <= 0) return;
    hipLaunchKernelGGL(k_split_bf16, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, X, rows, D, mu, padded,
                       (u32x4 *)img, any_lo);
}

// Error budget of one approximate value e = ||b||^2 - 2 <a, b>, D <= 128, worst case:
//   representation: |v - hi - lo| <= 2^-16 |v| on both operands and the dropped lo.lo term give
//     3 * 2^-16 |a||b| on the inner product, twice that on e                      (9.2e-5 |a||b|);
//   fp32 accumulation of the 3 D products in any order: <= 3 D 2^-24 |a||b| on the inner
//     product, twice that on e                                                     (4.6e-5 |a||b|);
//   together < 1.4e-4 |a||b| <= 7e-5 (||a||^2 + ||b||^2).  A comparison involves two values, and
//   ||a||^2 + ||b||^2 <= 3 ||a||^2 + 2 d for a column at distance d, hence the band
//   1.4e-4 (3 ||a||^2 + 2 d).  (Typical errors are a factor sqrt(3 D) smaller; the band only
//   decides how many columns are re-evaluated exactly, never the result.)
#define BF16_BAND_NORM 1.4e-4f
// Columns past the end of B get this "norm": finite, so that index bits can be planted
// in the key, and beyond BF16_NO_KEY, from where on a key counts as absent.
#define BF16_NO_COLUMN 3e38f
#define BF16_NO_KEY 1e38f

// What the product kernel does with a finished 128 x 128 tile of e = ||b||^2 - 2 <a, b>
// (the row norm is common to a row and joins at the end):
//  MODE_NN    running two smallest per row slot of every lane; at the end every kept key inside
//             the band of the row minimum is emitted (encoding: nearest centroid);
//  MODE_MIN   running minimum per row slot of every lane, written out as 64 group minima per
//             (row, split) (search, first sweep);
//  MODE_EMIT  every column with e <= thr[row] is appended to the row's candidate list
//             (search, second sweep).
enum { MODE_NN = 0, MODE_MIN = 1, MODE_EMIT = 2 };

struct Bf16Args {
    const u32x4 *A; // image of the rows
    const u32x4 *B; // image of the columns
    const int *a_any_lo;
    int M, N, D;
    const float *an, *bn;
    int nsplit, tiles_per_split;
    int tile_stride; // a split takes every tile_stride-th tile of its range (1: all of them)
    // MODE_NN
    uint64_t *cand;
    int idx_bits; // low mantissa bits of a running key that hold (tile, column block)
    float band_dist;
    // MODE_MIN
    float *gmin; // [M x nsplit x 64]
    // MODE_EMIT
    const float *thr; // [M]
    int32_t *ccnt;    // [M]
    int32_t *cidx;    // [M x cap]
    int cap;
};

// SPT = D / 16 steps per tile; PDEPTH page pairs of B in flight in registers (divides SPT, so
// that every register set and ring half has a fixed role in the unrolled tile body).
// HI: the product of the hi parts alone (search sweeps): lo pages are neither loaded nor multiplied.
// An operand's hi part differs from it by at most 2^-8 of each component, so <a, b> - <a_h, b_h> =
// <a - a_h, b> + <a_h, b - b_h> is at most 2^-7 |a||b| (1 + 2^-8) in size, half of that when the rows are their
// own hi parts (integer-valued queries); e takes twice the product's error, and the fp32 accumulation of D <= 128
// products adds 2 D 2^-24 |a||b|, inside the 2 % the constant is rounded up by.  With |a| taken as the largest
// of the workgroup's 128 rows the error bound t of a column depends on the column alone and joins its norm:
// MODE_MIN works on e + t (an upper bound of the true value, so the threshold drawn from the minima still has
// enough columns at or below it), MODE_EMIT on e - t (a lower bound: no column at or below the threshold is missed).
template <int SPT, int MODE, bool HI>
__global__ __launch_bounds__(256, 2) void k_coarse_bf16(Bf16Args a)
{
    static_assert(!HI || MODE != MODE_NN, "the nearest-centroid mode needs the split product");
    constexpr int PDEPTH = SPT % 4 == 0 ? 4 : (SPT % 3 == 0 ? 3 : 2);
    static_assert(SPT % 2 == 0 && SPT % PDEPTH == 0, "steps per tile");
    // [A pages: SPT x 2][B ring: 2 x 2 pages]; the tail of the kernel reuses the front
    extern __shared__ u32x4 lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int64_t m0 = (int64_t)blockIdx.x * BT;
    const int split = blockIdx.y;
    const int ntiles = (a.N + BT - 1) / BT;
    const int t0 = split * a.tiles_per_split;
    const int t1 = min(ntiles, t0 + a.tiles_per_split);
    const int tstride = a.tile_stride;
    const int ntl = t1 > t0 ? (t1 - t0 + tstride - 1) / tstride : 0;
    const int last = ntl * SPT - 1; // last step of the split
    const bool use_lo = !HI && *a.a_any_lo != 0;
    // (kept in a lo page of the ring, which the hi-only form never fills: the operand pages take the
    // whole 80 KB that let two workgroups share a compute unit)
    float *strip_max = (float *)(lds + (SPT * 2 + 1) * PAGE);
    if (HI) {
        const int64_t row = m0 + (tid & (BT - 1));
        float v = row < a.M ? a.an[row] : 0.f;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
        if (lane == 0) strip_max[wave] = v;
    }
    u32x4 *Apages = lds;
    u32x4 *ring = lds + SPT * 2 * PAGE;

    // the block of A
    {
        const u32x4 *src = a.A + (int64_t)blockIdx.x * SPT * 2 * PAGE;
#pragma unroll
        for (int p = 0; p < SPT * 2; p += HI ? 2 : 1) Apages[p * PAGE + tid] = src[p * PAGE + tid];
    }

    // B pages: step j of this split is step j % SPT of its (j / SPT)-th tile, the page pair at
    // ((t0 + (j / SPT) * tstride) * SPT + j % SPT) * 2.  Loads past the last step re-read the
    // last pair, so that the number of loads in flight never varies.
    const u32x4 *bsrc = a.B + (int64_t)t0 * SPT * 2 * PAGE + tid;
    auto fetch = [&](u32x4 (&r)[2], int j) {
        j = min(j, last);
        const int jt = j / SPT;
        const int64_t pg = (int64_t)(j + jt * (tstride - 1) * SPT) * 2;
        r[0] = bsrc[pg * PAGE];
        if (!HI) r[1] = bsrc[(pg + 1) * PAGE];
    };
    u32x4 rb[PDEPTH][2];
    if (ntl > 0) {
#pragma unroll
        for (int j = 0; j < PDEPTH; ++j) fetch(rb[j], j);
        ring[tid] = rb[0][0];
        if (!HI) ring[PAGE + tid] = rb[0][1];
        fetch(rb[0], PDEPTH);
    }

    // fragment of a 32-row block: lane reads row (lane & 31), chunk (lane >> 5)
    const int frow = lane & 31;
    const int fpos = 2 * frow + ((lane >> 5) ^ ((frow >> 2) & 1));
    const int fa0 = 2 * wm + fpos, fa1 = fa0 + 64; // + 32 rows
    const int fb0 = 2 * wn + fpos, fb1 = fb0 + 64;
    // accumulator register r of block i holds row wm + 32 i + 8 (r / 4) + 4 (lane / 32) + r % 4
    auto slot_row = [&](int i, int r) { return wm + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); };

    // per row slot: MODE_NN smallest / second smallest key, MODE_MIN minimum, MODE_EMIT threshold
    float b1[2][16], b2[MODE == MODE_NN ? 2 : 1][16];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (MODE == MODE_EMIT) {
                const int64_t row = m0 + slot_row(i, r);
                b1[i][r] = row < a.M ? a.thr[row] : -INFINITY;
            } else {
                b1[i][r] = INFINITY;
                if (MODE == MODE_NN) b2[i][r] = INFINITY;
            }
        }
    const uint32_t keep = MODE == MODE_NN ? ~((1u << a.idx_bits) - 1u) : 0xFFFFFFFFu;

    // (the first product of a tile starts from a constant zero, so the accumulators are never cleared)
    f32x16 acc[2][2];
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    // MODE_EMIT over hi parts: the reported columns of the workgroup's 128 rows are collected in the lo pages
    // of A, which this form never fills (SPT * 8 slots per row; counters in the ring's first lo page), and
    // appended to the rows' global lists at the end: one global atomic per row and workgroup instead of one
    // per reported column, and no wait for its return inside the sweep.
    constexpr bool LBUF = HI && MODE == MODE_EMIT;
    constexpr int LSLOTS = SPT * 8;
    int *lcnt = (int *)(lds + (SPT * 2 + 1) * PAGE) + 16; // [BT] (behind the strip maxima)
    auto lslot = [&](int r, int sl) -> int * { // slot r * LSLOTS + sl of the SPT lo pages (1 024 words each) laid end to end
        const int flat = r * LSLOTS + sl;
        return (int *)(lds + (2 * (flat >> 10) + 1) * PAGE) + (flat & 1023);
    };
    if (LBUF && tid < BT) lcnt[tid] = 0;
    __syncthreads();
    float hi_band = 0.f; // error bound of e per unit of |b|
    if (HI)
        hi_band = sqrtf(fmaxf(fmaxf(strip_max[0], strip_max[1]), fmaxf(strip_max[2], strip_max[3]))) *
                  (*a.a_any_lo ? 0x1p-6f : 0x1p-7f) * 1.02f * (MODE == MODE_MIN ? 1.f : -1.f);
    // the hi fragments of the wave's 64 rows for all steps: the same for every tile, kept in registers
    bf16x8 ahr[SPT][2];
#pragma unroll
    for (int u = 0; u < SPT; ++u) {
        ahr[u][0] = __builtin_bit_cast(bf16x8, Apages[u * 2 * PAGE + fa0]);
        ahr[u][1] = __builtin_bit_cast(bf16x8, Apages[u * 2 * PAGE + fa1]);
    }
    int64_t pend_row = -1; // MODE_EMIT: a reported column whose place in the list is on its way
    int pend_col = 0, pend_pos = 0;
    for (int tl = 0; tl < ntl; ++tl) {
        // column norms of this tile, asked for now and used after its last step
        const int64_t n0 = (int64_t)(t0 + tl * tstride) * BT;
        float cb[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t col = n0 + wn + 32 * j + (lane & 31);
            cb[j] = a.bn[min(col, (int64_t)a.N - 1)];
            if (HI) cb[j] = fmaf(hi_band, sqrtf(fmaxf(cb[j], 0.f)), cb[j]);
            cb[j] = col < a.N ? cb[j] : BF16_NO_COLUMN;
        }
#pragma unroll
        for (int u = 0; u < SPT; ++u) {
            const int s = tl * SPT + u;
            // page pair of step s + 1 into the other half of the ring, its registers refilled
            {
                u32x4 *dst = ring + ((u + 1) & 1) * 2 * PAGE;
                dst[tid] = rb[(u + 1) % PDEPTH][0];
                if (!HI) dst[PAGE + tid] = rb[(u + 1) % PDEPTH][1];
                fetch(rb[(u + 1) % PDEPTH], s + 1 + PDEPTH);
            }
            const u32x4 *ap = Apages + u * 2 * PAGE;
            const u32x4 *bp = ring + (u & 1) * 2 * PAGE;
            bf16x8 ah[2], bh[2], bl[2];
            ah[0] = ahr[u][0];
            ah[1] = ahr[u][1];
            bh[0] = __builtin_bit_cast(bf16x8, bp[fb0]);
            bh[1] = __builtin_bit_cast(bf16x8, bp[fb1]);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bh[j], u == 0 ? zero16 : acc[i][j], 0, 0, 0);
            if (!HI) {
                bl[0] = __builtin_bit_cast(bf16x8, bp[PAGE + fb0]);
                bl[1] = __builtin_bit_cast(bf16x8, bp[PAGE + fb1]);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bl[j], acc[i][j], 0, 0, 0);
            }
            if (use_lo) {
                bf16x8 al[2];
                al[0] = __builtin_bit_cast(bf16x8, ap[PAGE + fa0]);
                al[1] = __builtin_bit_cast(bf16x8, ap[PAGE + fa1]);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], bh[j], acc[i][j], 0, 0, 0);
            }
            __syncthreads();
        }
        // ---- tile finished ----
        // MODE_EMIT: a column qualifies when thr - e = (thr - ||b||^2) + 2 <a, b> is not negative; the sign bits
        // are shifted into one word per column half, element (i, r) ending at bit 31 - (16 i + r)
        uint32_t miss[2] = {0u, 0u};
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t tj = (uint32_t)(tl * 2 + j);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    if (MODE == MODE_EMIT) {
                        const float t = fmaf(2.f, acc[i][j][r], b1[i][r] - cb[j]);
                        miss[j] = __builtin_amdgcn_alignbit(miss[j], __float_as_uint(t), 31);
                    } else {
                        const float e = fmaf(-2.f, acc[i][j][r], cb[j]);
                        if (MODE == MODE_NN) {
                            const float key = __uint_as_float((__float_as_uint(e) & keep) | tj);
                            b2[i][r] = __builtin_amdgcn_fmed3f(b1[i][r], b2[i][r], key);
                            b1[i][r] = fminf(b1[i][r], key);
                        } else {
                            b1[i][r] = fminf(b1[i][r], e);
                        }
                    }
                }
        }
        if (MODE == MODE_EMIT) {
            // A lane rarely has more than one column to report per tile.  The place of the first
            // one is asked for now and used after the next tile's products, so that the round trip
            // of the atomic is not waited for; further ones are placed at once.
            if (pend_row >= 0 && pend_pos < a.cap) a.cidx[pend_row * a.cap + pend_pos] = pend_col;
            pend_row = -1;
            bool first = true;
            uint64_t hits = ((uint64_t)~miss[1] << 32) | (uint32_t)~miss[0];
            while (hits) {
                const int bit = __ffsll((unsigned long long)hits) - 1;
                hits &= hits - 1;
                const int j = bit >> 5, el = 31 - (bit & 31), i = el >> 4, r = el & 15;
                const int64_t row = m0 + slot_row(i, r);
                const int col = (int)n0 + wn + 32 * j + (lane & 31);
                if (LBUF) {
                    const int sl = atomicAdd(&lcnt[slot_row(i, r)], 1);
                    if (sl < LSLOTS) {
                        *lslot(slot_row(i, r), sl) = col;
                        continue;
                    }
                }
                const int pos = atomicAdd(&a.ccnt[row], 1);
                if (first) {
                    pend_row = row;
                    pend_col = col;
                    pend_pos = pos;
                    first = false;
                } else if (pos < a.cap) {
                    a.cidx[row * a.cap + pos] = col;
                }
            }
        }
    }
    if (MODE == MODE_EMIT && pend_row >= 0 && pend_pos < a.cap) a.cidx[pend_row * a.cap + pend_pos] = pend_col;
    if (LBUF) {
        __syncthreads();
        int *lbase = lcnt + BT; // [BT] place of the row's first buffered column in its global list
        if (tid < BT) {
            const int nb = min(lcnt[tid], LSLOTS);
            lbase[tid] = nb > 0 ? atomicAdd(&a.ccnt[m0 + tid], nb) : 0; // (rows past the end report nothing)
        }
        __syncthreads();
        for (int t = tid; t < BT * LSLOTS; t += 256) {
            const int r = t / LSLOTS, sl = t - r * LSLOTS;
            const int pos = lbase[r] + sl;
            if (sl < min(lcnt[r], LSLOTS) && pos < a.cap) a.cidx[(m0 + r) * a.cap + pos] = *lslot(r, sl);
        }
    }

    if (MODE == MODE_EMIT) return;
    if (MODE == MODE_MIN) {
        // 64 group minima per (row, split): column class (lane & 31) of each column half
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + slot_row(i, r);
                if (row < a.M) a.gmin[(row * a.nsplit + split) * 64 + (wn >> 6) * 32 + (lane & 31)] = b1[i][r];
            }
        return;
    }

    // ---- MODE_NN: row minimum over the workgroup, then every kept key inside the band of it ----
    __syncthreads(); // the operand pages are dead from here on
    unsigned *rowmin = (unsigned *)lds;                                         // [BT]
    int *rowcnt = (int *)(rowmin + BT);                                         // [BT]
    int *rowovf = rowcnt + BT;                                                  // [BT]
    unsigned long long *rowcand = (unsigned long long *)(rowovf + BT);          // [BT][VLQ_NN_CANDS]
    if (tid < BT) {
        rowmin[tid] = 0xFFFFFFFFu;
        rowcnt[tid] = 0;
        rowovf[tid] = -1;
#pragma unroll
        for (int s = 0; s < VLQ_NN_CANDS; ++s) rowcand[tid * VLQ_NN_CANDS + s] = KEY_MAX;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (b1[i][r] < BF16_NO_KEY) atomicMin(&rowmin[slot_row(i, r)], f2ord(b1[i][r]));
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int rl = slot_row(i, r);
            const uint32_t mo = rowmin[rl];
            if (mo == 0xFFFFFFFFu || m0 + rl >= a.M) continue;
            const float ra = a.an[m0 + rl];
            const float emin = __uint_as_float(__float_as_uint(ord2f(mo)) & keep);
            const float dmin = fmaxf(emin + ra, 0.f);
            const float band = emin + a.band_dist * (ra + dmin) + BF16_BAND_NORM * (3.f * ra + 2.f * dmin);
            const float ks[2] = {b1[i][r], b2[MODE == MODE_NN ? i : 0][r]};
            // a lane keeps two keys per row: when its second one lies inside the band a third may
            // have been dropped, so the row is handed on as incomplete
            if (ks[1] < BF16_NO_KEY && __uint_as_float(__float_as_uint(ks[1]) & keep) <= band) {
                const int slot = (wn >> 6) * 32 + (lane & 31);
                const int old = atomicCAS(&rowovf[rl], -1, slot);
                if (old != -1 && old != slot) rowovf[rl] = 64; // several slots
            }
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                if (!(ks[s] < BF16_NO_KEY)) continue;
                const uint32_t u = __float_as_uint(ks[s]);
                const float e = __uint_as_float(u & keep);
                if (e <= band) {
                    const uint32_t tj = u & ~keep;
                    const uint32_t col = (uint32_t)(t0 + (int)(tj >> 1) * tstride) * BT + wn + 32 * (tj & 1) + (lane & 31);
                    if (col >= (uint32_t)a.N) continue;
                    const int pos = atomicAdd(&rowcnt[rl], 1);
                    const float d = fmaxf(e + ra, 0.f) + 0.f;
                    if (pos < VLQ_NN_CANDS)
                        rowcand[rl * VLQ_NN_CANDS + pos] = ((uint64_t)__float_as_uint(d) << 32) | col;
                }
            }
        }
    __syncthreads();
    if (tid < BT && m0 + tid < a.M) {
        uint64_t *dst = a.cand + ((m0 + tid) * a.nsplit + split) * VLQ_NN_CANDS;
        const int cnt = rowcnt[tid], sl = rowovf[tid];
        const bool all = cnt > VLQ_NN_CANDS || sl == 64 || (sl >= 0 && cnt >= VLQ_NN_CANDS);
#pragma unroll
        for (int s = 0; s < VLQ_NN_CANDS; ++s) {
            uint64_t key = rowcand[tid * VLQ_NN_CANDS + s];
            if (all && s == 0) key = ((uint64_t)VLQ_NN_MARK << 32) | VLQ_NN_ALL;
            if (!all && sl >= 0 && s == cnt) key = ((uint64_t)VLQ_NN_MARK << 32) | (uint32_t)sl;
            dst[s] = key;
        }
    }
}

template <int MODE, bool HI = false>
static int launch_mode(Bf16Args &a, hipStream_t st)
{
    const int ntiles = (a.N + BT - 1) / BT;
    a.tiles_per_split = (ntiles + a.nsplit - 1) / a.nsplit;
    if (a.tile_stride < 1) a.tile_stride = 1;
    const int spt = a.D / BSTEP;
    const size_t lds_bytes = (size_t)(spt * 2 + 4) * PAGE * 16;
    dim3 grid((unsigned)((a.M + BT - 1) / BT), (unsigned)a.nsplit);
    auto go = [&](auto kern) -> int {
        // more than 64 KB of dynamic LDS has to be asked for
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds_bytes);
        if (e != hipSuccess) return (int)e;
        hipLaunchKernelGGL(kern, grid, dim3(256), lds_bytes, st, a);
        return 0;
    };
    switch (spt) {
    case 2: return go(k_coarse_bf16<2, MODE, HI>);
    case 4: return go(k_coarse_bf16<4, MODE, HI>);
    case 6: return go(k_coarse_bf16<6, MODE, HI>);
    case 8: return go(k_coarse_bf16<8, MODE, HI>);
    }
    return (int)hipErrorInvalidValue;
}

int launch_coarse_gemm_nn_bf16(const void *Aimg, const int *a_any_lo, int M, const void *Bimg, int N, int D,
                               const float *an, const float *bn, uint64_t *cand, int nsplit, float *band_norm,
                               float *band_dist, hipStream_t st)
{
    Bf16Args a = {};
    a.A = (const u32x4 *)Aimg;
    a.B = (const u32x4 *)Bimg;
    a.a_any_lo = a_any_lo;
    a.M = M;
    a.N = N;
    a.D = D;
    a.an = an;
    a.bn = bn;
    a.cand = cand;
    a.nsplit = nsplit;
    const int ntiles = (N + BT - 1) / BT;
    const int per = (ntiles + nsplit - 1) / nsplit;
    int bits = 1;
    while ((1 << bits) < 2 * per) ++bits;
    a.idx_bits = bits;
    // planting the index moves a key by less than 2^(bits - 23) of its own size, and a key
    // e = d - ||a||^2 is at most ||a||^2 + d in size; minimum and candidate both carry it
    a.band_dist = 2.5f * ldexpf(1.f, bits - 23);
    *band_norm = BF16_BAND_NORM;
    *band_dist = a.band_dist;
    if (M <= 0 || N <= 0) return 0;
    return launch_mode<MODE_NN>(a, st);
}

// ---------------------------------------------------------------------------
// w1 nearest centroids of every query (Alg. 3, first loop) without the nq x k matrix.
//
// Sweep 1 leaves 64 * nsplit group minima per query; the want-th smallest of them, tau, has at
// least want columns at or below it, so it bounds the want-th smallest approximate value from
// above, and it is tight: the want smallest columns rarely share a group.  Sweep 2 recomputes
// the product and lists every column with e <= tau + band, where the band covers the error of
// both sweeps' values against the exact distances.  The listed columns (about want of them)
// get their distance again as direct fp32 sums of squared differences and are sorted by
// (distance, index): the first w1 are the cells, exactly as a full exact ranking would give.
// A query whose list overflows (masses of coinciding distances) is ranked exactly over all
// columns instead.
// ---------------------------------------------------------------------------
// tau = the want-th smallest of the G group minima of a row, found bit by bit from the top of the
// ordered bit patterns: a wave per row, every trial value is compared with all minima and the lanes
// that lie below are counted with ballots (scalar work, no sorting, no barriers).
// (The hi-only sweeps carry their own, wider error inside the values they compare; the band added here is that
// of the fp32 arithmetic and of the split product, which the hi-only bound exceeds by far.)
__global__ __launch_bounds__(256) void k_cell_threshold(const float *__restrict__ gmin, int G, int want, int nq,
                                                        const float *__restrict__ qn, float *__restrict__ thr,
                                                        int32_t *__restrict__ ccnt)
{
    extern __shared__ uint32_t tkeys[]; // [4 waves][G]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = blockIdx.x * 4 + wave;
    if (row >= nq) return;
    uint32_t *mine = tkeys + wave * G; // (a wave reads back only what it wrote itself)
    const float *grow = gmin + (int64_t)row * G;
    uint32_t result = 0;
    if (G <= 512) { // the usual case: the minima in registers, all loads in flight together
        uint32_t u[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { // (clamped, not branched: the loads go out back to back)
            const float gv = grow[min(lane + 64 * e, G - 1)];
            u[e] = lane + 64 * e < G ? f2ord(gv) : 0xFFFFFFFFu;
        }
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t trial = result | (1u << bit);
            int below = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) below += __popcll(__ballot(u[e] < trial)); // (a filler is below nothing)
            if (below < want) result = trial;
        }
    } else if (G <= 4096) { // small batches have many column splits: still in registers
        uint32_t u[64];
#pragma unroll
        for (int e = 0; e < 64; ++e) {
            const float gv = grow[min(lane + 64 * e, G - 1)];
            u[e] = lane + 64 * e < G ? f2ord(gv) : 0xFFFFFFFFu;
        }
        // Most of the minima cannot matter: the want-th smallest of the two smallest values of every lane (128
        // of the values) bounds the answer from above, and closely, since the smallest values are spread over the
        // lanes; the few values at or below it are compacted and searched eight to a lane.
        bool pruned = false;
        if (want <= 128) {
            uint32_t m1 = 0xFFFFFFFFu, m2 = 0xFFFFFFFFu;
#pragma unroll
            for (int e = 0; e < 64; ++e) {
                m2 = min(m2, max(m1, u[e]));
                m1 = min(m1, u[e]);
            }
            uint32_t bound = 0;
            for (int bit = 31; bit >= 0; --bit) {
                const uint32_t trial = bound | (1u << bit);
                if (__popcll(__ballot(m1 < trial)) + __popcll(__ballot(m2 < trial)) < want) bound = trial;
            }
            int keep = 0;
#pragma unroll
            for (int e = 0; e < 64; ++e) keep += u[e] <= bound;
            int at = keep;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_up(at, o, 64);
                if (lane >= o) at += t;
            }
            const int total = __shfl(at, 63, 64);
            if (total <= 512) {
                at -= keep;
#pragma unroll
                for (int e = 0; e < 64; ++e)
                    if (u[e] <= bound) mine[at++] = u[e];
                __builtin_amdgcn_wave_barrier();
                uint32_t v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = lane + 64 * e < total ? mine[lane + 64 * e] : 0xFFFFFFFFu;
                for (int bit = 31; bit >= 0; --bit) {
                    const uint32_t trial = result | (1u << bit);
                    int below = 0;
#pragma unroll
                    for (int e = 0; e < 8; ++e) below += __popcll(__ballot(v[e] < trial));
                    if (below < want) result = trial;
                }
                pruned = true;
            }
        }
        if (!pruned)
            for (int bit = 31; bit >= 0; --bit) {
                const uint32_t trial = result | (1u << bit);
                int below = 0;
#pragma unroll
                for (int e = 0; e < 64; ++e) below += __popcll(__ballot(u[e] < trial));
                if (below < want) result = trial;
            }
    } else {
        for (int i = lane; i < G; i += 64) mine[i] = f2ord(grow[i]);
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t trial = result | (1u << bit);
            int below = 0;
            for (int i = lane; i < G; i += 64) below += __popcll(__ballot(mine[i] < trial));
            // G is a multiple of 64, so every lane makes the same number of rounds and `below` is uniform
            if (below < want) result = trial;
        }
    }
    if (lane == 0) {
        const float tau = ord2f(result);
        const float ra = qn[row];
        const float dt = fmaxf(tau + ra, 0.f);
        // below BF16_NO_KEY, so that columns past the end never qualify
        thr[row] = fminf(tau + BF16_BAND_NORM * (3.f * ra + 2.f * dt), BF16_NO_KEY);
        ccnt[row] = 0;
    }
}

// direct ||y - c||^2 by 16 lanes (l16 = lane % 16), butterfly over the 16: same value in all of them
__device__ __forceinline__ float sqdist16(const float *yv, const float *__restrict__ rowp, int D, int l16, bool vec)
{
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
    return row16_sum(acc);
}

// the same sums for four rows at once (their loads in flight together)
__device__ __forceinline__ void sqdist16x4(const float *yv, const float *const (&rowp)[4], int D, int l16, bool vec,
                                           float (&out)[4])
{
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    if (vec) {
        for (int d = l16 * 4; d < D; d += 64) {
            f32x4 cv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) cv[u] = *(const f32x4 *)(rowp[u] + d);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float t0 = yv[d] - cv[u].x, t1 = yv[d + 1] - cv[u].y, t2 = yv[d + 2] - cv[u].z, t3 = yv[d + 3] - cv[u].w;
                acc[u] = fmaf(t0, t0, acc[u]);
                acc[u] = fmaf(t1, t1, acc[u]);
                acc[u] = fmaf(t2, t2, acc[u]);
                acc[u] = fmaf(t3, t3, acc[u]);
            }
        }
    } else {
        for (int d = l16; d < D; d += 16) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float t = yv[d] - rowp[u][d];
                acc[u] = fmaf(t, t, acc[u]);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) out[u] = row16_sum(acc[u]);
}

#define CELLS_FB 2048 // buffer of the exact ranking over all columns

__global__ __launch_bounds__(256) void k_cells_exact(const float *__restrict__ Q, int D,
                                                     const float *__restrict__ C, int k,
                                                     const int32_t *__restrict__ ccnt,
                                                     const int32_t *__restrict__ cidx, int cap, int w,
                                                     int32_t *__restrict__ cells, float *__restrict__ cell_dist,
                                                     int32_t *__restrict__ pair_cnt, int32_t *__restrict__ pair_rank)
{
    extern __shared__ uint64_t ckeys[]; // [max(cap, CELLS_FB)] then yv [D]
    __shared__ int sh_n;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub16 = lane >> 4, l16 = lane & 15;
    const int row = blockIdx.x;
    const int nkeys = cap > CELLS_FB ? cap : CELLS_FB;
    float *yv = (float *)(ckeys + nkeys);
    for (int d = tid; d < D; d += 256) yv[d] = Q[(int64_t)row * D + d];
    const bool vec = (D % 4 == 0) && (((uintptr_t)C) % 16 == 0);
    const int listed = ccnt[row];
    int cnt;
    __syncthreads();
    if (listed <= cap) {
        cnt = listed;
        for (int c0 = wave * 4; c0 < cnt; c0 += 64) { // four candidates per 16 lanes and round
            int ii[4];
            const float *rp[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + 16 * u + sub16;
                ii[u] = c < cnt ? cidx[(int64_t)row * cap + c] : 0;
                rp[u] = C + (int64_t)ii[u] * D;
            }
            float dd[4];
            sqdist16x4(yv, rp, D, l16, vec, dd);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + 16 * u + sub16;
                if (l16 == 0 && c < cnt) ckeys[c] = make_key(dd[u], (uint32_t)ii[u]);
            }
        }
        __syncthreads();
        if (cnt <= 256) {
            // a key per thread: its rank among the (distinct) keys is its place in the output
            const uint64_t mine = tid < cnt ? ckeys[tid] : KEY_MAX;
            int rank = 0;
            for (int c = 0; c < cnt; ++c) rank += ckeys[c] < mine;
            __syncthreads();
            if (tid < cnt) ckeys[rank] = mine;
            __syncthreads();
        } else {
            const int sz = next_pow2_dev(cnt);
            for (int c = cnt + tid; c < sz; c += 256) ckeys[c] = KEY_MAX;
            __syncthreads();
            block_bitonic_sort<256>(ckeys, sz, tid);
        }
    } else {
        // exact ranking over all columns: keys below the current w-th smallest are collected;
        // a full buffer is sorted and cut back to w
        uint64_t cut = KEY_MAX;
        if (tid == 0) sh_n = 0;
        __syncthreads();
        for (int i0 = 0; i0 < k; i0 += 16) {
            const int i = i0 + wave * 4 + sub16;
            const float d = sqdist16(yv, C + (int64_t)min(i, k - 1) * D, D, l16, vec);
            const uint64_t key = make_key(d, (uint32_t)i);
            if (l16 == 0 && i < k && key < cut) ckeys[atomicAdd(&sh_n, 1)] = key;
            __syncthreads();
            const int n = sh_n;
            __syncthreads(); // everyone has read the fill level before the next round appends
            if (n > CELLS_FB - 16 || i0 + 16 >= k) {
                const int sz = next_pow2_dev(n);
                for (int c = n + tid; c < sz; c += 256) ckeys[c] = KEY_MAX;
                __syncthreads();
                block_bitonic_sort<256>(ckeys, sz, tid);
                if (n >= w) cut = ckeys[w - 1];
                __syncthreads();
                if (tid == 0) sh_n = min(n, w);
                __syncthreads();
            }
        }
        cnt = sh_n;
    }
    for (int e = tid; e < w; e += 256) {
        const uint64_t key = ckeys[e];
        const bool ok = e < cnt && key != KEY_MAX;
        cells[(int64_t)row * w + e] = ok ? (int32_t)(uint32_t)key : -1;
        if (cell_dist) cell_dist[(int64_t)row * w + e] = ok ? ord2f((uint32_t)(key >> 32)) : INFINITY;
        // (query, cell) pairs per cell, for the cell-major pass over the neighbour centroids
        if (pair_cnt && ok) pair_rank[(int64_t)row * w + e] = atomicAdd(&pair_cnt[(uint32_t)key], 1);
    }
}

bool cells_bf16_plan(int nq, int k, int D, int w1, bool hi_only, int *nsplit, int *cap)
{
    if (!coarse_bf16_supported(D)) return false;
    const int ntiles = (k + BT - 1) / BT;
    const int strips = (nq + BT - 1) / BT;
    int ns = 512 / strips; // one round of two workgroups per CU
    const int need = (2 * w1 + 63) / 64; // at least twice as many groups as cells wanted
    if (ns < need) ns = need;
    if (ns > 64) ns = 64;
    if (ns > ntiles / 2) ns = ntiles / 2; // every group sees at least two tiles
    if (ns < 1 || ns < need) return false;
    const int per = (ntiles + ns - 1) / ns;
    ns = (ntiles + per - 1) / per; // no empty split
    if (ns < need) return false;
    *nsplit = ns;
    // the hi-only sweeps list more columns (wider band): room for eight times the cells wanted
    const int room = (hi_only ? 8 : 4) * w1;
    *cap = next_pow2(room > (hi_only ? 512 : 256) ? room : (hi_only ? 512 : 256));
    return true;
}

size_t cells_bf16_workspace(int nq, int nsplit, int cap, size_t *gmin_off, size_t *thr_off, size_t *ccnt_off,
                            size_t *cidx_off)
{
    size_t off = 0;
    auto take = [&](size_t bytes) {
        off = (off + 255) & ~(size_t)255;
        const size_t at = off;
        off += bytes;
        return at;
    };
    *gmin_off = take((size_t)nq * nsplit * 64 * 4);
    *thr_off = take((size_t)nq * 4);
    *ccnt_off = take((size_t)nq * 4);
    *cidx_off = take((size_t)nq * cap * 4);
    return off;
}

int launch_cells_bf16_coarse(const void *Qimg, const int *q_any_lo, int nq, const void *Cimg, int k, int D,
                             const float *qn, const float *cn, bool hi_only, int w1, int nsplit, int cap, void *ws,
                             hipStream_t st)
{
    size_t og, ot, oc, oi;
    cells_bf16_workspace(nq, nsplit, cap, &og, &ot, &oc, &oi);
    char *base = (char *)ws;
    Bf16Args a = {};
    a.A = (const u32x4 *)Qimg;
    a.B = (const u32x4 *)Cimg;
    a.a_any_lo = q_any_lo;
    a.M = nq;
    a.N = k;
    a.D = D;
    a.an = qn;
    a.bn = cn;
    a.nsplit = nsplit;
    a.gmin = (float *)(base + og);
    a.thr = (float *)(base + ot);
    a.ccnt = (int32_t *)(base + oc);
    a.cidx = (int32_t *)(base + oi);
    a.cap = cap;
    // The first sweep only has to bound the w1-th smallest distance from above, and the w1-th
    // smallest over any subset of the columns does: with many tiles per split it looks at every
    // other tile (half the work; about twice the columns pass the second sweep's threshold and are
    // re-evaluated exactly, still well inside the candidate lists).
    const int ntiles = (k + BT - 1) / BT;
    a.tile_stride = (ntiles + nsplit - 1) / nsplit >= 8 ? 2 : 1;
    int rc = hi_only ? launch_mode<MODE_MIN, true>(a, st) : launch_mode<MODE_MIN>(a, st);
    a.tile_stride = 1;
    if (rc) return rc;
    const int G = nsplit * 64;
    hipLaunchKernelGGL(k_cell_threshold, dim3((unsigned)((nq + 3) / 4)), dim3(256), (size_t)4 * G * 4, st, a.gmin, G,
                       w1, nq, qn, (float *)(base + ot), a.ccnt);
    return hi_only ? launch_mode<MODE_EMIT, true>(a, st) : launch_mode<MODE_EMIT>(a, st);
}

void launch_cells_bf16_exact(const float *Q, int nq, int D, const float *C, int k, int w1, int cap, const void *ws,
                             int nsplit, int32_t *cells, float *cell_dist, int32_t *pair_cnt, int32_t *pair_rank,
                             hipStream_t st)
{
    size_t og, ot, oc, oi;
    cells_bf16_workspace(nq, nsplit, cap, &og, &ot, &oc, &oi);
    const char *base = (const char *)ws;
    const int nkeys = cap > CELLS_FB ? cap : CELLS_FB;
    hipLaunchKernelGGL(k_cells_exact, dim3((unsigned)nq), dim3(256), (size_t)nkeys * 8 + (size_t)D * 4, st, Q, D, C, k,
                       (const int32_t *)(base + oc), (const int32_t *)(base + oi), cap, w1, cells, cell_dist, pair_cnt,
                       pair_rank);
}
