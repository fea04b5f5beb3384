// First-level quantiser on the bf16 matrix cores (Eq. 2; Alg. 1 "nearest centroid").
//
// An fp32 value v is split into two bf16 numbers, hi = rne(v) and lo = rne(v - hi),
// so that |v - hi - lo| <= 2^-18 |v|.  The inner product of two split vectors is
// taken as hi.hi + hi.lo + lo.hi with fp32 accumulation on
// v_mfma_f32_32x32x16_bf16; the dropped lo.lo term and the representation error
// together stay below 3 * 2^-18 |x| |c|.  The result only shortlists centroids: every
// column whose approximate distance lies within the error band of the row minimum
// is handed on and re-evaluated there as a direct fp32 sum of squared differences,
// so the decision itself is taken in fp32 exactly as by the fp32 path.
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
// 128 rows of A stay in LDS for the whole sweep (D <= 128: 64 KB); the pages of B
// stream global -> registers (four steps ahead) -> a two-page-pair ring in LDS, one
// barrier per step.  Two workgroups share a CU (2 x 80 KB of LDS), so one's
// selection epilogue overlaps the other's MFMAs.
#include "common.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

#define BT 128          // rows per block
#define BSTEP 16        // contraction indices per step
#define PAGE 256        // 16-byte chunks per page
#define BF16_MAX_D 128  // A block resident in LDS: D / 16 steps x 2 pages x 4 KB

__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// X [rows x D] fp32 -> image [ceil(rows / 128)][D / 16][hi page, lo page]; rows past
// the end are written as zeros.  *any_lo is raised when some lo is non-zero.
// One thread per (row, chunk of 8 values).
__global__ __launch_bounds__(256) void k_split_bf16(const float *__restrict__ X, int64_t rows, int D,
                                                    int64_t padded_rows, u32x4 *__restrict__ img,
                                                    int *__restrict__ any_lo)
{
    const int cpr = D / 8; // chunks per row
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    bool nz = false;
    if (i < padded_rows * cpr) {
        const int64_t row = i / cpr;
        const int ch = (int)(i - row * cpr);
        u32x4 ph = {0, 0, 0, 0}, pl = {0, 0, 0, 0};
        if (row < rows) {
            const f32x4 v0 = *(const f32x4 *)(X + row * D + ch * 8);
            const f32x4 v1 = *(const f32x4 *)(X + row * D + ch * 8 + 4);
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
    if (__ballot(nz) != 0 && (threadIdx.x & 63) == 0) atomicOr(any_lo, 1);
}

__global__ void k_zero_flag(int *p) { *p = 0; }

bool coarse_bf16_supported(int D) { return D == 32 || D == 64 || D == 96 || D == 128; }

size_t coarse_bf16_image_bytes(int64_t rows, int D)
{
    const int64_t blocks = (rows + BT - 1) / BT;
    return (size_t)blocks * BT * D * 4;
}

void launch_split_bf16(const float *X, int64_t rows, int D, void *img, int *any_lo, hipStream_t st)
{
    hipLaunchKernelGGL(k_zero_flag, dim3(1), dim3(1), 0, st, any_lo);
    const int64_t padded = (rows + BT - 1) / BT * BT;
    const int64_t n = padded * (D / 8);
    if (n <= 0) return;
    hipLaunchKernelGGL(k_split_bf16, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, X, rows, D, padded,
                       (u32x4 *)img, any_lo);
}

// Error of the split product relative to ||a||^2 + ||b||^2 <= 3 ||a||^2 + 2 d: minimum and
// candidate each carry 2 * 3 * 2^-18 |a| |b| <= 3 * 2^-18 (||a||^2 + ||b||^2), rounded up.
#define BF16_BAND_NORM 3e-5f
// Columns past the end of B get this "norm": finite, so that index bits can be planted
// in the key, and beyond BF16_NO_KEY, from where on a key counts as absent.
#define BF16_NO_COLUMN 3e38f
#define BF16_NO_KEY 1e38f

struct Bf16NNArgs {
    const u32x4 *A; // image of the rows
    const u32x4 *B; // image of the columns
    const int *a_any_lo;
    int M, N, D;
    const float *an, *bn;
    uint64_t *cand;
    int nsplit, tiles_per_split;
    int idx_bits; // low mantissa bits of a running key that hold (tile, column block)
    float band_dist;
};

// SPT = D / 16 steps per tile; PDEPTH page pairs of B in flight in registers (divides SPT, so
// that every register set and ring half has a fixed role in the unrolled tile body).
template <int SPT>
__global__ __launch_bounds__(256, 2) void k_coarse_nn_bf16(Bf16NNArgs a)
{
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
    const int ntl = t1 > t0 ? t1 - t0 : 0;
    const int last = ntl * SPT - 1; // last step of the split
    const bool use_lo = *a.a_any_lo != 0;
    u32x4 *Apages = lds;
    u32x4 *ring = lds + SPT * 2 * PAGE;

    // the block of A
    {
        const u32x4 *src = a.A + (int64_t)blockIdx.x * SPT * 2 * PAGE;
#pragma unroll
        for (int p = 0; p < SPT * 2; ++p) Apages[p * PAGE + tid] = src[p * PAGE + tid];
    }

    // B pages: step j of this split is the page pair at (t0 * SPT + j) * 2.  Loads past the
    // last step re-read the last pair, so that the number of loads in flight never varies.
    const u32x4 *bsrc = a.B + (int64_t)t0 * SPT * 2 * PAGE + tid;
    auto fetch = [&](u32x4 (&r)[2], int j) {
        j = min(j, last);
        r[0] = bsrc[(int64_t)(2 * j) * PAGE];
        r[1] = bsrc[(int64_t)(2 * j + 1) * PAGE];
    };
    u32x4 rb[PDEPTH][2];
    if (ntl > 0) {
#pragma unroll
        for (int j = 0; j < PDEPTH; ++j) fetch(rb[j], j);
        ring[tid] = rb[0][0];
        ring[PAGE + tid] = rb[0][1];
        fetch(rb[0], PDEPTH);
    }

    // fragment of a 32-row block: lane reads row (lane & 31), chunk (lane >> 5)
    const int frow = lane & 31;
    const int fpos = 2 * frow + ((lane >> 5) ^ ((frow >> 2) & 1));
    const int fa0 = 2 * wm + fpos, fa1 = fa0 + 64; // + 32 rows
    const int fb0 = 2 * wn + fpos, fb1 = fb0 + 64;

    float b1[2][16], b2[2][16];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) b1[i][r] = b2[i][r] = INFINITY;
    const uint32_t keep = ~((1u << a.idx_bits) - 1u);

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    __syncthreads();
    for (int tl = 0; tl < ntl; ++tl) {
        // column norms of this tile, asked for now and used after its last step
        const int64_t n0 = (int64_t)(t0 + tl) * BT;
        float cb[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t col = n0 + wn + 32 * j + (lane & 31);
            cb[j] = a.bn[min(col, (int64_t)a.N - 1)];
            cb[j] = col < a.N ? cb[j] : BF16_NO_COLUMN;
        }
#pragma unroll
        for (int u = 0; u < SPT; ++u) {
            const int s = tl * SPT + u;
            // page pair of step s + 1 into the other half of the ring, its registers refilled
            {
                u32x4 *dst = ring + ((u + 1) & 1) * 2 * PAGE;
                dst[tid] = rb[(u + 1) % PDEPTH][0];
                dst[PAGE + tid] = rb[(u + 1) % PDEPTH][1];
                fetch(rb[(u + 1) % PDEPTH], s + 1 + PDEPTH);
            }
            const u32x4 *ap = Apages + u * 2 * PAGE;
            const u32x4 *bp = ring + (u & 1) * 2 * PAGE;
            bf16x8 ah[2], bh[2], bl[2];
            ah[0] = __builtin_bit_cast(bf16x8, ap[fa0]);
            ah[1] = __builtin_bit_cast(bf16x8, ap[fa1]);
            bh[0] = __builtin_bit_cast(bf16x8, bp[fb0]);
            bh[1] = __builtin_bit_cast(bf16x8, bp[fb1]);
            bl[0] = __builtin_bit_cast(bf16x8, bp[PAGE + fb0]);
            bl[1] = __builtin_bit_cast(bf16x8, bp[PAGE + fb1]);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bh[j], acc[i][j], 0, 0, 0);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bl[j], acc[i][j], 0, 0, 0);
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
        // tile finished: fold e = ||b||^2 - 2 <a, b> (the row norm is common to a row and joins
        // at the end) into the running two smallest of every row slot of the lane
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t tj = (uint32_t)(tl * 2 + j);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float e = fmaf(-2.f, acc[i][j][r], cb[j]);
                    const float key = __uint_as_float((__float_as_uint(e) & keep) | tj);
                    b2[i][r] = __builtin_amdgcn_fmed3f(b1[i][r], b2[i][r], key);
                    b1[i][r] = fminf(b1[i][r], key);
                    acc[i][j][r] = 0.f;
                }
        }
    }

    // ---- row minimum over the workgroup, then every kept key inside the band of it ----
    __syncthreads(); // the operand pages are dead from here on
    unsigned *rowmin = (unsigned *)lds;                                         // [BT]
    int *rowcnt = (int *)(rowmin + BT);                                         // [BT]
    unsigned long long *rowcand = (unsigned long long *)(rowcnt + BT);          // [BT][VLQ_NN_CANDS]
    if (tid < BT) {
        rowmin[tid] = 0xFFFFFFFFu;
        rowcnt[tid] = 0;
#pragma unroll
        for (int s = 0; s < VLQ_NN_CANDS; ++s) rowcand[tid * VLQ_NN_CANDS + s] = KEY_MAX;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int rl = wm + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (b1[i][r] < BF16_NO_KEY) atomicMin(&rowmin[rl], f2ord(b1[i][r]));
        }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int rl = wm + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            const uint32_t mo = rowmin[rl];
            if (mo == 0xFFFFFFFFu || m0 + rl >= a.M) continue;
            const float ra = a.an[m0 + rl];
            const float emin = __uint_as_float(__float_as_uint(ord2f(mo)) & keep);
            const float dmin = fmaxf(emin + ra, 0.f);
            const float band = emin + a.band_dist * (ra + dmin) + BF16_BAND_NORM * (3.f * ra + 2.f * dmin);
            const float ks[2] = {b1[i][r], b2[i][r]};
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                if (!(ks[s] < BF16_NO_KEY)) continue;
                const uint32_t u = __float_as_uint(ks[s]);
                const float e = __uint_as_float(u & keep);
                if (e <= band) {
                    const uint32_t tj = u & ~keep;
                    const uint32_t col = (uint32_t)(t0 + (int)(tj >> 1)) * BT + wn + 32 * (tj & 1) + (lane & 31);
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
#pragma unroll
        for (int s = 0; s < VLQ_NN_CANDS; ++s) dst[s] = rowcand[tid * VLQ_NN_CANDS + s];
    }
}

int launch_coarse_gemm_nn_bf16(const void *Aimg, const int *a_any_lo, int M, const void *Bimg, int N, int D,
                               const float *an, const float *bn, uint64_t *cand, int nsplit, float *band_norm,
                               float *band_dist, hipStream_t st)
{
    Bf16NNArgs a;
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
    a.tiles_per_split = (ntiles + nsplit - 1) / nsplit;
    int bits = 1;
    while ((1 << bits) < 2 * a.tiles_per_split) ++bits;
    a.idx_bits = bits;
    // planting the index moves a key by less than 2^(bits - 23) of its own size, and a key
    // e = d - ||a||^2 is at most ||a||^2 + d in size; minimum and candidate both carry it
    a.band_dist = 2.5f * ldexpf(1.f, bits - 23);
    *band_norm = BF16_BAND_NORM;
    *band_dist = a.band_dist;
    if (M <= 0 || N <= 0) return 0;
    const int spt = D / BSTEP;
    const size_t lds_bytes = (size_t)(spt * 2 + 4) * PAGE * 16;
    dim3 grid((unsigned)((M + BT - 1) / BT), (unsigned)nsplit);
    auto go = [&](auto kern) -> int {
        // more than 64 KB of dynamic LDS has to be asked for once per kernel
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds_bytes);
        if (e != hipSuccess) return (int)e;
        hipLaunchKernelGGL(kern, grid, dim3(256), lds_bytes, st, a);
        return 0;
    };
    switch (spt) {
    case 2: return go(k_coarse_nn_bf16<2>);
    case 4: return go(k_coarse_nn_bf16<4>);
    case 6: return go(k_coarse_nn_bf16<6>);
    case 8: return go(k_coarse_nn_bf16<8>);
    }
    return (int)hipErrorInvalidValue;
}
