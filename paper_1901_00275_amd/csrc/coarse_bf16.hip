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
// Workgroup = 256 threads = 4 waves, tile 128 x 128, each wave a 64 x 64 quadrant
// (2 x 2 MFMA blocks).  Operands are streamed in slabs of 32 contraction indices:
// global -> registers -> LDS, double buffered, one barrier per slab; two workgroups
// share a CU so one's epilogue overlaps the other's MFMAs.  An LDS slab row is
// 64 bytes = four 16-byte chunks; chunk c of row r is stored at position
// c ^ ((r >> 1) & 3), which makes both the row-contiguous writes and the
// 32-rows-by-one-chunk fragment reads free of bank conflicts.
#include "common.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

#define BT 128
#define BK 32

__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// X [count] fp32 -> hi, lo [count] bf16; *any_lo is raised when some lo is non-zero.
__global__ __launch_bounds__(256) void k_split_bf16(const float *__restrict__ X, int64_t count4,
                                                    uint16_t *__restrict__ hi, uint16_t *__restrict__ lo,
                                                    int *__restrict__ any_lo)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    bool nz = false;
    if (i < count4) {
        const f32x4 v = ((const f32x4 *)X)[i];
        uint32_t h[4], l[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            h[e] = bf16_rne(v[e]);
            const float r = v[e] - __uint_as_float(h[e] << 16);
            l[e] = bf16_rne(r);
            nz |= (l[e] & 0x7FFFu) != 0;
        }
        u32x2 ph, pl;
        ph.x = h[0] | (h[1] << 16);
        ph.y = h[2] | (h[3] << 16);
        pl.x = l[0] | (l[1] << 16);
        pl.y = l[2] | (l[3] << 16);
        ((u32x2 *)hi)[i] = ph;
        ((u32x2 *)lo)[i] = pl;
    }
    if (__ballot(nz) != 0 && (threadIdx.x & 63) == 0) atomicOr(any_lo, 1);
}

__global__ void k_zero_flag(int *p) { *p = 0; }

void launch_split_bf16(const float *X, int64_t rows, int D, uint16_t *hi, uint16_t *lo, int *any_lo,
                       hipStream_t st)
{
    hipLaunchKernelGGL(k_zero_flag, dim3(1), dim3(1), 0, st, any_lo);
    const int64_t count4 = rows * D / 4;
    if (count4 <= 0) return;
    hipLaunchKernelGGL(k_split_bf16, dim3((unsigned)((count4 + 255) / 256)), dim3(256), 0, st, X, count4, hi, lo,
                       any_lo);
}

bool coarse_bf16_supported(int D) { return D % BK == 0; }

// Rounding band of the split product relative to ||a||^2 + ||b||^2 (both rows of a
// comparison carry the error, hence twice 2 * 3 * 2^-18 / 2, rounded up).
#define BF16_BAND_NORM 3e-5f
// Columns past the end of B get this "norm": finite, so that the index bits can be
// planted in it, and above BF16_INVALID_BITS, from where on a key counts as absent.
#define BF16_NO_COLUMN 3e38f
#define BF16_INVALID_BITS 0x7E000000u

struct Bf16NNArgs {
    const u32x4 *Ah, *Al; // [M x D/8]
    const u32x4 *Bh, *Bl; // [N x D/8]
    const int *a_any_lo;
    int M, N, D;
    const float *an, *bn;
    uint64_t *cand;
    int nsplit, tiles_per_split;
    int idx_bits; // low mantissa bits of a running key that hold (tile, column block)
    float band_dist;
};

__global__ __launch_bounds__(256, 2) void k_coarse_nn_bf16(Bf16NNArgs a)
{
    __shared__ u32x4 slab[2][4][BT * 4]; // [buffer][Ah, Al, Bh, Bl][row * 4 + swizzled chunk]
    __shared__ float ran[BT];
    __shared__ unsigned rowmin[BT];
    __shared__ int rowcnt[BT];
    __shared__ unsigned long long rowcand[BT][VLQ_NN_CANDS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int64_t m0 = (int64_t)blockIdx.x * BT;
    const int split = blockIdx.y;
    const int ntiles = (a.N + BT - 1) / BT;
    const int t0 = split * a.tiles_per_split;
    const int t1 = min(ntiles, t0 + a.tiles_per_split);
    const int DC = a.D / 8;   // 16-byte chunks per row
    const int SL = a.D / BK;  // slabs per tile
    const int total = (t1 - t0) * SL;
    const bool use_lo = *a.a_any_lo != 0;

    if (tid < BT) {
        ran[tid] = m0 + tid < a.M ? a.an[m0 + tid] : 0.f;
        rowmin[tid] = 0xFFFFFFFFu;
        rowcnt[tid] = 0;
#pragma unroll
        for (int s = 0; s < VLQ_NN_CANDS; ++s) rowcand[tid][s] = KEY_MAX;
    }

    // staging: thread moves chunks q = tid and tid + 256 of every operand slab
    int lrow[2], lpos[2];
    int64_t offA[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int q = tid + 256 * p;
        lrow[p] = q >> 2;
        const int c = q & 3;
        lpos[p] = lrow[p] * 4 + (c ^ ((lrow[p] >> 1) & 3));
        int64_t r = m0 + lrow[p];
        if (r > a.M - 1) r = a.M - 1; // rows past the end repeat the last one and are never emitted
        offA[p] = r * DC + c;
    }
    // fragment reads: lane reads row (lane & 31) of a 32-row block, chunk 2 s + (lane >> 5)
    const int frow = lane & 31;
    const int fsw = (frow >> 1) & 3;
    const int fch = lane >> 5;

    u32x4 ra_h[2], ra_l[2], rb_h[2], rb_l[2];
    auto issue = [&](int g) {
        const int t = t0 + g / SL, kc = (g % SL) * (BK / 8);
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            int64_t r = (int64_t)t * BT + lrow[p];
            if (r > a.N - 1) r = a.N - 1;
            const int64_t ob = r * DC + (tid & 3) + kc;
            ra_h[p] = a.Ah[offA[p] + kc];
            ra_l[p] = a.Al[offA[p] + kc];
            rb_h[p] = a.Bh[ob];
            rb_l[p] = a.Bl[ob];
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            slab[buf][0][lpos[p]] = ra_h[p];
            slab[buf][1][lpos[p]] = ra_l[p];
            slab[buf][2][lpos[p]] = rb_h[p];
            slab[buf][3][lpos[p]] = rb_l[p];
        }
    };

    float b1[2][16], b2[2][16];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) b1[i][r] = b2[i][r] = INFINITY;
    const uint32_t keep = ~((1u << a.idx_bits) - 1u);

    f32x16 acc[2][2];
    __syncthreads();
    auto reset_acc = [&]() {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                // the row norm enters through the accumulator: -2 acc = ||a||^2 - 2 <a, b>
                const float v = -0.5f * ran[wm + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)];
                acc[i][0][r] = v;
                acc[i][1][r] = v;
            }
    };
    reset_acc();

    if (total > 0) {
        issue(0);
        stash(0);
    }
    __syncthreads();
    for (int g = 0; g < total; ++g) {
        const int cur = g & 1;
        const bool more = g + 1 < total;
        if (more) issue(g + 1);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            bf16x8 ah[2], al[2], bh[2], bl[2];
            const int ch = ((2 * s + fch) ^ fsw);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int ia = (wm + 32 * i + frow) * 4 + ch;
                const int ib = (wn + 32 * i + frow) * 4 + ch;
                ah[i] = __builtin_bit_cast(bf16x8, slab[cur][0][ia]);
                al[i] = __builtin_bit_cast(bf16x8, slab[cur][1][ia]);
                bh[i] = __builtin_bit_cast(bf16x8, slab[cur][2][ib]);
                bl[i] = __builtin_bit_cast(bf16x8, slab[cur][3][ib]);
            }
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
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], bh[j], acc[i][j], 0, 0, 0);
            }
        }
        if (more) stash(cur ^ 1);
        __syncthreads();
        if (g % SL == SL - 1) {
            // tile finished: fold its 64 values per lane into the running two smallest per row slot
            const int tl = g / SL; // tile index inside this split
            const int64_t n0 = (int64_t)(t0 + tl) * BT;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int64_t col = n0 + wn + 32 * j + (lane & 31);
                const float cb = col < a.N ? a.bn[col] : BF16_NO_COLUMN;
                const uint32_t tj = (uint32_t)(tl * 2 + j);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float e = fmaf(-2.f, acc[i][j][r], cb);
                        const float key = __uint_as_float((__float_as_uint(e) & keep) | tj);
                        b2[i][r] = __builtin_amdgcn_fmed3f(b1[i][r], b2[i][r], key);
                        b1[i][r] = fminf(b1[i][r], key);
                    }
            }
            reset_acc();
        }
    }

    // ---- row minimum over the workgroup, then every kept key inside the band of it ----
    auto clamp_bits = [&](float v) -> uint32_t {
        const uint32_t u = __float_as_uint(v);
        return (u & 0x80000000u) ? (u & ~keep) : u; // negative approximations count as zero
    };
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int rl = wm + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            const uint32_t u = clamp_bits(b1[i][r]);
            if (u < BF16_INVALID_BITS) atomicMin(&rowmin[rl], u);
        }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int rl = wm + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            const uint32_t mn = rowmin[rl];
            if (mn >= BF16_INVALID_BITS) continue;
            const float dmin = __uint_as_float(mn & keep);
            const float band = dmin + a.band_dist * dmin + BF16_BAND_NORM * (3.f * ran[rl] + 2.f * dmin);
            const float ks[2] = {b1[i][r], b2[i][r]};
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const uint32_t u = clamp_bits(ks[s]);
                if (u >= BF16_INVALID_BITS) continue;
                const float d = __uint_as_float(u & keep);
                if (d <= band) {
                    const uint32_t tj = u & ~keep;
                    const uint32_t col = (uint32_t)(t0 + (int)(tj >> 1)) * BT + wn + 32 * (tj & 1) + (lane & 31);
                    if (col >= (uint32_t)a.N) continue;
                    const int pos = atomicAdd(&rowcnt[rl], 1);
                    if (pos < VLQ_NN_CANDS) rowcand[rl][pos] = ((uint64_t)(u & keep) << 32) | col;
                }
            }
        }
    __syncthreads();
    if (tid < BT && m0 + tid < a.M) {
        uint64_t *dst = a.cand + ((m0 + tid) * a.nsplit + split) * VLQ_NN_CANDS;
#pragma unroll
        for (int s = 0; s < VLQ_NN_CANDS; ++s) dst[s] = rowcand[tid][s];
    }
}

void launch_coarse_gemm_nn_bf16(const uint16_t *Ah, const uint16_t *Al, const int *a_any_lo, int M,
                                const uint16_t *Bh, const uint16_t *Bl, int N, int D, const float *an,
                                const float *bn, uint64_t *cand, int nsplit, float *band_norm,
                                float *band_dist, hipStream_t st)
{
    Bf16NNArgs a;
    a.Ah = (const u32x4 *)Ah;
    a.Al = (const u32x4 *)Al;
    a.Bh = (const u32x4 *)Bh;
    a.Bl = (const u32x4 *)Bl;
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
    // truncating the low mantissa bits moves a value by less than 2^(bits - 23) of itself;
    // minimum and candidate both carry it
    a.band_dist = 2.2f * ldexpf(1.f, bits - 23);
    *band_norm = BF16_BAND_NORM;
    *band_dist = a.band_dist;
    if (M <= 0 || N <= 0) return;
    dim3 grid((unsigned)((M + BT - 1) / BT), (unsigned)nsplit);
    hipLaunchKernelGGL(k_coarse_nn_bf16, grid, dim3(256), 0, st, a);
}
