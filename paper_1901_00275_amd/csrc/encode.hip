// Encoding on the GPU (Alg. 1 + Alg. 2): the second half, after the
// nearest-centroid candidates have come out of the matrix-core contraction.
#include "common.h"

#define ENC_NT 256
#define ENC_PB_MAX 32

// ||x - row||^2 by each group of 16 lanes (l16 = lane % 16): four components per lane and step, then
// the adder's lane-crossing sum.  Every exact evaluation of a centroid distance in this file goes
// through it, so that coinciding centroids get bit-identical values and ties fall to the smaller index.
__device__ __forceinline__ float sqdist16(const float *x, const float *__restrict__ row, int D, int l16, bool vec)
{
    float acc = 0.f;
    if (vec) {
        for (int d = l16 * 4; d < D; d += 64) {
            const f32x4 cv = *(const f32x4 *)(row + d);
            const float t0 = x[d] - cv.x, t1 = x[d + 1] - cv.y, t2 = x[d + 2] - cv.z, t3 = x[d + 3] - cv.w;
            acc = fmaf(t0, t0, acc);
            acc = fmaf(t1, t1, acc);
            acc = fmaf(t2, t2, acc);
            acc = fmaf(t3, t3, acc);
        }
    } else {
        for (int d = l16; d < D; d += 16) {
            const float t = x[d] - row[d];
            acc = fmaf(t, t, acc);
        }
    }
    return row16_sum(acc);
}

// Nearest row of C [k x D] to x by direct sums of squared differences, smallest (distance, index),
// over a set of `count` columns given by col_of(c), c = 0 .. count - 1 (columns >= k are skipped):
// 16 lanes per row, four rows per pass.  Serves the rows whose shortlist came back incomplete.
template <typename ColOf>
__device__ __forceinline__ uint64_t exact_nearest_of(const float *x, const float *__restrict__ C, int k, int D, int lane,
                                                     int count, ColOf col_of)
{
    const int sub = lane >> 4, l16 = lane & 15;
    const bool vec = (D % 4 == 0) && (((uintptr_t)C) % 16 == 0);
    uint64_t best = KEY_MAX;
    for (int c0 = 0; c0 < count; c0 += 4) {
        const int c = c0 + sub;
        const int i = c < count ? col_of(c) : k;
        const float acc = sqdist16(x, C + (int64_t)min(i, k - 1) * D, D, l16, vec);
        if (i < k) {
            const uint64_t key = make_key(acc, (uint32_t)i);
            best = key < best ? key : best;
        }
    }
    return wave_min_u64(best);
}

// The marker keys of a vector's shortlist (see VLQ_NN_MARK): every marked lane slot is searched
// exactly, a VLQ_NN_ALL marker asks for all columns.  cd [nc] are the keys of all splits, uniform
// over the wave.  Returns the best key found (KEY_MAX if there was no marker).
__device__ __forceinline__ uint64_t resolve_markers(const uint64_t *__restrict__ cd, int nc, int nsplit, const float *x,
                                                    const float *__restrict__ C, int k, int D, int lane)
{
    uint64_t best = KEY_MAX;
    const int ntiles = (k + VLQ_NN_TILE - 1) / VLQ_NN_TILE;
    const int per = (ntiles + nsplit - 1) / nsplit;
    for (int c0 = 0; c0 < nc; c0 += 64) {
        const uint64_t key = c0 + lane < nc ? cd[c0 + lane] : KEY_MAX;
        uint64_t mask = __ballot((uint32_t)(key >> 32) == VLQ_NN_MARK);
        while (mask) {
            const int src = __ffsll((unsigned long long)mask) - 1;
            mask &= mask - 1;
            const uint32_t slot = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)key, src);
            uint64_t got;
            if (slot == VLQ_NN_ALL) {
                got = exact_nearest_of(x, C, k, D, lane, k, [](int c) { return c; });
                mask = 0;
                c0 = nc; // nothing can add to a ranking over all columns
            } else {
                const int split = (c0 + src) / VLQ_NN_CANDS;
                const int t0 = split * per, t1 = min(ntiles, t0 + per);
                const int base = (int)(slot >> 5) * 64 + (int)(slot & 31);
                got = exact_nearest_of(x, C, k, D, lane, 2 * (t1 - t0),
                                       [=](int c) { return (t0 + (c >> 1)) * VLQ_NN_TILE + base + 32 * (c & 1); });
            }
            best = got < best ? got : best;
        }
    }
    return best;
}

// The byte of lambda and the residual for the chosen line (Eq. 12-13), in fp64 so that both are
// known to the rounding of their own size: lambda is taken as the projection
// <x - c_i, s_ij - c_i> / ||s_ij - c_i||^2, which is Eq. 8 with a, b and c written out (the same
// value without the cancellation of a + c - b), and the residual as (x - c_i) - l (s_ij - c_i) with
// l the grid value of the byte.  x (LDS, one wave's vector) is overwritten with the residual.
__device__ __forceinline__ float line_byte_and_residual(float *x, const float *__restrict__ ci,
                                                        const float *__restrict__ sj, int D, int lane,
                                                        double step, float zero, float *__restrict__ res_out)
{
    double g = 0.0, cc = 0.0;
    for (int d = lane; d < D; d += 64) {
        const double c = (double)ci[d], e = (double)sj[d] - c, z = (double)x[d] - c;
        g = fma(z, e, g);
        cc = fma(e, e, cc);
    }
    g = wave_sum_f64(g);
    cc = wave_sum_f64(cc);
    const double lam = cc > 0.0 ? g / cc : 0.0;
    double qd = rint(lam / step) + (double)zero;
    qd = fmin(fmax(qd, 0.0), 255.0);
    const double lh = (qd - (double)zero) * step;
    for (int d = lane; d < D; d += 64) {
        const double c = (double)ci[d];
        const float r = (float)(((double)x[d] - c) - lh * ((double)sj[d] - c));
        x[d] = r;
        if (res_out) res_out[d] = r;
    }
    return (float)qd;
}

// One workgroup encodes PB consecutive vectors.
//  phase 1 (a wave per vector): the candidates within the rounding band of the
//    smallest GEMM-form distance are re-evaluated as direct sums of squared
//    differences; the smallest (distance, index) is the cell (Eq. 2).  Then the
//    n lines of the cell: g_j = <x - c_i, s_ij - c_i>, lambda_j = g_j / c_j (Eq. 13), squared line
//    distance a - c lambda^2 (= Eq. 7 at that lambda); smallest (distance, j) is the edge.
//    lambda -> byte -> grid value; residual to the anchor of that grid value (Eq. 12).
//  phase 2 (thread = codeword): for every sub-space the nearest codeword by direct
//    squared distance, ties to the smaller codeword (Alg. 2).
template <int DS>
__global__ __launch_bounds__(ENC_NT) void k_encode_finish(EncodeArgs a, int PB)
{
    extern __shared__ unsigned char smem[];
    unsigned long long *best = (unsigned long long *)smem; // [PB][m]
    float *res = (float *)(best + PB * a.m);               // [PB][D]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int D = a.D, m = a.m, n = a.n;
    const int ds = DS > 0 ? DS : D / m;
    const int64_t g0 = (int64_t)blockIdx.x * PB;
    const int np = (int)min((int64_t)PB, a.nb - g0);

    for (int i = tid; i < PB * m; i += ENC_NT) best[i] = KEY_MAX;
    const bool vec16 = (D % 4 == 0) && (((uintptr_t)a.C) % 16 == 0);

    for (int pt = wave; pt < np; pt += ENC_NT / 64) {
        const int64_t gid = g0 + pt;
        float *x = res + pt * D;
        float xn = 0.f; // of the vector as the product saw it (centred when mu is given)
        for (int d = lane; d < D; d += 64) {
            const float v = a.X[gid * D + d];
            x[d] = v;
            const float vc = a.mu ? v - a.mu[d] : v;
            xn = fmaf(vc, vc, xn);
        }
        xn = wave_sum(xn);
        // candidates of all column splits
        const int nc = a.nsplit * VLQ_NN_CANDS;
        const uint64_t *cd = a.cand + gid * nc;
        uint64_t mn = KEY_MAX;
        bool marked = false;
        for (int c = lane; c < nc; c += 64) {
            const uint64_t key = cd[c];
            if ((uint32_t)(key >> 32) == VLQ_NN_MARK)
                marked = true;
            else
                mn = key < mn ? key : mn;
        }
        // incomplete shortlists first: the marked slots (or all columns) exactly
        uint64_t bk = __ballot(marked) ? resolve_markers(cd, nc, a.nsplit, x, a.C, a.k, D, lane) : KEY_MAX;
        mn = wave_min_u64(mn);
        if (mn != KEY_MAX) {
            const float dmin = __uint_as_float((uint32_t)(mn >> 32));
            const float band = dmin + a.band_dist * (xn + dmin) + a.band_norm * (3.f * xn + 2.f * dmin);
            for (int c = 0; c < nc; ++c) {
                const uint64_t key = cd[c]; // same address in all lanes
                if (key == KEY_MAX || (uint32_t)(key >> 32) == VLQ_NN_MARK || __uint_as_float((uint32_t)(key >> 32)) > band)
                    continue;
                const uint32_t idx = (uint32_t)key;
                const float d = sqdist16(x, a.C + (int64_t)idx * D, D, lane & 15, vec16);
                const uint64_t ek = make_key(d, idx);
                bk = ek < bk ? ek : bk;
            }
        }
        if (bk == KEY_MAX) { // only with non-finite input: keep indices in range
            const uint32_t idx = mn == KEY_MAX ? 0u : (uint32_t)mn;
            bk = make_key(sqdist16(x, a.C + (int64_t)idx * D, D, lane & 15, vec16), idx);
        }
        const int cell = (int)(uint32_t)bk;
        const float av = ord2f((uint32_t)(bk >> 32));
        if (!a.S) { // nearest centroid only (Lloyd iterations)
            if (lane == 0) a.cell[gid] = cell;
            continue;
        }
        // line quantisation inside the cell: Eq. 8's numerator (a + c - b) / 2 as the inner product
        // g = <x - c_i, s_ij - c_i> (no cancellation), squared line distance a - g^2 / c
        int bj = 0;
        float bd2 = INFINITY;
        const float *cc = a.C + (int64_t)cell * D;
        for (int j = 0; j < n; ++j) {
            const float *sr = a.C + (int64_t)a.S[(int64_t)cell * n + j] * D;
            float g = 0.f;
            for (int d = lane; d < D; d += 64) g = fmaf(x[d] - cc[d], sr[d] - cc[d], g);
            g = wave_sum(g);
            const float c = a.E[(int64_t)cell * n + j];
            const float lam = c > 0.f ? g / c : 0.f;
            const float d2 = av - g * lam;
            if (d2 < bd2) {
                bd2 = d2;
                bj = j;
            }
        }
        const float qf = line_byte_and_residual(x, a.C + (int64_t)cell * D, a.C + (int64_t)a.S[(int64_t)cell * n + bj] * D,
                                                D, lane, a.lam_step_d, a.lam_zero, a.res ? a.res + gid * D : nullptr);
        if (lane == 0) {
            if (a.cell) a.cell[gid] = cell;
            if (a.edge) a.edge[gid] = bj;
            if (a.lamq) a.lamq[gid] = (uint8_t)qf;
        }
    }
    __syncthreads();
    if (!a.codes) return;

    // phase 2: thread tid is codeword tid
    for (int p = 0; p < m; ++p) {
        const float *w = a.P + ((int64_t)p * 256 + tid) * ds;
        float wr[DS > 0 ? DS : 1];
        if (DS > 0) {
#pragma unroll
            for (int d = 0; d < DS; ++d) wr[d] = w[d];
        }
        for (int pt = 0; pt < np; ++pt) {
            const float *r = res + pt * D + p * ds;
            float s = 0.f;
            if (DS > 0) {
#pragma unroll
                for (int d = 0; d < DS; ++d) {
                    const float t = r[d] - wr[d];
                    s = fmaf(t, t, s);
                }
            } else {
                for (int d = 0; d < ds; ++d) {
                    const float t = r[d] - w[d];
                    s = fmaf(t, t, s);
                }
            }
            uint64_t key = wave_min_u64(make_key(s, (uint32_t)tid));
            if (lane == 0) atomicMin(&best[pt * m + p], (unsigned long long)key);
        }
    }
    __syncthreads();
    for (int i = tid; i < np * m; i += ENC_NT) a.codes[g0 * m + i] = (uint8_t)(best[i] & 0xFFu);
}


// ---------------------------------------------------------------------------
// The same two phases arranged for the common shapes (D <= 128 and a multiple
// of four, sub-spaces of up to 16 dimensions), 64 vectors per workgroup.
//  phase 1 (a wave per vector, as above) forms the n line distances four rows at
//    a time: 16 lanes per neighbour row, each lane eight components, so a pass
//    costs one short reduction instead of four wave-wide ones.
//  phase 2 turns the work round: a lane is a vector, a wave takes whole
//    sub-spaces, and the 256 codewords come in one after the other through uniform
//    loads.  Every lane keeps its own running (distance, codeword) minimum, so the
//    step has no cross-lane reduction at all; strict "<" in ascending codeword
//    order keeps the smaller codeword of a tie (Alg. 2).
// ---------------------------------------------------------------------------
#define ENC2_PB 64
typedef const float __attribute__((address_space(4))) cfloat;

template <int DS>
__global__ __launch_bounds__(ENC_NT) void k_encode_finish_lanes(EncodeArgs a)
{
    extern __shared__ unsigned char smem[];
    const int D = a.D, m = a.m, n = a.n;
    const int RS = D + 1; // odd row stride: lane = vector reads are conflict-free
    float *res = (float *)smem;                        // [ENC2_PB][RS]
    uint8_t *cod = (uint8_t *)(res + ENC2_PB * RS);    // [ENC2_PB][m]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int sub = lane >> 4, l16 = lane & 15;
    const int64_t g0 = (int64_t)blockIdx.x * ENC2_PB;
    const int np = (int)min((int64_t)ENC2_PB, a.nb - g0);
    const int d0 = l16 * 4, d1 = 64 + l16 * 4;
    const bool has0 = d0 < D, has1 = d1 < D;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    const bool vec16 = true; // this kernel serves D % 4 == 0 with aligned centroids only

    for (int pt = wave; pt < np; pt += ENC_NT / 64) {
        const int64_t gid = g0 + pt;
        float *x = res + pt * RS;
        float xn = 0.f; // of the vector as the product saw it (centred when mu is given)
        for (int d = lane; d < D; d += 64) {
            const float v = a.X[gid * D + d];
            x[d] = v;
            const float vc = a.mu ? v - a.mu[d] : v;
            xn = fmaf(vc, vc, xn);
        }
        xn = wave_sum(xn);
        const int nc = a.nsplit * VLQ_NN_CANDS;
        const uint64_t *cd = a.cand + gid * nc;
        uint64_t mn = KEY_MAX;
        bool marked = false;
        for (int c = lane; c < nc; c += 64) {
            const uint64_t key = cd[c];
            if ((uint32_t)(key >> 32) == VLQ_NN_MARK)
                marked = true;
            else
                mn = key < mn ? key : mn;
        }
        // incomplete shortlists first: the marked slots (or all columns) exactly
        uint64_t bk = __ballot(marked) ? resolve_markers(cd, nc, a.nsplit, x, a.C, a.k, D, lane) : KEY_MAX;
        mn = wave_min_u64(mn);
        if (mn != KEY_MAX) {
            const float dmin = __uint_as_float((uint32_t)(mn >> 32));
            const float band = dmin + a.band_dist * (xn + dmin) + a.band_norm * (3.f * xn + 2.f * dmin);
            for (int c0 = 0; c0 < nc; c0 += 64) { // the few candidates inside the band, found 64 keys at a time
                const uint64_t key = c0 + lane < nc ? cd[c0 + lane] : KEY_MAX;
                const bool inb = key != KEY_MAX && (uint32_t)(key >> 32) != VLQ_NN_MARK &&
                                 !(__uint_as_float((uint32_t)(key >> 32)) > band);
                uint64_t mask = __ballot(inb);
                while (mask) {
                    const int src = __ffsll((unsigned long long)mask) - 1;
                    mask &= mask - 1;
                    const uint32_t idx = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)key, src);
                    const float d = sqdist16(x, a.C + (int64_t)idx * D, D, lane & 15, vec16);
                    const uint64_t ek = make_key(d, idx);
                    bk = ek < bk ? ek : bk;
                }
            }
        }
        if (bk == KEY_MAX) { // only with non-finite input: keep indices in range
            const uint32_t idx = mn == KEY_MAX ? 0u : (uint32_t)mn;
            bk = make_key(sqdist16(x, a.C + (int64_t)idx * D, D, lane & 15, vec16), idx);
        }
        const int cell = (int)(uint32_t)bk;
        const float av = ord2f((uint32_t)(bk >> 32));
        // line quantisation inside the cell, four neighbour rows per pass
        // (Eq. 8's numerator (a + c - b) / 2 as the inner product g = <x - c_i, s_ij - c_i>: no
        // cancellation; squared line distance a - g^2 / c)
        const float *xg = a.X + gid * D;
        const float *cg = a.C + (int64_t)cell * D;
        f32x4 y0 = zero, y1 = zero, ci0 = zero, ci1 = zero; // y = x - c_i
        if (has0) {
            ci0 = *(const f32x4 *)(cg + d0);
            y0 = *(const f32x4 *)(xg + d0) - ci0;
        }
        if (has1) {
            ci1 = *(const f32x4 *)(cg + d1);
            y1 = *(const f32x4 *)(xg + d1) - ci1;
        }
        float bd2 = INFINITY;
        int bj = 0x7FFFFFFF;
        for (int j0 = 0; j0 < n; j0 += 16) { // 16 rows per round: their loads are all under way together
            int sidx[4];
            float ev[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = j0 + 4 * u + sub;
                const bool live = j < n;
                sidx[u] = live ? a.S[(int64_t)cell * n + j] : cell;
                ev[u] = live ? a.E[(int64_t)cell * n + j] : 0.f;
            }
            f32x4 c0[4], c1[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float *row = a.C + (int64_t)sidx[u] * D;
                c0[u] = has0 ? *(const f32x4 *)(row + d0) : zero;
                c1[u] = has1 ? *(const f32x4 *)(row + d1) : zero;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = j0 + 4 * u + sub;
                float acc = 0.f;
                {
                    const f32x4 e0 = c0[u] - ci0;
                    acc = fmaf(y0.x, e0.x, acc);
                    acc = fmaf(y0.y, e0.y, acc);
                    acc = fmaf(y0.z, e0.z, acc);
                    acc = fmaf(y0.w, e0.w, acc);
                }
                {
                    const f32x4 e1 = c1[u] - ci1;
                    acc = fmaf(y1.x, e1.x, acc);
                    acc = fmaf(y1.y, e1.y, acc);
                    acc = fmaf(y1.z, e1.z, acc);
                    acc = fmaf(y1.w, e1.w, acc);
                }
                acc = row16_sum(acc);
                if (j < n) {
                    const float c = ev[u];
                    const float lam = c > 0.f ? acc / c : 0.f;
                    const float d2 = av - acc * lam;
                    if (d2 < bd2) { // rows of a lane group come in ascending j
                        bd2 = d2;
                        bj = j;
                    }
                }
            }
        }
        // the four lane groups hold the best of their rows: smallest (distance, j) overall
#pragma unroll
        for (int o = 16; o <= 32; o <<= 1) {
            const float od = __shfl_xor(bd2, o, 64);
            const int oj = __shfl_xor(bj, o, 64);
            if (od < bd2 || (od == bd2 && oj < bj)) {
                bd2 = od;
                bj = oj;
            }
        }
        if (bj == 0x7FFFFFFF) bj = 0; // every line distance was NaN (non-finite input): keep the index in range
        const float qf = line_byte_and_residual(x, a.C + (int64_t)cell * D, a.C + (int64_t)a.S[(int64_t)cell * n + bj] * D,
                                                D, lane, a.lam_step_d, a.lam_zero, a.res ? a.res + gid * D : nullptr);
        if (lane == 0) {
            if (a.cell) a.cell[gid] = cell;
            if (a.edge) a.edge[gid] = bj;
            if (a.lamq) a.lamq[gid] = (uint8_t)qf;
        }
    }
    __syncthreads();

    // phase 2: lane = vector, wave = sub-space, codewords in ascending order
    for (int p = wave; p < m; p += ENC_NT / 64) {
        float r[DS];
#pragma unroll
        for (int d = 0; d < DS; ++d) r[d] = res[lane * RS + p * DS + d];
        // the codebooks are never written while the kernel runs: reading them through the constant
        // address space lets the uniform loads take the scalar path and the operands stay in SGPRs
        const cfloat *w = (const cfloat *)(uintptr_t)(a.P + (int64_t)p * 256 * DS);
        float best = INFINITY;
        int bt = 0;
        // CB codewords per batch (other waves of the SIMD cover the latency of the uniform loads:
        // issuing a batch a whole round ahead measured no faster)
        constexpr int CB = DS >= 12 ? 2 : (DS >= 6 ? 4 : 8);
        float wc[CB * DS], wn[CB * DS];
#pragma unroll
        for (int i = 0; i < CB * DS; ++i) wc[i] = w[i];
        for (int t = 0; t < 256; t += CB) {
            const int tn = t + CB < 256 ? t + CB : t;
#pragma unroll
            for (int i = 0; i < CB * DS; ++i) wn[i] = w[tn * DS + i];
#pragma unroll
            for (int u = 0; u < CB; ++u) {
                float s = 0.f;
#pragma unroll
                for (int d = 0; d < DS; ++d) {
                    const float tv = r[d] - wc[u * DS + d];
                    s = fmaf(tv, tv, s);
                }
                if (s < best) {
                    best = s;
                    bt = t + u;
                }
            }
#pragma unroll
            for (int i = 0; i < CB * DS; ++i) wc[i] = wn[i];
        }
        cod[lane * m + p] = (uint8_t)bt;
    }
    __syncthreads();
    for (int i = tid; i < np * m; i += ENC_NT) a.codes[g0 * m + i] = cod[i];
}

static bool encode_lanes_supported(const EncodeArgs &a)
{
    if (!a.S || !a.codes) return false;
    if (a.D > 128 || a.D % 4) return false;
    if ((((uintptr_t)a.X) | ((uintptr_t)a.C)) % 16) return false;
    const int ds = a.D / a.m;
    return ds == 4 || ds == 6 || ds == 8 || ds == 12 || ds == 16;
}

void launch_encode_finish(const EncodeArgs &a, hipStream_t st)
{
    if (a.nb <= 0) return;
    if (!a.wave_per_vector && encode_lanes_supported(a)) {
        const size_t smem2 = (size_t)ENC2_PB * (a.D + 1) * 4 + (size_t)ENC2_PB * a.m;
        const unsigned grid2 = (unsigned)((a.nb + ENC2_PB - 1) / ENC2_PB);
#define ENC2_LAUNCH(DSV)                                                                                       \
    hipLaunchKernelGGL(k_encode_finish_lanes<DSV>, dim3(grid2), dim3(ENC_NT), smem2, st, a)
        switch (a.D / a.m) {
        case 4: ENC2_LAUNCH(4); break;
        case 6: ENC2_LAUNCH(6); break;
        case 8: ENC2_LAUNCH(8); break;
        case 12: ENC2_LAUNCH(12); break;
        default: ENC2_LAUNCH(16); break;
        }
#undef ENC2_LAUNCH
        return;
    }
    int PB = (int)(65536 / ((size_t)a.D * 4));
    if (PB > ENC_PB_MAX) PB = ENC_PB_MAX;
    if (PB < 1) PB = 1;
    const size_t smem = (size_t)PB * a.D * 4 + (size_t)PB * a.m * 8;
    const unsigned grid = (unsigned)((a.nb + PB - 1) / PB);
    const int ds = a.D / a.m;
#define ENC_LAUNCH(DSV)                                                                                        \
    do {                                                                                                       \
        (void)hipFuncSetAttribute((const void *)k_encode_finish<DSV>, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                  (int)smem);                                                                  \
        hipLaunchKernelGGL(k_encode_finish<DSV>, dim3(grid), dim3(ENC_NT), smem, st, a, PB);                    \
    } while (0)
    switch (ds) {
    case 2: ENC_LAUNCH(2); break;
    case 4: ENC_LAUNCH(4); break;
    case 6: ENC_LAUNCH(6); break;
    case 8: ENC_LAUNCH(8); break;
    case 16: ENC_LAUNCH(16); break;
    default: ENC_LAUNCH(0); break;
    }
#undef ENC_LAUNCH
}
