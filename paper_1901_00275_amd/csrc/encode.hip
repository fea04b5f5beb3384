// Encoding on the GPU (Alg. 1 + Alg. 2): the second half, after the
// nearest-centroid candidates have come out of the matrix-core contraction.
#include "common.h"

#define ENC_NT 256
#define ENC_PB_MAX 32

// One workgroup encodes PB consecutive vectors.
//  phase 1 (a wave per vector): the candidates within the rounding band of the
//    smallest GEMM-form distance are re-evaluated as direct sums of squared
//    differences; the smallest (distance, index) is the cell (Eq. 2).  Then the
//    n lines of the cell: b_j direct, lambda_j by Eq. 13, squared line distance
//    a - c lambda^2 (= Eq. 7 at that lambda); smallest (distance, j) is the edge.
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

    for (int pt = wave; pt < np; pt += ENC_NT / 64) {
        const int64_t gid = g0 + pt;
        float *x = res + pt * D;
        float xn = 0.f;
        for (int d = lane; d < D; d += 64) {
            const float v = a.X[gid * D + d];
            x[d] = v;
            xn = fmaf(v, v, xn);
        }
        xn = wave_sum(xn);
        // candidates of all column splits
        const int nc = a.nsplit * VLQ_NN_CANDS;
        const uint64_t *cd = a.cand + gid * nc;
        uint64_t mn = KEY_MAX;
        for (int c = lane; c < nc; c += 64) {
            const uint64_t key = cd[c];
            mn = key < mn ? key : mn;
        }
        mn = wave_min_u64(mn);
        const float dmin = __uint_as_float((uint32_t)(mn >> 32));
        const float band = dmin + a.band_dist * (xn + dmin) + a.band_norm * (3.f * xn + 2.f * dmin);
        uint64_t bk = KEY_MAX;
        for (int c = 0; c < nc; ++c) {
            const uint64_t key = cd[c]; // same address in all lanes
            if (key == KEY_MAX || __uint_as_float((uint32_t)(key >> 32)) > band) continue;
            const uint32_t idx = (uint32_t)key;
            const float d = wave_sqdist(x, a.C + (int64_t)idx * D, D, lane);
            const uint64_t ek = make_key(d, idx);
            bk = ek < bk ? ek : bk;
        }
        if (bk == KEY_MAX) { // only with non-finite input: keep indices in range
            const uint32_t idx = mn == KEY_MAX ? 0u : (uint32_t)mn;
            bk = make_key(wave_sqdist(x, a.C + (int64_t)idx * D, D, lane), idx);
        }
        const int cell = (int)(uint32_t)bk;
        const float av = ord2f((uint32_t)(bk >> 32));
        if (!a.S) { // nearest centroid only (Lloyd iterations)
            if (lane == 0) a.cell[gid] = cell;
            continue;
        }
        // line quantisation inside the cell
        int bj = 0;
        float bl = 0.f, bd2 = INFINITY;
        for (int j = 0; j < n; ++j) {
            const int s = a.S[(int64_t)cell * n + j];
            const float b = wave_sqdist(x, a.C + (int64_t)s * D, D, lane);
            const float c = a.E[(int64_t)cell * n + j];
            const float lam = c > 0.f ? 0.5f * (av + c - b) / c : 0.f;
            const float d2 = av - c * lam * lam;
            if (d2 < bd2) {
                bd2 = d2;
                bj = j;
                bl = lam;
            }
        }
        float qf = rintf(bl / a.lam_step) + a.lam_zero;
        qf = fminf(fmaxf(qf, 0.f), 255.f);
        const float lh = (qf - a.lam_zero) * a.lam_step;
        const float *ci = a.C + (int64_t)cell * D;
        const float *sj = a.C + (int64_t)a.S[(int64_t)cell * n + bj] * D;
        for (int d = lane; d < D; d += 64) {
            const float c = ci[d];
            const float r = x[d] - fmaf(lh, sj[d] - c, c);
            x[d] = r;
            if (a.res) a.res[gid * D + d] = r;
        }
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

void launch_encode_finish(const EncodeArgs &a, hipStream_t st)
{
    if (a.nb <= 0) return;
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
