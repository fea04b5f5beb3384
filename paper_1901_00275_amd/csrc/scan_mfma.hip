// Fast path of the list scan (Sec. 3.3.2 - 3.3.3) for 8-byte codes:
// lookup tables built on the matrix cores, points prefetched under the
// table build, K-selection per wavefront without workgroup barriers.
//
// Same arithmetic as the generic kernel in search.hip:
//   dist = sum_p A[p][t_p] + l (2 sum_p B[p][t_p] - 2 g) + l^2 c
//   A[p][t] = ||z^p - P[p][t]||^2 = ||z^p||^2 - 2 <z^p, P[p][t]> + ||P[p][t]||^2,  z = y - c_i
//   B[p][t] = <e^p, P[p][t]>,  e = s_ij - c_i
// so every table entry is an inner product of a codeword with a sub-vector of
// z or e: a [256 m x D/m] by [D/m x 1] product per vector.
//
// Layout of the work
//  * one workgroup (512 threads, 8 waves) per (query, split); two workgroups
//    fit a compute unit, so one can build tables on the matrix pipe while the
//    other gathers from LDS;
//  * the PQ codebooks stay in registers for the whole workgroup: wave w owns
//    sub-spaces w*M/8 .. and, per sub-space, lane l holds codewords l, 64+l,
//    128+l, 192+l as A operands of v_mfma_f32_4x4x1_16b_f32 (16 blocks of
//    4 codewords x 4 vectors per instruction);
//  * a batch = one probed cell and up to 3 of its visited sub-regions: the 4
//    vector columns of the instruction are z, e_1, e_2, e_3.  Column 0 yields A,
//    which the other three lanes of each quad fetch with a DPP quad broadcast
//    and store interleaved with their B as float2 (one 64-bit LDS gather per
//    lookup); ||P||^2 enters through one extra contraction step (codeword
//    coordinate -||P||^2 / 2 against 1 for column 0, 0 elsewhere);
//  * codes and lambda bytes of the batch's lists are loaded into registers
//    before the table build and consumed after it; ids are loaded only for
//    points that beat the current threshold;
//  * every wave keeps its own sorted K-best list and candidate buffer in LDS
//    and merges them alone; the waves share only a monotonically decreasing
//    threshold.  The eight lists are merged once at the end.
#include "common.h"

#define S2_NT 512
#define S2_NW 8
#define S2_U 4
#define S2_WIN 512
#define S2_KP 128
#define S2_WSZ 256
#define S2_SUBS 3

__device__ __forceinline__ float quad_bcast0(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x00, 0xf, 0xf, false));
}

// wave-private bitonic sort of S2_WSZ keys in LDS (one wave: LDS operations of a
// wave complete in issue order, so no workgroup barrier is needed)
__device__ __forceinline__ void wave_sort256(volatile uint64_t *wk, int lane)
{
    for (int k = 2; k <= S2_WSZ; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
#pragma unroll
            for (int h = 0; h < S2_WSZ / 128; ++h) {
                const int i = lane + 64 * h;
                const int l = ((i & ~(j - 1)) << 1) | (i & (j - 1));
                const int r = l | j;
                const uint64_t x = wk[l], y = wk[r];
                if ((x > y) == ((l & k) == 0)) {
                    wk[l] = y;
                    wk[r] = x;
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
}

__device__ __forceinline__ void wave_merge(volatile uint64_t *wk, int &cnt, int K, int lane,
                                           unsigned long long *sh_thr)
{
    for (int i = S2_KP + cnt + lane; i < S2_WSZ; i += 64) wk[i] = KEY_MAX;
    __builtin_amdgcn_wave_barrier();
    wave_sort256(wk, lane);
    for (int i = K + lane; i < S2_KP; i += 64) wk[i] = KEY_MAX;
    __builtin_amdgcn_wave_barrier();
    cnt = 0;
    const uint64_t t = wk[K - 1];
    if (lane == 0 && t != KEY_MAX) atomicMin(sh_thr, (unsigned long long)t);
    __builtin_amdgcn_wave_barrier();
}

template <int M, int DS>
__global__ __launch_bounds__(S2_NT, 4) void k_scan_mfma(ScanArgs a)
{
    constexpr int D = M * DS;
    constexpr int TAB = M * 256;
    constexpr int NPW = M / S2_NW; // sub-spaces per wave
    constexpr int VLD = D + 4;     // row stride of the vector buffer (rows land in different banks)
    static_assert(M % S2_NW == 0, "M must be a multiple of 8");

    extern __shared__ unsigned char smem[];
    uint64_t *keys = (uint64_t *)smem;                         // [NW][WSZ]
    float2 *AB = (float2 *)(keys + S2_NW * S2_WSZ);            // [SUBS][TAB]
    float *vec = (float *)(AB + S2_SUBS * TAB);                // [4][VLD]
    float *yv = vec + 4 * VLD;                                 // [D]
    int32_t *s_label = (int32_t *)(yv + D);                    // [WIN]
    uint32_t *s_beg = (uint32_t *)(s_label + S2_WIN);          // [WIN]
    int32_t *s_len = (int32_t *)(s_beg + S2_WIN);              // [WIN]
    float *s_g = (float *)(s_len + S2_WIN);                    // [WIN]
    int32_t *s_nbr = (int32_t *)(s_g + S2_WIN);                // [WIN]
    uint32_t *s_batch = (uint32_t *)(s_nbr + S2_WIN);          // [WIN] 3 x 9-bit positions + 2-bit count
    __shared__ unsigned long long sh_thr;
    __shared__ int sh_nbatch;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = blockIdx.x / a.nsplit, split = blockIdx.x - q * a.nsplit;
    const int R0 = (int)((int64_t)a.w2 * split / a.nsplit), R1 = (int)((int64_t)a.w2 * (split + 1) / a.nsplit);
    const int K = a.K, n = a.n;
    volatile uint64_t *wk = keys + wave * S2_WSZ;
    int wcnt = 0;

    // ---- per-workgroup set-up: codebooks into registers ----
    float Preg[NPW][4][DS], Paug[NPW][4];
#pragma unroll
    for (int pp = 0; pp < NPW; ++pp)
#pragma unroll
        for (int tb = 0; tb < 4; ++tb) {
            const float *w = a.P + ((int64_t)(wave * NPW + pp) * 256 + tb * 64 + lane) * DS;
            float s = 0.f;
#pragma unroll
            for (int d = 0; d < DS; ++d) {
                Preg[pp][tb][d] = w[d];
                s = fmaf(w[d], w[d], s);
            }
            Paug[pp][tb] = -0.5f * s;
        }
    for (int d = tid; d < D; d += S2_NT) yv[d] = a.Q[(int64_t)q * D + d];
    for (int i = lane; i < S2_WSZ; i += 64) wk[i] = KEY_MAX;
    if (tid == 0) sh_thr = KEY_MAX;

    const int j = lane & 3, blk = lane >> 2;

    for (int ws = R0; ws < R1; ws += S2_WIN) {
        const int nwin = min(S2_WIN, R1 - ws);
        __syncthreads(); // previous window done with the s_* arrays
        for (int r = tid; r < nwin; r += S2_NT) {
            const int label = a.scan_label[(int64_t)q * a.w2 + ws + r];
            s_label[r] = label;
            int len = 0;
            uint32_t beg = 0;
            int nbr = 0;
            float g = 0.f;
            if (label >= 0) {
                const int64_t b0 = a.off[label], b1 = a.off[label + 1];
                beg = (uint32_t)b0;
                len = (int)(b1 - b0);
                nbr = a.S[label];
                g = a.scan_g[(int64_t)q * a.w2 + ws + r];
            }
            s_beg[r] = beg;
            s_len[r] = len;
            s_nbr[r] = nbr;
            s_g[r] = g;
        }
        __syncthreads();
        if (tid == 0) {
            // batches: runs of up to 3 non-empty sub-regions of one cell (labels are sorted)
            int nb = 0, r = 0;
            while (r < nwin) {
                if (s_len[r] <= 0) {
                    ++r;
                    continue;
                }
                const int cell = s_label[r] / n;
                uint32_t desc = 0;
                int cnt = 0;
                while (r < nwin && cnt < S2_SUBS) {
                    if (s_len[r] <= 0) {
                        ++r;
                        continue;
                    }
                    if (s_label[r] / n != cell) break;
                    desc |= (uint32_t)r << (9 * cnt);
                    ++cnt;
                    ++r;
                }
                s_batch[nb++] = desc | ((uint32_t)cnt << 27);
            }
            sh_nbatch = nb;
        }
        __syncthreads();
        const int nbatch = sh_nbatch;

        // vector element owned by this thread in the [4][D] vector block (row, dim)
        const int vrow = tid / D, vdim = tid - vrow * D; // D <= 128: one element per thread when 4 D <= 512
        auto load_vec_elem = [&](int b) -> float {
            if (b >= nbatch || vrow >= 4) return 0.f;
            const uint32_t desc = s_batch[b];
            const int cnt = (int)(desc >> 27);
            const int r0 = (int)(desc & 511u);
            const int cell = s_label[r0] / n;
            const float c = a.C[(int64_t)cell * D + vdim];
            if (vrow == 0) return yv[vdim] - c;
            if (vrow - 1 >= cnt) return 0.f;
            const int rr = (int)((desc >> (9 * (vrow - 1))) & 511u);
            return a.C[(int64_t)s_nbr[rr] * D + vdim] - c;
        };
        if (vrow < 4) vec[vrow * VLD + vdim] = load_vec_elem(0);
        __syncthreads();

        for (int b = 0; b < nbatch; ++b) {
            // ---- header ----
            const uint32_t desc = s_batch[b];
            const int cnt = (int)(desc >> 27);
            int rr[S2_SUBS], len[S2_SUBS];
            uint32_t beg[S2_SUBS];
            float gg[S2_SUBS], cc[S2_SUBS];
#pragma unroll
            for (int s = 0; s < S2_SUBS; ++s) {
                rr[s] = (int)((desc >> (9 * s)) & 511u);
                const bool ok = s < cnt;
                len[s] = ok ? s_len[rr[s]] : 0;
                beg[s] = ok ? s_beg[rr[s]] : 0u;
                gg[s] = ok ? s_g[rr[s]] : 0.f;
                cc[s] = ok ? a.E[s_label[rr[s]]] : 0.f;
            }
            const int cum1 = len[0], cum2 = len[0] + len[1], Np = cum2 + len[2];

            // ---- prefetch the first NT*U points of the batch and the next batch's vectors ----
            uint32_t cw[S2_U][M / 4];
            uint32_t lb[S2_U];
#pragma unroll
            for (int u = 0; u < S2_U; ++u) {
                const int gi = tid + u * S2_NT;
                lb[u] = 0;
#pragma unroll
                for (int x = 0; x < M / 4; ++x) cw[u][x] = 0;
                if (gi < Np) {
                    const int li = (gi >= cum1) + (gi >= cum2);
                    const int64_t t = (int64_t)(li == 0 ? beg[0] : (li == 1 ? beg[1] : beg[2])) +
                                      (gi - (li == 0 ? 0 : (li == 1 ? cum1 : cum2)));
                    const uint32_t *cp = (const uint32_t *)(a.codes + t * M);
#pragma unroll
                    for (int x = 0; x < M / 4; ++x) cw[u][x] = cp[x];
                    lb[u] = a.lam[t];
                }
            }
            const float vnext = load_vec_elem(b + 1);

            // ---- tables on the matrix cores ----
#pragma unroll
            for (int pp = 0; pp < NPW; ++pp) {
                const int p = wave * NPW + pp;
                float v[DS];
                float zz = 0.f;
#pragma unroll
                for (int d = 0; d < DS; ++d) {
                    v[d] = vec[j * VLD + p * DS + d];
                    zz = fmaf(v[d], v[d], zz);
                }
                const float vaug = j == 0 ? 1.f : 0.f;
                f32x4 acc[4];
#pragma unroll
                for (int tb = 0; tb < 4; ++tb) acc[tb] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int d = 0; d < DS; ++d)
#pragma unroll
                    for (int tb = 0; tb < 4; ++tb)
                        acc[tb] = __builtin_amdgcn_mfma_f32_4x4x1f32(Preg[pp][tb][d], v[d], acc[tb], 0, 0, 0);
#pragma unroll
                for (int tb = 0; tb < 4; ++tb)
                    acc[tb] = __builtin_amdgcn_mfma_f32_4x4x1f32(Paug[pp][tb], vaug, acc[tb], 0, 0, 0);
#pragma unroll
                for (int tb = 0; tb < 4; ++tb) {
                    float A4[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) A4[i] = quad_bcast0(fmaf(-2.f, acc[tb][i], zz));
                    if (j >= 1 && j - 1 < cnt) {
                        f32x4 *dst = (f32x4 *)(AB + (j - 1) * TAB + p * 256 + tb * 64 + blk * 4);
                        dst[0] = (f32x4){A4[0], acc[tb][0], A4[1], acc[tb][1]};
                        dst[1] = (f32x4){A4[2], acc[tb][2], A4[3], acc[tb][3]};
                    }
                }
            }
            __syncthreads(); // tables complete; the vector block is free again
            if (vrow < 4) vec[vrow * VLD + vdim] = vnext;

            // ---- scan ----
            auto score = [&](const uint32_t (&cwv)[M / 4], uint32_t lbyte, int li, int64_t t) {
                const float2 *tab = AB + li * TAB;
                float sa = 0.f, sb = 0.f;
#pragma unroll
                for (int x = 0; x < M / 4; ++x)
#pragma unroll
                    for (int bb = 0; bb < 4; ++bb) {
                        const float2 ab = tab[(x * 4 + bb) * 256 + ((cwv[x] >> (8 * bb)) & 255u)];
                        sa += ab.x;
                        sb += ab.y;
                    }
                const float l = ((float)lbyte - a.lam_zero) * a.lam_step;
                const float g = li == 0 ? gg[0] : (li == 1 ? gg[1] : gg[2]);
                const float c = li == 0 ? cc[0] : (li == 1 ? cc[1] : cc[2]);
                const float dist = fmaf(l, fmaf(l, c, 2.f * (sb - g)), sa);
                // K-selection: the id is only needed for points that can still enter
                const uint64_t thr = sh_thr;
                const float thr_d = ord2f((uint32_t)(thr >> 32));
                bool pass = t >= 0 && !(dist > thr_d);
                if (__ballot(pass)) {
                    uint64_t key = KEY_MAX;
                    if (pass) {
                        key = make_key(dist, (uint32_t)a.ids[t]);
                        pass = key < thr;
                    }
                    uint64_t mask = __ballot(pass);
                    int np = __popcll(mask);
                    if (np) {
                        if (wcnt + np > S2_WSZ - S2_KP) {
                            wave_merge(wk, wcnt, K, lane, &sh_thr);
                            pass = pass && key < sh_thr;
                            mask = __ballot(pass);
                            np = __popcll(mask);
                        }
                        if (pass) wk[S2_KP + wcnt + __popcll(mask & ((1ull << lane) - 1ull))] = key;
                        wcnt += np;
                    }
                }
            };
#pragma unroll
            for (int u = 0; u < S2_U; ++u) {
                const int gi = tid + u * S2_NT;
                if (u * S2_NT >= Np) break; // uniform
                const int li = (gi >= cum1) + (gi >= cum2);
                const int64_t t = gi < Np ? (int64_t)(li == 0 ? beg[0] : (li == 1 ? beg[1] : beg[2])) +
                                                (gi - (li == 0 ? 0 : (li == 1 ? cum1 : cum2)))
                                          : -1;
                score(cw[u], lb[u], li > 2 ? 2 : li, t);
            }
            for (int base = S2_U * S2_NT; base < Np; base += S2_NT) { // lists longer than the prefetch window
                const int gi = base + tid;
                const int li = (gi >= cum1) + (gi >= cum2);
                int64_t t = -1;
                uint32_t c2[M / 4];
                uint32_t l2 = 0;
#pragma unroll
                for (int x = 0; x < M / 4; ++x) c2[x] = 0;
                if (gi < Np) {
                    t = (int64_t)(li == 0 ? beg[0] : (li == 1 ? beg[1] : beg[2])) +
                        (gi - (li == 0 ? 0 : (li == 1 ? cum1 : cum2)));
                    const uint32_t *cp = (const uint32_t *)(a.codes + t * M);
#pragma unroll
                    for (int x = 0; x < M / 4; ++x) c2[x] = cp[x];
                    l2 = a.lam[t];
                }
                score(c2, l2, li > 2 ? 2 : li, t);
            }
            __syncthreads(); // tables may be overwritten; next vectors visible
        }
    }

    // ---- merge the eight wave lists ----
    wave_merge(wk, wcnt, K, lane, &sh_thr);
    for (int i = S2_KP + lane; i < S2_WSZ; i += 64) wk[i] = KEY_MAX;
    __syncthreads();
    block_bitonic_sort<S2_NT>(keys, S2_NW * S2_WSZ, tid);
    if (a.nsplit > 1) {
        uint64_t *dst = a.partial + ((int64_t)q * a.nsplit + split) * K;
        for (int i = tid; i < K; i += S2_NT) dst[i] = keys[i];
    } else {
        for (int i = tid; i < K; i += S2_NT) {
            const uint64_t key = keys[i];
            const bool ok = key != KEY_MAX;
            a.out_dist[(int64_t)q * K + i] = ok ? ord2f((uint32_t)(key >> 32)) : INFINITY;
            a.out_ids[(int64_t)q * K + i] = ok ? (int32_t)(uint32_t)key : -1;
        }
    }
}

static size_t scan_mfma_smem(int M, int D)
{
    return (size_t)S2_NW * S2_WSZ * 8 + (size_t)S2_SUBS * M * 256 * 8 + (size_t)4 * (D + 4) * 4 + (size_t)D * 4 +
           (size_t)S2_WIN * 4 * 6;
}

// Shapes served by this kernel; everything else takes the generic kernel.
bool scan_mfma_supported(const ScanArgs &a)
{
    return a.m == 8 && a.D == 128 && a.K <= S2_KP && (((uintptr_t)a.codes) % 8 == 0);
}

void launch_scan_mfma(const ScanArgs &a, hipStream_t st)
{
    if (a.nq <= 0) return;
    const size_t smem = scan_mfma_smem(a.m, a.D);
    (void)hipFuncSetAttribute((const void *)k_scan_mfma<8, 16>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    hipLaunchKernelGGL((k_scan_mfma<8, 16>), dim3((unsigned)(a.nq * a.nsplit)), dim3(S2_NT), smem, st, a);
}
