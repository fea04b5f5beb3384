// Second-level traversal, lookup tables, list scan and K-selection (Alg. 3).
#include "common.h"
#include <type_traits>

// ---------------------------------------------------------------------------
// Sub-region scores (Sec. 3.3.1): the query is line-quantised against every edge
// l(c_i, s_ij) of every probed cell.  With a = ||y-c_i||^2, b = ||y-s_ij||^2 and
// c = ||s_ij-c_i||^2, Eq. 8 gives the query's own lambda and Eq. 7 evaluated at
// that lambda collapses to a - c lambda^2.  Eq. 8's numerator (a + c - b) / 2 is the
// inner product g = <y - c_i, s_ij - c_i>; it is formed as that inner product, which
// keeps its rounding error proportional to |y - c_i| |s_ij - c_i| instead of a + b (a
// query far from a short edge would otherwise lose lambda to cancellation), so
// lambda = g / c, score = a - g lambda, and b - a = c - 2 g for the scan.  a is a
// direct sum of squared differences.  The w2 smallest by (score, label i*n+j) are kept.  On request the
// query's lambda is restricted to a range (the distance to a segment of the line).
//
// Outputs per query: the visited labels in (score, label) order (for callers
// that want the traversal) and the same set ordered by label, so that the
// sub-regions of one cell are adjacent, with g for the scan.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int wave_incl_scan(int v, int lane)
{
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(v, o, 64);
        if (lane >= o) v += t;
    }
    return v;
}

__global__ __launch_bounds__(256) void k_subregions(const float *__restrict__ Q, int D,
                                                    const float *__restrict__ C,
                                                    const int32_t *__restrict__ S,
                                                    const float *__restrict__ E, int n,
                                                    const int32_t *__restrict__ cells,
                                                    const float *__restrict__ cell_dist, int w1, int w2,
                                                    float lam_min, float lam_max,
                                                    int sz, int32_t *__restrict__ sub,
                                                    float *__restrict__ sub_score,
                                                    int32_t *__restrict__ scan_label,
                                                    float *__restrict__ scan_g,
                                                    const int64_t *__restrict__ off,
                                                    uint4 *__restrict__ desc,
                                                    const float *__restrict__ bpre)
{
    extern __shared__ unsigned char smem[];
    // With the distances precomputed and only the scan's descriptors asked for, the keys and the
    // positions of the selected sub-regions are all that lives in LDS (twice the workgroups per CU).
    const bool lean = bpre && !sub && !sub_score && !scan_label;
    uint64_t *keys = (uint64_t *)smem;          // [sz]
    float *bval = (float *)(keys + sz);          // [sz]   (not lean) g of every sub-region
    float *yv = bval + sz;                       // [D]    (not lean)
    uint16_t *pos = (uint16_t *)(yv + D);        // [sz]   (not lean)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = blockIdx.x;
    const int total = w1 * n;

    // [sz] neighbour centroid of every sub-region; later the positions of the selected ones
    int *nbr = lean ? (int *)(keys + sz) : (int *)(pos + sz);
    __shared__ int hist[256];
    __shared__ int sh4[4];
    __shared__ int sh_bin, sh_before, sh_inbin;
    __shared__ unsigned sh_lo, sh_hi;
    __shared__ unsigned long long sh_cut;
    __shared__ uint64_t ckeys[256];

    if (!lean)
        for (int d = tid; d < D; d += 256) yv[d] = Q[(int64_t)q * D + d];
    if (!bpre)
        for (int t = tid; t < total; t += 256) {
            const int e = t / n, j = t - e * n;
            const int i = cells[(int64_t)q * w1 + e];
            nbr[t] = i >= 0 ? S[(int64_t)i * n + j] : -1;
        }
    __syncthreads();

    // Line score of sub-region t = (probed cell e, edge j) from g = <y - c_i, s_ij - c_i>: lambda by
    // Eq. 8, squared distance to the line a - c lambda^2 = a - g lambda (Eq. 7 at that lambda)
    auto put_score = [&](int t, float g) {
        const int e = t / n, j = t - e * n;
        const int i = cells[(int64_t)q * w1 + e];
        uint64_t key = KEY_MAX;
        if (i >= 0) {
            const float a = cell_dist[(int64_t)q * w1 + e];
            const float c = E[(int64_t)i * n + j];
            const float lam = c > 0.f ? g / c : 0.f;
            float score = a - g * lam;
            // lambda restricted to [lam_min, lam_max] (the whole line by default): Eq. 7 at the
            // restricted value is the distance to the line plus c times the squared shift along it
            const float lc = fminf(fmaxf(lam, lam_min), lam_max);
            if (lc != lam) score = fmaf(c * (lc - lam), lc - lam, score);
            key = make_key(score, (uint32_t)(i * n + j));
        }
        keys[t] = key;
        if (!lean) {
            bval[t] = g;
            pos[t] = (uint16_t)t;
        }
    };
    if (bpre) {
        // the inner products were computed cell by cell beforehand (k_neighbour_dists)
        for (int t = tid; t < total; t += 256) put_score(t, bpre[(int64_t)q * total + t]);
    } else {
        // g = <y - c_i, s_ij - c_i> for all w1*n sub-regions: 16 lanes per centroid row, 4 rows per wave
        // instruction, 16 rows in flight per wave (the rows are scattered over the codebook, so
        // the loop lives on memory-level parallelism).  The order of the additions is fixed.
        const bool vec = (D % 4 == 0) && (((uintptr_t)C) % 16 == 0);
        const int sub16 = lane >> 4, l16 = lane & 15;
        for (int t0 = wave * 16; t0 < total; t0 += 64) {
            float part[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int t = t0 + g * 4 + sub16;
                const int s = t < total ? nbr[t] : -1;
                float acc = 0.f;
                if (s >= 0) {
                    const float *row = C + (int64_t)s * D;
                    const float *crow = C + (int64_t)cells[(int64_t)q * w1 + t / n] * D;
                    if (vec) {
                        for (int d = l16 * 4; d < D; d += 64) {
                            const f32x4 cv = *(const f32x4 *)(row + d);
                            const f32x4 cc = *(const f32x4 *)(crow + d);
                            acc = fmaf(yv[d] - cc.x, cv.x - cc.x, acc);
                            acc = fmaf(yv[d + 1] - cc.y, cv.y - cc.y, acc);
                            acc = fmaf(yv[d + 2] - cc.z, cv.z - cc.z, acc);
                            acc = fmaf(yv[d + 3] - cc.w, cv.w - cc.w, acc);
                        }
                    } else {
                        for (int d = l16; d < D; d += 16) {
                            const float cc = crow[d];
                            acc = fmaf(yv[d] - cc, row[d] - cc, acc);
                        }
                    }
                }
                part[g] = acc;
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) part[g] = row16_sum(part[g]);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int t = t0 + g * 4 + sub16;
                if (l16 == 0 && t < total) put_score(t, part[g]);
            }
        }
    }
    __syncthreads();

    // ---- the w2 smallest (score, label) keys: radix select of the cut key, then compaction ----
    int *selpos = nbr; // [w2] positions of the selected sub-regions (the neighbour ids are dead by now)
    int nvalid = 0;
    for (int t = tid; t < total; t += 256) nvalid += keys[t] != KEY_MAX;
    nvalid = wave_incl_scan(nvalid, lane);
    if (lane == 63) sh4[wave] = nvalid;
    __syncthreads();
    nvalid = sh4[0] + sh4[1] + sh4[2] + sh4[3];
    __syncthreads();
    const int w2eff = min(w2, nvalid);
    // rank-th smallest (0-based) value of one 32-bit half of the keys: the high half over all keys,
    // or the low half over the keys whose high half is `fixed`; 4 passes of 8 bits.  Leaves the
    // rank inside the final bin and the size of that bin.
    int res_rank = 0, res_inbin = 0;
    auto select32 = [&](bool low, uint32_t fixed, int rank) -> uint32_t {
        uint32_t prefix = 0;
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            hist[tid] = 0;
            __syncthreads();
            for (int t = tid; t < total; t += 256) {
                const uint64_t key = keys[t];
                if (key == KEY_MAX || (low && (uint32_t)(key >> 32) != fixed)) continue;
                const uint32_t u = low ? (uint32_t)key : (uint32_t)(key >> 32);
                if (pass == 0 || (u >> (shift + 8)) == (prefix >> (shift + 8))) atomicAdd(&hist[(u >> shift) & 255], 1);
            }
            __syncthreads();
            const int c = hist[tid];
            int inc = wave_incl_scan(c, lane);
            if (lane == 63) sh4[wave] = inc;
            __syncthreads();
            for (int w = 0; w < wave; ++w) inc += sh4[w];
            if (inc - c <= rank && rank < inc) {
                sh_bin = tid;
                sh_before = inc - c;
                sh_inbin = c;
            }
            __syncthreads();
            prefix |= (uint32_t)sh_bin << shift;
            rank -= sh_before;
            res_inbin = sh_inbin;
            __syncthreads();
        }
        res_rank = rank;
        return prefix;
    };
    // The cut key = the w2eff-th smallest key.  The scores between the smallest and the largest
    // are binned linearly (monotone in the score, so the bins partition the order); the bin that
    // holds the cut is binned again over its own range until it is small, then its keys are ranked
    // by counting.  Scores are handled as their ordered bit patterns.
    uint64_t cut = 0;
    if (w2eff > 0) {
        uint32_t olo = 0xFFFFFFFFu, ohi = 0u;
        for (int t = tid; t < total; t += 256) {
            const uint64_t key = keys[t];
            if (key == KEY_MAX) continue;
            const uint32_t o = (uint32_t)(key >> 32);
            olo = min(olo, o);
            ohi = max(ohi, o);
        }
        int need = w2eff; // rank (1-based) of the cut among the keys with olo <= score <= ohi
        int inbin = nvalid;
        for (int level = 0; level < 8; ++level) {
            // range of the undecided scores over the workgroup
            if (tid == 0) {
                sh_lo = 0xFFFFFFFFu;
                sh_hi = 0u;
            }
            hist[tid] = 0;
            __syncthreads();
            if (olo <= ohi) {
                atomicMin(&sh_lo, olo);
                atomicMax(&sh_hi, ohi);
            }
            __syncthreads();
            const uint32_t glo = sh_lo, ghi = sh_hi;
            if (inbin <= 256 || glo == ghi) {
                olo = glo;
                ohi = ghi;
                break;
            }
            const float flo = ord2f(glo), fhi = ord2f(ghi);
            if (!(fhi > flo)) { // one score (or not comparable): resolved below
                olo = glo;
                ohi = ghi;
                break;
            }
            const float scale = 256.f / (fhi - flo);
            for (int t = tid; t < total; t += 256) {
                const uint64_t key = keys[t];
                const uint32_t o = (uint32_t)(key >> 32);
                if (key == KEY_MAX || o < glo || o > ghi) continue;
                int b = (int)((ord2f(o) - flo) * scale);
                b = b > 255 ? 255 : (b < 0 ? 0 : b);
                atomicAdd(&hist[b], 1);
            }
            __syncthreads();
            const int c = hist[tid];
            int inc = wave_incl_scan(c, lane);
            if (lane == 63) sh4[wave] = inc;
            __syncthreads();
            for (int w = 0; w < wave; ++w) inc += sh4[w];
            if (inc - c < need && need <= inc) {
                sh_bin = tid;
                sh_before = inc - c;
                sh_inbin = c;
            }
            __syncthreads();
            const int B = sh_bin;
            need -= sh_before;
            inbin = sh_inbin;
            // the scores of bin B bound the next round
            olo = 0xFFFFFFFFu;
            ohi = 0u;
            for (int t = tid; t < total; t += 256) {
                const uint64_t key = keys[t];
                const uint32_t o = (uint32_t)(key >> 32);
                if (key == KEY_MAX || o < glo || o > ghi) continue;
                int b = (int)((ord2f(o) - flo) * scale);
                b = b > 255 ? 255 : (b < 0 ? 0 : b);
                if (b == B) {
                    olo = min(olo, o);
                    ohi = max(ohi, o);
                }
            }
            __syncthreads();
            if (level == 7) { // publish the last range as well
                if (tid == 0) {
                    sh_lo = 0xFFFFFFFFu;
                    sh_hi = 0u;
                }
                __syncthreads();
                if (olo <= ohi) {
                    atomicMin(&sh_lo, olo);
                    atomicMax(&sh_hi, ohi);
                }
                __syncthreads();
                olo = sh_lo;
                ohi = sh_hi;
            }
        }
        // the undecided keys: olo <= score <= ohi, `inbin` of them, the cut is the need-th smallest
        if (tid == 0) sh_bin = 0;
        __syncthreads();
        if (inbin <= 256) {
            uint64_t *ck = ckeys;
            for (int t = tid; t < total; t += 256) {
                const uint64_t key = keys[t];
                const uint32_t o = (uint32_t)(key >> 32);
                if (key == KEY_MAX || o < olo || o > ohi) continue;
                ck[atomicAdd(&sh_bin, 1)] = key;
            }
            __syncthreads();
            const int c = sh_bin;
            if (tid < c) {
                const uint64_t mine = ck[tid];
                int rank = 0;
                for (int j = 0; j < c; ++j) rank += ck[j] < mine;
                if (rank == need - 1) sh_cut = mine;
            }
            __syncthreads();
            cut = sh_cut;
        } else if (olo == ohi) {
            // more than 256 keys share one score: the smaller labels win
            const uint32_t lcut = select32(true, olo, need - 1);
            cut = ((uint64_t)olo << 32) | lcut;
        } else {
            // the range would not narrow (non-finite scores): radix select over all keys
            const uint32_t v = select32(false, 0u, w2eff - 1);
            uint32_t lcut = 0xFFFFFFFFu;
            if (res_inbin != res_rank + 1) lcut = select32(true, v, res_rank);
            cut = ((uint64_t)v << 32) | lcut;
        }
    }
    // every thread takes a contiguous range of positions, so the compacted order is that of the
    // positions: sub-regions of nearer cells first, which tightens the scan's bound early
    const int per = (total + 255) / 256;
    const int tb = tid * per, te = min(total, tb + per);
    int mysel = 0;
    if (w2eff > 0)
        for (int t = tb; t < te; ++t) mysel += keys[t] <= cut;
    int base = wave_incl_scan(mysel, lane);
    if (lane == 63) sh4[wave] = base;
    __syncthreads();
    for (int w = 0; w < wave; ++w) base += sh4[w];
    base -= mysel;
    if (w2eff > 0)
        for (int t = tb; t < te; ++t)
            if (keys[t] <= cut) selpos[base++] = t;
    __syncthreads();

    if (!sub && !sub_score && !scan_label) {
        // only the streaming scan follows: it takes the visited sub-regions in any order
        for (int r = tid; r < w2; r += 256) {
            uint4 dsc = make_uint4(0u, 0u, 0u, 0u);
            if (r < w2eff) {
                const int t = selpos[r];
                const int label = (int)(uint32_t)keys[t];
                const float a = cell_dist[(int64_t)q * w1 + t / n];
                const int64_t b0 = off[label], b1 = off[label + 1];
                const float g = lean ? bpre[(int64_t)q * total + t] : bval[t];
                // b - a = c - 2 g
                dsc = make_uint4((uint32_t)b0, (uint32_t)(b1 - b0), __float_as_uint(a), __float_as_uint(fmaf(-2.f, g, E[label])));
            }
            desc[(int64_t)q * w2 + r] = dsc;
        }
        return;
    }

    // the selected keys to the front, sorted by (score, label), original positions alongside
    const int sz2 = next_pow2_dev(w2);
    {
        uint64_t mk[8]; // w2 <= 2048 = 8 * 256
        int mp[8];
        int c = 0;
        for (int r = tid; r < w2; r += 256, ++c) {
            mk[c] = r < w2eff ? keys[selpos[r]] : KEY_MAX;
            mp[c] = r < w2eff ? selpos[r] : 0;
        }
        __syncthreads();
        c = 0;
        for (int r = tid; r < w2; r += 256, ++c) {
            keys[r] = mk[c];
            pos[r] = (uint16_t)mp[c];
        }
        for (int r = w2 + tid; r < sz2; r += 256) {
            keys[r] = KEY_MAX;
            pos[r] = 0;
        }
        __syncthreads();
        block_bitonic_sort_kv<256>(keys, pos, sz2, tid);
    }

    // (score, label) order for the caller; then re-key the visited ones by label
    uint64_t mine[8]; // w2 <= 2048 = 8 * 256
    int cnt = 0;
    for (int r = tid; r < w2; r += 256, ++cnt) {
        const uint64_t key = keys[r];
        const bool ok = key != KEY_MAX;
        const int label = ok ? (int)(uint32_t)key : -1;
        if (sub) sub[(int64_t)q * w2 + r] = label;
        if (sub_score) sub_score[(int64_t)q * w2 + r] = ok ? ord2f((uint32_t)(key >> 32)) : INFINITY;
        uint64_t k2 = KEY_MAX;
        uint4 dsc = make_uint4(0u, 0u, 0u, 0u);
        if (ok) {
            const int p = pos[r];
            const int e = p / n;
            const float a = cell_dist[(int64_t)q * w1 + e];
            const float g = bval[p];
            k2 = ((uint64_t)(uint32_t)label << 32) | __float_as_uint(g);
            if (desc) {
                const int64_t b0 = off[label], b1 = off[label + 1];
                dsc = make_uint4((uint32_t)b0, (uint32_t)(b1 - b0), __float_as_uint(a), __float_as_uint(fmaf(-2.f, g, E[label])));
            }
        }
        if (desc) desc[(int64_t)q * w2 + r] = dsc;
        mine[cnt] = k2;
    }
    if (!scan_label) return;
    __syncthreads();
    cnt = 0;
    for (int r = tid; r < w2; r += 256, ++cnt) keys[r] = mine[cnt];
    for (int r = w2 + tid; r < sz2; r += 256) keys[r] = KEY_MAX;
    __syncthreads();
    block_bitonic_sort<256>(keys, sz2, tid);
    for (int r = tid; r < w2; r += 256) {
        const uint64_t key = keys[r];
        const bool ok = key != KEY_MAX;
        scan_label[(int64_t)q * w2 + r] = ok ? (int32_t)(uint32_t)(key >> 32) : -1;
        scan_g[(int64_t)q * w2 + r] = ok ? __uint_as_float((uint32_t)key) : 0.f;
    }
}

// ---------------------------------------------------------------------------
// The same selection when only the scan's descriptors are asked for and the products g are there
// already (large batches): the w1*n keys of a query stay in registers, KPT consecutive ones per
// thread.  The cut, i.e. the w2-th smallest (score, label), is found bit by bit from the top of the
// ordered score pattern: every trial value is compared with all keys, the keys below it are
// counted with ballots and the four wave counts meet in LDS (one barrier per bit); scores equal to
// the cut's are then separated by label the same way.  The selected sub-regions keep the order of
// their positions (nearer cells first, which tightens the scan's bound early).
// ---------------------------------------------------------------------------
template <int KPT>
__global__ __launch_bounds__(256) void k_subregions_lean(const float *__restrict__ E, int n,
                                                         const int32_t *__restrict__ cells,
                                                         const float *__restrict__ cell_dist, int w1, int w2,
                                                         float lam_min, float lam_max,
                                                         const int64_t *__restrict__ off,
                                                         uint4 *__restrict__ desc,
                                                         const float *__restrict__ bpre)
{
    extern __shared__ uint32_t picked[]; // [w2] {label, b - a, probed cell} of the selected sub-regions
    __shared__ int slot[2][4];
    __shared__ int sh4[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = blockIdx.x;
    const int total = w1 * n;
    uint32_t o[KPT];     // ordered score bits; 0xFFFFFFFF = no sub-region
    uint32_t label[KPT];
    float bma[KPT];      // b - a = c - 2 g for the scan
    const int tb = tid * KPT;
    {
        // all loads without branches (indices clamped), so that they are in flight together
        int ci[KPT];
        float gv[KPT], av[KPT], cv[KPT];
#pragma unroll
        for (int e = 0; e < KPT; ++e) {
            const int t = min(tb + e, total - 1);
            ci[e] = cells[(int64_t)q * w1 + t / n];
            av[e] = cell_dist[(int64_t)q * w1 + t / n];
            gv[e] = bpre[(int64_t)q * total + t];
        }
#pragma unroll
        for (int e = 0; e < KPT; ++e) {
            const int t = min(tb + e, total - 1);
            cv[e] = E[(int64_t)max(ci[e], 0) * n + (t - (t / n) * n)];
        }
#pragma unroll
        for (int e = 0; e < KPT; ++e) {
            const int t = tb + e;
            const bool ok = t < total && ci[e] >= 0;
            const float c = cv[e];
            const float lam = c > 0.f ? gv[e] / c : 0.f;
            float score = av[e] - gv[e] * lam;
            const float lc = fminf(fmaxf(lam, lam_min), lam_max);
            if (lc != lam) score = fmaf(c * (lc - lam), lc - lam, score);
            label[e] = ok ? (uint32_t)(ci[e] * n + (t - (t / n) * n)) : 0xFFFFFFFFu;
            // (a score whose pattern is all ones would count as absent below: one step down keeps it present)
            o[e] = ok ? min(f2ord(score), 0xFFFFFFFEu) : 0xFFFFFFFFu;
            bma[e] = fmaf(-2.f, gv[e], c);
        }
    }
    // sum of a wave-uniform count over the four waves; `round` alternates the LDS slots, so one
    // barrier per call is enough
    int round = 0;
    auto block_sum = [&](int v) {
        if (lane == 0) slot[round & 1][wave] = v;
        __syncthreads();
        const int r = slot[round & 1][0] + slot[round & 1][1] + slot[round & 1][2] + slot[round & 1][3];
        ++round;
        return r;
    };
    int nv = 0;
#pragma unroll
    for (int e = 0; e < KPT; ++e) nv += __popcll(__ballot(o[e] != 0xFFFFFFFFu));
    const int nvalid = block_sum(nv);
    const int w2eff = min(w2, nvalid);
    uint32_t vcut = 0, lcut = 0xFFFFFFFFu;
    if (w2eff > 0) {
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t trial = vcut | (1u << bit);
            int below = 0;
#pragma unroll
            for (int e = 0; e < KPT; ++e) below += __popcll(__ballot(o[e] < trial)); // absent keys are below nothing
            if (block_sum(below) < w2eff) vcut = trial;
        }
        int less = 0, equal = 0;
#pragma unroll
        for (int e = 0; e < KPT; ++e) {
            less += __popcll(__ballot(o[e] < vcut));
            equal += __popcll(__ballot(o[e] == vcut));
        }
        less = block_sum(less);
        equal = block_sum(equal);
        const int need = w2eff - less; // of the keys with the cut's score, the smallest labels
        if (equal > need) {
            lcut = 0;
            for (int bit = 31; bit >= 0; --bit) {
                const uint32_t trial = lcut | (1u << bit);
                int below = 0;
#pragma unroll
                for (int e = 0; e < KPT; ++e)
                    below += __popcll(__ballot(o[e] == vcut && label[e] < trial));
                if (block_sum(below) < need) lcut = trial;
            }
        }
    }
    // the selected keys, in position order, into LDS
    int mysel = 0;
#pragma unroll
    for (int e = 0; e < KPT; ++e) {
        const bool sel = w2eff > 0 && (o[e] < vcut || (o[e] == vcut && label[e] <= lcut));
        mysel += sel;
    }
    int base = wave_incl_scan(mysel, lane);
    if (lane == 63) sh4[wave] = base;
    __syncthreads();
    for (int w = 0; w < wave; ++w) base += sh4[w];
    base -= mysel;
#pragma unroll
    for (int e = 0; e < KPT; ++e) {
        const bool sel = w2eff > 0 && (o[e] < vcut || (o[e] == vcut && label[e] <= lcut));
        if (sel && base < w2) { // (exactly w2eff keys are selected; the bound is a safeguard)
            picked[3 * base] = label[e];
            picked[3 * base + 1] = __float_as_uint(bma[e]);
            picked[3 * base + 2] = (uint32_t)((tb + e) / n);
            ++base;
        }
    }
    __syncthreads();
    // descriptors: a thread per selected sub-region, four at a time (their offset loads in flight together)
    for (int r0 = tid; r0 < w2; r0 += 1024) {
        uint32_t lb[4];
        int64_t b0[4], b1[4];
        float a[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = r0 + 256 * u;
            lb[u] = r < w2eff ? picked[3 * r] : 0u;
            b0[u] = off[lb[u]];
            b1[u] = off[lb[u] + 1];
            a[u] = cell_dist[(int64_t)q * w1 + (r < w2eff ? picked[3 * r + 2] : 0u)];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = r0 + 256 * u;
            if (r < w2)
                desc[(int64_t)q * w2 + r] = r < w2eff ? make_uint4((uint32_t)b0[u], (uint32_t)(b1[u] - b0[u]),
                                                                  __float_as_uint(a[u]), picked[3 * r + 1])
                                                      : make_uint4(0u, 0u, 0u, 0u);
        }
    }
}

// ---------------------------------------------------------------------------
// g = <y - c_i, s_ij - c_i> cell by cell (Alg. 3, second loop: the numerator of Eq. 8, from which
// b = a + c - 2 g follows).  A batch of queries probes most cells several times; the (query, probed
// cell) pairs are grouped by cell, a workgroup brings the centroid of its cell and the n edge vectors
// s_ij - c_i into LDS once and serves every pair of the cell from there.
// The sums are formed exactly as in k_subregions (16 lanes per row, fixed order).
// ---------------------------------------------------------------------------
__global__ void k_zero_i32(int32_t *p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0;
}

// Every pair learns its rank inside its cell while the cells are counted, so that the scatter
// after the prefix sum needs no second round of atomics.
__global__ void k_pair_count(const int32_t *__restrict__ cells, int64_t np, int32_t *__restrict__ cnt,
                             int32_t *__restrict__ rank)
{
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p < np) {
        const int c = cells[p];
        if (c >= 0) rank[p] = atomicAdd(&cnt[c], 1);
    }
}

__global__ void k_pair_scatter(const int32_t *__restrict__ cells, int64_t np, const int64_t *__restrict__ poff,
                               const int32_t *__restrict__ rank, int32_t *__restrict__ pairs,
                               const int64_t *__restrict__ woff, int4 *__restrict__ work, int chunk)
{
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p < np) {
        const int c = cells[p];
        if (c >= 0) {
            const int r = rank[p];
            const int64_t beg = poff[c];
            pairs[beg + r] = (int32_t)p;
            // the first pair of every chunk of its cell enters the chunk in the work list: {cell, place of the
            // chunk's first pair, pairs in the chunk}
            if (r % chunk == 0) {
                const int64_t left = poff[c + 1] - (beg + r);
                work[woff[c] + r / chunk] = make_int4(c, (int)(beg + r), (int)(left < chunk ? left : chunk), 0);
            }
        }
    }
}

#define ND_PCH 32 // pairs taken up at a time

// Grouped (pairs != nullptr): the pairs of a cell are cut into chunks of ND_PCH; a workgroup takes one
// chunk from the work list (woff[k] entries; the grid is an upper bound of that), brings the cell's rows
// into LDS and serves the chunk's pairs (a popular cell spreads over many workgroups).  Ungrouped (small
// batches): a workgroup per pair, in the pairs' own order, np_all of them.  Two pairs per wave, four
// rows per pass.
__global__ __launch_bounds__(256) void k_neighbour_dists(const float *__restrict__ Q, int D,
                                                         const float *__restrict__ C,
                                                         const int32_t *__restrict__ S, int n, int k, int w1,
                                                         const int32_t *__restrict__ cells,
                                                         const int64_t *__restrict__ poff,
                                                         const int32_t *__restrict__ pairs, int64_t np_all,
                                                         const int64_t *__restrict__ woff,
                                                         const int4 *__restrict__ work, float *__restrict__ bq)
{
    extern __shared__ float nrows[]; // [n][D] edge vectors s_ij - c_i, then [D] the centroid c_i
    __shared__ int sp[ND_PCH];
    float *crow = nrows + (size_t)n * D;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane >> 4, l16 = lane & 15;
    int64_t pbeg, pend;
    int cell;
    if (pairs) {
        if ((int64_t)blockIdx.x >= woff[k]) return;
        const int4 wi = work[blockIdx.x];
        cell = wi.x;
        pbeg = wi.y;
        pend = pbeg + wi.z;
    } else {
        pbeg = blockIdx.x;
        pend = pbeg + 1;
        if (pbeg >= np_all) return;
        cell = cells[pbeg];
        if (cell < 0) return; // a query with fewer than w1 cells
    }
    const bool vec = (D % 4 == 0) && ((((uintptr_t)C) | ((uintptr_t)Q)) % 16 == 0);
    const bool fast = vec && D <= 128;
    const int d0 = l16 * 4, d1 = 64 + l16 * 4;
    const bool has0 = fast && d0 < D, has1 = fast && d1 < D;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    // the first chunk's pairs are asked for now, beside the rows
    int first_p = 0;
    if (tid < min((int64_t)ND_PCH, pend - pbeg)) first_p = pairs ? pairs[pbeg + tid] : (int)(pbeg + tid);
    {
        const float *cg = C + (int64_t)cell * D;
        if (vec && D <= 128) {
            // half a wave per row, a lane per 16-byte chunk of it (so a thread subtracts the same chunk of the
            // centroid from all its rows); up to eight rows per thread and pass: their index loads first, then
            // their row loads, so that a pass costs two round trips
            const int d4 = D / 4, col = tid & 31, r8 = tid >> 5;
            const bool colok = col < d4;
            const f32x4 cvv = colok ? ((const f32x4 *)cg)[col] : zero;
            if (r8 == 0 && colok) ((f32x4 *)crow)[col] = cvv;
            for (int j0 = 0; j0 < n; j0 += 64) {
                int ss[8];
                f32x4 rv[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (j0 + 8 * u < n) ss[u] = S[(int64_t)cell * n + min(j0 + 8 * u + r8, n - 1)];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (j0 + 8 * u < n) rv[u] = colok ? ((const f32x4 *)(C + (int64_t)ss[u] * D))[col] : zero;
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int j = j0 + 8 * u + r8;
                    if (j0 + 8 * u < n && j < n && colok) ((f32x4 *)nrows)[j * d4 + col] = rv[u] - cvv;
                }
            }
        } else if (vec) {
            const int d4 = D / 4;
            for (int t = tid; t < (n + 1) * d4; t += 256) {
                const int j = t / d4, c = t - j * d4;
                const f32x4 cv = ((const f32x4 *)cg)[c];
                if (j < n) {
                    const int s = S[(int64_t)cell * n + j];
                    ((f32x4 *)nrows)[t] = ((const f32x4 *)(C + (int64_t)s * D))[c] - cv;
                } else {
                    ((f32x4 *)nrows)[t] = cv;
                }
            }
        } else {
            for (int t = tid; t < (n + 1) * D; t += 256) {
                const int j = t / D, d = t - j * D;
                nrows[t] = j < n ? C[(int64_t)S[(int64_t)cell * n + j] * D + d] - cg[d] : cg[d];
            }
        }
    }
    for (int64_t ch = pbeg; ch < pend; ch += ND_PCH) {
        const int i = 0, e = (int)min((int64_t)ND_PCH, pend - ch);
        __syncthreads(); // rows staged; the previous chunk's pair list no longer read
        if (tid < e) sp[tid] = ch == pbeg ? first_p : (pairs ? pairs[ch + tid] : (int)(ch + tid));
        __syncthreads();
        if (fast) {
            // A group of 16 lanes takes two pairs of the cell and a block of 16 rows: lane l keeps, for both
            // pairs, its share of the 16 dot products (the components 4 l .. 4 l + 3 and 64 + 4 l .. of
            // every row) in 2 x 16 registers, then the 16 x 16 partial sums of a pair are added across the
            // lanes and transposed at once: register s of lane l belongs to row s ^ g(l), with g chosen so that
            // each of the four lane-crossing steps of row16_sum (neighbour, other pair of the quad, other quad
            // of the half, other half) finds the same row in the partner's register s + 1, s + 2, s + 4, s + 8.
            // Half of the registers are given away at every step: 15 lane-crossing adds per pair instead of
            // 64, the same additions in the same association as row16_sum, so the sums are the same to the
            // bit; lane l ends with the sum of row g(l).
            const int gl = (l16 & 3) ^ ((l16 & 4) ? 7 : 0) ^ ((l16 & 8) ? 12 : 0);
            const int nb = (n + 15) >> 4;          // blocks of 16 rows
            const int npp = (e + 1) >> 1;          // pairs of pairs
            const int combos = npp * nb;
            for (int c0 = (wave << 2) + sub; c0 < ((combos + 15) & ~15); c0 += 16) {
                const bool live = c0 < combos;
                const int c = live ? c0 : 0;
                const int pp = c / nb, blk = c - pp * nb;
                const bool two = 2 * pp + 1 < e;
                const int pa = sp[2 * pp], pb = sp[two ? 2 * pp + 1 : 2 * pp];
                const float *ya = Q + (int64_t)(pa / w1) * D, *yb = Q + (int64_t)(pb / w1) * D;
                f32x4 a0 = zero, a1 = zero, b0 = zero, b1 = zero; // y - c_i
                if (has0) {
                    const f32x4 cc = *(const f32x4 *)(crow + d0);
                    a0 = *(const f32x4 *)(ya + d0) - cc;
                    b0 = *(const f32x4 *)(yb + d0) - cc;
                }
                if (has1) {
                    const f32x4 cc = *(const f32x4 *)(crow + d1);
                    a1 = *(const f32x4 *)(ya + d1) - cc;
                    b1 = *(const f32x4 *)(yb + d1) - cc;
                }
                float ra[16], rb[16];
#pragma unroll
                for (int sreg = 0; sreg < 16; ++sreg) {
                    const int j = min(blk * 16 + (sreg ^ gl), n - 1); // (rows past the end: computed, not stored)
                    const float *row = nrows + j * D;
                    float acca = 0.f, accb = 0.f;
                    if (has0) {
                        const f32x4 ev = *(const f32x4 *)(row + d0);
                        acca = fmaf(a0.x, ev.x, acca);
                        acca = fmaf(a0.y, ev.y, acca);
                        acca = fmaf(a0.z, ev.z, acca);
                        acca = fmaf(a0.w, ev.w, acca);
                        accb = fmaf(b0.x, ev.x, accb);
                        accb = fmaf(b0.y, ev.y, accb);
                        accb = fmaf(b0.z, ev.z, accb);
                        accb = fmaf(b0.w, ev.w, accb);
                    }
                    if (has1) {
                        const f32x4 ev = *(const f32x4 *)(row + d1);
                        acca = fmaf(a1.x, ev.x, acca);
                        acca = fmaf(a1.y, ev.y, acca);
                        acca = fmaf(a1.z, ev.z, acca);
                        acca = fmaf(a1.w, ev.w, acca);
                        accb = fmaf(b1.x, ev.x, accb);
                        accb = fmaf(b1.y, ev.y, accb);
                        accb = fmaf(b1.z, ev.z, accb);
                        accb = fmaf(b1.w, ev.w, accb);
                    }
                    ra[sreg] = acca;
                    rb[sreg] = accb;
                }
#define VLQ_DPP_GET(x, ctrl) __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), ctrl, 0xF, 0xF, true))
#pragma unroll
                for (int u = 0; u < 16; u += 2) { // neighbour in the pair: quad_perm [1, 0, 3, 2]
                    ra[u] += VLQ_DPP_GET(ra[u + 1], 0xB1);
                    rb[u] += VLQ_DPP_GET(rb[u + 1], 0xB1);
                }
#pragma unroll
                for (int u = 0; u < 16; u += 4) { // other pair of the quad: quad_perm [2, 3, 0, 1]
                    ra[u] += VLQ_DPP_GET(ra[u + 2], 0x4E);
                    rb[u] += VLQ_DPP_GET(rb[u + 2], 0x4E);
                }
#pragma unroll
                for (int u = 0; u < 16; u += 8) { // other quad of the half: row_half_mirror
                    ra[u] += VLQ_DPP_GET(ra[u + 4], 0x141);
                    rb[u] += VLQ_DPP_GET(rb[u + 4], 0x141);
                }
                ra[0] += VLQ_DPP_GET(ra[8], 0x140); // other half of the row: row_mirror
                rb[0] += VLQ_DPP_GET(rb[8], 0x140);
#undef VLQ_DPP_GET
                const int j = blk * 16 + gl;
                if (live && j < n) {
                    bq[(int64_t)pa * n + j] = ra[0];
                    if (two) bq[(int64_t)pb * n + j] = rb[0];
                }
            }
        } else
        for (int pi = i + wave; pi < e; pi += 4) {
            const int p = sp[pi];
            const float *y = Q + (int64_t)(p / w1) * D;
            for (int j0 = 0; j0 < n; j0 += 4) {
                const int j = j0 + sub;
                float acc = 0.f;
                if (j < n) {
                    const float *row = nrows + j * D;
                    if (vec) {
                        for (int d = l16 * 4; d < D; d += 64) {
                            const f32x4 ev = *(const f32x4 *)(row + d);
                            const f32x4 zv = *(const f32x4 *)(y + d) - *(const f32x4 *)(crow + d);
                            acc = fmaf(zv.x, ev.x, acc);
                            acc = fmaf(zv.y, ev.y, acc);
                            acc = fmaf(zv.z, ev.z, acc);
                            acc = fmaf(zv.w, ev.w, acc);
                        }
                    } else {
                        for (int d = l16; d < D; d += 16) acc = fmaf(y[d] - crow[d], row[d], acc);
                    }
                }
                acc = row16_sum(acc);
                if (l16 == 0 && j < n) bq[(int64_t)p * n + j] = acc;
            }
        }
    }
}

// Few pairs: grouping them by cell (count, prefix sum over all k cells, scatter) costs more than the
// row loads it saves; every pair is then served on its own.
bool neighbour_dists_grouped(int nq, int w1) { return (int64_t)nq * w1 > 4096; }

bool neighbour_dists_by_cell(int nq, int k, int n, int D, int w1)
{
    // the centroid of a cell and its n edge vectors must fit in LDS (two workgroups per compute unit)
    (void)nq; (void)k; (void)w1;
    return (size_t)(n + 1) * D * 4 <= 73728;
}

size_t neighbour_dists_workspace(int nq, int k, int n, int w1)
{
    size_t b = 0;
    b += (((size_t)k * 4) + 255) & ~(size_t)255;                   // counts
    b += (((size_t)(k + 1) * 8) + 255) & ~(size_t)255;             // offsets
    b += (((size_t)nq * w1 * 4) + 255) & ~(size_t)255;             // ranks
    b += (((size_t)nq * w1 * 4) + 255) & ~(size_t)255;             // pairs
    b += (((size_t)(k + 1) * 8) + 255) & ~(size_t)255;             // work offsets
    b += ((((size_t)nq * w1 / ND_PCH + k + 1) * 16) + 255) & ~(size_t)255; // work list
    b += (((size_t)nq * w1 * n * 4) + 255) & ~(size_t)255;         // distances
    return b;
}

PairWs neighbour_dists_carve(void *ws, int nq, int k, int n, int w1)
{
    char *base = (char *)ws;
    auto take = [&](size_t bytes) {
        char *at = base;
        base += (bytes + 255) & ~(size_t)255;
        return at;
    };
    PairWs pw;
    pw.cnt = (int32_t *)take((size_t)k * 4);
    pw.poff = (int64_t *)take((size_t)(k + 1) * 8);
    pw.rank = (int32_t *)take((size_t)nq * w1 * 4);
    pw.pairs = (int32_t *)take((size_t)nq * w1 * 4);
    pw.woff = (int64_t *)take((size_t)(k + 1) * 8);
    pw.work = (int4 *)take(((size_t)nq * w1 / ND_PCH + k + 1) * 16);
    pw.bq = (float *)take((size_t)nq * w1 * n * 4);
    return pw;
}

void launch_pair_counts_zero(const PairWs &pw, int k, hipStream_t st)
{
    hipLaunchKernelGGL(k_zero_i32, dim3((unsigned)(((int64_t)k + 255) / 256)), dim3(256), 0, st, pw.cnt, (int64_t)k);
}

void launch_subregions(const float *Q, int nq, int D, const float *C, const int32_t *S, const float *E,
                       int n, int k, const int32_t *cells, const float *cell_dist, int w1, int w2,
                       float lam_min, float lam_max, int32_t *sub, float *sub_score, int32_t *scan_label,
                       float *scan_g, const int64_t *off, uint4 *desc, void *ws, bool pairs_counted, hipStream_t st)
{
    if (nq <= 0) return;
    const float *bpre = nullptr;
    if (ws) {
        // neighbour distances cell by cell; ws has neighbour_dists_workspace() bytes
        const PairWs pw = neighbour_dists_carve(ws, nq, k, n, w1);
        int32_t *cnt = pw.cnt, *rank = pw.rank, *pairs = pw.pairs;
        int64_t *poff = pw.poff;
        float *bq = pw.bq;
        const int64_t np = (int64_t)nq * w1;
        const bool grouped = neighbour_dists_grouped(nq, w1);
        if (grouped) {
            if (!pairs_counted) {
                launch_pair_counts_zero(pw, k, st);
                hipLaunchKernelGGL(k_pair_count, dim3((unsigned)((np + 255) / 256)), dim3(256), 0, st, cells, np, cnt, rank);
            }
            launch_exclusive_scan_chunks(cnt, k, poff, ND_PCH, pw.woff, st);
            hipLaunchKernelGGL(k_pair_scatter, dim3((unsigned)((np + 255) / 256)), dim3(256), 0, st, cells, np, poff,
                               rank, pairs, pw.woff, pw.work, ND_PCH);
        }
        const size_t rows_bytes = (size_t)(n + 1) * D * 4;
        if (rows_bytes > 49152) // (48 KB of dynamic LDS beside the static part need no asking)
            (void)hipFuncSetAttribute((const void *)k_neighbour_dists, hipFuncAttributeMaxDynamicSharedMemorySize, (int)rows_bytes);
        // grouped: at most np / ND_PCH full chunks and one partial chunk per probed cell
        const int64_t most_cells = np < (int64_t)k ? np : (int64_t)k;
        hipLaunchKernelGGL(k_neighbour_dists, dim3((unsigned)(grouped ? np / ND_PCH + most_cells : np)), dim3(256), rows_bytes, st, Q,
                           D, C, S, n, k, w1, cells, poff, grouped ? pairs : nullptr, np, pw.woff, pw.work, bq);
        bpre = bq;
    }
    int sz = next_pow2(w1 * n);
    if (sz < next_pow2(w2)) sz = next_pow2(w2);
    if (sz < 2) sz = 2;
    const bool lean = bpre && !sub && !sub_score && !scan_label;
    if (lean && desc && w1 * n <= 4096) {
        // keys in registers: 4, 8 or 16 per thread
        const int total = w1 * n;
        const size_t pk = (size_t)w2 * 12;
        if (total <= 1024)
            hipLaunchKernelGGL(k_subregions_lean<4>, dim3((unsigned)nq), dim3(256), pk, st, E, n, cells, cell_dist, w1, w2,
                               lam_min, lam_max, off, desc, bpre);
        else if (total <= 2048)
            hipLaunchKernelGGL(k_subregions_lean<8>, dim3((unsigned)nq), dim3(256), pk, st, E, n, cells, cell_dist, w1, w2,
                               lam_min, lam_max, off, desc, bpre);
        else
            hipLaunchKernelGGL(k_subregions_lean<16>, dim3((unsigned)nq), dim3(256), pk, st, E, n, cells, cell_dist, w1, w2,
                               lam_min, lam_max, off, desc, bpre);
        return;
    }
    size_t smem = lean ? (size_t)sz * (8 + 4) : (size_t)sz * (8 + 4 + 2 + 4) + (size_t)D * 4;
    if (smem > 49152) // (48 KB of dynamic LDS beside the static part need no asking)
        (void)hipFuncSetAttribute((const void *)k_subregions, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    hipLaunchKernelGGL(k_subregions, dim3((unsigned)nq), dim3(256), smem, st, Q, D, C, S, E, n, cells,
                       cell_dist, w1, w2, lam_min, lam_max, sz, sub, sub_score, scan_label, scan_g, off, desc, bpre);
}

// ---------------------------------------------------------------------------
// Lookup tables + list scan + K-selection (Sec. 3.3.2 - 3.3.3).
//
// For a point x of sub-region (i, j) with code (t_1..t_m) and lambda byte value
// l, Eq. 14 is || (y - c_i) - l e - q2 ||^2 with e = s_ij - c_i and q2 the
// concatenation of the codewords.  Expanding around z = y - c_i gives
//
//   dist = sum_p A[p][t_p]  +  l * ( 2 sum_p B[p][t_p] - 2 g )  +  l^2 c
//   A[p][t] = || z^p - P[p][t] ||^2       per (query, cell)
//   B[p][t] = < e^p , P[p][t] >           per sub-region
//   g = <z, e>,  c = ||e||^2
//
// which is Eq. 16-17 with term2, term3 and term5 folded into A and
// term4 - term3 into B: 2m lookups per point, as counted in Sec. 3.3.2, but
// no large cancelling terms.  A and B are interleaved in LDS so that one
// 64-bit read serves both.
//
// A workgroup handles one (query, split) pair: a contiguous range of the
// query's visited sub-regions in label order.  Candidates below the current
// K-th key go to an LDS buffer that is merged into the sorted top-K by a
// bitonic sort whenever it fills.
// ---------------------------------------------------------------------------
#define SCAN_NT 256
#define SCAN_PTS 4 // points per thread between two buffer checks

template <int NT>
__device__ __forceinline__ void topk_merge(uint64_t *keys, int KP, int SZ, int K, int *cnt_p, uint64_t *thr_p,
                                           int tid)
{
    // keys[0..KP) current result (sorted, padded), keys[KP..KP+cnt) new candidates
    __syncthreads();
    const int cnt = *cnt_p;
    for (int i = KP + cnt + tid; i < SZ; i += NT) keys[i] = KEY_MAX;
    __syncthreads();
    block_bitonic_sort<NT>(keys, SZ, tid);
    for (int i = K + tid; i < KP; i += NT) keys[i] = KEY_MAX;
    if (tid == 0) {
        *cnt_p = 0;
        *thr_p = keys[K - 1];
    }
    __syncthreads();
}

__global__ __launch_bounds__(SCAN_NT) void k_scan(ScanArgs a, int KP, int SZ)
{
    extern __shared__ unsigned char smem[];
    const int m = a.m, D = a.D, ds = D / m;
    uint64_t *keys = (uint64_t *)smem;                 // [SZ]
    float2 *AB = (float2 *)(keys + SZ);                // [m * 256]
    float *yv = (float *)(AB + m * 256);               // [D]
    float *zv = yv + D;                                // [D]
    float *ev = zv + D;                                // [D]
    __shared__ int sh_cnt;
    __shared__ uint64_t sh_thr;

    const int tid = threadIdx.x;
    const int q = blockIdx.x / a.nsplit, split = blockIdx.x - q * a.nsplit;
    const int CB = SZ - KP;
    const int r0 = (int)((int64_t)a.w2 * split / a.nsplit), r1 = (int)((int64_t)a.w2 * (split + 1) / a.nsplit);

    for (int d = tid; d < D; d += SCAN_NT) yv[d] = a.Q[(int64_t)q * D + d];
    for (int i = tid; i < KP; i += SCAN_NT) keys[i] = KEY_MAX;
    if (tid == 0) {
        sh_cnt = 0;
        sh_thr = KEY_MAX;
    }
    __syncthreads();

    int cur_cell = -1;
    for (int r = r0; r < r1; ++r) {
        const int label = a.scan_label[(int64_t)q * a.w2 + r];
        if (label < 0) continue; // uniform over the workgroup
        const int64_t beg = a.off[label], end = a.off[label + 1];
        if (beg == end) continue;
        const int i = label / a.n, j = label - i * a.n;
        const bool new_cell = i != cur_cell;
        cur_cell = i;
        const float *ci = a.C + (int64_t)i * D;
        const float *sj = a.C + (int64_t)a.S[(int64_t)i * a.n + j] * D;
        __syncthreads(); // previous list fully scanned before the tables change
        for (int d = tid; d < D; d += SCAN_NT) {
            const float c = ci[d];
            zv[d] = yv[d] - c;
            ev[d] = sj[d] - c;
        }
        __syncthreads();
        // lookup tables
        for (int idx = tid; idx < m * 256; idx += SCAN_NT) {
            const int p = idx >> 8;
            const float *w = a.P + (int64_t)idx * ds;
            const float *zp = zv + p * ds, *ep = ev + p * ds;
            float sb = 0.f;
            for (int d = 0; d < ds; ++d) sb = fmaf(ep[d], w[d], sb);
            if (new_cell) {
                float sa = 0.f;
                for (int d = 0; d < ds; ++d) {
                    const float t = zp[d] - w[d];
                    sa = fmaf(t, t, sa);
                }
                AB[idx] = make_float2(sa, sb);
            } else {
                AB[idx].y = sb;
            }
        }
        const float cc = a.E[label];
        const float g = a.scan_g[(int64_t)q * a.w2 + r];
        __syncthreads();

        // scan the list
        for (int64_t base = beg; base < end; base += SCAN_NT * SCAN_PTS) {
            // the fill level is read between two barriers with no appends in between,
            // so every thread takes the same decision
            const int fill = sh_cnt;
            __syncthreads();
            if (fill > CB - SCAN_NT * SCAN_PTS) topk_merge<SCAN_NT>(keys, KP, SZ, a.K, &sh_cnt, &sh_thr, tid);
            const uint64_t thr = sh_thr;
#pragma unroll
            for (int u = 0; u < SCAN_PTS; ++u) {
                const int64_t t = base + u * SCAN_NT + tid;
                if (t < end) {
                    const uint8_t *code = a.codes + t * m;
                    float sa = 0.f, sb = 0.f;
                    if ((m & 3) == 0) {
                        const uint32_t *cw = (const uint32_t *)code;
                        for (int p4 = 0; p4 < m; p4 += 4) {
                            const uint32_t wv = cw[p4 >> 2];
#pragma unroll
                            for (int b = 0; b < 4; ++b) {
                                const float2 ab = AB[(p4 + b) * 256 + ((wv >> (8 * b)) & 255u)];
                                sa += ab.x;
                                sb += ab.y;
                            }
                        }
                    } else {
                        for (int p = 0; p < m; ++p) {
                            const float2 ab = AB[p * 256 + code[p]];
                            sa += ab.x;
                            sb += ab.y;
                        }
                    }
                    const float l = ((float)a.lam[t] - a.lam_zero) * a.lam_step;
                    const float dist = fmaf(l, fmaf(l, cc, 2.f * (sb - g)), sa);
                    const uint64_t key = make_key(dist, (uint32_t)a.ids[t]);
                    if (key < thr) {
                        const int pos = atomicAdd(&sh_cnt, 1);
                        keys[KP + pos] = key;
                    }
                }
            }
            __syncthreads();
        }
    }
    topk_merge<SCAN_NT>(keys, KP, SZ, a.K, &sh_cnt, &sh_thr, tid);
    if (a.nsplit > 1) {
        uint64_t *dst = a.partial + ((int64_t)q * a.nsplit + split) * a.K;
        for (int i = tid; i < a.K; i += SCAN_NT) dst[i] = keys[i];
    } else {
        for (int i = tid; i < a.K; i += SCAN_NT) {
            const uint64_t key = keys[i];
            const bool ok = key != KEY_MAX;
            a.out_dist[(int64_t)q * a.K + i] = ok ? ord2f((uint32_t)(key >> 32)) : INFINITY;
            a.out_ids[(int64_t)q * a.K + i] = ok ? (int32_t)(uint32_t)key : -1;
        }
    }
}

static void scan_sizes(int K, int *KP, int *SZ)
{
    *KP = next_pow2(K);
    int sz = 2 * *KP;
    if (sz < 2048) sz = 2048;
    *SZ = sz;
}

int scan_pick_nsplit(int nq, int w2, int K)
{
    // aim at >= 4 workgroups per compute unit (256 CUs); never more splits than lists
    int ns = (1024 + nq - 1) / nq;
    if (ns > w2) ns = w2;
    const int kp = next_pow2(K);
    const int cap = 8192 / kp; // the merge holds nsplit * K keys in LDS
    if (ns > cap) ns = cap;
    if (ns > 16) ns = 16;
    if (ns < 1) ns = 1;
    return ns;
}

bool scan_will_stream(const ScanArgs &a) { return !a.force_generic && scan_stream_supported(a); }

void launch_scan(const ScanArgs &a, hipStream_t st)
{
    if (a.nq <= 0) return;
    if (scan_will_stream(a)) {
        launch_scan_stream(a, st);
        return;
    }
    int KP, SZ;
    scan_sizes(a.K, &KP, &SZ);
    size_t smem = (size_t)SZ * 8 + (size_t)a.m * 256 * 8 + (size_t)a.D * 4 * 3;
    if (smem > 49152) // (48 KB of dynamic LDS beside the static part need no asking)
        (void)hipFuncSetAttribute((const void *)k_scan, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    hipLaunchKernelGGL(k_scan, dim3((unsigned)(a.nq * a.nsplit)), dim3(SCAN_NT), smem, st, a, KP, SZ);
}

// Merge of the per-split partial results of one query (second pass of the
// two-pass K-selection of Sec. 4).  Every partial list is sorted, so the place of a key in the
// merged order is its position in its own list plus the number of keys that precede it in every
// other list (a binary search each): no sorting.  Equal keys (possible only when the caller's ids
// repeat) are ordered by list, so that every place is taken once.
__global__ __launch_bounds__(256) void k_merge(const uint64_t *__restrict__ partial, int nsplit, int K,
                                               float *__restrict__ out_dist, int32_t *__restrict__ out_ids)
{
    extern __shared__ unsigned char smem[];
    uint64_t *keys = (uint64_t *)smem; // [nsplit][K]
    uint64_t *outk = keys + nsplit * K; // [K]
    const int tid = threadIdx.x, q = blockIdx.x;
    const int total = nsplit * K;
    for (int i = tid; i < total; i += 256) keys[i] = partial[(int64_t)q * total + i];
    for (int i = tid; i < K; i += 256) outk[i] = KEY_MAX;
    __syncthreads();
    for (int e = tid; e < total; e += 256) {
        const uint64_t x = keys[e];
        if (x == KEY_MAX) continue;
        const int s = e / K;
        int rank = e - s * K;
        for (int o = 0; o < nsplit && rank < K; ++o) {
            if (o == s) continue;
            const uint64_t *l = keys + o * K;
            int lo = 0, hi = K; // keys of list o that precede x: smaller ones, and equal ones of earlier lists
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (l[mid] < x || (o < s && l[mid] == x))
                    lo = mid + 1;
                else
                    hi = mid;
            }
            rank += lo;
        }
        if (rank < K) outk[rank] = x;
    }
    __syncthreads();
    for (int i = tid; i < K; i += 256) {
        const uint64_t key = outk[i];
        const bool ok = key != KEY_MAX;
        out_dist[(int64_t)q * K + i] = ok ? ord2f((uint32_t)(key >> 32)) : INFINITY;
        out_ids[(int64_t)q * K + i] = ok ? (int32_t)(uint32_t)key : -1;
    }
}

void launch_merge(const uint64_t *partial, int nq, int nsplit, int K, float *out_dist, int32_t *out_ids,
                  hipStream_t st)
{
    if (nq <= 0) return;
    size_t smem = (size_t)(nsplit + 1) * K * 8;
    if (smem > 49152) // (48 KB of dynamic LDS beside the static part need no asking)
        (void)hipFuncSetAttribute((const void *)k_merge, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    hipLaunchKernelGGL(k_merge, dim3((unsigned)nq), dim3(256), smem, st, partial, nsplit, K, out_dist, out_ids);
}
