// Inverted lists (Sec. 4): list lengths (as offsets), ids, codes and lambda
// bytes of the k*n sub-regions, list l = cell * n + edge, ascending id inside a
// list.  Built by a counting sort of the staged points.
#include "common.h"

__global__ void k_iota_i32(int32_t *p, int64_t n, int32_t start)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = start + (int32_t)i;
}
void launch_iota_i32(int32_t *p, int64_t n, int32_t start, hipStream_t st)
{
    if (n <= 0) return;
    hipLaunchKernelGGL(k_iota_i32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n, start);
}

__global__ void k_pack_labels(const int32_t *__restrict__ cell, const int32_t *__restrict__ edge, int n, int k,
                              int32_t *__restrict__ label, int64_t nb, int32_t *__restrict__ bad)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nb) return;
    const int c = cell[i], e = edge[i];
    if (c < 0 || c >= k || e < 0 || e >= n) {
        label[i] = -1;
        atomicOr(bad, 1);
    } else {
        label[i] = c * n + e;
    }
}
void launch_pack_labels(const int32_t *cell, const int32_t *edge, int n, int k, int32_t *label, int64_t nb,
                        int32_t *bad, hipStream_t st)
{
    if (nb <= 0) return;
    hipLaunchKernelGGL(k_pack_labels, dim3((unsigned)((nb + 255) / 256)), dim3(256), 0, st, cell, edge, n, k,
                       label, nb, bad);
}

__global__ void k_list_histogram(const int32_t *__restrict__ label, int64_t N, int32_t *__restrict__ cnt)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N; i += stride) {
        const int l = label[i];
        if (l >= 0) atomicAdd(&cnt[l], 1);
    }
}
void launch_list_histogram(const int32_t *label, int64_t N, int32_t *cnt, hipStream_t st)
{
    if (N <= 0) return;
    int64_t blocks = (N + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(k_list_histogram, dim3((unsigned)blocks), dim3(256), 0, st, label, N, cnt);
}

// off[i] = sum of cnt[0..i), off[nl] = total; one workgroup walks the array in tiles of 16 384
// (sixteen consecutive counts per thread: few rounds, each with two barriers), carrying the sum.
#define XS_PER 16
__global__ __launch_bounds__(1024) void k_exclusive_scan(const int32_t *__restrict__ cnt, int64_t nl,
                                                         int64_t *__restrict__ off)
{
    __shared__ int64_t wsum[16];
    __shared__ int64_t carry_sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool vec = ((uintptr_t)cnt) % 16 == 0;
    int64_t carry = 0;
    for (int64_t t0 = 0; t0 < nl; t0 += 1024 * XS_PER) {
        const int64_t i0 = t0 + XS_PER * tid;
        int32_t c[XS_PER];
        if (vec && i0 + XS_PER <= nl) {
#pragma unroll
            for (int e = 0; e < XS_PER; e += 4) {
                const int4 v = *(const int4 *)(cnt + i0 + e);
                c[e] = v.x;
                c[e + 1] = v.y;
                c[e + 2] = v.z;
                c[e + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int e = 0; e < XS_PER; ++e) c[e] = i0 + e < nl ? cnt[i0 + e] : 0;
        }
        int64_t mine = 0;
#pragma unroll
        for (int e = 0; e < XS_PER; ++e) mine += c[e];
        int64_t inc = mine; // inclusive scan over the wave
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int64_t v = __shfl_up(inc, o, 64);
            if (lane >= o) inc += v;
        }
        if (lane == 63) wsum[wave] = inc;
        __syncthreads();
        int64_t before = carry;
        for (int w = 0; w < wave; ++w) before += wsum[w];
        int64_t run = before + inc - mine;
#pragma unroll
        for (int e = 0; e < XS_PER; ++e) {
            if (i0 + e < nl) off[i0 + e] = run;
            run += c[e];
        }
        if (tid == 1023) carry_sh = run;
        __syncthreads();
        carry = carry_sh;
    }
    if (tid == 0) off[nl] = carry;
}
// The same for short arrays (the per-cell pair counts of a search) without the serial walk: a workgroup per
// 4 096 counts first adds up everything before its tile (read again by every later workgroup: a few
// hundred KB from L2 at most), then scans its own tile.
#define XB_TILE 4096
// With chunk > 0, a power of two, the scan of ceil(cnt / chunk) goes to off2 beside it (both are summed in one word, the counts
// in the low 32 bits, the chunk counts above them: for counts that add up to less than 2^31).
__global__ __launch_bounds__(256) void k_exclusive_scan_tiles(const int32_t *__restrict__ cnt, int64_t nl,
                                                              int64_t *__restrict__ off, int chunk,
                                                              int64_t *__restrict__ off2)
{
    __shared__ int64_t wsum[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t t0 = (int64_t)blockIdx.x * XB_TILE;
    // (chunk is a power of two)
    const int csh = chunk > 0 ? 31 - __clz(chunk) : 0;
    auto both = [&](int32_t c) { return (int64_t)c + (chunk > 0 ? (int64_t)((c + chunk - 1) >> csh) << 32 : 0); };
    const int64_t low = chunk > 0 ? (((int64_t)1 << 32) - 1) : ~(int64_t)0;
    int64_t before = 0;
    for (int64_t i = 4 * tid; i < t0; i += XB_TILE) { // t0 is a multiple of the tile: four loads in flight
        int4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = *(const int4 *)(cnt + i + 1024 * u);
#pragma unroll
        for (int u = 0; u < 4; ++u) before += both(v[u].x) + both(v[u].y) + both(v[u].z) + both(v[u].w);
    }
    const int64_t i0 = t0 + XS_PER * tid;
    int32_t c[XS_PER];
#pragma unroll
    for (int e = 0; e < XS_PER; ++e) c[e] = i0 + e < nl ? cnt[i0 + e] : 0;
    int64_t mine = 0;
#pragma unroll
    for (int e = 0; e < XS_PER; ++e) mine += both(c[e]);
    // the sum of `before` over the workgroup, and the scan of `mine`
    int64_t inc = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int64_t v = __shfl_up(inc, o, 64);
        if (lane >= o) inc += v;
        before += __shfl_xor(before, o, 64);
    }
    if (lane == 63) wsum[wave] = inc;
    __shared__ int64_t bsum[4];
    if (lane == 0) bsum[wave] = before;
    __syncthreads();
    int64_t run = bsum[0] + bsum[1] + bsum[2] + bsum[3] + inc - mine;
    for (int w = 0; w < wave; ++w) run += wsum[w];
#pragma unroll
    for (int e = 0; e < XS_PER; ++e) {
        if (i0 + e < nl) {
            off[i0 + e] = run & low;
            if (chunk > 0) off2[i0 + e] = run >> 32;
        }
        run += both(c[e]);
    }
    if (i0 <= nl - 1 && nl - 1 < i0 + XS_PER) { // the thread that holds the last count
        off[nl] = run & low;
        if (chunk > 0) off2[nl] = run >> 32;
    }
}

void launch_exclusive_scan(const int32_t *cnt, int64_t nl, int64_t *off, hipStream_t st)
{
    if (nl > 0 && nl <= ((int64_t)1 << 18) && ((uintptr_t)cnt) % 16 == 0)
        hipLaunchKernelGGL(k_exclusive_scan_tiles, dim3((unsigned)((nl + XB_TILE - 1) / XB_TILE)), dim3(256), 0, st, cnt,
                           nl, off, 0, (int64_t *)nullptr);
    else
        hipLaunchKernelGGL(k_exclusive_scan, dim3(1), dim3(1024), 0, st, cnt, nl, off);
}

void launch_exclusive_scan_chunks(const int32_t *cnt, int64_t nl, int64_t *off, int chunk, int64_t *off2, hipStream_t st)
{
    hipLaunchKernelGGL(k_exclusive_scan_tiles, dim3((unsigned)((nl + XB_TILE - 1) / XB_TILE)), dim3(256), 0, st, cnt, nl,
                       off, chunk, off2);
}

__global__ void k_list_scatter(const int32_t *__restrict__ label, const int32_t *__restrict__ st_ids,
                               const uint8_t *__restrict__ st_codes, const uint8_t *__restrict__ st_lam,
                               int64_t N, int m, const int64_t *__restrict__ off,
                               int32_t *__restrict__ cursor, int32_t *__restrict__ ids,
                               uint8_t *__restrict__ codes, uint8_t *__restrict__ lam)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N; i += stride) {
        const int l = label[i];
        if (l < 0) continue;
        const int64_t pos = off[l] + atomicAdd(&cursor[l], 1);
        ids[pos] = st_ids[i];
        lam[pos] = st_lam[i];
        if ((m & 3) == 0) {
            const uint32_t *s = (const uint32_t *)(st_codes + i * m);
            uint32_t *d = (uint32_t *)(codes + pos * m);
            for (int p = 0; p < m / 4; ++p) d[p] = s[p];
        } else {
            for (int p = 0; p < m; ++p) codes[pos * m + p] = st_codes[i * m + p];
        }
    }
}
void launch_list_scatter(const int32_t *label, const int32_t *st_ids, const uint8_t *st_codes,
                         const uint8_t *st_lam, int64_t N, int m, const int64_t *off, int32_t *cursor,
                         int32_t *ids, uint8_t *codes, uint8_t *lam, hipStream_t st)
{
    if (N <= 0) return;
    int64_t blocks = (N + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(k_list_scatter, dim3((unsigned)blocks), dim3(256), 0, st, label, st_ids, st_codes, st_lam,
                       N, m, off, cursor, ids, codes, lam);
}

// The scatter places the points of a list in arbitrary order; this pass orders
// every list by id.  One 64-thread workgroup per list sorts lists of up to
// SORT_MAX points in LDS; longer unsorted lists are reported to the host.
#define SORT_MAX 1024

__global__ __launch_bounds__(64) void k_list_sort(const int64_t *__restrict__ off, int64_t nl, int m,
                                                  int32_t *__restrict__ ids, uint8_t *__restrict__ codes,
                                                  uint8_t *__restrict__ lam, int32_t *__restrict__ long_lists,
                                                  int32_t *__restrict__ n_long, int max_long)
{
    extern __shared__ unsigned char smem[];
    uint64_t *keys = (uint64_t *)smem;            // [SORT_MAX]
    uint8_t *pay = (uint8_t *)(keys + SORT_MAX);  // [SORT_MAX * (m + 1)]
    __shared__ int unsorted;
    const int tid = threadIdx.x;
    const int64_t l = blockIdx.x;
    const int64_t beg = off[l];
    const int64_t len = off[l + 1] - beg;
    if (len <= 1) return;
    if (tid == 0) unsorted = 0;
    __syncthreads();
    for (int64_t i = tid; i + 1 < len; i += 64)
        if (ids[beg + i] > ids[beg + i + 1]) unsorted = 1;
    __syncthreads();
    if (!unsorted) return;
    if (len > SORT_MAX) {
        if (tid == 0) {
            const int p = atomicAdd(n_long, 1);
            if (p < max_long) long_lists[p] = (int32_t)l;
        }
        return;
    }
    const int sz = next_pow2_dev((int)len);
    for (int i = tid; i < sz; i += 64)
        keys[i] = i < len ? (((uint64_t)(uint32_t)ids[beg + i] << 32) | (uint32_t)i) : KEY_MAX;
    for (int64_t i = tid; i < len * m; i += 64) pay[i] = codes[beg * m + i];
    for (int i = tid; i < len; i += 64) pay[len * m + i] = lam[beg + i];
    __syncthreads();
    block_bitonic_sort<64>(keys, sz, tid);
    for (int i = tid; i < len; i += 64) {
        const uint64_t key = keys[i];
        const int src = (int)(uint32_t)key;
        ids[beg + i] = (int32_t)(uint32_t)(key >> 32);
        lam[beg + i] = pay[len * m + src];
        for (int p = 0; p < m; ++p) codes[(beg + i) * m + p] = pay[src * m + p];
    }
}
void launch_list_sort(const int64_t *off, int64_t nl, int m, int32_t *ids, uint8_t *codes, uint8_t *lam,
                      int32_t *long_lists, int32_t *n_long, int max_long, hipStream_t st)
{
    if (nl <= 0) return;
    const size_t smem = (size_t)SORT_MAX * 8 + (size_t)SORT_MAX * (m + 1);
    (void)hipFuncSetAttribute((const void *)k_list_sort, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    hipLaunchKernelGGL(k_list_sort, dim3((unsigned)nl), dim3(64), smem, st, off, nl, m, ids, codes, lam, long_lists,
                       n_long, max_long);
}

// Second tier: the lists the 64-thread pass reported (more than SORT_MAX points), one
// 256-thread workgroup each, keys and payload in up to 150 KB of LDS.  Lists beyond mid_max
// points are passed on to the third tier.
__global__ __launch_bounds__(256) void k_list_sort_mid(const int64_t *__restrict__ off, int m, int mid_max,
                                                       const int32_t *__restrict__ in_lists, int n_in,
                                                       int32_t *__restrict__ ids, uint8_t *__restrict__ codes,
                                                       uint8_t *__restrict__ lam, int32_t *__restrict__ out_lists,
                                                       int32_t *__restrict__ n_out, int max_out)
{
    extern __shared__ unsigned char smem[];
    uint64_t *keys = (uint64_t *)smem;           // [mid_max]
    uint8_t *pay = (uint8_t *)(keys + mid_max);  // [mid_max * (m + 1)]
    const int tid = threadIdx.x;
    if ((int)blockIdx.x >= n_in) return;
    const int64_t l = in_lists[blockIdx.x];
    const int64_t beg = off[l];
    const int64_t len = off[l + 1] - beg;
    if (len > mid_max) {
        if (tid == 0) {
            const int p = atomicAdd(n_out, 1);
            if (p < max_out) out_lists[p] = (int32_t)l;
        }
        return;
    }
    const int sz = next_pow2_dev((int)len);
    for (int i = tid; i < sz; i += 256)
        keys[i] = i < len ? (((uint64_t)(uint32_t)ids[beg + i] << 32) | (uint32_t)i) : KEY_MAX;
    for (int64_t i = tid; i < len * m; i += 256) pay[i] = codes[beg * m + i];
    for (int i = tid; i < len; i += 256) pay[len * m + i] = lam[beg + i];
    __syncthreads();
    block_bitonic_sort<256>(keys, sz, tid);
    for (int i = tid; i < len; i += 256) {
        const uint64_t key = keys[i];
        const int src = (int)(uint32_t)key;
        ids[beg + i] = (int32_t)(uint32_t)(key >> 32);
        lam[beg + i] = pay[len * m + src];
        for (int p = 0; p < m; ++p) codes[(beg + i) * m + p] = pay[src * m + p];
    }
}

int list_sort_mid_max(int m)
{
    // keys (8 B) + payload (m + 1 B) per point within 150 KB, as a power of two, at least 2 * SORT_MAX
    int mm = 8192;
    while (mm > 2 * SORT_MAX && (size_t)mm * (8 + m + 1) > 150 * 1024) mm >>= 1;
    return (size_t)mm * (8 + m + 1) <= 150 * 1024 ? mm : 0;
}

void launch_list_sort_mid(const int64_t *off, int m, const int32_t *in_lists, int n_in, int32_t *ids, uint8_t *codes,
                          uint8_t *lam, int32_t *out_lists, int32_t *n_out, int max_out, hipStream_t st)
{
    const int mm = list_sort_mid_max(m);
    if (n_in <= 0 || mm == 0) return;
    const size_t smem = (size_t)mm * (8 + m + 1);
    (void)hipFuncSetAttribute((const void *)k_list_sort_mid, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    hipLaunchKernelGGL(k_list_sort_mid, dim3((unsigned)n_in), dim3(256), smem, st, off, m, mm, in_lists, n_in, ids,
                       codes, lam, out_lists, n_out, max_out);
}

// A list too long for LDS: bitonic sort of (id, position) keys in global memory
// by a single workgroup, then the payload is permuted through a scratch copy.
__global__ __launch_bounds__(1024) void k_long_list_sort(int64_t beg, int64_t len, int64_t sz, int m,
                                                         int32_t *__restrict__ ids, uint8_t *__restrict__ codes,
                                                         uint8_t *__restrict__ lam, uint64_t *__restrict__ keys,
                                                         uint8_t *__restrict__ pay)
{
    const int tid = threadIdx.x;
    for (int64_t i = tid; i < sz; i += 1024)
        keys[i] = i < len ? (((uint64_t)(uint32_t)ids[beg + i] << 32) | (uint32_t)i) : KEY_MAX;
    for (int64_t i = tid; i < len * m; i += 1024) pay[i] = codes[beg * m + i];
    for (int64_t i = tid; i < len; i += 1024) pay[len * m + i] = lam[beg + i];
    __syncthreads();
    for (int64_t k = 2; k <= sz; k <<= 1)
        for (int64_t j = k >> 1; j > 0; j >>= 1) {
            for (int64_t i = tid; i < (sz >> 1); i += 1024) {
                const int64_t lo = ((i & ~(j - 1)) << 1) | (i & (j - 1)), hi = lo | j;
                const uint64_t x = keys[lo], y = keys[hi];
                if ((x > y) == ((lo & k) == 0)) {
                    keys[lo] = y;
                    keys[hi] = x;
                }
            }
            __syncthreads();
        }
    for (int64_t i = tid; i < len; i += 1024) {
        const uint64_t key = keys[i];
        const int64_t src = (int64_t)(uint32_t)key;
        ids[beg + i] = (int32_t)(uint32_t)(key >> 32);
        lam[beg + i] = pay[len * m + src];
        for (int p = 0; p < m; ++p) codes[(beg + i) * m + p] = pay[src * m + p];
    }
}
void launch_long_list_sort_at(int64_t beg, int64_t len, int m, int32_t *ids, uint8_t *codes, uint8_t *lam,
                              uint64_t *scratch_keys, uint8_t *scratch_payload, hipStream_t st)
{
    int64_t sz = 1;
    while (sz < len) sz <<= 1;
    hipLaunchKernelGGL(k_long_list_sort, dim3(1), dim3(1024), 0, st, beg, len, sz, m, ids, codes, lam, scratch_keys,
                       scratch_payload);
}

// Query-independent part of the ADC distance of every stored point (Eq. 15-17):
//   s_x = ||q2||^2 + 2 <q1 - mu, q2> + (l^2 - l) c,  q1 = c_i + l (s_ij - c_i),  q2 = codewords of x,
// i.e. term2 + 2 (1-l) term3 + 2 l term4 + (l^2 - l) term7 of Eq. 16-17 summed per point, with the
// inner products taken relative to a fixed vector mu (the scan's table is 2 <y - mu, q2>, so mu drops
// out of the distance; what it removes is the part of both inner products that grows with the
// distance of the data from the origin and would cancel between them in fp32).
// Summed in fp64 and rounded once.  One 64-thread workgroup per list: the edge length c is formed
// by the whole wave, then lanes stride over the points, every lane walking the D coordinates of its
// point (centroid rows come from L1/L2, the same for all lanes).
__global__ __launch_bounds__(64) void k_list_static(const int64_t *__restrict__ off, int n, int D, int m,
                                                    const float *__restrict__ C, const int32_t *__restrict__ S,
                                                    const float *__restrict__ P, const float *__restrict__ mu,
                                                    const uint8_t *__restrict__ codes,
                                                    const uint8_t *__restrict__ lam, double lam_step, float lam_zero,
                                                    float *__restrict__ sx)
{
    const int64_t l = blockIdx.x;
    const int64_t beg = off[l], end = off[l + 1];
    if (beg == end) return;
    const int i = (int)(l / n);
    const float *ci = C + (int64_t)i * D;
    const float *sj = C + (int64_t)S[l] * D;
    double c = 0.0;
    for (int d = threadIdx.x; d < D; d += 64) {
        const double e = (double)sj[d] - (double)ci[d];
        c = fma(e, e, c);
    }
    c = wave_sum_f64(c);
    const int ds = D / m;
    for (int64_t t = beg + threadIdx.x; t < end; t += 64) {
        const double lh = ((double)lam[t] - (double)lam_zero) * lam_step;
        double q2n = 0.0, q12 = 0.0;
        for (int p = 0; p < m; ++p) {
            const float *w = P + ((int64_t)p * 256 + codes[t * m + p]) * ds;
            for (int d = 0; d < ds; ++d) {
                const int g = p * ds + d;
                const double cv = (double)ci[g], wv = (double)w[d];
                const double q1 = (cv - (double)mu[g]) + lh * ((double)sj[g] - cv);
                q2n = fma(wv, wv, q2n);
                q12 = fma(q1, wv, q12);
            }
        }
        sx[t] = (float)(q2n + 2.0 * q12 + (lh * lh - lh) * c);
    }
}
void launch_list_static(const int64_t *off, int64_t nl, int n, int D, int m, const float *C, const int32_t *S,
                        const float *P, const float *mu, const uint8_t *codes, const uint8_t *lam, double lam_step,
                        float lam_zero, float *sx, hipStream_t st)
{
    if (nl <= 0) return;
    hipLaunchKernelGGL(k_list_static, dim3((unsigned)nl), dim3(64), 0, st, off, n, D, m, C, S, P, mu, codes, lam,
                       lam_step, lam_zero, sx);
}
