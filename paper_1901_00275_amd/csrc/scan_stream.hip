// Streaming list scan with fused K-selection (Sec. 3.3.2 - 3.3.3): the fast path.
//
// Eq. 15 splits the ADC distance ||y - q1 - q2||^2 (Eq. 14) into
//     ||y - q1||^2  +  ||q2||^2 + 2 <q1, q2>  -  2 <y, q2>
// and Eq. 17 writes the first part with the coarse distances a = ||y - c_i||^2,
// b = ||y - s_ij||^2 and the edge length c:  (1-l) a + l b + (l^2 - l) c.
// Everything that does not depend on the query,
//     s_x = ||q2||^2 + 2 <q1 - mu, q2> + (l^2 - l) c     (term2 + term3/4 + the term7 part),
// is summed once per point when the lists are built and streamed with the code,
// so that a query needs ONE lookup table for the whole scan,
//     T[p][t] = 2 <(y - mu)^p, P[p][t]>                    (term5, 256 D multiply-adds),
// and per point m table reads:
//     dist = s_x + a + l (b - a) - sum_p T[p][t_p].
// mu is one vector fixed per index (the mean of the centroids); it cancels between s_x and T and
// keeps both inner products, and with them the rounding error of the sum, independent of where
// the data lie relative to the origin.
// a and b come from the traversal kernels (term6 / term8 are by-products of the
// region traversal), so the scan itself touches no centroid.
//
// Streams per point: m code bytes, 1 lambda byte, 4 bytes s_x.  Vector ids are
// not streamed: candidates are tracked by their position in the list arrays and
// ids are looked up for the K survivors only (the paper keeps ids off the scan
// path in the same way, Sec. 4).
//
// Work layout: one workgroup of 512 threads (8 waves) per (query, split).  The
// table lives in LDS.  Waves take whole lists from a shared counter; a wave
// issues all loads of up to 8 chunks of 64 points before it consumes the first,
// and enough waves are resident per compute unit to cover the memory latency.
// K-selection: every wave keeps its own sorted K-best list and a candidate
// buffer in LDS and merges them alone; the waves share one monotonically
// decreasing upper bound of the K-th best key; the eight lists are merged once
// at the end, ids are resolved and the result is ordered by (distance, id).
#include "common.h"

#define SS_NT 512
#define SS_NW 8
#define SS_CH 8      // chunks of 64 points loaded ahead per wave
#define SS_KP 128    // per-wave sorted list (K <= 128)
#define SS_WSZ 256   // per-wave keys: list + candidate buffer
#define SS_GL 16     // packed form: lists taken at a time
#define SS_PCH 4     // packed form: chunks loaded ahead

typedef __attribute__((address_space(3))) unsigned long long lds_u64;
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

// Wave-private merge of the candidate buffer wk[SS_KP .. SS_WSZ) (unsorted, padded with KEY_MAX) into
// the sorted list wk[0 .. SS_KP): the candidates are sorted in descending order, which makes the whole
// array one bitonic sequence; a single compare-exchange stage against the list leaves the SS_KP
// smallest keys (still bitonic) in the list's place, and a bitonic merge orders them.  About half
// the LDS traffic of sorting all SS_WSZ keys.  (LDS operations of one wave complete in issue
// order, so no workgroup barrier is needed.)
// bitonic sequence of SS_KP keys -> ascending (one wave, one comparator per lane and stage)
__device__ __forceinline__ void wave_bitonic_merge(volatile lds_u64 *wk, int lane)
{
    for (int j = SS_KP >> 1; j > 0; j >>= 1) {
        const int l = ((lane & ~(j - 1)) << 1) | (lane & (j - 1));
        const int r = l | j;
        const uint64_t x = wk[l], y = wk[r];
        if (x > y) {
            wk[l] = y;
            wk[r] = x;
        }
        __builtin_amdgcn_wave_barrier();
    }
}

__device__ __forceinline__ void wave_merge_candidates(volatile lds_u64 *wk, int lane)
{
    static_assert(SS_KP == 128 && SS_WSZ == 256, "one comparator per lane and stage");
    volatile lds_u64 *c = wk + SS_KP;
    for (int k = 2; k <= SS_KP; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            const int l = ((lane & ~(j - 1)) << 1) | (lane & (j - 1));
            const int r = l | j;
            const uint64_t x = c[l], y = c[r];
            if ((x < y) == ((l & k) == 0)) { // descending
                c[l] = y;
                c[r] = x;
            }
            __builtin_amdgcn_wave_barrier();
        }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int i = lane + 64 * h;
        const uint64_t x = wk[i], y = c[i];
        if (y < x) wk[i] = y;
    }
    __builtin_amdgcn_wave_barrier();
    wave_bitonic_merge(wk, lane);
}

// Two sorted lists a, b of SS_KP keys each -> the SS_KP smallest of both, sorted, in a (one wave).
__device__ __forceinline__ void wave_merge_lists(volatile lds_u64 *a, volatile lds_u64 *b, int lane)
{
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int i = lane + 64 * h;
        const uint64_t x = a[i], y = b[SS_KP - 1 - i];
        if (y < x) a[i] = y;
    }
    __builtin_amdgcn_wave_barrier();
    wave_bitonic_merge(a, lane);
}

// PACKED: the lists are short (a few tens of points): a wave takes SS_GL lists at a time and lays
// their points end to end over its lanes, so that a chunk of 64 lanes holds several lists; each
// lane finds its list from the running lengths and carries its own a, b - a.
template <int M, bool PACKED>
__global__ __launch_bounds__(SS_NT, 4) void k_scan_stream(ScanArgs a, const uint4 *__restrict__ desc)
{
    // all LDS is static: the table sits at a fixed address, which folds into the lookups' offsets
    __shared__ float T[M * 256];
    __shared__ uint64_t keys[SS_NW * SS_WSZ];
    __shared__ float yv[VLQ_MAX_DIM];
    __shared__ unsigned long long sh_thr;              // upper bound of the K-th smallest key of the workgroup
    __shared__ unsigned long long sh_q[SS_NW];         // every wave's ceil(K/8)-th key
    __shared__ int sh_next;                            // next list to hand out

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = blockIdx.x / a.nsplit, split = blockIdx.x - q * a.nsplit;
    const int r0 = (int)((int64_t)a.w2 * split / a.nsplit), r1 = (int)((int64_t)a.w2 * (split + 1) / a.nsplit);
    const int K = a.K, D = a.D, ds = D / M;
    const int KQ = (K + SS_NW - 1) / SS_NW;
    volatile lds_u64 *wk = (volatile lds_u64 *)(keys + wave * SS_WSZ);
    int wcnt = 0;

    for (int d = tid; d < D; d += SS_NT) yv[d] = a.Q[(int64_t)q * D + d] - a.mu[d];
    for (int i = lane; i < SS_WSZ; i += 64) wk[i] = KEY_MAX;
    if (tid == 0) {
        sh_thr = KEY_MAX;
        sh_next = r0;
    }
    if (tid < SS_NW) sh_q[tid] = KEY_MAX;
    __syncthreads();
    // the query's table: T[p][t] = 2 <(y - mu)^p, P[p][t]>
    for (int idx = tid; idx < M * 256; idx += SS_NT) {
        const float *w = a.P + (int64_t)idx * ds;
        const float *yp = yv + (idx >> 8) * ds;
        float s = 0.f;
        for (int d = 0; d < ds; ++d) s = fmaf(yp[d], w[d], s);
        T[idx] = 2.f * s;
    }
    __syncthreads();

    // Merge of this wave's candidates into its sorted list.  Publishes two upper bounds of
    // the K-th smallest key of the whole workgroup: the wave's own K-th key, and the largest
    // of all waves' ceil(K/8)-th keys (8 * ceil(K/8) >= K keys lie at or below it).
    auto merge_wave = [&]() {
        for (int i = SS_KP + wcnt + lane; i < SS_WSZ; i += 64) wk[i] = KEY_MAX;
        __builtin_amdgcn_wave_barrier();
        wave_merge_candidates(wk, lane);
        for (int i = K + lane; i < SS_KP; i += 64) wk[i] = KEY_MAX;
        __builtin_amdgcn_wave_barrier();
        wcnt = 0;
        if (lane == 0) sh_q[wave] = wk[KQ - 1];
        __builtin_amdgcn_wave_barrier();
        uint64_t bound = 0;
#pragma unroll
        for (int w = 0; w < SS_NW; ++w) {
            const uint64_t t = ((volatile lds_u64 *)sh_q)[w];
            bound = t > bound ? t : bound;
        }
        const uint64_t own = wk[K - 1];
        bound = own < bound ? own : bound;
        if (lane == 0 && bound != KEY_MAX) atomicMin(&sh_thr, (unsigned long long)bound);
        __builtin_amdgcn_wave_barrier();
    };

    uint64_t thr = KEY_MAX;
    float thr_f = INFINITY;
    // one chunk of 64 points: m table reads per point, the distance, and the candidates that pass
    auto score_chunk = [&](const uint32_t (&cw)[M / 4], uint32_t lbv, float sxv, float av, float bav, uint32_t gpos,
                           bool live) __attribute__((always_inline)) {
        float ts = 0.f;
#pragma unroll
        for (int x = 0; x < M / 4; ++x)
#pragma unroll
            for (int bb = 0; bb < 4; ++bb) {
                const uint32_t byte_off = ((cw[x] >> (8 * bb)) & 255u) << 2;
                ts += *(const float *)((const char *)(T + (x * 4 + bb) * 256) + byte_off);
            }
        const float l = ((float)lbv - a.lam_zero) * a.lam_step;
        const float dist = (sxv - ts) + fmaf(l, bav, av);
        // cheap test on the distance alone; the exact (distance, position) key only for the few that pass
        bool pass = live && dist <= thr_f;
        uint64_t mask = __ballot(pass);
        if (mask) {
            const uint64_t key = make_key(dist, gpos);
            pass = pass && key < thr;
            mask = __ballot(pass);
            int np = __popcll(mask);
            if (np && wcnt + np > SS_WSZ - SS_KP) {
                merge_wave();
                thr = sh_thr;
                thr_f = thr == KEY_MAX ? INFINITY : ord2f((uint32_t)(thr >> 32));
                pass = pass && key < thr;
                mask = __ballot(pass);
                np = __popcll(mask);
            }
            if (pass) wk[SS_KP + wcnt + __popcll(mask & ((1ull << lane) - 1ull))] = key;
            wcnt += np;
        }
    };
    if (PACKED) {
        // up to SS_GL lists per turn, fewer when the workgroup has few lists, so that all waves get some
        int gl = (r1 - r0) / SS_NW;
        gl = gl < 1 ? 1 : (gl > SS_GL ? SS_GL : gl);
        for (;;) {
            int s = 0;
            if (lane == 0) s = atomicAdd(&sh_next, gl);
            s = __builtin_amdgcn_readfirstlane(s);
            if (s >= r1) break;
            // lane i < gl holds the descriptor of list s + i
            uint4 dsc = make_uint4(0u, 0u, 0u, 0u);
            if (lane < gl && s + lane < r1) dsc = desc[(int64_t)q * a.w2 + s + lane];
            const int len = max((int)dsc.y, 0);
            int end = len; // inclusive prefix sum: where the list ends in the concatenation
#pragma unroll
            for (int o = 1; o < SS_GL; o <<= 1) {
                const int t = __shfl_up(end, o, 64);
                if (lane >= o) end += t;
            }
            const int start = end - len;
            const int total = __builtin_amdgcn_readlane(end, SS_GL - 1);
            if (total <= 0) continue;
            int ends[SS_GL]; // uniform copies
#pragma unroll
            for (int i = 0; i < SS_GL; ++i) ends[i] = __builtin_amdgcn_readlane(end, i);
            thr = sh_thr;
            thr_f = thr == KEY_MAX ? INFINITY : ord2f((uint32_t)(thr >> 32));
            for (int base = 0; base < total; base += 64 * SS_PCH) {
                uint32_t cw[SS_PCH][M / 4];
                uint32_t lb[SS_PCH], gp[SS_PCH];
                float sv[SS_PCH], fav[SS_PCH], fbav[SS_PCH];
#pragma unroll
                for (int u = 0; u < SS_PCH; ++u) {
                    if (base + 64 * u < total) { // uniform over the wave
                        const int p = min(base + 64 * u + lane, total - 1); // idle lanes repeat the last point
                        int j = 0; // the list that holds position p: the lists before it end at or before p
#pragma unroll
                        for (int i = 0; i < SS_GL - 1; ++i) j += ends[i] <= p;
                        const uint32_t g = (uint32_t)__shfl((int)dsc.x, j, 64) + (uint32_t)(p - __shfl(start, j, 64));
                        fav[u] = __uint_as_float((uint32_t)__shfl((int)dsc.z, j, 64));
                        fbav[u] = __uint_as_float((uint32_t)__shfl((int)dsc.w, j, 64));
                        gp[u] = g;
                        const uint32_t *cp = (const uint32_t *)(a.codes + (size_t)g * M);
                        if (M == 8) {
                            const u32x2_t c2 = *(const u32x2_t *)cp;
                            cw[u][0] = c2.x;
                            cw[u][1] = c2.y;
                        } else {
                            const u32x4_t c4 = *(const u32x4_t *)cp;
#pragma unroll
                            for (int x = 0; x < M / 4; ++x) cw[u][x] = c4[x];
                        }
                        lb[u] = a.lam[g];
                        sv[u] = a.sx[g];
                    }
                }
#pragma unroll
                for (int u = 0; u < SS_PCH; ++u)
                    if (base + 64 * u < total)
                        score_chunk(cw[u], lb[u], sv[u], fav[u], fbav[u], gp[u], base + 64 * u + lane < total);
            }
        }
    } else {
    for (;;) {
        int s = 0;
        if (lane == 0) s = atomicAdd(&sh_next, 1);
        s = __builtin_amdgcn_readfirstlane(s);
        if (s >= r1) break;
        const uint4 dsc = desc[(int64_t)q * a.w2 + s]; // uniform address: scalar load
        const uint32_t beg = dsc.x;
        const int len = (int)dsc.y;
        const float av = __uint_as_float(dsc.z), bav = __uint_as_float(dsc.w);
        if (len <= 0) continue;
        // range-checked raw buffers over the three streams of this list: reads past the end
        // return zero and are masked out, so the chunk loop needs no address arithmetic
        const __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc((void *)(a.codes + (int64_t)beg * M), 0, len * M, 0x00020000);
        const __amdgpu_buffer_rsrc_t rl = __builtin_amdgcn_make_buffer_rsrc((void *)(a.lam + beg), 0, len, 0x00020000);
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)(a.sx + beg), 0, len * 4, 0x00020000);
        thr = sh_thr;
        thr_f = thr == KEY_MAX ? INFINITY : ord2f((uint32_t)(thr >> 32));
        for (int base = 0; base < len; base += 64 * SS_CH) {
            // ---- all loads of up to SS_CH chunks ----
            uint32_t cw[SS_CH][M / 4];
            uint32_t lb[SS_CH];
            float sv[SS_CH];
#pragma unroll
            for (int u = 0; u < SS_CH; ++u) {
                if (base + 64 * u < len) { // uniform over the wave
                    const int so = base + 64 * u;
                    if (M == 8) {
                        const u32x2_t c2 = __builtin_bit_cast(u32x2_t, __builtin_amdgcn_raw_buffer_load_b64(rc, lane * 8, so * 8, 0));
                        cw[u][0] = c2.x;
                        cw[u][1] = c2.y;
                    } else {
                        const u32x4_t c4 = __builtin_bit_cast(u32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rc, lane * 16, so * 16, 0));
#pragma unroll
                        for (int x = 0; x < M / 4; ++x) cw[u][x] = c4[x];
                    }
                    lb[u] = __builtin_amdgcn_raw_buffer_load_b8(rl, lane, so, 0);
                    sv[u] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, lane * 4, so * 4, 0));
                }
            }
            // ---- score ----
#pragma unroll
            for (int u = 0; u < SS_CH; ++u)
                if (base + 64 * u < len) {
                    const int within = base + 64 * u + lane;
                    score_chunk(cw[u], lb[u], sv[u], av, bav, beg + (uint32_t)within, within < len);
                }
        }
    }
    }

    // ---- merge the eight wave lists; resolve ids; order by (distance, id) ----
    // Every wave's list is sorted: a tree of three rounds merges them pairwise, each merge keeping
    // the SS_KP smallest keys of its two lists (one wave per merge, no sorting).
    merge_wave();
    const int KP = next_pow2_dev(K);
#pragma unroll
    for (int step = SS_NW / 2; step >= 1; step >>= 1) {
        __syncthreads();
        if (wave < step) wave_merge_lists(wk, (volatile lds_u64 *)(keys + (wave + step) * SS_WSZ), lane);
    }
    __syncthreads();
    // The first wave resolves the ids of the K survivors and orders them by (distance, id): the list is
    // in (distance, position) order, so only keys of equal distance can move (a wave-private sort).
    if (wave != 0) return;
    {
        uint64_t mine[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int i = lane + 64 * h;
            const uint64_t key = i < K ? wk[i] : KEY_MAX;
            mine[h] = key != KEY_MAX ? ((key & 0xFFFFFFFF00000000ull) | (uint32_t)a.ids[(uint32_t)key]) : KEY_MAX;
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) wk[lane + 64 * h] = mine[h];
        __builtin_amdgcn_wave_barrier();
        for (int k = 2; k <= KP; k <<= 1)
            for (int j = k >> 1; j > 0; j >>= 1) {
                const int l = ((lane & ~(j - 1)) << 1) | (lane & (j - 1));
                const int r = l | j;
                if (r < KP) {
                    const uint64_t x = wk[l], y = wk[r];
                    if ((x > y) == ((l & k) == 0)) {
                        wk[l] = y;
                        wk[r] = x;
                    }
                }
                __builtin_amdgcn_wave_barrier();
            }
    }
    if (a.nsplit > 1) {
        uint64_t *dst = a.partial + ((int64_t)q * a.nsplit + split) * K;
        for (int i = lane; i < K; i += 64) dst[i] = wk[i];
    } else {
        for (int i = lane; i < K; i += 64) {
            const uint64_t key = wk[i];
            const bool ok = key != KEY_MAX;
            a.out_dist[(int64_t)q * K + i] = ok ? ord2f((uint32_t)(key >> 32)) : INFINITY;
            a.out_ids[(int64_t)q * K + i] = ok ? (int32_t)(uint32_t)key : -1;
        }
    }
}


// Shapes served by this kernel; everything else takes the generic kernel.
bool scan_stream_supported(const ScanArgs &a)
{
    return (a.m == 8 || a.m == 16) && a.K <= SS_KP && a.sx != nullptr && a.mu != nullptr && a.desc != nullptr &&
           (((uintptr_t)a.codes) % 16 == 0);
}

void launch_scan_stream(const ScanArgs &a, hipStream_t st)
{
    if (a.nq <= 0) return;
    const dim3 grid((unsigned)(a.nq * a.nsplit));
    const uint4 *desc = (const uint4 *)a.desc;
    if (a.m == 8) {
        if (a.packed)
            hipLaunchKernelGGL((k_scan_stream<8, true>), grid, dim3(SS_NT), 0, st, a, desc);
        else
            hipLaunchKernelGGL((k_scan_stream<8, false>), grid, dim3(SS_NT), 0, st, a, desc);
    } else {
        if (a.packed)
            hipLaunchKernelGGL((k_scan_stream<16, true>), grid, dim3(SS_NT), 0, st, a, desc);
        else
            hipLaunchKernelGGL((k_scan_stream<16, false>), grid, dim3(SS_NT), 0, st, a, desc);
    }
}
