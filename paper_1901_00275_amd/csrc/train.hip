// Lloyd iterations (k-means) for the codebooks of Sec. 2.1 / Sec. 3.1: the update half.
// The assignment half is the nearest-centroid search of the encoder (coarse_bf16.hip /
// coarse.hip + k_encode_finish in nearest-only mode).
//
// Member sums are accumulated in 64-bit fixed point, so the result does not depend on the
// order in which the atomics land: x is scaled by 2^shift / s, s = the smallest power of two
// >= max |x| over the sample, shift = 62 - ceil(log2(points)); the sum of all members cannot
// overflow and the resolution is s * 2^-shift (2^-38 s for 16 M points).
#include "common.h"

__global__ __launch_bounds__(256) void k_absmax(const float *__restrict__ X, int64_t count, uint32_t *__restrict__ out)
{
    uint32_t m = 0;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += stride) {
        const uint32_t u = __float_as_uint(X[i]) & 0x7FFFFFFFu;
        if (u < 0x7F800000u) m = max(m, u); // finite values only
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, o, 64));
    if ((threadIdx.x & 63) == 0) atomicMax(out, m);
}

void launch_absmax(const float *X, int64_t count, uint32_t *out_bits, hipStream_t st)
{
    if (count <= 0) return;
    int64_t blocks = (count + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_absmax, dim3((unsigned)blocks), dim3(256), 0, st, X, count, out_bits);
}

// power of two >= the largest magnitude (1 for an all-zero sample)
__device__ __forceinline__ double scale_of(uint32_t absmax_bits)
{
    const float m = __uint_as_float(absmax_bits);
    if (!(m > 0.f)) return 1.0;
    int e;
    frexpf(m, &e); // m = f * 2^e, 0.5 <= f < 1
    return ldexp(1.0, e);
}

// one thread per (vector, dimension)
__global__ __launch_bounds__(256) void k_kmeans_accumulate(const float *__restrict__ X, int64_t nb, int D,
                                                           const int32_t *__restrict__ assign,
                                                           const uint32_t *__restrict__ absmax_bits, int shift,
                                                           long long *__restrict__ sums, int32_t *__restrict__ cnt)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= nb * D) return;
    const int64_t row = i / D;
    const int d = (int)(i - row * D);
    const int c = assign[row];
    if (c < 0) return;
    const double f = ldexp(1.0, shift) / scale_of(*absmax_bits);
    const float x = X[i];
    if (__float_as_uint(x) << 1 < 0xFF000000u) // finite
        atomicAdd((unsigned long long *)&sums[(int64_t)c * D + d], (unsigned long long)llrint((double)x * f));
    if (d == 0) atomicAdd(&cnt[c], 1);
}

void launch_kmeans_accumulate(const float *X, int64_t nb, int D, const int32_t *assign, const uint32_t *absmax_bits,
                              int shift, long long *sums, int32_t *cnt, hipStream_t st)
{
    const int64_t n = nb * D;
    if (n <= 0) return;
    hipLaunchKernelGGL(k_kmeans_accumulate, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, X, nb, D, assign,
                       absmax_bits, shift, sums, cnt);
}

// a centroid with members moves to their mean; one without stays
__global__ __launch_bounds__(256) void k_kmeans_update(float *__restrict__ C, int k, int D,
                                                       const long long *__restrict__ sums,
                                                       const int32_t *__restrict__ cnt,
                                                       const uint32_t *__restrict__ absmax_bits, int shift)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)k * D) return;
    const int c = (int)(i / D);
    const int n = cnt[c];
    if (n <= 0) return;
    const double inv = scale_of(*absmax_bits) / ldexp(1.0, shift);
    C[i] = (float)((double)sums[i] * inv / (double)n);
}

void launch_kmeans_update(float *C, int k, int D, const long long *sums, const int32_t *cnt,
                          const uint32_t *absmax_bits, int shift, hipStream_t st)
{
    const int64_t n = (int64_t)k * D;
    hipLaunchKernelGGL(k_kmeans_update, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, C, k, D, sums, cnt,
                       absmax_bits, shift);
}
