// Validation and preparation kernels: unpack codes, reconstruct W_F, feedback quantizer.
// None of these is on the inference hot path; they are written for clarity, one thread per element.
#include <hip/hip_fp16.h>

#include "fbq_internal.h"

namespace fbq {

typedef _Float16 half_t;

// Code k of a packed row, assembled field by field from the device layout.
__device__ __forceinline__ uint32_t code_of_row(const uint32_t *row, int bits, int k)
{
    if (bits == 4) return (row[k >> 3] >> ((k & 7) * 4)) & 15u;
    const uint32_t *u = row + (k >> 5) * 3;
    const int j = k & 31;
    if (j == 30) return ((u[0] >> 15) & 1u) | (((u[1] >> 15) & 1u) << 1) | (((u[2] >> 15) & 1u) << 2);
    if (j == 31) return (u[0] >> 31) | ((u[1] >> 31) << 1) | ((u[2] >> 31) << 2);
    const int wd = j / 10, f = j % 10;
    const int sh = f < 5 ? 3 * f : 16 + 3 * (f - 5);
    return (u[wd] >> sh) & 7u;
}

__global__ __launch_bounds__(256) void fbq_unpack_kernel(const uint32_t *__restrict__ qw, uint8_t *__restrict__ codes,
                                                         int N, int K, int bits, int row_words)
{
    const int n = blockIdx.y;
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (n < N && k < K) codes[(size_t)n * K + k] = (uint8_t)code_of_row(qw + (size_t)n * row_words, bits, k);
}

hipError_t launch_unpack(const fbq_desc &d, const uint32_t *qw, uint8_t *codes, hipStream_t stream)
{
    hipLaunchKernelGGL(fbq_unpack_kernel, dim3(ceil_div(d.K, 256), d.N), dim3(256), 0, stream, qw, codes, d.N, d.K, d.bits,
                       (int)row_words(d.K, d.bits));
    return hipGetLastError();
}

// W_F[n,k] = s*(q - z) + sum_j At[j,k] * Bt[n,j]   (Sec. 4.1: W_F = Q(W - Sigma) + Sigma), fp32.
__global__ __launch_bounds__(256) void fbq_reconstruct_kernel(const uint32_t *__restrict__ qw, const uint16_t *__restrict__ scales,
                                                              const uint16_t *__restrict__ zeros, const uint16_t *__restrict__ At,
                                                              const uint16_t *__restrict__ Bt, float *__restrict__ W_hat, int N,
                                                              int K, int r, int bits, int row_words)
{
    const int n = blockIdx.y;
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (n >= N || k >= K) return;
    const int G = K / kGroup;
    const float s = (float)__builtin_bit_cast(half_t, scales[(size_t)n * G + k / kGroup]);
    const float z = (float)__builtin_bit_cast(half_t, zeros[(size_t)n * G + k / kGroup]);
    const float q = (float)code_of_row(qw + (size_t)n * row_words, bits, k);
    float sigma = 0.0f;
    for (int j = 0; j < r; ++j)
        sigma = fmaf((float)__builtin_bit_cast(half_t, At[(size_t)j * K + k]),
                     (float)__builtin_bit_cast(half_t, Bt[(size_t)n * r + j]), sigma);
    W_hat[(size_t)n * K + k] = s * (q - z) + sigma;
}

hipError_t launch_reconstruct(const fbq_desc &d, const uint32_t *qw, const uint16_t *scales, const uint16_t *zeros,
                              const uint16_t *At, const uint16_t *Bt, float *W_hat, hipStream_t stream)
{
    hipLaunchKernelGGL(fbq_reconstruct_kernel, dim3(ceil_div(d.K, 256), d.N), dim3(256), 0, stream, qw, scales, zeros, At, Bt,
                       W_hat, d.N, d.K, d.r, d.bits, (int)row_words(d.K, d.bits));
    return hipGetLastError();
}

// ------------------------------------------------------------------ feedback quantizer (fp64)

__device__ __forceinline__ double half_bits_to_double(uint16_t h) { return (double)__builtin_bit_cast(half_t, h); }

// double -> fp16 bits, round to nearest even, done on integers so that no intermediate fp32
// rounding can occur.  Input is finite and non-negative here, or negative for the zero point.
__device__ uint16_t double_to_half_bits(double d)
{
    const uint64_t u = __builtin_bit_cast(uint64_t, d);
    const uint16_t sign = (uint16_t)((u >> 48) & 0x8000u);
    const int e = (int)((u >> 52) & 0x7ff) - 1023;           // unbiased exponent
    const uint64_t man = (u & 0xFFFFFFFFFFFFFull) | (1ull << 52);
    if (((u >> 52) & 0x7ff) == 0) return sign;               // zero / fp64 subnormal
    if (e >= 16) return sign | 0x7c00u;                      // overflow (callers never get here with inf/nan)
    if (e < -25) return sign;                                // below half of the smallest subnormal
    // value = man * 2^(e-52).  fp16 keeps bits down to 2^(max(e,-14) - 10).
    const int drop = 52 - 10 + (e < -14 ? -14 - e : 0);      // low bits of man to round away
    uint64_t keep = man >> drop;
    const uint64_t rem = man & ((1ull << drop) - 1), half = 1ull << (drop - 1);
    if (rem > half || (rem == half && (keep & 1))) keep += 1;
    // keep is now in units of the fp16 ulp at this exponent; re-encode (carry handled by addition)
    if (e < -14) return sign | (uint16_t)keep;               // subnormal (or rounds up into the first normal)
    const uint32_t bits = ((uint32_t)(e + 15) << 10) + (uint32_t)(keep - 1024);
    return bits >= 0x7c00u ? (sign | 0x7c00u) : (sign | (uint16_t)bits);
}

// One block of 128 threads per (row, group).  fp64 with no fused multiply-add, so that the result
// does not depend on contraction choices.
__global__ __launch_bounds__(128) void fbq_quantize_kernel(const uint16_t *__restrict__ W, const uint16_t *__restrict__ At,
                                                           const uint16_t *__restrict__ Bt, uint32_t *__restrict__ qw,
                                                           uint16_t *__restrict__ scales, uint16_t *__restrict__ zeros, int N,
                                                           int K, int r, int bits, int row_words)
{
#pragma clang fp contract(off)
    __shared__ double smin[128], smax[128];
    __shared__ uint16_t sz[2];
    __shared__ uint8_t scode[128];
    const int n = blockIdx.y, g = blockIdx.x, i = threadIdx.x;
    const int k = g * kGroup + i;
    const int qmax = (1 << bits) - 1;

    double sigma = 0.0;
    for (int j = 0; j < r; ++j) sigma = sigma + half_bits_to_double(At[(size_t)j * K + k]) * half_bits_to_double(Bt[(size_t)n * r + j]);
    const double R = half_bits_to_double(W[(size_t)n * K + k]) - sigma;       // feedback: quantize W - Sigma

    smin[i] = R;
    smax[i] = R;
    __syncthreads();
    for (int off = 64; off > 0; off >>= 1) {
        if (i < off) {
            smin[i] = fmin(smin[i], smin[i + off]);
            smax[i] = fmax(smax[i], smax[i + off]);
        }
        __syncthreads();
    }
    if (i == 0) {
        const double mn = smin[0], mx = smax[0];
        double s = (mx - mn) / (double)qmax;
        if (!(s > 0.0)) s = 1.0;
        uint16_t s16 = double_to_half_bits(s);
        if (s16 < 0x0400u) s16 = 0x0400u;
        uint16_t z16;
        for (;;) {
            const double sd = half_bits_to_double(s16);
            z16 = double_to_half_bits(-mn / sd);
            const double zd = half_bits_to_double(z16);
            if ((mn / sd + zd >= -0.5 && mx / sd + zd <= (double)qmax + 0.5) || s16 >= 0x7bffu) break;
            s16 += 1;
        }
        sz[0] = s16;
        sz[1] = z16;
        scales[(size_t)n * (K / kGroup) + g] = s16;
        zeros[(size_t)n * (K / kGroup) + g] = z16;
    }
    __syncthreads();
    const double sd = half_bits_to_double(sz[0]), zd = half_bits_to_double(sz[1]);
    double q = rint(R / sd + zd);                                             // ties to even
    q = fmin(fmax(q, 0.0), (double)qmax);
    scode[i] = (uint8_t)q;
    __syncthreads();

    uint32_t *row = qw + (size_t)n * row_words;
    if (bits == 4) {
        if (i < 16) {
            uint32_t w = 0;
            for (int c = 0; c < 8; ++c) w |= (uint32_t)scode[i * 8 + c] << (4 * c);
            row[g * 16 + i] = w;
        }
    } else if (i < 12) {
        const int u = i / 3, wd = i % 3;
        const uint8_t *cu = scode + u * 32;
        uint32_t w = 0;
        for (int f = 0; f < 5; ++f) {
            w |= (uint32_t)cu[wd * 10 + f] << (3 * f);
            w |= (uint32_t)cu[wd * 10 + 5 + f] << (16 + 3 * f);
        }
        w |= ((uint32_t)(cu[30] >> wd) & 1u) << 15;
        w |= ((uint32_t)(cu[31] >> wd) & 1u) << 31;
        row[g * 12 + i] = w;
    }
}

hipError_t launch_quantize(const fbq_desc &d, const uint16_t *W, const uint16_t *At, const uint16_t *Bt, uint32_t *qw,
                           uint16_t *scales, uint16_t *zeros, hipStream_t stream)
{
    hipLaunchKernelGGL(fbq_quantize_kernel, dim3(d.K / kGroup, d.N), dim3(128), 0, stream, W, At, Bt, qw, scales, zeros, d.N,
                       d.K, d.r, d.bits, (int)row_words(d.K, d.bits));
    return hipGetLastError();
}

}  // namespace fbq
