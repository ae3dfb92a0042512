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

// A double from the lane that the data-parallel control word names (quad permutations, row mirrors).
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v)
{
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_mov_dpp((int)(uint32_t)u, CTRL, 0xF, 0xF, true);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_mov_dpp((int)(uint32_t)(u >> 32), CTRL, 0xF, 0xF, true);
    return __builtin_bit_cast(double, (uint64_t)lo | ((uint64_t)hi << 32));
}

// One block of 128 threads per group of 128 input features and kQuantRows consecutive rows: thread i
// keeps column k = 128 g + i of At in registers (32 taps at a time, fetched by the block as a tile) and
// walks over the rows with it, so At is read once per 16 rows and Bt is converted once per block (LDS,
// broadcast reads).  fp64, the
// taps in index order, no contraction left to the compiler; the one fused multiply-add is exact
// by construction: the product of two fp16 values has 22 significant bits and is exact in fp64, so
// fma(a, b, c) and (a * b) + c round the same number.
// With D16 / Dt16 given, the kernel also writes what the reconstruction step needs from the same
// registers: Delta_F = (W - Sigma) - s (q - z), times `gain`, as fp16 in both orientations
// (D16 [N][K]; Dt16 [K][ldt] with columns N..ldt-1 zero).
constexpr int kQuantRows = 16;
constexpr int kQuantTaps = 32;

__global__ __launch_bounds__(128) void fbq_quantize_kernel(const uint16_t *__restrict__ W, const uint16_t *__restrict__ At,
                                                           const uint16_t *__restrict__ Bt, uint32_t *__restrict__ qw,
                                                           uint16_t *__restrict__ scales, uint16_t *__restrict__ zeros, int N,
                                                           int K, int r, int bits, int row_words, uint16_t *__restrict__ D16,
                                                           uint16_t *__restrict__ Dt16, int ldt, float gain)
{
#pragma clang fp contract(off)
    __shared__ double smin[2][kQuantRows], smax[2][kQuantRows];
    __shared__ uint16_t sz[kQuantRows][2];
    __shared__ uint8_t scode[kQuantRows][128];
    __shared__ __align__(16) uint16_t at_tile[kQuantTaps][kGroup];   // the block's tile of At
    __shared__ float bt[kQuantRows][kQuantTaps];      // the block's rows of Bt (fp16 values are exact in fp32; half the LDS bytes of fp64)
    const int g = blockIdx.x, n0 = blockIdx.y * kQuantRows, i = threadIdx.x;
    const int rows = min(kQuantRows, N - n0);
    const int k = g * kGroup + i;
    const int qmax = (1 << bits) - 1;

    double sigma[kQuantRows];
#pragma unroll
    for (int row = 0; row < kQuantRows; ++row) sigma[row] = 0.0;
    for (int j0 = 0; j0 < r; j0 += kQuantTaps) {
        // taps past r enter as zeros (adding 0 * b changes nothing); rows past N repeat the last row and are never stored
        // the 32 x 128 tile of At: 16-byte loads (four per thread) into LDS, from where a thread takes its column
        // (32 two-byte global loads per thread cost the load path eight times the instructions)
        __syncthreads();
#pragma unroll
        for (int pc = 0; pc < kQuantTaps * kGroup / 8 / 128; ++pc) {
            const int piece = pc * 128 + i, jj = piece / (kGroup / 8), k8 = piece % (kGroup / 8);
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (j0 + jj < r) v = *reinterpret_cast<const uint4 *>(At + (size_t)(j0 + jj) * K + g * kGroup + k8 * 8);
            *reinterpret_cast<uint4 *>(&at_tile[jj][k8 * 8]) = v;
        }
        for (int idx = i; idx < kQuantRows * kQuantTaps; idx += 128) {
            const int row = idx / kQuantTaps, jj = idx % kQuantTaps;
            bt[row][jj] = j0 + jj < r ? (float)__builtin_bit_cast(half_t, Bt[(size_t)min(n0 + row, N - 1) * r + j0 + jj]) : 0.0f;
        }
        __syncthreads();
        double at[kQuantTaps];
#pragma unroll
        for (int jj = 0; jj < kQuantTaps; ++jj) at[jj] = half_bits_to_double(at_tile[jj][i]);   // zero past r
#pragma unroll
        for (int row = 0; row < kQuantRows; ++row)
#pragma unroll
            for (int jj = 0; jj < kQuantTaps; ++jj) sigma[row] = __builtin_fma(at[jj], (double)bt[row][jj], sigma[row]);
    }

    // feedback: quantize R = W - Sigma.  Extremes over the group: lanes by shuffles, then the two waves.
    double R[kQuantRows];
#pragma unroll
    for (int row = 0; row < kQuantRows; ++row) {
        R[row] = row < rows ? half_bits_to_double(W[(size_t)(n0 + row) * K + k]) - sigma[row] : 0.0;
        double mn = R[row], mx = R[row];
        // within rows of 16 lanes by data-parallel moves (no LDS traffic), across the four rows by two shuffles
        mn = fmin(mn, dpp_move<0xB1>(mn)); mx = fmax(mx, dpp_move<0xB1>(mx));       // neighbours
        mn = fmin(mn, dpp_move<0x4E>(mn)); mx = fmax(mx, dpp_move<0x4E>(mx));       // pairs of a quad
        mn = fmin(mn, dpp_move<0x141>(mn)); mx = fmax(mx, dpp_move<0x141>(mx));     // quads of a half row (mirror)
        mn = fmin(mn, dpp_move<0x140>(mn)); mx = fmax(mx, dpp_move<0x140>(mx));     // halves of a row (mirror)
        mn = fmin(mn, __shfl_xor(mn, 16, 64)); mx = fmax(mx, __shfl_xor(mx, 16, 64));
        mn = fmin(mn, __shfl_xor(mn, 32, 64)); mx = fmax(mx, __shfl_xor(mx, 32, 64));
        if ((i & 63) == 0) {
            smin[i >> 6][row] = mn;
            smax[i >> 6][row] = mx;
        }
    }
    __syncthreads();
    if (i < rows) {
        const double mn = fmin(smin[0][i], smin[1][i]), mx = fmax(smax[0][i], smax[1][i]);
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
        sz[i][0] = s16;
        sz[i][1] = z16;
        scales[(size_t)(n0 + i) * (K / kGroup) + g] = s16;
        zeros[(size_t)(n0 + i) * (K / kGroup) + g] = z16;
    }
    __syncthreads();
#pragma unroll
    for (int row = 0; row < kQuantRows; ++row) {
        if (row >= rows) continue;
        const double sd = half_bits_to_double(sz[row][0]), zd = half_bits_to_double(sz[row][1]);
        double q = rint(R[row] / sd + zd);                                    // ties to even
        q = fmin(fmax(q, 0.0), (double)qmax);
        scode[row][i] = (uint8_t)q;
        R[row] = R[row] - sd * (q - zd);                                      // Delta_F (Sec. 4.2)
    }
    __syncthreads();
    if (D16) {
        typedef _Float16 half8 __attribute__((ext_vector_type(8)));
        half8 lo, hi;
#pragma unroll
        for (int row = 0; row < kQuantRows; ++row) {
            const half_t v = row < rows ? (half_t)(float)((double)gain * R[row]) : (half_t)0.0f;
            if (row < rows) D16[(size_t)(n0 + row) * K + k] = __builtin_bit_cast(uint16_t, v);
            if (row < 8) lo[row] = v;
            else hi[row - 8] = v;
        }
        half8 *col = reinterpret_cast<half8 *>(Dt16 + (size_t)k * ldt + n0);   // n0 a multiple of 16, ldt of 64
        col[0] = lo;
        col[1] = hi;
        if (n0 + kQuantRows >= N) {                                            // last block of rows: clear the padding
            const half8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
            for (int c = n0 + kQuantRows; c < ldt; c += 8) *reinterpret_cast<half8 *>(Dt16 + (size_t)k * ldt + c) = zero;
        }
    }

    const int words = bits == 4 ? 16 : 12;                                    // packed words per row and group
    for (int idx = i; idx < rows * words; idx += 128) {
        const int row = idx / words, wi = idx % words;
        uint32_t *out = qw + (size_t)(n0 + row) * row_words + g * words;
        uint32_t w = 0;
        if (bits == 4) {
            for (int c = 0; c < 8; ++c) w |= (uint32_t)scode[row][wi * 8 + c] << (4 * c);
        } else {
            const int u = wi / 3, wd = wi % 3;
            const uint8_t *cu = scode[row] + u * 32;
            for (int f = 0; f < 5; ++f) {
                w |= (uint32_t)cu[wd * 10 + f] << (3 * f);
                w |= (uint32_t)cu[wd * 10 + 5 + f] << (16 + 3 * f);
            }
            w |= ((uint32_t)(cu[30] >> wd) & 1u) << 15;
            w |= ((uint32_t)(cu[31] >> wd) & 1u) << 31;
        }
        out[wi] = w;
    }
}

hipError_t launch_quantize(const fbq_desc &d, const uint16_t *W, const uint16_t *At, const uint16_t *Bt, uint32_t *qw,
                           uint16_t *scales, uint16_t *zeros, hipStream_t stream, uint16_t *D16, uint16_t *Dt16, int ldt, float gain)
{
    hipLaunchKernelGGL(fbq_quantize_kernel, dim3(d.K / kGroup, ceil_div(d.N, kQuantRows)), dim3(128), 0, stream, W, At, Bt, qw, scales,
                       zeros, d.N, d.K, d.r, d.bits, (int)row_words(d.K, d.bits), D16, Dt16, ldt, gain);
    return hipGetLastError();
}

// ------------------------------------------------------------------ read-stream yardstick

// Reads every 16-byte piece of a buffer once and writes nothing: what the memory system delivers to a
// launch of a given size, measured with the same launch protocol as the decode kernels, is the
// ceiling they are judged against beside the nominal HBM peak.  Eight loads per thread in flight.
__global__ __launch_bounds__(256) void fbq_read_stream_kernel(const uint4 *__restrict__ p, unsigned long long n16)
{
    constexpr int kUnroll = 8;
    unsigned long long i = ((unsigned long long)blockIdx.x * kUnroll) * 256 + threadIdx.x;
    const unsigned long long stride = (unsigned long long)gridDim.x * kUnroll * 256;
    for (; i < n16; i += stride) {
        uint4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const unsigned long long j = i + (unsigned long long)u * 256;
            v[u] = p[j < n16 ? j : n16 - 1];             // past the end: the last piece again, never out of bounds
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) asm volatile("" ::"v"(v[u].x), "v"(v[u].y), "v"(v[u].z), "v"(v[u].w));   // keeps the loads alive
    }
}

hipError_t launch_read_stream(const void *buf, size_t bytes, hipStream_t stream)
{
    const unsigned long long n16 = bytes / 16;
    const int blocks = (int)std::min<unsigned long long>(1024, (n16 + 2047) / 2048);
    hipLaunchKernelGGL(fbq_read_stream_kernel, dim3(blocks), dim3(256), 0, stream, (const uint4 *)buf, n16);
    return hipGetLastError();
}

// ------------------------------------------------------------------ conventional sub-branch (comparator)

// The arrangement the fused kernel replaces (Sec. 3.2, Fig. 4 left): after the quantized main path has written
// y, the sub-branch runs as launches of its own - t = x.A, rounded to fp16 as a stand-alone kernel's output is,
// then y += t.B, which reads y back and writes it again.  Plain kernels: this path exists to be measured against.

// t[m][j] = sum_k x[m][k] At[j][k]: one block per (column j, token m), 256 threads along K.
__global__ __launch_bounds__(256) void fbq_unfused_down_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ At,
                                                               uint16_t *__restrict__ t, int K, int r)
{
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    __shared__ float part[4];
    const int j = blockIdx.x, m = blockIdx.y, tid = threadIdx.x;
    const uint4 *xr = reinterpret_cast<const uint4 *>(x + (size_t)m * K), *ar = reinterpret_cast<const uint4 *>(At + (size_t)j * K);
    float acc = 0.0f;
    for (int i = tid; i < K / 8; i += 256) {
        const uint4 a = xr[i], b = ar[i];
        const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, aw[q]), __builtin_bit_cast(h2, bw[q]), acc, false);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
    if ((tid & 63) == 0) part[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0) t[(size_t)m * r + j] = __builtin_bit_cast(uint16_t, (_Float16)(part[0] + part[1] + part[2] + part[3]));
}

// y[m][n] += sum_j t[m][j] Bt[n][j]: one thread per output, t of the token in LDS.
__global__ __launch_bounds__(256) void fbq_unfused_up_kernel(const uint16_t *__restrict__ t, const uint16_t *__restrict__ Bt,
                                                             uint16_t *__restrict__ y, int N, int r)
{
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    __shared__ uint32_t tl[kMaxRank / 2];
    const int m = blockIdx.y, n = blockIdx.x * 256 + threadIdx.x;
    for (int i = threadIdx.x; i < r / 2; i += 256) tl[i] = reinterpret_cast<const uint32_t *>(t + (size_t)m * r)[i];
    __syncthreads();
    if (n >= N) return;
    const uint4 *br = reinterpret_cast<const uint4 *>(Bt + (size_t)n * r);
    float acc = (float)__builtin_bit_cast(_Float16, y[(size_t)m * N + n]);
    for (int i = 0; i < r / 8; ++i) {
        const uint4 b = br[i];
        const uint32_t bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, tl[4 * i + q]), __builtin_bit_cast(h2, bw[q]), acc, false);
    }
    y[(size_t)m * N + n] = __builtin_bit_cast(uint16_t, (_Float16)acc);
}

hipError_t launch_unfused_branch(const LinearArgs &a, uint16_t *t, hipStream_t stream)
{
    hipLaunchKernelGGL(fbq_unfused_down_kernel, dim3(a.r, a.M), dim3(256), 0, stream, a.x, a.At, t, a.K, a.r);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(fbq_unfused_up_kernel, dim3(ceil_div(a.N, 256), a.M), dim3(256), 0, stream, t, a.Bt, a.y, a.N, a.r);
    return hipGetLastError();
}

}  // namespace fbq
