// Prefill path (M > 16 tokens): the fused kernel of Sec. 4.3 as an fp16 MFMA GEMM for gfx950.
//
//   y[M,N] = x[M,K] . Wq[N,K]^T + t[M,r] . B[r,N],   t = x . A
//
// Two launches: the down-projection t = x.A (a small MFMA GEMM, "requires relatively minimal time"
// in the paper's words) and the fused kernel, which de-quantizes in registers, multiplies on the
// matrix cores and folds the up-projection into the same accumulators as 2r extra K columns, so y
// is written once.
//
// Fused kernel.  Block = 4 waves side by side along N; block tile 128 (M) x 256 (N); a wave owns
// 128 x 64 = 4 x 2 tiles of v_mfma_f32_32x32x16_f16.  K advances in super-steps of 64:
//   * activations: a 128 x 64 fp16 tile per super-step goes global -> registers -> LDS (double
//     buffered, rows padded to 144 B so that 128-bit reads are conflict free); every wave reads
//     all of it (4 fragments per K step of 16);
//   * weights never touch LDS: lane (n = lane % 32, h = lane / 32) loads the 32 codes
//     k = 64u + 32h .. +31 of row n (INT4: one 16-byte load, INT3: one 12-byte load) and turns them
//     into the four 8 x fp16 operands of the super-step's four K steps in registers.  The MFMA only
//     needs both operands to agree on which k sits in which slot, so the activations are stored in
//     LDS in the order the code extraction produces (pairs (c, c+4) for INT4, (f, f+5) for INT3).
//   * de-quantization: mask+OR puts a code into the mantissa of 1024.0 (or 1024 + 16c, 1024 + 8c,
//     1024 + 64c for fields at higher bit offsets); one exact packed add or fma recovers the integer
//     code, then (q - z) * s in packed fp16: two roundings per weight, each 2^-11 relative at most.
// The sub-branch enters as t = t_hi + t_lo (two fp16 halves, ~22 bits) against B^T rows.
#include <hip/hip_fp16.h>

#include "fbq_internal.h"

namespace fbq {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int kBM = 128;             // block tile rows (tokens)
constexpr int kTM = 4;               // 32-row MFMA tiles per wave along M
constexpr int kTN = 2;               // 32-column MFMA tiles per wave along N
constexpr int kWavesN = 4;           // waves per block, side by side along N
constexpr int kBN = kWavesN * kTN * 32;   // 256
constexpr int kBK = 64;              // K per super-step
constexpr int kLdsRow = 144;         // bytes per activation row in LDS (128 + 16 padding)

__device__ __forceinline__ half2_t h2_of(uint32_t v) { return __builtin_bit_cast(half2_t, v); }
__device__ __forceinline__ half2_t h2_splat(half_t v) { return half2_t{v, v}; }

struct PrefillParams {
    const uint32_t *qw;
    const uint16_t *scales;
    const uint16_t *zeros;
    const uint16_t *Bt;    // [N][r]
    const uint16_t *x;     // [M][K]
    const uint16_t *thl;   // [M][2r]: t_hi | t_lo
    uint16_t *y;           // [M][N]
    int M, N, K, r;
    int row_words, G;
};

// Order in which the 32 activations of a lane's code block must sit so that slot s of K step i
// (s = 0..7) meets the code the extraction puts there.
template <int BITS>
__device__ __forceinline__ constexpr int slot_source(int s)
{
    if (BITS == 4) {                 // word j = s / 8 yields pairs (0,4) (1,5) (2,6) (3,7)
        const int j = s / 8, t = s % 8;
        return 8 * j + (t / 2) + 4 * (t % 2);
    }
    if (s >= 30) return s;           // the two spread codes pair up last
    const int w = s / 10, t = s % 10;   // word w yields pairs (f, f+5)
    return 10 * w + (t / 2) + 5 * (t % 2);
}

// The lane's 32 codes of one super-step as 16 fp16 pairs s * (q - z), in slot order.
template <int BITS>
struct WeightRegs {
    static constexpr int kWords = BITS == 4 ? 4 : 3;
    uint32_t w[kWords];

    __device__ __forceinline__ void load(const uint32_t *row, int u, int h)
    {
        const uint32_t *p = row + (2 * u + h) * kWords;
        if (BITS == 4) {
            const uint4 q = *reinterpret_cast<const uint4 *>(p);
            w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w;
        } else {
            w[0] = p[0]; w[1] = p[1]; w[2] = p[2];
        }
    }

    __device__ __forceinline__ void dequant(half2_t s2, half2_t nz2, half2_t (&out)[16]) const
    {
        const half2_t k1024 = h2_splat((half_t)-1024.0f);
        if (BITS == 4) {
            const half2_t r16 = h2_splat((half_t)0.0625f), k64 = h2_splat((half_t)-64.0f);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t a = w[j], b = w[j] >> 8;
                const half2_t q0 = h2_of((a & 0x000F000Fu) | 0x64006400u) + k1024;
                const half2_t q1 = h2_of((a & 0x00F000F0u) | 0x64006400u) * r16 + k64;
                const half2_t q2 = h2_of((b & 0x000F000Fu) | 0x64006400u) + k1024;
                const half2_t q3 = h2_of((b & 0x00F000F0u) | 0x64006400u) * r16 + k64;
                out[4 * j + 0] = (q0 + nz2) * s2;
                out[4 * j + 1] = (q1 + nz2) * s2;
                out[4 * j + 2] = (q2 + nz2) * s2;
                out[4 * j + 3] = (q3 + nz2) * s2;
            }
        } else {
            const half2_t r8 = h2_splat((half_t)0.125f), k128 = h2_splat((half_t)-128.0f);
            const half2_t r64 = h2_splat((half_t)0.015625f), k16 = h2_splat((half_t)-16.0f);
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const uint32_t a = w[j], b = w[j] >> 9;
                const half2_t q0 = h2_of((a & 0x00070007u) | 0x64006400u) + k1024;
                const half2_t q1 = h2_of((a & 0x00380038u) | 0x64006400u) * r8 + k128;
                const half2_t q2 = h2_of((a & 0x01C001C0u) | 0x64006400u) * r64 + k16;
                const half2_t q3 = h2_of((b & 0x00070007u) | 0x64006400u) + k1024;
                const half2_t q4 = h2_of((b & 0x00380038u) | 0x64006400u) * r8 + k128;
                out[5 * j + 0] = (q0 + nz2) * s2;
                out[5 * j + 1] = (q1 + nz2) * s2;
                out[5 * j + 2] = (q2 + nz2) * s2;
                out[5 * j + 3] = (q3 + nz2) * s2;
                out[5 * j + 4] = (q4 + nz2) * s2;
            }
            const uint32_t e = ((w[0] >> 15) & 0x00010001u) | ((w[1] >> 14) & 0x00020002u) | ((w[2] >> 13) & 0x00040004u);
            out[15] = (h2_of(e | 0x64006400u) + k1024 + nz2) * s2;
        }
    }
};

__device__ __forceinline__ half8_t pack8(half2_t a, half2_t b, half2_t c, half2_t d)
{
    return half8_t{a.x, a.y, b.x, b.y, c.x, c.y, d.x, d.y};
}

template <int BITS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void fbq_gemm_kernel(const PrefillParams p)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][kBM * kLdsRow];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, h = lane >> 5;
    const int m0 = blockIdx.y * kBM;
    const int nw = blockIdx.x * kBN + wave * (kTN * 32);
    const int U = p.K / kBK;         // even: K is a multiple of 128

    // this lane's weight rows (clamped: columns past N are computed on a valid row and never stored)
    const uint32_t *wrow[kTN];
    int nrow[kTN];
#pragma unroll
    for (int tn = 0; tn < kTN; ++tn) {
        nrow[tn] = min(nw + tn * 32 + col, p.N - 1);
        wrow[tn] = p.qw + (size_t)nrow[tn] * p.row_words;
    }

    // this thread's share of the activation tile: row tid/2, 32 activations (64 B) of block tid%2
    const int xr = tid >> 1, xb = tid & 1;
    const uint16_t *xsrc = p.x + (size_t)min(m0 + xr, p.M - 1) * p.K + xb * 32;
    uint4 xreg[4];
    auto x_fetch = [&](int u) __attribute__((always_inline)) {
        const uint4 *s = reinterpret_cast<const uint4 *>(xsrc + u * kBK);
#pragma unroll
        for (int i = 0; i < 4; ++i) xreg[i] = s[i];
    };
    auto x_store = [&](int buf) __attribute__((always_inline)) {
        half_t v[32];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t wds[4] = {xreg[i].x, xreg[i].y, xreg[i].z, xreg[i].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const half2_t hh = h2_of(wds[j]);
                v[i * 8 + j * 2] = hh.x;
                v[i * 8 + j * 2 + 1] = hh.y;
            }
        }
        uint4 *dst = reinterpret_cast<uint4 *>(&lds[buf][xr * kLdsRow + xb * 64]);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            half2_t o[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] = half2_t{v[slot_source<BITS>(i * 8 + 2 * j)], v[slot_source<BITS>(i * 8 + 2 * j + 1)]};
            dst[i] = make_uint4(__builtin_bit_cast(uint32_t, o[0]), __builtin_bit_cast(uint32_t, o[1]),
                                __builtin_bit_cast(uint32_t, o[2]), __builtin_bit_cast(uint32_t, o[3]));
        }
    };

    float16_t acc[kTM][kTN];
#pragma unroll
    for (int tm = 0; tm < kTM; ++tm)
#pragma unroll
        for (int tn = 0; tn < kTN; ++tn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.0f;

    half2_t s2[kTN], nz2[kTN];
    auto load_sz = [&](int g) __attribute__((always_inline)) {
#pragma unroll
        for (int tn = 0; tn < kTN; ++tn) {
            const half_t s = __builtin_bit_cast(half_t, p.scales[(size_t)nrow[tn] * p.G + g]);
            const half_t z = __builtin_bit_cast(half_t, p.zeros[(size_t)nrow[tn] * p.G + g]);
            s2[tn] = h2_splat(s);
            nz2[tn] = h2_splat(-z);
        }
    };

    // one super-step: four K steps of 16 on the tile in lds[buf]
    auto compute = [&](const WeightRegs<BITS> (&wr)[kTN], int buf) __attribute__((always_inline)) {
        half2_t wv[kTN][16];
#pragma unroll
        for (int tn = 0; tn < kTN; ++tn) wr[tn].dequant(s2[tn], nz2[tn], wv[tn]);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            half8_t bf[kTN];
#pragma unroll
            for (int tn = 0; tn < kTN; ++tn) bf[tn] = pack8(wv[tn][4 * i], wv[tn][4 * i + 1], wv[tn][4 * i + 2], wv[tn][4 * i + 3]);
#pragma unroll
            for (int tm = 0; tm < kTM; ++tm) {
                const half8_t af = *reinterpret_cast<const half8_t *>(&lds[buf][(tm * 32 + col) * kLdsRow + h * 64 + i * 16]);
#pragma unroll
                for (int tn = 0; tn < kTN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af, bf[tn], acc[tm][tn], 0, 0, 0);
            }
        }
    };

    WeightRegs<BITS> wa[kTN], wb[kTN];
#pragma unroll
    for (int tn = 0; tn < kTN; ++tn) wa[tn].load(wrow[tn], 0, h);
    load_sz(0);
    x_fetch(0);
    x_store(0);
    __syncthreads();

    for (int u = 0; u < U; u += 2) {                    // one quantization group (128 k) per iteration
#pragma unroll
        for (int tn = 0; tn < kTN; ++tn) wb[tn].load(wrow[tn], u + 1, h);
        x_fetch(u + 1);
        compute(wa, 0);
        x_store(1);
        __syncthreads();
        const bool more = u + 2 < U;                    // block-uniform
        if (more) {
#pragma unroll
            for (int tn = 0; tn < kTN; ++tn) wa[tn].load(wrow[tn], u + 2, h);
            x_fetch(u + 2);
        }
        compute(wb, 1);
        if (more) {
            load_sz((u + 2) / 2);
            x_store(0);
        }
        __syncthreads();
    }

    // up-projection: 2r extra K columns, t_hi and t_lo against the same B^T rows
    if (p.r > 0) {
        const int steps = (2 * p.r) / 16;
        for (int st = 0; st < steps; ++st) {
            const int jj = st * 16 + h * 8;             // column of [t_hi | t_lo]
            const int jb = jj >= p.r ? jj - p.r : jj;   // tap of B
            half8_t bf[kTN];
#pragma unroll
            for (int tn = 0; tn < kTN; ++tn) bf[tn] = *reinterpret_cast<const half8_t *>(p.Bt + (size_t)nrow[tn] * p.r + jb);
#pragma unroll
            for (int tm = 0; tm < kTM; ++tm) {
                const int m = min(m0 + tm * 32 + col, p.M - 1);
                const half8_t af = *reinterpret_cast<const half8_t *>(p.thl + (size_t)m * (2 * p.r) + jj);
#pragma unroll
                for (int tn = 0; tn < kTN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af, bf[tn], acc[tm][tn], 0, 0, 0);
            }
        }
    }

    // single store of y: accumulator register v of a lane holds row 8*(v/4) + 4*h + v%4, column `col`
#pragma unroll
    for (int tn = 0; tn < kTN; ++tn) {
        const int n = nw + tn * 32 + col;
        if (n >= p.N) continue;
#pragma unroll
        for (int tm = 0; tm < kTM; ++tm) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + tm * 32 + 8 * (v / 4) + 4 * h + (v % 4);
                if (m < p.M) p.y[(size_t)m * p.N + n] = __builtin_bit_cast(uint16_t, (half_t)acc[tm][tn][v]);
            }
        }
    }
}

// ------------------------------------------------------------------ down-projection (prefill)

// t[m][j] = sum_k x[m][k] * At[j][k] for one 32-row tile of tokens and all r columns; the block's
// four waves take a quarter of K each and add their tiles up through LDS in wave order.  Written as
// t_hi = fp16(t), t_lo = fp16(t - t_hi).  RT = 32-column tiles (r <= 32 * RT).
template <int RT>
__global__ __launch_bounds__(256) void fbq_down_proj_prefill_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ At,
                                                                    uint16_t *__restrict__ thl, int M, int K, int r)
{
    extern __shared__ float sum[];                      // [32][32 * RT]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, h = lane >> 5;
    const int m0 = blockIdx.x * 32;
    const int kq = K / 4;                               // K is a multiple of 128
    const uint16_t *xrow = x + (size_t)min(m0 + col, M - 1) * K + wave * kq + h * 8;
    const uint16_t *arow[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) arow[rt] = At + (size_t)min(rt * 32 + col, r - 1) * K + wave * kq + h * 8;

    float16_t acc[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[rt][v] = 0.0f;

#pragma unroll 4
    for (int kk = 0; kk < kq; kk += 16) {
        const half8_t af = *reinterpret_cast<const half8_t *>(xrow + kk);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const half8_t bf = *reinterpret_cast<const half8_t *>(arow[rt] + kk);
            acc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af, bf, acc[rt], 0, 0, 0);
        }
    }

    const int ld = 32 * RT;
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int i = 8 * (v / 4) + 4 * h + (v % 4);
                    float *dst = &sum[i * ld + rt * 32 + col];
                    *dst = w == 0 ? acc[rt][v] : *dst + acc[rt][v];
                }
        }
        __syncthreads();
    }
    for (int idx = tid; idx < 32 * r; idx += 256) {
        const int i = idx / r, j = idx - i * r;
        if (m0 + i < M) {
            const float t = sum[i * ld + j];
            const half_t hi = (half_t)t;
            const half_t lo = (half_t)(t - (float)hi);
            thl[(size_t)(m0 + i) * (2 * r) + j] = __builtin_bit_cast(uint16_t, hi);
            thl[(size_t)(m0 + i) * (2 * r) + r + j] = __builtin_bit_cast(uint16_t, lo);
        }
    }
}

size_t prefill_workspace_bytes(int M, int r) { return (size_t)M * 2 * r * sizeof(uint16_t); }

hipError_t launch_down_proj_prefill(const LinearArgs &a, hipStream_t stream)
{
    const dim3 grid(ceil_div(a.M, 32));
    const int rt = ceil_div(a.r, 32);
    uint16_t *thl = (uint16_t *)a.workspace;
    if (rt <= 1) hipLaunchKernelGGL(fbq_down_proj_prefill_kernel<1>, grid, dim3(256), 32 * 32 * sizeof(float), stream, a.x, a.At, thl, a.M, a.K, a.r);
    else if (rt <= 2) hipLaunchKernelGGL(fbq_down_proj_prefill_kernel<2>, grid, dim3(256), 32 * 64 * sizeof(float), stream, a.x, a.At, thl, a.M, a.K, a.r);
    else if (rt <= 4) hipLaunchKernelGGL(fbq_down_proj_prefill_kernel<4>, grid, dim3(256), 32 * 128 * sizeof(float), stream, a.x, a.At, thl, a.M, a.K, a.r);
    else hipLaunchKernelGGL(fbq_down_proj_prefill_kernel<8>, grid, dim3(256), 32 * 256 * sizeof(float), stream, a.x, a.At, thl, a.M, a.K, a.r);
    return hipGetLastError();
}

hipError_t launch_gemm_prefill(const LinearArgs &a, hipStream_t stream)
{
    PrefillParams p;
    p.qw = a.qw; p.scales = a.scales; p.zeros = a.zeros; p.Bt = a.Bt; p.x = a.x; p.y = a.y;
    p.thl = (const uint16_t *)a.workspace;
    p.M = a.M; p.N = a.N; p.K = a.K; p.r = a.r;
    p.row_words = (int)row_words(a.K, a.bits);
    p.G = a.K / kGroup;
    const dim3 grid(ceil_div(a.N, kBN), ceil_div(a.M, kBM));
    if (a.bits == 4) hipLaunchKernelGGL(fbq_gemm_kernel<4>, grid, dim3(256), 0, stream, p);
    else hipLaunchKernelGGL(fbq_gemm_kernel<3>, grid, dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace fbq
