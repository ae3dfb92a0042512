// Decode path (M <= 16 tokens): the fused kernel of Sec. 4.3 as a memory-streaming GEMV for gfx950.
//
//   down-projection   t = x.A            small split-K kernel, fp32 partial sums in the workspace
//   fused kernel      y = x.Wq^T + t.B   one pass over the packed codes; de-quantization, main
//                                        projection and up-projection share one fp32 accumulator
//                                        and y is written once
//
// Work decomposition of the fused kernel.  A wave owns kRows consecutive output rows and a
// contiguous K range; its 64 lanes lie along K.  One wave-wide load covers 2048 codes
// (INT4: 16 B per lane, INT3: 12 B per lane, both fully coalesced), so a lane always holds 32
// consecutive codes of one quantization group.  The lane's 32 activations stay in registers for
// the whole kernel (they are the same for every row), pre-arranged as the fp16 pairs that the
// code extraction produces.
//
// Code extraction without conversion instructions.  Masking a packed word with 0x000F000F (INT4)
// or 0x00070007 (INT3) leaves two codes, one per 16-bit half, each in the low mantissa bits of an
// fp16 with a zero exponent field: the subnormal q * 2^-24.  v_dot2_f32_f16 multiplies such a pair
// with an activation pair exactly and accumulates in fp32, so a field at bit offset o only needs
// its accumulator scaled by 2^(24-o) once per 32 codes.  The group's scale and zero are applied
// once per lane and chunk:  s * (sum q.x - z * sum x).
#include <hip/hip_fp16.h>

#include "fbq_internal.h"

namespace fbq {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half_t;

__device__ __forceinline__ half2_t as_h2(uint32_t v) { return __builtin_bit_cast(half2_t, v); }
__device__ __forceinline__ float dot2(uint32_t codes, half2_t xp, float acc)
{
    return __builtin_amdgcn_fdot2(as_h2(codes), xp, acc, false);
}

// Sum over the 64 lanes of a wave; every lane ends with the total.
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// ------------------------------------------------------------------ activations in registers

// The lane's 32 activations of one chunk as the 16 pairs matching the code extraction order, and
// their plain sum.  INT4: word j holds codes 8j..8j+7 and yields pairs (0,4) (1,5) (2,6) (3,7).
// INT3: word w holds codes 10w..10w+9 and yields pairs (f, f+5), f = 0..4; codes 30, 31 pair up.
template <int BITS>
struct XFrag {
    half2_t p[16];
    float sum;

    __device__ __forceinline__ void load(const uint16_t *xrow, int k0, bool valid)
    {
        half_t v[32];
        if (valid) {
            const uint4 *src = reinterpret_cast<const uint4 *>(xrow + k0);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint4 q = src[i];
                uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    half2_t h = as_h2(w[j]);
                    v[i * 8 + j * 2] = h.x;
                    v[i * 8 + j * 2 + 1] = h.y;
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < 32; ++i) v[i] = (half_t)0.0f;
        }
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < 32; ++i) s += (float)v[i];
        sum = s;
        if (BITS == 4) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int f = 0; f < 4; ++f) p[j * 4 + f] = half2_t{v[8 * j + f], v[8 * j + f + 4]};
        } else {
#pragma unroll
            for (int w = 0; w < 3; ++w)
#pragma unroll
                for (int f = 0; f < 5; ++f) p[w * 5 + f] = half2_t{v[10 * w + f], v[10 * w + f + 5]};
            p[15] = half2_t{v[30], v[31]};
        }
    }
};

// sum_k q[k] * x[k] over the lane's 32 codes (exact products, fp32 accumulation).
__device__ __forceinline__ float dot_codes_int4(const uint32_t (&w)[4], const half2_t (&p)[16])
{
    float lo = 0.0f, hi = 0.0f;   // fields at bit 0 (unit 2^-24) and at bit 4 (unit 2^-20)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t a = w[j], b = w[j] >> 8;
        lo = dot2(a & 0x000F000Fu, p[j * 4 + 0], lo);
        hi = dot2(a & 0x00F000F0u, p[j * 4 + 1], hi);
        lo = dot2(b & 0x000F000Fu, p[j * 4 + 2], lo);
        hi = dot2(b & 0x00F000F0u, p[j * 4 + 3], hi);
    }
    return lo * 16777216.0f + hi * 1048576.0f;
}

__device__ __forceinline__ float dot_codes_int3(const uint32_t (&w)[3], const half2_t (&p)[16])
{
    float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f;   // fields at bit 0, 3, 6: units 2^-24, 2^-21, 2^-18
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        const uint32_t a = w[j], b = w[j] >> 9;
        a0 = dot2(a & 0x00070007u, p[j * 5 + 0], a0);
        a1 = dot2(a & 0x00380038u, p[j * 5 + 1], a1);
        a2 = dot2(a & 0x01C001C0u, p[j * 5 + 2], a2);
        a0 = dot2(b & 0x00070007u, p[j * 5 + 3], a0);
        a1 = dot2(b & 0x00380038u, p[j * 5 + 4], a1);
    }
    const uint32_t e = ((w[0] >> 15) & 0x00010001u) | ((w[1] >> 14) & 0x00020002u) | ((w[2] >> 13) & 0x00040004u);
    a0 = dot2(e, p[15], a0);
    return a0 * 16777216.0f + a1 * 2097152.0f + a2 * 262144.0f;
}

template <int BITS>
struct CodeWords;
template <>
struct CodeWords<4> {
    uint32_t w[4];
    __device__ __forceinline__ void load(const uint32_t *p)
    {
        uint4 q = *reinterpret_cast<const uint4 *>(p);
        w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w;
    }
    __device__ __forceinline__ void zero() { w[0] = w[1] = w[2] = w[3] = 0; }
    __device__ __forceinline__ float dot(const half2_t (&p)[16]) const { return dot_codes_int4(w, p); }
};
template <>
struct CodeWords<3> {
    uint32_t w[3];
    __device__ __forceinline__ void load(const uint32_t *p)
    {
        w[0] = p[0]; w[1] = p[1]; w[2] = p[2];
    }
    __device__ __forceinline__ void zero() { w[0] = w[1] = w[2] = 0; }
    __device__ __forceinline__ float dot(const half2_t (&p)[16]) const { return dot_codes_int3(w, p); }
};

// ------------------------------------------------------------------ fused GEMV kernel

struct GemvParams {
    const uint32_t *qw;
    const uint16_t *scales;
    const uint16_t *zeros;
    const uint16_t *Bt;
    const float *tpart;   // [kSplitT][M][r]
    const uint16_t *x;    // [M][K]
    uint16_t *y;          // [M][N]
    int M, N, K, r;
    int row_words;        // words per packed row
    int G;                // groups per row
};

// BITS: 3 or 4.  CPW: chunks (of 2048 codes) per wave.  KS: waves of a block that split K.
// ROWS: rows per wave.  RI: ceil(r/128), 0 = branch-free twin.
template <int BITS, int CPW, int KS, int ROWS, int RI>
__global__ __launch_bounds__(256) void fbq_gemv_kernel(const GemvParams p)
{
    constexpr int kWaves = 4;
    constexpr int kRowSets = kWaves / KS;               // row sets per block
    constexpr int kLaneWords = BITS == 4 ? 4 : 3;
    __shared__ float red[KS > 1 ? kWaves * ROWS : 1];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int ks = wave % KS;                           // which K slice
    const int rs = wave / KS;                           // which row set of the block
    const int m = blockIdx.y;
    const int n0 = (blockIdx.x * kRowSets + rs) * ROWS;
    const bool wave_active = n0 < p.N;
    const int chunk0 = ks * CPW;

    // activations of this wave's K range, kept for all rows
    XFrag<BITS> xf[CPW];
    const uint16_t *xrow = p.x + (size_t)m * p.K;
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
        const int k0 = (chunk0 + c) * kChunk + lane * kLaneCodes;
        xf[c].load(xrow, k0, wave_active && k0 < p.K);
    }

    // down-projection result for this lane's taps: t[j], j = (i*64 + lane)*2 + {0,1}
    float t0[RI > 0 ? RI : 1], t1[RI > 0 ? RI : 1];
    if (RI > 0) {
#pragma unroll
        for (int i = 0; i < RI; ++i) {
            t0[i] = t1[i] = 0.0f;
            const int j = (i * 64 + lane) * 2;
            if (wave_active && ks == 0 && j < p.r) {
                for (int s = 0; s < kSplitT; ++s) {
                    const float2 v = *reinterpret_cast<const float2 *>(p.tpart + ((size_t)s * p.M + m) * p.r + j);
                    t0[i] += v.x;
                    t1[i] += v.y;
                }
            }
        }
    }

    // issue every load of this wave's rows before using any of them
    CodeWords<BITS> cw[ROWS][CPW];
    half_t sc[ROWS][CPW], zp[ROWS][CPW];
    uint32_t bt[ROWS][RI > 0 ? RI : 1];
#pragma unroll
    for (int i = 0; i < ROWS; ++i) {
        const int n = min(n0 + i, p.N - 1);             // clamp: tail rows re-read a valid row, result discarded
        const uint32_t *qrow = p.qw + (size_t)n * p.row_words;
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            const int k0 = (chunk0 + c) * kChunk + lane * kLaneCodes;
            if (wave_active && k0 < p.K) {
                cw[i][c].load(qrow + (size_t)(k0 / kLaneCodes) * kLaneWords);
                const int g = k0 / kGroup;
                sc[i][c] = __builtin_bit_cast(half_t, p.scales[(size_t)n * p.G + g]);
                zp[i][c] = __builtin_bit_cast(half_t, p.zeros[(size_t)n * p.G + g]);
            } else {
                cw[i][c].zero();
                sc[i][c] = (half_t)0.0f;
                zp[i][c] = (half_t)0.0f;
            }
        }
        if (RI > 0) {
#pragma unroll
            for (int q = 0; q < RI; ++q) {
                const int j = (q * 64 + lane) * 2;
                bt[i][q] = (wave_active && ks == 0 && j < p.r)
                               ? *reinterpret_cast<const uint32_t *>(p.Bt + (size_t)n * p.r + j)
                               : 0u;
            }
        }
    }

    float out = 0.0f;   // lane i of the wave ends up holding row n0 + i
#pragma unroll
    for (int i = 0; i < ROWS; ++i) {
        float acc = 0.0f;
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            const float qx = cw[i][c].dot(xf[c].p);
            const float s = (float)sc[i][c], z = (float)zp[i][c];
            acc = fmaf(s, fmaf(-z, xf[c].sum, qx), acc);
        }
        if (RI > 0) {
#pragma unroll
            for (int q = 0; q < RI; ++q) {
                const half2_t b = as_h2(bt[i][q]);
                acc = fmaf(t0[q], (float)b.x, acc);
                acc = fmaf(t1[q], (float)b.y, acc);
            }
        }
        acc = wave_sum(acc);
        if (lane == i) out = acc;
    }

    if (KS > 1) {
        if (lane < ROWS) red[wave * ROWS + lane] = out;
        __syncthreads();
        if (ks == 0 && lane < ROWS) {
            out = 0.0f;
#pragma unroll
            for (int q = 0; q < KS; ++q) out += red[(wave + q) * ROWS + lane];
        }
    }
    if (wave_active && ks == 0 && lane < ROWS && n0 + lane < p.N)
        p.y[(size_t)m * p.N + n0 + lane] = __builtin_bit_cast(uint16_t, (half_t)out);
}

// ------------------------------------------------------------------ down-projection (decode)

// t[m][j] = sum_k x[m][k] * A[k][j], split over kSplitT blocks along K; block s writes its
// partial sums to tpart[s][m][j].  Threads: (r/2) column pairs x (256/(r/2)) K sub-slices.
template <int MT>
__global__ __launch_bounds__(256) void fbq_down_proj_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ A,
                                                            float *__restrict__ tpart, int M, int K, int r, int m_base)
{
    extern __shared__ float lds[];                      // [ksub][MT][r]
    const int pairs = r >> 1;                           // r is a multiple of 8
    const int ksub_n = 256 / pairs > 0 ? 256 / pairs : 1;
    const int jp = threadIdx.x % pairs;
    const int ksub = threadIdx.x / pairs;
    const int kper = (K + kSplitT - 1) / kSplitT;
    const int kbeg = blockIdx.x * kper;
    const int kend = min(K, kbeg + kper);

    float acc0[MT], acc1[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) acc0[m] = acc1[m] = 0.0f;

    if (ksub < ksub_n && threadIdx.x < pairs * ksub_n) {
        for (int k = kbeg + ksub; k < kend; k += ksub_n) {
            const half2_t a = as_h2(*reinterpret_cast<const uint32_t *>(A + (size_t)k * r + 2 * jp));
            const float a0 = (float)a.x, a1 = (float)a.y;
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                if (m_base + m < M) {
                    const float xv = (float)__builtin_bit_cast(half_t, x[(size_t)(m_base + m) * K + k]);
                    acc0[m] = fmaf(xv, a0, acc0[m]);
                    acc1[m] = fmaf(xv, a1, acc1[m]);
                }
            }
        }
        for (int m = 0; m < MT; ++m) {
            lds[(ksub * MT + m) * r + 2 * jp] = acc0[m];
            lds[(ksub * MT + m) * r + 2 * jp + 1] = acc1[m];
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < MT * r; idx += 256) {
        const int m = idx / r, j = idx - m * r;
        if (m_base + m < M) {
            float s = 0.0f;
            for (int q = 0; q < ksub_n; ++q) s += lds[(q * MT + m) * r + j];
            tpart[((size_t)blockIdx.x * M + m_base + m) * r + j] = s;
        }
    }
}

template <int MT>
static void launch_down_proj_mt(const LinearArgs &a, hipStream_t stream)
{
    const int pairs = a.r / 2;
    const int ksub_n = 256 / pairs > 0 ? 256 / pairs : 1;
    const size_t lds_bytes = (size_t)ksub_n * MT * a.r * sizeof(float);
    hipLaunchKernelGGL(fbq_down_proj_kernel<MT>, dim3(kSplitT), dim3(256), lds_bytes, stream, a.x, a.A, a.tpart, a.M, a.K, a.r,
                       0);
}

hipError_t launch_down_proj_decode(const LinearArgs &a, hipStream_t stream)
{
    if (a.M == 1) launch_down_proj_mt<1>(a, stream);
    else if (a.M <= 4) launch_down_proj_mt<4>(a, stream);
    else if (a.M <= 8) launch_down_proj_mt<8>(a, stream);
    else launch_down_proj_mt<16>(a, stream);
    return hipGetLastError();
}

// ------------------------------------------------------------------ dispatch

template <int BITS, int CPW, int KS, int ROWS>
static hipError_t launch_gemv_ri(const GemvParams &p, hipStream_t stream)
{
    constexpr int kRowSets = 4 / KS;
    const dim3 grid(ceil_div(p.N, kRowSets * ROWS), p.M);
    const int ri = ceil_div(p.r, 128);
    switch (ri) {
    case 0: hipLaunchKernelGGL((fbq_gemv_kernel<BITS, CPW, KS, ROWS, 0>), grid, dim3(256), 0, stream, p); break;
    case 1: hipLaunchKernelGGL((fbq_gemv_kernel<BITS, CPW, KS, ROWS, 1>), grid, dim3(256), 0, stream, p); break;
    default: hipLaunchKernelGGL((fbq_gemv_kernel<BITS, CPW, KS, ROWS, 2>), grid, dim3(256), 0, stream, p); break;
    }
    return hipGetLastError();
}

template <int BITS, int CPW, int KS>
static hipError_t launch_gemv_rows(const GemvParams &p, hipStream_t stream)
{
    // enough waves to cover the chip several times over, otherwise fewer rows per wave
    const long waves4 = (long)ceil_div(p.N, 4) * KS * p.M;
    if (waves4 >= 2048) return launch_gemv_ri<BITS, CPW, KS, 4>(p, stream);
    return launch_gemv_ri<BITS, CPW, KS, 2>(p, stream);
}

template <int BITS>
static hipError_t launch_gemv_bits(const GemvParams &p, hipStream_t stream)
{
    const int chunks = ceil_div(p.K, kChunk);
    if (chunks <= 4) {
        switch (chunks) {
        case 1: return launch_gemv_rows<BITS, 1, 1>(p, stream);
        case 2: return launch_gemv_rows<BITS, 2, 1>(p, stream);
        case 3: return launch_gemv_rows<BITS, 3, 1>(p, stream);
        default: return launch_gemv_rows<BITS, 4, 1>(p, stream);
        }
    }
    if (chunks <= 8) {
        switch (ceil_div(chunks, 2)) {
        case 3: return launch_gemv_rows<BITS, 3, 2>(p, stream);
        default: return launch_gemv_rows<BITS, 4, 2>(p, stream);
        }
    }
    if (chunks <= 16) {
        switch (ceil_div(chunks, 4)) {
        case 3: return launch_gemv_rows<BITS, 3, 4>(p, stream);
        default: return launch_gemv_rows<BITS, 4, 4>(p, stream);
        }
    }
    return hipErrorInvalidValue;   // K > 32768: rejected by the caller's shape check
}

hipError_t launch_gemv_decode(const LinearArgs &a, hipStream_t stream)
{
    GemvParams p;
    p.qw = a.qw; p.scales = a.scales; p.zeros = a.zeros; p.Bt = a.Bt; p.tpart = a.tpart; p.x = a.x; p.y = a.y;
    p.M = a.M; p.N = a.N; p.K = a.K; p.r = a.r;
    p.row_words = (int)row_words(a.K, a.bits);
    p.G = a.K / kGroup;
    return a.bits == 4 ? launch_gemv_bits<4>(p, stream) : launch_gemv_bits<3>(p, stream);
}

}  // namespace fbq
