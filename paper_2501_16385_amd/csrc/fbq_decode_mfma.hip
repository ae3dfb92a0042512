// Decode path for a few tokens (2 <= M <= 16): the fused kernel of Sec. 4.3 with the packed codes
// still streamed exactly once, the tokens riding along as the 16 rows of a matrix-core tile.
//
//   y[M,N] = x[M,K] . Wq[N,K]^T + t[M,r] . B[r,N],   t = x . A
//
// Two launches, as in the paper: a small down-projection, then the fused kernel.
//
// Fused kernel.  A block owns 16 TN consecutive output columns and walks over K in chunks of 2048
// codes.  The packed words go from HBM straight into LDS (global_load_lds), one instruction per row
// and chunk: 64 lanes x 16 B (INT4) or 12 B (INT3) = one contiguous kilobyte of a single row, the
// access pattern the memory likes, double buffered so that the next chunk streams in while this one
// is worked on.  The block's four waves take four quantization groups of the chunk each and add
// their tiles up through LDS at the end.  v_mfma_f32_16x16x32_f16 multiplies a 16 (token) x 32 (k)
// activation fragment with a 32 (k) x 16 (column) weight fragment.  Lane (c = lane % 16,
// q = lane / 16) holds 8 values of k for token c in the first and for column c in the second, and
// the instruction only needs both operands to agree on which k that is.  So for one group of 128
// lane (c, q) takes the 32 codes k = 32 q .. 32 q + 31 of its column - one 16- or 12-byte LDS read
// (rows padded by 16 B: no bank conflicts) - and the same 32 activations of its token, read from
// L2 and arranged in registers into the pair order the code extraction produces; the four matrix
// instructions of the group use 8 of the 32 each.
//
// De-quantization is split around the matrix instruction so that nothing is rounded on the way:
// the weight operand carries the plain codes q (small integers, exact in fp16), the group's tile
// D = sum_k x q comes back in fp32, a fifth matrix instruction against an all-ones operand gives
// X = sum_k x in the same register layout, and the lane that holds column n adds s (D - z X) to its
// accumulator in fp32.  The up-projection enters the same accumulators as r more values of k, with
// t split into two fp16 halves (t_hi + t_lo carries 22 bits of the fp32 sum).
#include <hip/hip_fp16.h>

#include "fbq_internal.h"

namespace fbq {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));

constexpr int kTokens = 16;          // rows of the matrix-core tile; M is padded up to it
constexpr int kMaxSlices = 4;        // K slices of the down-projection

__device__ __forceinline__ half2_t h2_of(uint32_t v) { return __builtin_bit_cast(half2_t, v); }
__device__ __forceinline__ half2_t h2_splat(half_t v) { return half2_t{v, v}; }
__device__ __forceinline__ half8_t pack8(half2_t a, half2_t b, half2_t c, half2_t d)
{
    return half8_t{a.x, a.y, b.x, b.y, c.x, c.y, d.x, d.y};
}
__device__ __forceinline__ int ceil_div_dev(int a, int b) { return (a + b - 1) / b; }
__device__ __forceinline__ float4_t mfma(half8_t a, half8_t b, float4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

struct SmallParams {
    const uint32_t *qw;
    const uint16_t *scales;
    const uint16_t *zeros;
    const uint16_t *At;    // [r][K]
    const uint16_t *Bt;    // [N][r]
    const uint16_t *x;     // [M][K]
    uint16_t *y;           // [M][N]
    float *tpart;          // workspace: [slices][16][r] partial sums of t
    int M, N, K, r;
    int row_words, G;
    int slices, kslice;    // down-projection: number of K slices and their length (a multiple of 128)
};

// (w & mask) | 0x6400 in both halves: the masked field lands in the mantissa of 1024.0
__device__ __forceinline__ half2_t field(uint32_t w, uint32_t mask, uint32_t k6400)
{
    uint32_t v;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(v) : "v"(w), "s"(mask), "v"(k6400));
    return h2_of(v);
}

// The lane's 32 codes of one group as 16 exact fp16 pairs, in extraction order:
// INT4 word j -> pairs (8j+f, 8j+f+4), f = 0..3;  INT3 word j -> pairs (10j+f, 10j+f+5), f = 0..4,
// and codes (30, 31) last.
template <int BITS>
struct SmallCodes {
    static constexpr int kWords = BITS == 4 ? 4 : 3;
    uint32_t w[kWords];

    __device__ __forceinline__ void load(const uint32_t *p)
    {
        if (BITS == 4) {
            const uint4 q = *reinterpret_cast<const uint4 *>(p);
            w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w;
        } else {
            w[0] = p[0]; w[1] = p[1]; w[2] = p[2];
        }
    }

    __device__ __forceinline__ void pairs(uint32_t k6400, half2_t (&out)[16]) const
    {
        const half2_t k1024 = h2_splat((half_t)-1024.0f);
        if (BITS == 4) {
            const half2_t r16 = h2_splat((half_t)0.0625f), k64 = h2_splat((half_t)-64.0f);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t a = w[j], b = w[j] >> 8;
                out[4 * j + 0] = field(a, 0x000F000Fu, k6400) + k1024;
                out[4 * j + 1] = field(a, 0x00F000F0u, k6400) * r16 + k64;
                out[4 * j + 2] = field(b, 0x000F000Fu, k6400) + k1024;
                out[4 * j + 3] = field(b, 0x00F000F0u, k6400) * r16 + k64;
            }
        } else {
            const half2_t r8 = h2_splat((half_t)0.125f), k128 = h2_splat((half_t)-128.0f);
            const half2_t r64 = h2_splat((half_t)0.015625f), k16 = h2_splat((half_t)-16.0f);
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const uint32_t a = w[j], b = w[j] >> 9;
                out[5 * j + 0] = field(a, 0x00070007u, k6400) + k1024;
                out[5 * j + 1] = field(a, 0x00380038u, k6400) * r8 + k128;
                out[5 * j + 2] = field(a, 0x01C001C0u, k6400) * r64 + k16;
                out[5 * j + 3] = field(b, 0x00070007u, k6400) + k1024;
                out[5 * j + 4] = field(b, 0x00380038u, k6400) * r8 + k128;
            }
            const uint32_t e = ((w[0] >> 15) & 0x00010001u) | ((w[1] >> 14) & 0x00020002u) | ((w[2] >> 13) & 0x00040004u);
            out[15] = h2_of(e | 0x64006400u) + k1024;
        }
    }
};

// The lane's 32 activations of one group in the same pair order.
template <int BITS>
__device__ __forceinline__ void arrange_x(const uint4 (&raw)[4], half2_t (&p)[16])
{
    half_t v[32];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t w[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const half2_t h = h2_of(w[j]);
            v[i * 8 + j * 2] = h.x;
            v[i * 8 + j * 2 + 1] = h.y;
        }
    }
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

// Scales and zeros of the wave's four groups of one chunk for the lane's TN columns (fp16 bits):
// lane (c, q) loads those of group g0 + q, and group i's are fetched from lane (c, i) when needed.
template <int TN>
struct ScaleRegs {
    uint32_t sc[TN], zp[TN];
    __device__ __forceinline__ void load(const SmallParams &p, const size_t (&sz)[TN], int g)
    {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            sc[tn] = p.scales[sz[tn] + g];
            zp[tn] = p.zeros[sz[tn] + g];
        }
    }
    // value held by lane (c, i), as a float
    static __device__ __forceinline__ float from_group(uint32_t v, int src_lane)
    {
        const uint32_t u = (uint32_t)__builtin_amdgcn_ds_bpermute(src_lane * 4, (int)v);
        return (float)__builtin_bit_cast(half_t, (uint16_t)u);
    }
};

// The lane's 32 activations of one group as loaded; xl: token row + 32 q.
struct SmallXRegs {
    uint4 raw[4];
    __device__ __forceinline__ void load(const uint16_t *xl, int g)
    {
        const uint4 *src = reinterpret_cast<const uint4 *>(xl + (size_t)g * kGroup);
#pragma unroll
        for (int i = 0; i < 4; ++i) raw[i] = src[i];
    }
};

constexpr int kChunkCodes = 2048;    // codes per row one wave-wide copy brings in: 16 quantization groups
constexpr int kWaves = 4;            // waves per block; wave w works on groups 4 w .. 4 w + 3 of every chunk

template <int BITS>
struct SmallStage {
    static constexpr int kLaneBytes = BITS == 4 ? 16 : 12;          // 32 codes
    static constexpr int kRowBytes = 64 * kLaneBytes;               // one chunk of one row
    static constexpr int kPitch = kRowBytes + 16;                   // LDS row pitch: 4 banks further per row
};

template <int BITS, int TN>
constexpr int small_m_lds_bytes() { return 2 * 16 * TN * SmallStage<BITS>::kPitch + kWaves * TN * 64 * (int)sizeof(float4_t); }

// BITS: 3 or 4.  TN: 16-column tiles per block.  BRANCH: r > 0.
template <int BITS, int TN, bool BRANCH>
__global__ __launch_bounds__(64 * kWaves) void fbq_gemv_mfma_kernel(const SmallParams p)
{
    typedef SmallStage<BITS> St;
    constexpr int kRows = 16 * TN;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int kStageBytes = kRows * St::kPitch;    // stage s of the packed words starts at smem + s * kStageBytes
    float4_t *red = reinterpret_cast<float4_t *>(smem + 2 * kStageBytes);   // [kWaves][TN][64]

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, q = lane >> 4;
    const int n0 = blockIdx.x * kRows;
    const int chunks = ceil_div_dev(p.K, kChunkCodes);

    // columns past N re-read the last row and tokens past M the last token: computed, never stored
    size_t sz[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) sz[tn] = (size_t)min(n0 + 16 * tn + c, p.N - 1) * p.G;
    const uint16_t *xl = p.x + (size_t)min(c, p.M - 1) * p.K + 32 * q;

    // copies of this wave: rows wave, wave + 4, ... of the block, one chunk of 2048 codes each.  INT4:
    // one instruction of 64 x 16 B.  INT3: three of 64 x 4 B, each a contiguous 256 B piece of the 768.
    // Lanes past the end of a row (last chunk only) re-read the row's start, which nobody uses.
    auto copy_chunk = [&](int ch, int stage) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < kRows / kWaves; ++i) {
            const int row = wave + kWaves * i;
            const uint32_t *src = p.qw + (size_t)min(n0 + row, p.N - 1) * p.row_words;
            unsigned char *dst = &smem[stage * kStageBytes + row * St::kPitch];
            if constexpr (BITS == 4) {                  // the size argument must be a literal
                const int w = (ch * 64 + lane) * 4;
                __builtin_amdgcn_global_load_lds(src + (w < p.row_words ? w : 0), (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
            } else {
#pragma unroll
                for (int j = 0; j < 3; ++j) {
                    const int w = ch * 192 + j * 64 + lane;
                    __builtin_amdgcn_global_load_lds(src + (w < p.row_words ? w : 0),
                                                     (__attribute__((address_space(3))) void *)(dst + j * 256), 4, 0, 0);
                }
            }
        }
    };

    uint32_t k6400 = 0x64006400u;
    asm volatile("" : "+v"(k6400));                     // keep the constant in a VGPR for v_and_or_b32
    const half2_t one2 = h2_splat((half_t)1.0f);
    const half8_t ones = pack8(one2, one2, one2, one2);
    const float4_t zero4 = {0.0f, 0.0f, 0.0f, 0.0f};

    float4_t acc[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) acc[tn] = zero4;

    // one quantization group: block index blk = 4 (group within the chunk) + q of this lane's row segment
    auto process = [&](const unsigned char *stage, int i, const ScaleRegs<TN> &sr, const SmallXRegs &xr) __attribute__((always_inline)) {
        const int blk = 4 * (4 * wave + i) + q;         // the lane's 32-code block of the row's chunk
        half2_t xp[16];
        arrange_x<BITS>(xr.raw, xp);
        half8_t a[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = pack8(xp[4 * i], xp[4 * i + 1], xp[4 * i + 2], xp[4 * i + 3]);
        float4_t X = zero4;                             // sum of the group's activations, per token
#pragma unroll
        for (int i = 0; i < 4; ++i) X = mfma(a[i], ones, X);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            SmallCodes<BITS> cw;
            cw.load(reinterpret_cast<const uint32_t *>(stage + (16 * tn + c) * St::kPitch + blk * St::kLaneBytes));
            half2_t d[16];
            cw.pairs(k6400, d);
            float4_t D = zero4;
#pragma unroll
            for (int i = 0; i < 4; ++i) D = mfma(a[i], pack8(d[4 * i], d[4 * i + 1], d[4 * i + 2], d[4 * i + 3]), D);
            const float s = ScaleRegs<TN>::from_group(sr.sc[tn], 16 * i + c);
            const float nzs = -ScaleRegs<TN>::from_group(sr.zp[tn], 16 * i + c) * s;
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[tn][v] = fmaf(s, D[v], fmaf(nzs, X[v], acc[tn][v]));
        }
    };

    // Activations come from L2 one group ahead, scales and zeros one chunk ahead, each in two register
    // sets used alternately; loads past the last group re-read it and are dropped.
    const int g_last = p.G - 1;
    ScaleRegs<TN> sr[2];
    SmallXRegs xr[2];
    sr[0].load(p, sz, min(4 * wave + q, g_last));
    xr[0].load(xl, min(4 * wave, g_last));
    copy_chunk(0, 0);

    auto chunk = [&](int ch, const ScaleRegs<TN> &sc_cur, ScaleRegs<TN> &sc_nxt) __attribute__((always_inline)) {
        const unsigned char *cur = smem + (ch & 1) * kStageBytes;
        __builtin_amdgcn_s_waitcnt(0x0F70);             // vmcnt(0): this wave's copies of chunk ch have landed
        __syncthreads();                                // ... and everybody's; everybody is done with the other stage
        if (ch + 1 < chunks) copy_chunk(ch + 1, (ch + 1) & 1);   // block-uniform
        const int g0 = ch * 16 + 4 * wave;              // this wave's four groups of the chunk
        sc_nxt.load(p, sz, min(g0 + 16 + q, g_last));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            // next group of this wave: the following one of the chunk, or the first of the next chunk
            const int gn = i < 3 ? g0 + i + 1 : g0 + 16;
            xr[(i + 1) & 1].load(xl, min(gn, g_last));
            if (g0 + i < p.G) process(cur, i, sc_cur, xr[i & 1]);   // wave-uniform
        }
    };
    int ch = 0;
    for (; ch + 1 < chunks; ch += 2) {
        chunk(ch, sr[0], sr[1]);
        chunk(ch + 1, sr[1], sr[0]);
    }
    if (ch < chunks) chunk(ch, sr[0], sr[1]);

    // K split: every wave leaves its tiles in LDS; wave tn adds them up for tile tn, folds the
    // up-projection in and stores.
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) red[(wave * TN + tn) * 64 + lane] = acc[tn];
    __syncthreads();
    for (int tn = wave; tn < TN; tn += kWaves) {        // wave-uniform
        float4_t sum = red[tn * 64 + lane];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) sum += red[(w * TN + tn) * 64 + lane];

        const int n = n0 + 16 * tn + c;
        if (BRANCH) {
            // t[token c][j], j = 32 js + 8 q .. + 7, from the slices' partial sums; B^T row of column n
            const uint16_t *brow = p.Bt + (size_t)min(n, p.N - 1) * p.r;
            for (int js = 0; js * 32 < p.r; ++js) {
                const int j = js * 32 + q * 8;
                half8_t thi, tlo, bf;
#pragma unroll
                for (int e = 0; e < 8; ++e) { thi[e] = (half_t)0.0f; tlo[e] = (half_t)0.0f; bf[e] = (half_t)0.0f; }
                if (j < p.r) {                          // r is a multiple of 8: all eight taps or none
                    float t[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) t[e] = 0.0f;
                    for (int sl = 0; sl < p.slices; ++sl) {
                        const float4 *src = reinterpret_cast<const float4 *>(p.tpart + ((size_t)sl * kTokens + c) * p.r + j);
                        const float4 lo = src[0], hi = src[1];
                        t[0] += lo.x; t[1] += lo.y; t[2] += lo.z; t[3] += lo.w;
                        t[4] += hi.x; t[5] += hi.y; t[6] += hi.z; t[7] += hi.w;
                    }
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        thi[e] = (half_t)t[e];
                        tlo[e] = (half_t)(t[e] - (float)thi[e]);
                    }
                    bf = *reinterpret_cast<const half8_t *>(brow + j);
                }
                sum = mfma(thi, bf, sum);
                sum = mfma(tlo, bf, sum);
            }
        }
        // lane (c, q) holds column n and tokens 4 q + v
        if (n < p.N) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int m = 4 * q + v;
                if (m < p.M) p.y[(size_t)m * p.N + n] = __builtin_bit_cast(uint16_t, (half_t)sum[v]);
            }
        }
    }
}

// Down-projection for up to 16 tokens: block (column tile of 16, K slice); the block's sixteen waves
// take a sixteenth of the slice each.  partial[slice][token][j] = sum over the slice of
// x[token][k] At[j][k]; token rows past M repeat the last token.
constexpr int kDownWaves = 16;

__global__ __launch_bounds__(64 * kDownWaves) void fbq_down_proj_small_kernel(const SmallParams p)
{
    __shared__ float4_t red[kDownWaves][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, q = lane >> 4;
    const int j0 = blockIdx.x * 16, slice = blockIdx.y;
    const int kw = p.kslice / kDownWaves;               // a multiple of 32
    const int kbeg = slice * p.kslice + wave * kw;
    const int kend = min(p.K, kbeg + kw);
    const uint16_t *xr = p.x + (size_t)min(c, p.M - 1) * p.K + 8 * q;
    const uint16_t *ar = p.At + (size_t)min(j0 + c, p.r - 1) * p.K + 8 * q;
    float4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 8
    for (int k = kbeg; k < kend; k += 32)
        acc = mfma(*reinterpret_cast<const half8_t *>(xr + k), *reinterpret_cast<const half8_t *>(ar + k), acc);
    red[wave][lane] = acc;
    __syncthreads();
    if (wave == 0) {
        float4_t sum = red[0][lane];
#pragma unroll
        for (int w = 1; w < kDownWaves; ++w) sum += red[w][lane];
        const int j = j0 + c;                           // lane (c, q) holds column j and tokens 4 q + v
        if (j < p.r) {
#pragma unroll
            for (int v = 0; v < 4; ++v) p.tpart[((size_t)slice * kTokens + 4 * q + v) * p.r + j] = sum[v];
        }
    }
}

static int cu_count()
{
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
            n = 256;
        return n;
    }();
    return cus;
}

template <int BITS, int TN>
static hipError_t launch_variant(const SmallParams &p, hipStream_t stream)
{
    constexpr int lds = small_m_lds_bytes<BITS, TN>();
    // more than 64 KiB of LDS per block has to be asked for, once per kernel (and device)
    static const hipError_t prepared = [] {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&fbq_gemv_mfma_kernel<BITS, TN, true>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&fbq_gemv_mfma_kernel<BITS, TN, false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        return e;
    }();
    if (prepared != hipSuccess) return prepared;
    const dim3 grid(ceil_div(p.N, 16 * TN)), block(64 * kWaves);
    if (p.r > 0) hipLaunchKernelGGL((fbq_gemv_mfma_kernel<BITS, TN, true>), grid, block, lds, stream, p);
    else hipLaunchKernelGGL((fbq_gemv_mfma_kernel<BITS, TN, false>), grid, block, lds, stream, p);
    return hipGetLastError();
}

template <int BITS>
static hipError_t launch_bits(const SmallParams &p, hipStream_t stream)
{
    // Wider blocks re-read the activations less often; narrower ones give more blocks.  Take the
    // widest that still leaves two blocks per CU.
    const int want = 2 * cu_count();
    if (ceil_div(p.N, 64) >= want) return launch_variant<BITS, 4>(p, stream);
    if (ceil_div(p.N, 32) >= want) return launch_variant<BITS, 2>(p, stream);
    return launch_variant<BITS, 1>(p, stream);
}

// workspace: [slices][16][r] fp32 partial sums of t
size_t small_m_workspace_bytes(int r) { return (size_t)kMaxSlices * kTokens * r * sizeof(float); }

hipError_t launch_gemv_small_m(const LinearArgs &a, hipStream_t stream)
{
    if (a.M < 1 || a.M > kTokens) return hipErrorInvalidValue;
    SmallParams p;
    p.qw = a.qw; p.scales = a.scales; p.zeros = a.zeros; p.At = a.At; p.Bt = a.Bt; p.x = a.x; p.y = a.y;
    p.tpart = (float *)a.workspace;
    p.M = a.M; p.N = a.N; p.K = a.K; p.r = a.r;
    p.row_words = (int)row_words(a.K, a.bits);
    p.G = a.K / kGroup;
    p.kslice = ceil_div(ceil_div(a.K, kMaxSlices), 32 * kDownWaves) * (32 * kDownWaves);
    p.slices = ceil_div(a.K, p.kslice);
    if (a.r > 0) {
        hipLaunchKernelGGL(fbq_down_proj_small_kernel, dim3(ceil_div(a.r, 16), p.slices), dim3(64 * kDownWaves), 0, stream, p);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return a.bits == 4 ? launch_bits<4>(p, stream) : launch_bits<3>(p, stream);
}

}  // namespace fbq
