// Decode path (M <= 16 tokens): the fused kernel of Sec. 4.3 as a memory-streaming GEMV for gfx950.
//
//   down-projection   t = x.A            a few producer blocks at the front of the SAME launch, each
//                                        owning four columns of A over all of K (the paper keeps
//                                        it a separate small kernel; on this GPU a launch costs as
//                                        much as streaming a 4096^2 layer, so it rides along)
//   fused kernel      y = x.Wq^T + t.B   one pass over the packed codes; de-quantization, main
//                                        projection and up-projection share one fp32 accumulator
//                                        and y is written once.  t is needed only for the last few
//                                        instructions of a wave, so waiting for it hides behind
//                                        the weight stream.
//
// Hand-over of t inside one launch.  Every t[j] travels as one 8-byte word {value, tag}; the tag
// identifies the launch (AQL dispatch id mixed with the queue address: distinct for every launch,
// also for every replay of a captured graph, identical for all blocks of one launch).  Consumers
// poll the words they need until the tags match: no flag, no counter, no atomic read-modify-write
// (each costs microseconds across the eight L2s) and nothing to reset afterwards.  Words are
// written and read with device-scope (sc1) accesses, which do not linger in a per-XCD L2.
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

// v + (v moved across lanes by a DPP control); lanes the move does not reach add zero.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v)
{
    const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, false);
    return v + __builtin_bit_cast(float, moved);
}

// Sum over the 64 lanes of a wave, returned wave-uniform.  Butterfly inside each row of 16 lanes,
// then row 0 -> 1, 2 -> 3 (row_bcast:15) and rows 0+1 -> 2, 3 (row_bcast:31); lane 63 has the total.
__device__ __forceinline__ float wave_sum(float v)
{
    v = dpp_add<0xB1, 0xF>(v);    // quad_perm [1,0,3,2]
    v = dpp_add<0x4E, 0xF>(v);    // quad_perm [2,3,0,1]
    v = dpp_add<0x141, 0xF>(v);   // row_half_mirror
    v = dpp_add<0x140, 0xF>(v);   // row_mirror
    v = dpp_add<0x142, 0xA>(v);   // row_bcast:15 into rows 1 and 3
    v = dpp_add<0x143, 0xC>(v);   // row_bcast:31 into rows 2 and 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// ------------------------------------------------------------------ activations in registers

// The lane's 32 activations of one chunk as the 16 pairs matching the code extraction order, and
// their plain sum.  INT4: word j holds codes 8j..8j+7 and yields pairs (0,4) (1,5) (2,6) (3,7).
// INT3: word w holds codes 10w..10w+9 and yields pairs (f, f+5), f = 0..4; codes 30, 31 pair up.
template <int BITS>
struct XFrag {
    half2_t p[16];
    float sum;

    // raw: 32 consecutive fp16 activations as loaded; valid == false gives an all-zero fragment
    __device__ __forceinline__ void arrange(const uint4 (&raw)[4], bool valid)
    {
        half_t v[32];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t w[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const half2_t h = as_h2(valid ? w[j] : 0u);
                v[i * 8 + j * 2] = h.x;
                v[i * 8 + j * 2 + 1] = h.y;
            }
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
    __device__ __forceinline__ float dot(const half2_t (&p)[16]) const { return dot_codes_int4(w, p); }
};
template <>
struct CodeWords<3> {
    uint32_t w[3];
    __device__ __forceinline__ void load(const uint32_t *p)
    {
        w[0] = p[0]; w[1] = p[1]; w[2] = p[2];
    }
    __device__ __forceinline__ float dot(const half2_t (&p)[16]) const { return dot_codes_int3(w, p); }
};

// ------------------------------------------------------------------ fused GEMV kernel

struct GemvParams {
    const uint32_t *qw;
    const uint16_t *scales;
    const uint16_t *zeros;
    const uint16_t *At;   // [r][K]
    const uint16_t *Bt;   // [N][r]
    const uint16_t *x;    // [M][K]
    uint16_t *y;          // [M][N]
    uint64_t *ttag;       // workspace: [M][r] words {fp32 value (low half), launch tag (high half)}
    int M, N, K, r;
    int row_words;        // words per packed row
    int G;                // groups per row
    int producers;        // producer blocks at the front of the grid (0 when r == 0)
};

constexpr int kProdCols = 4;          // columns of A per producer block
constexpr int kSpinLimit = 1 << 15;   // polls (~0.3 us each) before a wave gives up and computes t itself
constexpr int kCacheSc1 = 16 | (1 << 31);   // buffer-load policy: device scope (sc1), and volatile so that a poll is never hoisted or merged

extern "C" __device__ unsigned long long fbq_llvm_dispatch_id(void) __asm("llvm.amdgcn.dispatch.id");

// Identity of this launch, the same in every block: never zero, so a zero-filled workspace never matches.
__device__ __forceinline__ uint32_t launch_tag()
{
    const uint64_t id = fbq_llvm_dispatch_id();
    const uint64_t q = (uint64_t)__builtin_amdgcn_queue_ptr();
    const uint32_t tag = (uint32_t)id + (uint32_t)(q >> 6) * 0x9E3779B1u;
    return tag ? tag : 0x80000000u;
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t dev_buffer(const void *p, int bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, bytes, 0x00020000);
}

typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));

// Producer block b of token m: t[j] for its kProdCols columns, lanes along K like the main kernel.
__device__ void produce_t(const GemvParams &p, int m, int b, uint32_t tag, float *lds)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint16_t *xrow = p.x + (size_t)m * p.K;
    const int j0 = b * kProdCols;
    float acc[kProdCols];
#pragma unroll
    for (int c = 0; c < kProdCols; ++c) acc[c] = 0.0f;
#pragma unroll 2
    for (int k0 = tid * 8; k0 < p.K; k0 += 256 * 8) {
        const uint4 xv = *reinterpret_cast<const uint4 *>(xrow + k0);
        uint4 av[kProdCols];
#pragma unroll
        for (int c = 0; c < kProdCols; ++c) {
            const int j = min(j0 + c, p.r - 1);         // r is a multiple of 8: never clamps, keeps loads unconditional
            av[c] = *reinterpret_cast<const uint4 *>(p.At + (size_t)j * p.K + k0);
        }
#pragma unroll
        for (int c = 0; c < kProdCols; ++c) {
            acc[c] = dot2(av[c].x, as_h2(xv.x), acc[c]);
            acc[c] = dot2(av[c].y, as_h2(xv.y), acc[c]);
            acc[c] = dot2(av[c].z, as_h2(xv.z), acc[c]);
            acc[c] = dot2(av[c].w, as_h2(xv.w), acc[c]);
        }
    }
#pragma unroll
    for (int c = 0; c < kProdCols; ++c) {
        const float s = wave_sum(acc[c]);
        if (lane == 0) lds[wave * kProdCols + c] = s;
    }
    __syncthreads();
    if (tid < kProdCols && j0 + tid < p.r) {
        const float s = (lds[tid] + lds[kProdCols + tid]) + (lds[2 * kProdCols + tid] + lds[3 * kProdCols + tid]);
        const uint64_t word = (uint64_t)__builtin_bit_cast(uint32_t, s) | ((uint64_t)tag << 32);
        __hip_atomic_store(p.ttag + (size_t)m * p.r + j0 + tid, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// BITS: 3 or 4.  CPW: chunks (of 2048 codes) per wave.  KS: waves of a block that split K.
// ROWS: rows per wave.  RI: ceil(r/128), 0 = branch-free twin.
template <int BITS, int CPW, int KS, int ROWS, int RI>
__global__ __launch_bounds__(256) void fbq_gemv_kernel(const GemvParams p)
{
    constexpr int kWaves = 4;
    constexpr int kRowSets = kWaves / KS;               // row sets per block
    constexpr int kLaneWords = BITS == 4 ? 4 : 3;
    constexpr int kRI = RI > 0 ? RI : 1;
    __shared__ float red[kWaves * (ROWS > kProdCols ? ROWS : kProdCols)];   // K-split sums, or the producer's wave sums

    const int m = blockIdx.y;
    int bx = blockIdx.x;
    uint32_t tag = 0;
    if (RI > 0) {
        tag = launch_tag();
        if (bx < p.producers) {                         // block-uniform: producer blocks only produce
            produce_t(p, m, bx, tag, red);
            return;
        }
        bx -= p.producers;
    }

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int ks = wave % KS;                           // which K slice
    const int rs = wave / KS;                           // which row set of the block
    const int n0 = (bx * kRowSets + rs) * ROWS;

    // Every load below is unconditional (addresses clamped into the tensors) so that the whole
    // wave's traffic is in flight before anything waits; clamped lanes are zeroed afterwards.
    int kc[CPW];
    bool kv[CPW];
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
        const int k0 = ((ks * CPW + c) * 64 + lane) * kLaneCodes;
        kv[c] = k0 < p.K;
        kc[c] = kv[c] ? k0 : 0;
    }
    int jc[kRI];
    bool jv[kRI];
#pragma unroll
    for (int q = 0; q < kRI; ++q) {
        const int j = (q * 64 + lane) * 2;
        jv[q] = RI > 0 && j < p.r;
        jc[q] = jv[q] ? j : 0;
    }

    uint4 xraw[CPW][4];
    const uint16_t *xrow = p.x + (size_t)m * p.K;
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
        const uint4 *src = reinterpret_cast<const uint4 *>(xrow + kc[c]);
#pragma unroll
        for (int i = 0; i < 4; ++i) xraw[c][i] = src[i];
    }

    CodeWords<BITS> cw[ROWS][CPW];
    uint16_t sc[ROWS][CPW], zp[ROWS][CPW];
    uint32_t bt[ROWS][kRI];
#pragma unroll
    for (int i = 0; i < ROWS; ++i) {
        const int n = min(n0 + i, p.N - 1);             // rows past the end re-read the last row; never stored
        const uint32_t *qrow = p.qw + (size_t)n * p.row_words;
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            cw[i][c].load(qrow + (kc[c] / kLaneCodes) * kLaneWords);
            sc[i][c] = p.scales[(size_t)n * p.G + kc[c] / kGroup];
            zp[i][c] = p.zeros[(size_t)n * p.G + kc[c] / kGroup];
        }
        if (RI > 0) {
#pragma unroll
            for (int q = 0; q < RI; ++q) bt[i][q] = *reinterpret_cast<const uint32_t *>(p.Bt + (size_t)n * p.r + jc[q]);
        }
    }

    // One early look at t: if the producers are already done it is in hand before the arithmetic.
    // A lane needs t[j], t[j+1]: one 16-byte device-scope load {value, tag, value, tag}.
    const __amdgpu_buffer_rsrc_t tbuf = dev_buffer(p.ttag + (size_t)m * p.r, (RI > 0 ? p.r : 1) * 8);
    uint4_t tw[kRI];
    bool ready = false;
    if (RI > 0 && ks == 0) {
        bool ok = true;
#pragma unroll
        for (int q = 0; q < RI; ++q) {
            tw[q] = __builtin_amdgcn_raw_buffer_load_b128(tbuf, jc[q] * 8, 0, kCacheSc1);
            ok = ok && (!jv[q] || (tw[q].y == tag && tw[q].w == tag));
        }
        ready = __all(ok);
    }

    XFrag<BITS> xf[CPW];
#pragma unroll
    for (int c = 0; c < CPW; ++c) xf[c].arrange(xraw[c], kv[c]);

    // main path: de-quantize and multiply; clamped lanes hold zero activations and add nothing
    float acc[ROWS];
#pragma unroll
    for (int i = 0; i < ROWS; ++i) {
        float a = 0.0f;
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            const float qx = cw[i][c].dot(xf[c].p);
            const float s = (float)__builtin_bit_cast(half_t, sc[i][c]);
            const float z = (float)__builtin_bit_cast(half_t, zp[i][c]);
            a = fmaf(s, fmaf(-z, xf[c].sum, qx), a);
        }
        acc[i] = a;
    }

    // up-projection into the same accumulators (the K-slice-0 wave of each row set only)
    if (RI > 0 && ks == 0) {
        float t0[kRI], t1[kRI];
        if (!ready) {
#pragma unroll
            for (int i = 0; i < ROWS; ++i) asm volatile("" : "+v"(acc[i]));   // finish the arithmetic before waiting
            for (int it = 0; it < kSpinLimit && !ready; ++it) {
                bool ok = true;
#pragma unroll
                for (int q = 0; q < RI; ++q) {
                    tw[q] = __builtin_amdgcn_raw_buffer_load_b128(tbuf, jc[q] * 8, 0, kCacheSc1);
                    ok = ok && (!jv[q] || (tw[q].y == tag && tw[q].w == tag));
                }
                ready = __all(ok);
                if (!ready) __builtin_amdgcn_s_sleep(2);
            }
        }
#pragma unroll
        for (int q = 0; q < RI; ++q) {
            if (ready) {
                const uint32_t v0 = tw[q].x, v1 = tw[q].z;   // scalars first: bit_cast of a vector component reads the wrong lane
                t0[q] = __builtin_bit_cast(float, v0);
                t1[q] = __builtin_bit_cast(float, v1);
            } else {                                    // producers never showed up in time: do it here
                t0[q] = t1[q] = 0.0f;
                const uint16_t *a0 = p.At + (size_t)jc[q] * p.K, *a1 = a0 + p.K;
                for (int k = 0; k < p.K; ++k) {
                    const float xv = (float)__builtin_bit_cast(half_t, xrow[k]);
                    t0[q] = fmaf(xv, (float)__builtin_bit_cast(half_t, a0[k]), t0[q]);
                    t1[q] = fmaf(xv, (float)__builtin_bit_cast(half_t, a1[k]), t1[q]);
                }
            }
            const float u0 = jv[q] ? t0[q] : 0.0f, u1 = jv[q] ? t1[q] : 0.0f;
#pragma unroll
            for (int i = 0; i < ROWS; ++i) {
                const half2_t b = as_h2(bt[i][q]);
                acc[i] = fmaf(u0, (float)b.x, acc[i]);
                acc[i] = fmaf(u1, (float)b.y, acc[i]);
            }
        }
    }

    float out = 0.0f;   // lane i of the wave ends up holding row n0 + i
#pragma unroll
    for (int i = 0; i < ROWS; ++i) {
        const float tot = wave_sum(acc[i]);
        if (lane == i) out = tot;
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
    if (ks == 0 && lane < ROWS && n0 + lane < p.N)
        p.y[(size_t)m * p.N + n0 + lane] = __builtin_bit_cast(uint16_t, (half_t)out);
}

// ------------------------------------------------------------------ dispatch

template <int BITS, int CPW, int KS, int ROWS>
static hipError_t launch_gemv_ri(const GemvParams &p, hipStream_t stream)
{
    constexpr int kRowSets = 4 / KS;
    const dim3 grid(ceil_div(p.N, kRowSets * ROWS) + p.producers, p.M);
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

size_t decode_workspace_bytes(int M, int r) { return (size_t)M * r * sizeof(uint64_t); }

hipError_t launch_gemv_decode(const LinearArgs &a, hipStream_t stream)
{
    GemvParams p;
    p.qw = a.qw; p.scales = a.scales; p.zeros = a.zeros; p.At = a.At; p.Bt = a.Bt; p.x = a.x; p.y = a.y;
    p.M = a.M; p.N = a.N; p.K = a.K; p.r = a.r;
    p.row_words = (int)row_words(a.K, a.bits);
    p.G = a.K / kGroup;
    p.producers = ceil_div(a.r, kProdCols);
    p.ttag = (uint64_t *)a.workspace;
    return a.bits == 4 ? launch_gemv_bits<4>(p, stream) : launch_gemv_bits<3>(p, stream);
}

}  // namespace fbq
