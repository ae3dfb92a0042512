// Decode path for one or two tokens: the fused kernel of Sec. 4.3 as a memory-streaming GEMV for gfx950.
//
//   down-projection   t = x.A            inside the SAME launch: each of the first r blocks takes one
//                                        column of A as a small job before its first tile (the paper keeps it a separate small kernel;
//                                        on this GPU a launch costs as much as streaming a 4096^2
//                                        layer, so it rides along, and it holds no block slot)
//   fused kernel      y = x.Wq^T + t.B   one pass over the packed codes; de-quantization, main
//                                        projection and up-projection share one fp32 accumulator
//                                        and y is written once.  t is needed only for the second
//                                        half of a tile (up-projection, sum, store), which is
//                                        postponed by one trip, so waiting for it hides behind
//                                        the weight stream.
//
// Hand-over of t inside one launch.  Every t[j] travels as one 8-byte word {value, tag}; the tag
// identifies the launch (AQL dispatch id mixed with the queue address: distinct for every launch,
// also for every replay of a captured graph, identical for all blocks of one launch).  Consumers
// poll the words they need until the tags match: no flag, no counter, no atomic read-modify-write
// (each costs microseconds across the eight L2s) and nothing to reset afterwards.  Words are
// written and read with device-scope (sc1) accesses, which do not linger in a per-XCD L2.
//
// Work decomposition of the fused kernel.  Waves are persistent: a wave owns a contiguous K range
// and walks over tiles of ROWS consecutive output rows with a fixed stride, with two tile buffers in
// registers: a buffer is requested again, for the tile two trips ahead, as soon as its arithmetic is
// done.  Its 64 lanes lie along K.  One wave-wide load covers 2048
// codes (INT4: 16 B per lane, INT3: 12 B per lane, both fully coalesced), so a lane always holds
// 32 consecutive codes of one quantization group.  The token's activations are fetched once per
// block, handed to the waves through LDS and stay in registers for every tile (they are the same
// for every row), pre-arranged as the fp16 pairs that the code extraction produces.  One launch can
// serve several layers with the same K (q/k/v, gate/up): grid.y is the layer, and blocks are shared
// out in proportion to the layers' sizes.
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
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));
typedef uint32_t uint3_t __attribute__((ext_vector_type(3)));

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

    // 32 consecutive fp16 values as loaded -> the 16 pairs in extraction order (also used for a column of A,
    // so that its dot product with the activations can run on the pairs the wave already holds)
    static __device__ __forceinline__ void pairs(const uint4 (&raw)[4], bool valid, half2_t (&p)[16], half_t (&v)[32])
    {
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

    // raw: 32 consecutive fp16 activations as loaded; valid == false gives an all-zero fragment
    __device__ __forceinline__ void arrange(const uint4 (&raw)[4], bool valid)
    {
        half_t v[32];
        pairs(raw, valid, p, v);
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < 32; ++i) s += (float)v[i];
        sum = s;
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
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t buf, int lane_off, int row_off)
    {
        const uint4_t q = __builtin_amdgcn_raw_buffer_load_b128(buf, lane_off, row_off, 0);
        w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w;
    }
    __device__ __forceinline__ float dot(const half2_t (&p)[16]) const { return dot_codes_int4(w, p); }
};
template <>
struct CodeWords<3> {
    uint32_t w[3];
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t buf, int lane_off, int row_off)
    {
        const uint3_t q = __builtin_amdgcn_raw_buffer_load_b96(buf, lane_off, row_off, 0);
        w[0] = q.x; w[1] = q.y; w[2] = q.z;
    }
    __device__ __forceinline__ float dot(const half2_t (&p)[16]) const { return dot_codes_int3(w, p); }
};

// ------------------------------------------------------------------ fused GEMV kernel

struct LayerParams {
    const uint32_t *qw;
    const uint16_t *scales;
    const uint16_t *zeros;
    const uint16_t *At;   // [r][K]
    const uint16_t *Bt;   // [N][r]
    const uint16_t *x;    // [M][K]
    uint16_t *y;          // [M][N]
    uint64_t *ttag;       // workspace: [M][tslices][r] words {fp32 partial sum (low half), launch tag (high half)}
    int N, K, r;
    int row_words;        // words per packed row
    int G;                // groups per row
    int tslices;          // K slices of the down-projection = waves of a block that split K (1, 2 or 4); consumers add the partial sums
    int blocks;           // blocks of this layer
    int spin_limit;       // polls for t before a wave computes it itself; negative: at once (test hook)
};

struct GemvGroup {
    LayerParams layer[kMaxGroup];
};

constexpr int kNowhere = 1 << 30;     // a byte offset beyond any buffer a layer has
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

// Everything one wave loads for one tile of ROWS rows.  All loads are buffer loads: the row base is a
// scalar offset (the rows of a tile are the same for every lane), the lane's position inside a row is
// a byte offset computed once, and a tile that is not wanted is "loaded" through descriptors of size
// zero, which answer zero without touching memory - so every wave issues the same number of loads
// on every trip and the compiler can count exactly how many loads are younger than the data it
// waits for.
struct TileBuffers {
    __amdgpu_buffer_rsrc_t qw, scales, zeros, bt;
};

__device__ __forceinline__ TileBuffers tile_buffers(const LayerParams &p, bool enabled)
{
    TileBuffers b;
    const int on = enabled ? 1 : 0;   // sizes fit 32 bits: K <= 32768 and the rows of one layer stay far below 2^31 bytes
    b.qw = dev_buffer(p.qw, on * (int)((size_t)p.N * p.row_words * 4));
    b.scales = dev_buffer(p.scales, on * p.N * p.G * 2);
    b.zeros = dev_buffer(p.zeros, on * p.N * p.G * 2);
    b.bt = dev_buffer(p.Bt, on * p.N * p.r * 2);
    return b;
}

template <int BITS, int CPW, int ROWS>
struct RowTile {
    static constexpr int kLaneWords = BITS == 4 ? 4 : 3;
    CodeWords<BITS> cw[ROWS][CPW];
    uint32_t sc[ROWS][CPW], zp[ROWS][CPW];   // fp16 bits, one per register: packing two would stall the load stream

    // Rows past the end re-read the last row (never stored); lanes past K aim beyond the buffer and get
    // zeros (their activations are zero too).  qoff: byte offset of the lane's words inside a packed row, goff: of its
    // group's scale / zero inside a row of scales.
    __device__ __forceinline__ void load(const LayerParams &p, const TileBuffers &b, int n0, const int (&qoff)[CPW], const int (&goff)[CPW])
    {
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            const int n = min(n0 + i, p.N - 1);
#pragma unroll
            for (int c = 0; c < CPW; ++c) {
                cw[i][c].load(b.qw, qoff[c], n * p.row_words * 4);
                sc[i][c] = __builtin_amdgcn_raw_buffer_load_b16(b.scales, goff[c], n * p.G * 2, 0);
                zp[i][c] = __builtin_amdgcn_raw_buffer_load_b16(b.zeros, goff[c], n * p.G * 2, 0);
            }
        }
    }
};

// The lane's two taps of each of the tile's ROWS rows of Bt (taps past r aim beyond the buffer and read as zero; their t is zero too).
template <int ROWS, int RI>
__device__ __forceinline__ void load_taps(uint32_t (&bt)[ROWS][RI], const LayerParams &p, const TileBuffers &b, int n0, const int (&joff)[RI])
{
#pragma unroll
    for (int i = 0; i < ROWS; ++i) {
        const int n = min(n0 + i, p.N - 1);
#pragma unroll
        for (int q = 0; q < RI; ++q) bt[i][q] = __builtin_amdgcn_raw_buffer_load_b32(b.bt, joff[q], n * p.r * 2, 0);
    }
}

// Where a wave covers four chunks of K the kernel has no registers to spare for a column of A next to its tiles:
// there the first blocks of a layer do nothing but the down-projection (one column per row set of the block, each
// wave over its own K range, everything in natural order straight from memory) and leave.
template <int CPW, int KS>
__device__ __forceinline__ void job_only_block(const LayerParams &p, int m, int bx, int wave, int lane, uint32_t tag)
{
    const int ks = wave % KS;
    const int jcol = bx * (4 / KS) + wave / KS;          // one column per row set of the block
    if (jcol >= p.r) return;
    const __amdgpu_buffer_rsrc_t abuf = dev_buffer(p.At, p.r * p.K * 2);
    const __amdgpu_buffer_rsrc_t xbuf = dev_buffer(p.x + (size_t)m * p.K, p.K * 2);
    __builtin_amdgcn_s_setprio(3);                      // every other block of the layer waits for these words
    uint4_t xr[CPW][4], ar[CPW][4];
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            // a wave-wide load covers 512 consecutive activations: fully coalesced, x and the column alike
            const int k0 = ks * CPW * kChunk + ((c * 4 + i) * 64 + lane) * 8;
            const int off = k0 < p.K ? k0 * 2 : kNowhere;    // past K: zeros from both buffers
            xr[c][i] = __builtin_amdgcn_raw_buffer_load_b128(xbuf, off, 0, 0);
            ar[c][i] = __builtin_amdgcn_raw_buffer_load_b128(abuf, off, jcol * p.K * 2, 0);
        }
    }
    float tj = 0.0f;
#pragma unroll
    for (int c = 0; c < CPW; ++c)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            tj = dot2(ar[c][i].x, as_h2(xr[c][i].x), tj);
            tj = dot2(ar[c][i].y, as_h2(xr[c][i].y), tj);
            tj = dot2(ar[c][i].z, as_h2(xr[c][i].z), tj);
            tj = dot2(ar[c][i].w, as_h2(xr[c][i].w), tj);
        }
    tj = wave_sum(tj);
    if (lane == 0) {
        const uint64_t word = (uint64_t)__builtin_bit_cast(uint32_t, tj) | ((uint64_t)tag << 32);
        __hip_atomic_store(p.ttag + ((size_t)m * p.tslices + ks) * p.r + jcol, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// BITS: 3 or 4.  CPW: chunks (of 2048 codes) per wave.  KS: waves of a block that split K.
// ROWS: rows per tile.  RI: ceil(r/128), 0 = branch-free twin.
template <int BITS, int CPW, int KS, int ROWS, int RI>
__global__ __launch_bounds__(256) void fbq_gemv_kernel(const GemvGroup g)
{
    constexpr int kWaves = 4;
    constexpr int kRowSets = kWaves / KS;               // row sets per block
    constexpr int kRI = RI > 0 ? RI : 1;
    constexpr int kXChunks = CPW * KS;                  // chunks of 2048 activations the block covers
    __shared__ float red[kWaves * ROWS];                                    // K-split sums
    __shared__ uint4 x_lds[kXChunks * 256];                                 // the token's activations, 16-byte pieces swizzled

    // Grid: x = layer of the group, y = block of the layer, z = token: blocks are dispatched x first, so the first
    // blocks of every layer - the ones with a share of the down-projection - start before anybody's later blocks.
    // The layer comes from the block index, not from a table in the kernel arguments: its parameters
    // are then fetched in one go with everything else (a second, dependent round trip to the kernel
    // arguments costs more than half a microsecond here).  Layers with fewer blocks than the widest
    // one of the group leave the surplus blocks at once.
    const int m = blockIdx.z;
    const LayerParams p = g.layer[blockIdx.x];
    // (all of them before the first branch: left alone, the compiler fetches only what the branch needs first)
    asm volatile("" :: "s"(p.qw), "s"(p.scales), "s"(p.zeros), "s"(p.x), "s"(p.y), "s"(p.N), "s"(p.K), "s"(p.row_words), "s"(p.G));
    if (RI > 0) asm volatile("" :: "s"(p.At), "s"(p.Bt), "s"(p.ttag), "s"(p.r), "s"(p.tslices), "s"(p.spin_limit));
    constexpr bool kInlineJob = CPW <= 3;               // else: the first r blocks do the down-projection and nothing else
    int bx = blockIdx.y;
    const int job_blocks = RI > 0 && !kInlineJob ? (p.r + kRowSets - 1) / kRowSets : 0;
    if (bx >= p.blocks + job_blocks) return;
    const uint32_t tag = RI > 0 ? launch_tag() : 0u;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same in all lanes: lets row offsets live in scalar registers
    if (RI > 0 && !kInlineJob) {
        if (bx < job_blocks) {                          // block-uniform
            job_only_block<CPW, KS>(p, blockIdx.z, bx, wave, lane, tag);
            return;
        }
        bx -= job_blocks;
    }
    const int ks = wave % KS;                           // which K slice
    const int rs = wave / KS;                           // which row set of the block
    const int ntiles = (p.N + ROWS - 1) / ROWS;
    const int tstride = p.blocks * kRowSets;
    const int trips = (ntiles - bx * kRowSets + tstride - 1) / tstride;   // block-uniform; < 1 only in blocks launched for their share of the down-projection alone
    int tile = bx * kRowSets + rs;

    // The token's activations: the block fetches them once (each thread 16 bytes per chunk) ...
    const uint16_t *xrow = p.x + (size_t)m * p.K;
    uint4 xin[kXChunks];
#pragma unroll
    for (int i = 0; i < kXChunks; ++i) {
        const int k = (i * 256 + tid) * 8;
        xin[i] = k < p.K ? *reinterpret_cast<const uint4 *>(xrow + k) : make_uint4(0u, 0u, 0u, 0u);
    }

    // ... and right behind them the first tile goes out, before anything waits.
    int qoff[CPW], goff[CPW], koff[CPW];
    bool kv[CPW];
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
        const int k0 = ((ks * CPW + c) * 64 + lane) * kLaneCodes;
        kv[c] = k0 < p.K;
        // lanes past K aim beyond every buffer (no layer's codes reach 2^30 bytes): the buffer unit answers zero
        // without touching memory, and the lane's activations are zero as well
        koff[c] = kv[c] ? k0 * 2 : kNowhere;            // the same position in a row of fp16 values (a column of A)
        qoff[c] = kv[c] ? (k0 / kLaneCodes) * RowTile<BITS, CPW, ROWS>::kLaneWords * 4 : kNowhere;
        goff[c] = kv[c] ? (k0 / kGroup) * 2 : kNowhere;
    }
    int joff[kRI];
    bool jv[kRI];
#pragma unroll
    for (int q = 0; q < kRI; ++q) {
        const int j = (q * 64 + lane) * 2;
        jv[q] = RI > 0 && j < p.r;
        joff[q] = jv[q] ? j * 2 : kNowhere;
    }
    // Down-projection.  Column j of A is a job for block j of the layer: the waves of its first row set take it,
    // each over its own K range.  So the first r blocks of a layer - the first in dispatch order - do all of it, a
    // sliver each, and nobody holds a block slot for it.  (A compute unit fetches at its share of the memory
    // system's pace, about 20 KB per microsecond when the whole GPU streams: four columns of a 4096-wide A on one
    // compute unit would keep t back by more than a microsecond, one column does not.)  The column's words are
    // asked for BEFORE the first tile: loads come back in the order they were made, and every other block waits
    // for t.
    const int jcol = bx;
    const bool has_job = RI > 0 && kInlineJob && rs == 0 && jcol < p.r;   // wave-uniform
    uint4 acol[CPW][4];
    if (has_job) {
        const __amdgpu_buffer_rsrc_t abuf = dev_buffer(p.At, p.r * p.K * 2);
#pragma unroll
        for (int c = 0; c < CPW; ++c)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint4_t v = __builtin_amdgcn_raw_buffer_load_b128(abuf, koff[c] + i * 16, jcol * p.K * 2, 0);
                acol[c][i] = make_uint4(v.x, v.y, v.z, v.w);
            }
    }
    RowTile<BITS, CPW, ROWS> cur, nxt;                  // even and odd trips
    uint32_t bt0[ROWS][kRI], bt1[ROWS][kRI];            // their rows of Bt
    cur.load(p, tile_buffers(p, true), min(tile, ntiles - 1) * ROWS, qoff, goff);
    if (RI > 0) load_taps<ROWS, kRI>(bt0, p, tile_buffers(p, ks == 0), min(tile, ntiles - 1) * ROWS, joff);   // only the K-slice-0 wave applies them
    __builtin_amdgcn_sched_barrier(0);

    // Activations into LDS (piece j at j ^ ((j >> 4) & 3): the 16 lanes of a quarter wave then read 16
    // different bank groups), and from there the wave's K range into registers, used for every tile.
#pragma unroll
    for (int i = 0; i < kXChunks; ++i) {
        const int j = i * 256 + tid;
        x_lds[j ^ ((j >> 4) & 3)] = xin[i];
    }
    __syncthreads();
    XFrag<BITS> xf[CPW];
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
        uint4 raw[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int j = ((ks * CPW + c) * 64 + lane) * 4 + i;
            raw[i] = x_lds[j ^ ((j >> 4) & 3)];
        }
        xf[c].arrange(raw, kv[c]);
    }
    // The job: t[jcol] over this wave's K range, on the pairs the wave holds anyway (lanes past K hold zeros),
    // summed over the wave in a fixed order and handed over as one tagged word.
    const int tslices = RI > 0 ? p.tslices : 1;
    auto t_partial = [&](const uint4 (&col)[CPW][4]) __attribute__((always_inline)) {
        float tj = 0.0f;
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            half2_t ap[16];
            half_t unused[32];
            XFrag<BITS>::pairs(col[c], true, ap, unused);
#pragma unroll
            for (int q = 0; q < 16; ++q) tj = __builtin_amdgcn_fdot2(ap[q], xf[c].p[q], tj, false);
        }
        return wave_sum(tj);
    };
    auto hand_over = [&](int j, float tj) __attribute__((always_inline)) {
        if (lane == 0) {
            const uint64_t word = (uint64_t)__builtin_bit_cast(uint32_t, tj) | ((uint64_t)tag << 32);
            __hip_atomic_store(p.ttag + ((size_t)m * tslices + ks) * p.r + j, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };
    if (RI > 0) {
        if (has_job) hand_over(jcol, t_partial(acol));
        if (trips <= 0) return;                         // a block that exists for its job only (a layer with a handful of rows)
    }
    // The second tile goes out only now: the memory pipeline serves a compute unit's requests in the
    // order they were made, and the first tiles of all its waves should come before any second tile.
#pragma unroll
    for (int c = 0; c < CPW; ++c) asm volatile("" : "+v"(xf[c].sum));
    __builtin_amdgcn_sched_barrier(0);
    nxt.load(p, tile_buffers(p, trips > 1), min(tile + tstride, ntiles - 1) * ROWS, qoff, goff);
    __builtin_amdgcn_sched_barrier(0);

    // t: a lane needs t[j], t[j+1]: one 16-byte device-scope load {value, tag, value, tag}.  With several
    // K slices there is one such word pair per slice, and the lane adds the partial sums.
    const __amdgpu_buffer_rsrc_t tbuf = dev_buffer(p.ttag + (size_t)m * tslices * p.r, (RI > 0 ? tslices * p.r : 1) * 8);
    uint4_t tw[kRI][kMaxTSlices];
    float t0[kRI], t1[kRI];
    bool have_t = false;
    auto request_t = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < RI; ++q)
#pragma unroll
            for (int sl = 0; sl < kMaxTSlices; ++sl)
                // lanes without a tap, and slices the layer does not have, aim past the end: the buffer unit answers zero without touching memory
                tw[q][sl] = __builtin_amdgcn_raw_buffer_load_b128(tbuf, jv[q] && sl < tslices ? (sl * p.r) * 8 + joff[q] * 4 : tslices * p.r * 8, 0, kCacheSc1);
    };
    auto t_arrived = [&]() __attribute__((always_inline)) {
        bool ok = true;
#pragma unroll
        for (int q = 0; q < RI; ++q)
#pragma unroll
            for (int sl = 0; sl < kMaxTSlices; ++sl)
                if (sl < tslices) ok = ok && (!jv[q] || (tw[q][sl].y == tag && tw[q][sl].w == tag));
        return (bool)__all(ok);
    };

    // Every wave that applies the up-projection (the K-slice-0 wave of each row set) takes t for itself - asked for
    // one tile earlier, see below - and waits if it is not there yet: no barrier, so a wave whose tiles come early
    // is not held back to the pace of the slowest wave of its block.
    const bool needs_t = RI > 0 && ks == 0;             // wave-uniform
    auto take_t = [&]() __attribute__((always_inline)) {
        if (needs_t) {
            bool ready = p.spin_limit >= 0 && t_arrived();
            // Not there yet: every wave of the launch would now ask for the same few hundred bytes over and over, and
            // the one memory channel that holds them also serves its share of everybody's weights.  So a poll asks
            // for a single word - the one stored by the last wave in dispatch order that has a job - and only when
            // that has come is all of t asked for again.
            for (int spin = 0; spin < p.spin_limit && !ready; ++spin) {
                const uint32_t probe_tag = __builtin_amdgcn_raw_buffer_load_b32(tbuf, 0, (tslices * p.r - 1) * 8 + 4, kCacheSc1);
                if (probe_tag == tag) {
                    request_t();
                    ready = t_arrived();
                }
                if (!ready) __builtin_amdgcn_s_sleep(4);
            }
#pragma unroll
            for (int q = 0; q < RI; ++q) {
                float u0 = 0.0f, u1 = 0.0f;
                if (ready) {
#pragma unroll
                    for (int sl = 0; sl < kMaxTSlices; ++sl) {
                        if (sl < tslices) {
                            const uint32_t v0 = tw[q][sl].x, v1 = tw[q][sl].z;   // scalars first: bit_cast of a vector component reads the wrong lane
                            u0 += __builtin_bit_cast(float, v0);
                            u1 += __builtin_bit_cast(float, v1);
                        }
                    }
                } else {                            // the words never showed up in time: do it here
                    const uint16_t *a0 = p.At + (size_t)(jv[q] ? joff[q] / 2 : 0) * p.K, *a1 = a0 + p.K;   // lanes without a tap: column 0, ignored
                    for (int k = 0; k < p.K; ++k) {
                        const float xv = (float)__builtin_bit_cast(half_t, xrow[k]);
                        u0 = fmaf(xv, (float)__builtin_bit_cast(half_t, a0[k]), u0);
                        u1 = fmaf(xv, (float)__builtin_bit_cast(half_t, a1[k]), u1);
                    }
                }
                t0[q] = jv[q] ? u0 : 0.0f;
                t1[q] = jv[q] ? u1 : 0.0f;
            }
        }
        have_t = true;
    };

    // Second half of a tile: up-projection into the same accumulators (the K-slice-0 wave of each row
    // set only), sum over the wave (and over the K slices), one store per row.
    auto finish = [&](float (&acc)[ROWS], const uint32_t (&bt)[ROWS][kRI], int tile) __attribute__((always_inline)) {
        if (RI > 0 && ks == 0) {
#pragma unroll
            for (int q = 0; q < RI; ++q) {
#pragma unroll
                for (int i = 0; i < ROWS; ++i) {
                    const half2_t b = as_h2(bt[i][q]);
                    acc[i] = fmaf(t0[q], (float)b.x, acc[i]);
                    acc[i] = fmaf(t1[q], (float)b.y, acc[i]);
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
            __syncthreads();                            // previous trip's sums have been read
            if (lane < ROWS) red[wave * ROWS + lane] = out;
            __syncthreads();
            if (ks == 0 && lane < ROWS) {
                out = 0.0f;
#pragma unroll
                for (int q = 0; q < KS; ++q) out += red[(wave + q) * ROWS + lane];
            }
        }
        const int n0 = tile * ROWS;
        if (ks == 0 && lane < ROWS && tile < ntiles && n0 + lane < p.N)
            p.y[(size_t)m * p.N + n0 + lane] = __builtin_bit_cast(uint16_t, (half_t)out);
    };

    // One trip.  The tile's registers are refilled (with the tile two trips ahead, or with nothing) as
    // soon as the arithmetic has consumed them.  With a sub-branch the second half of a tile is
    // postponed by one trip: t is requested when the next tile's arithmetic starts and taken when it
    // ends, so waiting for the down-projection hides behind a whole tile of the weight stream (a wave with a
    // single trip has nothing to hide behind and waits at once).  Even trips use (cur, bt0, acc0), odd
    // trips (nxt, bt1, acc1): the rows of Bt for trip j + 1 are fetched in trip j, when the previous
    // owner of that buffer, trip j - 1, has been finished.
    float acc0[ROWS], acc1[ROWS];
    auto step = [&](RowTile<BITS, CPW, ROWS> &T, float (&acc)[ROWS], float (&acc_prev)[ROWS], uint32_t (&bt_mine)[ROWS][kRI],
                    uint32_t (&bt_prev)[ROWS][kRI], int j, int tile) __attribute__((always_inline)) {
        // main path: de-quantize and multiply; clamped lanes hold zero activations and add nothing
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            // t is asked for as late as possible - when the tile's first row has arrived and its arithmetic
            // is about to start - so that the answer is still fresh when the tile is done
            if (i == 1 && needs_t && !have_t && (j > 0 || trips == 1)) {
                asm volatile("" : "+v"(acc[0]));
                __builtin_amdgcn_sched_barrier(0);
                request_t();
                __builtin_amdgcn_sched_barrier(0);
            }
            float a = 0.0f;
#pragma unroll
            for (int c = 0; c < CPW; ++c) {
                const float qx = T.cw[i][c].dot(xf[c].p);
                const float s = (float)__builtin_bit_cast(half_t, (uint16_t)T.sc[i][c]);
                const float z = (float)__builtin_bit_cast(half_t, (uint16_t)T.zp[i][c]);
                a = fmaf(s, fmaf(-z, xf[c].sum, qx), a);
            }
            acc[i] = a;
        }
#pragma unroll
        for (int i = 0; i < ROWS; ++i) asm volatile("" : "+v"(acc[i]));   // the arithmetic is done before the registers are handed back
        __builtin_amdgcn_sched_barrier(0);
        T.load(p, tile_buffers(p, j + 2 < trips), min(tile + 2 * tstride, ntiles - 1) * ROWS, qoff, goff);
        __builtin_amdgcn_sched_barrier(0);
        if (RI == 0) {
            finish(acc, bt_mine, tile);
            return;
        }
        if (j > 0) {
            if (!have_t) take_t();
            finish(acc_prev, bt_prev, tile - tstride);
        }
        __builtin_amdgcn_sched_barrier(0);
        load_taps<ROWS, kRI>(bt_prev, p, tile_buffers(p, j + 1 < trips && ks == 0), min(tile + tstride, ntiles - 1) * ROWS, joff);
        __builtin_amdgcn_sched_barrier(0);
    };

    // trips is block-uniform; the loop body is straight-line, so the number of loads in flight at every
    // wait is known at compile time.
    int j = 0;
    for (; j + 1 < trips; j += 2) {
        step(cur, acc0, acc1, bt0, bt1, j, tile);
        step(nxt, acc1, acc0, bt1, bt0, j + 1, tile + tstride);
        tile += 2 * tstride;
    }
    if (j < trips) {
        step(cur, acc0, acc1, bt0, bt1, j, tile);
        tile += tstride;
    }
    if (RI > 0) {                                       // the last trip's second half
        if (!have_t) take_t();
        if (trips & 1) finish(acc0, bt0, tile - tstride);
        else finish(acc1, bt1, tile - tstride);
    }
}

// ------------------------------------------------------------------ dispatch

static int device_cu_count()
{
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
            n = 256;
        return n;
    }();
    return cus;
}

// Variant of the kernel a layer needs: it depends on K (chunks per wave, K split), bits and rank class.
struct Variant {
    int bits, cpw, ks, ri;
    bool operator==(const Variant &o) const { return bits == o.bits && cpw == o.cpw && ks == o.ks; }
};

static Variant variant_of(int K, int bits, int r)
{
    const int chunks = ceil_div(K, kChunk);
    Variant v{bits, 0, 0, ceil_div(r, 128)};
    if (chunks <= 4) { v.ks = 1; v.cpw = chunks; }
    else if (chunks <= 8) { v.ks = 2; v.cpw = ceil_div(chunks, 2); }
    else { v.ks = 4; v.cpw = ceil_div(chunks, 4) < 3 ? 3 : ceil_div(chunks, 4); }
    if (v.ks > 1 && v.cpw < 3) v.cpw = 3;
    return v;
}

template <int BITS, int CPW, int KS, int ROWS>
static hipError_t launch_ri(const GemvGroup &g, int ri, dim3 grid, hipStream_t stream)
{
    switch (ri) {
    case 0: hipLaunchKernelGGL((fbq_gemv_kernel<BITS, CPW, KS, ROWS, 0>), grid, dim3(256), 0, stream, g); break;
    case 1: hipLaunchKernelGGL((fbq_gemv_kernel<BITS, CPW, KS, ROWS, 1>), grid, dim3(256), 0, stream, g); break;
    default: hipLaunchKernelGGL((fbq_gemv_kernel<BITS, CPW, KS, ROWS, 2>), grid, dim3(256), 0, stream, g); break;
    }
    return hipGetLastError();
}

template <int BITS, int CPW, int KS>
static hipError_t launch_rows(const GemvGroup &g, int rows, int ri, dim3 grid, hipStream_t stream)
{
    if constexpr (CPW == 1) {                           // wider tiles only where a row is a single chunk
        if (rows == 4) return launch_ri<BITS, CPW, KS, 4>(g, ri, grid, stream);
    }
    return launch_ri<BITS, CPW, KS, 2>(g, ri, grid, stream);
}

template <int BITS>
static hipError_t launch_bits(const GemvGroup &g, const Variant &v, int rows, dim3 grid, hipStream_t stream)
{
    switch (v.ks * 10 + v.cpw) {
    case 11: return launch_rows<BITS, 1, 1>(g, rows, v.ri, grid, stream);
    case 12: return launch_rows<BITS, 2, 1>(g, rows, v.ri, grid, stream);
    case 13: return launch_rows<BITS, 3, 1>(g, rows, v.ri, grid, stream);
    case 14: return launch_rows<BITS, 4, 1>(g, rows, v.ri, grid, stream);
    case 23: return launch_rows<BITS, 3, 2>(g, rows, v.ri, grid, stream);
    case 24: return launch_rows<BITS, 4, 2>(g, rows, v.ri, grid, stream);
    case 43: return launch_rows<BITS, 3, 4>(g, rows, v.ri, grid, stream);
    case 44: return launch_rows<BITS, 4, 4>(g, rows, v.ri, grid, stream);
    }
    return hipErrorInvalidValue;   // K > 32768: rejected by the caller's shape check
}

static_assert((size_t)kPerTokenMaxM * kMaxTSlices * kMaxRank * sizeof(uint64_t) <= kStaticScratchBytes, "the static scratch must hold the largest GEMV hand-over");
// One tagged word per token, K slice (= wave of a block along K) and column of A.
size_t decode_workspace_bytes(int M, int K, int r) { return (size_t)M * variant_of(K, 4, r).ks * r * sizeof(uint64_t); }

// Layers may share a launch when they need the same kernel variant.  A branch-free layer never joins
// layers with a sub-branch: the fused kernel reads Bt unconditionally, and a branch-free layer has none.
bool decode_group_compatible(const LinearArgs &a, const LinearArgs &b)
{
    return variant_of(a.K, a.bits, a.r) == variant_of(b.K, b.bits, b.r) && a.M == b.M && (a.r > 0) == (b.r > 0);
}

hipError_t launch_gemv_decode(const LinearArgs *layers, int n_layers, hipStream_t stream)
{
    if (n_layers < 1 || n_layers > kMaxGroup) return hipErrorInvalidValue;
    Variant v = variant_of(layers[0].K, layers[0].bits, layers[0].r);
    const int M = layers[0].M;
    double total_work = 0.0;
    for (int i = 0; i < n_layers; ++i) {
        if (!decode_group_compatible(layers[0], layers[i])) return hipErrorInvalidValue;
        v.ri = std::max(v.ri, ceil_div(layers[i].r, 128));
        total_work += (double)layers[i].N * layers[i].K;
    }
    const int row_sets = 4 / v.ks;
    // Blocks to share out: two per CU keeps enough bytes in flight; a token dimension multiplies the grid.
    int budget = std::max(1, 2 * device_cu_count() / std::max(1, std::min(M, 2)));
    // Tiles of 4 rows when that still leaves every wave at least one tile, and registers allow; else 2.
    long tiles4 = 0, tiles = 0;
    for (int i = 0; i < n_layers; ++i) tiles4 += ceil_div(layers[i].N, 4);
    const int rows = (v.cpw == 1 && tiles4 >= (long)budget * row_sets) ? 4 : 2;
    // A launch in which no wave would get a second tile (one 4096 x 4096 layer) runs one block per CU instead, two
    // tiles per wave: half as many blocks fetch and arrange the activations, and the wait for t - which a wave
    // with a single tile has nothing to hide behind - disappears behind the second tile (5.0 -> 4.7 us with a
    // sub-branch, 4.1 -> 3.7 us without).
    for (int i = 0; i < n_layers; ++i) tiles += ceil_div(layers[i].N, rows);
    if (tiles <= (long)budget * row_sets && tiles > (long)budget * row_sets / 2) budget = std::max(1, budget / 2);

    // Where the down-projection has blocks of its own (see job_only_block) they come out of the same budget: the
    // other blocks have fixed tile lists and must all be resident from the start.
    const bool inline_job = v.cpw <= 3;
    if (!inline_job) {
        int job_blocks = 0;
        for (int i = 0; i < n_layers; ++i) job_blocks += ceil_div(layers[i].r, row_sets);
        budget = std::max(budget / 2, budget - job_blocks);
    }
    GemvGroup g;
    int widest = 0;
    for (int i = 0; i < n_layers; ++i) {
        const LinearArgs &a = layers[i];
        LayerParams &p = g.layer[i];
        p.qw = a.qw; p.scales = a.scales; p.zeros = a.zeros; p.At = a.At; p.Bt = a.Bt; p.x = a.x; p.y = a.y;
        p.ttag = (uint64_t *)a.workspace;
        p.N = a.N; p.K = a.K; p.r = a.r;
        p.row_words = (int)row_words(a.K, a.bits);
        p.G = a.K / kGroup;
        p.tslices = v.ks;
        p.spin_limit = spin_limit();
        const int max_blocks = ceil_div(ceil_div(a.N, rows), row_sets);
        const int share = (int)(budget * ((double)a.N * a.K / total_work));
        if (inline_job) {
            // every column of A needs a block: a layer with fewer row tiles than that gets blocks that only do their job
            p.blocks = std::max({1, std::min(max_blocks, share), a.r});
            widest = std::max(widest, p.blocks);
        } else {
            p.blocks = std::max(1, std::min(max_blocks, share));
            widest = std::max(widest, p.blocks + ceil_div(a.r, row_sets));  // blocks in front that only do the down-projection
        }
    }
    for (int i = n_layers; i < kMaxGroup; ++i) g.layer[i] = g.layer[0];   // never indexed: grid.x stops at n_layers
    const dim3 grid(n_layers, widest, M);
    return v.bits == 4 ? launch_bits<4>(g, v, rows, grid, stream) : launch_bits<3>(g, v, rows, grid, stream);
}

}  // namespace fbq
