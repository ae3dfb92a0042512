// Decode path for a few tokens (3 <= M <= 16): the fused kernel of Sec. 4.3 with the packed codes
// streamed exactly once, the tokens riding along as the 16 rows of a matrix-core tile.
//
//   y[M,N] = x[M,K] . Wq[N,K]^T + t[M,r] . B[r,N],   t = x . A
//
// One launch.  The first blocks of a grid row do the layer's down-projection and hand t over inside
// the launch (every partial sum travels as one 8-byte word {value, launch tag}, written and read at
// device scope: no flag, no fence, nothing to reset); all others stream weights from the start and
// ask for t only when their main part is done.  (The paper has a second launch there; on this GPU
// a launch boundary costs 4-5 us, a third of this kernel.)
//
// v_mfma_f32_16x16x32_f16 multiplies a 16 (token) x 32 (k) activation fragment with a 32 (k) x 16
// (output row) weight fragment.  Lane (c = lane % 16, q = lane / 16) supplies 8 values of k for
// token c in the first operand and for output row c in the second, and the instruction only needs
// both operands to agree on which k that is.
//
// Weights.  For one quantization group (128 codes) of 16 consecutive output rows, lane (c, q) needs
// the 32 codes k = 32 q .. 32 q + 31 of row c: one 16-byte (INT4) or 12-byte (INT3) load straight
// from the packed row into registers, no LDS memory in between (in most instances a neighbouring
// lane does the load, so that the four lanes of a load quad read one row, and the words change lanes
// afterwards).  A wave owns four consecutive groups, so the 16 row segments it reads are 256 (192)
// contiguous bytes each.  Masking a packed word with
// 0x000F000F and OR-ing 0x64006400 leaves two codes as the fp16 pair (1024 + q, 1024 + q'); fields
// that sit 4 (3, 6) bits higher come out as 1024 + 16 q (8 q, 64 q).  These go into the matrix
// instruction as they are: one v_and_or_b32 per two codes is all the de-quantization the inner
// loop does.
//
// Activations.  For every group, lane (c, q) reads the 32 activations k = 32 q .. 32 q + 31 of token c
// (four 16-byte loads, while the weights are under way) and re-orders them in registers into the four
// operands that meet its weight operands - divided by 16 (8, 64) where the weight field is scaled.
// A wave keeps the operands of its four groups in registers and walks over the block's row tiles
// with them, so a block reads the activations once, whatever the number of rows it owns.  Per group
// and token, X = sum x and XS = 1024 sum x' (x' the scaled activations) come from the matrix core as
// well: the operands against a column of ones, and against the column of field gains.
//
// One group of one row tile then is  D' = sum x' (1024 + m q) = XS + sum x q  (four matrix
// instructions, fp32, every product exact), and the lane that holds output row n adds
// s (D' - XS - z X) to its accumulator: the same factorisation as in the one-token kernel.
//
// A block's eight waves split K.  The up-projection enters the same accumulators as r more values of
// k (t split into two fp16 halves: t_hi + t_lo carries 22 bits of the fp32 sum), in units of
// (tile, 32 taps) dealt out to the waves; then the waves' partial tiles meet in LDS and y is stored
// once.  Layers that read the same activations (q/k/v, gate/up) share the launch.
#include <hip/hip_fp16.h>

#include "fbq_internal.h"


namespace fbq {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t uint2_t __attribute__((ext_vector_type(2)));
typedef uint32_t uint3_t __attribute__((ext_vector_type(3)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));

constexpr int kTokens = 16;          // rows of the matrix-core tile; M is padded up to it
constexpr int kMainWaves = 8;        // waves per block of the fused kernel; they split K
constexpr int kWaveGroups = 4;       // consecutive quantization groups a wave takes per pass over the block's tiles
constexpr int kPassGroups = kMainWaves * kWaveGroups;   // groups one pass covers (4096 codes)
constexpr int kMaxTiles = 4;         // 16-row tiles per block (more would not fit the register file next to the activations)

__device__ __forceinline__ half2_t h2_of(uint32_t v) { return __builtin_bit_cast(half2_t, v); }
__device__ __forceinline__ half8_t pack8(half2_t a, half2_t b, half2_t c, half2_t d)
{
    return half8_t{a.x, a.y, b.x, b.y, c.x, c.y, d.x, d.y};
}
__device__ __forceinline__ float4_t mfma(half8_t a, half8_t b, float4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ __amdgpu_buffer_rsrc_t buffer_of(const void *p, long bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

struct SmallParams {
    const uint32_t *qw;
    const uint16_t *scales;
    const uint16_t *zeros;
    const uint16_t *At;    // [r][K]
    const uint16_t *Bt;    // [N][r]
    const uint16_t *x;     // [M][K]
    uint16_t *y;           // [M][N]
    uint64_t *tpart;       // workspace: [slices][16][r] words {fp32 partial sum of t = x.A over one K slice, launch tag}
    uint64_t *tsum;        // workspace: [16][r] words {t, launch tag}: the slices added up
    int M, N, K, r;
    int row_words, G;
    int slices, kslice;    // down-projection: number of K slices and their length (a multiple of 512)
    int down_blocks;       // blocks at the start of this layer's grid row that do its down-projection, slice by slice ...
    int sum_blocks;        // ... and the blocks after them that add the slices up (16 columns each)
    int tiles_per_block;   // 16-row tiles a consumer block owns
    int spin_limit;        // polls for t before a wave computes it itself; negative: at once (test hook)
};

// Layers that share their activations (q/k/v, gate/up) share the launch.  In the grid y is the layer
// and x the block of that layer; the layer's parameters are found from the block index alone, so
// they are fetched in one go with the rest of the kernel arguments (a second, dependent round trip
// to them costs more than half a microsecond).  Surplus blocks of rows with fewer blocks than the
// widest leave at once.
struct SmallGroup {
    int n_layers;
    SmallParams layer[kMaxSmallGroup];
};

// What the weight field of pair p (0..15, in extraction order) is multiplied by; the activation that meets it is divided by it.
template <int BITS>
__device__ __forceinline__ constexpr float field_gain(int p)
{
    if (BITS == 4) return (p & 1) ? 16.0f : 1.0f;
    if (p == 15) return 1.0f;
    const int f = p % 5;
    return f == 1 || f == 4 ? 8.0f : (f == 2 ? 64.0f : 1.0f);
}

// (w & mask) | 0x6400 in both halves: the masked field lands in the mantissa of 1024.0.  Plain C on
// purpose (it becomes one v_and_or_b32): the result feeds a matrix instruction directly, and only
// for instructions it has selected itself does the compiler keep the required distance.
__device__ __forceinline__ half2_t field(uint32_t w, uint32_t mask, uint32_t k6400)
{
    return h2_of((w & mask) | k6400);
}

// The lane's 32 codes of one group and their four matrix operands.  Pair order (also the order of
// the arranged activations): INT4 word j -> codes (8j+f, 8j+f+4), f = 0..3;  INT3 word j -> codes
// (10j+f, 10j+f+5), f = 0..4, and codes (30, 31) last.
template <int BITS>
struct SmallCodes {
    static constexpr int kWords = BITS == 4 ? 4 : 3;
    uint32_t w[kWords];

    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t buf, int lane_off, int tile_off)
    {
        if constexpr (BITS == 4) {
            const uint4_t v = __builtin_amdgcn_raw_buffer_load_b128(buf, lane_off, tile_off, 0);
            w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
        } else {
            const uint3_t v = __builtin_amdgcn_raw_buffer_load_b96(buf, lane_off, tile_off, 0);
            w[0] = v.x; w[1] = v.y; w[2] = v.z;
        }
    }

    // With from_lane >= 0 the words arrived in load order (lane l: row l / 4, quarter l % 4) and move to matrix order first.
    __device__ __forceinline__ void operands(uint32_t k6400, int from_lane, half8_t (&b)[4])
    {
        if (from_lane >= 0) {
#pragma unroll
            for (int j = 0; j < kWords; ++j) w[j] = (uint32_t)__builtin_amdgcn_ds_bpermute(from_lane, (int)w[j]);
        }
        if constexpr (BITS == 4) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t lo = w[j], hi = w[j] >> 8;
                b[j] = pack8(field(lo, 0x000F000Fu, k6400), field(lo, 0x00F000F0u, k6400), field(hi, 0x000F000Fu, k6400),
                             field(hi, 0x00F000F0u, k6400));
            }
        } else {
            half2_t d[16];
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const uint32_t lo = w[j], hi = w[j] >> 9;
                d[5 * j + 0] = field(lo, 0x00070007u, k6400);
                d[5 * j + 1] = field(lo, 0x00380038u, k6400);
                d[5 * j + 2] = field(lo, 0x01C001C0u, k6400);
                d[5 * j + 3] = field(hi, 0x00070007u, k6400);
                d[5 * j + 4] = field(hi, 0x00380038u, k6400);
            }
            const uint32_t e = ((w[0] >> 15) & 0x00010001u) | ((w[1] >> 14) & 0x00020002u) | ((w[2] >> 13) & 0x00040004u);
            d[15] = h2_of(e | 0x64006400u);
#pragma unroll
            for (int t = 0; t < 4; ++t) b[t] = pack8(d[4 * t], d[4 * t + 1], d[4 * t + 2], d[4 * t + 3]);
        }
    }
};

// fp16 number i (0..4) of three consecutive words
__device__ __forceinline__ half_t half_at(uint3_t w, int i)
{
    const uint32_t lo = i < 2 ? w.x : (i < 4 ? w.y : w.z);
    return __builtin_bit_cast(half_t, (uint16_t)((i & 1) ? lo >> 16 : lo));
}

// ------------------------------------------------------------------ down-projection, inside the launch

constexpr int kCacheSc1 = 16 | (1 << 31);   // buffer-load policy: device scope (sc1), and volatile so that a poll is never hoisted or merged

constexpr int kPrepWaves = 8;      // = kMainWaves: preparing blocks and consumers are blocks of the same launch

// Down-projection for up to 16 tokens: block b = (K slice, column tile of 16); the block's eight
// waves take an eighth of the slice each.  partial[slice][token][j] = sum over the slice of
// x[token][k] At[j][k], stored with the launch tag in the other half of its 8-byte word; token rows
// past M repeat the last token.  The slices only exist to put more compute units to work on this
// short, latency-bound step; the consumers add them up.
__device__ void down_proj_block(const SmallParams &p, int b, uint32_t tag, float4_t (*red)[64])
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, q = lane >> 4;
    const int col_tiles = (p.r + 15) / 16;
    const int slice = b / col_tiles, j0 = (b - slice * col_tiles) * 16;
    const int kw = p.kslice / kPrepWaves;               // a multiple of 32
    const int kbeg = slice * p.kslice + wave * kw;
    const int kend = min(p.K, kbeg + kw);
    // As in the consumers: lane l fetches the piece l % 4 of row l / 4 (a load quad reads 64 contiguous bytes
    // of one row), and lane (c, q) then takes the words of lane 4 c + q.
    const int ld_row = lane >> 2, ld_piece = lane & 3, from_lane = (4 * c + q) * 4;
    const uint16_t *xr = p.x + (size_t)min(ld_row, p.M - 1) * p.K + 8 * ld_piece;
    const uint16_t *ar = p.At + (size_t)min(j0 + ld_row, p.r - 1) * p.K + 8 * ld_piece;
    auto to_matrix_order = [&](uint4 v) __attribute__((always_inline)) {
        const uint4_t w = {(uint32_t)__builtin_amdgcn_ds_bpermute(from_lane, (int)v.x), (uint32_t)__builtin_amdgcn_ds_bpermute(from_lane, (int)v.y),
                           (uint32_t)__builtin_amdgcn_ds_bpermute(from_lane, (int)v.z), (uint32_t)__builtin_amdgcn_ds_bpermute(from_lane, (int)v.w)};
        return __builtin_bit_cast(half8_t, w);
    };
    float4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 4
    for (int k = kbeg; k < kend; k += 32)
        acc = mfma(to_matrix_order(*reinterpret_cast<const uint4 *>(xr + k)), to_matrix_order(*reinterpret_cast<const uint4 *>(ar + k)), acc);
    red[wave][lane] = acc;
    __syncthreads();
    if (wave == 0) {
        float4_t sum = red[0][lane];
#pragma unroll
        for (int w = 1; w < kPrepWaves; ++w) sum += red[w][lane];
        const int j = j0 + c;                           // lane (c, q) holds column j and tokens 4 q + v
        if (j < p.r) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float partial = sum[v];        // a scalar first: bit_cast of a vector component reads the wrong element
                const uint64_t word = (uint64_t)__builtin_bit_cast(uint32_t, partial) | ((uint64_t)tag << 32);
                __hip_atomic_store(p.tpart + ((size_t)slice * kTokens + 4 * q + v) * p.r + j, word, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

// Second step of the down-projection: block b adds up the K slices of columns 16 b .. 16 b + 15 for all
// 16 token rows (one thread per sum) as soon as their words carry this launch's tag, and passes t on
// in the same form.  Consumers then read one word per value, whatever the number of slices.
constexpr int kSumSlices = 16;        // = the most K slices a layer can have
__device__ void sum_slices_block(const SmallParams &p, int b, uint32_t tag)
{
    const int tid = threadIdx.x;
    if (tid >= 256) return;                             // whole waves
    const int token = tid >> 4, j = 16 * b + (tid & 15);
    const bool mine = j < p.r;
    const __amdgpu_buffer_rsrc_t pb = buffer_of(p.tpart, (long)p.slices * kTokens * p.r * 8);
    float t = 0.0f;
    bool ready = false;
    for (int spin = 0; spin < p.spin_limit && !ready; ++spin) {
        bool ok = true;
        t = 0.0f;
        // all slices are asked for at once (one device-scope round trip per poll, not one per slice);
        // slices the layer does not have aim past the buffer: zero, no access
        uint2_t w[kSumSlices];
#pragma unroll
        for (int sl = 0; sl < kSumSlices; ++sl)
            w[sl] = __builtin_amdgcn_raw_buffer_load_b64(pb, mine && sl < p.slices ? ((sl * kTokens + token) * p.r + j) * 8 : 0x7FFFFFF0, 0, kCacheSc1);
#pragma unroll
        for (int sl = 0; sl < kSumSlices; ++sl) {
            const uint32_t v = w[sl].x;
            t += __builtin_bit_cast(float, v);               // (zero for the slices that are not there)
            ok = ok && (!mine || sl >= p.slices || w[sl].y == tag);
        }
        ready = __all(ok);
        if (!ready) __builtin_amdgcn_s_sleep(4);
    }
    if (!mine) return;
    if (!ready) {                                       // the slices never showed up: the whole sum, here
        const uint16_t *xr = p.x + (size_t)min(token, p.M - 1) * p.K, *ar = p.At + (size_t)j * p.K;
        t = 0.0f;
        for (int k = 0; k < p.K; ++k) t = fmaf((float)__builtin_bit_cast(half_t, xr[k]), (float)__builtin_bit_cast(half_t, ar[k]), t);
    }
    const uint64_t word = (uint64_t)__builtin_bit_cast(uint32_t, t) | ((uint64_t)tag << 32);
    __hip_atomic_store(p.tsum + (size_t)token * p.r + j, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Activation operands of one group: the lane's 32 activations (four 16-byte pieces, k ascending) become
// the four operands that meet its weight operands, pair by pair in extraction order, each divided by
// the gain of the weight field it meets (exact unless the quotient is subnormal).  One byte
// permutation picks the two activations of a pair out of the 16 dwords, one packed multiply scales
// the pairs whose field has a gain.
template <int BITS>
__device__ __forceinline__ void arrange_operands(const uint4_t (&raw)[4], half8_t (&ops)[4])
{
    uint32_t d[16];
#pragma unroll
    for (int i = 0; i < 4; ++i) { d[4 * i] = raw[i].x; d[4 * i + 1] = raw[i].y; d[4 * i + 2] = raw[i].z; d[4 * i + 3] = raw[i].w; }
    half2_t pr[16];
#pragma unroll
    for (int pi = 0; pi < 16; ++pi) {
        int first, second;                              // the two codes of pair pi
        if (BITS == 4) { first = 8 * (pi / 4) + pi % 4; second = first + 4; }
        else if (pi == 15) { first = 30; second = 31; }
        else { first = 10 * (pi / 5) + pi % 5; second = first + 5; }
        // result bytes 0,1 <- half `first` (bytes 0..3 of the selector's view are its dword), bytes 2,3 <- half `second`
        const uint32_t sel = (uint32_t)(2 * (first & 1)) | ((uint32_t)(2 * (first & 1) + 1) << 8) |
                             ((uint32_t)(4 + 2 * (second & 1)) << 16) | ((uint32_t)(4 + 2 * (second & 1) + 1) << 24);
        const half2_t both = h2_of(__builtin_amdgcn_perm(d[second / 2], d[first / 2], sel));
        const float gain = field_gain<BITS>(pi);
        const half_t inv = (half_t)(1.0f / gain);
        pr[pi] = gain == 1.0f ? both : both * half2_t{inv, inv};
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) ops[t] = pack8(pr[4 * t], pr[4 * t + 1], pr[4 * t + 2], pr[4 * t + 3]);
}

// The gains of the eight weight fields that operand t holds: against this column the scaled
// activations sum to X = sum x.
template <int BITS>
__device__ __forceinline__ half8_t gain_operand(int t)
{
    half8_t g;
#pragma unroll
    for (int e = 0; e < 8; ++e) g[e] = (half_t)field_gain<BITS>(4 * t + e / 2);
    return g;
}

// ------------------------------------------------------------------ hand-over inside the launch


extern "C" __device__ unsigned long long fbq_small_m_dispatch_id(void) __asm("llvm.amdgcn.dispatch.id");

// Identity of this launch, the same in every block and different for every launch (also for every
// replay of a captured graph): never zero, so a zero-filled workspace never matches.
__device__ __forceinline__ uint32_t small_m_launch_tag()
{
    const uint64_t id = fbq_small_m_dispatch_id();
    const uint64_t q = (uint64_t)__builtin_amdgcn_queue_ptr();
    const uint32_t tag = (uint32_t)id + (uint32_t)(q >> 6) * 0x9E3779B1u;
    return tag ? tag : 0x80000000u;
}

// ------------------------------------------------------------------ fused kernel

// BITS: 3 or 4.  T: 16-row tiles per block.  BRANCH: r > 0.
// TAIL: some layer of the launch has an odd number of scales (N G odd): see where scale and zero are taken.
template <int BITS, int T, bool BRANCH, bool TAIL>
__global__ __launch_bounds__(64 * kMainWaves) void fbq_small_m_kernel(const SmallGroup g)
{
    constexpr int kPiece = BITS == 4 ? 16 : 12;         // bytes of 32 codes
    __shared__ float4_t red[kMainWaves][T][64];
    // one group of activations per wave on its way from row order (as loaded, coalesced) to lane order:
    // [token][16 pieces of 16 bytes + 1 of padding], the padding keeps both directions free of bank conflicts
    __shared__ uint4_t xslab[kMainWaves][kTokens * 17];
    float4_t (*red_prep)[64] = reinterpret_cast<float4_t (*)[64]>(&red[0][0][0]);   // [8][64], what a down-projection block needs

    const SmallParams p = g.layer[blockIdx.y];
    // (all of them before the first branch: left alone, the compiler fetches only what the branch needs first)
    asm volatile("" :: "s"(p.qw), "s"(p.scales), "s"(p.zeros), "s"(p.x), "s"(p.y), "s"(p.M), "s"(p.N), "s"(p.K), "s"(p.row_words), "s"(p.G), "s"(p.tiles_per_block));
    if (BRANCH) asm volatile("" :: "s"(p.Bt), "s"(p.At), "s"(p.tpart), "s"(p.tsum), "s"(p.r), "s"(p.slices), "s"(p.kslice), "s"(p.down_blocks), "s"(p.sum_blocks), "s"(p.spin_limit));
    const uint32_t tag = BRANCH ? small_m_launch_tag() : 0u;

    // The first blocks of a grid row do the layer's down-projection.  They come first in dispatch
    // order, so whoever waits for their words waits for blocks that are already running.
    if (BRANCH && (int)blockIdx.x < p.down_blocks + p.sum_blocks) {
        if ((int)blockIdx.x < p.down_blocks) down_proj_block(p, blockIdx.x, tag, red_prep);
        else sum_slices_block(p, blockIdx.x - p.down_blocks, tag);
        return;
    }
    const int block = blockIdx.x - (BRANCH ? p.down_blocks + p.sum_blocks : 0);
    if (block * p.tiles_per_block >= (p.N + 15) / 16) return;   // a narrower layer of the group
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int c = lane & 15, q = lane >> 4;
    const int ntiles = (p.N + 15) / 16;
    const int tile0 = block * p.tiles_per_block;
    const int row_bytes = p.row_words * 4;

    const __amdgpu_buffer_rsrc_t qbuf = buffer_of(p.qw, (long)p.N * row_bytes);
    // The range check is per dword, so the count is rounded up to whole dwords: with N·G odd the last
    // half shares an aligned dword with two bytes past the array (same cache line, never another page).
    const __amdgpu_buffer_rsrc_t sbuf = buffer_of(p.scales, ((long)p.N * p.G * 2 + 3) & ~3L);
    const __amdgpu_buffer_rsrc_t zbuf = buffer_of(p.zeros, ((long)p.N * p.G * 2 + 3) & ~3L);
    const __amdgpu_buffer_rsrc_t xbuf = buffer_of(p.x, (long)p.M * p.K * 2);
    // activations are fetched a group at a time in four loads of four token rows each: 16 lanes per row,
    // 256 contiguous bytes (the lane's own 64 bytes of its token would make every load a 64-segment gather)
    const int xtok = lane >> 4, xpiece = lane & 15;

    // Who loads what.  The matrix instruction wants lane (c, q) = lane q * 16 + c to hold quarter q of row c,
    // but loaded that way the four neighbouring lanes of a load quad read four different rows, i.e. four
    // cache lines, and a wave-wide load costs the address path 64 cycles.  So lane l fetches quarter l % 4 of
    // row l / 4 - a quad reads 64 (48) contiguous bytes of one row, 16 cycles per load - and the words change
    // lanes afterwards (ds_bpermute: lane (c, q) takes those of lane 4 c + q).  Scale and zero likewise: the
    // four lanes of a quad read the same 12 bytes of row l / 4, lane (c, q) takes them from lane 4 c.
    // Measured: 4096 -> 11008 11.9 -> 10.8 us, the {gate,up} pair 21.2 -> 19.9, 28672 -> 8192 52.7 -> 49.1.  Not
    // for INT4 with four tiles per block (the extra lane traffic costs more than the address path gains: q/k/v
    // 13.3 -> 14.0; INT3 with four tiles gains, 14.3 -> 13.0) and not for INT3 with two tiles (that instance then spills).
    // Rows past N re-read the last row: computed, never stored.
    constexpr bool kQuadLoads = BITS == 4 ? T <= 3 : T != 2;
    const int from_lane = (4 * c + q) * 4, from_quad = (4 * c) * 4;   // byte addresses of the source lanes
    int qrow[T], srow[T], odd[T];
#pragma unroll
    for (int ti = 0; ti < T; ++ti) {
        const int n = min((tile0 + ti) * 16 + c, p.N - 1);
        const int n_ld = kQuadLoads ? min((tile0 + ti) * 16 + (lane >> 2), p.N - 1) : n;
        qrow[ti] = n_ld * row_bytes + (kQuadLoads ? lane & 3 : q) * kPiece;
        srow[ti] = n_ld * p.G * 2;
        odd[ti] = (n * p.G) & 1;                        // of the row the lane ends up with; the wave's first group is a multiple of four
    }

    // Up-projection: r more values of k, in units of (tile, 32 taps) dealt out to the waves.  Lane (c, q)
    // needs t[token c][j .. j + 7] and Bt[row c of the tile][j .. j + 7], j = 32 js + 8 q; taps past r read
    // beyond the buffers, i.e. zeros.  The Bt part of the wave's first unit (cold, from HBM) is requested
    // here with everything else; t (a few KB that every block reads) is fetched when it is needed.
    const int tap_steps = BRANCH ? (p.r + 31) / 32 : 0;
    const int units = T * tap_steps;
    const __amdgpu_buffer_rsrc_t tbuf = buffer_of(p.tsum, BRANCH ? (long)kTokens * p.r * 8 : 0);
    const __amdgpu_buffer_rsrc_t bbuf = buffer_of(p.Bt, BRANCH ? (long)p.N * p.r * 2 : 0);
    constexpr int kNowhere = 0x7FFFFFF0;                // beyond every buffer
    half8_t ubf;
    auto request_taps = [&](int u) __attribute__((always_inline)) {
        const int ti = u / max(tap_steps, 1), js = u - ti * tap_steps;
        const int j = js * 32 + q * 8;
        const bool on = u < units && j < p.r;          // r is a multiple of 8: all eight taps or none
        const int n = min((tile0 + ti) * 16 + c, p.N - 1);
        ubf = __builtin_bit_cast(half8_t, __builtin_amdgcn_raw_buffer_load_b128(bbuf, on ? (n * p.r + j) * 2 : kNowhere, 0, 0));
    };
    if (BRANCH) request_taps(wave);

    uint32_t k6400 = 0x64006400u;
    asm volatile("" : "+v"(k6400));                     // keep the constant in a VGPR for v_and_or_b32
    const float4_t zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    float4_t acc[T];
#pragma unroll
    for (int ti = 0; ti < T; ++ti) acc[ti] = zero4;

    // One pass: the wave's four groups g0 .. g0 + 3 against every tile of the block.  Everything the
    // pass needs is requested up front.  Every offset that depends on the group is part of the
    // bounds-checked per-lane offset of its buffer load: groups past the end of K read activation
    // operands and sums beyond their buffers, i.e. zeros without a memory access, and add nothing
    // (their weights are whatever follows in the row, or zero behind the last row: finite either way;
    // their scales and zeros are replaced by zero).
    const int passes = (p.G + kPassGroups - 1) / kPassGroups;
    for (int pass = 0; pass < passes; ++pass) {
        const int g0 = pass * kPassGroups + wave * kWaveGroups;
        // Token rows past M are all zero and are not fetched (their lanes aim beyond the buffer).
        // Order of the requests: the first tile's weights, then the activations, then the other tiles -
        // the weights are the long pole (HBM), so some are under way before the block's share of the
        // activations (L2) occupies the load path, and the first tile can be worked on while the rest streams.
        half8_t xa[kWaveGroups][4];
        float4_t X[kWaveGroups], XS[kWaveGroups];
        SmallCodes<BITS> cw[T][kWaveGroups];
        // Four fp16 scales / zeros, groups g0 .. g0 + 3 of the lane's row: they start at an even or an odd
        // fp16 index, so three aligned words are loaded and shifted by a half where needed.
        uint3_t sc[T], zp[T];
        auto request_tile = [&](int ti) __attribute__((always_inline)) {
#pragma unroll
            for (int gi = 0; gi < kWaveGroups; ++gi) cw[ti][gi].load(qbuf, qrow[ti] + (g0 + gi) * 4 * kPiece, 0);
            sc[ti] = __builtin_amdgcn_raw_buffer_load_b96(sbuf, (srow[ti] + g0 * 2) & ~3, 0, 0);
            zp[ti] = __builtin_amdgcn_raw_buffer_load_b96(zbuf, (srow[ti] + g0 * 2) & ~3, 0, 0);
        };
        request_tile(0);
        // Activations: all four groups at once, or two at a time where the instance is short of registers (INT3,
        // four tiles): the second pair is then requested when the first has been arranged, long before the weights are in.
        constexpr int kXG = BITS == 4 && T <= 3 ? kWaveGroups : 2;
        uint4_t xraw[kXG][4];
        auto request_x = [&](int part) __attribute__((always_inline)) {
#pragma unroll
            for (int gj = 0; gj < kXG; ++gj)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int grp = g0 + kXG * part + gj;
                    xraw[gj][i] = __builtin_amdgcn_raw_buffer_load_b128(xbuf, 4 * i + xtok < p.M && grp < p.G ? (4 * i + xtok) * p.K * 2 + grp * 256 + xpiece * 16 : kNowhere, 0, 0);
                }
        };
        request_x(0);
#pragma unroll
        for (int ti = 1; ti < T; ++ti) request_tile(ti);
        __builtin_amdgcn_sched_barrier(0);
        // while the weights stream: operands, and both sums per token from the matrix core (accumulator
        // register v of lane (., q) belongs to token 4 q + v, which is where the sums are needed)
        half8_t ones;
#pragma unroll
        for (int e = 0; e < 8; ++e) ones[e] = (half_t)1.0f;
#pragma unroll
        for (int part = 0; part < kWaveGroups / kXG; ++part) {
            uint4_t mine[kXG][4];
#pragma unroll
            for (int gj = 0; gj < kXG; ++gj) {
                // through the wave's slab: token rows in, the lane's 64 bytes (token c, quarter q) out
#pragma unroll
                for (int i = 0; i < 4; ++i) xslab[wave][(4 * i + xtok) * 17 + xpiece] = xraw[gj][i];
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int i = 0; i < 4; ++i) mine[gj][i] = xslab[wave][c * 17 + 4 * q + i];
                __builtin_amdgcn_wave_barrier();
            }
            if (part + 1 < kWaveGroups / kXG) request_x(part + 1);
#pragma unroll
            for (int gj = 0; gj < kXG; ++gj) {
                const int gi = kXG * part + gj;
                arrange_operands<BITS>(mine[gj], xa[gi]);
                float4_t sx = zero4, sxs = zero4;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    sx = mfma(xa[gi][t], gain_operand<BITS>(t), sx);
                    sxs = mfma(xa[gi][t], ones, sxs);
                }
                X[gi] = sx;
                XS[gi] = 1024.0f * sxs;
            }
        }
#pragma unroll
        for (int ti = 0; ti < T; ++ti) {
            // scale and zero of the lane's row from the lane that fetched them
            if constexpr (kQuadLoads) {
            sc[ti] = uint3_t{(uint32_t)__builtin_amdgcn_ds_bpermute(from_quad, (int)sc[ti].x), (uint32_t)__builtin_amdgcn_ds_bpermute(from_quad, (int)sc[ti].y),
                             (uint32_t)__builtin_amdgcn_ds_bpermute(from_quad, (int)sc[ti].z)};
            zp[ti] = uint3_t{(uint32_t)__builtin_amdgcn_ds_bpermute(from_quad, (int)zp[ti].x), (uint32_t)__builtin_amdgcn_ds_bpermute(from_quad, (int)zp[ti].y),
                             (uint32_t)__builtin_amdgcn_ds_bpermute(from_quad, (int)zp[ti].z)};
            }
            // Groups past the end of K add nothing as long as what is read in their place is finite: the next row's
            // scales, or zero beyond the descriptor.  One half is neither: with N G odd the descriptor, whole dwords,
            // also admits the two bytes behind the array, which may hold anything, a NaN included.  That half is cleared
            // (any row within a pass's 32 groups of the array's end can have fetched it).
            if (TAIL && ((p.N * p.G) & 1)) {               // block-uniform; an instance of its own, so that layers with an even number of scales run the code they always ran
                const int n = min((tile0 + ti) * 16 + c, p.N - 1);
                const int kk = ((p.N * p.G) >> 1) - ((n * p.G + g0) >> 1);   // which of the lane's three dwords is the array's last
                sc[ti] = uint3_t{kk == 0 ? sc[ti].x & 0xFFFFu : sc[ti].x, kk == 1 ? sc[ti].y & 0xFFFFu : sc[ti].y, kk == 2 ? sc[ti].z & 0xFFFFu : sc[ti].z};
                zp[ti] = uint3_t{kk == 0 ? zp[ti].x & 0xFFFFu : zp[ti].x, kk == 1 ? zp[ti].y & 0xFFFFu : zp[ti].y, kk == 2 ? zp[ti].z & 0xFFFFu : zp[ti].z};
            }
#pragma unroll
            for (int gi = 0; gi < kWaveGroups; ++gi) {
                half8_t b[4];
                cw[ti][gi].operands(k6400, kQuadLoads ? from_lane : -1, b);
                float4_t D = zero4;
#pragma unroll
                for (int t = 0; t < 4; ++t) D = mfma(xa[gi][t], b[t], D);
                const float s = (float)half_at(sc[ti], gi + odd[ti]), z = (float)half_at(zp[ti], gi + odd[ti]);
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[ti][v] = fmaf(s, D[v] - fmaf(z, X[gi][v], XS[gi][v]), acc[ti][v]);
            }
        }
    }

    if (BRANCH) {
        for (int u = wave; u < units; u += kMainWaves) {   // wave-uniform; the first unit's Bt operand is already here
            const int ti = u / tap_steps, js = u - ti * tap_steps;
            const int j = js * 32 + q * 8;
            // t[token c][j .. j + 7]: eight words {t, launch tag} (four 16-byte device-scope loads), written long ago
            // as a rule.  Should the tags not turn up, the lane computes its eight values itself.
            float t[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};   // (taps past r stay zero also when nothing is ever polled)
            bool ready = false;
            const int off = j < p.r ? (c * p.r + j) * 8 : kNowhere;
            for (int spin = 0; spin < p.spin_limit && !ready; ++spin) {
                bool ok = true;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint4_t w = __builtin_amdgcn_raw_buffer_load_b128(tbuf, off + 16 * i, 0, kCacheSc1);
                    const uint32_t v0 = w.x, v1 = w.z;
                    t[2 * i] = __builtin_bit_cast(float, v0);
                    t[2 * i + 1] = __builtin_bit_cast(float, v1);
                    ok = ok && (j >= p.r || (w.y == tag && w.w == tag));
                }
                ready = __all(ok);
                if (!ready) __builtin_amdgcn_s_sleep(4);
            }
            if (!ready && j < p.r) {
                const uint16_t *xr = p.x + (size_t)min(c, p.M - 1) * p.K;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint16_t *ar = p.At + (size_t)(j + e) * p.K;
                    float a = 0.0f;
                    for (int k = 0; k < p.K; ++k) a = fmaf((float)__builtin_bit_cast(half_t, xr[k]), (float)__builtin_bit_cast(half_t, ar[k]), a);
                    t[e] = a;
                }
            }
            half8_t thi, tlo;                           // t_hi + t_lo carries 22 bits of the fp32 sum
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                thi[e] = (half_t)t[e];
                tlo[e] = (half_t)(t[e] - (float)thi[e]);
            }
            float4_t d = mfma(thi, ubf, zero4);
            d = mfma(tlo, ubf, d);
#pragma unroll
            for (int k = 0; k < T; ++k)
                if (k == ti) acc[k] += d;
            if (u + kMainWaves < units) request_taps(u + kMainWaves);
        }
    }

    // K split: every wave leaves its tiles in LDS; wave ti adds them up for tile ti and stores.
#pragma unroll
    for (int ti = 0; ti < T; ++ti) red[wave][ti][lane] = acc[ti];
    __syncthreads();
    for (int ti = wave; ti < T; ti += kMainWaves) {     // wave-uniform
        if (tile0 + ti >= ntiles) break;
        float4_t sum = red[0][ti][lane];
#pragma unroll
        for (int w = 1; w < kMainWaves; ++w) sum += red[w][ti][lane];
        const int n = (tile0 + ti) * 16 + c;
        // lane (c, q) holds output row n and tokens 4 q + v
        if (n < p.N) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int m = 4 * q + v;
                if (m < p.M) p.y[(size_t)m * p.N + n] = __builtin_bit_cast(uint16_t, (half_t)sum[v]);
            }
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

template <int BITS, int T, bool TAIL>
static hipError_t launch_tiles(const SmallGroup &g, bool branch, dim3 grid, hipStream_t stream)
{
    // (the INT3 three- and four-tile instances without the branch come out of the compiler with spills of
    // 160 bytes and more; the ones with the branch spill nothing or 36 bytes, and with r = 0 they do the same work)
    if constexpr (BITS == 3 && T >= 3) {
        hipLaunchKernelGGL((fbq_small_m_kernel<BITS, T, true, TAIL>), grid, dim3(64 * kMainWaves), 0, stream, g);
    } else {
        if (branch) hipLaunchKernelGGL((fbq_small_m_kernel<BITS, T, true, TAIL>), grid, dim3(64 * kMainWaves), 0, stream, g);
        else hipLaunchKernelGGL((fbq_small_m_kernel<BITS, T, false, TAIL>), grid, dim3(64 * kMainWaves), 0, stream, g);
    }
    return hipGetLastError();
}

template <int BITS>
static hipError_t launch_bits(const SmallGroup &g, int row_blocks, hipStream_t stream)
{
    const bool branch = g.layer[0].r > 0;
    const dim3 grid(row_blocks, g.n_layers);
    bool tail = false;                                  // a layer whose scale array ends in the middle of a dword
    for (int i = 0; i < g.n_layers; ++i) tail = tail || (((long)g.layer[i].N * g.layer[i].G) & 1);
    switch (g.layer[0].tiles_per_block * 2 + (tail ? 1 : 0)) {
    case 2: return launch_tiles<BITS, 1, false>(g, branch, grid, stream);
    case 3: return launch_tiles<BITS, 1, true>(g, branch, grid, stream);
    case 4: return launch_tiles<BITS, 2, false>(g, branch, grid, stream);
    case 5: return launch_tiles<BITS, 2, true>(g, branch, grid, stream);
    case 6: return launch_tiles<BITS, 3, false>(g, branch, grid, stream);
    case 7: return launch_tiles<BITS, 3, true>(g, branch, grid, stream);
    case 8: return launch_tiles<BITS, 4, false>(g, branch, grid, stream);
    default: return launch_tiles<BITS, 4, true>(g, branch, grid, stream);
    }
}

// workspace: [16 slices][16][r] 8-byte words {fp32 partial sum of t, launch tag}, then [16][r] words {t, launch tag};
// zero-filled once by the caller
constexpr int kMaxSlices = 16;       // K slices of the down-projection
static_assert(kMaxSlices == kSumSlices, "the summing blocks ask for every slice at once");
static_assert((size_t)(kMaxSlices + 1) * kTokens * kMaxRank * 8 <= kStaticScratchBytes, "the static scratch must hold the largest few-token hand-over");
size_t small_m_workspace_bytes(int K, int r) { (void)K; return (size_t)(kMaxSlices + 1) * kTokens * r * 8; }

static int tiles_per_block_of(int total_tiles, int preparing_blocks, int passes)
{
    // Blocks run one per compute unit, in rounds; a block's time grows with passes x (tiles + about one tile's
    // worth of fixed work: arranging the activations, the reduction).  The blocks that do the down-projection come
    // first in the grid and are gone after about two such units - which only matters where they and the
    // consumers together do not fit the GPU at once: then some consumers start that much later.  (Counting them
    // as full blocks of a round, as an earlier version did, chose one tile per block for long K with few rows:
    // 28672 -> 8192 at 16 tokens 58 us, with two tiles 46; 13824 -> 5120 28.6 and 24.7.)  So: the tile count that
    // makes rounds x passes x (tiles + 1), plus that delay where it applies, smallest.  4096 rows: two tiles in
    // one round beside the preparing blocks instead of one tile and a late start; q/k/v together: four tiles
    // instead of three for the same reason; gate/up together: three tiles in two full rounds rather than four in
    // one and a half; 11008 -> 4096: one tile per block (16.3 us against 17.9 with two).
    constexpr int kPrepUnits = 2;
    int best = 1, best_cost = 1 << 30;
    for (int t = 1; t <= kMaxTiles; ++t) {
        const int consumers = ceil_div(total_tiles, t);
        const int cost = ceil_div(consumers, cu_count()) * passes * (t + 1) + (consumers + preparing_blocks > cu_count() ? kPrepUnits : 0);
        if (cost < best_cost) { best = t; best_cost = cost; }
    }
    return best;
}

static int slice_length(int K)
{
    // slices of 1024 (they only exist to put more compute units to work on a short, latency-bound step), longer where K > 16384
    return std::max(1024, ceil_div(ceil_div(K, kMaxSlices), 32 * kPrepWaves) * (32 * kPrepWaves));
}

// What the kernel itself needs of the layers of one launch: the same instance (a branch-free layer never joins layers
// with a sub-branch).  Activations, token count, outputs and workspace are per layer.
static bool same_instance(const LinearArgs &a, const LinearArgs &b)
{
    return a.K == b.K && a.bits == b.bits && (a.r > 0) == (b.r > 0);
}

// Layers of a grouped call share the launch when they also read the same activations.
bool small_m_group_compatible(const LinearArgs &a, const LinearArgs &b)
{
    return a.x == b.x && a.M == b.M && same_instance(a, b);
}

hipError_t launch_gemv_small_m(const LinearArgs *layers, int n_layers, hipStream_t stream)
{
    if (n_layers < 1 || n_layers > kMaxSmallGroup) return hipErrorInvalidValue;
    const LinearArgs &first = layers[0];
    int total_tiles = 0;
    for (int i = 0; i < n_layers; ++i) {
        if (layers[i].M < 1 || layers[i].M > kTokens || !same_instance(first, layers[i])) return hipErrorInvalidValue;
        total_tiles += ceil_div(layers[i].N, 16);
    }
    int preparing = 0;
    for (int i = 0; i < n_layers; ++i)
        if (layers[i].r > 0) preparing += ceil_div(layers[i].r, 16) * (ceil_div(layers[i].K, slice_length(layers[i].K)) + 1);
    const int tpb = tiles_per_block_of(total_tiles, preparing, ceil_div(first.K / kGroup, kPassGroups));
    SmallGroup g;
    g.n_layers = n_layers;
    int row_blocks = 0;                                  // widest row of the grid
    for (int i = 0; i < n_layers; ++i) {
        const LinearArgs &a = layers[i];
        SmallParams &p = g.layer[i];
        p.qw = a.qw; p.scales = a.scales; p.zeros = a.zeros; p.At = a.At; p.Bt = a.Bt; p.x = a.x; p.y = a.y;
        p.tpart = (uint64_t *)a.workspace;               // each layer's own partial sums of t ...
        p.tsum = p.tpart + (size_t)kMaxSlices * kTokens * a.r;   // ... and their sums
        p.M = a.M; p.N = a.N; p.K = a.K; p.r = a.r;
        p.row_words = (int)row_words(a.K, a.bits);
        p.G = a.K / kGroup;
        // Every consumer block reads all of t at device scope, slice by slice, so few slices: one up to K = 8192 (its
        // producers have the whole main part of the consumers to finish in), at most four.
        p.kslice = slice_length(a.K);
        p.slices = ceil_div(a.K, p.kslice);
        p.down_blocks = a.r > 0 ? ceil_div(a.r, 16) * p.slices : 0;
        p.sum_blocks = a.r > 0 ? ceil_div(a.r, 16) : 0;
        p.tiles_per_block = tpb;
        p.spin_limit = spin_limit();
        row_blocks = std::max(row_blocks, p.down_blocks + p.sum_blocks + ceil_div(ceil_div(a.N, 16), tpb));
    }
    for (int i = n_layers; i < kMaxSmallGroup; ++i) g.layer[i] = g.layer[0];   // never indexed: grid.y stops at n_layers
    return first.bits == 4 ? launch_bits<4>(g, row_blocks, stream) : launch_bits<3>(g, row_blocks, stream);
}

}  // namespace fbq
