// Layer-wise reconstruction (Alg. 1, Sec. 4.2): one gradient-descent iteration on the sub-branch
// of one layer.
//
// The loss and its gradient depend on the calibration activations X [T,K] only through
// H = X^T X (Sec. 4.2: L = tr(Delta_F H Delta_F^T), dL/dSigma = -2 Delta_F H with the feedback
// detached), so H is formed once per layer and an iteration is
//
//   A16, B16   <- fp16 of the fp32 masters                               (cast kernel)
//   q, s, z    <- Q(W - Sigma16)               feedback quantizer  } fbq_quantize_kernel: fp64, Delta_F
//   Delta_F    <- (W - Sigma16) - s (q - z)                        } from the registers that hold W - Sigma16
//   Q          <- Bt^T Delta_F        [r,K]                              (GEMM, K split)
//   dL/dAt     <- -2 Q H              [r,K]    } one GEMM on the stacked                                 
//   V^T        <- At H                [r,K]    } operand [Q; At], K split
//   dL/dBt     <- -2 Delta_F V        [N,r]                              (GEMM, K split)
//   L          <- sum Delta_F o (Delta_F H)    only if the caller asks   (GEMM, 2 N K^2 flop, + reduction)
//   masters    <- masters - lr gradient                                  (update kernel)
//
// with Sigma[n,k] = sum_j Bt[n,j] At[j,k] in the device layouts At [r,K], Bt [N,r].  Multiplying
// Delta_F H out costs 2 N K^2 flop; the gradients need only products with r rows or columns
// (8 N K r + 4 r K^2 flop, a twentieth of that at r = 64, K = 4096) because H is symmetric:
// Delta_F H At^T = Delta_F (At H)^T.  The loss is the one quantity that needs Delta_F H itself.
//
// One matrix-core kernel serves every contraction: C[m,n] = sum_k A[m,k] B[n,k] with both operands
// contiguous along k (fp16 in, fp32 accumulate, v_mfma_f32_32x32x16_f16).  128x128 block tile,
// 4 waves of 64x64, k advancing 64 at a time; both operand tiles go global -> registers -> LDS with
// coalesced 16-byte loads (rows of 128 bytes, whole cache lines) and are read back as matrix
// operands with ds_read_b128, the 16-byte chunks of a row XOR-swizzled so that neither side has a
// bank conflict; the next step's global loads are in flight while the current one is multiplied.
// Rows past the end of an operand are fetched through a bounds-checked buffer descriptor and
// arrive as zeros.  fp16 operands carry Delta_F times 256 and H times the caller's h_scale, so
// that neither leaves the normal range; the factors come out again in the epilogues.
#include <hip/hip_fp16.h>

#include "fbq_internal.h"

namespace fbq {

typedef _Float16 half_t;
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));

constexpr int kStepK = 64;           // k per step: one 128-byte row segment per operand row
constexpr float kDeltaGain = 256.0f; // Delta_F is stored as fp16(256 Delta_F)
constexpr int kXcds = 8;

struct GemmArgs {
    const uint16_t *A;   // [Mr][lda] fp16
    const uint16_t *B;   // [Nr][ldb] fp16
    int Mr, Nr, Kd;      // Kd a multiple of 64
    int lda, ldb;        // elements
    // store epilogue (any of the three may be absent)
    float *C32; int ldc32; float alpha; int c32_rows;   // C32[m,n] = alpha acc for rows m < c32_rows
    uint16_t *C16; int ldc16; float beta; int c16_row0; // C16[m - c16_row0, n] = fp16(beta acc) for rows m >= c16_row0
    const uint16_t *D; int ldd; float *dot;      // dot[tile] = sum over the tile of acc D[m,n]  (splits == 1 only)
    // K split over `splits` blocks per tile (few tiles, long K): raw sums go to part [splits][Mr][Nr]
    // and fbq_sum_splits_kernel applies the store epilogue
    int splits; float *part;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t rows_buffer(const void *p, long bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

// 16-byte chunk c (0..7) of row `row` of an operand tile sits at chunk c ^ key(row): 8 or 16
// consecutive rows reading the same c touch every bank once, whether the LDS serves 128 or 256
// bytes per clock.
__device__ __forceinline__ int swizzle_key(int row) { return ((row >> 1) & 7) ^ ((row & 1) << 2); }

__device__ __forceinline__ void store_result(const GemmArgs &g, int m, int n, float a)
{
    if (g.C32 && m < g.c32_rows) g.C32[(size_t)m * g.ldc32 + n] = g.alpha * a;
    if (g.C16 && m >= g.c16_row0) g.C16[(size_t)(m - g.c16_row0) * g.ldc16 + n] = __builtin_bit_cast(uint16_t, (half_t)(g.beta * a));
}

// WM x WN: 32x32 tiles a wave owns (rows x columns); the block's 2 x 2 waves cover 64 WM x 64 WN.
template <int WM, int WN>
__global__ __launch_bounds__(256, (WM * WN > 4 ? 1 : 2)) void fbq_gemm_nt_kernel(GemmArgs g)
{
    extern __shared__ __align__(16) unsigned char lds[];   // [buffer][A rows | B rows][128 bytes]
    constexpr int BM = 64 * WM, BN = 64 * WN;
    constexpr int kABytes = BM * kStepK * 2, kBufferBytes = (BM + BN) * kStepK * 2;
    constexpr int LA = BM * 8 / 256, LB = BN * 8 / 256;     // 16-byte loads per thread and step

    // Consecutive tiles (same rows of A, neighbouring rows of B) run on the same XCD and share its L2.
    const int tiles_n = (g.Nr + BN - 1) / BN, tiles_m = (g.Mr + BM - 1) / BM;
    const int total = tiles_m * tiles_n * g.splits, per_xcd = (total + kXcds - 1) / kXcds;
    const int unit = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    if (unit >= total) return;
    const int tile = unit / g.splits, split = unit % g.splits;
    const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int col = lane & 31, h = lane >> 5;

    const __amdgpu_buffer_rsrc_t abuf = rows_buffer(g.A + (size_t)m0 * g.lda, (long)min(BM, g.Mr - m0) * g.lda * 2);
    const __amdgpu_buffer_rsrc_t bbuf = rows_buffer(g.B + (size_t)n0 * g.ldb, (long)min(BN, g.Nr - n0) * g.ldb * 2);

    // thread t fetches chunk t % 8 of rows t / 8, t / 8 + 32, ...: every wave-wide load covers whole 128-byte row segments
    const int lrow = tid >> 3, lch = tid & 7;
    const int goff_a = lrow * g.lda * 2 + lch * 16, goff_b = lrow * g.ldb * 2 + lch * 16;
    const int gstep_a = 32 * g.lda * 2, gstep_b = 32 * g.ldb * 2;
    const int loff = lrow * 128 + ((lch ^ swizzle_key(lrow)) * 16);     // rows 32 apart share the key
    uint4_t ra[LA], rb[LB];
    auto fetch = [&](int s) {
#pragma unroll
        for (int i = 0; i < LA; ++i) ra[i] = __builtin_bit_cast(uint4_t, __builtin_amdgcn_raw_buffer_load_b128(abuf, goff_a + i * gstep_a + s * 128, 0, 0));
#pragma unroll
        for (int i = 0; i < LB; ++i) rb[i] = __builtin_bit_cast(uint4_t, __builtin_amdgcn_raw_buffer_load_b128(bbuf, goff_b + i * gstep_b + s * 128, 0, 0));
    };
    auto stash = [&](int buf) {
        unsigned char *la = lds + buf * kBufferBytes, *lb = la + kABytes;
#pragma unroll
        for (int i = 0; i < LA; ++i) *reinterpret_cast<uint4_t *>(la + loff + i * 32 * 128) = ra[i];
#pragma unroll
        for (int i = 0; i < LB; ++i) *reinterpret_cast<uint4_t *>(lb + loff + i * 32 * 128) = rb[i];
    };

    float16_t acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // operand rows of this lane: 32 rows apart, so they share the swizzle key
    const int key = swizzle_key(col);
    const int arow = (wm * 32 * WM + col) * 128, brow = (wn * 32 * WN + col) * 128;
    auto multiply = [&](int buf) {
        const unsigned char *la = lds + buf * kBufferBytes, *lb = la + kABytes;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int chunk = ((kk * 2 + h) ^ key) * 16;
            half8_t af[WM], bf[WN];
#pragma unroll
            for (int i = 0; i < WM; ++i) af[i] = *reinterpret_cast<const half8_t *>(la + arow + i * 32 * 128 + chunk);
#pragma unroll
            for (int j = 0; j < WN; ++j) bf[j] = *reinterpret_cast<const half8_t *>(lb + brow + j * 32 * 128 + chunk);
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
    };

    const int all_steps = g.Kd / kStepK, per_split = (all_steps + g.splits - 1) / g.splits;
    const int first = split * per_split, steps = min(all_steps, first + per_split) - first;   // >= 1: the launcher sees to it
    fetch(first);
    stash(0);
    __syncthreads();
    for (int s = 0; s < steps; ++s) {
        if (s + 1 < steps) fetch(first + s + 1);
        multiply(s & 1);
        if (s + 1 < steps) stash((s + 1) & 1);   // the other buffer: every wave finished reading it before the last barrier
        __syncthreads();
    }

    // accumulator register v of a lane: row 8 (v / 4) + 4 h + v % 4 of the 32x32 tile, column `col`
    {
        float dot = 0.0f;
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int j = 0; j < WN; ++j) {
                const int n = n0 + (wn * WN + j) * 32 + col;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + (wm * WM + i) * 32 + 8 * (v / 4) + 4 * h + (v % 4);
                    if (m >= g.Mr || n >= g.Nr) continue;
                    const float a = acc[i][j][v];
                    if (g.splits > 1) {
                        g.part[((size_t)split * g.Mr + m) * g.Nr + n] = a;
                        continue;
                    }
                    store_result(g, m, n, a);
                    if (g.D) dot = fmaf(a, (float)__builtin_bit_cast(half_t, g.D[(size_t)m * g.ldd + n]), dot);
                }
            }
        if (g.dot) {
            // fixed order: lanes by xor-shuffles, then the four waves in turn
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) dot += __shfl_xor(dot, off, 64);
            float *wsum = reinterpret_cast<float *>(lds);
            if (lane == 0) wsum[wave] = dot;
            __syncthreads();
            if (tid == 0) g.dot[tile] = ((wsum[0] + wsum[1]) + wsum[2]) + wsum[3];
        }
    }
}

// The store epilogue over the sum of the K splits' partial results, splits in index order.
__global__ __launch_bounds__(256) void fbq_sum_splits_kernel(GemmArgs g)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x, count = (size_t)g.Mr * g.Nr;
    if (i >= count) return;
    float a = 0.0f;
    for (int sp = 0; sp < g.splits; ++sp) a += g.part[(size_t)sp * count + i];
    store_result(g, (int)(i / g.Nr), (int)(i % g.Nr), a);
}

// Tile shapes: 128 x 128 in general, 64 rows or 64 columns where an operand has no more than that (the
// r-row products at r <= 64).  Larger tiles (256 x 128 at one block per CU: 4096^3 at 547 instead of
// 650 TFLOP/s; 256 x 256: spills) were measured and dropped: with a single block per CU nothing runs
// while its waves wait at the barrier.  K steps of 32 with up to four blocks per CU: 594 instead of 624 TFLOP/s.
struct TileShape { int wm, wn; };
static TileShape tile_for(int Mr, int Nr)
{
    if (Mr <= 64) return {1, 2};
    if (Nr <= 64) return {2, 1};
    return {2, 2};
}
static int tiles_of(int Mr, int Nr)
{
    const TileShape t = tile_for(Mr, Nr);
    return ceil_div(Mr, 64 * t.wm) * ceil_div(Nr, 64 * t.wn);
}

// Blocks that split K for one tile: enough to give every CU a block when the tiles alone do not,
// at least 4 steps each, and none left without a step.
static int splits_for(int Mr, int Nr, int Kd)
{
    const int tiles = tiles_of(Mr, Nr), steps = Kd / kStepK;
    const int want = std::min(256 / std::max(tiles, 1), steps / 4);
    if (want < 2) return 1;
    return ceil_div(steps, ceil_div(steps, want));
}

static size_t split_scratch_bytes(int Mr, int Nr, int Kd)
{
    const int sp = splits_for(Mr, Nr, Kd);
    return sp > 1 ? (size_t)sp * Mr * Nr * 4 : 0;
}

template <int WM, int WN>
static void launch_gemm_tile(const GemmArgs &g, dim3 grid, hipStream_t stream)
{
    constexpr int bytes = 2 * (64 * WM + 64 * WN) * kStepK * 2;
    static_assert(bytes <= 65536, "more LDS than a launch may ask for without raising the function's limit");
    hipLaunchKernelGGL((fbq_gemm_nt_kernel<WM, WN>), grid, dim3(256), bytes, stream, g);
}

static hipError_t launch_gemm(GemmArgs g, float *split_scratch, hipStream_t stream)
{
    g.splits = (!g.dot && split_scratch) ? splits_for(g.Mr, g.Nr, g.Kd) : 1;
    g.part = split_scratch;
    const TileShape t = tile_for(g.Mr, g.Nr);
    const int units = tiles_of(g.Mr, g.Nr) * g.splits;
    const dim3 grid(ceil_div(units, kXcds) * kXcds);
    if (t.wm == 1) launch_gemm_tile<1, 2>(g, grid, stream);
    else if (t.wn == 1) launch_gemm_tile<2, 1>(g, grid, stream);
    else launch_gemm_tile<2, 2>(g, grid, stream);
    if (g.splits > 1)
        hipLaunchKernelGGL(fbq_sum_splits_kernel, dim3((unsigned)(((size_t)g.Mr * g.Nr + 255) / 256)), dim3(256), 0, stream, g);
    return hipGetLastError();
}

static GemmArgs gemm_args(const uint16_t *A, int Mr, int lda, const uint16_t *B, int Nr, int ldb, int Kd)
{
    GemmArgs g{};
    g.A = A; g.B = B; g.Mr = Mr; g.Nr = Nr; g.Kd = Kd; g.lda = lda; g.ldb = ldb;
    g.c32_rows = Mr; g.c16_row0 = 0; g.splits = 1;
    return g;
}

// dst [C][ldd] = transpose of src [R][C] (fp16), columns R..ldd-1 of dst zero.  Block (32, 8), tile 32x32.
__global__ __launch_bounds__(256) void fbq_transpose_f16_kernel(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst,
                                                                int R, int C, int ldd)
{
    __shared__ uint16_t t[32][33];
    const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
    for (int i = threadIdx.y; i < 32; i += 8) {
        const int r = r0 + i, c = c0 + threadIdx.x;
        t[i][threadIdx.x] = (r < R && c < C) ? src[(size_t)r * C + c] : (uint16_t)0;
    }
    __syncthreads();
    for (int i = threadIdx.y; i < 32; i += 8) {
        const int c = c0 + i, r = r0 + threadIdx.x;
        if (c < C && r < ldd) dst[(size_t)c * ldd + r] = t[threadIdx.x][i];
    }
}

// fp16 views of the fp32 masters: At16 [r][K] and Bt16 [N][r] (the inference layouts, outputs of the
// step; At16 once more as the lower half of the stacked operand [Q; At]) and Bc [r][Np] = B with
// rows contiguous along n, columns N..Np-1 zero.
__global__ __launch_bounds__(256) void fbq_cast_masters_kernel(const float *__restrict__ At32, const float *__restrict__ Bt32,
                                                               uint16_t *__restrict__ At16, uint16_t *__restrict__ Bt16,
                                                               uint16_t *__restrict__ At16_stacked, uint16_t *__restrict__ Bc,
                                                               int N, int K, int r, int Np)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t nA = (size_t)r * K, nB = (size_t)N * r, nC = (size_t)r * Np;
    if (i < nA) {
        const uint16_t v = __builtin_bit_cast(uint16_t, (half_t)At32[i]);
        At16[i] = v;
        At16_stacked[i] = v;
    } else if (i < nA + nB) {
        Bt16[i - nA] = __builtin_bit_cast(uint16_t, (half_t)Bt32[i - nA]);
    } else if (i < nA + nB + nC) {
        const size_t e = i - nA - nB;
        const int j = (int)(e / Np), n = (int)(e % Np);
        Bc[e] = n < N ? __builtin_bit_cast(uint16_t, (half_t)Bt32[(size_t)n * r + j]) : (uint16_t)0;
    }
}

// loss = scale * (sum of the tiles' partial sums, in index order), by one block.
__global__ __launch_bounds__(256) void fbq_loss_kernel(const float *__restrict__ part, int n, float scale, float *__restrict__ loss)
{
    __shared__ double s[256];
    double a = 0.0;
    for (int i = threadIdx.x; i < n; i += 256) a += (double)part[i];
    s[threadIdx.x] = a;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) s[threadIdx.x] += s[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = (float)(s[0] * (double)scale);
}

// masters <- masters - lr gradient  (Alg. 1, the update line), both arrays in one launch.
__global__ __launch_bounds__(256) void fbq_descent_kernel(float *__restrict__ At32, const float *__restrict__ gAt, size_t nA,
                                                          float *__restrict__ Bt32, const float *__restrict__ gBt, size_t nB, float lr)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < nA) At32[i] = At32[i] - lr * gAt[i];
    else if (i < nA + nB) Bt32[i - nA] = Bt32[i - nA] - lr * gBt[i - nA];
}

static size_t pad256(size_t b) { return (b + 255) & ~(size_t)255; }
static int pad64(int v) { return (v + 63) & ~63; }

constexpr float kVGain = 64.0f;      // V^T = At H is stored as fp16(64 h_scale At H)

struct TrainLayout {
    size_t Bc, D16, Dt16, S16, Vt16, dot, split, total;
};

static TrainLayout train_layout(int N, int K, int r)
{
    const int Np = pad64(N);
    TrainLayout l{};
    size_t o = 0;
    l.Bc = o;   o += pad256((size_t)r * Np * 2);
    l.D16 = o;  o += pad256((size_t)N * K * 2);
    l.Dt16 = o; o += pad256((size_t)K * Np * 2);
    l.S16 = o;  o += pad256((size_t)2 * r * K * 2);          // stacked operand [Q; At]
    l.Vt16 = o; o += pad256((size_t)r * K * 2);
    l.dot = o;  o += pad256((size_t)ceil_div(N, 64) * ceil_div(K, 64) * 4);           // enough for any tile shape
    l.split = o;
    o += pad256(std::max(std::max(split_scratch_bytes(r, K, Np), split_scratch_bytes(2 * r, K, K)), split_scratch_bytes(N, r, K)));
    l.total = o;
    return l;
}

size_t train_workspace_bytes(int N, int K, int r, int T)
{
    const int Tp = pad64(T);
    return std::max(train_layout(N, K, r).total, pad256((size_t)K * Tp * 2) + pad256(split_scratch_bytes(K, K, Tp)));
}

hipError_t launch_gram(int K, int T, const uint16_t *X, float h_scale, uint16_t *H16, void *workspace, hipStream_t stream)
{
    const int Tp = pad64(T);
    uint16_t *Xt = (uint16_t *)workspace;                       // [K][Tp], tokens past T zero
    float *scratch = (float *)((unsigned char *)workspace + pad256((size_t)K * Tp * 2));
    hipLaunchKernelGGL(fbq_transpose_f16_kernel, dim3(ceil_div(K, 32), ceil_div(Tp, 32)), dim3(32, 8), 0, stream, X, Xt, T, K, Tp);
    GemmArgs g = gemm_args(Xt, K, Tp, Xt, K, Tp, Tp);
    g.C16 = H16; g.ldc16 = K; g.beta = h_scale;
    return launch_gemm(g, scratch, stream);
}

hipError_t launch_train_step(const TrainArgs &a, hipStream_t stream)
{
    const int N = a.d.N, K = a.d.K, r = a.d.r, Np = pad64(N);
    const TrainLayout l = train_layout(N, K, r);
    unsigned char *ws = (unsigned char *)a.workspace;
    uint16_t *Bc = (uint16_t *)(ws + l.Bc);
    uint16_t *D16 = (uint16_t *)(ws + l.D16), *Dt16 = (uint16_t *)(ws + l.Dt16);
    uint16_t *S16 = (uint16_t *)(ws + l.S16), *Vt16 = (uint16_t *)(ws + l.Vt16);
    float *dot = (float *)(ws + l.dot), *scratch = (float *)(ws + l.split);
    const int tiles = tiles_of(N, K);

    // fp16 views of the masters: what the forward pass of Alg. 1 computes with
    const size_t casts = (size_t)r * K + (size_t)N * r + (size_t)r * Np;
    hipLaunchKernelGGL(fbq_cast_masters_kernel, dim3((unsigned)((casts + 255) / 256)), dim3(256), 0, stream, a.At32, a.Bt32, a.At16,
                       a.Bt16, S16 + (size_t)r * K, Bc, N, K, r, Np);
    // Q(W - Sigma16), written in the inference layout, and Delta_F = (W - Sigma16) - Q(W - Sigma16), times 256,
    // in both orientations
    hipError_t e = launch_quantize(a.d, a.W, a.At16, a.Bt16, a.qw, a.scales, a.zeros, stream, D16, Dt16, Np, kDeltaGain);
    if (e != hipSuccess) return e;
    // Q = Bt^T Delta_F (times 256), the upper half of the stacked operand
    {
        GemmArgs g = gemm_args(Bc, r, Np, Dt16, K, Np, Np);
        g.C16 = S16; g.ldc16 = K; g.beta = 1.0f;
        if ((e = launch_gemm(g, scratch, stream)) != hipSuccess) return e;
    }
    // [Q; At] H (H symmetric): rows of Q give dL/dAt = -2 Q H, rows of At give V^T = At H
    {
        GemmArgs g = gemm_args(S16, 2 * r, K, a.H16, K, K, K);
        g.C32 = a.gAt; g.ldc32 = K; g.alpha = -2.0f / (kDeltaGain * a.h_scale); g.c32_rows = r;
        g.C16 = Vt16; g.ldc16 = K; g.beta = kVGain; g.c16_row0 = r;
        if ((e = launch_gemm(g, scratch, stream)) != hipSuccess) return e;
    }
    // dL/dBt = -2 Delta_F H At^T = -2 Delta_F V
    {
        GemmArgs g = gemm_args(D16, N, K, Vt16, r, K, K);
        g.C32 = a.gBt; g.ldc32 = r; g.alpha = -2.0f / (kDeltaGain * kVGain * a.h_scale);
        if ((e = launch_gemm(g, scratch, stream)) != hipSuccess) return e;
    }
    // L = sum Delta_F o (Delta_F H): the only use of the full product, and only on request
    if (a.loss) {
        GemmArgs g = gemm_args(D16, N, K, a.H16, K, K, K);
        g.D = D16; g.ldd = K; g.dot = dot;
        if ((e = launch_gemm(g, nullptr, stream)) != hipSuccess) return e;
        hipLaunchKernelGGL(fbq_loss_kernel, dim3(1), dim3(256), 0, stream, dot, tiles, 1.0f / (kDeltaGain * kDeltaGain * a.h_scale),
                           a.loss);
    }
    // gradient descent on the masters
    const size_t nA = (size_t)r * K, nB = (size_t)N * r;
    hipLaunchKernelGGL(fbq_descent_kernel, dim3((unsigned)((nA + nB + 255) / 256)), dim3(256), 0, stream, a.At32, a.gAt, nA, a.Bt32,
                       a.gBt, nB, a.lr);
    return hipGetLastError();
}

}  // namespace fbq
