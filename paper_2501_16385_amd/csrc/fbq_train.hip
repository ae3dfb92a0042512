// Layer-wise reconstruction (Alg. 1, Sec. 4.2): one gradient-descent iteration on the sub-branch
// of one layer.
//
// The loss and its gradient depend on the calibration activations X [T,K] only through
// H = X^T X (Sec. 4.2: L = tr(Delta_F H Delta_F^T), dL/dSigma = -2 Delta_F H with the feedback
// detached), so H is formed once per layer and an iteration is
//
//   A16, B16   <- fp16 of the fp32 masters                               (cast kernel)
//   q, s, z    <- Q(W - Sigma16)               feedback quantizer        (fbq_quantize_kernel)
//   Delta_F    <- W - s (q - z) - Sigma16      Sigma16 by matrix cores   (GEMM, "delta" epilogue)
//   P          <- Delta_F H                    the dominant contraction  (GEMM, 2 N K^2 flop)
//   L          <- sum Delta_F o P                                        (same launch, then a reduction)
//   dL/dBt     <- -2 P At^T           [N,r]                              (GEMM)
//   dL/dAt     <- -2 (Bt^T Delta_F) H [r,K]                              (two GEMMs)
//   masters    <- masters - lr gradient                                  (update kernel)
//
// with Sigma[n,k] = sum_j Bt[n,j] At[j,k] in the device layouts At [r,K], Bt [N,r].
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

constexpr int kTile = 128;           // block tile, both ways
constexpr int kStepK = 64;           // k per step: one 128-byte row segment per operand row
constexpr float kDeltaGain = 256.0f; // Delta_F is stored as fp16(256 Delta_F)
constexpr int kXcds = 8;

enum { kEpiStore = 0, kEpiDelta = 1 };

struct GemmArgs {
    const uint16_t *A;   // [Mr][lda] fp16
    const uint16_t *B;   // [Nr][ldb] fp16
    int Mr, Nr, Kd;      // Kd a multiple of 64
    int lda, ldb;        // elements
    // store epilogue (any of the three may be absent)
    float *C32; int ldc32; float alpha;          // C32[m,n] = alpha acc
    uint16_t *C16; int ldc16; float beta;        // C16[m,n] = fp16(beta acc)
    const uint16_t *D; int ldd; float *dot;      // dot[tile] = sum over the tile of acc D[m,n]
    // delta epilogue: acc is Sigma[m,n] (m a weight row, n an input feature)
    const uint16_t *W; const uint32_t *qw; const uint16_t *scales; const uint16_t *zeros;
    uint16_t *D16; uint16_t *Dt16; int ldt;      // D16 [Mr][Nr], Dt16 [Nr][ldt] = its transpose; both 256 Delta_F
    int bits, row_words;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t rows_buffer(const void *p, long bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

// 16-byte chunk c (0..7) of row `row` of an operand tile sits at chunk c ^ key(row): 8 or 16
// consecutive rows reading the same c touch every bank once, whether the LDS serves 128 or 256
// bytes per clock.
__device__ __forceinline__ int swizzle_key(int row) { return ((row >> 1) & 7) ^ ((row & 1) << 2); }

__device__ __forceinline__ uint32_t packed_code(const uint32_t *row, int bits, int k)
{
    if (bits == 4) return (row[k >> 3] >> ((k & 7) * 4)) & 15u;
    const uint32_t *u = row + (k >> 5) * 3;
    const int j = k & 31;
    if (j == 30) return ((u[0] >> 15) & 1u) | (((u[1] >> 15) & 1u) << 1) | (((u[2] >> 15) & 1u) << 2);
    if (j == 31) return (u[0] >> 31) | ((u[1] >> 31) << 1) | ((u[2] >> 31) << 2);
    const int wd = j / 10, f = j % 10;
    return (u[wd] >> (f < 5 ? 3 * f : 16 + 3 * (f - 5))) & 7u;
}

template <int EPI>
__global__ __launch_bounds__(256, 2) void fbq_gemm_nt_kernel(GemmArgs g)
{
    __shared__ __align__(16) unsigned char lds[2 * 2 * kTile * kStepK * 2];   // [buffer][operand][row][128 bytes]
    constexpr int kOperandBytes = kTile * kStepK * 2;

    // Consecutive tiles (same rows of A, neighbouring rows of B) run on the same XCD and share its L2.
    const int tiles_n = (g.Nr + kTile - 1) / kTile, tiles_m = (g.Mr + kTile - 1) / kTile;
    const int total = tiles_m * tiles_n, per_xcd = (total + kXcds - 1) / kXcds;
    const int tile = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    if (tile >= total) return;
    const int m0 = (tile / tiles_n) * kTile, n0 = (tile % tiles_n) * kTile;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int col = lane & 31, h = lane >> 5;

    const __amdgpu_buffer_rsrc_t abuf = rows_buffer(g.A + (size_t)m0 * g.lda, (long)min(kTile, g.Mr - m0) * g.lda * 2);
    const __amdgpu_buffer_rsrc_t bbuf = rows_buffer(g.B + (size_t)n0 * g.ldb, (long)min(kTile, g.Nr - n0) * g.ldb * 2);

    int goff_a[4], goff_b[4], loff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = tid + 256 * i, row = c >> 3, ch = c & 7;
        goff_a[i] = row * g.lda * 2 + ch * 16;
        goff_b[i] = row * g.ldb * 2 + ch * 16;
        loff[i] = row * 128 + ((ch ^ swizzle_key(row)) * 16);
    }
    uint4_t ra[4], rb[4];
    auto fetch = [&](int s) {
#pragma unroll
        for (int i = 0; i < 4; ++i) ra[i] = __builtin_bit_cast(uint4_t, __builtin_amdgcn_raw_buffer_load_b128(abuf, goff_a[i] + s * 128, 0, 0));
#pragma unroll
        for (int i = 0; i < 4; ++i) rb[i] = __builtin_bit_cast(uint4_t, __builtin_amdgcn_raw_buffer_load_b128(bbuf, goff_b[i] + s * 128, 0, 0));
    };
    auto stash = [&](int buf) {
        unsigned char *la = lds + (buf * 2 + 0) * kOperandBytes, *lb = lds + (buf * 2 + 1) * kOperandBytes;
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4_t *>(la + loff[i]) = ra[i];
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4_t *>(lb + loff[i]) = rb[i];
    };

    float16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // operand rows of this lane: 32 rows apart, so they share the swizzle key
    const int key = swizzle_key(col);
    const int arow = (wm * 64 + col) * 128, brow = (wn * 64 + col) * 128;
    auto multiply = [&](int buf) {
        const unsigned char *la = lds + (buf * 2 + 0) * kOperandBytes, *lb = lds + (buf * 2 + 1) * kOperandBytes;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int chunk = ((kk * 2 + h) ^ key) * 16;
            half8_t af[2], bf[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) af[i] = *reinterpret_cast<const half8_t *>(la + arow + i * 32 * 128 + chunk);
#pragma unroll
            for (int j = 0; j < 2; ++j) bf[j] = *reinterpret_cast<const half8_t *>(lb + brow + j * 32 * 128 + chunk);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
    };

    const int steps = g.Kd / kStepK;
    fetch(0);
    stash(0);
    __syncthreads();
    for (int s = 0; s < steps; ++s) {
        if (s + 1 < steps) fetch(s + 1);
        multiply(s & 1);
        if (s + 1 < steps) stash((s + 1) & 1);   // the other buffer: every wave finished reading it before the last barrier
        __syncthreads();
    }

    // accumulator register v of a lane: row 8 (v / 4) + 4 h + v % 4 of the 32x32 tile, column `col`
    if (EPI == kEpiStore) {
        float dot = 0.0f;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int n = n0 + wn * 64 + j * 32 + col;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + wm * 64 + i * 32 + 8 * (v / 4) + 4 * h + (v % 4);
                    if (m >= g.Mr || n >= g.Nr) continue;
                    const float a = acc[i][j][v];
                    if (g.C32) g.C32[(size_t)m * g.ldc32 + n] = g.alpha * a;
                    if (g.C16) g.C16[(size_t)m * g.ldc16 + n] = __builtin_bit_cast(uint16_t, (half_t)(g.beta * a));
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
    } else {
        // Delta_F = W - s (q - z) - Sigma for weight row m and input feature n, times 256, in both orientations
        const int G = g.Nr / kGroup;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int n = n0 + wn * 64 + j * 32 + col;
                if (n >= g.Nr) continue;
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    const int mb = m0 + wm * 64 + i * 32 + 8 * vq + 4 * h;
                    half4_t out;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int m = mb + e;
                        float val = 0.0f;
                        if (m < g.Mr) {
                            const float w = (float)__builtin_bit_cast(half_t, g.W[(size_t)m * g.Nr + n]);
                            const float s = (float)__builtin_bit_cast(half_t, g.scales[(size_t)m * G + n / kGroup]);
                            const float z = (float)__builtin_bit_cast(half_t, g.zeros[(size_t)m * G + n / kGroup]);
                            const float q = (float)packed_code(g.qw + (size_t)m * g.row_words, g.bits, n);
                            val = kDeltaGain * (w - s * (q - z) - acc[i][j][vq * 4 + e]);
                            g.D16[(size_t)m * g.Nr + n] = __builtin_bit_cast(uint16_t, (half_t)val);
                        }
                        out[e] = (half_t)val;
                    }
                    if (mb < g.ldt) *reinterpret_cast<half4_t *>(g.Dt16 + (size_t)n * g.ldt + mb) = out;   // rows past Mr: zeros
                }
            }
    }
}

static hipError_t launch_gemm(const GemmArgs &g, int epi, hipStream_t stream)
{
    const int tiles = ceil_div(g.Mr, kTile) * ceil_div(g.Nr, kTile);
    const dim3 grid(ceil_div(tiles, kXcds) * kXcds);
    if (epi == kEpiStore) hipLaunchKernelGGL(fbq_gemm_nt_kernel<kEpiStore>, grid, dim3(256), 0, stream, g);
    else hipLaunchKernelGGL(fbq_gemm_nt_kernel<kEpiDelta>, grid, dim3(256), 0, stream, g);
    return hipGetLastError();
}

static GemmArgs gemm_args(const uint16_t *A, int Mr, int lda, const uint16_t *B, int Nr, int ldb, int Kd)
{
    GemmArgs g{};
    g.A = A; g.B = B; g.Mr = Mr; g.Nr = Nr; g.Kd = Kd; g.lda = lda; g.ldb = ldb;
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
// step), and zero-padded operand copies: Ac [K][rp] (A, contiguous along r), Bp [N][rp], Bc [r][Np].
__global__ __launch_bounds__(256) void fbq_cast_masters_kernel(const float *__restrict__ At32, const float *__restrict__ Bt32,
                                                               uint16_t *__restrict__ At16, uint16_t *__restrict__ Bt16,
                                                               uint16_t *__restrict__ Ac, uint16_t *__restrict__ Bp,
                                                               uint16_t *__restrict__ Bc, int N, int K, int r, int rp, int Np)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t nA = (size_t)K * rp, nB = (size_t)N * rp, nC = (size_t)r * Np;
    if (i < nA) {
        const int k = (int)(i / rp), j = (int)(i % rp);
        uint16_t v = 0;
        if (j < r) {
            v = __builtin_bit_cast(uint16_t, (half_t)At32[(size_t)j * K + k]);
            At16[(size_t)j * K + k] = v;
        }
        Ac[i] = v;
    } else if (i < nA + nB) {
        const size_t e = i - nA;
        const int n = (int)(e / rp), j = (int)(e % rp);
        uint16_t v = 0;
        if (j < r) {
            v = __builtin_bit_cast(uint16_t, (half_t)Bt32[(size_t)n * r + j]);
            Bt16[(size_t)n * r + j] = v;
        }
        Bp[e] = v;
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

struct TrainLayout {
    size_t Ac, Bp, Bc, D16, Dt16, P16, Q16, dot, total;
};

static TrainLayout train_layout(int N, int K, int r)
{
    const int rp = pad64(r), Np = pad64(N);
    TrainLayout l{};
    size_t o = 0;
    l.Ac = o;   o += pad256((size_t)K * rp * 2);
    l.Bp = o;   o += pad256((size_t)N * rp * 2);
    l.Bc = o;   o += pad256((size_t)r * Np * 2);
    l.D16 = o;  o += pad256((size_t)N * K * 2);
    l.Dt16 = o; o += pad256((size_t)K * Np * 2);
    l.P16 = o;  o += pad256((size_t)N * K * 2);
    l.Q16 = o;  o += pad256((size_t)r * K * 2);
    l.dot = o;  o += pad256((size_t)ceil_div(N, kTile) * ceil_div(K, kTile) * 4);
    l.total = o;
    return l;
}

size_t train_workspace_bytes(int N, int K, int r, int T)
{
    return std::max(train_layout(N, K, r).total, pad256((size_t)K * pad64(T) * 2));
}

hipError_t launch_gram(int K, int T, const uint16_t *X, float h_scale, uint16_t *H16, void *workspace, hipStream_t stream)
{
    const int Tp = pad64(T);
    uint16_t *Xt = (uint16_t *)workspace;                       // [K][Tp], tokens past T zero
    hipLaunchKernelGGL(fbq_transpose_f16_kernel, dim3(ceil_div(K, 32), ceil_div(Tp, 32)), dim3(32, 8), 0, stream, X, Xt, T, K, Tp);
    GemmArgs g = gemm_args(Xt, K, Tp, Xt, K, Tp, Tp);
    g.C16 = H16; g.ldc16 = K; g.beta = h_scale;
    return launch_gemm(g, kEpiStore, stream);
}

hipError_t launch_train_step(const TrainArgs &a, hipStream_t stream)
{
    const int N = a.d.N, K = a.d.K, r = a.d.r, rp = pad64(r), Np = pad64(N);
    const TrainLayout l = train_layout(N, K, r);
    unsigned char *ws = (unsigned char *)a.workspace;
    uint16_t *Ac = (uint16_t *)(ws + l.Ac), *Bp = (uint16_t *)(ws + l.Bp), *Bc = (uint16_t *)(ws + l.Bc);
    uint16_t *D16 = (uint16_t *)(ws + l.D16), *Dt16 = (uint16_t *)(ws + l.Dt16), *P16 = (uint16_t *)(ws + l.P16);
    uint16_t *Q16 = (uint16_t *)(ws + l.Q16);
    float *dot = (float *)(ws + l.dot);
    const int tiles = ceil_div(N, kTile) * ceil_div(K, kTile);

    // fp16 views of the masters: what the forward pass of Alg. 1 computes with
    const size_t casts = (size_t)K * rp + (size_t)N * rp + (size_t)r * Np;
    hipLaunchKernelGGL(fbq_cast_masters_kernel, dim3((unsigned)((casts + 255) / 256)), dim3(256), 0, stream, a.At32, a.Bt32, a.At16,
                       a.Bt16, Ac, Bp, Bc, N, K, r, rp, Np);
    // Q(W - Sigma16): the feedback quantizer, written in the inference layout
    hipError_t e = launch_quantize(a.d, a.W, a.At16, a.Bt16, a.qw, a.scales, a.zeros, stream);
    if (e != hipSuccess) return e;
    // Delta_F = W - Q(W - Sigma16) - Sigma16, Sigma16[n,k] = sum_j Bt16[n,j] A16[k,j]
    {
        GemmArgs g = gemm_args(Bp, N, rp, Ac, K, rp, rp);
        g.W = a.W; g.qw = a.qw; g.scales = a.scales; g.zeros = a.zeros;
        g.D16 = D16; g.Dt16 = Dt16; g.ldt = Np; g.bits = a.d.bits; g.row_words = (int)row_words(K, a.d.bits);
        if ((e = launch_gemm(g, kEpiDelta, stream)) != hipSuccess) return e;
    }
    // P = Delta_F H (H symmetric), kept as fp16(256 h_scale P); the tiles' shares of sum Delta_F o P
    {
        GemmArgs g = gemm_args(D16, N, K, a.H16, K, K, K);
        g.C16 = P16; g.ldc16 = K; g.beta = 1.0f;
        g.D = D16; g.ldd = K; g.dot = dot;
        if ((e = launch_gemm(g, kEpiStore, stream)) != hipSuccess) return e;
    }
    hipLaunchKernelGGL(fbq_loss_kernel, dim3(1), dim3(256), 0, stream, dot, tiles, 1.0f / (kDeltaGain * kDeltaGain * a.h_scale), a.loss);
    const float gscale = -2.0f / (kDeltaGain * a.h_scale);
    // dL/dBt = -2 P At^T
    {
        GemmArgs g = gemm_args(P16, N, K, a.At16, r, K, K);
        g.C32 = a.gBt; g.ldc32 = r; g.alpha = gscale;
        if ((e = launch_gemm(g, kEpiStore, stream)) != hipSuccess) return e;
    }
    // dL/dAt = -2 (Bt^T Delta_F) H
    {
        GemmArgs g = gemm_args(Bc, r, Np, Dt16, K, Np, Np);
        g.C16 = Q16; g.ldc16 = K; g.beta = 1.0f;
        if ((e = launch_gemm(g, kEpiStore, stream)) != hipSuccess) return e;
        GemmArgs g2 = gemm_args(Q16, r, K, a.H16, K, K, K);
        g2.C32 = a.gAt; g2.ldc32 = K; g2.alpha = gscale;
        if ((e = launch_gemm(g2, kEpiStore, stream)) != hipSuccess) return e;
    }
    // gradient descent on the masters
    const size_t nA = (size_t)r * K, nB = (size_t)N * r;
    hipLaunchKernelGGL(fbq_descent_kernel, dim3((unsigned)((nA + nB + 255) / 256)), dim3(256), 0, stream, a.At32, a.gAt, nA, a.Bt32,
                       a.gBt, nB, a.lr);
    return hipGetLastError();
}

}  // namespace fbq
