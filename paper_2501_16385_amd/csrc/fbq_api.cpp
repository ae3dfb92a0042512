// C ABI of the library: argument validation, host-side packing and kernel dispatch.
// Every operation is defined in include/fbq.h; nothing here computes on the CPU except fbq_pack
// (a one-off layout conversion that is off the hot path by definition).
#include <string.h>

#include <atomic>

#include "fbq_internal.h"

using namespace fbq;

extern "C" const char *fbq_status_string(fbq_status s)
{
    switch (s) {
    case FBQ_OK: return "ok";
    case FBQ_ERR_NULL: return "null pointer";
    case FBQ_ERR_SHAPE: return "bad shape or value";
    case FBQ_ERR_UNSUPPORTED: return "unsupported configuration";
    case FBQ_ERR_ALIGN: return "device pointer not 16-byte aligned";
    case FBQ_ERR_WORKSPACE: return "workspace too small";
    case FBQ_ERR_HIP: return "HIP launch error";
    }
    return "unknown status";
}

extern "C" fbq_status fbq_check_desc(const fbq_desc *d)
{
    if (!d) return FBQ_ERR_NULL;
    if (d->bits != 3 && d->bits != 4) return FBQ_ERR_UNSUPPORTED;
    if (d->group != kGroup) return FBQ_ERR_UNSUPPORTED;
    if (d->N < 1 || d->K < 1 || d->r < 0) return FBQ_ERR_SHAPE;
    if (d->K % d->group || d->K % 32 || d->r % 8) return FBQ_ERR_SHAPE;
    if (d->r > kMaxRank || d->K > kMaxK) return FBQ_ERR_UNSUPPORTED;
    // the kernels address a layer's buffers with 32-bit byte offsets and keep 2^30 as "nowhere"
    if ((size_t)d->N * row_words(d->K, d->bits) * sizeof(uint32_t) >= ((size_t)1 << 30)) return FBQ_ERR_UNSUPPORTED;
    if ((size_t)d->N * d->r * sizeof(uint16_t) >= ((size_t)1 << 30)) return FBQ_ERR_UNSUPPORTED;   // (B^T likewise)
    return FBQ_OK;
}

extern "C" size_t fbq_packed_bytes(const fbq_desc *d)
{
    if (fbq_check_desc(d) != FBQ_OK) return 0;
    return (size_t)d->N * row_words(d->K, d->bits) * sizeof(uint32_t);
}

// 17..64 tokens: whether the few-token kernel, the sets of 16 tokens side by side in one launch, is expected to beat
// the prefill GEMM.  It streams the packed words once per set, in passes of 4096 along K; the GEMM reads them once
// but has a long start (three launches, few tiles) and a K loop per tile that few tiles cannot hide.  Fitted to
// measurements of both at 32, 48 and 64 tokens on ten shapes (us; MC = millions of codes, K counted in whole passes
// for the sets): the sets take about 2 + sets x (2.2 + 0.165 MC), the GEMM 30 + 0.135 MC + 1.5 K / 1024 (with INT3
// and INT4 alike).  Examples, sets / GEMM: 8192 -> 28672 at 32 tokens 84 / 71, at 64 160 / 83; 28672 -> 8192 at 32
// tokens 80 / 101, at 48 122 / 101; 4096 -> 11008 at 64 tokens 35 / 41; 13824 -> 5120 at 48 tokens 50 / 62.
static bool sets_beat_gemm(int M, int N, int K)
{
    const int sets = (M + kDecodeMaxM - 1) / kDecodeMaxM;
    const double k_passes = 4096.0 * ((K + 4095) / 4096);
    const double cost_sets = 2.0 + sets * (2.2 + 0.165e-6 * N * k_passes);
    const double cost_gemm = 30.0 + 0.135e-6 * N * (double)K + 1.5 * K / 1024.0;
    return cost_sets <= cost_gemm;
}

// In front of what the prefill path keeps in a workspace: room for the hand-over words of the decode paths, which the
// prefill path never touches.  A workspace that serves calls of every token count then only ever holds words with a
// launch's tag, or the zeros it started with, where the decode kernels look for tags - never activations or partial
// sums that happen to look like one.
static size_t handover_reserve(int K, int r)
{
    return r > 0 ? (size_t)kMaxSmallGroup * small_m_workspace_bytes(K, r) : 0;
}

extern "C" size_t fbq_workspace_bytes(const fbq_desc *d, int M)
{
    if (fbq_check_desc(d) != FBQ_OK || M < 1) return 0;
    if (M <= kPerTokenMaxM) return d->r == 0 ? 0 : decode_workspace_bytes(M, d->K, d->r);
    // up to 64 tokens go through the few-token kernel 16 at a time, all in one launch, every 16 tokens with hand-over
    // words of their own (one or two left over go through the GEMV afterwards, whose words fit the first set);
    // nothing to hand over without a sub-branch
    if (M <= kDecodeMaxM) return small_m_workspace_bytes(d->K, d->r);
    if (M <= kChunkedMaxM && sets_beat_gemm(M, d->N, d->K))
        return (size_t)((M + kDecodeMaxM - 1) / kDecodeMaxM) * small_m_workspace_bytes(d->K, d->r);
    return handover_reserve(d->K, d->r) + prefill_workspace_bytes(M, d->N, d->K, d->r);      // holds the re-ordered activations even when r == 0
}

// ------------------------------------------------------------------ host-side packing

// Bit c of code k within a packed row: word index and bit position (layout in fbq.h).
static inline void code_bit_slot(int bits, int k, int c, size_t *word, int *bit)
{
    if (bits == 4) {
        *word = (size_t)k >> 3;
        *bit = ((k & 7) << 2) + c;
        return;
    }
    const int unit = k >> 5, j = k & 31;
    if (j >= 30) {
        *word = (size_t)unit * 3 + c;
        *bit = j == 30 ? 15 : 31;
        return;
    }
    const int wd = j / 10, f = j - wd * 10;
    *word = (size_t)unit * 3 + wd;
    *bit = (f >= 5 ? 16 + 3 * (f - 5) : 3 * f) + c;
}

extern "C" fbq_status fbq_pack(const fbq_desc *d, const uint8_t *codes, const uint16_t *scales, const uint16_t *zeros,
                               const uint16_t *A, const uint16_t *B, uint32_t *qweight_out, uint16_t *scales_out,
                               uint16_t *zeros_out, uint16_t *At_out, uint16_t *Bt_out)
{
    fbq_status st = fbq_check_desc(d);
    if (st != FBQ_OK) return st;
    if (!codes || !scales || !zeros || !qweight_out || !scales_out || !zeros_out) return FBQ_ERR_NULL;
    if (d->r > 0 && (!A || !B || !At_out || !Bt_out)) return FBQ_ERR_NULL;

    const int N = d->N, K = d->K, r = d->r, bits = d->bits;
    const size_t rw = row_words(K, bits);
    const unsigned qmax = (1u << bits) - 1u;
    memset(qweight_out, 0, rw * (size_t)N * sizeof(uint32_t));
    for (int n = 0; n < N; ++n) {
        uint32_t *row = qweight_out + rw * (size_t)n;
        const uint8_t *crow = codes + (size_t)n * K;
        for (int k = 0; k < K; ++k) {
            const unsigned q = crow[k];
            if (q > qmax) return FBQ_ERR_SHAPE;
            for (int c = 0; c < bits; ++c) {
                size_t w;
                int bit;
                code_bit_slot(bits, k, c, &w, &bit);
                row[w] |= ((q >> c) & 1u) << bit;
            }
        }
    }
    const size_t ng = (size_t)N * (K / d->group);
    memcpy(scales_out, scales, ng * sizeof(uint16_t));
    memcpy(zeros_out, zeros, ng * sizeof(uint16_t));
    if (r > 0) {
        for (int k = 0; k < K; ++k)
            for (int j = 0; j < r; ++j) At_out[(size_t)j * K + k] = A[(size_t)k * r + j];
        for (int n = 0; n < N; ++n)
            for (int j = 0; j < r; ++j) Bt_out[(size_t)n * r + j] = B[(size_t)j * N + n];
    }
    return FBQ_OK;
}

// ------------------------------------------------------------------ device entry points

static inline bool misaligned(const void *p) { return ((uintptr_t)p & 15u) != 0; }

namespace fbq {
fbq_status hip_status(hipError_t e)
{
    if (e == hipSuccess) e = hipGetLastError();
    return e == hipSuccess ? FBQ_OK : FBQ_ERR_HIP;
}
}  // namespace fbq

namespace fbq {

// Validates one layer's arguments and fills the launch record; nothing is launched here.
fbq_status check_layer(const fbq_desc *d, int M, const void *x, const void *qweight, const void *scales,
                              const void *zeros, const void *At, const void *Bt, void *y, void *workspace,
                              size_t workspace_bytes, LinearArgs *a)
{
    fbq_status st = fbq_check_desc(d);
    if (st != FBQ_OK) return st;
    if (M < 1) return FBQ_ERR_SHAPE;
    if (!x || !qweight || !scales || !zeros || !y) return FBQ_ERR_NULL;
    if (d->r > 0 && (!At || !Bt)) return FBQ_ERR_NULL;
    const size_t need = fbq_workspace_bytes(d, M);
    if (need > 0 && !workspace) return FBQ_ERR_NULL;
    if (misaligned(x) || misaligned(qweight) || misaligned(scales) || misaligned(zeros) || misaligned(y)) return FBQ_ERR_ALIGN;
    if (d->r > 0 && (misaligned(At) || misaligned(Bt))) return FBQ_ERR_ALIGN;
    if (need > 0 && misaligned(workspace)) return FBQ_ERR_ALIGN;
    if (workspace_bytes < need) return FBQ_ERR_WORKSPACE;
    a->qw = (const uint32_t *)qweight;
    a->scales = (const uint16_t *)scales;
    a->zeros = (const uint16_t *)zeros;
    a->At = (const uint16_t *)At;
    a->Bt = (const uint16_t *)Bt;
    a->x = (const uint16_t *)x;
    a->y = (uint16_t *)y;
    a->workspace = workspace;
    a->M = M; a->N = d->N; a->K = d->K; a->r = d->r; a->bits = d->bits;
    return FBQ_OK;
}

static hipError_t launch_prefill(const LinearArgs &call, hipStream_t s)
{
    LinearArgs a = call;
    a.workspace = (char *)call.workspace + handover_reserve(call.K, call.r);
    hipError_t e = launch_prepass_prefill(a, s);
    if (e == hipSuccess) e = launch_gemm_prefill(a, s);
    return e;
}

// One or two tokens: streaming GEMV, one pass per token, with the down-projection inside the launch.
// 3..16 tokens: one pass over the packed words against a matrix-core tile of tokens.  17..64 tokens:
// the same, 16 tokens at a time, the sets of 16 side by side in ONE launch as if they were layers of a group
// (the prefill GEMM has too few tiles to fill the GPU there), unless the layer is so large that reading its packed words
// three or four times costs more than the GEMM's long start.  More: the prefill GEMM.
hipError_t launch_one(const LinearArgs &a, hipStream_t s)
{
    if (a.M <= kPerTokenMaxM) return launch_gemv_decode(&a, 1, s);
    if (a.M <= kDecodeMaxM) return launch_gemv_small_m(&a, 1, s);
    if (a.M <= kChunkedMaxM && sets_beat_gemm(a.M, a.N, a.K)) {
        static_assert(kChunkedMaxM <= kMaxSmallGroup * kDecodeMaxM, "the sets of 16 tokens must fit one grouped launch");
        LinearArgs set[kMaxSmallGroup], rest = a;
        const size_t ws_each = small_m_workspace_bytes(a.K, a.r);
        int n = 0;
        rest.M = 0;
        for (int m0 = 0; m0 < a.M; m0 += kDecodeMaxM) {
            LinearArgs c = a;
            c.M = std::min(kDecodeMaxM, a.M - m0);
            c.x = a.x + (size_t)m0 * a.K;
            c.y = a.y + (size_t)m0 * a.N;
            if (c.M <= kPerTokenMaxM) { rest = c; continue; }   // one or two tokens left over: the GEMV is cheaper
            c.workspace = a.workspace ? (char *)a.workspace + (size_t)n * ws_each : nullptr;
            set[n++] = c;
        }
        hipError_t e = launch_gemv_small_m(set, n, s);
        // (the GEMV runs behind the grouped launch on the stream and marks its words with its own tag, whoever wrote there before)
        if (e == hipSuccess && rest.M > 0) e = launch_gemv_decode(&rest, 1, s);
        return e;
    }
    return launch_prefill(a, s);
}

}  // namespace fbq

extern "C" fbq_status fbq_linear_unfused(const fbq_desc *d, int M, const void *x, const void *qweight, const void *scales,
                                         const void *zeros, const void *At, const void *Bt, void *y, void *workspace,
                                         size_t workspace_bytes, fbq_stream stream)
{
    LinearArgs a;
    const fbq_status st = check_layer(d, M, x, qweight, scales, zeros, At, Bt, y, workspace, workspace_bytes, &a);
    if (st != FBQ_OK) return st;
    if (M > kDecodeMaxM) return FBQ_ERR_UNSUPPORTED;
    if (d->r > 0 && workspace_bytes < (size_t)M * d->r * sizeof(uint16_t)) return FBQ_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    LinearArgs main_path = a;                           // the quantized layer without its sub-branch ...
    main_path.r = 0; main_path.At = nullptr; main_path.Bt = nullptr;
    hipError_t e = launch_one(main_path, s);
    if (e == hipSuccess && d->r > 0) e = launch_unfused_branch(a, (uint16_t *)workspace, s);   // ... and the sub-branch on top
    return hip_status(e);
}

extern "C" fbq_status fbq_linear(const fbq_desc *d, int M, const void *x, const void *qweight, const void *scales,
                                 const void *zeros, const void *At, const void *Bt, void *y, void *workspace,
                                 size_t workspace_bytes, fbq_stream stream)
{
    LinearArgs a;
    const fbq_status st = check_layer(d, M, x, qweight, scales, zeros, At, Bt, y, workspace, workspace_bytes, &a);
    if (st != FBQ_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    return hip_status(launch_one(a, s));
}

extern "C" fbq_status fbq_linear_group(const fbq_layer_call *calls, int n, int M, fbq_stream stream)
{
    constexpr int kMaxCalls = 64;
    if (!calls) return FBQ_ERR_NULL;
    if (n < 1 || n > kMaxCalls) return FBQ_ERR_SHAPE;
    LinearArgs args[kMaxCalls];
    for (int i = 0; i < n; ++i) {
        const fbq_layer_call &c = calls[i];
        const fbq_status st = check_layer(&c.desc, M, c.x, c.qweight, c.scales, c.zeros, c.At, c.Bt, c.y, c.workspace,
                                          c.workspace_bytes, &args[i]);
        if (st != FBQ_OK) return st;
    }
    // Layers that share a launch carry the same launch tag: two of them writing their hand-over words into the same
    // memory would accept each other's t.  Workspaces must not overlap.
    for (int i = 0; i < n; ++i) {
        const size_t ni = fbq_workspace_bytes(&calls[i].desc, M);
        if (!ni) continue;
        const uintptr_t ai = (uintptr_t)calls[i].workspace;
        for (int j = i + 1; j < n; ++j) {
            const size_t nj = fbq_workspace_bytes(&calls[j].desc, M);
            const uintptr_t aj = (uintptr_t)calls[j].workspace;
            if (nj && ai < aj + nj && aj < ai + ni) return FBQ_ERR_WORKSPACE;
        }
    }
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    if (M > kDecodeMaxM) {
        for (int i = 0; i < n && e == hipSuccess; ++i) e = launch_one(args[i], s);
        return hip_status(e);
    }
    // Decode: layers that fit one launch (the same kernel instance; for 4..16 tokens also the same
    // activations) are served together.
    const bool few = M > kPerTokenMaxM;
    const int cap = few ? kMaxSmallGroup : kMaxGroup;
    bool done[kMaxCalls] = {false};
    for (int i = 0; i < n && e == hipSuccess; ++i) {
        if (done[i]) continue;
        LinearArgs batch[kMaxGroup];
        int nb = 0;
        for (int j = i; j < n && nb < cap; ++j) {
            if (!done[j] && (few ? small_m_group_compatible(args[i], args[j]) : decode_group_compatible(args[i], args[j]))) {
                batch[nb++] = args[j];
                done[j] = true;
            }
        }
        e = few ? launch_gemv_small_m(batch, nb, s) : launch_gemv_decode(batch, nb, s);
    }
    return hip_status(e);
}

extern "C" fbq_status fbq_reconstruct(const fbq_desc *d, const void *qweight, const void *scales, const void *zeros,
                                      const void *At, const void *Bt, float *W_hat, fbq_stream stream)
{
    fbq_status st = fbq_check_desc(d);
    if (st != FBQ_OK) return st;
    if (!qweight || !scales || !zeros || !W_hat) return FBQ_ERR_NULL;
    if (d->r > 0 && (!At || !Bt)) return FBQ_ERR_NULL;
    if (misaligned(qweight) || misaligned(scales) || misaligned(zeros) || misaligned(W_hat)) return FBQ_ERR_ALIGN;
    if (d->r > 0 && (misaligned(At) || misaligned(Bt))) return FBQ_ERR_ALIGN;
    return hip_status(launch_reconstruct(*d, (const uint32_t *)qweight, (const uint16_t *)scales, (const uint16_t *)zeros,
                                         (const uint16_t *)At, (const uint16_t *)Bt, W_hat, (hipStream_t)stream));
}

extern "C" fbq_status fbq_unpack_codes(const fbq_desc *d, const void *qweight, uint8_t *codes_out, fbq_stream stream)
{
    fbq_status st = fbq_check_desc(d);
    if (st != FBQ_OK) return st;
    if (!qweight || !codes_out) return FBQ_ERR_NULL;
    if (misaligned(qweight) || misaligned(codes_out)) return FBQ_ERR_ALIGN;
    return hip_status(launch_unpack(*d, (const uint32_t *)qweight, codes_out, (hipStream_t)stream));
}

extern "C" fbq_status fbq_quantize_feedback(const fbq_desc *d, const void *W, const void *At, const void *Bt,
                                            void *qweight_out, void *scales_out, void *zeros_out, fbq_stream stream)
{
    fbq_status st = fbq_check_desc(d);
    if (st != FBQ_OK) return st;
    if (!W || !qweight_out || !scales_out || !zeros_out) return FBQ_ERR_NULL;
    if (d->r > 0 && (!At || !Bt)) return FBQ_ERR_NULL;
    if (misaligned(W) || misaligned(qweight_out) || misaligned(scales_out) || misaligned(zeros_out)) return FBQ_ERR_ALIGN;
    if (d->r > 0 && (misaligned(At) || misaligned(Bt))) return FBQ_ERR_ALIGN;
    return hip_status(launch_quantize(*d, (const uint16_t *)W, (const uint16_t *)At, (const uint16_t *)Bt,
                                      (uint32_t *)qweight_out, (uint16_t *)scales_out, (uint16_t *)zeros_out,
                                      (hipStream_t)stream));
}

namespace fbq {
static std::atomic<int> g_spin_limit{kDefaultSpinLimit};
int spin_limit() { return g_spin_limit.load(std::memory_order_relaxed); }
}  // namespace fbq

extern "C" int fbq_test_set_spin_limit(int polls)
{
    const int clamped = polls < 0 ? -1 : std::min(polls, kDefaultSpinLimit);
    return g_spin_limit.exchange(clamped, std::memory_order_relaxed);
}

extern "C" fbq_status fbq_measure_read_stream(const void *buf, size_t bytes, fbq_stream stream)
{
    if (!buf) return FBQ_ERR_NULL;
    if (bytes < 16) return FBQ_ERR_SHAPE;
    if (misaligned(buf)) return FBQ_ERR_ALIGN;
    return hip_status(launch_read_stream(buf, bytes, (hipStream_t)stream));
}

extern "C" size_t fbq_train_workspace_bytes(const fbq_desc *d, int T)
{
    if (fbq_check_desc(d) != FBQ_OK || d->r < 1 || T < 1) return 0;
    return train_workspace_bytes(d->N, d->K, d->r, T);
}

extern "C" fbq_status fbq_gram(const fbq_desc *d, int T, const void *X, float h_scale, void *H16_out, void *workspace,
                               size_t workspace_bytes, fbq_stream stream)
{
    fbq_status st = fbq_check_desc(d);
    if (st != FBQ_OK) return st;
    if (T < 1 || T > (1 << 20) || !(h_scale > 0.0f)) return FBQ_ERR_SHAPE;
    if (!X || !H16_out || !workspace) return FBQ_ERR_NULL;
    if (misaligned(X) || misaligned(H16_out) || misaligned(workspace)) return FBQ_ERR_ALIGN;
    if (workspace_bytes < train_workspace_bytes(d->N, d->K, d->r > 0 ? d->r : 8, T)) return FBQ_ERR_WORKSPACE;
    return hip_status(launch_gram(d->K, T, (const uint16_t *)X, h_scale, (uint16_t *)H16_out, workspace, (hipStream_t)stream));
}

extern "C" fbq_status fbq_train_step(const fbq_desc *d, const void *W, const void *H16, float h_scale, float *At32, float *Bt32,
                                     float lr, void *qweight_out, void *scales_out, void *zeros_out, void *At16_out,
                                     void *Bt16_out, float *grad_At, float *grad_Bt, float *loss, void *workspace,
                                     size_t workspace_bytes, fbq_stream stream)
{
    fbq_status st = fbq_check_desc(d);
    if (st != FBQ_OK) return st;
    if (d->r < 1 || !(h_scale > 0.0f) || !(lr >= 0.0f)) return FBQ_ERR_SHAPE;
    if (!W || !H16 || !At32 || !Bt32 || !qweight_out || !scales_out || !zeros_out || !At16_out || !Bt16_out || !grad_At ||
        !grad_Bt || !workspace)
        return FBQ_ERR_NULL;
    if (misaligned(W) || misaligned(H16) || misaligned(At32) || misaligned(Bt32) || misaligned(qweight_out) ||
        misaligned(scales_out) || misaligned(zeros_out) || misaligned(At16_out) || misaligned(Bt16_out) || misaligned(grad_At) ||
        misaligned(grad_Bt) || misaligned(workspace))
        return FBQ_ERR_ALIGN;
    if (workspace_bytes < train_workspace_bytes(d->N, d->K, d->r, 1)) return FBQ_ERR_WORKSPACE;
    TrainArgs a{};
    a.d = *d;
    a.W = (const uint16_t *)W; a.H16 = (const uint16_t *)H16; a.h_scale = h_scale; a.lr = lr;
    a.At32 = At32; a.Bt32 = Bt32;
    a.qw = (uint32_t *)qweight_out; a.scales = (uint16_t *)scales_out; a.zeros = (uint16_t *)zeros_out;
    a.At16 = (uint16_t *)At16_out; a.Bt16 = (uint16_t *)Bt16_out;
    a.gAt = grad_At; a.gBt = grad_Bt; a.loss = loss; a.workspace = workspace;
    return hip_status(launch_train_step(a, (hipStream_t)stream));
}
