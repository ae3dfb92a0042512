// Internal declarations shared by the library's own translation units (not part of the ABI).
#ifndef FBQ_INTERNAL_H
#define FBQ_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "fbq.h"

namespace fbq {

constexpr int kGroup = 128;          // codes per (scale, zero) pair
constexpr int kLaneCodes = 32;       // codes one lane takes from one wave-wide load
constexpr int kChunk = 64 * kLaneCodes;   // codes one wave-wide load covers (2048)
constexpr int kMaxRank = 256;
constexpr int kMaxK = 16 * kChunk;      // 32768: the decode kernel keeps a wave's activations in registers
constexpr int kDecodeMaxM = 16;
constexpr int kChunkedMaxM = 64;     // up to here the few-token kernel, 16 tokens at a time, can beat the prefill GEMM
constexpr int kPerTokenMaxM = 2;     // up to here the GEMV streams the weights once per token; above, the matrix-core tile wins
constexpr int kMaxTSlices = 4;       // K slices of the decode down-projection: kMaxK / (4 passes * 2048)
constexpr int kMaxGroup = 8;         // layers one grouped decode launch can serve
constexpr int kMaxSmallGroup = 4;    // ... for 4..16 tokens

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// How often a consumer polls for the down-projection's words before it computes them itself.  The value
// in force is process-wide and only the test hook fbq_test_set_spin_limit changes it: a negative value
// makes every consumer take the fall-back path at once (every kernel still runs to its end), so the
// path that a healthy run never takes can be checked against the oracle.
constexpr int kDefaultSpinLimit = 1 << 15;   // polls of about 0.3 us each
int spin_limit();

// Words per packed row.
inline size_t row_words(int K, int bits) { return (size_t)K * bits / 32; }

struct LinearArgs {
    const uint32_t *qw;
    const uint16_t *scales;
    const uint16_t *zeros;
    const uint16_t *At;
    const uint16_t *Bt;
    const uint16_t *x;
    uint16_t *y;
    void *workspace;  // see decode_workspace_bytes / small_m_workspace_bytes / prefill_workspace_bytes
    int M, N, K, r, bits;
};

// Launchers (validated arguments only).  Each returns the hipError_t of its launches.
hipError_t launch_gemv_decode(const LinearArgs *layers, int n_layers, hipStream_t stream);
bool decode_group_compatible(const LinearArgs &a, const LinearArgs &b);
hipError_t launch_gemv_small_m(const LinearArgs *layers, int n_layers, hipStream_t stream);
bool small_m_group_compatible(const LinearArgs &a, const LinearArgs &b);
hipError_t launch_prepass_prefill(const LinearArgs &a, hipStream_t stream);
hipError_t launch_gemm_prefill(const LinearArgs &a, hipStream_t stream);
hipError_t launch_unpack(const fbq_desc &d, const uint32_t *qw, uint8_t *codes, hipStream_t stream);
hipError_t launch_reconstruct(const fbq_desc &d, const uint32_t *qw, const uint16_t *scales, const uint16_t *zeros,
                              const uint16_t *At, const uint16_t *Bt, float *W_hat, hipStream_t stream);
// D16 / Dt16 (optional): Delta_F times `gain` as fp16, [N][K] and transposed [K][ldt] (ldt a multiple of 64, >= N).
hipError_t launch_quantize(const fbq_desc &d, const uint16_t *W, const uint16_t *At, const uint16_t *Bt, uint32_t *qw,
                           uint16_t *scales, uint16_t *zeros, hipStream_t stream, uint16_t *D16 = nullptr,
                           uint16_t *Dt16 = nullptr, int ldt = 0, float gain = 0.0f);

hipError_t launch_read_stream(const void *buf, size_t bytes, hipStream_t stream);
// the sub-branch as two launches of its own on top of a y the main path has written (t: [M][r] fp16 scratch)
hipError_t launch_unfused_branch(const LinearArgs &a, uint16_t *t, hipStream_t stream);

// Arguments of one reconstruction iteration (validated): see fbq_train_step.
struct TrainArgs {
    fbq_desc d;
    const uint16_t *W;
    const uint16_t *H16;
    float h_scale, lr;
    float *At32, *Bt32;
    uint32_t *qw;
    uint16_t *scales, *zeros, *At16, *Bt16;
    float *gAt, *gBt, *loss;
    void *workspace;
};
hipError_t launch_gram(int K, int T, const uint16_t *X, float h_scale, uint16_t *H16, void *workspace, hipStream_t stream);
hipError_t launch_train_step(const TrainArgs &a, hipStream_t stream);
size_t train_workspace_bytes(int N, int K, int r, int T);

// Shared by the entry points (fbq_api.cpp, fbq_static.hip): argument validation that fills the launch
// record without launching, the dispatch on the token count, and the mapping of a HIP error to a status.
fbq_status check_layer(const fbq_desc *d, int M, const void *x, const void *qweight, const void *scales, const void *zeros,
                       const void *At, const void *Bt, void *y, void *workspace, size_t workspace_bytes, LinearArgs *a);
hipError_t launch_one(const LinearArgs &a, hipStream_t s);
fbq_status hip_status(hipError_t e);

// Largest hand-over scratch any call of up to kDecodeMaxM tokens needs (r = kMaxRank): 16 K slices and their
// sums, 16 token rows each, one 8-byte word per value.
constexpr size_t kStaticScratchBytes = (size_t)(16 + 1) * 16 * kMaxRank * 8;

size_t decode_workspace_bytes(int M, int K, int r);
size_t small_m_workspace_bytes(int K, int r);
size_t prefill_workspace_bytes(int M, int N, int K, int r);

}  // namespace fbq

#endif
