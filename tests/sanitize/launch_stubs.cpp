// Stand-ins for the library's kernel launchers, so that its host part (fbq_api.cpp) links without any device code
// for the sanitizer run: validation happens before a launch, and the sanitizer run only exercises what comes
// before.  A launcher that is reached reports an error.
#include "fbq_internal.h"

namespace fbq {
hipError_t launch_gemv_decode(const LinearArgs *, int, hipStream_t) { return hipErrorNotSupported; }
bool decode_group_compatible(const LinearArgs &, const LinearArgs &) { return false; }
hipError_t launch_gemv_small_m(const LinearArgs *, int, hipStream_t) { return hipErrorNotSupported; }
bool small_m_group_compatible(const LinearArgs &, const LinearArgs &) { return false; }
hipError_t launch_prepass_prefill(const LinearArgs &, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gemm_prefill(const LinearArgs &, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_unpack(const fbq_desc &, const uint32_t *, uint8_t *, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_reconstruct(const fbq_desc &, const uint32_t *, const uint16_t *, const uint16_t *, const uint16_t *, const uint16_t *,
                              float *, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_quantize(const fbq_desc &, const uint16_t *, const uint16_t *, const uint16_t *, uint32_t *, uint16_t *, uint16_t *,
                           hipStream_t, uint16_t *, uint16_t *, int, float) { return hipErrorNotSupported; }
hipError_t launch_read_stream(const void *, size_t, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_unfused_branch(const LinearArgs &, uint16_t *, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gram(int, int, const uint16_t *, float, uint16_t *, void *, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_train_step(const TrainArgs &, hipStream_t) { return hipErrorNotSupported; }
size_t train_workspace_bytes(int, int, int, int) { return 256; }
size_t decode_workspace_bytes(int M, int, int r) { return (size_t)M * 4 * r * 8; }
size_t small_m_workspace_bytes(int, int r) { return (size_t)17 * 16 * r * 8; }
size_t prefill_workspace_bytes(int M, int, int K, int r) { return (size_t)(M + 256) * K * 2 + (size_t)M * r * 40; }
}  // namespace fbq
