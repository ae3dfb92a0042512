// placeholder until the MFMA path lands
#include "fbq_internal.h"
namespace fbq {
size_t prefill_workspace_bytes(int M, int r) { return (size_t)M * r * 8; }
hipError_t launch_down_proj_prefill(const LinearArgs &, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gemm_prefill(const LinearArgs &, hipStream_t) { return hipErrorNotSupported; }
}
