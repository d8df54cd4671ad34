// Fast-transform realisation (placeholder until the kernels land).
#include "fc_common.h"

namespace fc {
bool fft_supported(const fc_kv_desc&, int32_t) { return false; }
FftLayout fft_layout(const fc_kv_desc&, int32_t) { return FftLayout{}; }
hipError_t fft_prepare(const fc_kv_desc&, int32_t, const FftLayout&, void*, hipStream_t) { return hipErrorNotSupported; }
hipError_t fft_score(const void*, const void*, const fc_kv_desc&, int32_t, const FftLayout&, float*, double*, void*, hipStream_t) { return hipErrorNotSupported; }
}  // namespace fc
