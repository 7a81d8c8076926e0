// temporary: MFMA kernels not built yet
#include "cca_internal.h"
namespace cca {
bool attention_mfma_supported(const Dims &) { return false; }
hipError_t attention_mfma_bf16(const Dims &, const void *, const void *, const void *, void *, float *, hipStream_t) { return hipErrorNotSupported; }
bool prologue_fused_supported(const Dims &) { return false; }
hipError_t prologue_fused_bf16(const Dims &, const cca_weights &, const void *, void *, void *, void *, hipStream_t) { return hipErrorNotSupported; }
}
