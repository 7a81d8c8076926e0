// temporary: MFMA kernels not built yet
#include "cca_internal.h"
namespace cca {
bool prologue_fused_supported(const Dims &) { return false; }
hipError_t prologue_fused_bf16(const Dims &, const cca_weights &, const void *, void *, void *, void *, hipStream_t) { return hipErrorNotSupported; }
}
