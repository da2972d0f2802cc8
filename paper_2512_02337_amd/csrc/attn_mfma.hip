#include "internal.h"
namespace specpv {
bool attn_ctx_mfma_supported(const Shape &, int) { return false; }
hipError_t launch_attn_ctx_mfma(const Shape &, const int32_t *, const int32_t *, int, Partials, hipStream_t)
{ return hipErrorNotSupported; }
}
