#include "internal.h"
namespace specpv {
bool score_mfma_supported(const Shape &, int) { return false; }
hipError_t launch_scores_mfma(const Shape &, const void *, const void *, int, int, float *, hipStream_t)
{ return hipErrorNotSupported; }
}
