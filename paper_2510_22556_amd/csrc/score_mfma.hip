// MFMA window scoring for bf16, D = 128, G*W = 128 (placeholder until the tile kernel lands).
#include "sablock_internal.h"

namespace sablock {

bool score_mfma_supported(const Dims &) { return false; }
size_t score_mfma_ws_bytes(const Dims &) { return 0; }
hipError_t launch_score_mfma(const Dims &, const void *, const void *, const float *, float, float *, float *,
                             void *, hipStream_t)
{
    return hipErrorNotSupported;
}

}  // namespace sablock
