// Matrix-core scoring path (bf16 inputs, head_dim 128) -- placeholder until the kernels land.
#include "internal.h"
namespace obc {
void mfma_plan(int, int, int, int, int, int, int, ScoreWorkspace *ws, size_t *) { ws->use_mfma = 0; }
hipError_t launch_score_mfma(const ScoreArgs &, const ScoreWorkspace &, char *, hipStream_t) { return hipErrorNotSupported; }
}  // namespace obc
