// ec_prefill_score, matrix-core path for bf16 inputs (placeholder: forwards to the vector-ALU path).
#include "ec_common.h"

namespace ec {
int score_simt_dispatch(const void* q, const void* k, const void* v, void* out, float* lse,
                        float* head_imp, int B, int H, int T, int D, int dt, float scale,
                        hipStream_t stream);

int score_mfma_dispatch(const void* q, const void* k, const void* v, void* out, float* lse,
                        float* head_imp, int B, int H, int T, int D, int dt, float scale,
                        hipStream_t stream)
{
    return score_simt_dispatch(q, k, v, out, lse, head_imp, B, H, T, D, dt, scale, stream);
}
}  // namespace ec
