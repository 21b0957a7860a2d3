// Backward of gist-masked attention, bf16 path (placeholder wiring: routes to the
// plain-ALU kernels until the MFMA kernels land).
#include "common.h"

namespace unigist {

size_t bwd_mfma_workspace(const AttnShape& s) {
    return (((size_t)s.B * s.Hq * s.L * sizeof(float)) + 255) & ~(size_t)255;
}

hipError_t launch_bwd_mfma(const void* q, const void* k, const void* v, const void* out, const float* lse,
                           const void* dout, void* dq, void* dk, void* dv, void* ws, const AttnShape& s,
                           hipStream_t st) {
    return launch_bwd_simple(q, k, v, out, lse, dout, dq, dk, dv, (float*)ws, s, UNIGIST_BF16, st);
}

}  // namespace unigist
