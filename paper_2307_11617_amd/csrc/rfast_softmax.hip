// Softmax-regression gradient (bf16 MFMA) — placeholder until the kernels land.
#include "rfast_internal.h"
hipError_t rfast_softmax_gradient(rfast_ctx*, const int32_t*, bool) { return hipErrorNotSupported; }
size_t rfast_softmax_scratch_bytes(int32_t, const rfast_problem*) { return 0; }
