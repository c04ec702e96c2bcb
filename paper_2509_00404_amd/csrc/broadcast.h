// C = A V0 over all rows (see broadcast.hip).  C must be zero on entry (fp32 atomics
// accumulate the contraction chunks); *amax_bits (optional) must be zero on entry.
#pragma once
#include "common.h"
int launch_broadcast(hipStream_t s, const bf16_t* A, int64_t lda, int64_t M, int64_t N, const bf16_t* V0hi,
                     const bf16_t* V0lo, int k, float* C, uint32_t* amax_bits);
