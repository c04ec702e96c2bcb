// C = A V0 over all rows (see broadcast.hip).  The contraction is cut in broadcast_splits(M, N)
// ranges; range y writes its partial product to Cpart + y*M*k (plain stores, every entry written);
// C is the sum of the parts.  *amax_bits (optional) must be zero on entry.
#pragma once
#include "common.h"
int broadcast_splits(int64_t M, int64_t N);
int launch_broadcast(hipStream_t s, const bf16_t* A, int64_t lda, int64_t M, int64_t N, const bf16_t* V0hi,
                     const bf16_t* V0lo, int k, float* Cpart, uint32_t* amax_bits);
