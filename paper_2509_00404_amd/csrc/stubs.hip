// Entry points not implemented yet: they refuse loudly instead of computing anything.
#include "common.h"
extern "C" int metis_split_quantize(void*, const metis_mat*, const float*, const float*, const float*, int,
                                    metis_split*, float*) { return METIS_UNSUPPORTED; }
extern "C" size_t metis_linear_workspace_bytes(int64_t, int64_t, int64_t, int) { return 0; }
extern "C" int metis_fp4_linear_fwd(void*, const metis_split*, const metis_split*, metis_mat*, void*, size_t) { return METIS_UNSUPPORTED; }
extern "C" int metis_fp4_linear_dgrad(void*, const metis_split*, const metis_split*, metis_mat*, void*, size_t) { return METIS_UNSUPPORTED; }
extern "C" int metis_fp4_linear_wgrad(void*, const metis_split*, const metis_split*, metis_mat*, void*, size_t) { return METIS_UNSUPPORTED; }
