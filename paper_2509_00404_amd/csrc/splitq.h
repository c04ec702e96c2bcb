// Pieces of the split + quantize step (splitq.hip) that the fused decomposition + split path also uses.
#pragma once
#include "common.h"

int padded_rank(int k);          // rank rounded up to what the residual kernel is built for: 16, 32, 64 or 128

// shape and pointer checks of a split output for A [M, N] at rank k (METIS_OK or the status to return)
int check_split_out(int64_t M, int64_t N, int k, const metis_split* out);

// V [N, k] fp32 -> bf16 hi / lo parts [N, kp] (columns k .. kp zero)
int launch_v_factors(hipStream_t s, const float* V, int64_t N, int k, int kp, bf16_t* v_hi, bf16_t* v_lo);

// C = sum of nparts partial products [rows, k] fp32 (part_stride elements apart), written to C_out, and -C as bf16
// hi / lo parts [rows, kp]: the left operand of R = A - C V0^T
int launch_band_factors(hipStream_t s, const float* parts, int nparts, int64_t part_stride, int64_t rows, int k, int kp,
                        float* C_out, bf16_t* us_hi, bf16_t* us_lo);

// R = A + us V^T, quantized along the columns (codes, scales) and optionally along the rows (ct, st: pointers at
// this band's first row inside outputs whose rows are Mt long); A may be a band of rows starting at row row_off
int launch_residual_quant(hipStream_t s, const bf16_t* A, int64_t lda, int64_t M, int64_t N, int64_t Mt, int64_t row_off,
                          const bf16_t* us_hi, const bf16_t* us_lo, const bf16_t* v_hi, const bf16_t* v_lo, int kp, float g,
                          uint8_t* codes, uint8_t* scales, uint8_t* ct, uint8_t* st, float* R_debug, bool sr, uint64_t seed);

// Q(U^T) and Q(V^T) into out->Ut / out->Vt, S copied to out->S
int quantize_factors(hipStream_t s, const float* U, const float* S, const float* V, int64_t M, int64_t N, int k,
                     metis_split* out, bool sr, uint64_t seed);

// quant.hip: the two transposed factor quantizations (and the copy of S when S_src is not null) in one launch.
// U [M, k] and V [N, k] fp32 contiguous; Ut [k, M] and Vt [k, N] with M % 16 == 0 and N % 16 == 0
int launch_quantize_factors_t(hipStream_t s, const float* U, int64_t M, const float* V, int64_t N, int k, const metis_fp4& Ut,
                              const metis_fp4& Vt, bool sr, uint64_t seed_u, uint64_t seed_v, const float* S_src, float* S_dst);
