/*
 * metis.h -- C ABI of the MI355X-native Metis hot path (spectral split + NVFP4
 * quantization + FP4 GEMMs of one linear layer; Metis, arXiv 2509.00404).
 *
 * Conventions that hold for every entry point
 *   - Every matrix pointer is DEVICE memory owned by the caller, row-major.
 *     Scalars and the structs themselves are HOST memory, read before return.
 *   - `stream` is a hipStream_t passed as void*; all work is enqueued on it and
 *     the call returns without synchronising.  Nothing is allocated or freed.
 *   - Return value: METIS_OK (0) or a negative metis_status.  Argument and shape
 *     errors are detected on the host before anything is enqueued.
 *   - Layout of one linear layer (PyTorch convention): X[L,K] activations,
 *     W[N,K] weight, Y = X W^T [L,N], G = dL/dY [L,N].  The paper's W (Sec. 3.2)
 *     is the transpose of this W.
 */
#ifndef METIS_H
#define METIS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    METIS_OK = 0,
    METIS_INVALID_ARG = -1,      /* null pointer, k < 1, rho outside (0,1], unknown dtype */
    METIS_BAD_SHAPE = -2,        /* quantized axis not a multiple of 16, k+p too large, mismatched operands */
    METIS_WORKSPACE_TOO_SMALL = -3,
    METIS_HIP_ERROR = -4,        /* a launch failed; hipGetLastError() has the reason */
    METIS_UNSUPPORTED = -5,      /* size outside what the kernels are built for (e.g. k+p > 96) */
    METIS_SCRATCH_TOO_SMALL = -6 /* the input needs more than the library's built-in scratch array holds */
} metis_status;

enum { METIS_BF16 = 0, METIS_F32 = 1 };

/* Dense device matrix, row-major, leading dimension `ld` in elements. */
typedef struct {
    void*   ptr;
    int64_t rows, cols, ld;
    int     dtype;               /* METIS_BF16 or METIS_F32 */
} metis_mat;

/*
 * NVFP4-quantized device matrix (Sec. 2.3; value set in App. C.1).
 *   codes  [rows, cols/2]  two E2M1 codes per byte, low nibble = even column,
 *                          nibble = sign<<3 | magnitude code (0..7 -> 0,.5,1,1.5,2,3,4,6)
 *   scales [rows, cols/16] one FP8-E4M3 bit pattern (0x00..0x7E) per block of 16
 *                          consecutive columns
 *   tscale                 per-tensor power-of-two scale g; element value =
 *                          grid[code] * e4m3(scale) * g.  g = 1 is the paper's text verbatim.
 * Blocks always run along `cols` (the contiguous axis).  A matrix that must be
 * blocked along its rows is stored transposed.
 */
typedef struct {
    uint8_t* codes;
    uint8_t* scales;
    float    tscale;
    int64_t  rows, cols;
} metis_fp4;

/*
 * Split-quantized operand A[M,N] ~ U diag(S) V^T + R  (Sec. 3.2: Q_b is applied to
 * U, V and R separately, S stays in high precision).
 *   Ut  Q(U^T) [k,M]   each left singular vector contiguous, blocks along M
 *   Vt  Q(V^T) [k,N]
 *   R   Q(R)   [M,N]   blocks along N (for a GEMM contracting over A's columns)
 *   Rt  Q(R^T) [N,M]   blocks along M (for a GEMM contracting over A's rows); may be
 *                      all-null if the caller does not need that orientation
 *   S   fp32 [k]
 * k = 0: not split; R (and Rt) hold Q(A), Ut/Vt/S are ignored.
 */
typedef struct {
    metis_fp4 Ut, Vt, R, Rt;
    float*    S;
    int       k;
} metis_split;

const char* metis_status_string(int status);
int metis_version(void);

/*
 * Per-tensor scale of a metis_fp4 for data whose largest magnitude is `amax` (host-only helper, no
 * GPU work): the smallest power of two g with 6 * 448 * g >= amax, so that the largest block scale
 * still fits FP8-E4M3.  The paper's text has no such scale (g = 1); this build's reading adds it so
 * that small-magnitude tensors (singular vectors, gradients) do not fall into E4M3's subnormals,
 * and keeps it a power of two so that every quantizer comparison stays exact.  amax <= 0 or not
 * finite returns 1.  Callers typically take amax from a previous step (metis_decompose's amax_out).
 */
float metis_tensor_scale(float amax);

/* ---- random draws of the decomposition (Sec. 3.1) ------------------------------------- */

/* Number of sampled rows l_k = min(M, max(k+p, ceil(rho*M))). Host-only helper. */
int64_t metis_sample_count(int64_t M, int k, int p, double rho);

/*
 * Row sample (Sec. 3.1, sparse random sampling): idx[Ms] (device, uint32), ascending,
 * distinct, one row per stratum [floor(j*M/Ms), floor((j+1)*M/Ms)), offset = word j of
 * Philox4x32-10 stream 1 under `seed`, modulo the stratum length.
 */
int metis_sample_rows(void* stream, uint64_t seed, int64_t M, int64_t Ms, uint32_t* idx);

/*
 * Sequence-granular sample (Sec. 3.1 speaks of sampling sequences, i.e. runs of consecutive token rows): the M
 * rows are M / group sequences of `group` consecutive rows (M % group == 0); whole sequences are drawn exactly as
 * metis_sample_rows draws rows -- one sequence per stratum of sequences, offset = word j of Philox stream 1 modulo
 * the stratum length -- and each contributes its rows in order.  metis_sample_count_sequences gives the number of
 * sampled ROWS: ceil(rho * M / group) sequences, at least ceil((k+p) / group), at most M / group, times group
 * (0 on invalid arguments); group = 1 is metis_sample_count / metis_sample_rows.  idx: device uint32 [Ms].
 * Errors: METIS_INVALID_ARG, METIS_BAD_SHAPE (M or Ms not a multiple of group, Ms > M).
 */
int64_t metis_sample_count_sequences(int64_t M, int k, int p, double rho, int64_t group);
int metis_sample_sequences(void* stream, uint64_t seed, int64_t M, int64_t Ms, int64_t group, uint32_t* idx);

/*
 * Gaussian test matrix (Sec. 3.1, random projection): omega[N,r] (device, bf16 bits as
 * uint16, row-major).  Entry e = n*r+c: Box-Muller on words 2e, 2e+1 of Philox stream 2,
 * u1 = ((w0>>9)+0.5)*2^-23, u2 = (w1>>8)*2^-24, z = sqrt(-2 ln u1) cos(2 pi u2), rounded
 * to bf16 (nearest even).
 */
int metis_gaussian_omega(void* stream, uint64_t seed, int64_t N, int r, uint16_t* omega);

/* ---- decomposition (Sec. 3.1 + the split of Sec. 3.2) ---------------------------------- */

/* Bytes of device workspace metis_decompose needs for an M x N input. */
size_t metis_decompose_workspace_bytes(int64_t M, int64_t N, int k, int p, double rho);

/*
 * A[M,N] (bf16) -> U[M,k], S[k], V[N,k] (all fp32, row-major, device) such that
 * U diag(S) V^T = A V V^T, U^T U = V^T V = I, S descending; span(V) is the top-k right
 * singular subspace of the sampled, sketched matrix:
 *   sample l_k rows -> Z = A_s Omega -> thin QR (CholeskyQR2) Z = H R -> B = H^T A_s ->
 *   top-k right singular vectors V0 of B -> broadcast C = A V0 over ALL rows ->
 *   SVD of C = U S W^T, V = V0 W.
 * No power iteration.  `amax_out` (device fp32[1], optional) receives max|A|.
 * `idx` / `omega` (optional, device): explicit draws replacing the seeded ones (n_idx rows;
 * omega is [N, k+p] bf16); pass NULL/0 to draw from `seed`.
 * `info` (device int32[1], optional): set non-zero if a Cholesky pivot was not positive
 * (rank-deficient sketch); the outputs are then unspecified.
 * The result is a function of the arguments alone: split contractions write partial products that are added in a
 * fixed order (no floating-point atomics), so two calls give the same bits.
 * Errors: INVALID_ARG, BAD_SHAPE (k+p > min(l_k, N)), UNSUPPORTED (k+p > 96, dtype not
 * bf16), WORKSPACE_TOO_SMALL.
 */
int metis_decompose(void* stream, const metis_mat* A, int k, int oversample, double sample_rate,
                    uint64_t seed, float* U, float* S, float* V, float* amax_out,
                    void* workspace, size_t workspace_bytes,
                    const uint32_t* idx, int64_t n_idx, const uint16_t* omega, int32_t* info);

/*
 * Decomposition and split in one call, with one pass over A in HBM (Sec. 3.2's residual A - U S V^T equals
 * A - (A V0) V0^T, V0 being the subspace found on the sampled rows, so it does not have to wait for the
 * singular-value form of the factors).  A is processed in bands of rows small enough to stay in the
 * last-level cache (64 MiB of A): a band's C = A V0 is formed, then the band is read again -- from cache -- for
 * the residual and its quantization into out->R (and out->Rt when its codes pointer is non-null).  Afterwards
 * U, S, V are brought to singular-value form as in metis_decompose and Q(U^T), Q(V^T), S go to out.
 * Arguments as for metis_decompose and metis_split_quantize (out->R.tscale etc. are read as the tensor
 * scales); workspace: metis_decompose_split_workspace_bytes.  U, S, V equal those of metis_decompose; the
 * residual differs from the two-call form only by fp32 rounding (both subtract the same product in different
 * factorizations), so quantization codes may differ where a value sits within rounding of a decision threshold.
 * Errors: those of metis_decompose and metis_split_quantize.
 */
size_t metis_decompose_split_workspace_bytes(int64_t M, int64_t N, int k, int p, double rho);
int metis_decompose_split_quantize(void* stream, const metis_mat* A, int k, int oversample, double sample_rate,
                                   uint64_t seed, float* U, float* S, float* V, float* amax_out, metis_split* out,
                                   float* R_debug, void* workspace, size_t workspace_bytes,
                                   const uint32_t* idx, int64_t n_idx, const uint16_t* omega, int32_t* info);

/*
 * Several decompositions in one call (Sec. 3.2: activations and output gradients are re-decomposed at every
 * step, so one training step decomposes many matrices; they are independent of each other).  Each job has
 * the arguments of metis_decompose; results are what n_jobs separate calls would give.  The stages that
 * run on a single workgroup (Cholesky factorizations, the two eigen-decompositions) are launched once for
 * all jobs of the same k + oversample (resp. k), so they cost one problem's latency instead of n_jobs
 * times it; the stages that stream the matrices are enqueued job after job.  Jobs may differ in every
 * argument; their workspaces and outputs must not overlap.  The array is host memory, read before return.
 * Errors: those of metis_decompose, for the first offending job, before anything is enqueued.
 */
typedef struct {
    const metis_mat* A;
    int      k, oversample;
    double   sample_rate;
    uint64_t seed;
    float*   U;
    float*   S;
    float*   V;
    float*   amax_out;          /* optional */
    void*    workspace;
    size_t   workspace_bytes;
    const uint32_t* idx;        /* optional explicit draws, as for metis_decompose */
    int64_t  n_idx;
    const uint16_t* omega;
    int32_t* info;              /* optional */
    metis_split* split;         /* optional: also split-quantize A as metis_decompose_split_quantize does; the
                                   workspace is then metis_decompose_split_workspace_bytes */
    float*   R_debug;           /* optional, with split: fp32 [M,N] dump of the quantizer's input */
    int64_t  sample_group;      /* 0 or 1: rows are sampled; > 1: whole sequences of that many consecutive rows
                                   (metis_sample_sequences; needs M % sample_group == 0) */
} metis_decompose_job;
int metis_decompose_batch(void* stream, int n_jobs, const metis_decompose_job* jobs);

/* ---- quantization (Sec. 2.3) and split (Sec. 3.2) -------------------------------------- */

/*
 * Plain NVFP4 quantization of A[M,N] (bf16 or fp32): per block of 16 along the columns,
 * scale = smallest E4M3 s with 6*s*g >= block amax (saturating at 448), codes = nearest
 * E2M1 value of e/(s*g), ties to the even code.  `out` (blocks along N, may be NULL) and
 * `out_t` (A^T [N,M], blocks along M, may be NULL) are filled from the same input; their
 * tscale members are read as g.
 */
int metis_quantize(void* stream, const metis_mat* A, metis_fp4* out, metis_fp4* out_t);

/*
 * Stochastically rounded variant (Sec. 4, "FP4 Training": stochastic rounding is the default of
 * every FP4 run).  Block scales as above.  With y = e/(s*g) (fp32 quotient, |y| clipped at 6)
 * between the neighbouring E2M1 magnitudes lo <= |y| <= hi, the element goes to hi with
 * probability (|y| - lo)/(hi - lo), else to lo; values on the grid do not move.  The draw of an
 * element is u = (w >> 8) * 2^-24, w = Philox4x32-10 word under `seed` whose index is the
 * element's row-major position in the output it belongs to (stream 3 for `out`, stream 4 for
 * `out_t`; word w = lane w%4 of the block with counter (w/4 low, w/4 high, stream, 0)); it goes
 * up iff u < t.  Same arguments, layouts and errors as metis_quantize; results are
 * reproducible bit for bit from (A, g, seed).
 */
int metis_quantize_sr(void* stream, const metis_mat* A, uint64_t seed, metis_fp4* out, metis_fp4* out_t);

/*
 * The recipe the paper compares with (Sec. 4.3, "Comparison with Nvidia's Recipe"; Sec. 5, "Hadamard
 * transformations"): a random Hadamard rotation in front of the stochastically rounded quantizer.  The paper
 * gives no definition; this build's reading: every block of 16 consecutive columns is rotated,
 * z = (x * d) H_16 / 4 (H_16 the Sylvester Hadamard matrix in natural order, d_i = -1 iff the top bit of word i of
 * Philox stream 5 under `seed` is set, the same 16 signs for every block), evaluated in fp32 by the radix-2
 * butterfly in natural order (h = 1, 2, 4, 8: pairs (i, i + h) -> (a + b, a - b)), then z is quantized as
 * metis_quantize_sr does (draws: `seed`, stream 3).  H_16 / 4 is orthogonal, so two operands rotated along their
 * common contraction axis with the same seed keep their product.  A: device bf16 [M,N], N % 16 == 0, 16-byte
 * aligned rows; out as for metis_quantize (blocks along N).
 * Errors: METIS_INVALID_ARG, METIS_BAD_SHAPE, METIS_UNSUPPORTED (A not bf16).
 */
int metis_quantize_rht_sr(void* stream, const metis_mat* A, uint64_t seed, metis_fp4* out);

/*
 * Split + quantize: R = A - U diag(S) V^T in fp32 (unquantized factors, Sec. 3.2), then
 * Q(R) into out->R (and Q(R^T) into out->Rt when its codes pointer is non-null), Q(U^T)
 * into out->Ut, Q(V^T) into out->Vt, S copied to out->S.  out->k must equal k.
 * `R_debug` (device fp32 [M,N], optional) receives the exact quantizer input.
 * `workspace`: metis_split_workspace_bytes(M, N, k) bytes of device scratch.
 * Errors: INVALID_ARG, BAD_SHAPE (N % 16, or M % 16 when Rt is requested, mismatched out),
 * UNSUPPORTED (A not bf16, k > 128), WORKSPACE_TOO_SMALL.
 */
size_t metis_split_workspace_bytes(int64_t M, int64_t N, int k);
int metis_split_quantize(void* stream, const metis_mat* A, const float* U, const float* S,
                         const float* V, int k, metis_split* out, float* R_debug,
                         void* workspace, size_t workspace_bytes);

/*
 * metis_split_quantize for callers that cannot allocate device memory or hand over a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments minus
 * the workspace, same kernels, same results bit for bit.  The factor staging (-U S and V as bf16 pairs,
 * metis_split_workspace_bytes(M, N, k) bytes) lives in an array built into the library,
 * METIS_SPLIT_STATIC_SCRATCH_BYTES per GPU, held until the process ends; an input that needs more
 * returns METIS_SCRATCH_TOO_SMALL before anything is enqueued ((M + N) * 4 * k' <= 8 MiB with k' = k
 * rounded up to 16/32/64/128: e.g. 16384 x 14336 at k = 64 fits).  The call itself allocates nothing
 * and never synchronises.  All calls on one GPU share that GPU's array: calls that may overlap on one
 * GPU (different streams, concurrent graph branches) race on it and must be serialised by the caller;
 * calls on one stream are ordered and safe.  Nothing in the array needs clearing between calls (every
 * byte read is rewritten first by the same call).
 */
#define METIS_SPLIT_STATIC_SCRATCH_BYTES (8u << 20)
int metis_split_quantize_static(void* stream, const metis_mat* A, const float* U, const float* S,
                                const float* V, int k, metis_split* out, float* R_debug);

/*
 * Stochastically rounded split (Sec. 4, "FP4 Training"): as metis_split_quantize, with every
 * quantizer replaced by the rule of metis_quantize_sr.  Draws: R from `seed` (stream 3), R^T from
 * `seed` (stream 4), Q(U^T) from `seed + 1` and Q(V^T) from `seed + 2` (stream 4 each), the word
 * index being the element's row-major position in the tensor it is written to.
 */
int metis_split_quantize_sr(void* stream, const metis_mat* A, const float* U, const float* S,
                            const float* V, int k, uint64_t seed, metis_split* out, float* R_debug,
                            void* workspace, size_t workspace_bytes);

/*
 * Split of a weight whose parts are stored, not recomputed (Sec. 3.2: for parameters the low-rank
 * factors and the residual are separate trainable variables, updated independently).  Q_b on
 * U, V and W_R as given; S copied to out->S; no subtraction and no workspace.
 *   W_R  device, bf16 or fp32, [M,N] row stride ld >= N (N % 16 == 0; M % 16 == 0 when out->Rt is wanted)
 *   U [M,k], S [k], V [N,k]  device fp32, contiguous; 1 <= k <= 128, k == out->k
 *   out  as for metis_split_quantize (Rt all-null: that orientation is skipped)
 * The _sr form rounds stochastically with the keys of metis_split_quantize_sr
 * (W_R: seed, U: seed+1, V: seed+2).  Asynchronous on `stream`.
 * Errors: METIS_INVALID_ARG, METIS_BAD_SHAPE (as metis_quantize).
 */
int metis_split_from_parts(void* stream, const metis_mat* W_R, const float* U, const float* S,
                           const float* V, int k, metis_split* out);
int metis_split_from_parts_sr(void* stream, const metis_mat* W_R, const float* U, const float* S,
                              const float* V, int k, uint64_t seed, metis_split* out);

/* ---- FP4 GEMMs on split operands (Eq. 2, Eq. 3, and the W_R gradient after Eq. 3) ------ */

/* Bytes of device workspace the three GEMM calls need (max over them). */
size_t metis_linear_workspace_bytes(int64_t L, int64_t N, int64_t K, int k);

/* Y[L,N]  = Xbar Wbar^T   uses X.R [L,K], W.R [N,K]                       (Eq. 2) */
int metis_fp4_linear_fwd(void* stream, const metis_split* X, const metis_split* W, metis_mat* Y,
                         void* workspace, size_t workspace_bytes);
/* dX[L,K] = Gbar Wbar     uses G.R [L,N], W.Rt [K,N]                      (Eq. 3) */
int metis_fp4_linear_dgrad(void* stream, const metis_split* G, const metis_split* W, metis_mat* dX,
                           void* workspace, size_t workspace_bytes);
/* dW[N,K] = Gbar^T Xbar   uses G.Rt [N,L], X.Rt [K,L]   (dL/dW_R of Sec. 3.2, transposed) */
int metis_fp4_linear_wgrad(void* stream, const metis_split* G, const metis_split* X, metis_mat* dW,
                           void* workspace, size_t workspace_bytes);

/*
 * The same three products in two phases, for callers that want to run the pre-pass of several products side by
 * side (it is a handful of small kernels: the skinny products with the factors and the assembly of the low-rank
 * columns, Sec. 3.3's extra terms) and their main kernels back to back afterwards:
 *   product  METIS_LINEAR_FWD (a = X, b = W), METIS_LINEAR_DGRAD (a = G, b = W), METIS_LINEAR_WGRAD (a = G, b = X)
 *   phase    METIS_LINEAR_PREPARE writes only the workspace; METIS_LINEAR_APPLY reads what PREPARE of the same
 *            product, operands and workspace left there and writes `out`; METIS_LINEAR_ALL = both, which is what
 *            the three calls above do.  `out` may be null for PREPARE.
 * Between PREPARE and APPLY the workspace must not be used by anything else (one workspace per product in flight).
 * Same argument rules, workspace size and errors as the three calls above; METIS_INVALID_ARG for an unknown
 * product or phase.  Asynchronous on `stream`.
 */
enum { METIS_LINEAR_FWD = 0, METIS_LINEAR_DGRAD = 1, METIS_LINEAR_WGRAD = 2 };
enum { METIS_LINEAR_ALL = 0, METIS_LINEAR_PREPARE = 1, METIS_LINEAR_APPLY = 2 };
int metis_fp4_linear_phase(void* stream, int product, int phase, const metis_split* a, const metis_split* b,
                           metis_mat* out, void* workspace, size_t workspace_bytes);

/* ---- gradients of the weight's low-rank factors (Sec. 3.2, backward formulas after Eq. 3) --- */

/* Bytes of device workspace metis_fp4_factor_grads needs for W[N,K] split at rank k. */
size_t metis_factor_grads_workspace_bytes(int64_t N, int64_t K, int k);

/*
 * Gradients with respect to the factors of W[N,K] = U diag(S) V^T + W_R, given the dense
 * dW[N,K] = Gbar^T Xbar that metis_fp4_linear_wgrad wrote (which is also dL/dW_R).  The
 * paper's sums over the split terms of X and of the output gradient collect into dW:
 *     dU[N,k] = dW Vbar diag(S)      dS[k,k] = Ubar^T dW Vbar      dV[K,k] = dW^T Ubar diag(S)
 * Ubar, Vbar are the dequantized W->Ut [k,N], W->Vt [k,K]; S = W->S stays fp32.  (This
 * build's U [N,k] holds the paper's V_k and its V [K,k] the paper's U_k, because W is stored
 * [out, in].)  dS is the full k x k matrix, row-major; a diagonal S takes its diagonal.
 *   dW   device, fp32 or bf16, [N,K] with row stride ld >= K
 *   W    only Ut, Vt, S and k are read; 1 <= k <= 128; N, K multiples of 16
 *   dU, dS, dV   device fp32, caller-owned, contiguous row-major, overwritten
 *   workspace    device, 16-byte aligned, >= metis_factor_grads_workspace_bytes(N, K, k)
 * Products accumulate in fp64 and round once to fp32.  Asynchronous on `stream`.
 * Errors: METIS_INVALID_ARG (null pointer, dtype, k out of range, misaligned workspace),
 * METIS_BAD_SHAPE (factor shapes do not match dW), METIS_WORKSPACE_TOO_SMALL.
 */
int metis_fp4_factor_grads(void* stream, const metis_mat* dW, const metis_split* W,
                           float* dU, float* dS, float* dV,
                           void* workspace, size_t workspace_bytes);

/* ---- MXFP4 variant (the microscaling block format named in Sec. 2.3 beside NVFP4) ------------ */

/*
 * MXFP4-quantized device matrix (OCP Microscaling Formats v1.0):
 *   codes  [rows, cols/2]   two E2M1 codes per byte, same nibble layout as metis_fp4
 *   scales [rows, cols/32]  one E8M0 byte per block of 32 consecutive columns, value 2^(byte - 127)
 * element value = grid[code] * 2^(scale - 127).  Blocks run along `cols`.
 */
typedef struct {
    uint8_t* codes;
    uint8_t* scales;
    int64_t  rows, cols;
} metis_mxfp4;

/*
 * Quantize A (device, bf16 or fp32, [rows, cols], cols % 32 == 0, rows 16-byte aligned) to MXFP4:
 * per block X = 2^(floor(log2 amax) - 2) (the specification's conversion rule), elements round to the
 * nearest E2M1 value of e / X, ties to the even code, magnitudes above 6 saturate; an all-zero block
 * stores scale byte 0.  out's buffers are caller-owned and overwritten.  Asynchronous on `stream`.
 * Errors: METIS_INVALID_ARG, METIS_BAD_SHAPE (shape mismatch or misaligned rows).
 */
int metis_quantize_mx(void* stream, const metis_mat* A, metis_mxfp4* out);

/*
 * C[M,N] = A[M,K] B[N,K]^T on the block-scaled FP4 matrix instruction (the scales are applied by
 * the hardware, fp32 accumulation).  K % 32 == 0 (whole blocks; a K that is not a multiple of 256 takes a
 * somewhat slower variant of the kernel); C device, bf16 or fp32, row stride ld >= N.
 * Errors: METIS_INVALID_ARG, METIS_BAD_SHAPE, METIS_UNSUPPORTED (an operand larger than 4 GiB of codes).
 */
int metis_mxfp4_gemm_nt(void* stream, const metis_mxfp4* A, const metis_mxfp4* B, metis_mat* C);

/* ---- measurement aid ---------------------------------------------------------------------- */

/*
 * Bracket every launch of one hot kernel with caller-owned HIP events (hipEvent_t passed as
 * void*), recorded on the stream the kernel is launched on: launch i uses start[i % n] and
 * stop[i % n].  kernel_id: 0 main FP4 GEMM kernel of the three linear calls (the kernel that
 * writes Y / dX / dW), 1 broadcast C = A V0, 2 fused residual + quantize, 3 plain row
 * quantizer.  n = 0 switches it off.  The arrays (host memory) must stay valid while set.
 * Host-side state, not thread-safe; for benchmarks only.
 */
int metis_profile_events(int kernel_id, void** start, void** stop, int n);

/*
 * Measured ceilings of the GPU the library runs on, for quoting roofline fractions against what the chip
 * sustains as well as against its datasheet peaks.  Asynchronous on `stream`; the caller times them.
 *   metis_ceiling_copy   dst[0..bytes) = src[0..bytes) (device, 16-byte aligned, bytes % 16 == 0): a plain
 *                        streaming copy, 2 * bytes of traffic.
 *   metis_ceiling_read   streams src once; sink: device uint32[2048], normally left untouched.
 *   metis_ceiling_mfma   512 workgroups x 4 waves issue iters x 8 independent 32x32x16 fp16 matrix instructions
 *                        from registers; *flops_out (host, optional) = floating-point operations of the launch;
 *                        sink: device float[512 * 256], normally left untouched.
 *   metis_ceiling_mfma_mix  the FP4 GEMM's instruction mix without its memory system: one workgroup of four
 *                        waves per CU and per `waves_per_simd` (1 or 2), every wave issuing iters x 4 matrix
 *                        instructions (accumulators in the accumulation registers), each followed by
 *                        `valu_per_mfma` (0, 2, 4, 5, 6 or 8) independent packed fp16 multiplies on registers; shows
 *                        what the chip sustains when a wave has to issue that much vector work per matrix
 *                        instruction.  With valu_per_mfma = METIS_MIX_GEMM_EXPANSION (waves_per_simd 1) a wave
 *                        runs `iters` (rounded up to even) steps of the GEMM's own stage loop on registers instead:
 *                        eight fragments expanded from raw words (4 FP4 -> fp16 conversions + 4 packed multiplies
 *                        each), then the 16 matrix instructions of a 128 x 128 wave tile, in the compiler's order --
 *                        the GEMM without LDS traffic, global loads, waits and barrier.  METIS_MIX_GEMM_EXPANSION_FP6
 *                        is that loop with the codes in 6-bit containers, expanded by the 32-wide FP6 converter (two
 *                        instructions per step instead of 32): what a wider container format would buy.
 *                        *flops_out as above; sink as above.
 * Errors: METIS_INVALID_ARG.
 */
#define METIS_MIX_GEMM_EXPANSION (-1)
#define METIS_MIX_GEMM_EXPANSION_FP6 (-2)
int metis_ceiling_mfma_mix(void* stream, int iters, int valu_per_mfma, int waves_per_simd, float* sink, double* flops_out);
int metis_ceiling_copy(void* stream, const void* src, void* dst, size_t bytes);
int metis_ceiling_read(void* stream, const void* src, size_t bytes, uint32_t* sink);
int metis_ceiling_mfma(void* stream, int iters, float* sink, double* flops_out);

#ifdef __cplusplus
}
#endif
#endif /* METIS_H */
