// Gradients of the weight's low-rank factors (Sec. 3.2, backward pass: the formulas after Eq. 3).
// Layout of this build: W[N,K] = U S V^T + W_R, U [N,k], V [K,k]; dW[N,K] = Gbar^T Xbar is the output
// of metis_fp4_linear_wgrad.  With the quantized factors Ubar, Vbar and the unquantized S:
//     dL/dU = dW Vbar S [N,k],   dL/dS = Ubar^T dW Vbar [k,k],   dL/dV = dW^T Ubar S [K,k]
// (the paper's four-term sums with Xbar^T (P T Q^T + D_R) collected into dW).  Three skinny products of the
// dense dW with the dequantized factors on the fp64 matrix cores, contraction split over workgroups.
#include "common.h"
#include "dgemm.h"
#include <algorithm>
#include "dgemm_skinny.h"
#include "../../include/metis.h"

namespace {

// out[j][c] = value of the FP4 factor entry (j, c), times scale[j] when given
__global__ void k_dequant_factor(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales, int k, int64_t cols,
                                 float g, const float* __restrict__ rowscale, float* __restrict__ out) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)k * cols) return;
    const int64_t j = t / cols, c = t - j * cols;
    const uint32_t byte = codes[j * (cols / 2) + c / 2];
    const uint32_t nib = (c & 1) ? (byte >> 4) : (byte & 15u);
    const float grid[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};
    float v = grid[nib & 7u] * e4m3_decode(scales[j * (cols / 16) + c / 16]) * g;
    if (nib & 8u) v = -v;
    out[t] = rowscale ? v * rowscale[j] : v;
}

// The same values laid out for the skinny kernels: bf16 [cols][k] (exact: a code times an E4M3 scale times a power
// of two has at most 5 significant bits), or fp64 [cols][k] times rowscale[j]
template <typename TO>
__global__ void k_dequant_factor_t(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales, int k, int64_t cols,
                                   float g, const float* __restrict__ rowscale, TO* __restrict__ out) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)k * cols) return;
    const int64_t c = t / k;
    const int j = (int)(t - c * k);
    const uint32_t byte = codes[j * (cols / 2) + c / 2];
    const uint32_t nib = (c & 1) ? (byte >> 4) : (byte & 15u);
    const float grid[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};
    float v = grid[nib & 7u] * e4m3_decode(scales[j * (cols / 16) + c / 16]) * g;
    if (nib & 8u) v = -v;
    if constexpr (sizeof(TO) == 2) out[t] = f32_to_bf16_rne(v);
    else out[t] = (double)v * (double)rowscale[j];
}

// out[c][j] = (float) in[j][c]
__global__ void k_f64_to_f32_t(const double* __restrict__ in, int k, int64_t cols, float* __restrict__ out) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)k * cols) return;
    const int64_t c = t / k;
    const int j = (int)(t - c * k);
    out[t] = (float)in[(int64_t)j * cols + c];
}


// out[r][j] = (float)(in[r][j] * colscale[j])  (colscale optional)
__global__ void k_f64_to_f32_cols(const double* __restrict__ in, int64_t rows, int k, const float* __restrict__ colscale,
                                  float* __restrict__ out) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= rows * k) return;
    const int j = (int)(t % k);
    out[t] = (float)(colscale ? in[t] * (double)colscale[j] : in[t]);
}

int splits_for(int64_t Kc, int64_t tiles) {
    int64_t s = 1024 / (tiles > 1024 ? 1024 : tiles), maxs = Kc / 64;
    if (s > maxs) s = maxs;
    return (int)(s < 1 ? 1 : s);
}

struct FgLayout {
    size_t off_t, off_dv, off_ds, off_vd, off_ud, off_uds, off_vbf, off_h64, off_parts, total;
};

FgLayout fg_layout(int64_t N, int64_t K, int k) {
    FgLayout L;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    L.off_t = take((size_t)N * k * 8);
    L.off_dv = take((size_t)K * k * 8);
    L.off_ds = take((size_t)k * k * 8);
    L.off_vd = take((size_t)k * K * 4);
    L.off_ud = take((size_t)k * N * 4);
    L.off_uds = take((size_t)k * N * 4);
    L.off_vbf = take((size_t)K * k * 2);
    L.off_h64 = take((size_t)N * k * 8);
    {
        // partial products of whichever split contraction is running (fast and generic kernels), added in a fixed order
        const int64_t tk = ceil_div64(k, 32);
        const size_t tp = std::max(sketch_parts(N, K), dgemm_parts<EPI_PART_F64>(N, k, K, splits_for(K, ceil_div64(N, 32) * tk)));
        const size_t vp = std::max(project_parts(N, K), dgemm_parts<EPI_PART_F64>(K, k, N, splits_for(N, ceil_div64(K, 32) * tk)));
        const size_t sp = dgemm_parts<EPI_PART_F64>(k, k, N, splits_for(N, tk * tk));
        size_t need = std::max(tp * (size_t)N * k, vp * (size_t)K * k);
        need = std::max(need, sp * (size_t)k * k);
        L.off_parts = take(need * 8);
    }
    L.total = o;
    return L;
}

DOperand opnd(const void* p, int64_t s_outer, int64_t s_k) {
    DOperand o;
    o.p = p; o.s_outer = s_outer; o.s_k = s_k; o.map_outer = nullptr; o.map_k = nullptr; o.nparts = 1; o.part_stride = 0;
    return o;
}

DEpilogue epi64(double* c, int64_t ldc) {
    DEpilogue e;
    e.c = c; e.ldc = ldc; e.hi_t = nullptr; e.lo_t = nullptr; e.ld_t = 0; e.skip = nullptr; e.part_stride = 0;
    return e;
}

DEpilogue epi_part(double* parts, int64_t M, int64_t N) {
    DEpilogue e = epi64(parts, N);
    e.part_stride = M * N;
    return e;
}

bool fp4_ok(const metis_fp4& f, int64_t rows, int64_t cols) {
    return f.codes && f.scales && f.rows == rows && f.cols == cols && cols % 16 == 0 && f.tscale > 0.0f;
}

template <typename TW>
int run(hipStream_t s, const TW* dW, int64_t ld, int64_t N, int64_t K, int k, const metis_split* W, float* dU, float* dS,
        float* dV, char* ws, const FgLayout& L) {
    double* T = (double*)(ws + L.off_t);
    double* dV64 = (double*)(ws + L.off_dv);
    double* dS64 = (double*)(ws + L.off_ds);
    float* Vd = (float*)(ws + L.off_vd);
    float* Ud = (float*)(ws + L.off_ud);
    float* UdS = (float*)(ws + L.off_uds);
    double* parts = (double*)(ws + L.off_parts);
    SumList sums;
    hipLaunchKernelGGL(k_dequant_factor, dim3((unsigned)ceil_div64((int64_t)k * K, 256)), dim3(256), 0, s, W->Vt.codes,
                       W->Vt.scales, k, K, W->Vt.tscale, (const float*)nullptr, Vd);
    hipLaunchKernelGGL(k_dequant_factor, dim3((unsigned)ceil_div64((int64_t)k * N, 256)), dim3(256), 0, s, W->Ut.codes,
                       W->Ut.scales, k, N, W->Ut.tscale, (const float*)nullptr, Ud);
    hipLaunchKernelGGL(k_dequant_factor, dim3((unsigned)ceil_div64((int64_t)k * N, 256)), dim3(256), 0, s, W->Ut.codes,
                       W->Ut.scales, k, N, W->Ut.tscale, W->S, UdS);
    METIS_LAUNCH_CHECK();
    const int64_t tk = ceil_div64(k, 32);
    // A bf16 dW of aligned rows takes the decomposition's skinny kernels (same shapes as its sketch and projection)
    bool fast = false;
    if constexpr (sizeof(TW) == 2) fast = skinny_ok((const bf16_t*)dW, ld, K, k) && N % 8 == 0;
    if (fast) {
        bf16_t* Vbf = (bf16_t*)(ws + L.off_vbf);
        double* H64 = (double*)(ws + L.off_h64);
        hipLaunchKernelGGL(k_dequant_factor_t<bf16_t>, dim3((unsigned)ceil_div64((int64_t)k * K, 256)), dim3(256), 0, s,
                           W->Vt.codes, W->Vt.scales, k, K, W->Vt.tscale, (const float*)nullptr, Vbf);
        hipLaunchKernelGGL(k_dequant_factor_t<double>, dim3((unsigned)ceil_div64((int64_t)k * N, 256)), dim3(256), 0, s,
                           W->Ut.codes, W->Ut.scales, k, N, W->Ut.tscale, W->S, H64);
        METIS_LAUNCH_CHECK();
        int st;
        // T = dW Vbar                  [N,k], contraction over K
        if ((st = launch_sketch(s, (const bf16_t*)dW, ld, nullptr, N, K, Vbf, k, parts)) != METIS_OK) return st;
        sums.add(parts, sketch_parts(N, K), N * (int64_t)k, N * (int64_t)k, T);
        sums.launch(s);
        // dV^T = (Ubar S)^T dW         [k,K], contraction over N
        if ((st = launch_project(s, H64, nullptr, nullptr, k, (const bf16_t*)dW, ld, nullptr, N, K, parts)) != METIS_OK)
            return st;
        sums.add(parts, project_parts(N, K), K * (int64_t)k, K * (int64_t)k, dV64);
        sums.launch(s);
    } else {
        // T = dW Vbar                  [N,k], contraction over K
        int want = splits_for(K, ceil_div64(N, 32) * tk);
        launch_dgemm<TW, float, EPI_PART_F64>(s, opnd(dW, ld, 1), opnd(Vd, K, 1), N, k, K, want, epi_part(parts, N, k));
        sums.add(parts, dgemm_parts<EPI_PART_F64>(N, k, K, want), N * (int64_t)k, N * (int64_t)k, T);
        sums.launch(s);
        // dV = dW^T (Ubar S)           [K,k], contraction over N
        want = splits_for(N, ceil_div64(K, 32) * tk);
        launch_dgemm<TW, float, EPI_PART_F64>(s, opnd(dW, 1, ld), opnd(UdS, N, 1), K, k, N, want, epi_part(parts, K, k));
        sums.add(parts, dgemm_parts<EPI_PART_F64>(K, k, N, want), K * (int64_t)k, K * (int64_t)k, dV64);
        sums.launch(s);
    }
    METIS_LAUNCH_CHECK();
    // dS = Ubar^T T                    [k,k], contraction over N
    {
        const int want = splits_for(N, tk * tk);
        launch_dgemm<float, double, EPI_PART_F64>(s, opnd(Ud, N, 1), opnd(T, 1, k), k, k, N, want, epi_part(parts, k, k));
        sums.add(parts, dgemm_parts<EPI_PART_F64>(k, k, N, want), (int64_t)k * k, (int64_t)k * k, dS64);
        sums.launch(s);
    }
    METIS_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_f64_to_f32_cols, dim3((unsigned)ceil_div64(N * k, 256)), dim3(256), 0, s, T, N, k, W->S, dU);
    if (fast)
        hipLaunchKernelGGL(k_f64_to_f32_t, dim3((unsigned)ceil_div64(K * k, 256)), dim3(256), 0, s, dV64, k, K, dV);
    else
        hipLaunchKernelGGL(k_f64_to_f32_cols, dim3((unsigned)ceil_div64(K * k, 256)), dim3(256), 0, s, dV64, K, k,
                           (const float*)nullptr, dV);
    hipLaunchKernelGGL(k_f64_to_f32_cols, dim3((unsigned)ceil_div64((int64_t)k * k, 256)), dim3(256), 0, s, dS64,
                       (int64_t)k, k, (const float*)nullptr, dS);
    METIS_LAUNCH_CHECK();
    return METIS_OK;
}

}  // namespace

extern "C" size_t metis_factor_grads_workspace_bytes(int64_t N, int64_t K, int k) {
    if (N < 1 || K < 1 || k < 1) return 0;
    return fg_layout(N, K, k).total;
}

extern "C" int metis_fp4_factor_grads(void* stream, const metis_mat* dW, const metis_split* W, float* dU, float* dS,
                                      float* dV, void* workspace, size_t workspace_bytes) {
    if (!dW || !dW->ptr || !W || !dU || !dS || !dV || !workspace) return METIS_INVALID_ARG;
    if (dW->dtype != METIS_F32 && dW->dtype != METIS_BF16) return METIS_INVALID_ARG;
    const int64_t N = dW->rows, K = dW->cols;
    const int k = W->k;
    if (N < 1 || K < 1 || dW->ld < K) return METIS_BAD_SHAPE;
    if (k < 1 || k > 128 || !W->S) return METIS_INVALID_ARG;
    if (!fp4_ok(W->Ut, k, N) || !fp4_ok(W->Vt, k, K)) return METIS_BAD_SHAPE;
    const FgLayout L = fg_layout(N, K, k);
    if (workspace_bytes < L.total) return METIS_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(workspace) % 16) return METIS_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    if (dW->dtype == METIS_F32)
        return run<float>(s, (const float*)dW->ptr, dW->ld, N, K, k, W, dU, dS, dV, (char*)workspace, L);
    return run<bf16_t>(s, (const bf16_t*)dW->ptr, dW->ld, N, K, k, W, dU, dS, dV, (char*)workspace, L);
}
