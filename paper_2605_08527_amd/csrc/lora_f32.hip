// fp32 path: the same layer in plain fp32 ALU arithmetic for fp32 inputs (no
// matrix cores, no rounding of inputs).  Sized for small problems; it exists
// so that fp32 data is never silently down-cast to bf16.
#include "common.h"

namespace marlaas {

__device__ __forceinline__ float lora_elem(const float* L, int form, int64_t ld_c, int r, int64_t c, int q) {
  // form FORM_NN: L[c * r + q]; FORM_NT: L[q * ld_c + c]
  return form == FORM_NN ? L[c * r + q] : L[(int64_t)q * ld_c + c];
}

__global__ __launch_bounds__(256) void shrink_f32_kernel(const float* X, int64_t ldx, int64_t C,
                                                         const int32_t* perm, const int32_t* seg_off,
                                                         int n, const AdapterEntry* table, int which,
                                                         int lform, float* u, int r_stride, int64_t T_lora) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= T_lora * r_stride) return;
  const int64_t m = idx / r_stride;
  const int q = (int)(idx - m * r_stride);
  const int t = segment_of(seg_off, n, (int)m);
  const AdapterEntry e = table[t];
  float sum = 0.f;
  if (q < e.rank) {
    const float* L = (const float*)(which ? e.B : e.A);
    const int64_t tok = perm ? perm[m] : m;
    const float* xr = X + tok * ldx;
    for (int64_t c = 0; c < C; ++c) sum = fmaf(xr[c], lora_elem(L, lform, C, e.rank, c, q), sum);
    sum *= e.scale;
  }
  u[idx] = sum;
}

// one thread per output element; x index runs along the output columns
template <bool OUT_F32>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* Aop, int64_t lda, const float* Bop,
                                                       int64_t ldb, int form, int64_t T, int64_t Kc,
                                                       int64_t Nout, const int32_t* perm,
                                                       const int32_t* seg_off, int n,
                                                       const AdapterEntry* table, int which,
                                                       const float* U, int r_stride, void* out, int64_t ldo) {
  const int64_t col = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t m = blockIdx.y;
  if (col >= Nout || m >= T) return;
  const int64_t tok = perm ? perm[m] : m;
  const float* ar = Aop + tok * lda;
  float base = 0.f;
  if (form == FORM_NN) for (int64_t k = 0; k < Kc; ++k) base = fmaf(ar[k], Bop[k * ldb + col], base);
  else for (int64_t k = 0; k < Kc; ++k) base = fmaf(ar[k], Bop[col * ldb + k], base);
  float lora = 0.f;
  if (n > 0 && U != nullptr && m < seg_off[n]) {
    const int t = segment_of(seg_off, n, (int)m);
    const AdapterEntry e = table[t];
    const float* L = (const float*)(which ? e.B : e.A);
    // L_t(q, col): FORM_NN stored [r, Nout], FORM_NT stored [Nout, r]
    for (int q = 0; q < e.rank; ++q)
      lora = fmaf(U[m * r_stride + q], form == FORM_NN ? L[(int64_t)q * Nout + col] : L[col * e.rank + q], lora);
  }
  const float y = base + lora;
  if (OUT_F32) ((float*)out)[tok * ldo + col] = y;
  else ((bf16_t*)out)[tok * ldo + col] = float_to_bf16_bits(y);
}

__global__ __launch_bounds__(256) void reduce_f32_kernel(const float* X, int64_t ldx, int64_t C,
                                                         const int32_t* perm, const int32_t* seg_off,
                                                         const AdapterEntry* table, const GradEntry* grads,
                                                         int which, int oform, const float* V,
                                                         int r_stride, int accumulate) {
  const int t = blockIdx.y;
  const AdapterEntry e = table[t];
  const int r = e.rank;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= C * r) return;
  // consecutive threads walk the contiguous index of the output
  int64_t c; int q;
  if (oform == FORM_NN) { c = idx / r; q = (int)(idx - c * r); }
  else { q = (int)(idx / C); c = idx - (int64_t)q * C; }
  float sum = 0.f;
  for (int m = seg_off[t]; m < seg_off[t + 1]; ++m) {
    const int64_t tok = perm ? perm[m] : m;
    sum = fmaf(X[tok * ldx + c], V[(int64_t)m * r_stride + q], sum);
  }
  float* o = (which ? grads[t].dB : grads[t].dA) + idx;
  *o = accumulate ? *o + sum : sum;
}

hipError_t launch_shrink_f32(const float* X, int64_t ldx, int64_t C, const int32_t* perm,
                             const int32_t* seg_off, int n_adapters, const AdapterEntry* table,
                             int which, int lora_form, float* u, int r_stride, int64_t T_lora,
                             hipStream_t stream) {
  if (n_adapters <= 0 || T_lora <= 0) return hipSuccess;
  const int64_t total = T_lora * r_stride;
  hipLaunchKernelGGL(shrink_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                     X, ldx, C, perm, seg_off, n_adapters, table, which, lora_form, u, r_stride, T_lora);
  return hipGetLastError();
}

hipError_t launch_gemm_f32(const float* Aop, int64_t lda, const float* Bop, int64_t ldb, int form,
                           int64_t T, int64_t Kc, int64_t Nout, const int32_t* perm,
                           const int32_t* seg_off, int n_adapters, const AdapterEntry* table,
                           int which, const float* U, int r_stride, void* out, int64_t ldo,
                           int out_is_f32, hipStream_t stream) {
  if (T <= 0 || Nout <= 0) return hipSuccess;
  if (T > 65535) return hipErrorInvalidValue;   // grid.y limit of this simple path
  dim3 grid((unsigned)((Nout + 255) / 256), (unsigned)T);
  if (out_is_f32)
    hipLaunchKernelGGL(gemm_f32_kernel<true>, grid, dim3(256), 0, stream, Aop, lda, Bop, ldb, form, T, Kc,
                       Nout, perm, seg_off, n_adapters, table, which, U, r_stride, out, ldo);
  else
    hipLaunchKernelGGL(gemm_f32_kernel<false>, grid, dim3(256), 0, stream, Aop, lda, Bop, ldb, form, T, Kc,
                       Nout, perm, seg_off, n_adapters, table, which, U, r_stride, out, ldo);
  return hipGetLastError();
}

hipError_t launch_reduce_f32(const float* X, int64_t ldx, int64_t C, const int32_t* perm,
                             const int32_t* seg_off, int n_adapters, const AdapterEntry* table,
                             const GradEntry* grads, int which, int out_form, const float* V,
                             int r_stride, int accumulate, hipStream_t stream) {
  if (n_adapters <= 0) return hipSuccess;
  dim3 grid((unsigned)((C * r_stride + 255) / 256), (unsigned)n_adapters);
  hipLaunchKernelGGL(reduce_f32_kernel, grid, dim3(256), 0, stream, X, ldx, C, perm, seg_off, table,
                     grads, which, out_form, V, r_stride, accumulate);
  return hipGetLastError();
}

}  // namespace marlaas
