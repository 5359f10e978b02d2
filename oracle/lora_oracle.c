/*
 * fp64 CPU oracle for the mixed-tenant multi-LoRA linear layer.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the test-suite, the
 * smoke check and the cpu_baseline leg of the benchmark may call it.  It
 * shares no source, header, helper or table with the HIP library, and the HIP
 * library never calls into it.
 *
 * What it computes is the plain definition of the layer (the multi-LoRA
 * shared-base design of the paper's Section 1 principle (1) and Section 4.5,
 * "Multi-LoRA Rollout with Single-Task Training"; LoRA itself is the cited
 * low-rank-update method, Section 2.3):
 *
 *   forward   u_i   = x_i A_t                      (t = adapter of token i)
 *             y_i   = x_i W + s_t * u_i B_t        (t < 0: y_i = x_i W)
 *   backward  v_i   = s_t * dY_i B_t^T
 *             dX_i  = dY_i W^T + v_i A_t^T
 *             dB_t  = s_t * sum_{i in seg(t)} u_i^T dY_i
 *             dA_t  =       sum_{i in seg(t)} x_i^T v_i
 *
 * The backward lines are the derivative of the forward line for a loss whose
 * gradient w.r.t. y is dY; W is frozen (only the per-task LoRA parameters are
 * trained: Section 4.2), so there is no dW.
 *
 * Inputs arrive as the already-rounded bit patterns the GPU sees (bf16 or
 * fp32); they are widened exactly to double and nothing is ever rounded to a
 * narrower type here.  Every token is handled on its own from token_adapter[i]
 * (no segment map is built), and per-adapter sums run over tokens in increasing
 * i, so results are reproducible and row-permutation-equivariant bit for bit.
 *
 * Pins (tests/test_oracle_pins.py): exact rational brute force on tiny inputs,
 * a hand-computed integer example, B=0, single adapter = dense merged weight
 * (numpy matmul), permutation equivariance, finite differences, adjoint
 * identities, output variance of the seeded init, linearity.  The paper prints
 * no worked numeric example of the layer, so parity against paper-printed
 * values is unpinned.
 *
 * Layout flag: 0 = "math"  W[d_in,d_out], A_t[d_in,r], B_t[r,d_out]
 *              1 = "torch" W[d_out,d_in], A_t[r,d_in], B_t[d_out,r]
 * all row-major; x[T,d_in], dY[T,d_out] row-major with leading dimensions.
 * dtype flag: 0 = bf16 bit patterns (uint16), 1 = IEEE fp32.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double widen(const void* p, int dtype, int64_t idx) {
  if (dtype == 0) {
    uint32_t bits = ((uint32_t)((const uint16_t*)p)[idx]) << 16;
    float f;
    memcpy(&f, &bits, 4);
    return (double)f;
  }
  return (double)((const float*)p)[idx];
}

/* W as double in [d_in][d_out] orientation (pure data movement). */
static double* widen_W(const void* W, int dtype, int layout, int64_t ldw, int64_t K, int64_t N) {
  double* Wd = (double*)malloc(sizeof(double) * (size_t)K * (size_t)N);
  if (!Wd) return NULL;
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < K; ++k)
    for (int64_t j = 0; j < N; ++j)
      Wd[k * N + j] = layout == 0 ? widen(W, dtype, k * ldw + j) : widen(W, dtype, j * ldw + k);
  return Wd;
}

/* A_t as double [d_in][r]; B_t as double [r][d_out]. */
static double* widen_A(const void* A, int dtype, int layout, int64_t K, int64_t r) {
  double* Ad = (double*)malloc(sizeof(double) * (size_t)K * (size_t)(r > 0 ? r : 1));
  if (!Ad) return NULL;
  for (int64_t k = 0; k < K; ++k)
    for (int64_t q = 0; q < r; ++q)
      Ad[k * r + q] = layout == 0 ? widen(A, dtype, k * r + q) : widen(A, dtype, q * K + k);
  return Ad;
}
static double* widen_B(const void* B, int dtype, int layout, int64_t r, int64_t N) {
  double* Bd = (double*)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1) * (size_t)N);
  if (!Bd) return NULL;
  for (int64_t q = 0; q < r; ++q)
    for (int64_t j = 0; j < N; ++j)
      Bd[q * N + j] = layout == 0 ? widen(B, dtype, q * N + j) : widen(B, dtype, j * r + q);
  return Bd;
}

static void free_list(double** p, int n) {
  if (!p) return;
  for (int t = 0; t < n; ++t) free(p[t]);
  free(p);
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/*
 * Forward.  rows == NULL: all T tokens, y is [T, d_out]; otherwise y (and u)
 * hold one line per entry of rows[0..n_rows).  u (nullable) is [*, r_max] with
 * u_i = x_i A_t in its first r_t entries and zeros after.
 * Returns 0, or -1 on allocation failure / a token id outside [-1, n_adapters).
 */
int oracle_fwd(int dtype, int layout, int64_t T, int64_t K, int64_t N, int n_adapters,
               const void* x, int64_t ldx, const void* W, int64_t ldw,
               const void* const* A, const void* const* B, const int32_t* ranks,
               const double* scales, const int32_t* token_adapter,
               const int64_t* rows, int64_t n_rows, double* y, double* u, int64_t r_max) {
  int64_t n_out = rows ? n_rows : T;
  for (int64_t i = 0; i < T; ++i)
    if (token_adapter[i] < -1 || token_adapter[i] >= n_adapters) return -1;
  double* Wd = widen_W(W, dtype, layout, ldw, K, N);
  double** Ad = (double**)calloc((size_t)(n_adapters > 0 ? n_adapters : 1), sizeof(double*));
  double** Bd = (double**)calloc((size_t)(n_adapters > 0 ? n_adapters : 1), sizeof(double*));
  if (!Wd || !Ad || !Bd) return -1;
  for (int t = 0; t < n_adapters; ++t) {
    Ad[t] = widen_A(A[t], dtype, layout, K, ranks[t]);
    Bd[t] = widen_B(B[t], dtype, layout, ranks[t], N);
    if (!Ad[t] || !Bd[t]) return -1;
  }
  int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t o = 0; o < n_out; ++o) {
    int64_t i = rows ? rows[o] : o;
    int t = token_adapter[i];
    double* base = (double*)calloc((size_t)N, sizeof(double));
    double* lora = (double*)calloc((size_t)N, sizeof(double));
    double* ui = (double*)calloc((size_t)(r_max > 0 ? r_max : 1), sizeof(double));
    if (!base || !lora || !ui) { fail = 1; free(base); free(lora); free(ui); continue; }
    for (int64_t k = 0; k < K; ++k) {           /* base_j = sum_k x_ik W_kj */
      double xk = widen(x, dtype, i * ldx + k);
      const double* Wk = Wd + k * N;
      for (int64_t j = 0; j < N; ++j) base[j] += xk * Wk[j];
    }
    if (t >= 0) {
      int64_t r = ranks[t];
      for (int64_t k = 0; k < K; ++k) {         /* u_q = sum_k x_ik A_kq */
        double xk = widen(x, dtype, i * ldx + k);
        for (int64_t q = 0; q < r; ++q) ui[q] += xk * Ad[t][k * r + q];
      }
      for (int64_t q = 0; q < r; ++q)           /* lora_j = sum_q u_q B_qj */
        for (int64_t j = 0; j < N; ++j) lora[j] += ui[q] * Bd[t][q * N + j];
      for (int64_t j = 0; j < N; ++j) y[o * N + j] = base[j] + scales[t] * lora[j];
    } else {
      for (int64_t j = 0; j < N; ++j) y[o * N + j] = base[j];
    }
    if (u) for (int64_t q = 0; q < r_max; ++q) u[o * r_max + q] = ui[q];
    free(base); free(lora); free(ui);
  }
  free(Wd); free_list(Ad, n_adapters); free_list(Bd, n_adapters);
  return fail ? -1 : 0;
}

/*
 * Backward.  dX (nullable) is computed for rows[0..n_rows) (all T tokens when
 * rows == NULL), one line of d_in doubles each.  dA/dB (nullable) are host
 * arrays with one double buffer per entry of sel[0..n_sel): dA[s] has the
 * shape of A_{sel[s]} in the math layout [d_in, r]; dB[s] is [r, d_out]
 * (math layout regardless of the input layout flag).  An adapter with no
 * tokens gets zeros.
 */
int oracle_bwd(int dtype, int layout, int64_t T, int64_t K, int64_t N, int n_adapters,
               const void* x, int64_t ldx, const void* W, int64_t ldw,
               const void* const* A, const void* const* B, const int32_t* ranks,
               const double* scales, const int32_t* token_adapter,
               const void* dY, int64_t lddy,
               const int64_t* rows, int64_t n_rows, double* dX,
               const int32_t* sel, int n_sel, double* const* dA, double* const* dB) {
  for (int64_t i = 0; i < T; ++i)
    if (token_adapter[i] < -1 || token_adapter[i] >= n_adapters) return -1;
  double** Ad = (double**)calloc((size_t)(n_adapters > 0 ? n_adapters : 1), sizeof(double*));
  double** Bd = (double**)calloc((size_t)(n_adapters > 0 ? n_adapters : 1), sizeof(double*));
  if (!Ad || !Bd) return -1;
  for (int t = 0; t < n_adapters; ++t) {
    Ad[t] = widen_A(A[t], dtype, layout, K, ranks[t]);
    Bd[t] = widen_B(B[t], dtype, layout, ranks[t], N);
    if (!Ad[t] || !Bd[t]) return -1;
  }
  int fail = 0;
  if (dX) {
    int64_t n_out = rows ? n_rows : T;
    double* Wd = widen_W(W, dtype, layout, ldw, K, N);
    if (!Wd) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t o = 0; o < n_out; ++o) {
      int64_t i = rows ? rows[o] : o;
      int t = token_adapter[i];
      double* out = dX + o * K;
      for (int64_t k = 0; k < K; ++k) {         /* dX_k = sum_j dY_ij W_kj */
        const double* Wk = Wd + k * N;
        double acc = 0.0;
        for (int64_t j = 0; j < N; ++j) acc += widen(dY, dtype, i * lddy + j) * Wk[j];
        out[k] = acc;
      }
      if (t >= 0) {
        int64_t r = ranks[t];
        for (int64_t q = 0; q < r; ++q) {       /* v_q = s sum_j dY_ij B_qj */
          double acc = 0.0;
          for (int64_t j = 0; j < N; ++j) acc += widen(dY, dtype, i * lddy + j) * Bd[t][q * N + j];
          double vq = scales[t] * acc;
          for (int64_t k = 0; k < K; ++k) out[k] += vq * Ad[t][k * r + q];
        }
      }
    }
    free(Wd);
  }
  if (dA && dB) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < n_sel; ++s) {
      int t = sel[s];
      int64_t r = ranks[t];
      double* gA = dA[s];
      double* gB = dB[s];
      memset(gA, 0, sizeof(double) * (size_t)K * (size_t)r);
      memset(gB, 0, sizeof(double) * (size_t)r * (size_t)N);
      double* ui = (double*)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
      double* vi = (double*)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
      if (!ui || !vi) { fail = 1; free(ui); free(vi); continue; }
      for (int64_t i = 0; i < T; ++i) {         /* tokens of seg(t), increasing i */
        if (token_adapter[i] != t) continue;
        for (int64_t q = 0; q < r; ++q) { ui[q] = 0.0; vi[q] = 0.0; }
        for (int64_t k = 0; k < K; ++k) {
          double xk = widen(x, dtype, i * ldx + k);
          for (int64_t q = 0; q < r; ++q) ui[q] += xk * Ad[t][k * r + q];
        }
        for (int64_t q = 0; q < r; ++q) {
          double acc = 0.0;
          for (int64_t j = 0; j < N; ++j) acc += widen(dY, dtype, i * lddy + j) * Bd[t][q * N + j];
          vi[q] = scales[t] * acc;
        }
        for (int64_t q = 0; q < r; ++q)         /* dB_qj += s u_q dY_ij */
          for (int64_t j = 0; j < N; ++j)
            gB[q * N + j] += scales[t] * ui[q] * widen(dY, dtype, i * lddy + j);
        for (int64_t k = 0; k < K; ++k) {       /* dA_kq += x_ik v_q */
          double xk = widen(x, dtype, i * ldx + k);
          for (int64_t q = 0; q < r; ++q) gA[k * r + q] += xk * vi[q];
        }
      }
      free(ui); free(vi);
    }
  }
  free_list(Ad, n_adapters); free_list(Bd, n_adapters);
  return fail ? -1 : 0;
}

/*
 * One optimizer step on the LoRA parameters of the task being trained.
 *
 * The manager keeps, per task, the LoRA parameters theta_t and an optimizer
 * state phi_t, and the training engine maps (theta_t, phi_t) of version v to
 * version v + 1 (Section 4.2; the PolicyUpdate line of Algorithm 1).  The
 * paper does not name the optimizer.  Reading taken here: AdamW, i.e. Adam
 * with decoupled weight decay as published by Loshchilov and Hutter
 * ("Decoupled Weight Decay Regularization", their Algorithm 2, schedule
 * multiplier 1), with phi_t = (first moment m, second moment v, step count):
 *
 *   step  = number of this update, 1 for the first
 *   p    <- p - lr * wd * p
 *   m    <- beta1 * m + (1 - beta1) * g
 *   v    <- beta2 * v + (1 - beta2) * g * g
 *   p    <- p - lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
 *
 * element by element, in place, in fp64.  g is the gradient the backward
 * above produces (dA_t or dB_t).  Returns -1 on a negative size or step < 1.
 */
int oracle_adamw_step(int64_t n, double* p, double* m, double* v, const double* g,
                      double lr, double beta1, double beta2, double eps, double wd, int64_t step) {
  if (n < 0 || step < 1) return -1;
  const double c1 = 1.0 - pow(beta1, (double)step);
  const double c2 = 1.0 - pow(beta2, (double)step);
  for (int64_t i = 0; i < n; ++i) {
    p[i] -= lr * wd * p[i];
    m[i] = beta1 * m[i] + (1.0 - beta1) * g[i];
    v[i] = beta2 * v[i] + (1.0 - beta2) * g[i] * g[i];
    p[i] -= lr * (m[i] / c1) / (sqrt(v[i] / c2) + eps);
  }
  return 0;
}
