// Element-wise and row-reduction kernels of the NG-SGD step (gfx950, 64-lane wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "state.h"

namespace ngsgd {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}

// Sum over a workgroup (any multiple of 64 threads up to 1024); `scratch` holds >= 16 doubles.
__device__ __forceinline__ double block_sum(double v, double* scratch) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  v = wave_sum(v);
  __syncthreads();
  if (lane == 0) scratch[wave] = v;
  __syncthreads();
  double t = 0.0;
  for (int w = 0; w < nw; ++w) t += scratch[w];
  return t;
}
__device__ __forceinline__ double block_max(double v, double* scratch) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmax(v, __shfl_xor(v, off));
  __syncthreads();
  if (lane == 0) scratch[wave] = v;
  __syncthreads();
  double t = scratch[0];
  for (int w = 1; w < nw; ++w) t = fmax(t, scratch[w]);
  return t;
}

// ---- fills and copies ----------------------------------------------------------------------------
__global__ void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

// out[n][0..D) = x[n][0..D), out[n][D] = 1, out[n][D+1..ldo) = 0   (input with the bias 1 appended, Sec. 4.4)
__global__ void copy_append_ones_kernel(const float* __restrict__ x, int ldx, float* __restrict__ out, int ldo,
                                        int N, int D) {
  const int row = blockIdx.y;
  for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < ldo; c += gridDim.x * blockDim.x)
    out[(size_t)row * ldo + c] = c < D ? x[(size_t)row * ldx + c] : (c == D ? 1.f : 0.f);
}

// dense rows x cols  <->  padded (ld) copies
__global__ void copy2d_kernel(const float* __restrict__ src, int lds_, float* __restrict__ dst, int ldd, int rows,
                              int cols, float scale, const double* scale_dev) {
  const int row = blockIdx.y;
  float s = scale;
  if (scale_dev != nullptr) s *= (float)(*scale_dev);
  for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < cols; c += gridDim.x * blockDim.x)
    dst[(size_t)row * ldd + c] = s * src[(size_t)row * lds_ + c];
}

__global__ void scale_rows_kernel(float* __restrict__ M, int ld, int N, int D, const double* __restrict__ gamma) {
  const int row = blockIdx.y;
  const float s = (float)(*gamma);
  for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < D; c += gridDim.x * blockDim.x)
    M[(size_t)row * ld + c] *= s;
}

// ---- nonlinearities ------------------------------------------------------------------------------
// Y[n][j] = tanh(A[n][j]); Y[n][D] = 1; padding zero.
__global__ void tanh_forward_kernel(const float* __restrict__ A, int lda, float* __restrict__ Y, int ldy, int N,
                                    int D) {
  const int row = blockIdx.y;
  for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < ldy; c += gridDim.x * blockDim.x)
    Y[(size_t)row * ldy + c] = c < D ? tanhf(A[(size_t)row * lda + c]) : (c == D ? 1.f : 0.f);
}

// The derivative w.r.t. a layer's input arrives as n_slabs partial products (split-K slabs of the backward
// GEMM, slab_stride floats apart) that are summed here in a fixed order.
__device__ __forceinline__ float slab_sum(const float* __restrict__ p, int n_slabs, size_t slab_stride) {
  float v = p[0];
  for (int s = 1; s < n_slabs; ++s) v += p[(size_t)s * slab_stride];
  return v;
}

// O[n][j] = dY[n][j] * (1 - Y[n][j]^2)
__global__ void tanh_backward_kernel(const float* __restrict__ dY, int ldd, int n_slabs, size_t slab_stride,
                                     const float* __restrict__ Y, int ldy, float* __restrict__ O, int ldo, int N,
                                     int D) {
  const int row = blockIdx.y;
  for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < D; c += gridDim.x * blockDim.x) {
    const float y = Y[(size_t)row * ldy + c];
    O[(size_t)row * ldo + c] = slab_sum(dY + (size_t)row * ldd + c, n_slabs, slab_stride) * (1.f - y * y);
  }
}

// p-norm (p = 2) over groups of G adjacent columns, one wavefront per row:
//   y_j = sqrt(sum_k a_{Gj+k}^2);  with renorm: y <- y / max(rms(y), floor), sigma[n] = that divisor.
// Writes Y[n][0..groups), Y[n][groups] = 1, padding zero.
constexpr float kRenormFloor = 1.0e-20f;

__global__ __launch_bounds__(256) void pnorm_forward_kernel(const float* __restrict__ A, int lda,
                                                            float* __restrict__ Y, int ldy,
                                                            float* __restrict__ sigma, int N, int groups, int G,
                                                            int renorm) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= N) return;
  const float* a = A + (size_t)row * lda;
  float* y = Y + (size_t)row * ldy;
  float ss = 0.f;
  for (int j = lane; j < groups; j += 64) {
    float s = 0.f;
    for (int k = 0; k < G; ++k) {
      const float v = a[j * G + k];
      s += v * v;
    }
    ss += s;              // sum_j y_j^2
    y[j] = sqrtf(s);
  }
  float inv = 1.f;
  if (renorm) {
    ss = wave_sum(ss);
    const float sg = fmaxf(sqrtf(ss / (float)groups), kRenormFloor);
    inv = 1.f / sg;
    if (lane == 0) sigma[row] = sg;
    for (int j = lane; j < groups; j += 64) y[j] *= inv;   // same lane wrote y[j] above
  }
  for (int c = groups + lane; c < ldy; c += 64) y[c] = c == groups ? 1.f : 0.f;
}

// Backward through (renorm o p-norm), one wavefront per row, in place over the affine outputs:
//   AO[n][Gj+k] <- dy_j * a_{Gj+k} / y_j   (0 where y_j = 0)
// with dy = dYn, y = Yn without renorm; with renorm  y = Yn*sigma, dy = (dYn - Yn * mean_j(dYn_j Yn_j)) / sigma.
__global__ __launch_bounds__(256) void pnorm_backward_kernel(const float* __restrict__ dYn, int ldd, int n_slabs,
                                                             size_t slab_stride,
                                                             const float* __restrict__ Yn, int ldy,
                                                             const float* __restrict__ sigma,
                                                             float* __restrict__ AO, int lda, int N, int groups,
                                                             int G, int renorm) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= N) return;
  const float* dy = dYn + (size_t)row * ldd;
  const float* yn = Yn + (size_t)row * ldy;
  float* ao = AO + (size_t)row * lda;
  float proj = 0.f, sg = 1.f;
  if (renorm) {
    float dot = 0.f;
    for (int j = lane; j < groups; j += 64) dot += slab_sum(dy + j, n_slabs, slab_stride) * yn[j];
    dot = wave_sum(dot);
    sg = sigma[row];
    proj = sg > kRenormFloor ? dot / (float)groups : 0.f;
  }
  const float inv_sg = 1.f / sg;
  for (int j = lane; j < groups; j += 64) {
    const float ynj = yn[j];
    const float d = (slab_sum(dy + j, n_slabs, slab_stride) - ynj * proj) * inv_sg;
    const float yj = ynj * sg;
    const float f = yj > 0.f ? d / yj : 0.f;
    for (int k = 0; k < G; ++k) ao[j * G + k] *= f;
  }
}

// ---- log-softmax, objective and its derivative (Sec. 2) ------------------------------------------
// One workgroup per row, in place: AO[n][c] <- [c == y_n] - softmax(a_n)_c;  rowobj[n] = log p(y_n | x_n).
__global__ __launch_bounds__(256) void softmax_xent_kernel(float* __restrict__ AO, int ld,
                                                           const int32_t* __restrict__ labels, int N, int C,
                                                           double* __restrict__ rowobj) {
  __shared__ double scratch[16];
  const int row = blockIdx.x;
  float* a = AO + (size_t)row * ld;
  float m = -INFINITY;
  for (int c = threadIdx.x; c < C; c += blockDim.x) m = fmaxf(m, a[c]);
  m = (float)block_max((double)m, scratch);
  double s = 0.0;
  for (int c = threadIdx.x; c < C; c += blockDim.x) s += (double)expf(a[c] - m);
  s = block_sum(s, scratch);
  const float lse = m + (float)log(s);
  const int y = labels[row];
  const bool valid = y >= 0 && y < C;        // an out-of-range label yields NaN, never an out-of-bounds access
  __syncthreads();
  if (threadIdx.x == 0) rowobj[row] = valid ? (double)a[y] - ((double)m + log(s)) : (double)NAN;
  __syncthreads();
  for (int c = threadIdx.x; c < C; c += blockDim.x) {
    const float p = expf(a[c] - lse);
    a[c] = (c == y ? 1.f : 0.f) - p;
  }
}

__global__ __launch_bounds__(256) void sum_double_kernel(const double* __restrict__ v, int n,
                                                         double* __restrict__ out) {
  __shared__ double scratch[16];
  double s = 0.0;
  for (int i = threadIdx.x; i < n; i += blockDim.x) s += v[i];
  s = block_sum(s, scratch);
  if (threadIdx.x == 0) *out = s;
}

// ---- preconditioner helpers -----------------------------------------------------------------------
// After Xhat = X - H W: reduce the partial sums, gamma_t = sqrt(tr(X X^T) / tr(Xhat Xhat^T)) (eq. gammat;
// 1 if the denominator is 0), per-row squared norms of the output.  One workgroup per instance.
struct FinishArgs {
  PrecondScalars* st;
  const double* sumsq_part;  // partial sums of squares of X
  int n_sumsq;
  const float* rownorm_part; // [n_col_tiles][N] partial row norms of Xhat
  int n_col_tiles;
  int N;
  double* prow;              // out: p_i (eq. pi), N doubles
  float* gamma_out;          // optional
  float* rownorm2_out;       // optional, gamma^2 p_i
};
struct FinishGroup {
  int count;
  FinishArgs a[kMaxInstances];
};

__global__ __launch_bounds__(256) void finish_apply_kernel(const FinishGroup g) {
  __shared__ double scratch[16];
  const FinishArgs& a = g.a[blockIdx.x];
  double t = 0.0;
  for (int i = threadIdx.x; i < a.n_sumsq; i += blockDim.x) t += a.sumsq_part[i];
  const double tr_M = block_sum(t, scratch);
  double ph = 0.0;
  for (int r = threadIdx.x; r < a.N; r += blockDim.x) {
    double p = 0.0;
    for (int c = 0; c < a.n_col_tiles; ++c) p += (double)a.rownorm_part[(size_t)c * a.N + r];
    a.prow[r] = p;
    ph += p;
  }
  const double tr_Mhat = block_sum(ph, scratch);
  const double gamma = tr_Mhat > 0.0 ? sqrt(tr_M / tr_Mhat) : 1.0;
  if (threadIdx.x == 0) {
    a.st->gamma = gamma;
    a.st->tr_M = tr_M;
    a.st->tr_Mhat = tr_Mhat;
    if (a.gamma_out != nullptr) *a.gamma_out = (float)gamma;
  }
  if (a.rownorm2_out != nullptr)
    for (int r = threadIdx.x; r < a.N; r += blockDim.x) a.rownorm2_out[r] = (float)(gamma * gamma * a.prow[r]);
}

// Rank 0: no factor, the output is the input; only the row norms are produced.  One workgroup per row block.
__global__ __launch_bounds__(256) void rownorm_kernel(const float* __restrict__ M, int ld, int N, int D,
                                                      double* __restrict__ prow, float* __restrict__ rownorm2_out) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= N) return;
  float s = 0.f;
  for (int c = lane; c < D; c += 64) {
    const float v = M[(size_t)row * ld + c];
    s += v * v;
  }
  s = wave_sum(s);
  if (lane == 0) {
    prow[row] = (double)s;
    if (rownorm2_out != nullptr) rownorm2_out[row] = s;
  }
}

// B_t = J_t + (N (1 - eta) / eta) (D_t + rho_t I) W_t, written over J (eq. wt1).  Grid (col blocks, R).
// Must run while st still holds D_t and rho_t, i.e. before the R x R update kernel.
__global__ void make_bt_kernel(float* __restrict__ J, const float* __restrict__ W, int ld, int D,
                               const PrecondScalars* __restrict__ st, int N, double num_samples_history) {
  const int i = blockIdx.y;
  const double eta = 1.0 - exp(-(double)N / num_samples_history);
  const float f = (float)((double)N * (1.0 - eta) / eta * (st->d[i] + st->rho));
  for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < D; c += gridDim.x * blockDim.x)
    J[(size_t)i * ld + c] += f * W[(size_t)i * ld + c];
}

// W = E^{1/2} R from a state given in definitional form (eq. beta2, etii, wt:def).  One workgroup per row.
__global__ __launch_bounds__(256) void set_state_kernel(const double* __restrict__ Rm, const double* __restrict__ d,
                                                        double rho, double alpha, int R, int D,
                                                        float* __restrict__ W, int ld, PrecondScalars* st) {
  const int i = blockIdx.x;
  double sum_d = 0.0;
  for (int k = 0; k < R; ++k) sum_d += d[k];
  const double beta = rho * (1.0 + alpha) + alpha / (double)D * sum_d;
  const double e = 1.0 / (beta / d[i] + 1.0);
  const double s = sqrt(e);
  for (int c = threadIdx.x; c < ld; c += blockDim.x) W[(size_t)i * ld + c] = c < D ? (float)(s * Rm[(size_t)i * D + c]) : 0.f;
  if (threadIdx.x == 0) {
    st->d[i] = d[i];
    st->e[i] = e;
    if (i == 0) {
      st->rho = rho;
      st->beta = beta;
      st->flags = 0;
    }
  }
}

// ---- maximum parameter change per minibatch (App. C.3) ---------------------------------------------
// a = min(1, N * max_change_per_sample / (lr * sum_i ||obar_i|| ||xbar_i||)), one workgroup per layer.
struct MaxChangeArgs {
  const double* prow_o;
  const double* prow_x;
  const double* gamma_o;
  const double* gamma_x;
  double* scale_out;
  int N;
};
struct MaxChangeGroup {
  int count;
  double lr, max_change_per_sample;
  MaxChangeArgs a[kMaxInstances];
};
__global__ __launch_bounds__(256) void max_change_kernel(const MaxChangeGroup g) {
  __shared__ double scratch[16];
  const MaxChangeArgs& a = g.a[blockIdx.x];
  double s = 0.0;
  for (int r = threadIdx.x; r < a.N; r += blockDim.x) s += sqrt(a.prow_o[r] * a.prow_x[r]);
  s = block_sum(s, scratch);
  if (threadIdx.x == 0) {
    double scale = 1.0;
    if (g.max_change_per_sample > 0.0) {
      const double bound = g.lr * (*a.gamma_o) * (*a.gamma_x) * s;
      if (bound > 0.0) scale = fmin(1.0, (double)a.N * g.max_change_per_sample / bound);
    }
    *a.scale_out = scale;
  }
}

// ---- parameter averaging (Sec. 3.1) -------------------------------------------------------------
struct AverageArgs {
  int n;
  size_t count;
  float* params[kMaxReplicas];
};
__global__ void average_kernel(const AverageArgs a) {
  const float inv = 1.f / (float)a.n;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < a.count; i += (size_t)gridDim.x * blockDim.x) {
    float s = 0.f;
    for (int r = 0; r < a.n; ++r) s += a.params[r][i];
    s *= inv;
    for (int r = 0; r < a.n; ++r) a.params[r][i] = s;
  }
}

}  // namespace ngsgd
