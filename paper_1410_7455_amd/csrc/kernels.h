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
__device__ __forceinline__ double wave_max_d(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmax(v, __shfl_xor(v, off));
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

// Clears several buffers in one launch: grid (blocks, count).
struct FillGroup {
  int count;
  uint32_t* ptr[kMaxInstances];
  size_t n[kMaxInstances];
};
__global__ void fill_zero_group_kernel(const FillGroup g) {
  uint32_t* p = g.ptr[blockIdx.y];
  const size_t n = g.n[blockIdx.y];
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

// out[n][0..D) = x[n][0..D), out[n][D] = 1, out[n][D+1..ldo) = 0   (input with the bias 1 appended, Sec. 4.4)
// Also clears *clear (the step's objective accumulator), if given.
__global__ void copy_append_ones_kernel(const float* __restrict__ x, int ldx, float* __restrict__ out, int ldo,
                                        int N, int D, double* __restrict__ clear) {
  const int row = blockIdx.y;
  if (row >= N) return;   // the grid's second dimension is the row count
  if (clear != nullptr && row == 0 && blockIdx.x == 0 && threadIdx.x == 0) *clear = 0.0;
  for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < ldo; c += gridDim.x * blockDim.x)
    out[(size_t)row * ldo + c] = c < D ? x[(size_t)row * ldx + c] : (c == D ? 1.f : 0.f);
}

// dense rows x cols  <->  padded (ld) copies
__global__ void copy2d_kernel(const float* __restrict__ src, int lds_, float* __restrict__ dst, int ldd, int rows,
                              int cols, float scale, const double* scale_dev) {
  const int row = blockIdx.y;
  if (row >= rows) return;   // the grid's second dimension is the row count
  float s = scale;
  if (scale_dev != nullptr) s *= (float)(*scale_dev);
  for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < cols; c += gridDim.x * blockDim.x)
    dst[(size_t)row * ldd + c] = s * src[(size_t)row * lds_ + c];
}

// Rows are 16-byte aligned and ld is a multiple of 4 (checked by the callers): 16 bytes per lane, tail by elements.
__global__ void scale_rows_kernel(float* __restrict__ M, int ld, int N, int D, const double* __restrict__ gamma) {
  const int row = blockIdx.y;
  if (row >= N) return;   // the grid's second dimension is the row count
  const float s = (float)(*gamma);
  float* m = M + (size_t)row * ld;
  const int d4 = D & ~3;
  for (int c = 4 * (blockIdx.x * blockDim.x + threadIdx.x); c < d4; c += 4 * gridDim.x * blockDim.x) {
    float4 v = *reinterpret_cast<float4*>(m + c);
    v.x *= s; v.y *= s; v.z *= s; v.w *= s;
    *reinterpret_cast<float4*>(m + c) = v;
  }
  if (blockIdx.x == 0 && threadIdx.x < D - d4) m[d4 + threadIdx.x] *= s;
}

// ---- nonlinearities ------------------------------------------------------------------------------
// Y[n][j] = tanh(A[n][j]); Y[n][D] = 1; padding zero.
__global__ void tanh_forward_kernel(const float* __restrict__ A, int lda, float* __restrict__ Y, int ldy, int N,
                                    int D) {
  const int row = blockIdx.y;
  if (row >= N) return;   // the grid's second dimension is the row count
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
  if (row >= N) return;   // the grid's second dimension is the row count
  for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < D; c += gridDim.x * blockDim.x) {
    const float y = Y[(size_t)row * ldy + c];
    O[(size_t)row * ldo + c] = slab_sum(dY + (size_t)row * ldd + c, n_slabs, slab_stride) * (1.f - y * y);
  }
}

// Workgroup-wide float sum / max for NT-thread workgroups (NT / 64 wavefronts); `red` holds >= NT / 64 floats.
template <int NT>
__device__ __forceinline__ float block_sum_f(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int w = 1; w < NT / 64; ++w) r += red[w];
  return r;
}
template <int NT>
__device__ __forceinline__ float block_max_f(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int w = 1; w < NT / 64; ++w) r = fmaxf(r, red[w]);
  return r;
}
__device__ __forceinline__ float block256_sum(float v, float* red) { return block_sum_f<256>(v, red); }
__device__ __forceinline__ float block256_max(float v, float* red) { return block_max_f<256>(v, red); }

// p-norm (p = 2) over groups of G adjacent columns, one NT-thread workgroup per row:
//   y_j = sqrt(sum_k a_{Gj+k}^2);  with renorm: y <- y / max(rms(y), floor), sigma[n] = that divisor.
// Writes Y[n][0..groups), Y[n][groups] = 1, padding zero.
constexpr float kRenormFloor = 1.0e-20f;

template <int NT>
__global__ __launch_bounds__(NT) void pnorm_forward_kernel(const float* __restrict__ A, int lda,
                                                            float* __restrict__ Y, int ldy,
                                                            float* __restrict__ sigma, int N, int groups, int G,
                                                            int renorm) {
  __shared__ float red[NT / 64];
  const int row = blockIdx.x;
  if (row >= N) return;   // one workgroup per row (uniform over the workgroup)
  const float* a = A + (size_t)row * lda;
  float* y = Y + (size_t)row * ldy;
  float ss = 0.f;
  // a thread keeps the (few) groups it computes in registers until the row's scale is known
  constexpr int kMaxOwn = 2048 / NT;   // groups per thread: rows of up to 2048 groups stay in registers
  float own[kMaxOwn];
#pragma unroll
  for (int u = 0; u < kMaxOwn; ++u) {
    const int j = threadIdx.x + u * NT;
    float s = 0.f;
    if (j < groups) {
      const float* g = a + (size_t)j * G;
      if ((G & 1) == 0) {
        for (int k = 0; k < G; k += 2) {
          const float2 v = *reinterpret_cast<const float2*>(g + k);
          s += v.x * v.x + v.y * v.y;
        }
      } else {
        for (int k = 0; k < G; ++k) s += g[k] * g[k];
      }
    }
    own[u] = sqrtf(s);
    ss += s;
  }
  for (int j = threadIdx.x + kMaxOwn * NT; j < groups; j += NT) {   // very wide rows: through memory
    float s = 0.f;
    for (int k = 0; k < G; ++k) s += a[(size_t)j * G + k] * a[(size_t)j * G + k];
    y[j] = sqrtf(s);
    ss += s;
  }
  float inv = 1.f;
  if (renorm) {
    ss = block_sum_f<NT>(ss, red);
    const float sg = fmaxf(sqrtf(ss / (float)groups), kRenormFloor);
    inv = 1.f / sg;
    if (threadIdx.x == 0) sigma[row] = sg;
    for (int j = threadIdx.x + kMaxOwn * NT; j < groups; j += NT) y[j] *= inv;   // written by this thread above
  }
#pragma unroll
  for (int u = 0; u < kMaxOwn; ++u) {
    const int j = threadIdx.x + u * NT;
    if (j < groups) y[j] = own[u] * inv;
  }
  for (int c = groups + threadIdx.x; c < ldy; c += NT) y[c] = c == groups ? 1.f : 0.f;
}

// Backward through (renorm o p-norm), one NT-thread workgroup per row, in place over the affine outputs:
//   AO[n][Gj+k] <- dy_j * a_{Gj+k} / y_j   (0 where y_j = 0)
// with dy = dYn, y = Yn without renorm; with renorm  y = Yn*sigma, dy = (dYn - Yn * mean_j(dYn_j Yn_j)) / sigma.
// dYn arrives as n_slabs partial products (see slab_sum).  The per-group factor dy_j / y_j goes through LDS.
constexpr int kPnormMaxGroupsLds = 4096;
constexpr int kPnormPrefetchPairs = 2048;   // float2 per row held in registers across the reductions (4096 outputs)

template <int NT>
__global__ __launch_bounds__(NT) void pnorm_backward_kernel(const float* __restrict__ dYn, int ldd, int n_slabs,
                                                             size_t slab_stride,
                                                             const float* __restrict__ Yn, int ldy,
                                                             const float* __restrict__ sigma,
                                                             float* __restrict__ AO, int lda, int N, int groups,
                                                             int G, int renorm) {
  constexpr int kPnormPrefetch = kPnormPrefetchPairs / NT;
  __shared__ float red[NT / 64];
  __shared__ float s_f[kPnormMaxGroupsLds];   // first dy_j, then the factor dy_j / y_j
  const int row = blockIdx.x;
  if (row >= N) return;   // one workgroup per row (uniform over the workgroup)
  const float* dy = dYn + (size_t)row * ldd;
  const float* yn = Yn + (size_t)row * ldy;
  float* ao = AO + (size_t)row * lda;
  const int D = groups * G;
  // the affine outputs this thread will rescale are requested first: they arrive while the row's factors are made
  const bool vec2 = (G & 1) == 0 && (lda & 1) == 0;
  float2* ao2 = reinterpret_cast<float2*>(ao);
  float2 pre[kPnormPrefetch];
  if (vec2) {
#pragma unroll
    for (int u = 0; u < kPnormPrefetch; ++u) {
      const int c2 = threadIdx.x + u * NT;
      if (c2 < D / 2) pre[u] = ao2[c2];
    }
  }
  float dot = 0.f;
  for (int j = threadIdx.x; j < groups; j += NT) {
    const float d = slab_sum(dy + j, n_slabs, slab_stride);
    s_f[j] = d;
    dot += d * yn[j];
  }
  float proj = 0.f, sg = 1.f;
  if (renorm) {
    dot = block_sum_f<NT>(dot, red);
    sg = sigma[row];
    proj = sg > kRenormFloor ? dot / (float)groups : 0.f;
  }
  const float inv_sg = 1.f / sg;
  for (int j = threadIdx.x; j < groups; j += NT) {   // each thread rewrites the entries it wrote above
    const float ynj = yn[j];
    const float d = (s_f[j] - ynj * proj) * inv_sg;
    const float yj = ynj * sg;
    s_f[j] = yj > 0.f ? d / yj : 0.f;
  }
  __syncthreads();
  if (vec2) {
    const int half_g = G / 2;
#pragma unroll
    for (int u = 0; u < kPnormPrefetch; ++u) {
      const int c2 = threadIdx.x + u * NT;
      if (c2 < D / 2) {
        const float f = s_f[c2 / half_g];
        ao2[c2] = make_float2(pre[u].x * f, pre[u].y * f);
      }
    }
    for (int c2 = threadIdx.x + kPnormPrefetch * NT; c2 < D / 2; c2 += NT) {
      const float f = s_f[c2 / half_g];
      float2 v = ao2[c2];
      v.x *= f;
      v.y *= f;
      ao2[c2] = v;
    }
  } else {
    for (int c = threadIdx.x; c < D; c += NT) ao[c] *= s_f[c / G];
  }
}

// ---- log-softmax, objective and its derivative (Sec. 2) ------------------------------------------
// One NT-thread workgroup per row, in place: AO[n][c] <- [c == y_n] - softmax(a_n)_c;
// rowobj[n] = log p(y_n | x_n), also added to *total.  Rows of up to 4 * kSoftmaxRowVec classes are read once and kept in registers.
constexpr int kSoftmaxRowVec = 2048;   // float4 per row held in registers

template <int NT>
__global__ __launch_bounds__(NT) void softmax_xent_kernel(float* __restrict__ AO, int ld,
                                                           const int32_t* __restrict__ labels, int N, int C,
                                                           double* __restrict__ rowobj, double* __restrict__ total) {
  constexpr int kSoftmaxVec = kSoftmaxRowVec / NT;   // float4 per thread
  __shared__ float red[NT / 64];
  const int row = blockIdx.x;
  if (row >= N) return;   // one workgroup per row (uniform over the workgroup)
  float* a = AO + (size_t)row * ld;
  const int y = labels[row];
  const bool valid = y >= 0 && y < C;        // an out-of-range label yields NaN, never an out-of-bounds access
  if (C <= 4 * kSoftmaxRowVec) {
    float4 v[kSoftmaxVec];
    float m = -INFINITY;
#pragma unroll
    for (int u = 0; u < kSoftmaxVec; ++u) {
      const int c = (threadIdx.x + u * NT) * 4;
      float4 t = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
      if (c + 3 < C) {
        t = *reinterpret_cast<const float4*>(a + c);
      } else if (c < C) {
        t.x = a[c];
        if (c + 1 < C) t.y = a[c + 1];
        if (c + 2 < C) t.z = a[c + 2];
      }
      v[u] = t;
      m = fmaxf(fmaxf(m, fmaxf(t.x, t.y)), fmaxf(t.z, t.w));
    }
    m = block_max_f<NT>(m, red);
    float s = 0.f;
#pragma unroll
    for (int u = 0; u < kSoftmaxVec; ++u) {
      v[u].x = expf(v[u].x - m);
      v[u].y = expf(v[u].y - m);
      v[u].z = expf(v[u].z - m);
      v[u].w = expf(v[u].w - m);
      s += (v[u].x + v[u].y) + (v[u].z + v[u].w);
    }
    s = block_sum_f<NT>(s, red);
    if (threadIdx.x == 0) {
      const double lp = valid ? (double)a[y] - ((double)m + log((double)s)) : (double)NAN;
      rowobj[row] = lp;
      unsafeAtomicAdd(total, lp);   // the objective, cleared at the start of the step (fp64: order does not matter)
    }
    __syncthreads();   // a[y] is read before any thread overwrites the row
    const float inv = 1.f / s;
#pragma unroll
    for (int u = 0; u < kSoftmaxVec; ++u) {
      const int c = (threadIdx.x + u * NT) * 4;
      float4 o;
      o.x = (c == y ? 1.f : 0.f) - v[u].x * inv;
      o.y = (c + 1 == y ? 1.f : 0.f) - v[u].y * inv;
      o.z = (c + 2 == y ? 1.f : 0.f) - v[u].z * inv;
      o.w = (c + 3 == y ? 1.f : 0.f) - v[u].w * inv;
      if (c + 3 < C) {
        *reinterpret_cast<float4*>(a + c) = o;
      } else if (c < C) {
        a[c] = o.x;
        if (c + 1 < C) a[c + 1] = o.y;
        if (c + 2 < C) a[c + 2] = o.z;
      }
    }
    return;
  }
  // wider rows: three passes over memory
  float m = -INFINITY;
  for (int c = threadIdx.x; c < C; c += NT) m = fmaxf(m, a[c]);
  m = block_max_f<NT>(m, red);
  float s = 0.f;
  for (int c = threadIdx.x; c < C; c += NT) s += expf(a[c] - m);
  s = block_sum_f<NT>(s, red);
  const float lse = m + logf(s);
  if (threadIdx.x == 0) {
    const double lp = valid ? (double)a[y] - ((double)m + log((double)s)) : (double)NAN;
    rowobj[row] = lp;
    unsafeAtomicAdd(total, lp);
  }
  __syncthreads();
  for (int c = threadIdx.x; c < C; c += NT) a[c] = (c == y ? 1.f : 0.f) - expf(a[c] - lse);
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
  // patches the fused apply kernel left undone (its bounded wait ran out): Xhat = X - H W is completed here
  const int* deferred_count; // nullptr: none
  const int* deferred;       // rb * n_col_tiles + chunk for each such patch of 64 rows x chunk_cols columns
  float* X;                  // N x D, in place
  const float* W;            // R x D
  const float* H;            // N x ldh, final
  int ldx, ldw, ldh, D, R, chunk_cols;
  // what the fused apply kernel accumulated into (arrival counters and H, contiguous): cleared on exit, so that the
  // next call without a factor update needs no clearing launch in front of it (nullptr: left as it is)
  float* clear_ptr;
  int clear_floats;          // a multiple of 4
};
struct FinishGroup {
  int count;
  FinishArgs a[kMaxInstances];
};

__global__ __launch_bounds__(1024) void finish_apply_kernel(const FinishGroup g) {
  __shared__ double scratch[32];
  const FinishArgs& a = g.a[blockIdx.x];
  const int n_deferred = a.deferred_count != nullptr ? *a.deferred_count : 0;
  if (n_deferred > 0) {
    // 16 threads per row of a 64-row patch; plain dot products over the rank (this path is rare and small)
    const int sub = threadIdx.x & 15;
    for (int e = 0; e < n_deferred; ++e) {
      const int id = a.deferred[e];
      const int rb = id / a.n_col_tiles, chunk = id % a.n_col_tiles;
      const int r = rb * 64 + (threadIdx.x >> 4);
      const int c_end = min(a.D, (chunk + 1) * a.chunk_cols);
      float sq = 0.f;
      if (r < a.N && threadIdx.x < 1024) {
        const float* h = a.H + (size_t)r * a.ldh;
        float* x = a.X + (size_t)r * a.ldx;
        for (int c = chunk * a.chunk_cols + sub; c < c_end; c += 16) {
          float s = 0.f;
          for (int j = 0; j < a.R; ++j) s = fmaf(h[j], a.W[(size_t)j * a.ldw + c], s);
          const float v = x[c] - s;
          x[c] = v;
          sq = fmaf(v, v, sq);
        }
      }
      sq += __shfl_xor(sq, 1);
      sq += __shfl_xor(sq, 2);
      sq += __shfl_xor(sq, 4);
      sq += __shfl_xor(sq, 8);
      if (r < a.N && sub == 0) const_cast<float*>(a.rownorm_part)[(size_t)chunk * a.N + r] = sq;
    }
    __threadfence();
    __syncthreads();   // the partial row norms written above are read below by other lanes
  }
  // Everything below hangs on a few rounds of loads from memory that no cache of this workgroup's die holds yet:
  // they are issued together, and what a row's four lanes find stays in registers until gamma is known.
  double t = 0.0;
  for (int i = threadIdx.x; i < a.n_sumsq; i += blockDim.x) t += a.sumsq_part[i];
  // four lanes share a row: each adds every fourth column tile (independent loads), then the quad is combined
  const int part = threadIdx.x & 3;
  const int N = a.N, nct = a.n_col_tiles;
  const int rows_per_pass = blockDim.x >> 2;
  auto row_sum = [&](int r) -> double {
    float p0 = 0.f, p1 = 0.f;
    if (r < N) {
      int c = part;
      for (; c + 4 < nct; c += 8) {
        p0 += a.rownorm_part[(size_t)c * N + r];
        p1 += a.rownorm_part[(size_t)(c + 4) * N + r];
      }
      if (c < nct) p0 += a.rownorm_part[(size_t)c * N + r];
    }
    double p = (double)p0 + (double)p1;
    p += __shfl_xor(p, 1);
    p += __shfl_xor(p, 2);
    return p;
  };
  constexpr int kKeep = 4;   // passes whose row sums stay in registers (N <= 1024 with 1024 threads)
  double pv[kKeep];
  double ph = 0.0;
#pragma unroll
  for (int ps = 0; ps < kKeep; ++ps) {
    const int r = ps * rows_per_pass + (threadIdx.x >> 2);
    pv[ps] = row_sum(r);
    if (r < N && part == 0) {
      a.prow[r] = pv[ps];
      ph += pv[ps];
    }
  }
  for (int r0 = kKeep * rows_per_pass; r0 < N; r0 += rows_per_pass) {   // (larger minibatches: through memory)
    const int r = r0 + (threadIdx.x >> 2);
    const double p = row_sum(r);
    if (r < N && part == 0) {
      a.prow[r] = p;
      ph += p;
    }
  }
  // tr(X X^T) and tr(Xhat Xhat^T) in one reduction
  {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    t = wave_sum(t);
    ph = wave_sum(ph);
    __syncthreads();
    if (lane == 0) {
      scratch[wave] = t;
      scratch[16 + wave] = ph;
    }
    __syncthreads();
    t = 0.0;
    ph = 0.0;
    for (int w = 0; w < nw; ++w) {
      t += scratch[w];
      ph += scratch[16 + w];
    }
  }
  const double tr_M = t, tr_Mhat = ph;
  const double gamma = tr_Mhat > 0.0 ? sqrt(tr_M / tr_Mhat) : 1.0;
  if (threadIdx.x == 0) {
    a.st->gamma = gamma;
    a.st->tr_M = tr_M;
    a.st->tr_Mhat = tr_Mhat;
    if (a.gamma_out != nullptr) *a.gamma_out = (float)gamma;
  }
  if (a.rownorm2_out != nullptr) {
#pragma unroll
    for (int ps = 0; ps < kKeep; ++ps) {
      const int r = ps * rows_per_pass + (threadIdx.x >> 2);
      if (r < N && part == 0) a.rownorm2_out[r] = (float)(gamma * gamma * pv[ps]);
    }
    if (N > kKeep * rows_per_pass) {
      __syncthreads();   // prow was written by other lanes
      for (int r = kKeep * rows_per_pass + threadIdx.x; r < N; r += blockDim.x)
        a.rownorm2_out[r] = (float)(gamma * gamma * a.prow[r]);
    }
  }
  if (a.clear_ptr != nullptr) {   // (every read of H and of the deferred count lies before a barrier above)
    float4* z = reinterpret_cast<float4*>(a.clear_ptr);
    for (int i = threadIdx.x; i < a.clear_floats / 4; i += blockDim.x) z[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
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

// B_t = J_t + (N (1 - eta) / eta) (D_t + rho_t I) W_t, written over J (eq. wt1).  Grid (col blocks, R, instance).
// Must run while st still holds D_t and rho_t, i.e. before the R x R update kernel.
struct BtArgs {
  float* J;
  const float* W;
  const PrecondScalars* st;
  int ld, D, R, N;
};
struct BtGroup {
  int count;
  double num_samples_history;
  BtArgs a[kMaxInstances];
};
__global__ void make_bt_kernel(const BtGroup g) {
  const BtArgs& a = g.a[blockIdx.z];
  const int i = blockIdx.y;
  if (i >= a.R) return;
  const double eta = 1.0 - exp(-(double)a.N / g.num_samples_history);
  const float f = (float)((double)a.N * (1.0 - eta) / eta * (a.st->d[i] + a.st->rho));
  for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < a.D; c += gridDim.x * blockDim.x)
    a.J[(size_t)i * a.ld + c] += f * a.W[(size_t)i * a.ld + c];
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
