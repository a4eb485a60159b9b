// Simple natural-gradient method (App. A): Fisher factors from the other rows of the same minibatch.
//
// For an N x D matrix X the efficient form (App. A.3) needs one symmetric positive-definite inverse of size
// n = min(N, D):  G = beta I + X^T X / (N-1)  (column space, N > D)  or  beta I + X X^T / (N-1)  (row space),
// Q = X G^{-1} resp. G^{-1} X, then a_i = x_i . q_i, b_i = 1 + a_i / (N-1-a_i), xhat_i = b_i q_i, and the
// rescaling gamma of App. A.2.
//
// The Gram matrix and Q are products for the matrix units (gemm.h).  The inverse is a blocked Gauss-Jordan
// elimination in fp64 without pivoting (G is positive definite, its condition number is at most about 1 + D/alpha):
// one launch per 32-wide pivot block k, every workgroup of the launch inverts the pivot block itself in LDS and
// then replaces its own 32 x 32 blocks,
//     (k,k) <- P = A_kk^{-1},   (k,j) <- P A_kj,   (i,k) <- -A_ik P,   (i,j) <- A_ij - A_ik P A_kj,
// reading the old matrix from one buffer and writing the new one to the other, so a launch has no ordering
// among its workgroups.  After the last pivot block the buffer holds G^{-1}.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"
#include "state.h"

namespace ngsgd {

constexpr int kSimpleBlock = 32;      // pivot block of the inversion
constexpr int kSimpleMaxGroup = 16;   // matrices per grouped launch (the argument block stays within 4 KB)

struct SimpleArgs {
  float* M;         // N x D, ld: X on entry, Xhat (or gamma Xhat) on exit
  float* Q;         // N x D, ldq: scratch for Q
  int ld, ldq;
  int N, D;
  int n, np, nblk;  // size of the Gram matrix, padded to a multiple of 32, number of pivot blocks
  double alpha, epsilon;
  double* buf[2];   // np x np each; the Gram matrix is accumulated in buf[1]
  float* ginv;      // np x np, G^{-1} rounded to fp32 for the Q product
  double* prow;     // N: ||xhat_i||^2
  double* scal;     // [0] tr(X^T X), [1] beta
  double* gamma;    // gamma (App. A.2)
  float* gamma_out;     // optional copies for the caller
  float* rownorm2_out;  // optional: gamma^2 ||xhat_i||^2
};
struct SimpleGroup {
  int count;
  SimpleArgs a[kSimpleMaxGroup];
};

// G = beta I + S / (N-1) with beta = alpha max(tr S, epsilon) / (N D) (App. A.2); rows and columns beyond n carry
// the identity so that the padded matrix stays positive definite.  Grid (np/32, np/32, count), 256 threads.
__global__ __launch_bounds__(256) void simple_prepare_kernel(const SimpleGroup g) {
  const SimpleArgs& a = g.a[blockIdx.z];
  if ((int)blockIdx.x >= a.nblk || (int)blockIdx.y >= a.nblk) return;
  __shared__ double scratch[16];
  const int tid = threadIdx.x, np = a.np, n = a.n;
  const double* __restrict__ S = a.buf[1];
  double t = 0.0;
  for (int i = tid; i < n; i += 256) t += S[(size_t)i * np + i];
  const double tr = block_sum(t, scratch);
  const double beta = a.alpha * fmax(tr, a.epsilon) / ((double)a.N * (double)a.D);
  if (blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) {
    a.scal[0] = tr;
    a.scal[1] = beta;
  }
  const double inv_nm1 = 1.0 / (double)(a.N - 1);
  double* __restrict__ G = a.buf[0];
  for (int e = tid; e < kSimpleBlock * kSimpleBlock; e += 256) {
    const int i = blockIdx.y * kSimpleBlock + (e >> 5), j = blockIdx.x * kSimpleBlock + (e & 31);
    double v;
    if (i < n && j < n) v = S[(size_t)i * np + j] * inv_nm1 + (i == j ? beta : 0.0);
    else v = i == j ? 1.0 : 0.0;
    G[(size_t)i * np + j] = v;
  }
}

// One pivot block of the blocked Gauss-Jordan inversion.  Grid (ceil(nblk_max/2), ceil(nblk_max/2), count),
// 256 threads: wavefront w of workgroup (x, y) owns block (2y + w/2, 2x + w%2).
// v_mfma_f64_16x16x4_f64: lane l supplies A[l%16][l/16] and B[l/16][l%16]; register r of lane l holds
// row 4r + l/16, column l%16 of the 16 x 16 result.
__global__ __launch_bounds__(256) void simple_sweep_kernel(const SimpleGroup g, const int k) {
  const SimpleArgs& a = g.a[blockIdx.z];
  const int nblk = a.nblk;
  if (k >= nblk || 2 * (int)blockIdx.x >= nblk || 2 * (int)blockIdx.y >= nblk) return;   // uniform per workgroup
  constexpr int B = kSimpleBlock;
  __shared__ double sP[B][B + 1];
  __shared__ double sT[4][B][B + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int np = a.np;
  const double* __restrict__ src = a.buf[k & 1];
  double* __restrict__ dst = a.buf[(k & 1) ^ 1];
  const size_t k0 = (size_t)k * B;

  for (int e = tid; e < B * B; e += 256) sP[e >> 5][e & 31] = src[(k0 + (e >> 5)) * np + k0 + (e & 31)];
  __syncthreads();
  // in-place Gauss-Jordan on the pivot block: thread owns column c of rows r0, r0+8, r0+16, r0+24
  {
    const int c = tid & 31, r0 = tid >> 5;
    for (int p = 0; p < B; ++p) {
      const double inv = 1.0 / sP[p][p];
      const double rowv = sP[p][c] * inv;
      double colv[4], cur[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        colv[q] = sP[r0 + 8 * q][p];
        cur[q] = sP[r0 + 8 * q][c];
      }
      __syncthreads();
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int r = r0 + 8 * q;
        double v;
        if (r == p) v = c == p ? inv : rowv;
        else if (c == p) v = -colv[q] * inv;
        else v = cur[q] - colv[q] * rowv;
        sP[r][c] = v;
      }
      __syncthreads();
    }
  }

  const int bi = 2 * blockIdx.y + (wave >> 1), bj = 2 * blockIdx.x + (wave & 1);
  const bool active = bi < nblk && bj < nblk;
  const int l16 = lane & 15, g4 = lane >> 4;
  const size_t i0 = (size_t)bi * B, j0 = (size_t)bj * B;
  typedef double doublex4 __attribute__((ext_vector_type(4)));
  doublex4 acc[2][2];

  // T = A_ik P  (bi != k)  or  -P  (bi == k), kept in LDS in row-major form for the second product
  if (active) {
    if (bi != k) {
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int nj = 0; nj < 2; ++nj) acc[mi][nj] = doublex4{0, 0, 0, 0};
#pragma unroll
      for (int ks = 0; ks < B / 4; ++ks) {
        double af[2], bf[2];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) af[mi] = src[(i0 + mi * 16 + l16) * np + k0 + ks * 4 + g4];
#pragma unroll
        for (int nj = 0; nj < 2; ++nj) bf[nj] = sP[ks * 4 + g4][nj * 16 + l16];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
          for (int nj = 0; nj < 2; ++nj)
            acc[mi][nj] = __builtin_amdgcn_mfma_f64_16x16x4f64(af[mi], bf[nj], acc[mi][nj], 0, 0, 0);
      }
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int nj = 0; nj < 2; ++nj)
#pragma unroll
          for (int r = 0; r < 4; ++r) sT[wave][mi * 16 + 4 * r + g4][nj * 16 + l16] = acc[mi][nj][r];
    } else {
      for (int e = lane; e < B * B; e += 64) sT[wave][e >> 5][e & 31] = -sP[e >> 5][e & 31];
    }
  }
  __syncthreads();
  if (!active) return;

  // new block: (bj != k)  C0 - T A_kj with C0 = A_ij (bi != k) or 0;   (bj == k)  -T
  if (bj != k) {
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int nj = 0; nj < 2; ++nj)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          acc[mi][nj][r] = bi != k ? src[(i0 + mi * 16 + 4 * r + g4) * np + j0 + nj * 16 + l16] : 0.0;
#pragma unroll
    for (int ks = 0; ks < B / 4; ++ks) {
      double af[2], bf[2];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi) af[mi] = -sT[wave][mi * 16 + l16][ks * 4 + g4];
#pragma unroll
      for (int nj = 0; nj < 2; ++nj) bf[nj] = src[(k0 + ks * 4 + g4) * np + j0 + nj * 16 + l16];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int nj = 0; nj < 2; ++nj)
          acc[mi][nj] = __builtin_amdgcn_mfma_f64_16x16x4f64(af[mi], bf[nj], acc[mi][nj], 0, 0, 0);
    }
  } else {
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int nj = 0; nj < 2; ++nj)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[mi][nj][r] = -sT[wave][mi * 16 + 4 * r + g4][nj * 16 + l16];
  }
  const bool last = k == nblk - 1;
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int nj = 0; nj < 2; ++nj)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const size_t at = (i0 + mi * 16 + 4 * r + g4) * np + j0 + nj * 16 + l16;
        dst[at] = acc[mi][nj][r];
        if (last) a.ginv[at] = (float)acc[mi][nj][r];
      }
}

// a_i = x_i . q_i, b_i = 1 + a_i / (N - 1 - a_i), xhat_i = b_i q_i (App. A.3), ||xhat_i||^2.  Grid (N_max, count).
__global__ __launch_bounds__(256) void simple_rows_kernel(const SimpleGroup g) {
  const SimpleArgs& a = g.a[blockIdx.y];
  const int i = blockIdx.x;
  if (i >= a.N) return;
  __shared__ double scratch[16];
  const int tid = threadIdx.x;
  float* __restrict__ x = a.M + (size_t)i * a.ld;
  const float* __restrict__ q = a.Q + (size_t)i * a.ldq;
  double dot = 0.0, qq = 0.0;
  for (int c = tid; c < a.D; c += 256) {
    const double xv = x[c], qv = q[c];
    dot += xv * qv;
    qq += qv * qv;
  }
  dot = block_sum(dot, scratch);
  qq = block_sum(qq, scratch);
  const double b = 1.0 + dot / ((double)(a.N - 1) - dot);
  for (int c = tid; c < a.D; c += 256) x[c] = (float)(b * (double)q[c]);
  if (tid == 0) a.prow[i] = b * b * qq;
}

// gamma = sqrt(tr(X^T X) / tr(Xhat^T Xhat)), 1 if the denominator is 0 (App. A.2).  Grid (count), 256 threads.
__global__ __launch_bounds__(256) void simple_gamma_kernel(const SimpleGroup g) {
  const SimpleArgs& a = g.a[blockIdx.x];
  __shared__ double scratch[16];
  const int tid = threadIdx.x;
  double den = 0.0;
  for (int i = tid; i < a.N; i += 256) den += a.prow[i];
  den = block_sum(den, scratch);
  const double gamma = den > 0.0 ? sqrt(a.scal[0] / den) : 1.0;
  if (tid == 0) {
    *a.gamma = gamma;
    if (a.gamma_out != nullptr) *a.gamma_out = (float)gamma;
  }
  if (a.rownorm2_out != nullptr)
    for (int i = tid; i < a.N; i += 256) a.rownorm2_out[i] = (float)(gamma * gamma * a.prow[i]);
}

}  // namespace ngsgd
