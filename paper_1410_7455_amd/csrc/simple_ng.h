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
constexpr int kSimpleGramTile = 128;  // the Gram matrix is computed in tiles of this size, upper triangle only
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
  double* pinv[2];  // 32 x 32 each: inverse of the pivot block of the current / the next elimination step
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

// Gauss-Jordan inversion of a 32 x 32 positive-definite block by a workgroup of 256 threads, without pivoting.
// Thread (c = tid % 32, r0 = tid / 32) holds column c of rows r0, r0+8, r0+16, r0+24 in cur[] on entry (the
// block) and on exit (its inverse).  A step only needs the pivot row and the pivot column, which their owners
// publish (for the next step, into the other pair of arrays) as soon as they have them: one barrier and a few
// LDS words per step, and the arithmetic is branch-free.  sRow, sCol: LDS, [2][32] each.
__device__ __forceinline__ void invert_block_32(double (&cur)[4], double (*sRow)[kSimpleBlock],
                                                double (*sCol)[kSimpleBlock]) {
  constexpr int B = kSimpleBlock;
  const int tid = threadIdx.x, c = tid & 31, r0 = tid >> 5;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    if (r0 + 8 * q == 0) sRow[0][c] = cur[q];
    if (c == 0) sCol[0][r0 + 8 * q] = cur[q];
  }
  __syncthreads();
  for (int p = 0; p < B; ++p) {
    const int par = p & 1;
    const double piv = sRow[par][p];
    const double rv = sRow[par][c];
    double colv[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) colv[q] = sCol[par][r0 + 8 * q];
    double inv = __builtin_amdgcn_rcp(piv);        // hardware estimate, two Newton steps
    inv = fma(fma(-piv, inv, 1.0), inv, inv);
    inv = fma(fma(-piv, inv, 1.0), inv, inv);
    const double rowv = rv * inv;
    const double on_row = c == p ? inv : rowv;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r = r0 + 8 * q;
      const double off_row = c == p ? -colv[q] * inv : fma(-colv[q], rowv, cur[q]);
      cur[q] = r == p ? on_row : off_row;
    }
    // row p+1 is register (p+1)/8 of the threads with r0 = (p+1) % 8; column p+1 is all four registers of two lanes
    const int qn = (p + 1) >> 3;
    const double next_row = qn == 0 ? cur[0] : (qn == 1 ? cur[1] : (qn == 2 ? cur[2] : cur[3]));
    if (r0 == ((p + 1) & 7)) sRow[par ^ 1][c] = next_row;
    if (c == p + 1) {
#pragma unroll
      for (int q = 0; q < 4; ++q) sCol[par ^ 1][r0 + 8 * q] = cur[q];
    }
    __syncthreads();
  }
}

// G = beta I + S / (N-1), S given by its tiles on and above the diagonal, with beta = alpha max(tr S, epsilon) / (N D)
// (App. A.2); rows and columns beyond n carry the identity so that the padded matrix stays positive definite.
// The workgroup of block (0, 0) also inverts it: the pivot block of the first elimination step.
// Grid (np/32, np/32, count), 256 threads.
__global__ __launch_bounds__(256) void simple_prepare_kernel(const SimpleGroup g) {
  const SimpleArgs& a = g.a[blockIdx.z];
  if ((int)blockIdx.x >= a.nblk || (int)blockIdx.y >= a.nblk) return;
  __shared__ double scratch[16];
  __shared__ double sRow[2][kSimpleBlock], sCol[2][kSimpleBlock];
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
  double blk[4];   // element tid + 256 q of the block: row (tid / 32) + 8 q, column tid % 32
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int e = tid + 256 * q;
    const int i = blockIdx.y * kSimpleBlock + (e >> 5), j = blockIdx.x * kSimpleBlock + (e & 31);
    double v;
    if (i < n && j < n) {
      const bool upper = i / kSimpleGramTile <= j / kSimpleGramTile;   // tiles below the diagonal were not computed
      v = (upper ? S[(size_t)i * np + j] : S[(size_t)j * np + i]) * inv_nm1 + (i == j ? beta : 0.0);
    } else {
      v = i == j ? 1.0 : 0.0;
    }
    G[(size_t)i * np + j] = v;
    blk[q] = v;
  }
  if (blockIdx.x == 0 && blockIdx.y == 0) {
    invert_block_32(blk, sRow, sCol);
#pragma unroll
    for (int q = 0; q < 4; ++q) a.pinv[0][tid + 256 * q] = blk[q];
  }
}

// One pivot block k of the blocked Gauss-Jordan inversion.  Grid (ceil(nblk_max/2) + 1, ceil(nblk_max/2), count),
// 256 threads: wavefront w of workgroup (x, y) owns block (2y + w/2, 2x + w%2) and replaces it, using the inverse
// P_k of the pivot block that the previous launch left in pinv[k % 2].  The one workgroup of the extra grid column
// looks ahead: it forms the next pivot block (k+1, k+1) as this step leaves it and inverts it into pinv[(k+1) % 2],
// so the 32-step elimination is done once per matrix and step, beside the block updates and not before them.
// v_mfma_f64_16x16x4_f64: lane l supplies A[l%16][l/16] and B[l/16][l%16]; register r of lane l holds
// row 4r + l/16, column l%16 of the 16 x 16 result.
__global__ __launch_bounds__(256) void simple_sweep_kernel(const SimpleGroup g, const int k) {
  const SimpleArgs& a = g.a[blockIdx.z];
  const int nblk = a.nblk;
  const bool ahead = blockIdx.x == gridDim.x - 1;
  if (k >= nblk) return;                                                                  // uniform per workgroup
  if (ahead && (blockIdx.y != 0 || k + 1 >= nblk)) return;
  if (!ahead && (2 * (int)blockIdx.x >= nblk || 2 * (int)blockIdx.y >= nblk)) return;
  constexpr int B = kSimpleBlock;
  __shared__ double sP[B][B + 1];      // P_k
  __shared__ double sRow[2][B], sCol[2][B];
  __shared__ double sT[4][B][B + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int np = a.np;
  const double* __restrict__ src = a.buf[k & 1];
  double* __restrict__ dst = a.buf[(k & 1) ^ 1];
  const size_t k0 = (size_t)k * B;

  const int bi = ahead ? k + 1 : 2 * blockIdx.y + (wave >> 1), bj = ahead ? k + 1 : 2 * blockIdx.x + (wave & 1);
  const bool active = ahead ? wave == 0 : (bi < nblk && bj < nblk);
  const int l16 = lane & 15, g4 = lane >> 4;
  const size_t i0 = (size_t)bi * B, j0 = (size_t)bj * B;
  typedef double doublex4 __attribute__((ext_vector_type(4)));

  // everything this wavefront needs is requested up front: P_k, A_ik by rows (it goes to LDS), A_kj as B-operand
  // fragments, A_ij as accumulators
  double pv[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) pv[q] = a.pinv[k & 1][tid + 256 * q];
  double aik[16];
  double bf[B / 4][2];
  doublex4 acc[2][2];
  if (active) {
    if (bi != k) {
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int e = lane + 64 * q;
        aik[q] = src[(i0 + (e >> 5)) * np + k0 + (e & 31)];
      }
    }
    if (bj != k) {
#pragma unroll
      for (int ks = 0; ks < B / 4; ++ks)
#pragma unroll
        for (int nj = 0; nj < 2; ++nj) bf[ks][nj] = src[(k0 + ks * 4 + g4) * np + j0 + nj * 16 + l16];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int nj = 0; nj < 2; ++nj)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            acc[mi][nj][r] = bi != k ? src[(i0 + mi * 16 + 4 * r + g4) * np + j0 + nj * 16 + l16] : 0.0;
    }
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int e = tid + 256 * q;
    sP[e >> 5][e & 31] = pv[q];
  }
  __syncthreads();
  const double (*P)[B + 1] = sP;

  // T = A_ik P  (bi != k)  or  -P  (bi == k), kept in LDS in row-major form for the second product.  The
  // barriers are outside every wave-dependent branch; they also order the wavefront's own LDS writes and reads.
  const bool mult = active && bi != k;
  if (mult) {
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int e = lane + 64 * q;
      sT[wave][e >> 5][e & 31] = aik[q];
    }
  }
  __syncthreads();
  doublex4 t[2][2];
  if (mult) {
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int nj = 0; nj < 2; ++nj) t[mi][nj] = doublex4{0, 0, 0, 0};
#pragma unroll
    for (int ks = 0; ks < B / 4; ++ks) {
      double af[2], pf[2];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi) af[mi] = sT[wave][mi * 16 + l16][ks * 4 + g4];
#pragma unroll
      for (int nj = 0; nj < 2; ++nj) pf[nj] = P[ks * 4 + g4][nj * 16 + l16];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int nj = 0; nj < 2; ++nj)
          t[mi][nj] = __builtin_amdgcn_mfma_f64_16x16x4f64(af[mi], pf[nj], t[mi][nj], 0, 0, 0);
    }
  }
  __syncthreads();
  if (mult) {
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int nj = 0; nj < 2; ++nj)
#pragma unroll
        for (int r = 0; r < 4; ++r) sT[wave][mi * 16 + 4 * r + g4][nj * 16 + l16] = t[mi][nj][r];
  } else if (active) {
    for (int e = lane; e < B * B; e += 64) sT[wave][e >> 5][e & 31] = -P[e >> 5][e & 31];
  }
  __syncthreads();
  if (!active && !ahead) return;

  // new block: (bj != k)  C0 - T A_kj with C0 = A_ij (bi != k) or 0;   (bj == k)  -T
  if (!active) {
    // look-ahead workgroup, wavefronts 1..3: nothing to multiply
  } else if (bj != k) {
#pragma unroll
    for (int ks = 0; ks < B / 4; ++ks) {
      double af[2];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi) af[mi] = -sT[wave][mi * 16 + l16][ks * 4 + g4];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int nj = 0; nj < 2; ++nj)
          acc[mi][nj] = __builtin_amdgcn_mfma_f64_16x16x4f64(af[mi], bf[ks][nj], acc[mi][nj], 0, 0, 0);
    }
  } else {
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int nj = 0; nj < 2; ++nj)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[mi][nj][r] = -sT[wave][mi * 16 + 4 * r + g4][nj * 16 + l16];
  }
  if (ahead) {
    // the next pivot block is in wavefront 0's accumulators: through LDS to the elimination's layout, invert, publish
    if (active) {
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int nj = 0; nj < 2; ++nj)
#pragma unroll
          for (int r = 0; r < 4; ++r) sT[1][mi * 16 + 4 * r + g4][nj * 16 + l16] = acc[mi][nj][r];
    }
    __syncthreads();
    double blk[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int e = tid + 256 * q;
      blk[q] = sT[1][e >> 5][e & 31];
    }
    invert_block_32(blk, sRow, sCol);
#pragma unroll
    for (int q = 0; q < 4; ++q) a.pinv[(k + 1) & 1][tid + 256 * q] = blk[q];
    return;
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
  const int tid = threadIdx.x, D = a.D, D4 = D >> 2;
  float* __restrict__ x = a.M + (size_t)i * a.ld;           // rows start on 16-byte boundaries
  const float* __restrict__ q = a.Q + (size_t)i * a.ldq;
  float4* __restrict__ x4 = reinterpret_cast<float4*>(x);
  const float4* __restrict__ q4 = reinterpret_cast<const float4*>(q);
  double dot = 0.0, qq = 0.0;
  for (int c = tid; c < D4; c += 256) {
    const float4 xv = x4[c], qv = q4[c];
    dot += (double)xv.x * qv.x + (double)xv.y * qv.y + (double)xv.z * qv.z + (double)xv.w * qv.w;
    qq += (double)qv.x * qv.x + (double)qv.y * qv.y + (double)qv.z * qv.z + (double)qv.w * qv.w;
  }
  for (int c = 4 * D4 + tid; c < D; c += 256) {
    const double xv = x[c], qv = q[c];
    dot += xv * qv;
    qq += qv * qv;
  }
  dot = block_sum(dot, scratch);
  qq = block_sum(qq, scratch);
  const double b = 1.0 + dot / ((double)(a.N - 1) - dot);
  for (int c = tid; c < D4; c += 256) {
    const float4 qv = q4[c];
    x4[c] = make_float4((float)(b * qv.x), (float)(b * qv.y), (float)(b * qv.z), (float)(b * qv.w));
  }
  for (int c = 4 * D4 + tid; c < D; c += 256) x[c] = (float)(b * (double)q[c]);
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
