// Initialisation of the online natural-gradient state from the first minibatch (App. B.3.2):
// top-R eigenpairs of S_0 = X_0^T X_0 / N, rho_0, D_0, then W_0 = E_0^{1/2} R_0.
//
// The eigenproblem is solved on the smaller of the D x D covariance and the N x N Gram matrix (same
// non-zero spectrum; an eigenvector u of the Gram matrix gives X_0^T u / sqrt(N lambda)).  The n x n
// symmetric matrix (n <= 1024..) is diagonalised in fp64 by a cyclic Jacobi method whose rounds are
// whole-GPU launches: a round applies n/2 disjoint rotations A <- J^T A J, every thread owning one
// 2x2 block, reading from one buffer and writing the other.  This runs once per process (and after
// each parameter-averaging round), never inside the steady-state step.
#pragma once

#include <hip/hip_runtime.h>

#include "kernels.h"
#include "small_update.h"
#include "state.h"

namespace ngsgd {

constexpr double kNullEigRatio = 1.0e-12;          // eigenvalues of S_0 at or below this ratio carry no direction
constexpr double kCompletionMinResidual = 0.1;     // Gram-Schmidt completion threshold
constexpr int kInitSweeps = 12;

struct InitArgs {
  PrecondScalars* st;
  const float* M;      // N x D first minibatch
  int ld;
  int N, D, R;
  int n;               // min(N, D): size of the eigenproblem
  int use_cov;         // 1: n = D, matrix X^T X / N; 0: n = N, matrix X X^T / N
  double* A[2];        // n x n ping-pong
  double* V[2];        // n x n eigenvector accumulators (columns)
  int* idx;            // R: column of V for each kept eigenpair, -1 if the direction is null
  float* W;            // R x ldw
  int ldw;
  double* vwork;       // D doubles
};
struct InitGroup {
  int count;
  double alpha, epsilon;
  InitArgs a[kMaxInstances];
};

// C = (1/N) X^T X (use_cov) or (1/N) X X^T, fp64 accumulation of fp32 data; V = I.  Grid (tiles, tiles, instance).
__global__ __launch_bounds__(256) void init_gram_kernel(const InitGroup g) {
  const InitArgs& a = g.a[blockIdx.z];
  const int n = a.n;
  const int i0 = blockIdx.y * 32, j0 = blockIdx.x * 32;
  if (i0 >= n || j0 >= n) return;
  __shared__ float sa[32][33], sb[32][33];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;   // 16 x 16 threads, 2 x 2 outputs each
  double acc[2][2] = {{0.0, 0.0}, {0.0, 0.0}};
  const int K = a.use_cov ? a.N : a.D;
  for (int k0 = 0; k0 < K; k0 += 32) {
    for (int t = threadIdx.x; t < 32 * 32; t += 256) {
      const int r = t >> 5, c = t & 31;
      float va = 0.f, vb = 0.f;
      if (a.use_cov) {   // element (i, k) = X[k][i]: r indexes k, c indexes i
        const int k = k0 + r;
        if (k < K) {
          if (i0 + c < n) va = a.M[(size_t)k * a.ld + i0 + c];
          if (j0 + c < n) vb = a.M[(size_t)k * a.ld + j0 + c];
        }
        sa[r][c] = va;   // [k][i]
        sb[r][c] = vb;
      } else {           // element (i, k) = X[i][k]: r indexes i, c indexes k
        const int k = k0 + c;
        if (k < K) {
          if (i0 + r < n) va = a.M[(size_t)(i0 + r) * a.ld + k];
          if (j0 + r < n) vb = a.M[(size_t)(j0 + r) * a.ld + k];
        }
        sa[c][r] = va;   // stored [k][i] as well
        sb[c][r] = vb;
      }
    }
    __syncthreads();
#pragma unroll 4
    for (int k = 0; k < 32; ++k) {
      const double a0 = sa[k][ty], a1 = sa[k][ty + 16];
      const double b0 = sb[k][tx], b1 = sb[k][tx + 16];
      acc[0][0] += a0 * b0;
      acc[0][1] += a0 * b1;
      acc[1][0] += a1 * b0;
      acc[1][1] += a1 * b1;
    }
    __syncthreads();
  }
  const double inv_n = 1.0 / (double)a.N;
  for (int u = 0; u < 2; ++u)
    for (int v = 0; v < 2; ++v) {
      const int i = i0 + ty + 16 * u, j = j0 + tx + 16 * v;
      if (i < n && j < n) {
        a.A[0][(size_t)i * n + j] = acc[u][v] * inv_n;
        a.V[0][(size_t)i * n + j] = i == j ? 1.0 : 0.0;
      }
    }
}

// One Jacobi round on every instance: A_out = J^T A_in J, V_out = V_in J.  Grid (blocks, 1, instance).
// `round` counts from 0 over all sweeps; an instance of size n uses round % (m-1) with m = n rounded up to even.
__global__ __launch_bounds__(256) void init_jacobi_round_kernel(const InitGroup g, int round, int src) {
  const InitArgs& a = g.a[blockIdx.z];
  const int n = a.n;
  const int m = (n + 1) & ~1, half = m / 2;
  const int r = round % (m - 1);
  const double* __restrict__ Ain = a.A[src];
  double* __restrict__ Aout = a.A[src ^ 1];
  const double* __restrict__ Vin = a.V[src];
  double* __restrict__ Vout = a.V[src ^ 1];
  const long long n_blk = (long long)half * half;
  const long long n_v = (long long)n * half;
  for (long long w = blockIdx.x * (long long)blockDim.x + threadIdx.x; w < n_blk + n_v;
       w += (long long)gridDim.x * blockDim.x) {
    if (w < n_blk) {
      const int bi = (int)(w / half), bj = (int)(w % half);
      int pi, qi, pj, qj;
      round_robin_pair(m, r, bi, pi, qi);
      round_robin_pair(m, r, bj, pj, qj);
      double ci = 1.0, si = 0.0, cj = 1.0, sj = 0.0;
      if (qi < n) sym_schur2(Ain[(size_t)pi * n + pi], Ain[(size_t)qi * n + qi], Ain[(size_t)pi * n + qi], ci, si);
      if (bj == bi) {
        cj = ci;
        sj = si;
      } else if (qj < n) {
        sym_schur2(Ain[(size_t)pj * n + pj], Ain[(size_t)qj * n + qj], Ain[(size_t)pj * n + qj], cj, sj);
      }
      const bool ri = qi < n, rj = qj < n;   // false: the pair holds the padding index, only p is real
      const double x00 = Ain[(size_t)pi * n + pj];
      const double x01 = rj ? Ain[(size_t)pi * n + qj] : 0.0;
      const double x10 = ri ? Ain[(size_t)qi * n + pj] : 0.0;
      const double x11 = (ri && rj) ? Ain[(size_t)qi * n + qj] : 0.0;
      const double y00 = ci * x00 - si * x10, y01 = ci * x01 - si * x11;
      const double y10 = si * x00 + ci * x10, y11 = si * x01 + ci * x11;
      double b00 = y00 * cj - y01 * sj, b01 = y00 * sj + y01 * cj;
      double b10 = y10 * cj - y11 * sj, b11 = y10 * sj + y11 * cj;
      if (bi == bj) b01 = b10 = 0.0;
      Aout[(size_t)pi * n + pj] = b00;
      if (rj) Aout[(size_t)pi * n + qj] = b01;
      if (ri) Aout[(size_t)qi * n + pj] = b10;
      if (ri && rj) Aout[(size_t)qi * n + qj] = b11;
    } else {
      const long long v = w - n_blk;
      const int row = (int)(v / half), bj = (int)(v % half);
      int pj, qj;
      round_robin_pair(m, r, bj, pj, qj);
      if (qj < n) {
        double cj, sj;
        sym_schur2(Ain[(size_t)pj * n + pj], Ain[(size_t)qj * n + qj], Ain[(size_t)pj * n + qj], cj, sj);
        const double u0 = Vin[(size_t)row * n + pj], u1 = Vin[(size_t)row * n + qj];
        Vout[(size_t)row * n + pj] = u0 * cj - u1 * sj;
        Vout[(size_t)row * n + qj] = u0 * sj + u1 * cj;
      } else {
        Vout[(size_t)row * n + pj] = Vin[(size_t)row * n + pj];
      }
    }
  }
}

// Top-R eigenvalues, rho_0, D_0, E_0 (App. B.3.2 with eq. beta2, etii).  One workgroup per instance.
// `src` is the buffer holding the diagonalised matrix.
__global__ __launch_bounds__(1024) void init_select_kernel(const InitGroup g, int src) {
  __shared__ double scratch[16];
  __shared__ double s_lam[kMaxRank];
  __shared__ int s_idx[kMaxRank];
  const InitArgs& a = g.a[blockIdx.x];
  const int n = a.n, R = a.R, D = a.D;
  const double* A = a.A[src];
  PrecondScalars* st = a.st;
  double tr = 0.0;
  for (int i = threadIdx.x; i < n; i += blockDim.x) tr += A[(size_t)i * n + i];
  tr = block_sum(tr, scratch);
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    const double li = A[(size_t)i * n + i];
    int rank = 0;
    for (int j = 0; j < n; ++j) {
      const double lj = A[(size_t)j * n + j];
      rank += (lj > li || (lj == li && j < i)) ? 1 : 0;
    }
    if (rank < R) {
      s_lam[rank] = li;
      s_idx[rank] = i;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    const double lmax = s_lam[0];
    double sum_l = 0.0;
    for (int k = 0; k < R; ++k) {
      const bool keep = lmax > 0.0 && s_lam[k] > kNullEigRatio * lmax;
      if (!keep) {
        s_lam[k] = 0.0;
        s_idx[k] = -1;
      }
      sum_l += s_lam[k];
    }
    const double rho0 = fmax((tr - sum_l) / (double)(D - R), g.epsilon);
    double sum_d = 0.0;
    for (int k = 0; k < R; ++k) {
      const double d = fmax(g.epsilon, s_lam[k] - rho0);
      st->d[k] = d;
      sum_d += d;
    }
    const double beta = rho0 * (1.0 + g.alpha) + g.alpha / (double)D * sum_d;
    for (int k = 0; k < R; ++k) st->e[k] = 1.0 / (beta / st->d[k] + 1.0);
    st->rho = rho0;
    st->beta = beta;
    st->trace_S0 = tr;
    st->flags = 0;
    st->sweeps = 0;
    // eigenvalue kept for the Gram route's 1/sqrt(N lambda); parked in gamma/tr fields is not possible: use vwork
    for (int k = 0; k < R; ++k) {
      a.idx[k] = s_idx[k];
      a.vwork[k] = s_lam[k];
    }
  }
}

// W_0 rows of the kept eigenpairs: sqrt(e_i) v_i with v_i a column of V (covariance route) or
// X_0^T u_i / sqrt(N lambda_i) (Gram route); zero for null directions.  Grid (col blocks of 64, R, instance).
__global__ __launch_bounds__(256) void init_rows_kernel(const InitGroup g, int src) {
  const InitArgs& a = g.a[blockIdx.z];
  const int i = blockIdx.y;
  if (i >= a.R) return;
  const int col = blockIdx.x * 64 + (threadIdx.x & 63);
  const int part = threadIdx.x >> 6;   // 4 slices of the row range
  if (blockIdx.x * 64 >= a.ldw) return;
  __shared__ double s_acc[4][64];
  const int src_col = a.idx[i];
  const double* V = a.V[src];
  const int n = a.n;
  double acc = 0.0;
  if (src_col >= 0 && col < a.D) {
    if (a.use_cov) {
      if (part == 0) acc = V[(size_t)col * n + src_col];
    } else {
      const int rows_per = (a.N + 3) / 4;
      const int r0 = part * rows_per, r1 = min(a.N, r0 + rows_per);
      for (int r = r0; r < r1; ++r) acc += (double)a.M[(size_t)r * a.ld + col] * V[(size_t)r * n + src_col];
    }
  }
  s_acc[part][threadIdx.x & 63] = acc;
  __syncthreads();
  if (part == 0 && col < a.ldw) {
    double v = s_acc[0][threadIdx.x] + s_acc[1][threadIdx.x] + s_acc[2][threadIdx.x] + s_acc[3][threadIdx.x];
    if (src_col >= 0 && col < a.D) {
      double scale = sqrt(a.st->e[i]);
      if (!a.use_cov) scale /= sqrt((double)a.N * a.vwork[i]);
      v *= scale;
    } else {
      v = 0.0;
    }
    a.W[(size_t)i * a.ldw + col] = (float)v;
  }
}

// Rows of R_0 for null directions: Gram-Schmidt completion from the standard basis e_0, e_1, ... (each
// candidate orthogonalised twice against all rows fixed so far, accepted when its residual exceeds 0.1).
// One workgroup per instance; returns at once when every direction was kept.
__global__ __launch_bounds__(1024) void init_complete_kernel(const InitGroup g) {
  __shared__ double scratch[16];
  __shared__ int s_fixed[kMaxRank];
  __shared__ int s_nfixed, s_missing;
  const InitArgs& a = g.a[blockIdx.x];
  const int R = a.R, D = a.D, ldw = a.ldw;
  const int tid = threadIdx.x, nt = blockDim.x;
  if (tid == 0) {
    int nf = 0, miss = 0;
    for (int k = 0; k < R; ++k) {
      if (a.idx[k] >= 0) s_fixed[nf++] = k; else ++miss;
    }
    s_nfixed = nf;
    s_missing = miss;
  }
  __syncthreads();
  if (s_missing == 0) return;
  double* v = a.vwork + kMaxRank;   // first kMaxRank entries hold the eigenvalues
  float* W = a.W;
  const PrecondScalars* st = a.st;
  int cand = 0;
  for (int i = 0; i < R; ++i) {
    if (a.idx[i] >= 0) continue;    // uniform
    bool accepted = false;
    while (!accepted && cand < D) {
      for (int c = tid; c < D; c += nt) v[c] = c == cand ? 1.0 : 0.0;
      ++cand;
      __syncthreads();
      for (int pass = 0; pass < 2; ++pass) {
        const int nf = s_nfixed;
        for (int f = 0; f < nf; ++f) {
          const int j = s_fixed[f];
          const double inv = 1.0 / sqrt(st->e[j]);
          double dot = 0.0;
          for (int c = tid; c < D; c += nt) dot += (double)W[(size_t)j * ldw + c] * inv * v[c];
          dot = block_sum(dot, scratch);
          for (int c = tid; c < D; c += nt) v[c] -= dot * (double)W[(size_t)j * ldw + c] * inv;
          __syncthreads();
        }
      }
      double nrm = 0.0;
      for (int c = tid; c < D; c += nt) nrm += v[c] * v[c];
      nrm = sqrt(block_sum(nrm, scratch));
      if (nrm > kCompletionMinResidual) {
        const double s = sqrt(st->e[i]) / nrm;
        for (int c = tid; c < ldw; c += nt) W[(size_t)i * ldw + c] = c < D ? (float)(s * v[c]) : 0.f;
        __syncthreads();
        if (tid == 0) s_fixed[s_nfixed++] = i;
        __syncthreads();
        accepted = true;
      }
    }
  }
}

}  // namespace ngsgd
