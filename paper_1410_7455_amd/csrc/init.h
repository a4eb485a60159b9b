// Initialisation of the online natural-gradient state from the first minibatch (App. B.3.2):
// top-R eigenpairs of S_0 = X_0^T X_0 / N, rho_0, D_0, then W_0 = E_0^{1/2} R_0.
//
// The eigenproblem is solved on the smaller of the D x D covariance and the N x N Gram matrix (same
// non-zero spectrum; an eigenvector u of the Gram matrix gives X_0^T u / sqrt(N lambda)).  The n x n
// symmetric matrix (n <= 1024..) is diagonalised in fp64 by a two-sided block Jacobi method: the indices are
// cut into blocks of 32; in a round every workgroup holds two blocks, applies that round's rotations to their
// 64 x 64 sub-matrix in LDS and keeps the accumulated rotation Q; a second launch applies A <- Q^T A Q,
// V <- V Q tile by tile on the fp64 matrix unit.  A sweep over n = 512 is 16 rounds of two launches that touch
// the matrix once each (the element-wise method it replaces took 511 launches per sweep, each a pass over the
// whole matrix) and rotates every index pair once.  This runs once per process (and after each
// parameter-averaging round), never inside the steady-state step.
#pragma once

#include <hip/hip_runtime.h>

#include "kernels.h"
#include "small_update.h"
#include "state.h"

namespace ngsgd {

constexpr double kNullEigRatio = 1.0e-12;          // eigenvalues of S_0 at or below this ratio carry no direction
constexpr double kCompletionMinResidual = 0.1;     // Gram-Schmidt completion threshold
constexpr int kInitBlock = 32;                     // index block of the block Jacobi method
constexpr int kInitPair = 2 * kInitBlock;          // two blocks: the sub-problem a workgroup holds in a round
constexpr int kInitMaxSweeps = 18;                 // block sweeps enqueued; the kernels return at once after convergence
constexpr double kInitRotateTol = 1.0e-8;          // entries below this, relative to their diagonal pair, are not rotated ...
constexpr double kInitCountFloor = 3.0e-14;        // ... nor those below this fraction of the trace (the rounding noise
                                                   // that applying a round's rotations leaves in every entry)
constexpr int kInitSolveLds = 4 * kInitPair * (kInitPair + 1) * (int)sizeof(double);   // two copies of A_sub and Q

struct InitArgs {
  PrecondScalars* st;
  const float* M;      // N x D first minibatch
  int ld;
  int N, D, R;
  int n;               // min(N, D): size of the eigenproblem
  int np;              // n rounded up to a multiple of 64 (zero padding, decoupled from the rest)
  int use_cov;         // 1: n = D, matrix X^T X / N; 0: n = N, matrix X X^T / N
  double* A;           // np x np, diagonalised in place
  double* V;           // np x np eigenvector accumulator (columns)
  double* Q;           // (np / 64) x 64 x 64: the rotation of every workgroup of the current round
  double* stat;        // [0] trace of the matrix, [1] block sweeps run
  int* cnt;            // [3]: rotations of block sweep s in cnt[s % 3]
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

// The initialisation is some hundreds of small launches: the instance list is stored in device memory once and the
// kernels take a pointer to it (a launch that carries the 3.6 KB list by value costs the host three times as much).
__global__ void init_store_group_kernel(const InitGroup g, InitGroup* __restrict__ dst) {
  const uint32_t* src = reinterpret_cast<const uint32_t*>(&g);
  uint32_t* out = reinterpret_cast<uint32_t*>(dst);
  for (int i = threadIdx.x; i < (int)(sizeof(InitGroup) / sizeof(uint32_t)); i += blockDim.x) out[i] = src[i];
}

// C = (1/N) X^T X (use_cov) or (1/N) X X^T, fp64 accumulation of fp32 data; V = I.  Grid (tiles, tiles, instance).
__global__ __launch_bounds__(256) void init_gram_kernel(const InitGroup* __restrict__ gp) {
  const InitArgs& a = gp->a[blockIdx.z];
  const int n = a.n, np = a.np;
  const int i0 = blockIdx.y * 32, j0 = blockIdx.x * 32;
  if (i0 >= np || j0 >= np) return;
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
      if (i < np && j < np) {
        a.A[(size_t)i * np + j] = (i < n && j < n) ? acc[u][v] * inv_n : 0.0;
        a.V[(size_t)i * np + j] = i == j ? 1.0 : 0.0;
      }
    }
}

// Trace of the matrix (the scale of the convergence test) and cleared rotation counters.  One workgroup per instance.
__global__ __launch_bounds__(256) void init_scale_kernel(const InitGroup* __restrict__ gp) {
  const InitArgs& a = gp->a[blockIdx.x];
  __shared__ double scratch[16];
  double t = 0.0;
  for (int i = threadIdx.x; i < a.n; i += 256) t += a.A[(size_t)i * a.np + i];
  t = block_sum(t, scratch);
  if (threadIdx.x == 0) {
    a.stat[0] = t;
    a.stat[1] = 0.0;
    a.cnt[0] = a.cnt[1] = a.cnt[2] = 0;
  }
}

// A block sweep is one "inside" round, in which every block rotates the index pairs it contains, followed by the
// nb - 1 rounds of a round-robin over the blocks, in which a block pair (I, J) rotates the pairs (i in I, j in J):
// every index pair once per sweep, as in the element-wise cyclic method.  An instance keeps iterating while the
// previous sweep made at least one rotation.
struct InitRound {
  int nb, npairs, sweep, r;   // r = 0: inside round; r >= 1: round-robin round r - 1
  bool active;
};
__device__ __forceinline__ InitRound init_round(const InitArgs& a, int ground) {
  InitRound o;
  o.nb = a.np / kInitBlock;
  o.npairs = o.nb / 2;
  const int per_sweep = o.nb;
  o.sweep = ground / per_sweep;
  o.r = ground % per_sweep;
  o.active = o.sweep == 0 || a.cnt[(o.sweep + 2) % 3] != 0;
  return o;
}
// the two blocks that workgroup `pair` holds in this round
__device__ __forceinline__ void init_block_pair(const InitRound& rd, int pair, int& I, int& J) {
  if (rd.r == 0) {
    I = 2 * pair;
    J = 2 * pair + 1;
  } else {
    round_robin_pair(rd.nb, rd.r - 1, pair, I, J);
  }
}
// global index of local index l (0..63) of the blocks (I, J)
__device__ __forceinline__ int init_pair_index(int I, int J, int l) {
  return (l < kInitBlock ? I : J) * kInitBlock + (l & (kInitBlock - 1));
}
// index pair k (0..31) of inner round ir, as local indices (0..63) of the two blocks: inside round (31 inner
// rounds): pairs within the first block for k < 16, within the second otherwise; cross round (32 inner rounds):
// (k, 32 + (k + ir) % 32)
__device__ __forceinline__ void init_inner_pair(bool inside, int ir, int k, int& p, int& q) {
  if (inside) {
    const int off = k < kInitBlock / 2 ? 0 : kInitBlock;
    round_robin_pair(kInitBlock, ir, k & (kInitBlock / 2 - 1), p, q);
    p += off;
    q += off;
  } else {
    p = k;
    q = kInitBlock + ((k + ir) & (kInitBlock - 1));
  }
}

// The rotations of one round for the two blocks of a workgroup (31 or 32 inner rounds of 32 disjoint rotations) on
// their 64 x 64 sub-matrix, in LDS; the accumulated rotation goes to Q.  The first 32 threads compute an inner
// round's rotations (division-free); then thread t updates the 2 x 2 block (pair t / 32, pair t % 32) of the
// sub-matrix and two rows of Q's column pair t % 32; both are double-buffered, two barriers per inner round.
// Grid (pairs, count), 1024 threads, kInitSolveLds bytes of dynamic LDS.
__global__ __launch_bounds__(1024) void init_block_solve_kernel(const InitGroup* __restrict__ gp, const int ground) {
  const InitArgs& a = gp->a[blockIdx.y];
  const InitRound rd = init_round(a, ground);
  const int pair = blockIdx.x;
  // the counter of the next sweep is cleared whether or not this instance still iterates (nobody reads or adds to
  // it during this sweep), so that an instance that has converged stays so
  if (pair == 0 && rd.r == 0 && threadIdx.x == 0) a.cnt[(rd.sweep + 1) % 3] = 0;
  if (pair >= rd.npairs || !rd.active) return;   // uniform over the workgroup
  constexpr int P = kInitPair, LD = kInitPair + 1;
  extern __shared__ double dyn_init[];
  double* sA = dyn_init;                 // [2][P][LD]
  double* sQ = dyn_init + 2 * P * LD;    // [2][P][LD]
  __shared__ double scratch[16];
  __shared__ double s_c[kInitBlock], s_s[kInitBlock];
  const int tid = threadIdx.x, np = a.np;
  int I, J;
  init_block_pair(rd, pair, I, J);
  const bool inside = rd.r == 0;
  const int inner_rounds = inside ? kInitBlock - 1 : kInitBlock;
  for (int e = tid; e < P * P; e += 1024) {
    const int li = e >> 6, lj = e & 63;
    sA[li * LD + lj] = a.A[(size_t)init_pair_index(I, J, li) * np + init_pair_index(I, J, lj)];
    sQ[li * LD + lj] = li == lj ? 1.0 : 0.0;
  }
  __syncthreads();
  const double floor_abs = kInitCountFloor * a.stat[0];
  if (pair == 0 && rd.r == 0 && tid == 0) a.stat[1] = (double)(rd.sweep + 1);   // block sweeps this instance has run
  const int bi = tid >> 5, bj = tid & 31;
  int significant = 0;
  for (int ir = 0; ir < inner_rounds; ++ir) {
    const double* Ain = sA + (ir & 1) * P * LD;
    double* Aout = sA + ((ir & 1) ^ 1) * P * LD;
    const double* Qin = sQ + (ir & 1) * P * LD;
    double* Qout = sQ + ((ir & 1) ^ 1) * P * LD;
    if (tid < kInitBlock) {
      int p, q;
      init_inner_pair(inside, ir, tid, p, q);
      const double app = Ain[p * LD + p], aqq = Ain[q * LD + q], apq = Ain[p * LD + q];
      // Entries below the relative threshold are left: inside a cluster of (nearly) equal eigenvalues any
      // orthonormal basis serves, and rotating its small entries would only diagonalise the cluster's own
      // perturbation, sweep after sweep; across separated eigenvalues such an entry moves an eigenvector by less
      // than the threshold.  Entries at the level of the rounding noise are left as well.
      double c = 1.0, s = 0.0;
      if (fabs(apq) > kInitRotateTol * sqrt(fabs(app * aqq)) && fabs(apq) > floor_abs) {
        bool large;
        jacobi_rotation(app, aqq, apq, 0.0, c, s, large);
        ++significant;
      }
      s_c[tid] = c;
      s_s[tid] = s;
    }
    __syncthreads();
    int pi, qi, pj, qj;
    init_inner_pair(inside, ir, bi, pi, qi);
    init_inner_pair(inside, ir, bj, pj, qj);
    const double ci = s_c[bi], si = s_s[bi], cj = s_c[bj], sj = s_s[bj];
    const double x00 = Ain[pi * LD + pj], x01 = Ain[pi * LD + qj], x10 = Ain[qi * LD + pj], x11 = Ain[qi * LD + qj];
    const double y00 = ci * x00 - si * x10, y01 = ci * x01 - si * x11;
    const double y10 = si * x00 + ci * x10, y11 = si * x01 + ci * x11;
    double b00 = y00 * cj - y01 * sj, b01 = y00 * sj + y01 * cj;
    double b10 = y10 * cj - y11 * sj, b11 = y10 * sj + y11 * cj;
    if (bi == bj) b01 = b10 = 0.0;
    Aout[pi * LD + pj] = b00;
    Aout[pi * LD + qj] = b01;
    Aout[qi * LD + pj] = b10;
    Aout[qi * LD + qj] = b11;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int row = bi + 32 * h;
      const double u0 = Qin[row * LD + pj], u1 = Qin[row * LD + qj];
      Qout[row * LD + pj] = u0 * cj - u1 * sj;
      Qout[row * LD + qj] = u0 * sj + u1 * cj;
    }
    __syncthreads();
  }
  const double* Qfin = sQ + (inner_rounds & 1) * P * LD;
  double* Qg = a.Q + (size_t)pair * P * P;
  for (int e = tid; e < P * P; e += 1024) Qg[e] = Qfin[(e >> 6) * LD + (e & 63)];
  const double total = block_sum((double)significant, scratch);
  if (tid == 0 && total > 0.0) atomicAdd(&a.cnt[rd.sweep % 3], (int)total);
}

// Applies the round's rotations: A <- Q^T A Q on the 64 x 64 tile (workgroup x's blocks, workgroup y's blocks), or
// V <- V Q on the tile (64 rows, workgroup y's blocks), in place (a tile depends on itself only).
// Grid (pairs + row chunks, pairs, count), 256 threads: wavefront w owns the 32 x 32 quadrant (w / 2, w % 2).
// v_mfma_f64_16x16x4_f64: lane l supplies A[l%16][l/16] and B[l/16][l%16]; register r holds row 4r + l/16, column l%16.
__global__ __launch_bounds__(256) void init_block_apply_kernel(const InitGroup* __restrict__ gp, const int ground, const int pairs_max) {
  const InitArgs& a = gp->a[blockIdx.z];
  const InitRound rd = init_round(a, ground);
  const int pb = blockIdx.y;
  const bool is_v = (int)blockIdx.x >= pairs_max;
  const int pa = is_v ? 0 : blockIdx.x, chunk = is_v ? (int)blockIdx.x - pairs_max : 0;
  if (!rd.active || pb >= rd.npairs) return;                                   // uniform over the workgroup
  if (is_v ? chunk * kInitPair >= a.np : pa >= rd.npairs) return;
  constexpr int P = kInitPair, LD = kInitPair + 1;
  __shared__ double sT[P][LD];
  typedef double doublex4 __attribute__((ext_vector_type(4)));
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, g4 = lane >> 4;
  const int qi = wave >> 1, qj = wave & 1;
  const int np = a.np;
  int Ia = 0, Ja = 0, Ib, Jb;
  init_block_pair(rd, pb, Ib, Jb);
  if (!is_v) init_block_pair(rd, pa, Ia, Ja);
  double* __restrict__ X = is_v ? a.V : a.A;
  const double* __restrict__ Qb = a.Q + (size_t)pb * P * P;
  auto grow = [&](const int l) { return is_v ? chunk * P + l : init_pair_index(Ia, Ja, l); };   // row of the tile's row l
  int gcol[2];
#pragma unroll
  for (int nj = 0; nj < 2; ++nj) gcol[nj] = init_pair_index(Ib, Jb, qj * 32 + nj * 16 + l16);

  if (is_v) {
    // the tile itself is the left factor
    for (int e = tid; e < P * P; e += 256) {
      const int lr = e >> 6, lc = e & 63;
      sT[lr][lc] = X[(size_t)grow(lr) * np + init_pair_index(Ib, Jb, lc)];
    }
  } else {
    // T = Q_a^T (tile): this wavefront's quadrant, K = 64
    const double* __restrict__ Qa = a.Q + (size_t)pa * P * P;
    doublex4 t[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int nj = 0; nj < 2; ++nj) t[mi][nj] = doublex4{0, 0, 0, 0};
#pragma unroll 4
    for (int ks = 0; ks < P / 4; ++ks) {
      const int k = ks * 4 + g4;
      double af[2], bf[2];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi) af[mi] = Qa[k * P + qi * 32 + mi * 16 + l16];
      const size_t xrow = (size_t)grow(k) * np;
#pragma unroll
      for (int nj = 0; nj < 2; ++nj) bf[nj] = X[xrow + gcol[nj]];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int nj = 0; nj < 2; ++nj)
          t[mi][nj] = __builtin_amdgcn_mfma_f64_16x16x4f64(af[mi], bf[nj], t[mi][nj], 0, 0, 0);
    }
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int nj = 0; nj < 2; ++nj)
#pragma unroll
        for (int r = 0; r < 4; ++r) sT[qi * 32 + mi * 16 + 4 * r + g4][qj * 32 + nj * 16 + l16] = t[mi][nj][r];
  }
  __syncthreads();   // every wavefront has read what it needs of the tile: it may be overwritten now
  // (left factor) Q_b
  doublex4 acc[2][2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int nj = 0; nj < 2; ++nj) acc[mi][nj] = doublex4{0, 0, 0, 0};
#pragma unroll 4
  for (int ks = 0; ks < P / 4; ++ks) {
    const int k = ks * 4 + g4;
    double af[2], bf[2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi) af[mi] = sT[qi * 32 + mi * 16 + l16][k];
#pragma unroll
    for (int nj = 0; nj < 2; ++nj) bf[nj] = Qb[k * P + qj * 32 + nj * 16 + l16];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int nj = 0; nj < 2; ++nj)
        acc[mi][nj] = __builtin_amdgcn_mfma_f64_16x16x4f64(af[mi], bf[nj], acc[mi][nj], 0, 0, 0);
  }
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const size_t xrow = (size_t)grow(qi * 32 + mi * 16 + 4 * r + g4) * np;
#pragma unroll
      for (int nj = 0; nj < 2; ++nj) X[xrow + gcol[nj]] = acc[mi][nj][r];
    }
}

// Top-R eigenvalues, rho_0, D_0, E_0 (App. B.3.2 with eq. beta2, etii).  One workgroup per instance.
__global__ __launch_bounds__(1024) void init_select_kernel(const InitGroup* __restrict__ gp) {
  __shared__ double scratch[16];
  __shared__ double s_lam[kMaxRank];
  __shared__ int s_idx[kMaxRank];
  const InitArgs& a = gp->a[blockIdx.x];
  const int n = a.n, R = a.R, D = a.D;
  const size_t lda = a.np;
  const double* A = a.A;
  PrecondScalars* st = a.st;
  double tr = 0.0;
  for (int i = threadIdx.x; i < n; i += blockDim.x) tr += A[i * lda + i];
  tr = block_sum(tr, scratch);
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    const double li = A[i * lda + i];
    int rank = 0;
    for (int j = 0; j < n; ++j) {
      const double lj = A[j * lda + j];
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
    const double rho0 = fmax((tr - sum_l) / (double)(D - R), gp->epsilon);
    double sum_d = 0.0;
    for (int k = 0; k < R; ++k) {
      const double d = fmax(gp->epsilon, s_lam[k] - rho0);
      st->d[k] = d;
      sum_d += d;
    }
    const double beta = rho0 * (1.0 + gp->alpha) + gp->alpha / (double)D * sum_d;
    for (int k = 0; k < R; ++k) st->e[k] = 1.0 / (beta / st->d[k] + 1.0);
    st->rho = rho0;
    st->beta = beta;
    st->trace_S0 = tr;
    st->flags = a.cnt[((int)a.stat[1] + 2) % 3] != 0 ? kFlagNoConverge : 0;   // the last sweep run still rotated
    st->sweeps = (int)a.stat[1];   // block sweeps of the initial eigen-decomposition
    // eigenvalue kept for the Gram route's 1/sqrt(N lambda); parked in gamma/tr fields is not possible: use vwork
    for (int k = 0; k < R; ++k) {
      a.idx[k] = s_idx[k];
      a.vwork[k] = s_lam[k];
    }
  }
}

// W_0 rows of the kept eigenpairs: sqrt(e_i) v_i with v_i a column of V (covariance route) or
// X_0^T u_i / sqrt(N lambda_i) (Gram route); zero for null directions.  Grid (col blocks of 64, R, instance).
__global__ __launch_bounds__(256) void init_rows_kernel(const InitGroup* __restrict__ gp) {
  const InitArgs& a = gp->a[blockIdx.z];
  const int i = blockIdx.y;
  if (i >= a.R) return;
  const int col = blockIdx.x * 64 + (threadIdx.x & 63);
  const int part = threadIdx.x >> 6;   // 4 slices of the row range
  if ((int)blockIdx.x * 64 >= a.ldw) return;
  __shared__ double s_acc[4][64];
  const int src_col = a.idx[i];
  const double* V = a.V;
  const int n = a.np;   // leading dimension of V
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
// One workgroup per instance; returns at once when every direction was kept.  A pass takes all its inner
// products against the same vector (every wavefront a share of the fixed rows) and then subtracts them together.
__global__ __launch_bounds__(1024) void init_complete_kernel(const InitGroup* __restrict__ gp) {
  __shared__ double scratch[16];
  __shared__ int s_fixed[kMaxRank];
  __shared__ double s_dot[kMaxRank], s_inv[kMaxRank];
  __shared__ int s_nfixed, s_missing;
  const InitArgs& a = gp->a[blockIdx.x];
  const int R = a.R, D = a.D, ldw = a.ldw;
  const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
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
  for (int k = tid; k < R; k += nt) s_inv[k] = 1.0 / sqrt(st->e[k]);   // rows of W are sqrt(e) times rows of R_0
  __syncthreads();
  int cand = 0;
  for (int i = 0; i < R; ++i) {
    if (a.idx[i] >= 0) continue;    // uniform
    bool accepted = false;
    while (!accepted && cand < D) {
      for (int c = tid; c < D; c += nt) v[c] = c == cand ? 1.0 : 0.0;
      ++cand;
      __syncthreads();
      const int nf = s_nfixed;
      for (int pass = 0; pass < 2; ++pass) {
        for (int f = wave; f < nf; f += nw) {
          const int j = s_fixed[f];
          const float* wj = W + (size_t)j * ldw;
          double dot = 0.0;
          for (int c = lane; c < D; c += 64) dot += (double)wj[c] * v[c];
          dot = wave_sum(dot);
          if (lane == 0) s_dot[f] = dot * s_inv[j];
        }
        __syncthreads();
        for (int c = tid; c < D; c += nt) {
          double x = v[c];
          for (int f = 0; f < nf; ++f) {
            const int j = s_fixed[f];
            x -= s_dot[f] * (double)W[(size_t)j * ldw + c] * s_inv[j];
          }
          v[c] = x;
        }
        __syncthreads();
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
