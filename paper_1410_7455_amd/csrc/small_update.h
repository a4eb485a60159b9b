// The R x R part of the online natural-gradient update, entirely on the device (App. B.3, B.3.1).
//
// One workgroup per instance holds Z_t and the eigenvector matrix in LDS (fp64) and runs a cyclic
// Jacobi eigen-solver with a round-robin ordering: every round applies floor(R/2) disjoint plane
// rotations, each thread updating whole 2x2 blocks, so a round costs two barriers.  Z_t is close to
// diagonal once the factor tracks the data (the rows of Y_t are then nearly eigenvectors scaled by
// their eigenvalues), so a few sweeps suffice.
#pragma once

#include <hip/hip_runtime.h>

#include "kernels.h"
#include "state.h"

namespace ngsgd {

constexpr int kSmallThreads = 1024;
constexpr int kMaxSweeps = 30;
constexpr double kJacobiTol = 1.0e-13;       // a pair is left alone once |z_pq| <= tol * sqrt(z_pp z_qq)
constexpr double kJacobiAbsTol = 1.0e-15;    // ... or once |z_pq| <= this * max_i z_ii (rounding noise level)
constexpr double kOrthoCondLimit = 1.0e6;    // App. B.3.1
constexpr double kOrthoTolerance = 1.0e-3;   // App. B.3.1

struct SmallArgs {
  PrecondScalars* st;
  double* K;         // R x R, J J^T; cleared on exit (the orthogonality check accumulates W W^T into it)
  const double* L;   // R x R, H^T H
  float* At;         // out: A_t (eq. wt1), R x ldat
  int ldat;
  int R, D, N;
};
struct SmallGroup {
  int count;
  double alpha, epsilon, num_samples_history;
  SmallArgs a[kMaxInstances];
};

// Rotation that diagonalises [[app, apq], [apq, aqq]] as J^T A J with J = [[c, s], [-s, c]].  Returns false (and
// the identity) when the off-diagonal entry is already negligible relative to the diagonal pair; that relative
// test is what gives small eigenvalues of a graded positive definite matrix their relative accuracy.
__device__ __forceinline__ bool sym_schur2(double app, double aqq, double apq, double& c, double& s,
                                           double abs_tol = 0.0) {
  c = 1.0;
  s = 0.0;
  if (!(fabs(apq) > fmax(kJacobiTol * sqrt(fabs(app * aqq)), abs_tol)) || fabs(apq) <= 1.0e-300) return false;
  const double tau = (aqq - app) / (2.0 * apq);
  const double t = (tau >= 0.0 ? 1.0 : -1.0) / (fabs(tau) + sqrt(1.0 + tau * tau));
  c = 1.0 / sqrt(1.0 + t * t);
  s = t * c;
  return true;
}

// Round-robin pairing of m (even) players: in round r, pair k is (m-1, r) for k = 0 and
// ((r+k) mod (m-1), (r-k) mod (m-1)) otherwise; over rounds 0..m-2 every pair meets once.
__device__ __forceinline__ void round_robin_pair(int m, int r, int k, int& p, int& q) {
  if (k == 0) {
    p = r;
    q = m - 1;
  } else {
    p = (r + k) % (m - 1);
    q = (r - k + (m - 1)) % (m - 1);
  }
  if (p > q) {
    const int t = p;
    p = q;
    q = t;
  }
}

__global__ __launch_bounds__(kSmallThreads) void small_update_kernel(const SmallGroup g) {
  extern __shared__ __attribute__((aligned(16))) double dyn[];
  __shared__ double scratch[16];
  __shared__ double s_d[kMaxRank], s_ise[kMaxRank], s_dr[kMaxRank], s_c[kMaxRank], s_enew[kMaxRank];
  __shared__ double s_cs[kMaxRank / 2 + 1], s_sn[kMaxRank / 2 + 1];
  __shared__ int s_p[kMaxRank / 2 + 1], s_q[kMaxRank / 2 + 1], s_perm[kMaxRank];
  __shared__ double s_scal[8];
  __shared__ int s_flag[2];
  __shared__ int s_rotations;

  const SmallArgs& a = g.a[blockIdx.x];
  const int R = a.R, D = a.D, N = a.N;
  const int tid = threadIdx.x, nt = blockDim.x;
  const int Rs = R | 1;                       // odd row stride
  double* Z = dyn;
  double* U = dyn + (size_t)R * Rs;
  PrecondScalars* st = a.st;

  const double eta = 1.0 - exp(-(double)N / g.num_samples_history);   // eq. eta:ns
  const double rho = st->rho;
  if (tid < R) s_d[tid] = st->d[tid];
  __syncthreads();
  if (tid == 0) {
    double sum_d = 0.0;
    for (int i = 0; i < R; ++i) sum_d += s_d[i];
    s_scal[0] = sum_d;
    s_scal[1] = rho * (1.0 + g.alpha) + g.alpha / (double)D * sum_d;  // beta_t, eq. beta2
  }
  __syncthreads();
  const double sum_d = s_scal[0], beta = s_scal[1];
  if (tid < R) {
    const double e = 1.0 / (beta / s_d[tid] + 1.0);                   // eq. etii
    s_ise[tid] = 1.0 / sqrt(e);
    s_dr[tid] = s_d[tid] + rho;
  }
  __syncthreads();

  // Z_t from K_t and L_t (eq. zt:compute), symmetrised; U = I
  const double ck = (eta / N) * (eta / N), cl = eta * (1.0 - eta) / N;
  for (int idx = tid; idx < R * R; idx += nt) {
    const int i = idx / R, j = idx % R;
    const double kij = 0.5 * (a.K[i * R + j] + a.K[j * R + i]);
    const double lij = 0.5 * (a.L[i * R + j] + a.L[j * R + i]);
    double z = (ck * kij + cl * lij * (s_dr[i] + s_dr[j])) * s_ise[i] * s_ise[j];
    if (i == j) z += (1.0 - eta) * (1.0 - eta) * s_dr[i] * s_dr[i];
    Z[i * Rs + j] = z;
    U[i * Rs + j] = i == j ? 1.0 : 0.0;
  }
  __syncthreads();

  // cyclic Jacobi, Z = U C U^T; a sweep in which no pair needed a rotation ends the iteration
  double zmax = 0.0;
  for (int i = tid; i < R; i += nt) zmax = fmax(zmax, Z[i * Rs + i]);
  const double abs_tol = kJacobiAbsTol * block_max(zmax, scratch);
  const int m = (R + 1) & ~1;
  const int half = m / 2;
  int sweeps = 0;
  bool converged = false;
  for (; sweeps < kMaxSweeps; ++sweeps) {
    if (tid == 0) s_rotations = 0;
    __syncthreads();
    for (int r = 0; r < m - 1; ++r) {
      if (tid < half) {
        int p, q;
        round_robin_pair(m, r, tid, p, q);
        double c = 1.0, s = 0.0;
        if (q < R && sym_schur2(Z[p * Rs + p], Z[q * Rs + q], Z[p * Rs + q], c, s, abs_tol))
          atomicAdd(&s_rotations, 1);
        s_p[tid] = p;
        s_q[tid] = q;
        s_cs[tid] = c;
        s_sn[tid] = s;
      }
      __syncthreads();
      for (int blk = tid; blk < half * half; blk += nt) {
        const int bi = blk / half, bj = blk % half;
        const int pi = s_p[bi], qi = s_q[bi], pj = s_p[bj], qj = s_q[bj];
        if (s_sn[bi] == 0.0 && s_sn[bj] == 0.0) continue;   // both rotations are the identity
        if (qi >= R || qj >= R) {
          // a pair with the padding index: only the real member's row/column takes part
          if (qi >= R && qj >= R) continue;
          if (qi >= R) {        // row pi unchanged by the row rotation; apply column rotation of pair bj
            const double cj = s_cs[bj], sj = s_sn[bj];
            const double x0 = Z[pi * Rs + pj], x1 = Z[pi * Rs + qj];
            Z[pi * Rs + pj] = x0 * cj - x1 * sj;
            Z[pi * Rs + qj] = x0 * sj + x1 * cj;
          } else {              // column pj unchanged; apply row rotation of pair bi
            const double ci = s_cs[bi], si = s_sn[bi];
            const double x0 = Z[pi * Rs + pj], x1 = Z[qi * Rs + pj];
            Z[pi * Rs + pj] = ci * x0 - si * x1;
            Z[qi * Rs + pj] = si * x0 + ci * x1;
          }
          continue;
        }
        const double ci = s_cs[bi], si = s_sn[bi], cj = s_cs[bj], sj = s_sn[bj];
        const double x00 = Z[pi * Rs + pj], x01 = Z[pi * Rs + qj];
        const double x10 = Z[qi * Rs + pj], x11 = Z[qi * Rs + qj];
        const double y00 = ci * x00 - si * x10, y01 = ci * x01 - si * x11;
        const double y10 = si * x00 + ci * x10, y11 = si * x01 + ci * x11;
        double b00 = y00 * cj - y01 * sj, b01 = y00 * sj + y01 * cj;
        double b10 = y10 * cj - y11 * sj, b11 = y10 * sj + y11 * cj;
        if (bi == bj) b01 = b10 = 0.0;      // the rotated pair itself is annihilated exactly
        Z[pi * Rs + pj] = b00;
        Z[pi * Rs + qj] = b01;
        Z[qi * Rs + pj] = b10;
        Z[qi * Rs + qj] = b11;
      }
      for (int idx = tid; idx < R * half; idx += nt) {
        const int row = idx / half, bj = idx % half;
        const int pj = s_p[bj], qj = s_q[bj];
        const double cj = s_cs[bj], sj = s_sn[bj];
        if (qj >= R || sj == 0.0) continue;
        const double u0 = U[row * Rs + pj], u1 = U[row * Rs + qj];
        U[row * Rs + pj] = u0 * cj - u1 * sj;
        U[row * Rs + qj] = u0 * sj + u1 * cj;
      }
      __syncthreads();
    }
    if (s_rotations == 0) {   // same value for every thread: read after the round's closing barrier
      converged = true;
      ++sweeps;
      break;
    }
    __syncthreads();          // everyone has read the counter before it is cleared again
  }

  // eigenvalues, floor (after eq. zt:eig:repeat), decreasing order
  const double floor_c = (1.0 - eta) * (1.0 - eta) * rho * rho;
  if (tid == 0) s_flag[0] = 0;
  __syncthreads();
  if (tid < R) {
    double c = Z[tid * Rs + tid];
    if (!(c >= floor_c)) {
      c = floor_c;
      atomicOr(&s_flag[0], 1);
    }
    s_c[tid] = c;
  }
  __syncthreads();
  if (tid < R) {
    int rank = 0;
    const double c = s_c[tid];
    for (int j = 0; j < R; ++j) rank += (s_c[j] > c || (s_c[j] == c && j < tid)) ? 1 : 0;
    s_perm[rank] = tid;   // s_perm[k] = index of the k-th largest eigenvalue
  }
  __syncthreads();
  if (tid == 0) {
    double sum_sqrt = 0.0;
    for (int i = 0; i < R; ++i) sum_sqrt += sqrt(s_c[i]);
    // eq. rhodash2, dt1, rhot1
    const double rho_dash = ((eta / N) * st->tr_M + (1.0 - eta) * ((double)D * rho + sum_d) - sum_sqrt) / (double)(D - R);
    const double rho_new = fmax(g.epsilon, rho_dash);
    double sum_dn = 0.0;
    for (int k = 0; k < R; ++k) {
      const double dn = fmax(sqrt(s_c[s_perm[k]]) - rho_dash, g.epsilon);
      s_enew[k] = dn;     // temporarily d_{t+1}
      sum_dn += dn;
    }
    const double beta_new = rho_new * (1.0 + g.alpha) + g.alpha / (double)D * sum_dn;
    s_scal[2] = rho_new;
    s_scal[3] = beta_new;
    const double cmax = s_c[s_perm[0]], cmin = s_c[s_perm[R - 1]];
    int flags = 0;
    if (s_flag[0]) flags |= kFlagFloored | kFlagOrthCheck;
    if (cmax > kOrthoCondLimit * cmin) flags |= kFlagOrthCheck;
    if (!converged) flags |= kFlagNoConverge;
    st->flags = flags;
    st->sweeps = sweeps;
    st->rho = rho_new;
    st->beta = beta_new;
  }
  __syncthreads();
  const double beta_new = s_scal[3];
  double en = 0.0;
  if (tid < R) {
    const double dn = s_enew[tid];
    en = 1.0 / (beta_new / dn + 1.0);
    st->d[tid] = dn;
    st->e[tid] = en;
  }
  __syncthreads();
  if (tid < R) s_enew[tid] = en;   // from here on e_{t+1}
  __syncthreads();
  // A_t = (eta/N) E_{t+1}^{1/2} C_t^{-1/2} U_t^T E_t^{-1/2}   (eq. wt1), rows in decreasing-eigenvalue order
  for (int idx = tid; idx < R * a.ldat; idx += nt) {
    const int k = idx / a.ldat, j = idx % a.ldat;
    float v = 0.f;
    if (j < R) {
      const int src = s_perm[k];
      v = (float)((eta / N) * sqrt(s_enew[k] / s_c[src]) * U[j * Rs + src] * s_ise[j]);
    }
    a.At[(size_t)k * a.ldat + j] = v;
  }
  for (int idx = tid; idx < R * R; idx += nt) a.K[idx] = 0.0;
}

// App. B.3.1 on the new factor: O = E^{-1/2} (W W^T) E^{-1/2}; if any entry is off the identity by more than
// 1e-3, W <- E^{1/2} L^{-1} E^{-1/2} W with O = L L^T.  Runs only when the update asked for the check.
struct OrthArgs {
  PrecondScalars* st;
  const double* G;   // R x R, W W^T of the new factor (accumulated only when the check was requested)
  float* W;
  int ld;
  int R, D;
};
struct OrthGroup {
  int count;
  OrthArgs a[kMaxInstances];
};

__global__ __launch_bounds__(kSmallThreads) void orth_fix_kernel(const OrthGroup g) {
  extern __shared__ __attribute__((aligned(16))) double dyn[];
  __shared__ double scratch[16];
  const OrthArgs& a = g.a[blockIdx.x];
  PrecondScalars* st = a.st;
  if (!(st->flags & kFlagOrthCheck)) return;   // uniform over the workgroup
  const int R = a.R, D = a.D, ld = a.ld;
  const int tid = threadIdx.x, nt = blockDim.x;
  const int Rs = R | 1;
  double* O = dyn;                    // R x Rs, becomes L
  double* X = dyn + (size_t)R * Rs;   // R x Rs, L^{-1} then the mixing matrix

  double dev = 0.0;
  for (int idx = tid; idx < R * R; idx += nt) {
    const int i = idx / R, j = idx % R;
    if (j <= i) {
      const double s = 0.5 * (a.G[i * R + j] + a.G[j * R + i]) / sqrt(st->e[i] * st->e[j]);
      O[i * Rs + j] = s;
      dev = fmax(dev, fabs(s - (i == j ? 1.0 : 0.0)));
    }
  }
  dev = block_max(dev, scratch);
  if (!(dev > kOrthoTolerance)) {
    __syncthreads();
    if (tid == 0) st->flags &= ~kFlagOrthCheck;
    return;
  }
  __syncthreads();
  // Cholesky O = L L^T in place (lower triangle), one column at a time
  for (int j = 0; j < R; ++j) {
    if (tid == 0) {
      double s = O[j * Rs + j];
      for (int k = 0; k < j; ++k) s -= O[j * Rs + k] * O[j * Rs + k];
      O[j * Rs + j] = sqrt(fmax(s, 1.0e-300));
    }
    __syncthreads();
    for (int i = j + 1 + tid; i < R; i += nt) {
      double s = O[i * Rs + j];
      for (int k = 0; k < j; ++k) s -= O[i * Rs + k] * O[j * Rs + k];
      O[i * Rs + j] = s / O[j * Rs + j];
    }
    __syncthreads();
  }
  // X = L^{-1} by forward substitution, one column per thread
  for (int c = tid; c < R; c += nt) {
    for (int i = 0; i < R; ++i) {
      double s = i == c ? 1.0 : 0.0;
      for (int k = c; k < i; ++k) s -= O[i * Rs + k] * X[k * Rs + c];
      X[i * Rs + c] = i < c ? 0.0 : s / O[i * Rs + i];
    }
  }
  __syncthreads();
  for (int idx = tid; idx < R * R; idx += nt) {
    const int i = idx / R, j = idx % R;
    X[i * Rs + j] *= sqrt(st->e[i] / st->e[j]);
  }
  __syncthreads();
  // W <- X W, X lower triangular: rows from last to first so the product can be formed in place
  float* Wm = a.W;
  for (int c = tid; c < D; c += nt) {
    for (int i = R - 1; i >= 0; --i) {
      double s = 0.0;
      for (int k = 0; k <= i; ++k) s += X[i * Rs + k] * (double)Wm[(size_t)k * ld + c];
      Wm[(size_t)i * ld + c] = (float)s;
    }
  }
  __syncthreads();
  if (tid == 0) st->flags = (st->flags & ~kFlagOrthCheck) | kFlagReorth;
}

}  // namespace ngsgd
