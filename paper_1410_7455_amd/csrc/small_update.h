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

constexpr int kSmallThreads = 1024;          // orthogonality fix kernel
constexpr int kEigThreads = 1024;            // R x R eigen-update kernel

constexpr int kEigvecThreads = 256;          // eigenvector kernel: 4 wavefronts, one row of U each
constexpr int kEigvecChunk = 32;             // rounds of the rotation log staged in LDS at a time
constexpr int kMaxSweeps = 20;
constexpr int kMaxHalf = kMaxRank / 2;
constexpr int kMaxRounds = kMaxSweeps * (kMaxRank - 1);
constexpr double kJacobiTol = 1.0e-13;       // a pair is left alone once |z_pq| <= tol * sqrt(z_pp z_qq)
constexpr double kJacobiAbsTol = 1.0e-13;    // ... or once |z_pq| <= this * max_i z_ii (rounding noise level)
constexpr double kOrthoCondLimit = 1.0e6;    // App. B.3.1
constexpr double kOrthoTolerance = 1.0e-3;   // App. B.3.1

// What the eigen-update kernel leaves for the eigenvector kernel (device memory, per instance).
struct EigWork {
  int n_rounds;                  // Jacobi rounds executed (rotation log length / half)
  int pad;
  int rank_of[kMaxRank];         // position of eigenpair i in decreasing-eigenvalue order
  double colscale[kMaxRank];     // (eta/N) sqrt(e_{t+1,k} / c_i) for eigenpair i at position k
  double rowscale[kMaxRank];     // e_{t,j}^{-1/2}
};

struct SmallArgs {
  PrecondScalars* st;
  double* K;         // R x R, J J^T; cleared on exit (the orthogonality check accumulates W W^T into it)
  const double* L;   // R x R, H^T H
  float* At;         // out: A_t (eq. wt1), R x ldat (written by the eigenvector kernel)
  int ldat;
  int R, D, N;
  double2* rotlog;   // [kMaxRounds][half] (c, s) of every pair of every round
  EigWork* work;
};
struct SmallGroup {
  int count;
  double alpha, epsilon, num_samples_history;
  SmallArgs a[kMaxInstances];
};

__device__ __forceinline__ double fast_rsqrt(double x) {
  double y = __builtin_amdgcn_rsq(x);
  y = y * (1.5 - 0.5 * x * y * y);
  y = y * (1.5 - 0.5 * x * y * y);
  return y;
}
__device__ __forceinline__ double fast_rcp(double x) {
  double r = __builtin_amdgcn_rcp(x);
  r = r * (2.0 - x * r);
  r = r * (2.0 - x * r);
  return r;
}

// Rotation that diagonalises [[app, apq], [apq, aqq]] as J^T A J with J = [[c, s], [-s, c]].  Returns false (and
// the identity) when the off-diagonal entry is already negligible: relative to the diagonal pair (that relative
// test is what gives small eigenvalues of a graded positive definite matrix their relative accuracy) or in
// absolute terms (abs_tol2 is the squared absolute threshold).  Division and square roots go through the
// hardware reciprocal estimates plus Newton steps: the rotation sits on the critical path of every round.
__device__ __forceinline__ bool jacobi_rotation(double app, double aqq, double apq, double abs_tol2, double& c,
                                                double& s) {
  c = 1.0;
  s = 0.0;
  const double apq2 = apq * apq;
  if (!(apq2 > kJacobiTol * kJacobiTol * fabs(app * aqq)) || !(apq2 > abs_tol2) || !(apq2 > 1.0e-290)) return false;
  const double h = 0.5 * (aqq - app);
  const double x = h * h + apq2;
  const double r = x * fast_rsqrt(x);
  const double t = apq * fast_rcp(h + (h >= 0.0 ? r : -r));
  c = fast_rsqrt(1.0 + t * t);
  s = t * c;
  return true;
}

// Exact variant used by the (not latency critical) initialisation.
__device__ __forceinline__ bool sym_schur2(double app, double aqq, double apq, double& c, double& s) {
  c = 1.0;
  s = 0.0;
  if (!(fabs(apq) > kJacobiTol * sqrt(fabs(app * aqq))) || fabs(apq) <= 1.0e-300) return false;
  const double tau = (aqq - app) / (2.0 * apq);
  const double t = (tau >= 0.0 ? 1.0 : -1.0) / (fabs(tau) + sqrt(1.0 + tau * tau));
  c = 1.0 / sqrt(1.0 + t * t);
  s = t * c;
  return true;
}

// Round-robin pairing of m (even) players: in round r, pair k is (m-1, r) for k = 0 and
// ((r+k) mod (m-1), (r-k) mod (m-1)) otherwise; over rounds 0..m-2 every pair meets once.  Returned with p < q.
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

// The Jacobi iteration works in "position space" (Brent-Luk): position 2k is the first and 2k+1 the second
// member of pair k, rotations always act on (2k, 2k+1), and after every round the matrix is permuted so that the
// next round's partners sit together again.  The permutation is the same every round,
//   first_k -> first_{k-1} (k >= 1),  first_0 -> second_1,  second_k -> second_{k+1} (1 <= k < half-1),
//   second_{half-1} -> first_{half-1},  second_0 stays,
// which is the circle method of a round-robin tournament with `second_0` as the fixed player: over m-1 rounds
// every two players meet once.  Because it is fixed, every thread reads and writes the same LDS addresses in
// every round and needs no index arithmetic in the loop.
__device__ __forceinline__ int next_position(int pos, int half) {
  if (half == 1) return pos;
  const int k = pos >> 1;
  if ((pos & 1) == 0) return k >= 1 ? 2 * (k - 1) : 3;          // first members
  if (k == 0) return 1;                                          // the fixed player
  return k == half - 1 ? 2 * (half - 1) : 2 * (k + 1) + 1;       // second members
}
// Player standing at `pos` after `rounds` rounds; players m-1-k start as second members, m-1 is the fixed one.
__device__ __forceinline__ int player_at(int pos, int rounds, int m) {
  const int k = pos >> 1;
  if (m == 2) return pos;
  const int r = rounds % (m - 1);
  if ((pos & 1) == 0) return (r + k) % (m - 1);
  return k == 0 ? m - 1 : (r - k + (m - 1)) % (m - 1);
}

// Z_t (eq. zt:compute), its eigenvalues by cyclic Jacobi, then rho_{t+1}, D_{t+1}, E_{t+1} (eq. rhodash2, dt1,
// rhot1, beta2, etii).  One workgroup per instance.  Only Z is rotated here (upper triangle in position space,
// two LDS copies used alternately); every rotation is logged, and the eigenvector kernel replays the log on the
// rows of the identity.  A round is: wave 0 computes the half rotations | barrier | every thread rotates its
// 2x2 blocks from one copy into their next positions in the other copy | barrier.
template <int ITEMS>
__global__ __launch_bounds__(kEigThreads) void eig_update_kernel(const SmallGroup g) {
  extern __shared__ __attribute__((aligned(16))) double dyn[];   // two copies of Z, m x ms, entries (a <= b) live
  __shared__ double scratch[16];
  __shared__ double s_d[kMaxRank], s_ise[kMaxRank], s_dr[kMaxRank], s_c[kMaxRank + 1], s_enew[kMaxRank];
  __shared__ double2 s_rot[kMaxHalf];
  __shared__ int s_perm[kMaxRank];
  __shared__ double s_scal[8];
  __shared__ int s_flag[2];
  __shared__ int s_rotated;

  const SmallArgs& a = g.a[blockIdx.x];
  const int R = a.R, D = a.D, N = a.N;
  const int tid = threadIdx.x;
  constexpr int nt = kEigThreads;
  const int m = (R + 1) & ~1;
  const int half = m / 2;
  const int ms = m;   // even row stride: the two entries (a, 2k), (a, 2k+1) of a block row are one aligned 16 bytes
  const int zcopy = m * ms;   // offset of the second copy (offsets, not pointers: the accesses stay LDS instructions)
  PrecondScalars* st = a.st;

  const double eta = 1.0 - exp(-(double)N / g.num_samples_history);   // eq. eta:ns
  const double rho = st->rho;
  for (int i = tid; i < R; i += nt) s_d[i] = st->d[i];
  __syncthreads();
  if (tid == 0) {
    double sum_d = 0.0;
    for (int i = 0; i < R; ++i) sum_d += s_d[i];
    s_scal[0] = sum_d;
    s_scal[1] = rho * (1.0 + g.alpha) + g.alpha / (double)D * sum_d;  // beta_t, eq. beta2
  }
  __syncthreads();
  const double sum_d = s_scal[0], beta = s_scal[1];
  for (int i = tid; i < R; i += nt) {
    const double e = 1.0 / (beta / s_d[i] + 1.0);                     // eq. etii
    s_ise[i] = 1.0 / sqrt(e);
    s_dr[i] = s_d[i] + rho;
  }
  __syncthreads();

  // Z_t from K_t and L_t (eq. zt:compute), symmetrised, laid out by position; the padding player of an odd R has
  // an all-zero row and column and is never rotated
  const double ck = (eta / N) * (eta / N), cl = eta * (1.0 - eta) / N;
  double zmax = 0.0;
  for (int idx = tid; idx < m * m; idx += nt) {
    const int pa = idx / m, pb = idx % m;
    if (pa > pb) continue;
    const int i = player_at(pa, 0, m), j = player_at(pb, 0, m);
    double z = 0.0;
    if (i < R && j < R) {
      const double kij = 0.5 * (a.K[i * R + j] + a.K[j * R + i]);
      const double lij = 0.5 * (a.L[i * R + j] + a.L[j * R + i]);
      z = (ck * kij + cl * lij * (s_dr[i] + s_dr[j])) * s_ise[i] * s_ise[j];
      if (i == j) {
        z += (1.0 - eta) * (1.0 - eta) * s_dr[i] * s_dr[i];
        zmax = fmax(zmax, z);
      }
    }
    dyn[pa * ms + pb] = z;
  }
  zmax = block_max(zmax, scratch);
  const double abs_tol = kJacobiAbsTol * zmax;
  const double abs_tol2 = abs_tol * abs_tol;

  // the blocks (bi <= bj) this thread owns, numbered row by row so that neighbouring lanes read neighbouring
  // 16-byte pieces: fixed source rows (two double2 loads) and destination offsets of their four entries
  const int n_blocks = half * (half + 1) / 2;
  int blk_i[ITEMS], blk_j[ITEMS];
  int src[ITEMS][2], dst[ITEMS][4];
#pragma unroll
  for (int it = 0; it < ITEMS; ++it) {
    const int item = tid + it * nt;
    int bi = 0, rem = item < n_blocks ? item : 0;
    while (rem >= half - bi) {   // row bi holds the blocks (bi, bi), (bi, bi+1), ..., (bi, half-1)
      rem -= half - bi;
      ++bi;
    }
    const int bj = bi + rem;
    blk_i[it] = bi;
    blk_j[it] = bj;
    src[it][0] = (2 * bi) * ms + 2 * bj;
    src[it][1] = (2 * bi + 1) * ms + 2 * bj;   // its first entry lies below the diagonal when bi == bj: ignored
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int na = next_position(2 * bi + (e >> 1), half), nb = next_position(2 * bj + (e & 1), half);
      dst[it][e] = na <= nb ? na * ms + nb : nb * ms + na;
    }
  }
  const bool odd_pad = (R & 1) != 0;   // pair 0 then holds the padding player
  if (tid == 0) s_rotated = 0;
  __syncthreads();

  // cyclic Jacobi; a sweep in which no pair needed a rotation ends the iteration
  int sweeps = 0, rounds = 0, cur = 0;
  bool converged = false;
  for (; sweeps < kMaxSweeps && !converged; ++sweeps) {
    for (int r = 0; r < m - 1; ++r, ++rounds, cur ^= 1) {
      const int co = cur ? zcopy : 0, no = cur ? 0 : zcopy;
      if (tid < half) {
        const int pt = 2 * tid, pb = 2 * tid + 1;
        double c = 1.0, s = 0.0;
        if (!(odd_pad && tid == 0) &&
            jacobi_rotation(dyn[co + pt * ms + pt], dyn[co + pb * ms + pb], dyn[co + pt * ms + pb], abs_tol2, c, s))
          s_rotated = 1;
        const double2 cs = make_double2(c, s);
        s_rot[tid] = cs;
        a.rotlog[(size_t)rounds * half + tid] = cs;
      }
      __syncthreads();
#pragma unroll
      for (int it = 0; it < ITEMS; ++it) {
        if (ITEMS > 1 && tid + it * nt >= n_blocks) continue;
        if (ITEMS == 1 && tid >= n_blocks) continue;
        const int bi = blk_i[it], bj = blk_j[it];
        const double2 ri = s_rot[bi], rj = s_rot[bj];
        const double ci = ri.x, si = ri.y, cj = rj.x, sj = rj.y;
        const double2 row0 = *reinterpret_cast<const double2*>(&dyn[co + src[it][0]]);
        const double2 row1 = *reinterpret_cast<const double2*>(&dyn[co + src[it][1]]);
        if (bi == bj) {   // the rotated pair itself: entries (t,t), (t,b), (b,b)
          const double att = row0.x, atb = row0.y, abb = row1.y;
          dyn[no + dst[it][0]] = ci * ci * att - 2.0 * ci * si * atb + si * si * abb;
          dyn[no + dst[it][3]] = si * si * att + 2.0 * ci * si * atb + ci * ci * abb;
          dyn[no + dst[it][1]] = si == 0.0 ? atb : 0.0;
          continue;
        }
        const double x00 = row0.x, x01 = row0.y, x10 = row1.x, x11 = row1.y;
        const double y00 = ci * x00 - si * x10, y01 = ci * x01 - si * x11;
        const double y10 = si * x00 + ci * x10, y11 = si * x01 + ci * x11;
        dyn[no + dst[it][0]] = y00 * cj - y01 * sj;
        dyn[no + dst[it][1]] = y00 * sj + y01 * cj;
        dyn[no + dst[it][2]] = y10 * cj - y11 * sj;
        dyn[no + dst[it][3]] = y10 * sj + y11 * cj;
      }
      __syncthreads();
    }
    if (s_rotated == 0) converged = true;   // same value for every thread: read after the round's closing barrier
    __syncthreads();                        // everyone has read the flag before it is cleared again
    if (tid == 0) s_rotated = 0;
  }

  // eigenvalues (by player), floor (after eq. zt:eig:repeat), decreasing order
  const int fo = cur ? zcopy : 0;
  const double floor_c = (1.0 - eta) * (1.0 - eta) * rho * rho;
  if (tid == 0) s_flag[0] = 0;
  __syncthreads();
  for (int pos = tid; pos < m; pos += nt) {
    const int i = player_at(pos, rounds, m);
    if (i >= R) continue;
    double c = dyn[fo + pos * ms + pos];
    if (!(c >= floor_c)) {
      c = floor_c;
      s_flag[0] = 1;
    }
    s_c[i] = c;
  }
  __syncthreads();
  for (int i = tid; i < R; i += nt) {
    int rank = 0;
    const double c = s_c[i];
    for (int j = 0; j < R; ++j) rank += (s_c[j] > c || (s_c[j] == c && j < i)) ? 1 : 0;
    s_perm[rank] = i;   // s_perm[k] = index of the k-th largest eigenvalue
    a.work->rank_of[i] = rank;
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
    a.work->n_rounds = rounds;
  }
  __syncthreads();
  const double beta_new = s_scal[3];
  for (int k = tid; k < R; k += nt) {
    const double dn = s_enew[k];
    const double en = 1.0 / (beta_new / dn + 1.0);
    st->d[k] = dn;
    st->e[k] = en;
    // A_t = (eta/N) E_{t+1}^{1/2} C_t^{-1/2} U_t^T E_t^{-1/2}  (eq. wt1): scale of row k / eigenpair s_perm[k]
    a.work->colscale[s_perm[k]] = (eta / N) * sqrt(en / s_c[s_perm[k]]);
    a.work->rowscale[k] = s_ise[k];
  }
  for (int idx = tid; idx < R * R; idx += nt) a.K[idx] = 0.0;
}

// U_t by replaying the rotation log on rows of the identity, then A_t (eq. wt1).  U <- U J only mixes two
// columns, so rows are independent: each wavefront owns one row and keeps it in registers.  Lane k holds the two
// columns that pair k rotates; between rounds the columns move to the neighbouring lanes exactly as the players
// of the round-robin schedule do (the first lane's second player never moves).  The log is staged through LDS
// in chunks of kEigvecChunk rounds, the next chunk being fetched while the current one is replayed.
__global__ __launch_bounds__(kEigvecThreads) void eigvec_kernel(const SmallGroup g) {
  __shared__ double2 s_log[2][kEigvecChunk * kMaxHalf];
  const SmallArgs& a = g.a[blockIdx.x];
  const int R = a.R;
  const int m = (R + 1) & ~1, half = m / 2;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = blockIdx.y * (kEigvecThreads / 64) + wave;   // rows >= R idle along (they share the barriers)
  const int n_rounds = a.work->n_rounds;
  const bool active = lane < half;
  // players held by this lane in round 0: first k, second m-1-k (lane 0: the fixed player m-1)
  int tp = lane, bp = m - 1 - lane;
  double top = (active && tp == row) ? 1.0 : 0.0;
  double bot = (active && bp == row) ? 1.0 : 0.0;

  constexpr int kLoads = (kEigvecChunk * kMaxHalf + kEigvecThreads - 1) / kEigvecThreads;
  const int chunk_elems = kEigvecChunk * half;   // the log is padded to whole chunks
  double2 stage[kLoads];
#pragma unroll
  for (int u = 0; u < kLoads; ++u) {
    const int e = tid + u * kEigvecThreads;
    if (e < chunk_elems) s_log[0][e] = a.rotlog[e];
  }
  __syncthreads();
  for (int base = 0, buf = 0; base < n_rounds; base += kEigvecChunk, buf ^= 1) {
    const bool more = base + kEigvecChunk < n_rounds;
    if (more) {
#pragma unroll
      for (int u = 0; u < kLoads; ++u) {
        const int e = tid + u * kEigvecThreads;
        if (e < chunk_elems) stage[u] = a.rotlog[(size_t)(base + kEigvecChunk) * half + e];
      }
    }
    const int len = min(kEigvecChunk, n_rounds - base);
    const double2* lg = s_log[buf];
    for (int rr = 0; rr < len; ++rr) {
      const double2 cs = active ? lg[rr * half + lane] : make_double2(1.0, 0.0);
      const double c = cs.x, s = cs.y;
      // the logged rotation acts on (first, second) of the pair
      const double nt_ = top * c - bot * s, nb_ = top * s + bot * c;
      top = nt_;
      bot = nb_;
      // players move: firsts shift one lane down (the last lane takes its own second), seconds shift one lane
      // up (lane 1 takes lane 0's first); lane 0's second is fixed
      if (m > 2) {
        const double t_dn = __shfl_down(top, 1);
        const double b_up = __shfl_up(bot, 1);
        const double t0 = __shfl(top, 0);
        top = lane == half - 1 ? bot : t_dn;
        bot = lane == 0 ? bot : (lane == 1 ? t0 : b_up);
        tp = tp + 1 == m - 1 ? 0 : tp + 1;
        if (lane != 0) bp = bp + 1 == m - 1 ? 0 : bp + 1;
      }
    }
    if (more) {
#pragma unroll
      for (int u = 0; u < kLoads; ++u) {
        const int e = tid + u * kEigvecThreads;
        if (e < chunk_elems) s_log[buf ^ 1][e] = stage[u];
      }
    }
    __syncthreads();
  }
  if (!active || row >= R) return;
  const int j = row;   // row of U = column of A_t
  const double rs = a.work->rowscale[j];
  if (tp < R) a.At[(size_t)a.work->rank_of[tp] * a.ldat + j] = (float)(a.work->colscale[tp] * top * rs);
  if (bp < R) a.At[(size_t)a.work->rank_of[bp] * a.ldat + j] = (float)(a.work->colscale[bp] * bot * rs);
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
