// The R x R part of the online natural-gradient update, entirely on the device (App. B.3, B.3.1).
//
// eig_update_kernel: one workgroup per instance forms Z_t from K_t and L_t (eq. zt:compute) and finds its
// eigenvalues by cyclic Jacobi in fp64.  Only Z is rotated: its upper triangle lives in LDS in "position space"
// (Brent-Luk: the members of pair k stand at positions 2k and 2k+1, and a fixed permutation between rounds brings
// the next partners together), in two copies used alternately, so a round costs one barrier.  The first wavefront
// computes the next round's rotations while the others rotate the 2x2 blocks; every rotation is written to a log.
// The kernel then floors and orders the eigenvalues and produces rho_{t+1}, D_{t+1}, E_{t+1} and the scales of A_t.
// eigvec_kernel: replays the rotation log on the rows of the identity (one wavefront per row of U_t, the two
// columns of a pair in one lane, moved between lanes as the players move) and writes A_t (eq. wt1).
// orth_fix_kernel: the orthogonality check of App. B.3.1 and, when it fails, the Cholesky fix folded into A_t.
#pragma once

#include <hip/hip_runtime.h>

#include "kernels.h"
#include "state.h"

namespace ngsgd {

constexpr int kSmallThreads = 1024;          // orthogonality fix kernel
constexpr int kEigThreads = 1024;            // R x R eigen-update kernel
// most 2x2 blocks of the upper triangle one thread may own
constexpr int kEigMaxItems = ((kMaxRank / 2) * (kMaxRank / 2 - 1) / 2 + (kEigThreads - 64) - 1) / (kEigThreads - 64);

constexpr int kEigvecThreads = 256;          // eigenvector kernel: 4 wavefronts, one row of U each
constexpr int kEigvecChunk = 32;             // rounds of the rotation log staged in LDS at a time
constexpr int kMaxSweeps = 20;
constexpr int kMaxHalf = kMaxRank / 2;
constexpr int kMaxRounds = kMaxSweeps * (kMaxRank - 1);
constexpr double kJacobiTol = 1.0e-13;       // a pair is left alone once |z_pq| <= tol * sqrt(z_pp z_qq)
constexpr double kJacobiAbsTol = 1.0e-13;    // ... or once |z_pq| <= this * max_i z_ii (rounding noise level)
constexpr double kJacobiLargeTol = 1.0e-6;   // a sweep without a rotated entry above this (same measure) ...
constexpr double kJacobiLargeAbs = 1.0e3;    // ... and above this many absolute thresholds is the last
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
  const double* sumsq_part;   // partial sums of tr(X X^T) left by the H product
  int n_sumsq;
  double2* rotlog;   // [kMaxRounds][half] (c, s) of every pair of every round
  EigWork* work;
};
struct SmallGroup {
  int count;
  double alpha, epsilon, num_samples_history;
  SmallArgs a[kMaxInstances];
};

// Coupled Newton (Goldschmidt) iteration from the hardware estimate: on return g = sqrt(x), h = 1 / (2 sqrt(x)).
// Two dependent operations per step instead of the three of the plain Newton step for 1/sqrt.
__device__ __forceinline__ void sqrt_pair(double x, double& g, double& h) {
  const double y = __builtin_amdgcn_rsq(x);
  g = x * y;
  h = 0.5 * y;
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const double e = fma(-g, h, 0.5);
    g = fma(g, e, g);
    h = fma(h, e, h);
  }
}

// Rotation that diagonalises [[app, apq], [apq, aqq]] as J^T A J with J = [[c, s], [-s, c]] (the inner rotation,
// c >= 1/sqrt 2).  Returns false (and the identity) when the off-diagonal entry is already negligible: relative
// to the diagonal pair (that relative test is what gives small eigenvalues of a graded positive definite matrix
// their relative accuracy) or in absolute terms (abs_tol2 is the squared absolute threshold).  `large` reports
// whether the entry was above kJacobiLargeTol relative to the pair and well above the absolute noise threshold:
// Jacobi converges quadratically, so a sweep whose rotations were all smaller than that leaves entries of the order
// of their square and needs no further sweep.  With
// h = (aqq - app) / 2 and r = sqrt(h^2 + apq^2):  c^2 = (1 + |h| / r) / 2,  s = sign(h) apq / (2 r c).  Written
// this way the rotation costs two reciprocal square roots in sequence and no division: it sits on the critical
// path of every round.
__device__ __forceinline__ bool jacobi_rotation(double app, double aqq, double apq, double abs_tol2, double& c,
                                                double& s, bool& large) {
  c = 1.0;
  s = 0.0;
  large = false;
  const double apq2 = apq * apq, scale2 = fabs(app * aqq);
  if (!(apq2 > kJacobiTol * kJacobiTol * scale2) || !(apq2 > abs_tol2) || !(apq2 > 1.0e-290)) return false;
  large = apq2 > kJacobiLargeTol * kJacobiLargeTol * scale2 && apq2 > kJacobiLargeAbs * kJacobiLargeAbs * abs_tol2;
  const double h = 0.5 * (aqq - app);
  double r, half_rinv, half_cinv;
  sqrt_pair(fma(h, h, apq2), r, half_rinv);
  const double sa = (h >= 0.0 ? apq : -apq) * half_rinv;   // sign(h) apq / (2 r)
  sqrt_pair(fma(fabs(h), half_rinv, 0.5), c, half_cinv);
  s = sa * (half_cinv + half_cinv);
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
template <int ITEMS, int NT>
__global__ __launch_bounds__(NT) void eig_update_kernel(const SmallGroup g) {
  extern __shared__ __attribute__((aligned(16))) double dyn[];   // two copies of Z (upper triangle, four planes)
  __shared__ double scratch[16];
  __shared__ double s_d[kMaxRank], s_ise[kMaxRank], s_dr[kMaxRank], s_c[kMaxRank + 1], s_enew[kMaxRank];
  __shared__ __attribute__((aligned(16))) double2 s_cs[2][kMaxHalf];   // (c, s) of the pairs, this round's and the next's
  __shared__ int s_perm[kMaxRank];
  __shared__ double s_scal[8];
  __shared__ int s_flag[2];
  __shared__ int s_rotated[2];

  const SmallArgs& a = g.a[blockIdx.x];
  const int R = a.R, D = a.D, N = a.N;
  const int tid = threadIdx.x;
  constexpr int nt = NT;
  const int m = (R + 1) & ~1;
  const int half = m / 2;
  PrecondScalars* st = a.st;

  const double eta = 1.0 - exp(-(double)N / g.num_samples_history);   // eq. eta:ns
  const double rho = st->rho;
  double tr_part = 0.0;   // tr(X X^T), summed here: the kernel that finishes the output may still be running
  for (int i = tid; i < a.n_sumsq; i += nt) tr_part += a.sumsq_part[i];
  const double tr_M = block_sum(tr_part, scratch);
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

  // Z_t from K_t and L_t (eq. zt:compute), symmetrised, laid out by position in four planes: plane 2a+b holds the
  // entry (2 bi + a, 2 bj + b) of every 2x2 block bi <= bj.  Blocks are numbered diagonal by diagonal (first the
  // blocks (k, k), then (k, k+1), ...): the permutation between rounds moves a block along its diagonal or to
  // the second next one, the block waves own runs of one diagonal, and the rotation lanes need the blocks (k, k)
  // and (k-1, k+1); with this numbering neighbouring lanes touch neighbouring addresses in all of these accesses
  // (8-byte LDS accesses without bank conflicts).  The padding player of an odd R has an all-zero row and column
  // and is never rotated.
  const int n_blocks = half * (half + 1) / 2;
  const int np = n_blocks;        // plane stride
  const int zcopy = 4 * np;       // offset of the second copy (offsets, not pointers: accesses stay LDS instructions)
  auto diag_start = [half](int d) { return d * half - d * (d - 1) / 2; };   // number of the block (0, d)
  auto slot = [&](int bi, int bj) { return diag_start(bj - bi) + bi; };    // number of the block (bi, bj), bi <= bj
  auto place = [&](int pa, int pb) {   // LDS offset of the entry at positions (pa, pb) within a copy
    const int lo = pa < pb ? pa : pb, hi = pa < pb ? pb : pa;
    const int bi = lo >> 1, bj = hi >> 1;
    return (2 * (lo & 1) + (hi & 1)) * np + slot(bi, bj);
  };
  for (int idx = tid; idx < 2 * zcopy; idx += nt) dyn[idx] = 0.0;
  __syncthreads();
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
    dyn[place(pa, pb)] = z;
  }
  zmax = block_max(zmax, scratch);
  const double abs_tol = kJacobiAbsTol * zmax;
  const double abs_tol2 = abs_tol * abs_tol;

  // The off-diagonal blocks (bi < bj) this thread owns (the threads after the first wavefront, diagonal by
  // diagonal), where they are stored, and the (fixed) destinations of their four entries.  The diagonal blocks
  // are handled apart (three entries, a different formula), so this path is branch-free.
  const int n_off = half * (half - 1) / 2;
  int blk_i[ITEMS], blk_j[ITEMS], blk_t[ITEMS];
  int dst[ITEMS][4];
#pragma unroll
  for (int it = 0; it < ITEMS; ++it) {
    const int item = (tid - 64) + it * (nt - 64);
    int d = 1, rem = (item >= 0 && item < n_off) ? item : 0;
    while (half - d > 0 && rem >= half - d) {   // diagonal d holds the blocks (0, d), ..., (half-1-d, half-1)
      rem -= half - d;
      ++d;
    }
    const int bi = rem, bj = min(rem + d, half - 1);   // (an idle thread of a single-pair problem: bj = bi = 0)
    blk_i[it] = bi;
    blk_j[it] = bj;
    blk_t[it] = (item >= 0 && item < n_off) ? slot(bi, bj) : -1;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      dst[it][e] = place(next_position(2 * bi + (e >> 1), half), next_position(2 * min(bj, half - 1) + (e & 1), half));
  }
  // The diagonal block (k, k) is rotated by lane k of the second wavefront (on top of its off-diagonal block): the
  // rotation lanes' chain bounds the round and is kept as short as possible.  Destinations of (t,t), (t,b), (b,b):
  const int diag_k = tid - 64;
  const bool diag_lane = diag_k >= 0 && diag_k < half;
  int diag_t = 0, diag_dst[3] = {0, 0, 0};
  if (diag_lane) {
    diag_t = slot(diag_k, diag_k);
    diag_dst[0] = place(next_position(2 * diag_k, half), next_position(2 * diag_k, half));
    diag_dst[1] = place(next_position(2 * diag_k, half), next_position(2 * diag_k + 1, half));
    diag_dst[2] = place(next_position(2 * diag_k + 1, half), next_position(2 * diag_k + 1, half));
  }
  const bool odd_pad = (R & 1) != 0;   // pair 0 then holds the padding player

  // Rotation lanes (the first wavefront): while the 2x2 blocks of round r are being rotated, lane k of this wave
  // prepares pair k's rotation for round r+1.  The pair that will stand at (2k, 2k+1) is made of member A (the
  // later column) and member B (the earlier row) of the present layout; the lane recomputes their two diagonal
  // entries and their common entry after this round's rotations from the old copy, so a round needs one barrier.
  const int rot_k = tid;   // the first wavefront: the oldest wave of a SIMD is served first
  const bool rot_lane = rot_k < half;
  int rz_blk = 0, rz_da = 0, rz_db = 0, rz_pa = 0, rz_pb = 0;
  bool rz_sa0 = true, rz_sb0 = true;
  if (rot_lane && half >= 2) {
    const int k = rot_k;
    const int pa = k < half - 1 ? k + 1 : half - 1, sa = k < half - 1 ? 0 : 1;   // first member of the new pair
    const int pb = k >= 2 ? k - 1 : 0, sb = k == 1 ? 0 : 1;                       // second member (pb < pa)
    rz_pa = pa;
    rz_pb = pb;
    rz_sa0 = sa == 0;
    rz_sb0 = sb == 0;
    rz_blk = slot(pb, pa);
    rz_da = slot(pa, pa);
    rz_db = slot(pb, pb);
  }
  double2* __restrict__ rotlog = a.rotlog;
  if (tid < 64) __builtin_amdgcn_s_setprio(3);   // the rotation wave's dependent chain bounds the round
  if (tid < 2) s_rotated[tid] = 0;
  __syncthreads();
  if (rot_lane) {   // rotations of the very first round
    const int t = slot(rot_k, rot_k);
    double c = 1.0, s = 0.0;
    bool large = false;
    if (!(odd_pad && rot_k == 0)) jacobi_rotation(dyn[t], dyn[3 * np + t], dyn[np + t], abs_tol2, c, s, large);
    if (large) s_rotated[0] = 1;
    s_cs[0][rot_k] = make_double2(c, s);
    rotlog[rot_k] = make_double2(c, s);
  }
  __syncthreads();

  // cyclic Jacobi; a sweep in which no pair needed a large rotation ends the iteration
  int sweeps = 0, rounds = 0, cur = 0;
  bool converged = false;
  for (; sweeps < kMaxSweeps && !converged; ++sweeps) {
    for (int r = 0; r < m - 1; ++r, ++rounds, cur ^= 1) {
      const int co = cur ? zcopy : 0, no = cur ? 0 : zcopy;
      const double2* cs = s_cs[cur];
      if (rot_lane) {
        double c = 1.0, s = 0.0;
        if (half >= 2 && !(odd_pad && rot_k == 0)) {
          const double2 csi = cs[rz_pb], csj = cs[rz_pa];
          const double ci = csi.x, si = csi.y, cj = csj.x, sj = csj.y;
          const double x00 = dyn[co + rz_blk], x01 = dyn[co + np + rz_blk];
          const double x10 = dyn[co + 2 * np + rz_blk], x11 = dyn[co + 3 * np + rz_blk];
          const double da_tt = dyn[co + rz_da], da_tb = dyn[co + np + rz_da], da_bb = dyn[co + 3 * np + rz_da];
          const double db_tt = dyn[co + rz_db], db_tb = dyn[co + np + rz_db], db_bb = dyn[co + 3 * np + rz_db];
          __builtin_amdgcn_sched_barrier(0);   // all reads are in flight before the first use
          // a first member takes (c, -s) of its pair's rotation, a second member (s, c)
          const double r0 = rz_sb0 ? ci : si, r1 = rz_sb0 ? -si : ci;
          const double q0 = rz_sa0 ? cj : sj, q1 = rz_sa0 ? -sj : cj;
          const double zab = q0 * (r0 * x00 + r1 * x10) + q1 * (r0 * x01 + r1 * x11);
          const double zaa = q0 * q0 * da_tt + 2.0 * q0 * q1 * da_tb + q1 * q1 * da_bb;
          const double zbb = r0 * r0 * db_tt + 2.0 * r0 * r1 * db_tb + r1 * r1 * db_bb;
          // whether this rotation belongs to the present sweep or opens the next one
          bool large = false;
          jacobi_rotation(zaa, zbb, zab, abs_tol2, c, s, large);
          if (large) s_rotated[(sweeps + (r == m - 2 ? 1 : 0)) & 1] = 1;
        }
        s_cs[cur ^ 1][rot_k] = make_double2(c, s);
        rotlog[(size_t)(rounds + 1) * half + rot_k] = make_double2(c, s);
      }
      if (diag_lane) {   // this round's rotation of pair diag_k, applied to its diagonal block
        const double2 csk = cs[diag_k];
        const double ck = csk.x, sk = csk.y;
        const double att = dyn[co + diag_t], atb = dyn[co + np + diag_t], abb = dyn[co + 3 * np + diag_t];
        dyn[no + diag_dst[0]] = ck * ck * att - 2.0 * ck * sk * atb + sk * sk * abb;
        dyn[no + diag_dst[2]] = sk * sk * att + 2.0 * ck * sk * atb + ck * ck * abb;
        dyn[no + diag_dst[1]] = sk == 0.0 ? atb : 0.0;
      }
#pragma unroll
      for (int it = 0; it < ITEMS; ++it) {
        const int t = blk_t[it];
        if (t < 0) continue;
        const int bi = blk_i[it], bj = blk_j[it];
        const double2 csi = cs[bi], csj = cs[bj];
        const double ci = csi.x, si = csi.y, cj = csj.x, sj = csj.y;
        const double x00 = dyn[co + t], x01 = dyn[co + np + t], x10 = dyn[co + 2 * np + t], x11 = dyn[co + 3 * np + t];
        const double y00 = ci * x00 - si * x10, y01 = ci * x01 - si * x11;
        const double y10 = si * x00 + ci * x10, y11 = si * x01 + ci * x11;
        dyn[no + dst[it][0]] = y00 * cj - y01 * sj;
        dyn[no + dst[it][1]] = y00 * sj + y01 * cj;
        dyn[no + dst[it][2]] = y10 * cj - y11 * sj;
        dyn[no + dst[it][3]] = y10 * sj + y11 * cj;
      }
      __syncthreads();
    }
    if (s_rotated[sweeps & 1] == 0) converged = true;   // same value for every thread: read after the barrier
    __syncthreads();                                    // everyone has read the flag before it is cleared again
    if (tid == 0) s_rotated[sweeps & 1] = 0;
  }

  // eigenvalues (by player), floor (after eq. zt:eig:repeat), decreasing order
  const int fo = cur ? zcopy : 0;
  const double floor_c = (1.0 - eta) * (1.0 - eta) * rho * rho;
  if (tid == 0) s_flag[0] = 0;
  __syncthreads();
  for (int pos = tid; pos < m; pos += nt) {
    const int i = player_at(pos, rounds, m);
    if (i >= R) continue;
    double c = dyn[fo + place(pos, pos)];
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
    const double rho_dash = ((eta / N) * tr_M + (1.0 - eta) * ((double)D * rho + sum_d) - sum_sqrt) / (double)(D - R);
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

// Whole-wavefront shifts by one lane through the DPP path of the vector ALU (no LDS traffic): lane i receives the
// value of lane i-1 (up) or i+1 (down); the lane without a source receives zero.
__device__ __forceinline__ double wave_shift_up(double x) {
  int lo = __double2loint(x), hi = __double2hiint(x);
  lo = __builtin_amdgcn_update_dpp(0, lo, 0x138, 0xf, 0xf, true);   // wave_shr:1
  hi = __builtin_amdgcn_update_dpp(0, hi, 0x138, 0xf, 0xf, true);
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double wave_shift_down(double x) {
  int lo = __double2loint(x), hi = __double2hiint(x);
  lo = __builtin_amdgcn_update_dpp(0, lo, 0x130, 0xf, 0xf, true);   // wave_shl:1
  hi = __builtin_amdgcn_update_dpp(0, hi, 0x130, 0xf, 0xf, true);
  return __hiloint2double(hi, lo);
}

// U_t by replaying the rotation log on rows of the identity, then A_t (eq. wt1).  U <- U J only mixes two
// columns, so rows are independent: each wavefront owns one row and keeps it in registers.  Lane k holds the two
// columns that pair k rotates; between rounds the columns move to the neighbouring lanes exactly as the players
// of the round-robin schedule do (the first lane's second player never moves).  The log is staged through LDS
// in chunks of kEigvecChunk rounds, the next chunk being fetched while the current one is replayed.
__global__ __launch_bounds__(kEigvecThreads) void eigvec_kernel(const SmallGroup g) {
  __shared__ double2 s_log[2][kEigvecChunk * kMaxHalf];
  extern __shared__ double eigvec_reserved[];   // not used: see the launch
  const SmallArgs& a = g.a[blockIdx.x];
  const int R = a.R;
  const int m = (R + 1) & ~1, half = m / 2;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = blockIdx.y * (kEigvecThreads / 64) + wave;   // rows >= R idle along (they share the barriers)
  const int n_rounds = a.work->n_rounds;
  const bool active = lane < half;
  // Lanes beyond the last pair replay the last pair's rotations on zeros: nothing of theirs reaches an active
  // lane (a lane takes from its lower neighbour, and the last active lane takes its own second member).
  const int ll = active ? lane : half - 1;
  // players held by this lane in round 0: first k, second m-1-k (lane 0: the fixed player m-1)
  double top = (active && lane == row) ? 1.0 : 0.0;
  double bot = (active && m - 1 - lane == row) ? 1.0 : 0.0;
  const bool last_lane = lane == half - 1, lane0 = lane == 0, lane1 = lane == 1;
  const bool single = m == 2;   // one pair: nothing moves

  // the log is padded to whole chunks, and one chunk beyond the last round is allocated: staging needs no guards
  constexpr int kLoads = (kEigvecChunk * kMaxHalf + kEigvecThreads - 1) / kEigvecThreads;
  const int chunk_elems = kEigvecChunk * half;
  const double2* __restrict__ rotlog = a.rotlog;
  int src[kLoads];
#pragma unroll
  for (int u = 0; u < kLoads; ++u) src[u] = min(tid + u * kEigvecThreads, chunk_elems - 1);
  double stage_c[kLoads], stage_s[kLoads];   // plain scalars: they must stay in registers
#pragma unroll
  for (int u = 0; u < kLoads; ++u) s_log[0][src[u]] = rotlog[src[u]];
  __syncthreads();
  for (int base = 0, buf = 0; base < n_rounds; base += kEigvecChunk, buf ^= 1) {
    const bool more = base + kEigvecChunk < n_rounds;
    if (more) {   // in flight while this chunk is replayed
#pragma unroll
      for (int u = 0; u < kLoads; ++u) {
        const double2 v = rotlog[(size_t)(base + kEigvecChunk) * half + src[u]];
        stage_c[u] = v.x;
        stage_s[u] = v.y;
      }
    }
    const int len = min(kEigvecChunk, n_rounds - base);
    const double2* lg = s_log[buf] + ll;
    auto replay = [&](double2 cs) {
      // the logged rotation acts on (first, second) of the pair
      const double nt_ = top * cs.x - bot * cs.y, nb_ = top * cs.y + bot * cs.x;
      // players move: firsts shift one lane down (the last lane takes its own second), seconds shift one lane
      // up (lane 1 takes lane 0's first); lane 0's second is fixed.  With a single pair (m = 2) lane 0 is the
      // last lane as well and both members stay.
      const double t_dn = wave_shift_down(nt_);
      const double b_up = wave_shift_up(nb_);
      const double t_up = wave_shift_up(nt_);
      top = last_lane ? (single ? nt_ : nb_) : t_dn;
      bot = lane0 ? nb_ : (lane1 ? t_up : b_up);
    };
    int rr = 0;
    for (; rr + 4 <= len; rr += 4) {   // four rotations fetched ahead of their use
      const double2 c0 = lg[(rr + 0) * half], c1 = lg[(rr + 1) * half], c2 = lg[(rr + 2) * half], c3 = lg[(rr + 3) * half];
      replay(c0);
      replay(c1);
      replay(c2);
      replay(c3);
    }
    for (; rr < len; ++rr) replay(lg[rr * half]);
    if (more) {
#pragma unroll
      for (int u = 0; u < kLoads; ++u) s_log[buf ^ 1][src[u]] = make_double2(stage_c[u], stage_s[u]);
    }
    __syncthreads();
  }
  if (!active || row >= R) return;
  // the players standing at this lane's two positions after n_rounds rounds
  const int tp = player_at(2 * lane, n_rounds, m), bp = player_at(2 * lane + 1, n_rounds, m);
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
  float* At;         // R x R (ldat): A_t on entry; when the fix is needed, E^{1/2} L^{-1} E^{-1/2} A_t on return
  int ldat;
  int R;
};
struct OrthGroup {
  int count;
  OrthArgs a[kMaxInstances];
};

// The augmented matrix [O | B], R x 2R: O = E^{-1/2} (W W^T) E^{-1/2} (full, symmetric) and B = E^{-1/2} A_t.
// Gaussian elimination without pivoting (O is symmetric positive definite) turns O into D L1^T and B into
// L1^{-1} B, where O = L1 D L1^T with unit lower triangular L1; the Cholesky factor is L = L1 D^{1/2}, so
// L^{-1} B = D^{-1/2} (L1^{-1} B).  The matrix lives in registers as 4 x CT tiles: thread (ti, tj) holds the rows
// 4 ti .. 4 ti + 3 and the columns tj, tj + 32, ... (CT of them: the kernel is instantiated per rank class).  What a step
// needs from other threads (the pivot row, the pivot column and the reciprocal of the pivot) is published in LDS by
// its owners at the end of the step before, in one of two buffers used alternately; a step (two pivots, see below)
// is then one barrier, LDS reads without address arithmetic and multiply-adds (a tile needs 2.3 times fewer reads
// per element than a strip of one row); wavefronts whose rows all lie above the pivot skip the step.
constexpr int kOrthTileRows = 4;
constexpr int kOrthTileStride = 32;   // columns tj, tj + 32, ...: the threads of a row of tiles
constexpr int kOrthRowsPerWave = (64 / kOrthTileStride) * kOrthTileRows;
static_assert((kMaxRank + kOrthTileRows - 1) / kOrthTileRows * kOrthTileStride <= kSmallThreads, "one thread per tile");
inline int orth_columns_per_thread(int R) { return (2 * R + kOrthTileStride - 1) / kOrthTileStride; }

template <int CT>
__global__ __launch_bounds__(kSmallThreads) void orth_fix_kernel(const OrthGroup g) {
  extern __shared__ __attribute__((aligned(16))) double dyn[];   // W W^T of the instance, R x (R + 1)
  __shared__ double scratch[16];
  __shared__ double s_ise[kMaxRank];                       // E_ii^{-1/2}
  __shared__ double s_prow[2][2][kOrthTileStride * CT];    // the two pivot rows of a step
  __shared__ double s_pcol[2][2][kMaxRank + kOrthTileRows];   // the two pivot columns of a step
  __shared__ double s_invp[2];                             // reciprocal of the first pivot of a step
  __shared__ double s_dinv[kMaxRank];                      // D_ii^{-1/2}
  const OrthArgs& a = g.a[blockIdx.x];
  PrecondScalars* st = a.st;
  if (!(st->flags & kFlagOrthCheck)) return;   // uniform over the workgroup
  const int R = a.R;
  const int tid = threadIdx.x, nt = blockDim.x;
  // the check: G and E through LDS (coalesced reads), O symmetrised from there
  double* const Gs = dyn;   // R x (R + 1)
  const int SG = R + 1;
  for (int idx = tid; idx < R * R; idx += nt) Gs[(idx / R) * SG + idx % R] = a.G[idx];
  for (int k = tid; k < R; k += nt) s_ise[k] = rsqrt(st->e[k]);
  __syncthreads();
  double dev = 0.0;
  for (int idx = tid; idx < R * R; idx += nt) {
    const int r = idx / R, c = idx % R;
    if (c < r) continue;
    const double o = 0.5 * (Gs[r * SG + c] + Gs[c * SG + r]) * s_ise[r] * s_ise[c];
    dev = fmax(dev, fabs(o - (r == c ? 1.0 : 0.0)));
  }
  dev = block_max(dev, scratch);
  if (!(dev > kOrthoTolerance)) {
    __syncthreads();
    if (tid == 0) st->flags &= ~kFlagOrthCheck;
    return;
  }
  // The fix W <- E^{1/2} L^{-1} E^{-1/2} W is applied to the factor it came from: W = A_t B_t, so the triangular
  // mixing matrix goes into A_t and the product with B_t (still in its buffer) is simply launched again, gated on
  // the flag set below.
  const int ti = tid / kOrthTileStride, tj = tid % kOrthTileStride;
  const int row0 = ti * kOrthTileRows;
  const int wave_row0 = (tid >> 6) * kOrthRowsPerWave;   // first row held by this wavefront
  double v[kOrthTileRows][CT];
#pragma unroll
  for (int r = 0; r < kOrthTileRows; ++r) {
    const int i = row0 + r;
    const double ise_i = s_ise[min(i, R - 1)];
#pragma unroll
    for (int c = 0; c < CT; ++c) {
      const int j = tj + kOrthTileStride * c;
      v[r][c] = 0.0;
      if (i < R && j < R) v[r][c] = 0.5 * (Gs[i * SG + j] + Gs[j * SG + i]) * ise_i * s_ise[j];
      if (i < R && j >= R && j < 2 * R) v[r][c] = (double)a.At[i * a.ldat + (j - R)] * ise_i;
    }
  }
  // Two pivots per barrier.  What the pair (k, k + 1) reads: rows k and k + 1 as they stand after pivot k - 1 (with zeros
  // in the columns up to k, which the pair must leave alone), columns k and k + 1 likewise, and the reciprocal of
  // pivot k.  Every thread derives from them what pivot k makes of row k + 1, of column k + 1 and of pivot k + 1 (a
  // few operations on values it has read anyway) and applies both eliminations to its tile at once.  The four lines
  // of the next pair are published by their owners behind the update, in the other of two buffers: the registers of a
  // row or column are met in unrolled loops under uniform compares, so no register is picked by index.
  auto publish = [&](const int kn, const int nb) {   // rows and columns kn, kn + 1 and 1 / pivot kn into buffer nb
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int ku = kn + u;
      const int kr = ku % kOrthTileRows, kti = ku / kOrthTileRows;
      const int kc = ku / kOrthTileStride, ktj = ku % kOrthTileStride;
#pragma unroll
      for (int r = 0; r < kOrthTileRows; ++r) {
        if (r == kr && ti == kti) {
#pragma unroll
          for (int c = 0; c < CT; ++c)
            s_prow[nb][u][tj + kOrthTileStride * c] = (tj + kOrthTileStride * c > kn) ? v[r][c] : 0.0;
        }
      }
#pragma unroll
      for (int c = 0; c < CT; ++c) {
        if (c == kc && tj == ktj) {
#pragma unroll
          for (int r = 0; r < kOrthTileRows; ++r) {
            s_pcol[nb][u][row0 + r] = v[r][c];
            if (u == 0 && row0 + r == kn) s_invp[nb] = 1.0 / fmax(v[r][c], 1.0e-300);
          }
        }
      }
    }
  };
  if (row0 < R) publish(0, 0);
  for (int k = 0; k < R - 1; k += 2) {
    const int buf = (k >> 1) & 1, nb = buf ^ 1;
    __syncthreads();
    if (wave_row0 + kOrthRowsPerWave - 1 > k && wave_row0 < R) {   // (uniform over the wavefront) some row lies below k
      const int k1 = k + 1;   // (k1 <= R - 1: a row of the matrix; as the last row it eliminates nothing)
      const double inv0 = s_invp[buf];
      const double m = s_pcol[buf][0][k1] * inv0;            // what pivot k takes off row k + 1
      const double a01 = s_prow[buf][0][k1];                 // entry (k, k + 1)
      const double inv1 = 1.0 / fmax(s_pcol[buf][1][k1] - m * a01, 1.0e-300);   // pivot k + 1 after pivot k
      double f[kOrthTileRows], gq[kOrthTileRows], p0[CT], q1[CT];
#pragma unroll
      for (int r = 0; r < kOrthTileRows; ++r) {
        const int i = row0 + r;
        const double c0 = s_pcol[buf][0][i], c1 = s_pcol[buf][1][i];
        f[r] = (i > k && i < R) ? c0 * inv0 : 0.0;
        gq[r] = (i > k1 && i < R) ? (c1 - f[r] * a01) * inv1 : 0.0;
      }
#pragma unroll
      for (int c = 0; c < CT; ++c) {
        const int j = tj + kOrthTileStride * c;
        p0[c] = s_prow[buf][0][j];
        q1[c] = (j > k1) ? s_prow[buf][1][j] - m * p0[c] : 0.0;   // row k + 1 after pivot k, dead columns zero
      }
#pragma unroll
      for (int r = 0; r < kOrthTileRows; ++r)
#pragma unroll
        for (int c = 0; c < CT; ++c) v[r][c] -= f[r] * p0[c] + gq[r] * q1[c];
      if (k + 2 < R - 1) publish(k + 2, nb);
    }
  }
  // D_ii is the diagonal entry of row i as it stood when the row became the pivot row: rows are not touched afterwards
#pragma unroll
  for (int r = 0; r < kOrthTileRows; ++r)
#pragma unroll
    for (int c = 0; c < CT; ++c)
      if (row0 + r < R && tj + kOrthTileStride * c == row0 + r) s_dinv[row0 + r] = rsqrt(fmax(v[r][c], 1.0e-300));
  __syncthreads();
#pragma unroll
  for (int r = 0; r < kOrthTileRows; ++r) {
    const int i = row0 + r;
    if (i >= R) continue;
    const double scale = s_dinv[i] / s_ise[i];   // E_ii^{1/2} D_ii^{-1/2}
#pragma unroll
    for (int c = 0; c < CT; ++c) {
      const int j = tj + kOrthTileStride * c;
      if (j >= R && j < 2 * R) a.At[i * a.ldat + (j - R)] = (float)(scale * v[r][c]);
    }
  }
  if (tid == 0) st->flags = (st->flags & ~kFlagOrthCheck) | kFlagReorth;
}

}  // namespace ngsgd
