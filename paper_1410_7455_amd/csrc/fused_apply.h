// Fused apply path of the online natural-gradient preconditioner (App. B.3, eq. ht and hatxt:compute:2; App. B.3.3,
// eq. pi): Xhat = X - (X W^T) W with the squared row norms of Xhat and tr(X X^T), reading X once and writing Xhat
// once.  Used when the factor is not updated by the call (App. B.5, "without updating").
//
// A 256-thread workgroup owns a patch of 64 rows x BC columns.  Every lane loads its share of the patch straight
// into registers, laid out as the A operand of v_mfma_f32_16x16x4_f32 (lane (r, g) of a wavefront holds row r,
// columns 16 kk + 4 g .. + 3), and the workgroup stages the matching BC columns of W in LDS.
//   phase 1: the patch's contribution to H = X W^T (rows x rank) on the matrix unit, added to H in memory with
//            float atomics; the patch's sum of squares.
//   wait:    an arrival counter per block of 64 rows tells when all column chunks of the block have contributed.
//   phase 2: Xhat^T = X^T - W^T H^T, computed transposed: the accumulator layout of the product (column index from
//            the register, row index from the lane) is then exactly the layout the patch already has in registers,
//            so the registers holding X are the accumulator and leave as Xhat.  Row norms from the same registers.
//
// Exchange between workgroups.  The dies of the chip have separate L2 caches, and a device-wide fence writes the
// die's L2 back and invalidates it: measured here, two such fences per thread cost 27 us of a 58 us launch, and even
// one release / acquire pair per workgroup cost 8 us.  The exchange therefore uses nothing but operations that are
// performed at the memory side: float atomics for H (with return, see below), an atomic counter, and loads of H at
// device scope that bypass this die's caches.  Order is kept by construction: every wavefront waits until its atomics
// have returned their old values before the workgroup's barrier, the counter is incremented after that barrier, and
// H is loaded after the counter has been seen complete.
//
// Progress.  The workgroups of a row block only wait for each other, and the grid is ordered row block by row
// block, so a launch on its own always makes progress: on every die workgroups are started in index order, hence the
// oldest unfinished row block has all its workgroups running or next in line.  With other kernels competing for the
// compute units the wait is still bounded: after `spin_limit` ticks of the constant-rate clock a workgroup stops
// waiting, leaves its patch of X untouched, puts the patch on the instance's list of deferred patches and exits; the
// kernel that reduces the partial sums afterwards (finish_apply_kernel) completes those patches from H, which is
// final by then.  So every wave exits whatever else occupies the GPU.  (The patch cannot be completed here without
// H, and H cannot be recomputed here from X: the matrix is updated in place, and other workgroups may already have
// replaced their columns of these rows.)
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm.h"
#include "state.h"

namespace ngsgd {

constexpr int kFusedRows = 64;       // rows of a patch: four wavefronts of 16
constexpr int kFusedThreads = 256;
constexpr int kFusedChunk = 160;     // columns of a patch (BC): 40 registers per lane hold it

struct FusedArgs {
  const float* X;          // N x D, leading dimension ldx
  float* Xout;             // N x D, leading dimension ldo (may be X itself)
  const float* W;          // R x D, leading dimension ldw; entries beyond D in a row are never used
  float* H;                // N x ldh, all zero on entry; X W^T on exit
  int* arrive;             // one arrival counter per row block, zero on entry
  int* deferred_count;     // zero on entry; number of patches put on the list below
  int* deferred;           // [n_rb * n_chunks] patches left for the finishing kernel: rb * n_chunks + chunk
  float* rownorm_part;     // [n_chunks][N] squared row norms of Xhat per column chunk
  double* sumsq_part;      // [n_chunks * n_rb] sums of squares of X per patch
  int ldx, ldo, ldw, ldh;
  int N, D, R;
  int n_rb, n_chunks, n_chunks_pad;   // the chunk count is padded to a multiple of the die count
  int unit_begin;                     // first workgroup index of this instance (a multiple of the die count)
};
struct FusedGroup {
  int count;
  int total_units;
  long long spin_limit;    // ticks of wall_clock64() a workgroup waits for its row block; <= 0: does not wait at all
  FusedArgs a[kMaxInstances];
};

// 16-byte load at device scope (sc1): served from where the atomics of all dies are performed, never from a stale
// line of this die's caches.  The compiler does not track the load: wait_coherent_loads() must follow before use.
__device__ __forceinline__ void load_coherent_f4(floatx4& dst, const float* p) {
  asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(dst) : "v"(p) : "memory");
}
__device__ __forceinline__ void wait_coherent_loads(floatx4& dst) {
  asm volatile("s_waitcnt vmcnt(0)" : "+v"(dst) : : "memory");
}

// TIMING is for microbenchmarks only (bit 0: no atomics on H, bit 1: no wait); production code uses 0.
template <int RC, int BC, int TIMING = 0>
__global__ __launch_bounds__(kFusedThreads, (RC <= 80 ? 3 : 2)) void fused_apply_kernel(const FusedGroup g) {
  constexpr int TJ = RC / 16;        // 16-wide tiles of the rank dimension
  constexpr int KK = BC / 16;        // 16-column groups of the patch
  constexpr int LDW = BC + 4;        // LDS row stride of the W chunk: 16-byte reads along a row and 4-byte reads down a
                                     // column are both free of bank conflicts when BC is a multiple of 32
  static_assert(RC % 16 == 0 && BC % 32 == 0, "tile shape");
  __shared__ __attribute__((aligned(16))) float Ws[RC * LDW];
  __shared__ double red[kFusedThreads / 64];
  __shared__ int s_arrived;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, g4 = lane >> 4;

  const int unit = blockIdx.x;
  if (unit >= g.total_units) return;
  int pi = 0;
  for (int i = 1; i < g.count; ++i)
    if (unit >= g.a[i].unit_begin) pi = i;
  const FusedArgs& P = g.a[pi];
  const int local = unit - P.unit_begin;
  const int rb = local / P.n_chunks_pad, chunk = local % P.n_chunks_pad;
  if (rb >= P.n_rb || chunk >= P.n_chunks) return;   // padding units (uniform over the workgroup)
  const int N = P.N, D = P.D, R = P.R;
  const int c0 = chunk * BC;
  const int row = rb * kFusedRows + wave * 16 + r16;       // the row this lane holds
  const bool row_ok = row < N;
  const int last_f4 = (D - 1) & ~3;                        // the last 16-byte piece of a row that holds a column < D

  // ---- the patch of X into registers (columns beyond D and rows beyond N as zeros) -----------------------
  float4 xr[KK];
  {
    const float* xrow = P.X + (size_t)min(row, N - 1) * P.ldx;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const int col = c0 + 16 * kk + 4 * g4;
      xr[kk] = *reinterpret_cast<const float4*>(xrow + min(col, last_f4));
    }
  }
  // ---- the chunk of W into LDS: Ws[j][c] = W[j][c0 + c], zero for j >= R or c0 + c >= D ------------------------
  {
    constexpr int F4_PER_ROW = BC / 4;
    constexpr int TOTAL = RC * F4_PER_ROW;
    constexpr int ITER = (TOTAL + kFusedThreads - 1) / kFusedThreads;
    float4 wr[ITER];
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      const int f = min(tid + i * kFusedThreads, TOTAL - 1);
      const int j = f / F4_PER_ROW, c4 = (f % F4_PER_ROW) * 4;
      wr[i] = *reinterpret_cast<const float4*>(P.W + (size_t)min(j, R - 1) * P.ldw + min(c0 + c4, last_f4));
    }
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      const int f = tid + i * kFusedThreads;
      if (TOTAL % kFusedThreads != 0 && f >= TOTAL) continue;
      const int j = f / F4_PER_ROW, c4 = (f % F4_PER_ROW) * 4;
      const int left = (j < R) ? D - (c0 + c4) : 0;
      float4 v = wr[i];
      v.x = left > 0 ? v.x : 0.f;
      v.y = left > 1 ? v.y : 0.f;
      v.z = left > 2 ? v.z : 0.f;
      v.w = left > 3 ? v.w : 0.f;
      *reinterpret_cast<float4*>(&Ws[j * LDW + c4]) = v;
    }
  }
  float ssq = 0.f;
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    const int left = row_ok ? D - (c0 + 16 * kk + 4 * g4) : 0;
    xr[kk].x = left > 0 ? xr[kk].x : 0.f;
    xr[kk].y = left > 1 ? xr[kk].y : 0.f;
    xr[kk].z = left > 2 ? xr[kk].z : 0.f;
    xr[kk].w = left > 3 ? xr[kk].w : 0.f;
    ssq += xr[kk].x * xr[kk].x + xr[kk].y * xr[kk].y + xr[kk].z * xr[kk].z + xr[kk].w * xr[kk].w;
  }
  __syncthreads();

  // ---- phase 1: this patch's part of H = X W^T --------------------------------------------------------------
  // Two 16-wide tiles of the rank at a time, each in two MFMA chains (even and odd 16-column groups) that are
  // summed with an ordinary add: the chains stay short (the matrix unit does not round its accumulator additions
  // to nearest) and consecutive MFMAs never depend on each other.  The additions to H of a pair of tiles are
  // issued as soon as the pair is complete, so that they travel while the next pair is being multiplied.
  // Register q of lane (r16, g4) holds H[row block row 16 wave + 4 g4 + q][16 tj + r16].
  // The atomics return the old value: a wavefront then knows that its additions have been performed where all dies
  // see them once the values are back, which the acknowledgement of an atomic without return does not guarantee (with
  // other kernels loading the memory system the arrival counter was seen to overtake such additions).
  static_assert(KK % 2 == 0, "column groups are taken in pairs");
  float old[TJ][4];
#pragma unroll
  for (int tj0 = 0; tj0 < TJ; tj0 += 2) {
    constexpr int kPair = 2;
    floatx4 ch[kPair][2];
#pragma unroll
    for (int t = 0; t < kPair; ++t) ch[t][0] = ch[t][1] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KK; kk += 2) {
      float4 bf[kPair][2];
#pragma unroll
      for (int t = 0; t < kPair; ++t)
#pragma unroll
        for (int par = 0; par < 2; ++par)
          if (tj0 + t < TJ)
            bf[t][par] = *reinterpret_cast<const float4*>(&Ws[(16 * (tj0 + t) + r16) * LDW + 16 * (kk + par) + 4 * g4]);
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int par = 0; par < 2; ++par)
#pragma unroll
          for (int t = 0; t < kPair; ++t)
            if (tj0 + t < TJ)
              ch[t][par] = __builtin_amdgcn_mfma_f32_16x16x4f32(pick4(xr[kk + par], q), pick4(bf[t][par], q), ch[t][par], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);   // two 16-column groups at a time: keeps the fragments of later groups out of registers
    }
#pragma unroll
    for (int t = 0; t < kPair; ++t) {
      if (tj0 + t >= TJ) continue;
      const int tj = tj0 + t;
      const floatx4 tot = ch[t][0] + ch[t][1];
      const int j = 16 * tj + r16;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int hrow = rb * kFusedRows + wave * 16 + 4 * g4 + q;
        old[tj][q] = 0.f;
        if (!(TIMING & 1) && hrow < N && j < R) old[tj][q] = unsafeAtomicAdd(P.H + (size_t)hrow * P.ldh + j, tot[q]);
      }
    }
  }
#pragma unroll
  for (int tj = 0; tj < TJ; ++tj)
#pragma unroll
    for (int q = 0; q < 4; ++q) asm volatile("" : : "v"(old[tj][q]));   // the returned value must have arrived here
  {
    double s = (double)ssq;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if (lane == 0) red[wave] = s;
  }
  // every atomic of this wavefront has returned before the barrier lets thread 0 count the workgroup's arrival
  // (a workgroup-scope release: a wait on the memory counters, no cache maintenance)
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  if (tid == 0) {
    P.sumsq_part[chunk * P.n_rb + rb] = (red[0] + red[1]) + (red[2] + red[3]);
    const int before = __hip_atomic_fetch_add(&P.arrive[rb], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int arrived = (before + 1 >= P.n_chunks || (TIMING & 2)) ? 1 : 0;   // the last to arrive need not look again
    const long long t0 = wall_clock64();
    while (!arrived) {
      if (wall_clock64() - t0 >= g.spin_limit) break;   // bounded: the patch is deferred below
      __builtin_amdgcn_s_sleep(2);
      arrived = __hip_atomic_load(&P.arrive[rb], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= P.n_chunks ? 1 : 0;
    }
    s_arrived = arrived;
  }
  __syncthreads();
  if (s_arrived == 0) {   // (uniform) give up: the patch stays as it is and is completed by the finishing kernel
    if (tid == 0) {
      const int slot = __hip_atomic_fetch_add(P.deferred_count, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      P.deferred[slot] = rb * P.n_chunks + chunk;
    }
    return;
  }

  // ---- the H rows of this wavefront's 16 rows, as the second operand of phase 2 ---------------------------------
  // hb[jj] = -H[row][16 jj + 4 g4 .. + 3]; columns beyond the rank carry nothing (an instance narrower than the
  // launch's rank class has fewer than RC columns of H: the reads stay inside its rows)
  float4 hb[TJ];
  {
    const float* hrow = P.H + (size_t)min(row, N - 1) * P.ldh;
    floatx4 hv[TJ];
    {
#pragma unroll
      for (int jj = 0; jj < TJ; ++jj) load_coherent_f4(hv[jj], hrow + min(16 * jj + 4 * g4, P.ldh - 4));
#pragma unroll
      for (int jj = 0; jj < TJ; ++jj) wait_coherent_loads(hv[jj]);
    }
#pragma unroll
    for (int jj = 0; jj < TJ; ++jj) {
      const int left = R - (16 * jj + 4 * g4);
      hb[jj] = make_float4(left > 0 ? -hv[jj][0] : 0.f, left > 1 ? -hv[jj][1] : 0.f, left > 2 ? -hv[jj][2] : 0.f,
                           left > 3 ? -hv[jj][3] : 0.f);
    }
  }

  // ---- phase 2: Xhat^T = X^T - W^T H^T with the registers of X as the accumulator -----------------------------
  // Two 16-column groups at a time (two independent MFMA chains); a pair is stored as soon as it is complete, so
  // the stores of one pair travel while the next is being multiplied.  Squared row norms over this chunk (eq. pi).
  float sq = 0.f;
  float* const orow = P.Xout + (size_t)min(row, N - 1) * P.ldo;
#pragma unroll
  for (int cc0 = 0; cc0 < KK; cc0 += 2) {
    floatx4 xa[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) xa[u] = floatx4{xr[cc0 + u].x, xr[cc0 + u].y, xr[cc0 + u].z, xr[cc0 + u].w};
#pragma unroll
    for (int jj = 0; jj < TJ; ++jj) {
      float w[2][4];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const float* wp = &Ws[(16 * jj + 4 * g4) * LDW + 16 * (cc0 + u) + r16];
        w[u][0] = wp[0]; w[u][1] = wp[LDW]; w[u][2] = wp[2 * LDW]; w[u][3] = wp[3 * LDW];
      }
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int u = 0; u < 2; ++u)
          xa[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(w[u][q], pick4(hb[jj], q), xa[u], 0, 0, 0);
    }
    if (row_ok) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int col = c0 + 16 * (cc0 + u) + 4 * g4;
        const floatx4 v = xa[u];
        if (col + 3 < D) {
          *reinterpret_cast<float4*>(orow + col) = make_float4(v[0], v[1], v[2], v[3]);
          sq += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
        } else {
#pragma unroll
          for (int q = 0; q < 4; ++q)
            if (col + q < D) {
              orow[col + q] = v[q];
              sq += v[q] * v[q];
            }
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);   // one pair at a time
  }
  sq += __shfl_xor(sq, 16);
  sq += __shfl_xor(sq, 32);
  if (row_ok && g4 == 0) P.rownorm_part[(size_t)chunk * N + row] = sq;
}

}  // namespace ngsgd
