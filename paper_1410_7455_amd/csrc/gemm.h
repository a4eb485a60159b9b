// Grouped fp32 MFMA GEMM for gfx950 (CDNA4).
//
// One launch runs a list of independent problems C = alpha * op(A) * op(B) [+ beta * C]; every
// workgroup owns one (problem, split, tile_m, tile_n) unit.  All matrix products of the NG-SGD step
// go through this kernel: the layer GEMMs (forward A B^T, backward A B, update A^T B) and the
// skinny products of the online preconditioner (H = X W^T, J = H^T X, Xhat = X - H W, K = J J^T,
// L = H^T H, W_{t+1} = A_t B_t; App. B.3 of the paper).
//
// Tiling: 64-lane wavefronts, v_mfma_f32_16x16x4_f32.  A workgroup of WGM x WGN waves computes a
// BM x BN tile; a wave owns (BM/WGM) x (BN/WGN) as TM x TN MFMA tiles.  Operand tiles are staged
// through double-buffered LDS.  An operand whose K index is contiguous in memory is kept as
// [row][BK+4] and feeds four consecutive MFMAs from one ds_read_b128 (lane group g supplies
// k = 4g..4g+3, for A and B alike, so the assignment of k to lanes is consistent); an operand
// whose row index is contiguous is kept as [k][rows+4].
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ngsgd {

constexpr int kMaxGroup = 16;
constexpr int kPrefetch = 2;   // K-blocks in flight from memory per workgroup
constexpr int kXcds = 8;   // accelerator dies (XCDs) of the MI355X, each with a private L2

enum Epilogue : int {
  EPI_STORE = 0,        // C = alpha*acc + beta*C
  EPI_ATOMIC_F32 = 1,   // C += alpha*acc            (split-K, float atomics)
  EPI_ATOMIC_F64 = 2,   // (double)C += alpha*acc    (split-K, double atomics)
  EPI_SUB_ROWNORM = 3,  // C = C - acc; aux[tile_n][row] = sum over the tile's columns of C^2
};

struct GemmProblem {
  const float* A;
  const float* B;
  void* C;
  int M, N, K;
  int lda, ldb, ldc;
  float alpha, beta;
  const double* alpha_dev[3];  // optional device scalars multiplied into alpha
  int tiles_m, tiles_n, splits, k_per_split;
  int tile_begin;              // first workgroup index of this problem
  float* aux;                  // EPI_SUB_ROWNORM: [tiles_n][M] row-norm partials
  double* sumsq;               // SUMSQ_A: [splits*tiles_m] partial sums of squares of A
  long long c_split_stride;    // EPI_STORE with splits > 1: split s writes its partial product to C + s*stride
  const int* gate;             // optional: the problem is skipped unless (*gate & gate_mask) != 0
  int gate_mask;
};

struct GemmGroup {
  int count;
  int total_tiles;
  GemmProblem p[kMaxGroup];
};

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef double doublex4 __attribute__((ext_vector_type(4)));

// Four consecutive 16x16x4 MFMAs on the k values a lane group holds.  The double variant multiplies the fp32
// operands exactly and accumulates in fp64 (v_mfma_f64_16x16x4_f64, same operand and result layout).
__device__ __forceinline__ void mfma_k4(floatx4& c, const float4& a, const float4& b) {
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, b.x, c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, b.y, c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, b.z, c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, b.w, c, 0, 0, 0);
}
__device__ __forceinline__ void mfma_k4(doublex4& c, const float4& a, const float4& b) {
  c = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a.x, (double)b.x, c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a.y, (double)b.y, c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a.z, (double)b.z, c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a.w, (double)b.w, c, 0, 0, 0);
}
__device__ __forceinline__ float pick4(const float4& v, int q) { return q == 0 ? v.x : (q == 1 ? v.y : (q == 2 ? v.z : v.w)); }
__device__ __forceinline__ void mfma_k1(floatx4& c, const float4& a, const float4& b, int q) {
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(pick4(a, q), pick4(b, q), c, 0, 0, 0);
}
__device__ __forceinline__ void mfma_k1(doublex4& c, const float4& a, const float4& b, int q) {
  c = __builtin_amdgcn_mfma_f64_16x16x4f64((double)pick4(a, q), (double)pick4(b, q), c, 0, 0, 0);
}
template <bool ACC64>
struct AccType {
  using type = floatx4;
};
template <>
struct AccType<true> {
  using type = doublex4;
};

// ---- global -> register -> LDS staging ---------------------------------------------------------
// The staging objects keep one global pointer and one LDS offset per 16-byte piece, set up once per tile: the
// K loop only advances the pointers by a constant.  (With the address arithmetic, bounds selects and clamps in
// the loop, a wave that is alone on its SIMD spent about 600 of its 2100 cycles per K-block issuing them.)
// Rows beyond the operand are read from a clamped, valid address and left as they are: row m of A and row n of B
// only ever reach C(m, n), which is not stored for rows outside the problem.  Only the K tail has to be zeroed,
// and only in a tile's last K-block.  Relies on ld being a multiple of 4 that covers the contiguous extent.
//
// K-contiguous operand: element (row, k) at base[row*ld + k]; LDS layout [ROWS][BK+4].
template <int ROWS, int BK, int NT>
struct StageKC {
  static constexpr int F4_PER_ROW = BK / 4;
  static constexpr int TOTAL = ROWS * F4_PER_ROW;
  static constexpr int ITER = (TOTAL + NT - 1) / NT;
  static constexpr int LDS_FLOATS = ROWS * (BK + 4);
  using Regs = floatx4[ITER];   // one K-block's share of this thread; the caller keeps several in flight
  const float* ptr[ITER];   // where this thread's piece of the next K-block starts
  int kq[ITER];             // k offset of the piece inside a K-block
  int lds_off[ITER];        // -1: surplus lane (TOTAL is not a multiple of NT), nothing to store
  float row_ok[ITER];       // 1 for rows inside the operand (only the sum of squares needs it)

  __device__ __forceinline__ void init(const float* __restrict__ base, int ld, int row0, int rows_total, int k_begin,
                                       int tid) {
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      const int f = min(tid + i * NT, TOTAL - 1);
      const int r = f / F4_PER_ROW;
      kq[i] = (f % F4_PER_ROW) * 4;
      const int gr = row0 + r;
      ptr[i] = base + (size_t)min(gr, rows_total - 1) * ld + k_begin + kq[i];
      lds_off[i] = (TOTAL % NT == 0 || tid + i * NT < TOTAL) ? r * (BK + 4) + kq[i] : -1;
      row_ok[i] = (gr < rows_total && lds_off[i] >= 0) ? 1.f : 0.f;
    }
  }
  // loads the K-block that starts at k0 and steps the pointers to the next one; `last`: the block may reach past k_end
  __device__ __forceinline__ void load(Regs& reg, int k0, int k_end, bool last) {
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      const float* p = ptr[i];
      if (last) p -= max(0, k0 + kq[i] - ((k_end - 1) & ~3));   // stay inside the row: the piece is masked anyway
      reg[i] = *reinterpret_cast<const floatx4*>(p);
      ptr[i] += BK;
    }
  }
  // zeroes what lies past k_end (called for a tile's last K-block only, when the registers are consumed)
  __device__ __forceinline__ void mask_tail(Regs& reg, int k0, int k_end) const {
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      const int left = k_end - (k0 + kq[i]);
      reg[i].x = left > 0 ? reg[i].x : 0.f;
      reg[i].y = left > 1 ? reg[i].y : 0.f;
      reg[i].z = left > 2 ? reg[i].z : 0.f;
      reg[i].w = left > 3 ? reg[i].w : 0.f;
    }
  }
  __device__ __forceinline__ void store(const Regs& reg, float* lds) const {
#pragma unroll
    for (int i = 0; i < ITER; ++i)
      if (TOTAL % NT == 0 || lds_off[i] >= 0) *reinterpret_cast<floatx4*>(&lds[lds_off[i]]) = reg[i];
  }
  __device__ __forceinline__ float sumsq(const Regs& reg) const {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < ITER; ++i)
      s += row_ok[i] * (reg[i].x * reg[i].x + reg[i].y * reg[i].y + reg[i].z * reg[i].z + reg[i].w * reg[i].w);
    return s;
  }
  // Operand fragments of a wavefront's T MFMA tiles for k-group kk (16 k values): out[t] holds the four k values
  // 16 kk + 4 g + {0..3} of the tile row that lane r16 supplies.  Tile t covers rows row0 + 16 t + (0..15).
  template <int T>
  __device__ __forceinline__ static void frags(const float* lds, int row0, int r16, int kk, int g, float4 (&out)[T]) {
#pragma unroll
    for (int t = 0; t < T; ++t)
      out[t] = *reinterpret_cast<const float4*>(&lds[(row0 + t * 16 + r16) * (BK + 4) + kk * 16 + 4 * g]);
  }
  // row (inside the wavefront's T tiles) of MFMA tile t, tile row j
  template <int T>
  __device__ __forceinline__ static int tile_row(int t, int j) { return t * 16 + j; }
};

// Row-contiguous operand: element (row, k) at base[k*ld + row]; LDS layout [BK][ROWS+PAD].  T is the number of
// MFMA tiles a wavefront has along this operand's rows.  The tiles are interleaved: tile t covers rows
// row0 + T j + t (j = 0..15), so the T values a lane needs for one k are adjacent in LDS and come with one read of
// the widest width that divides T (one 16-byte read for T = 4 instead of four 4-byte reads).  PAD keeps the
// k rows that the four 16-lane groups of a read touch on different banks.
// With IL false the tiles are not interleaved (tile t covers rows row0 + 16 t + j, four 4-byte reads each): the
// atomic epilogues want a wavefront's 16 lanes on adjacent columns of C.
template <int ROWS, int BK, int NT, int T, bool IL>
struct StageRC {
  static constexpr int VW = !IL ? 1 : ((T % 4 == 0) ? 4 : ((T % 2 == 0) ? 2 : 1));   // floats per LDS read
  static constexpr int PAD = VW == 2 ? 8 : 4;
  static constexpr int LD = ROWS + PAD;
  static constexpr int F4_PER_K = ROWS / 4;
  static constexpr int TOTAL = BK * F4_PER_K;
  static constexpr int ITER = (TOTAL + NT - 1) / NT;
  static constexpr int LDS_FLOATS = BK * LD;
  using Regs = floatx4[ITER];
  const float* ptr[ITER];
  int kq[ITER];             // k index of the piece inside a K-block
  int lds_off[ITER];
  float row_ok[ITER][4];    // per component (rows are the contiguous direction here)
  size_t block_stride;      // BK * ld

  __device__ __forceinline__ void init(const float* __restrict__ base, int ld, int row0, int rows_total, int k_begin,
                                       int tid) {
    block_stride = (size_t)BK * ld;
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      const int f = min(tid + i * NT, TOTAL - 1);
      kq[i] = f / F4_PER_K;
      const int r4 = (f % F4_PER_K) * 4;
      const int gr = row0 + r4;
      ptr[i] = base + (size_t)(k_begin + kq[i]) * ld + min(gr, (rows_total - 1) & ~3);
      lds_off[i] = (TOTAL % NT == 0 || tid + i * NT < TOTAL) ? kq[i] * LD + r4 : -1;
#pragma unroll
      for (int c = 0; c < 4; ++c) row_ok[i][c] = (gr + c < rows_total && lds_off[i] >= 0) ? 1.f : 0.f;
    }
    ld_ = ld;
  }
  int ld_;
  __device__ __forceinline__ void load(Regs& reg, int k0, int k_end, bool last) {
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      const float* p = ptr[i];
      if (last) p -= (size_t)max(0, k0 + kq[i] - (k_end - 1)) * ld_;   // stay inside the operand: masked anyway
      reg[i] = *reinterpret_cast<const floatx4*>(p);
      ptr[i] += block_stride;
    }
  }
  __device__ __forceinline__ void mask_tail(Regs& reg, int k0, int k_end) const {
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      const bool ok = k0 + kq[i] < k_end;
      reg[i].x = ok ? reg[i].x : 0.f;
      reg[i].y = ok ? reg[i].y : 0.f;
      reg[i].z = ok ? reg[i].z : 0.f;
      reg[i].w = ok ? reg[i].w : 0.f;
    }
  }
  __device__ __forceinline__ void store(const Regs& reg, float* lds) const {
#pragma unroll
    for (int i = 0; i < ITER; ++i)
      if (TOTAL % NT == 0 || lds_off[i] >= 0) *reinterpret_cast<floatx4*>(&lds[lds_off[i]]) = reg[i];
  }
  __device__ __forceinline__ float sumsq(const Regs& reg) const {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < ITER; ++i)
      s += row_ok[i][0] * reg[i].x * reg[i].x + row_ok[i][1] * reg[i].y * reg[i].y + row_ok[i][2] * reg[i].z * reg[i].z +
           row_ok[i][3] * reg[i].w * reg[i].w;
    return s;
  }
  template <int T_>
  __device__ __forceinline__ static void frags(const float* lds, int row0, int r16, int kk, int g, float4 (&out)[T_]) {
    static_assert(T_ == T, "tiles per wavefront");
    if (!IL) {
#pragma unroll
      for (int t = 0; t < T; ++t) {
        const float* p = &lds[(kk * 16 + 4 * g) * LD + row0 + t * 16 + r16];
        out[t] = make_float4(p[0], p[LD], p[2 * LD], p[3 * LD]);
      }
      return;
    }
    const float* p = &lds[(kk * 16 + 4 * g) * LD + row0 + r16 * T];
    float v[4][T];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
      for (int t = 0; t < T; t += VW) {
        if (VW == 4) {
          const float4 x = *reinterpret_cast<const float4*>(p + q * LD + t);
          v[q][t] = x.x; v[q][t + 1] = x.y; v[q][t + 2] = x.z; v[q][t + 3] = x.w;
        } else if (VW == 2) {
          const float2 x = *reinterpret_cast<const float2*>(p + q * LD + t);
          v[q][t] = x.x; v[q][t + 1] = x.y;
        } else {
          v[q][t] = p[q * LD + t];
        }
      }
    }
#pragma unroll
    for (int t = 0; t < T; ++t) out[t] = make_float4(v[0][t], v[1][t], v[2][t], v[3][t]);
  }
  template <int T_>
  __device__ __forceinline__ static int tile_row(int t, int j) { return IL ? j * T + t : t * 16 + j; }
};

template <bool KC, int ROWS, int BK, int NT, int T, bool IL>
struct StageSelect {
  using type = StageKC<ROWS, BK, NT>;
};
template <int ROWS, int BK, int NT, int T, bool IL>
struct StageSelect<false, ROWS, BK, NT, T, IL> {
  using type = StageRC<ROWS, BK, NT, T, IL>;
};

// Sum over the 16 lanes of a DPP row, through the vector ALU's cross-lane path (no LDS traffic): xor 1 and xor 2
// inside a quad, then the two mirrors pair quads and half rows.  Every lane ends up with the total.
__device__ __forceinline__ float group16_sum(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xf, 0xf, true));   // quad_perm [1,0,3,2]
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xf, 0xf, true));   // quad_perm [2,3,0,1]
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xf, 0xf, true));  // row_half_mirror
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xf, 0xf, true));  // row_mirror
  return v;
}

// A_KC: A is M x K with K contiguous (else stored K x M).  B_KC: B is N x K with K contiguous
// (else stored K x N).  The product is always sum_k A(m,k) B(n,k).
//
// ACC_CHUNK > 0 selects two-level accumulation: the MFMA chain runs over ACC_CHUNK staged K-blocks from a zero
// accumulator and is then added to a running total with an ordinary (round-to-nearest) fp32 add.  A long MFMA
// chain adds small products into a large accumulator, and the matrix unit does not round those additions to
// nearest, so its error grows linearly with K; the two-level form restores sqrt-like growth.
//
// ACC64 accumulates in fp64 on the fp64 matrix unit (half the fp32 rate).  The factor update needs it: J, K and
// L hold nearly parallel rows while the factor is still turning towards the data, and the weak directions then
// sit in differences that fp32 accumulation wipes out.
template <int BM, int BN, int BK, int WGM, int WGN, bool A_KC, bool B_KC, int EPI, bool SUMSQ_A, int ACC_CHUNK = 0,
          bool ACC64 = false, int PF = kPrefetch>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_kernel(const GemmGroup g) {
  using acc_t = typename AccType<ACC64>::type;
  constexpr int NT = WGM * WGN * 64;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 16, TN = WN / 16;
  static_assert(WM % 16 == 0 && WN % 16 == 0, "wave tile must be a multiple of 16x16");
  static_assert(BK % 16 == 0, "BK must be a multiple of 16");
  // B's tiles set the columns a lane owns: interleaved, they are TN adjacent columns (vector stores); the atomic
  // epilogues keep the 16 lanes of a tile row on adjacent columns instead
  constexpr bool B_IL = EPI == EPI_STORE || EPI == EPI_SUB_ROWNORM;
  using StageA = typename StageSelect<A_KC, BM, BK, NT, TM, true>::type;
  using StageB = typename StageSelect<B_KC, BN, BK, NT, TN, B_IL>::type;
  constexpr int EPI_LDS = (EPI == EPI_SUB_ROWNORM) ? WGN * BM : 0;
  constexpr int LDS_TOTAL = 2 * (StageA::LDS_FLOATS + StageB::LDS_FLOATS);
  __shared__ __attribute__((aligned(16))) float lds[(LDS_TOTAL > EPI_LDS ? LDS_TOTAL : EPI_LDS)];
  __shared__ double red[NT / 64];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int r16 = lane & 15, g4 = lane >> 4;

  // Workgroups go to the eight accelerator dies round-robin by their index, and each die has its own L2: give
  // every die one contiguous eighth of the unit list, so that the workgroups sharing an L2 share operand panels.
  const int per_xcd = (g.total_tiles + kXcds - 1) / kXcds;
  const int unit = ((int)blockIdx.x % kXcds) * per_xcd + (int)blockIdx.x / kXcds;
  if (unit >= g.total_tiles) return;   // the grid is rounded up to a multiple of the die count
  int pi = 0;
  for (int i = 1; i < g.count; ++i)
    if (unit >= g.p[i].tile_begin) pi = i;
  const GemmProblem& P = g.p[pi];
  if (P.gate != nullptr && ((*P.gate) & P.gate_mask) == 0) return;   // uniform over the workgroup
  // Within a split the tiles are numbered along the shorter side of the tile grid first: a die's contiguous run of
  // units then covers a compact patch, all of the small operand's panels but only its own share of the large one's.
  int local = unit - P.tile_begin;
  const int per_split = P.tiles_m * P.tiles_n;
  const int split = local / per_split;
  local -= split * per_split;
  int tm, tn;
  if (P.tiles_m <= P.tiles_n) {
    tm = local % P.tiles_m;
    tn = local / P.tiles_m;
  } else {
    tn = local % P.tiles_n;
    tm = local / P.tiles_n;
  }
  const int m0 = tm * BM, n0 = tn * BN;
  const int k_begin = split * P.k_per_split;
  const int k_end = min(P.K, k_begin + P.k_per_split);
  const int M = P.M, N = P.N;

  // accumulator layout: register r of lane l holds tile column l%16 and tile row 4*(l/16)+r for
  // v_mfma_f32_16x16x4_f32, tile row 4*r+(l/16) for v_mfma_f64_16x16x4_f64; where a tile's rows and columns lie
  // in the wavefront's part of C is the operand staging's business (interleaved for row-contiguous operands)
  auto local_row = [&](const int i, const int r) {
    return wm * WM + StageA::template tile_row<TM>(i, ACC64 ? 4 * r + g4 : 4 * g4 + r);
  };
  auto local_col = [&](const int j) { return wn * WN + StageB::template tile_row<TN>(j, r16); };
  // C - acc: the old values of C do not depend on the product; they are requested before the K loop and arrive
  // under it.  A lane that owns two adjacent columns (interleaved B, TN = 2) moves them as one 8-byte word.
  constexpr bool SUB = EPI == EPI_SUB_ROWNORM;
  constexpr bool SUB_V2 = SUB && !B_KC && TN == 2;
  float c_old[SUB ? TM : 1][SUB ? 4 : 1][SUB ? TN : 1];
  auto request_c_old = [&]() {
    const float* C = static_cast<const float*>(P.C);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = m0 + local_row(i, r);
        const int col0 = n0 + local_col(0);
        if (SUB_V2 && row < M && col0 + 1 < N) {
          const float2 v = *reinterpret_cast<const float2*>(C + (size_t)row * P.ldc + col0);
          c_old[i][r][0] = v.x;
          c_old[i][r][TN - 1] = v.y;
        } else {
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            const int col = n0 + local_col(j);
            c_old[i][r][j] = (row < M && col < N) ? C[(size_t)row * P.ldc + col] : 0.f;
          }
        }
      }
  };

  float* const As = lds;                             // two buffers of StageA::LDS_FLOATS
  float* const Bs = lds + 2 * StageA::LDS_FLOATS;    // two buffers of StageB::LDS_FLOATS

  acc_t acc[TM][TN];
  acc_t total[ACC_CHUNK > 0 ? TM : 1][ACC_CHUNK > 0 ? TN : 1];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      acc[i][j] = acc_t{0, 0, 0, 0};
      if (ACC_CHUNK > 0) total[i][j] = acc_t{0, 0, 0, 0};
    }

  float ssq = 0.f;
  const int nk = (k_end - k_begin + BK - 1) / BK;
  auto fold_chunk = [&](const int i, const bool more) {
    if (ACC_CHUNK > 0 && ((i + 1) % (ACC_CHUNK > 0 ? ACC_CHUNK : 1) == 0 || !more)) {
#pragma unroll
      for (int ti = 0; ti < TM; ++ti)
#pragma unroll
        for (int tj = 0; tj < TN; ++tj) {
          total[ti][tj] += acc[ti][tj];
          acc[ti][tj] = acc_t{0, 0, 0, 0};
        }
    }
  };
  // Software pipeline: K-block i is multiplied out of LDS buffer i & 1 while block i+1 waits in registers to be
  // written to the other buffer and blocks i+2 .. i+PF are still on their way from memory.  Register set u holds
  // block i+1 for i = u (mod PF).  Blocks are requested in increasing order, so one set of pointers serves all.
  StageA sa;
  StageB sb;
  typename StageA::Regs ra[PF];
  typename StageB::Regs rb[PF];
  sa.init(P.A, P.lda, m0, M, k_begin, tid);
  sb.init(P.B, P.ldb, n0, N, k_begin, tid);
  auto fetch = [&](const int blk, const int set) {   // block `blk` of this tile into register set `set`
    const int k0 = k_begin + blk * BK;
    const bool last = blk == nk - 1;
    sa.load(ra[set], k0, k_end, last);
    sb.load(rb[set], k0, k_end, last);
  };
  auto commit = [&](const int blk, const int set, const int buf) {   // register set -> LDS buffer
    if (blk == nk - 1) {
      sa.mask_tail(ra[set], k_begin + blk * BK, k_end);
      sb.mask_tail(rb[set], k_begin + blk * BK, k_end);
    }
    if (SUMSQ_A) ssq += sa.sumsq(ra[set]);
    sa.store(ra[set], As + buf * StageA::LDS_FLOATS);
    sb.store(rb[set], Bs + buf * StageB::LDS_FLOATS);
  };
  if (nk > 0) {
    fetch(0, 0);
    if (SUB) request_c_old();   // behind the first operand block: the K loop starts while the tile of C streams in
    commit(0, 0, 0);
#pragma unroll
    for (int u = 0; u < PF; ++u)
      if (1 + u < nk) fetch(1 + u, u);
  }
  if (SUB && nk <= 0) request_c_old();
  __syncthreads();
  // one K-block: multiply block i out of LDS, then pass block i+1 from register set u to LDS and refill the set
  auto block_step = [&](const int i, const int u, const bool steady) {
    const int cur = i & 1;
    const bool more = steady || i + 1 < nk;
    const float* a_lds = As + cur * StageA::LDS_FLOATS;
    const float* b_lds = Bs + cur * StageB::LDS_FLOATS;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      float4 af[TM], bf[TN];
      StageA::template frags<TM>(a_lds, wm * WM, r16, kk, g4, af);
      StageB::template frags<TN>(b_lds, wn * WN, r16, kk, g4, bf);
      // one k value at a time over all TM x TN accumulators: consecutive MFMAs are independent, so a wave
      // that is alone on its SIMD still issues them back to back
#pragma unroll
      for (int kq = 0; kq < 4; ++kq)
#pragma unroll
        for (int ti = 0; ti < TM; ++ti)
#pragma unroll
          for (int tj = 0; tj < TN; ++tj) mfma_k1(acc[ti][tj], af[ti], bf[tj], kq);
    }
    fold_chunk(i, more);
    // nothing below may move above the products: touching the prefetched registers makes the wave wait for them
    __builtin_amdgcn_sched_barrier(0);
    if (more) {
      commit(i + 1, u, cur ^ 1);   // (in the steady state block i+1 is never the last one: no tail to mask)
      if (steady || i + 1 + PF < nk) fetch(i + 1 + PF, u);
    }
    __syncthreads();
  };
  int it = 0;
  // steady state: every block of the trip has a successor to store and a block PF ahead to fetch, so the body is
  // straight-line code with a fixed number of loads in flight
  for (; it + 2 * PF < nk; it += PF) {
#pragma unroll
    for (int u = 0; u < PF; ++u) block_step(it + u, u, true);
  }
  for (; it < nk; it += PF) {
#pragma unroll
    for (int u = 0; u < PF; ++u)
      if (it + u < nk) block_step(it + u, u, false);   // uniform over the workgroup
  }
  if (ACC_CHUNK > 0) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[i][j] = total[i][j];
  }

  if (SUMSQ_A) {
    // every element of A's row block is staged exactly once by the tile_n == 0 workgroups
    double s = (double)ssq;
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if (lane == 0) red[wave] = s;
    __syncthreads();
    if (tid == 0 && tn == 0 && P.sumsq != nullptr) {
      double t = 0.0;
      for (int w = 0; w < NT / 64; ++w) t += red[w];
      P.sumsq[split * P.tiles_m + tm] = t;
    }
  }

  float alpha = P.alpha;
#pragma unroll
  for (int i = 0; i < 3; ++i)
    if (P.alpha_dev[i] != nullptr) alpha *= (float)(*P.alpha_dev[i]);

  if (EPI == EPI_SUB_ROWNORM) {
    float* C = static_cast<float*>(P.C);
    float* rowsum = lds;  // [WGN][BM], operand tiles are no longer needed
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int lrow = local_row(i, r);
        const int row = m0 + lrow;
        float sq = 0.f;
        float v[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) v[j] = c_old[SUB ? i : 0][SUB ? r : 0][SUB ? j : 0] - (float)acc[i][j][r];
        const int col0 = n0 + local_col(0);
        if (SUB_V2 && row < M && col0 + 1 < N) {
          *reinterpret_cast<float2*>(C + (size_t)row * P.ldc + col0) = make_float2(v[0], v[TN - 1]);
          sq = v[0] * v[0] + v[TN - 1] * v[TN - 1];
        } else {
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            const int col = n0 + local_col(j);
            if (row < M && col < N) {
              C[(size_t)row * P.ldc + col] = v[j];
              sq += v[j] * v[j];
            }
          }
        }
        sq = group16_sum(sq);
        if (r16 == 0) rowsum[wn * BM + lrow] = sq;
      }
    }
    __syncthreads();
    for (int lrow = tid; lrow < BM; lrow += NT) {
      const int row = m0 + lrow;
      if (row < M) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < WGN; ++w) s += rowsum[w * BM + lrow];
        P.aux[(size_t)tn * M + row] = s;
      }
    }
    return;
  }

  if (EPI == EPI_STORE && !B_KC && (TN == 2 || TN == 4)) {
    // a lane owns TN adjacent columns of each of its rows: one vector store where the row allows it
    float* const C = static_cast<float*>(P.C) + (size_t)split * P.c_split_stride;
    const int col0 = n0 + local_col(0);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = m0 + local_row(i, r);
        if (row >= M || col0 >= N) continue;
        float v[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j)
          v[j] = ACC64 ? (float)((double)alpha * (double)acc[i][j][r]) : alpha * (float)acc[i][j][r];
        float* c = C + (size_t)row * P.ldc + col0;
        if (col0 + TN <= N && (reinterpret_cast<uintptr_t>(c) & (4 * TN - 1)) == 0) {
          if (TN == 4) {
            float4 o = make_float4(v[0], v[1], v[2], v[TN - 1]);
            if (P.beta != 0.f) {
              const float4 old = *reinterpret_cast<const float4*>(c);
              o.x += P.beta * old.x; o.y += P.beta * old.y; o.z += P.beta * old.z; o.w += P.beta * old.w;
            }
            *reinterpret_cast<float4*>(c) = o;
          } else {
            float2 o = make_float2(v[0], v[1]);
            if (P.beta != 0.f) {
              const float2 old = *reinterpret_cast<const float2*>(c);
              o.x += P.beta * old.x; o.y += P.beta * old.y;
            }
            *reinterpret_cast<float2*>(c) = o;
          }
        } else {
#pragma unroll
          for (int j = 0; j < TN; ++j)
            if (col0 + j < N) c[j] = (P.beta != 0.f) ? v[j] + P.beta * c[j] : v[j];
        }
      }
    }
    return;
  }

#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + local_col(j);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = m0 + local_row(i, r);
        if (row < M && col < N) {
          const float v = ACC64 ? (float)((double)alpha * (double)acc[i][j][r]) : alpha * (float)acc[i][j][r];
          if (EPI == EPI_STORE) {
            float* c = static_cast<float*>(P.C) + (size_t)split * P.c_split_stride + (size_t)row * P.ldc + col;
            *c = (P.beta != 0.f) ? v + P.beta * (*c) : v;
          } else if (EPI == EPI_ATOMIC_F32) {
            unsafeAtomicAdd(static_cast<float*>(P.C) + (size_t)row * P.ldc + col, v);
          } else if (EPI == EPI_ATOMIC_F64) {
            unsafeAtomicAdd(static_cast<double*>(P.C) + (size_t)row * P.ldc + col,
                            ACC64 ? (double)alpha * (double)acc[i][j][r] : (double)v);
          }
        }
      }
    }
  }
}

// ---- host side -------------------------------------------------------------------------------
struct GemmDesc {  // what a caller states; tiling is filled in by the launcher
  const float* A = nullptr;
  const float* B = nullptr;
  void* C = nullptr;
  int M = 0, N = 0, K = 0;
  int lda = 0, ldb = 0, ldc = 0;
  float alpha = 1.f, beta = 0.f;
  const double* alpha_dev[3] = {nullptr, nullptr, nullptr};
  float* aux = nullptr;
  double* sumsq = nullptr;
  int splits = 1;  // requested split-K factor (atomic epilogues, or EPI_STORE with c_split_stride)
  long long c_split_stride = 0;
  const int* gate = nullptr;
  int gate_mask = 0;
};

template <int BM, int BN, int BK>
inline void plan_tiles(const GemmDesc& d, GemmProblem& p) {
  p.A = d.A; p.B = d.B; p.C = d.C;
  p.M = d.M; p.N = d.N; p.K = d.K;
  p.lda = d.lda; p.ldb = d.ldb; p.ldc = d.ldc;
  p.alpha = d.alpha; p.beta = d.beta;
  for (int i = 0; i < 3; ++i) p.alpha_dev[i] = d.alpha_dev[i];
  p.aux = d.aux; p.sumsq = d.sumsq;
  p.c_split_stride = d.c_split_stride;
  p.gate = d.gate; p.gate_mask = d.gate_mask;
  p.tiles_m = (d.M + BM - 1) / BM;
  p.tiles_n = (d.N + BN - 1) / BN;
  const int ksteps = (d.K + BK - 1) / BK;
  int splits = d.splits < 1 ? 1 : d.splits;
  if (splits > ksteps) splits = ksteps > 0 ? ksteps : 1;
  const int steps_per = (ksteps + splits - 1) / splits;
  p.k_per_split = (steps_per > 0 ? steps_per : 1) * BK;
  p.splits = ksteps > 0 ? (ksteps + steps_per - 1) / steps_per : 1;
}

template <int BM, int BN, int BK, int WGM, int WGN, bool A_KC, bool B_KC, int EPI, bool SUMSQ_A, int ACC_CHUNK = 0,
          bool ACC64 = false, int PF = kPrefetch>
inline hipError_t launch_gemm_group(const GemmDesc* descs, int count, hipStream_t stream) {
  int done = 0;
  while (done < count) {
    GemmGroup grp;
    const int n = (count - done) < kMaxGroup ? (count - done) : kMaxGroup;
    grp.count = n;
    int total = 0;
    for (int i = 0; i < n; ++i) {
      plan_tiles<BM, BN, BK>(descs[done + i], grp.p[i]);
      grp.p[i].tile_begin = total;
      total += grp.p[i].tiles_m * grp.p[i].tiles_n * grp.p[i].splits;
    }
    grp.total_tiles = total;
    if (total > 0) {
      hipLaunchKernelGGL((gemm_kernel<BM, BN, BK, WGM, WGN, A_KC, B_KC, EPI, SUMSQ_A, ACC_CHUNK, ACC64, PF>),
                         dim3((total + kXcds - 1) / kXcds * kXcds),
                         dim3(WGM * WGN * 64), 0, stream, grp);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
    done += n;
  }
  return hipSuccess;
}

// number of K splits a problem is actually planned with
template <int BM, int BN, int BK>
inline int planned_splits(const GemmDesc& d) {
  GemmProblem p;
  plan_tiles<BM, BN, BK>(d, p);
  return p.splits;
}

// number of sumsq partials the SUMSQ_A variant writes for a problem planned with these tiles
template <int BM, int BN, int BK>
inline int planned_sumsq_partials(const GemmDesc& d) {
  GemmProblem p;
  plan_tiles<BM, BN, BK>(d, p);
  return p.splits * p.tiles_m;
}

}  // namespace ngsgd
