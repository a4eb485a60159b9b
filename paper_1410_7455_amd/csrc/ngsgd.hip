// C ABI of the NG-SGD minibatch-step library: host-side orchestration of the HIP kernels.
// Declarations and argument contracts are in include/ngsgd.h.
#include "ngsgd.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <new>
#include <vector>

#include "fused_apply.h"
#include "gemm.h"
#include "init.h"
#include "kernels.h"
#include "simple_ng.h"
#include "small_update.h"
#include "state.h"

using namespace ngsgd;

namespace {

thread_local int g_last_hip_error = 0;

#define HIP_TRY(expr)                         \
  do {                                        \
    hipError_t e__ = (expr);                  \
    if (e__ != hipSuccess) {                  \
      g_last_hip_error = (int)e__;            \
      return NGSGD_EHIP;                      \
    }                                         \
  } while (0)
#define NG_TRY(expr)                \
  do {                              \
    int rc__ = (expr);              \
    if (rc__ != NGSGD_OK) return rc__; \
  } while (0)
#define LAUNCH_CHECK() HIP_TRY(hipGetLastError())

inline int pad32(int x) { return (x + 31) / 32 * 32; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Carves typed arrays out of a caller-provided device workspace; with base == nullptr it only sizes.
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base(static_cast<char*>(b)) {}
  template <typename T>
  T* take(size_t n) {
    off = align_up(off, 256);
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += n * sizeof(T);
    return p;
  }
};

// ---- optional per-category kernel timing with HIP events on the launch stream ----------------------
struct Profiler {
  bool on = false;
  std::vector<hipEvent_t> pool;
  struct Rec {
    int cat;
    size_t e0;
  };
  std::vector<Rec> recs;
  size_t used = 0;
  size_t dropped = 0;   // launch groups that found the event pool full since the last read
};
Profiler g_prof;
constexpr size_t kProfMaxEvents = 1 << 16;

struct ProfScope {
  hipStream_t s;
  bool active = false;
  size_t e0 = 0;
  ProfScope(int cat, hipStream_t stream) : s(stream) {
    if (!g_prof.on) return;
    if (g_prof.used + 2 > kProfMaxEvents) {
      g_prof.dropped += 1;
      return;
    }
    while (g_prof.pool.size() < g_prof.used + 2) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) return;
      g_prof.pool.push_back(e);
    }
    e0 = g_prof.used;
    g_prof.used += 2;
    g_prof.recs.push_back({cat, e0});
    active = hipEventRecord(g_prof.pool[e0], s) == hipSuccess;
  }
  ~ProfScope() {
    if (active) (void)hipEventRecord(g_prof.pool[e0 + 1], s);
  }
};

constexpr int kSumsqMax = 1024;   // partial sums of squares per preconditioner call
constexpr int kWideRow = 2048;    // rows at least this wide get 512-thread workgroups in the row-wise kernels
constexpr int kTargetBlocks = 512;

inline int rank_class(int rank) { return rank <= 32 ? 32 : (rank <= 80 ? 80 : 96); }

}  // namespace

// The factor updates of a network's instances run on side streams so that they overlap the rest of the step and
// the next step's forward / backward pass; the new factor is first needed by the next preconditioning.  The
// instances are split over kSideStreams streams by the moment their matrix exists (the last layer's derivatives
// and all layer inputs after the forward pass, the other derivatives as the backward pass produces them), so that
// each group's products H, J and its R x R work start as early as possible.  Two streams are the default (the last
// layer's derivatives and the layer inputs; the other derivatives after the backward pass): a third, which starts the
// upper hidden layers' derivatives in the middle of the backward pass, measured 1 - 2 % slower on the speech-shaped
// network (its small launches share the chip with the backward pass, and every further hardware queue in use
// lengthens the gaps between dependent kernels on all of them, plain steps included).
constexpr int kSideStreams = 3;          // most
constexpr int kDefaultSideStreams = 2;
struct SideSync {
  hipStream_t stream = nullptr;
  hipEvent_t inputs_ready = nullptr;   // recorded on the caller's stream: the group's matrices exist
  hipEvent_t hj_done = nullptr;        // recorded on the side stream: H, J and the partial sums of tr(X X^T) are final
  hipEvent_t outputs_done = nullptr;   // recorded on the caller's stream: the last reader of W_t (Xhat) has been enqueued
  hipEvent_t done = nullptr;           // recorded on the side stream: W_{t+1}, D_{t+1}, rho_{t+1} are final
  bool pending = false;                // `done` has been recorded and the stepping stream has not waited for it yet
  hipStream_t owner = nullptr;         // the stream the network's latest step was issued on
};

// ---------------------------------------------------------------------------------------------------
struct ngsgd_precond {
  int dim = 0, rank = 0, max_batch = 0;
  double alpha = 4.0, num_samples_history = 2000.0, epsilon = 1e-10;
  int update_period = 4, always_update_first = 10;
  int64_t t = 0;
  int ldw = 0;   // leading dimension of W and J
  int ldh = 0;   // leading dimension of H and A_t (= rank class)
  PrecondScalars* st = nullptr;
  float* zero_region = nullptr;   // [arrival counters, deferred count | H | K | L], cleared before each call
  int clean_rows = 0;             // the counters and this many rows of H are known to be clear (left so by the
                                  // finishing kernel of a call that went through the fused apply kernel)
  size_t zero_floats_all = 0;
  size_t arrive_slots = 0;        // arrival counters of the fused apply kernel, one per block of 64 rows, and
  int* arrive = nullptr;          // (last slot) the number of patches it deferred; padded to 256 bytes
  int* deferred = nullptr;        // list of deferred patches
  float* H = nullptr;
  float* J = nullptr;
  double* K = nullptr;
  double* L = nullptr;
  float* W = nullptr;
  float* At = nullptr;
  float* rownorm_part = nullptr;
  int max_col_tiles = 0;
  double* sumsq_part = nullptr;
  double* prow = nullptr;
  // initialisation scratch
  int n_init_max = 0;
  double* Ai = nullptr;
  double* Vi = nullptr;
  double* Qi = nullptr;
  double* init_stat = nullptr;
  int* init_cnt = nullptr;
  InitGroup* init_group = nullptr;   // device copy of the instance list of an initialisation this instance leads
  int* idx = nullptr;
  double* vwork = nullptr;
  double2* rotlog = nullptr;      // Jacobi rotation log of the latest factor update
  EigWork* eigwork = nullptr;
  bool owned_by_net = false;
  SideSync* sync = nullptr;   // set for instances of a network
  int last_N = 0;             // rows of the latest call
  int n_sumsq = 0;            // partial sums of tr(X X^T) its H product left in sumsq_part
};

namespace {

void precond_layout(ngsgd_precond& p, Carver& c) {
  const int R = p.rank, D = p.dim, NB = p.max_batch;
  p.ldw = pad32(D);
  p.ldh = R > 0 ? rank_class(R) : 0;
  p.st = c.take<PrecondScalars>(1);
  p.prow = c.take<double>(NB);
  if (R == 0) return;
  const size_t h_floats = (size_t)NB * p.ldh, kl_floats = (size_t)4 * R * R;   // ldh is a multiple of 16
  p.arrive_slots = align_up((size_t)(NB + kFusedRows - 1) / kFusedRows + 1, 64);
  p.zero_floats_all = p.arrive_slots + h_floats + kl_floats;
  p.zero_region = c.take<float>(p.zero_floats_all);
  if (p.zero_region) {
    p.arrive = reinterpret_cast<int*>(p.zero_region);
    p.H = p.zero_region + p.arrive_slots;
    p.K = reinterpret_cast<double*>(p.H + h_floats);
    p.L = p.K + (size_t)R * R;
  }
  p.J = c.take<float>((size_t)R * p.ldw);
  p.W = c.take<float>((size_t)R * p.ldw);
  p.At = c.take<float>((size_t)R * p.ldh);
  p.max_col_tiles = (D + 63) / 64;
  p.rownorm_part = c.take<float>((size_t)p.max_col_tiles * NB);
  p.sumsq_part = c.take<double>(kSumsqMax);
  p.deferred = c.take<int>(kSumsqMax);
  p.n_init_max = NB < D ? NB : D;
  const size_t np_init = (size_t)(p.n_init_max + kInitPair - 1) / kInitPair * kInitPair;
  p.Ai = c.take<double>(np_init * np_init);
  p.Vi = c.take<double>(np_init * np_init);
  p.Qi = c.take<double>(np_init / kInitPair * kInitPair * kInitPair);
  p.init_stat = c.take<double>(2);
  p.init_cnt = c.take<int>(4);
  p.init_group = c.take<InitGroup>(1);
  p.idx = c.take<int>(kMaxRank);
  p.vwork = c.take<double>((size_t)kMaxRank + D);
  {
    const int m = (R + 1) & ~1;
    const size_t rounds = ((size_t)kMaxSweeps * (m - 1 > 0 ? m - 1 : 1) + kEigvecChunk - 1) / kEigvecChunk * kEigvecChunk;
    p.rotlog = c.take<double2>((rounds + kEigvecChunk) * (m / 2));   // padded: the log is read in whole chunks
    p.eigwork = c.take<EigWork>(1);
  }
}

int precond_check_config(int dim, int rank, int max_batch, float alpha, float S, float eps, int period, int first) {
  if (dim < 1 || rank < 0 || rank > NGSGD_MAX_RANK || rank >= dim || max_batch < 1) return NGSGD_EINVAL;
  if (!(alpha >= 0.f) || !(S > 0.f) || !(eps > 0.f) || period < 1 || first < 0) return NGSGD_EINVAL;
  return NGSGD_OK;
}

void precond_configure(ngsgd_precond& p, int dim, int rank, int max_batch, float alpha, float S, float eps,
                       int period, int first) {
  p.dim = dim;
  p.rank = rank;
  p.max_batch = max_batch;
  p.alpha = alpha;
  p.num_samples_history = S;
  p.epsilon = eps;
  p.update_period = period;
  p.always_update_first = first;
  p.t = 0;
}

bool g_attr_done = false;
constexpr int kEigLdsReserve = 126 * 1024;   // dynamic LDS of a large eigen-update workgroup (of 160 KB per compute unit)
constexpr int kEigReserveFromRank = 48;
constexpr int kEigvecLdsReserve = 76 * 1024;   // on top of the 48 KB of the staged rotation log

int ensure_kernel_attributes() {
  if (g_attr_done) return NGSGD_OK;
  const int max_dyn = std::max(kEigLdsReserve, 2 * kMaxRank * (kMaxRank | 1) * (int)sizeof(double));
  HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(eig_update_kernel<1, kEigThreads>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, max_dyn));
  HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(eig_update_kernel<2, kEigThreads>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, max_dyn));
  HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(eig_update_kernel<kEigMaxItems, kEigThreads>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, max_dyn));
  HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(eigvec_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              kEigvecLdsReserve));
  {
    const int orth_dyn = kMaxRank * (kMaxRank + 1) * (int)sizeof(double);
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(orth_fix_kernel<2>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, orth_dyn));
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(orth_fix_kernel<3>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, orth_dyn));
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(orth_fix_kernel<5>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, orth_dyn));
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(orth_fix_kernel<6>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, orth_dyn));
  }
  HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(init_block_solve_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kInitSolveLds));
  g_attr_done = true;
  return NGSGD_OK;
}

inline int choose_splits(int tiles, int ksteps) {
  int s = kTargetBlocks / (tiles > 0 ? tiles : 1);
  if (s < 1) s = 1;
  if (s > ksteps) s = ksteps;
  return s < 1 ? 1 : s;
}

// ---- GEMM dispatch ---------------------------------------------------------------------------------
constexpr int BK = 16;

enum LayerGemm { GEMM_FWD, GEMM_BWD, GEMM_UPD };
constexpr int LBK = 32;             // K-block of the layer GEMMs
constexpr int kBwdAccChunk = 4;     // K-blocks per MFMA chain in the backward GEMM (128 products per chain)
constexpr int kMaxBwdSplits = 8;    // split-K slabs of the backward GEMM, summed by the nonlinearity's backward kernel

// Tile shapes of the layer GEMMs.  The products of a minibatch step are small next to the chip (a few hundred
// 64x64 tiles for 256 compute units), so what decides the time is how evenly the tiles fill it: every shape is
// priced as (rounds of 512 workgroups) x (tile area), and the cheapest is taken (the first listed among equals).
enum LayerTile { TILE_64x64, TILE_64x48, TILE_64x80, TILE_64x96, TILE_32x96, TILE_128x128, TILE_COUNT };
constexpr int kTileBM[TILE_COUNT] = {64, 64, 64, 64, 32, 128};
constexpr int kTileBN[TILE_COUNT] = {64, 48, 80, 96, 96, 128};
constexpr int kComputeUnits = 256;

// Wavefronts per workgroup of each tile shape (see launch_layer_tile) and what a workgroup of that shape gets done
// per unit of tile area and time relative to a four-wavefront one when each fills a compute unit's round.
constexpr int kTileWaves[TILE_COUNT] = {8, 4, 4, 12, 4, 4};
inline LayerTile pick_layer_tile(const GemmDesc* d, int n) {
  LayerTile best = TILE_64x64;
  double best_cost = 0.0;
  for (int t = 0; t < TILE_COUNT; ++t) {
    long long tiles = 0;
    for (int i = 0; i < n; ++i)
      tiles += (long long)((d[i].M + kTileBM[t] - 1) / kTileBM[t]) * ((d[i].N + kTileBN[t] - 1) / kTileBN[t]) *
               std::max(1, d[i].splits);
    // eight wavefronts per compute unit make a round (two workgroups of four, or one of eight or twelve): one
    // four-wavefront workgroup alone leaves the matrix unit idle while it waits on LDS and memory
    const int per_cu = std::max(1, 8 / kTileWaves[t]);
    const double rounds = (double)((tiles + per_cu * kComputeUnits - 1) / (per_cu * kComputeUnits));
    const double area = (double)kTileBM[t] * kTileBN[t] * per_cu;
    // a large tile does more work per byte staged: it wins once the rounds are many; twelve wavefronts on one
    // 64 x 96 tile get through a round faster than two four-wavefront workgroups on 64 x 48 tiles each (measured
    // on the 512 x 3000 x 301 product: 14.5 against 15.8 us)
    const double speed = t == TILE_128x128 ? 1.25 : (kTileWaves[t] == 12 ? 1.09 : 1.0);
    const double cost = rounds * area / speed;
    if (t == 0 || cost < best_cost) {
      best_cost = cost;
      best = (LayerTile)t;
    }
  }
  return best;
}

template <bool A_KC, bool B_KC, int CHUNK>
hipError_t launch_layer_tile(LayerTile t, const GemmDesc* d, int n, hipStream_t s) {
  switch (t) {
    case TILE_64x48: return launch_gemm_group<64, 48, LBK, 4, 1, A_KC, B_KC, EPI_STORE, false, CHUNK>(d, n, s);
    case TILE_64x80: return launch_gemm_group<64, 80, LBK, 4, 1, A_KC, B_KC, EPI_STORE, false, CHUNK>(d, n, s);
    case TILE_64x96: return launch_gemm_group<64, 96, LBK, 4, 3, A_KC, B_KC, EPI_STORE, false, CHUNK>(d, n, s);
    case TILE_32x96: return launch_gemm_group<32, 96, LBK, 2, 2, A_KC, B_KC, EPI_STORE, false, CHUNK>(d, n, s);
    case TILE_128x128: return launch_gemm_group<128, 128, LBK, 2, 2, A_KC, B_KC, EPI_STORE, false, CHUNK>(d, n, s);
    default: return launch_gemm_group<64, 64, LBK, 4, 2, A_KC, B_KC, EPI_STORE, false, CHUNK>(d, n, s);
  }
}

int launch_layer_gemms(LayerGemm kind, const GemmDesc* d, int n, hipStream_t s) {
  ProfScope prof(kind == GEMM_FWD ? NGSGD_PROF_GEMM_FWD : (kind == GEMM_BWD ? NGSGD_PROF_GEMM_BWD : NGSGD_PROF_GEMM_UPD),
                 s);
  const LayerTile t = pick_layer_tile(d, n);
  hipError_t e = hipSuccess;
  switch (kind) {
    case GEMM_FWD: e = launch_layer_tile<true, true, 0>(t, d, n, s); break;
    case GEMM_BWD: e = launch_layer_tile<true, false, kBwdAccChunk>(t, d, n, s); break;   // long K: two-level sums
    case GEMM_UPD: e = launch_layer_tile<false, false, 0>(t, d, n, s); break;
  }
  HIP_TRY(e);
  return NGSGD_OK;
}

// H = X W^T (split over D, float atomics) with the sum of squares of X as a by-product; two-level accumulation
// (MFMA chains of 64 products) keeps the rounding error of a long split at the level of a short one
constexpr int HBK = 32;          // K-block of the H product
constexpr int kHAccChunk = 2;
template <int RC>
hipError_t launch_h(const GemmDesc* d, int n, hipStream_t s) {
  return launch_gemm_group<64, RC, HBK, 4, 1, true, true, EPI_ATOMIC_F32, true, kHAccChunk>(d, n, s);
}
// J = H^T X, accumulated in fp64 and rounded once to fp32; narrow column tiles instead of a split over the rows
template <int RC>
hipError_t launch_j(const GemmDesc* d, int n, hipStream_t s) {
  if (RC == 32) return launch_gemm_group<32, 32, 32, 2, 2, false, false, EPI_STORE, false, 0, true>(d, n, s);
  return launch_gemm_group<RC, 32, 32, RC / 16, 2, false, false, EPI_STORE, false, 0, true>(d, n, s);
}
// W_{t+1} = A_t B_t
template <int RC>
hipError_t launch_wnew(const GemmDesc* d, int n, hipStream_t s) {
  return launch_gemm_group<RC, 64, BK, RC / 16, 2, true, false, EPI_STORE, false>(d, n, s);
}

template <typename F32, typename F80, typename F96>
hipError_t by_rank_class(int rc, F32 f32, F80 f80, F96 f96) {
  return rc == 32 ? f32() : (rc == 80 ? f80() : f96());
}

// R x R Gram products of the factor update (K = J J^T, L = H^T H, W W^T), fp64 accumulation across the splits of the
// long dimension.  Ranks up to 32: one 32 x 32 tile per instance; above: 64 x 64 tiles (a single 80 x 80 tile with one
// row of MFMA tiles per wavefront was measured slower at rank 80: 399 instead of 387 us for the 512 x 5000 call,
// fewer and longer workgroups)
template <bool KC>
hipError_t launch_small_gram(int rc, const GemmDesc* d, int n, hipStream_t s) {
  if (rc == 32) return launch_gemm_group<32, 32, BK, 2, 1, KC, KC, EPI_ATOMIC_F64, false, 0, true>(d, n, s);
  return launch_gemm_group<64, 64, BK, 2, 2, KC, KC, EPI_ATOMIC_F64, false, 0, true>(d, n, s);
}
constexpr int kGramMinSplitSteps = 4;   // K-blocks per split of a 32 x 32 tile at least: below that the atomic epilogue dominates
inline int gram_splits(int rc, int rank, int instances, int k) {
  const int ksteps = (k + BK - 1) / BK;
  if (rc == 32) return std::min(choose_splits(instances, ksteps), std::max(1, ksteps / kGramMinSplitSteps));
  const int tiles = ((rank + 63) / 64) * ((rank + 63) / 64);
  return choose_splits(tiles * instances, ksteps);
}

struct PrecondCall {
  ngsgd_precond* p;
  float* M;
  int ld;
  int N;
  float* gamma_out;
  float* rownorm2_out;
};

int run_init(const std::vector<PrecondCall>& calls, hipStream_t s) {
  ProfScope prof(NGSGD_PROF_INIT, s);
  size_t done = 0;
  while (done < calls.size()) {
    InitGroup g;
    const int n = (int)std::min<size_t>(kMaxInstances, calls.size() - done);
    g.count = n;
    int n_max = 0, ldw_max = 0, r_max = 0;
    for (int i = 0; i < n; ++i) {
      const PrecondCall& c = calls[done + i];
      ngsgd_precond& p = *c.p;
      InitArgs& a = g.a[i];
      a.st = p.st;
      a.M = c.M;
      a.ld = c.ld;
      a.N = c.N;
      a.D = p.dim;
      a.R = p.rank;
      a.use_cov = p.dim <= c.N ? 1 : 0;
      a.n = a.use_cov ? p.dim : c.N;
      a.np = (a.n + kInitPair - 1) / kInitPair * kInitPair;
      a.A = p.Ai;
      a.V = p.Vi;
      a.Q = p.Qi;
      a.stat = p.init_stat;
      a.cnt = p.init_cnt;
      a.idx = p.idx;
      a.W = p.W;
      a.ldw = p.ldw;
      a.vwork = p.vwork;
      n_max = std::max(n_max, a.n);
      ldw_max = std::max(ldw_max, p.ldw);
      r_max = std::max(r_max, p.rank);
      g.alpha = p.alpha;       // one configuration per group (instances of one net share it)
      g.epsilon = p.epsilon;
    }
    const int np_max = (n_max + kInitPair - 1) / kInitPair * kInitPair;
    const int tiles = np_max / 32;
    InitGroup* gd = calls[done].p->init_group;
    static_assert(sizeof(InitGroup) % sizeof(uint32_t) == 0, "copied word by word");
    hipLaunchKernelGGL(init_store_group_kernel, dim3(1), dim3(256), 0, s, g, gd);
    LAUNCH_CHECK();
    hipLaunchKernelGGL(init_gram_kernel, dim3(tiles, tiles, n), dim3(256), 0, s, gd);
    LAUNCH_CHECK();
    hipLaunchKernelGGL(init_scale_kernel, dim3(n), dim3(256), 0, s, gd);
    LAUNCH_CHECK();
    // block Jacobi: every instance runs its own sweeps of (blocks) rounds inside the common launches and
    // drops out (its workgroups return at once) after a sweep without a rotation
    const int pairs_max = np_max / kInitPair, rounds_per_sweep = 2 * pairs_max;   // inside round + round-robin
    for (int r = 0; r < kInitMaxSweeps * rounds_per_sweep; ++r) {
      hipLaunchKernelGGL(init_block_solve_kernel, dim3(pairs_max, n), dim3(1024), kInitSolveLds, s, gd, r);
      hipLaunchKernelGGL(init_block_apply_kernel, dim3(2 * pairs_max, pairs_max, n), dim3(256), 0, s, gd, r, pairs_max);
    }
    LAUNCH_CHECK();
    hipLaunchKernelGGL(init_select_kernel, dim3(n), dim3(1024), 0, s, gd);
    LAUNCH_CHECK();
    hipLaunchKernelGGL(init_rows_kernel, dim3((ldw_max + 63) / 64, r_max, n), dim3(256), 0, s, gd);
    LAUNCH_CHECK();
    hipLaunchKernelGGL(init_complete_kernel, dim3(n), dim3(1024), 0, s, gd);
    LAUNCH_CHECK();
    done += n;
  }
  return NGSGD_OK;
}

// Makes stream s wait for a factor update still running on the side stream.  Any stream may ask (an inspection
// call, an averaging call); the update only stops being pending once the stream that steps the network has
// waited for it, because that is the stream the next step's readers of the new factor are ordered on.
int join_side(SideSync* sync, hipStream_t s) {
  if (sync != nullptr && sync->pending) {
    HIP_TRY(hipStreamWaitEvent(s, sync->done, 0));
    if (s == sync->owner) sync->pending = false;
  }
  return NGSGD_OK;
}

// Split-K factor of the H = X W^T product of an N x D input (bounded by the room for its sum-of-squares partials).
// `group` is the number of instances that share the launch: the split only has to fill the chip once for all of
// them, and a split shorter than kMinSplitSteps K-blocks would spend its time in the atomic epilogue.
constexpr int kMinSplitSteps = 6;
int h_splits(int N, int D, int group) {
  const int tiles_m = (N + 63) / 64, ksteps = (D + HBK - 1) / HBK;
  int splits = choose_splits(tiles_m * (group > 0 ? group : 1), ksteps);
  splits = std::min(splits, std::max(1, ksteps / kMinSplitSteps));
  while (splits > 1 && splits * tiles_m > kSumsqMax) --splits;
  return splits;
}

// The online natural-gradient call (App. B.5) for a list of independent instances, in two phases.
//
// precond_apply: everything that touches the N x D matrices (initialisation on the first call, H, J when the
// factor is going to be updated, Xhat, gamma).  With scale_output the matrices are left as gamma * Xhat; without
// it they are left as Xhat and gamma stays in the instance's state for the caller to fold into a later product.
// The instances whose factor is due for an update are appended to `to_update`.
//
// factor_begin / factor_finish: the R x R work and the new factor for those instances (App. B.3); they read only
// what the first phase left in the instances' buffers, so a network runs them on side streams (ngsgd_step).
int precond_validate(const std::vector<PrecondCall>& calls) {
  for (auto& c : calls) {
    const ngsgd_precond& p = *c.p;
    if (c.N < 1 || c.N > p.max_batch || c.ld < p.dim || (c.ld & 3) || !aligned16(c.M)) return NGSGD_EINVAL;
    if (p.rank > 0 && p.t == 0 && c.N <= p.rank) return NGSGD_EINVAL;
  }
  return NGSGD_OK;
}

inline bool factor_due(const ngsgd_precond& p) { return p.t < p.always_update_first || p.t % p.update_period == 0; }

// Clears the accumulation buffers of the listed instances (H always; K, L when the factor is updated).  With
// `keep_clean` (the fused apply path, whose finishing kernel clears what it used) an instance whose counters and
// H rows are still clear is skipped, and no kernel is launched when that holds for all of them.
int clear_accumulators(const std::vector<PrecondCall>& list, hipStream_t s, bool keep_clean = false) {
  for (size_t done = 0; done < list.size();) {
    FillGroup fg;
    const int n = (int)std::min<size_t>(kMaxInstances, list.size() - done);
    fg.count = n;
    size_t n_max = 0;
    for (int i = 0; i < n; ++i) {
      const PrecondCall& c = list[done + i];
      ngsgd_precond& p = *c.p;
      fg.ptr[i] = reinterpret_cast<uint32_t*>(p.zero_region);
      fg.n[i] = factor_due(p) ? p.zero_floats_all : p.arrive_slots + (size_t)c.N * p.ldh;
      if (keep_clean && p.clean_rows >= c.N) fg.n[i] = 0;
      if (!keep_clean) p.clean_rows = 0;   // the caller is about to accumulate into H and leaves it that way
      n_max = std::max(n_max, fg.n[i]);
    }
    done += n;
    if (n_max == 0) continue;
    ProfScope prof(NGSGD_PROF_PRECOND_MISC, s);
    const unsigned blocks = (unsigned)std::min<size_t>((n_max + 2047) / 2048, 64);
    hipLaunchKernelGGL(fill_zero_group_kernel, dim3(blocks > 0 ? blocks : 1, n), dim3(256), 0, s, fg);
    LAUNCH_CHECK();
  }
  return NGSGD_OK;
}

// H = X W^T   (eq. ht) and the partial sums of tr(X X^T) for the listed instances in one launch: the tile is as
// wide as the widest rank class present (a narrower instance wastes matrix-unit work that is small next to the
// cost of a launch of its own).
int launch_h_products(std::vector<PrecondCall>& list, hipStream_t s) {
  if (list.empty()) return NGSGD_OK;
  int rc = 0;
  int class_count[3] = {0, 0, 0};   // the split of an instance is chosen for the instances of its own rank class:
  for (auto& c : list) {            // they carry comparable work, the narrower classes add little to the launch
    rc = std::max(rc, c.p->ldh);
    class_count[c.p->ldh == 32 ? 0 : (c.p->ldh == 80 ? 1 : 2)] += 1;
  }
  std::vector<GemmDesc> d;
  for (auto& c : list) {
    ngsgd_precond& p = *c.p;
    GemmDesc g;
    g.A = c.M; g.lda = c.ld;
    g.B = p.W; g.ldb = p.ldw;
    g.C = p.H; g.ldc = p.ldh;
    g.M = c.N; g.N = p.rank; g.K = p.dim;
    g.sumsq = p.sumsq_part;
    g.splits = h_splits(c.N, p.dim, class_count[p.ldh == 32 ? 0 : (p.ldh == 80 ? 1 : 2)]);
    p.last_N = c.N;
    {
      GemmDesc hd = g;
      p.n_sumsq = planned_sumsq_partials<64, 32, HBK>(hd);   // independent of the tile width
    }
    d.push_back(g);
  }
  ProfScope prof(NGSGD_PROF_PRECOND_H, s);
  HIP_TRY(by_rank_class(rc, [&] { return launch_h<32>(d.data(), (int)d.size(), s); },
                        [&] { return launch_h<80>(d.data(), (int)d.size(), s); },
                        [&] { return launch_h<96>(d.data(), (int)d.size(), s); }));
  return NGSGD_OK;
}

// J = H^T X for the listed instances (must read X before it is overwritten by Xhat).
int launch_j_products(std::vector<PrecondCall>& list, hipStream_t s) {
  for (int rc : {32, 80, 96}) {
    std::vector<GemmDesc> d;
    for (auto& c : list) {
      ngsgd_precond& p = *c.p;
      if (p.ldh != rc) continue;
      GemmDesc g;
      g.A = p.H; g.lda = p.ldh;
      g.B = c.M; g.ldb = c.ld;
      g.C = p.J; g.ldc = p.ldw;
      g.M = p.rank; g.N = p.dim; g.K = c.N;
      d.push_back(g);
    }
    if (d.empty()) continue;
    ProfScope prof(NGSGD_PROF_PRECOND_J, s);
    HIP_TRY(by_rank_class(rc, [&] { return launch_j<32>(d.data(), (int)d.size(), s); },
                          [&] { return launch_j<80>(d.data(), (int)d.size(), s); },
                          [&] { return launch_j<96>(d.data(), (int)d.size(), s); }));
  }
  return NGSGD_OK;
}

// How long a workgroup of the fused apply kernel waits for the other column chunks of its row block before it
// forms the H rows itself (microseconds; the kernel's clock runs at 100 MHz).
std::atomic<long long> g_fused_wait_us{2000};

inline int fused_chunks(int D) { return (D + kFusedChunk - 1) / kFusedChunk; }
inline int fused_row_blocks(int N) { return (N + kFusedRows - 1) / kFusedRows; }

// Whether the fused kernel's bookkeeping has room for this call (partial sums of tr(X X^T) per patch).
inline bool fused_fits(const ngsgd_precond& p, int N) {
  return fused_chunks(p.dim) * fused_row_blocks(N) <= kSumsqMax && (size_t)fused_row_blocks(N) < p.arrive_slots;
}

// Xhat = X - (X W^T) W, row-norm partials and the partial sums of tr(X X^T) in one pass over each matrix
// (eq. ht, hatxt:compute:2, pi), for instances whose factor is not updated by this call.
int launch_fused_apply(std::vector<PrecondCall>& list, hipStream_t s) {
  for (size_t done = 0; done < list.size();) {
    FusedGroup g;
    const int n = (int)std::min<size_t>(kMaxInstances, list.size() - done);
    g.count = n;
    g.spin_limit = g_fused_wait_us.load() * 100;
    int units = 0, rc = 0;
    for (int i = 0; i < n; ++i) {
      const PrecondCall& c = list[done + i];
      ngsgd_precond& p = *c.p;
      FusedArgs& a = g.a[i];
      a.X = c.M; a.ldx = c.ld;
      a.Xout = c.M; a.ldo = c.ld;
      a.W = p.W; a.ldw = p.ldw;
      a.H = p.H; a.ldh = p.ldh;
      a.arrive = p.arrive;
      a.deferred_count = p.arrive + (p.arrive_slots - 1);
      a.deferred = p.deferred;
      a.rownorm_part = p.rownorm_part;
      a.sumsq_part = p.sumsq_part;
      a.N = c.N; a.D = p.dim; a.R = p.rank;
      a.n_rb = fused_row_blocks(c.N);
      a.n_chunks = fused_chunks(p.dim);
      a.n_chunks_pad = (a.n_chunks + kXcds - 1) / kXcds * kXcds;
      a.unit_begin = units;
      units += a.n_rb * a.n_chunks_pad;
      p.last_N = c.N;
      p.n_sumsq = a.n_chunks * a.n_rb;
      rc = std::max(rc, p.ldh);
    }
    g.total_units = units;
    ProfScope prof(NGSGD_PROF_PRECOND_FUSED, s);
    if (rc == 32) {
      hipLaunchKernelGGL((fused_apply_kernel<32, kFusedChunk>), dim3(units), dim3(kFusedThreads), 0, s, g);
    } else if (rc == 80) {
      hipLaunchKernelGGL((fused_apply_kernel<80, kFusedChunk>), dim3(units), dim3(kFusedThreads), 0, s, g);
    } else {
      hipLaunchKernelGGL((fused_apply_kernel<96, kFusedChunk>), dim3(units), dim3(kFusedThreads), 0, s, g);
    }
    LAUNCH_CHECK();
    done += n;
  }
  return NGSGD_OK;
}

// With hj_ready the caller has already produced H and J of every instance (all due for an update, none at t = 0)
// and ordered s behind them; only Xhat and gamma remain.
// do_products / do_finish select the two halves of the work on the matrices (the products; the reduction of the
// partial sums to gamma and the row norms), so that a caller can issue the products of different instances at
// different times and reduce once.
int precond_apply(std::vector<PrecondCall>& calls, bool scale_output, hipStream_t s,
                  std::vector<PrecondCall>& to_update_out, bool hj_ready = false, bool do_products = true,
                  bool do_finish = true) {
  std::vector<PrecondCall> full, to_init, to_update;
  for (auto& c : calls) {
    ngsgd_precond& p = *c.p;
    if (p.rank == 0) {
      hipLaunchKernelGGL(rownorm_kernel, dim3((c.N + 3) / 4), dim3(256), 0, s, c.M, c.ld, c.N, p.dim, p.prow,
                         c.rownorm2_out);
      LAUNCH_CHECK();
      if (c.gamma_out != nullptr) {
        const uint32_t one_bits = 0x3f800000u;
        hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(c.gamma_out),
                           (size_t)1, one_bits);
        LAUNCH_CHECK();
      }
      continue;
    }
    full.push_back(c);
    if (p.t == 0) to_init.push_back(c);
    if (factor_due(p)) to_update.push_back(c);
  }
  // No factor is updated by this call: one fused pass per matrix instead of the H and Xhat products.
  bool fused = !hj_ready && to_update.empty() && !full.empty();
  for (auto& c : full) fused = fused && fused_fits(*c.p, c.N);
  if (!do_products) {
    // the caller has issued the products already
  } else if (fused) {
    NG_TRY(clear_accumulators(full, s, true));
    for (auto& c : full) c.p->clean_rows = 0;   // until the finishing kernel below has been enqueued
    NG_TRY(launch_fused_apply(full, s));
  } else if (!hj_ready) {
    if (!to_init.empty()) NG_TRY(run_init(to_init, s));
    NG_TRY(clear_accumulators(full, s));
    NG_TRY(launch_h_products(full, s));
    NG_TRY(launch_j_products(to_update, s));
  }
  // Xhat = X - H W   (eq. hatxt:compute:2), row-norm partials (eq. pi)
  if (!fused && do_products && !full.empty()) {
    std::vector<GemmDesc> d;
    for (auto& c : full) {
      ngsgd_precond& p = *c.p;
      GemmDesc g;
      g.A = p.H; g.lda = p.ldh;
      g.B = p.W; g.ldb = p.ldw;
      g.C = c.M; g.ldc = c.ld;
      g.M = c.N; g.N = p.dim; g.K = p.rank;
      g.aux = p.rownorm_part;
      d.push_back(g);
    }
    ProfScope prof(NGSGD_PROF_PRECOND_XHAT, s);
    HIP_TRY((launch_gemm_group<64, 64, BK, 2, 2, true, false, EPI_SUB_ROWNORM, false>(d.data(), (int)d.size(), s)));
  }
  // gamma_t, tr(X X^T), tr(Xhat Xhat^T)
  for (size_t done = 0; do_finish && done < full.size();) {
    ProfScope prof(NGSGD_PROF_PRECOND_MISC, s);
    FinishGroup g;
    const int n = (int)std::min<size_t>(kMaxInstances, full.size() - done);
    g.count = n;
    for (int i = 0; i < n; ++i) {
      const PrecondCall& c = full[done + i];
      ngsgd_precond& p = *c.p;
      FinishArgs& a = g.a[i];
      a.st = p.st;
      a.sumsq_part = p.sumsq_part;
      a.n_sumsq = p.n_sumsq;
      a.rownorm_part = p.rownorm_part;
      a.n_col_tiles = fused ? fused_chunks(p.dim) : (p.dim + 63) / 64;
      a.N = c.N;
      a.prow = p.prow;
      a.gamma_out = c.gamma_out;
      a.rownorm2_out = c.rownorm2_out;
      a.deferred_count = fused ? p.arrive + (p.arrive_slots - 1) : nullptr;
      a.deferred = p.deferred;
      a.X = c.M; a.ldx = c.ld;
      a.W = p.W; a.ldw = p.ldw;
      a.H = p.H; a.ldh = p.ldh;
      a.D = p.dim; a.R = p.rank;
      a.chunk_cols = kFusedChunk;
      a.clear_ptr = fused ? p.zero_region : nullptr;
      a.clear_floats = p.arrive_slots + c.N * p.ldh;
    }
    hipLaunchKernelGGL(finish_apply_kernel, dim3(n), dim3(1024), 0, s, g);
    LAUNCH_CHECK();
    if (fused)
      for (int i = 0; i < n; ++i) full[done + i].p->clean_rows = full[done + i].N;
    done += n;
  }
  if (scale_output && do_finish) {
    ProfScope prof(NGSGD_PROF_PRECOND_MISC, s);
    for (auto& c : full) {
      ngsgd_precond& p = *c.p;
      hipLaunchKernelGGL(scale_rows_kernel, dim3((p.dim + 1023) / 1024, c.N), dim3(256), 0, s, c.M, c.ld, c.N, p.dim,
                         &p.st->gamma);
      LAUNCH_CHECK();
    }
  }
  if (do_products) to_update_out.insert(to_update_out.end(), to_update.begin(), to_update.end());
  return NGSGD_OK;
}

// Instances of one small-kernel launch share alpha / epsilon / S (instances of one net do): length of the run
// of compatible instances that starts at `done`.
int small_chunk(const std::vector<PrecondCall>& list, size_t done) {
  const ngsgd_precond& p0 = *list[done].p;
  int n = 0;
  while (n < kMaxInstances && done + n < list.size()) {
    const ngsgd_precond& p = *list[done + n].p;
    if (p.alpha != p0.alpha || p.epsilon != p0.epsilon || p.num_samples_history != p0.num_samples_history) break;
    ++n;
  }
  return n;
}

// First half of the factor update (App. B.3): K, L, B_t, then Z_t, its eigen-decomposition, rho_{t+1}, D_{t+1}
// and A_t.  Reads H, J and the partial sums of tr(X X^T); leaves W_t alone.
int factor_begin(std::vector<PrecondCall>& to_update, hipStream_t s) {
  if (to_update.empty()) return NGSGD_OK;
  {
    // K = J J^T, L = H^T H, fp64 accumulation across the splits
    std::vector<GemmDesc> dk, dl;
    int rc = 0;
    for (auto& c : to_update) rc = std::max(rc, c.p->ldh);
    for (auto& c : to_update) {
      ngsgd_precond& p = *c.p;
      GemmDesc g;
      g.A = p.J; g.lda = p.ldw;
      g.B = p.J; g.ldb = p.ldw;
      g.C = p.K; g.ldc = p.rank;
      g.M = p.rank; g.N = p.rank; g.K = p.dim;
      g.splits = gram_splits(rc, p.rank, (int)to_update.size(), p.dim);
      dk.push_back(g);
      GemmDesc h;
      h.A = p.H; h.lda = p.ldh;
      h.B = p.H; h.ldb = p.ldh;
      h.C = p.L; h.ldc = p.rank;
      h.M = p.rank; h.N = p.rank; h.K = p.last_N;
      h.splits = gram_splits(rc, p.rank, (int)to_update.size(), p.last_N);
      dl.push_back(h);
    }
    ProfScope prof(NGSGD_PROF_PRECOND_KL, s);
    HIP_TRY(launch_small_gram<true>(rc, dk.data(), (int)dk.size(), s));
    HIP_TRY(launch_small_gram<false>(rc, dl.data(), (int)dl.size(), s));
  }
  // B_t over J (needs D_t, rho_t: before the R x R update)
  for (size_t done = 0; done < to_update.size();) {
    ProfScope prof(NGSGD_PROF_PRECOND_MISC, s);
    BtGroup bg;
    bg.num_samples_history = to_update[done].p->num_samples_history;
    int n = 0, r_max = 0, d_max = 0;
    while (n < kMaxInstances && done + n < to_update.size()) {
      const PrecondCall& c = to_update[done + n];
      ngsgd_precond& p = *c.p;
      if (p.num_samples_history != bg.num_samples_history) break;
      bg.a[n] = BtArgs{p.J, p.W, p.st, p.ldw, p.dim, p.rank, p.last_N};
      r_max = std::max(r_max, p.rank);
      d_max = std::max(d_max, p.dim);
      ++n;
    }
    bg.count = n;
    hipLaunchKernelGGL(make_bt_kernel, dim3((d_max + 1023) / 1024, r_max, n), dim3(256), 0, s, bg);
    LAUNCH_CHECK();
    done += n;
  }
  // Z_t, eigen-decomposition, rho_{t+1}, D_{t+1}, A_t
  for (size_t done = 0; done < to_update.size();) {
    SmallGroup g;
    const ngsgd_precond& p0 = *to_update[done].p;
    g.alpha = p0.alpha;
    g.epsilon = p0.epsilon;
    g.num_samples_history = p0.num_samples_history;
    const int n = small_chunk(to_update, done);
    int r_max = 0;
    for (int i = 0; i < n; ++i) {
      const ngsgd_precond& p = *to_update[done + i].p;
      SmallArgs& a = g.a[i];
      a.st = p.st; a.K = p.K; a.L = p.L; a.At = p.At; a.ldat = p.ldh;
      a.R = p.rank; a.D = p.dim; a.N = p.last_N;
      a.rotlog = p.rotlog; a.work = p.eigwork;
      a.sumsq_part = p.sumsq_part;
      a.n_sumsq = p.n_sumsq;
      r_max = std::max(r_max, p.rank);
    }
    g.count = n;
    ProfScope prof(NGSGD_PROF_PRECOND_SMALL, s);
    {
      const int m_max = (r_max + 1) & ~1;
      const int n_blocks = (m_max / 2) * (m_max / 2 + 1) / 2;   // 2x2 blocks of the upper triangle
      size_t eig_dyn = (size_t)2 * 4 * n_blocks * sizeof(double);   // two copies of four planes
      // A large eigen-problem is a long sequential chain bound by LDS latency, on which the next step waits: it asks for
      // most of the compute unit's LDS, so that no workgroup of the layer products (which live on LDS bandwidth) is
      // placed next to it.  That costs the products one compute unit in 256 per instance.
      if (m_max >= kEigReserveFromRank) eig_dyn = std::max<size_t>(eig_dyn, kEigLdsReserve);
      const int n_off = (m_max / 2) * (m_max / 2 - 1) / 2;   // off-diagonal blocks, owned by the waves after the first
      const int items = std::max(1, (n_off + (kEigThreads - 64) - 1) / (kEigThreads - 64));
      if (items <= 1) {
        hipLaunchKernelGGL((eig_update_kernel<1, kEigThreads>), dim3(n), dim3(kEigThreads), eig_dyn, s, g);
      } else if (items == 2) {
        hipLaunchKernelGGL((eig_update_kernel<2, kEigThreads>), dim3(n), dim3(kEigThreads), eig_dyn, s, g);
      } else {
        hipLaunchKernelGGL((eig_update_kernel<kEigMaxItems, kEigThreads>), dim3(n), dim3(kEigThreads), eig_dyn, s, g);
      }
      LAUNCH_CHECK();
    }
    const int rows_per_block = kEigvecThreads / 64;
    hipLaunchKernelGGL(eigvec_kernel, dim3(n, (r_max + rows_per_block - 1) / rows_per_block), dim3(kEigvecThreads),
                       r_max >= kEigReserveFromRank ? kEigvecLdsReserve : 0, s, g);
    LAUNCH_CHECK();
    done += n;
  }
  return NGSGD_OK;
}

// Second half: W_{t+1} = A_t B_t (eq. wt1) and the orthogonality check of App. B.3.1.  Overwrites W_t, so the
// caller orders it behind the last reader of W_t.
int factor_finish(std::vector<PrecondCall>& to_update, hipStream_t s) {
  for (size_t done = 0; done < to_update.size();) {
    OrthGroup og;
    const int n = small_chunk(to_update, done);
    int r_max = 0;
    for (int i = 0; i < n; ++i) {
      const ngsgd_precond& p = *to_update[done + i].p;
      OrthArgs& o = og.a[i];
      o.st = p.st; o.G = p.K; o.At = p.At; o.ldat = p.ldh; o.R = p.rank;
      r_max = std::max(r_max, p.rank);
    }
    og.count = n;
    auto launch_new_factor = [&](const bool only_if_reorthogonalised) -> int {
      for (int rc : {32, 80, 96}) {
        std::vector<GemmDesc> d;
        for (int i = 0; i < n; ++i) {
          ngsgd_precond& p = *to_update[done + i].p;
          if (p.ldh != rc) continue;
          GemmDesc w;
          w.A = p.At; w.lda = p.ldh;
          w.B = p.J; w.ldb = p.ldw;
          w.C = p.W; w.ldc = p.ldw;
          w.M = p.rank; w.N = p.dim; w.K = p.rank;
          if (only_if_reorthogonalised) {
            w.gate = &p.st->flags;
            w.gate_mask = kFlagReorth;
          }
          d.push_back(w);
        }
        if (d.empty()) continue;
        ProfScope prof(only_if_reorthogonalised ? NGSGD_PROF_PRECOND_MISC : NGSGD_PROF_PRECOND_WNEW, s);
        HIP_TRY(by_rank_class(rc, [&] { return launch_wnew<32>(d.data(), (int)d.size(), s); },
                              [&] { return launch_wnew<80>(d.data(), (int)d.size(), s); },
                              [&] { return launch_wnew<96>(d.data(), (int)d.size(), s); }));
      }
      return NGSGD_OK;
    };
    NG_TRY(launch_new_factor(false));
    {
      // App. B.3.1: W W^T of the new factor, accumulated into K (cleared by the R x R kernel) only for the
      // instances whose update asked for the check, then the check itself and, if needed, the Cholesky fix
      ProfScope prof(NGSGD_PROF_PRECOND_MISC, s);
      std::vector<GemmDesc> dg;
      for (int i = 0; i < n; ++i) {
        ngsgd_precond& p = *to_update[done + i].p;
        GemmDesc w;
        w.A = p.W; w.lda = p.ldw;
        w.B = p.W; w.ldb = p.ldw;
        w.C = p.K; w.ldc = p.rank;
        w.M = p.rank; w.N = p.rank; w.K = p.dim;
        w.splits = gram_splits(rank_class(r_max), p.rank, n, p.dim);
        w.gate = &p.st->flags;
        w.gate_mask = kFlagOrthCheck;
        dg.push_back(w);
      }
      HIP_TRY(launch_small_gram<true>(rank_class(r_max), dg.data(), (int)dg.size(), s));
      const size_t dyn = (size_t)r_max * (r_max + 1) * sizeof(double);   // W W^T of an instance
      const int ct = orth_columns_per_thread(r_max);   // 2 R / 32 rounded up: 1 .. 6
      if (ct <= 2) {
        hipLaunchKernelGGL(orth_fix_kernel<2>, dim3(n), dim3(kSmallThreads), dyn, s, og);
      } else if (ct <= 3) {
        hipLaunchKernelGGL(orth_fix_kernel<3>, dim3(n), dim3(kSmallThreads), dyn, s, og);
      } else if (ct <= 5) {
        hipLaunchKernelGGL(orth_fix_kernel<5>, dim3(n), dim3(kSmallThreads), dyn, s, og);
      } else {
        hipLaunchKernelGGL(orth_fix_kernel<6>, dim3(n), dim3(kSmallThreads), dyn, s, og);
      }
      LAUNCH_CHECK();
    }
    // where the check failed the kernel has folded the fix into A_t: W_{t+1} = A_t B_t once more for those
    NG_TRY(launch_new_factor(true));
    done += n;
  }
  return NGSGD_OK;
}

// Both phases for one list of instances on one stream.
int precondition_many(std::vector<PrecondCall>& calls, bool scale_output, hipStream_t s) {
  NG_TRY(ensure_kernel_attributes());
  NG_TRY(precond_validate(calls));
  std::vector<PrecondCall> to_update;
  NG_TRY(precond_apply(calls, scale_output, s, to_update));
  NG_TRY(factor_begin(to_update, s));
  NG_TRY(factor_finish(to_update, s));
  for (auto& c : calls) c.p->t += 1;
  return NGSGD_OK;
}

}  // namespace

// ---------------------------------------------------------------------------------------------------
// preconditioner C ABI
// ---- simple method (App. A) --------------------------------------------------------------------------
namespace {

struct SimpleWork {   // device scratch of one matrix, carved for up to max_rows x dim
  double* scal = nullptr;
  double* prow = nullptr;
  double* buf[2] = {nullptr, nullptr};
  double* pinv[2] = {nullptr, nullptr};
  float* ginv = nullptr;
  float* Q = nullptr;
  int ldq = 0;
};

void simple_layout(SimpleWork& w, int max_rows, int dim, bool own_prow, Carver& c) {
  const size_t np = (size_t)pad32(std::min(max_rows, dim));
  w.scal = c.take<double>(4);
  w.prow = own_prow ? c.take<double>(max_rows) : nullptr;
  w.buf[0] = c.take<double>(np * np);
  w.buf[1] = c.take<double>(np * np);
  w.pinv[0] = c.take<double>(kSimpleBlock * kSimpleBlock);
  w.pinv[1] = c.take<double>(kSimpleBlock * kSimpleBlock);
  w.ginv = c.take<float>(np * np);
  w.ldq = pad32(dim);
  w.Q = c.take<float>((size_t)max_rows * w.ldq);
}

struct SimpleCall {
  float* M;
  int ld, N, D;
  double alpha, epsilon;
  SimpleWork w;
  double* prow;          // N doubles: ||xhat_i||^2
  double* gamma;         // 1 double
  float* gamma_out;      // optional
  float* rownorm2_out;   // optional
};

// Enqueues the simple method for a list of independent matrices; every stage is one grouped launch.  With
// scale_output the matrices are left as gamma * Xhat, without it as Xhat with gamma in *gamma.
int simple_many(const std::vector<SimpleCall>& calls, bool scale_output, hipStream_t s) {
  for (auto& c : calls)
    if (c.M == nullptr || c.N < 2 || c.D < 1 || c.ld < c.D || (c.ld & 3) || !aligned16(c.M) || !(c.alpha > 0.0) ||
        !(c.epsilon > 0.0))
      return NGSGD_EINVAL;
  for (size_t done = 0; done < calls.size();) {
    const int cnt = (int)std::min<size_t>(kSimpleMaxGroup, calls.size() - done);
    SimpleGroup g;
    g.count = cnt;
    int nblk_max = 0, n_max = 0;
    for (int i = 0; i < cnt; ++i) {
      const SimpleCall& c = calls[done + i];
      SimpleArgs& a = g.a[i];
      a.M = c.M; a.ld = c.ld; a.Q = c.w.Q; a.ldq = c.w.ldq;
      a.N = c.N; a.D = c.D;
      a.n = c.N > c.D ? c.D : c.N;     // column space if N > D, row space otherwise (App. A.3)
      a.np = pad32(a.n);
      a.nblk = a.np / kSimpleBlock;
      a.alpha = c.alpha; a.epsilon = c.epsilon;
      a.buf[0] = c.w.buf[0]; a.buf[1] = c.w.buf[1];
      a.pinv[0] = c.w.pinv[0]; a.pinv[1] = c.w.pinv[1];
      a.ginv = c.w.ginv;
      a.prow = c.prow; a.scal = c.w.scal; a.gamma = c.gamma;
      a.gamma_out = c.gamma_out; a.rownorm2_out = c.rownorm2_out;
      nblk_max = std::max(nblk_max, a.nblk);
      n_max = std::max(n_max, a.N);
    }
    {
      // Gram matrix in fp64 (split over the long dimension, double atomics)
      ProfScope prof(NGSGD_PROF_SIMPLE_GRAM, s);
      FillGroup fg;
      fg.count = cnt;
      size_t fill_max = 0;
      for (int i = 0; i < cnt; ++i) {
        fg.ptr[i] = reinterpret_cast<uint32_t*>(g.a[i].buf[1]);
        fg.n[i] = (size_t)g.a[i].np * g.a[i].np * 2;
        fill_max = std::max(fill_max, fg.n[i]);
      }
      const unsigned blocks = (unsigned)std::min<size_t>((fill_max + 2047) / 2048, 256);
      hipLaunchKernelGGL(fill_zero_group_kernel, dim3(blocks > 0 ? blocks : 1, cnt), dim3(256), 0, s, fg);
      LAUNCH_CHECK();
      // the Gram matrix is symmetric: only the 128 x 128 tiles on and above the diagonal are computed, one
      // problem per tile row; the kernel that forms G mirrors them
      std::vector<GemmDesc> rows, cols;
      int tiles_rows = 0, tiles_cols = 0;
      constexpr int T = kSimpleGramTile;
      for (int i = 0; i < cnt; ++i) {
        const SimpleArgs& a = g.a[i];
        const int tr = (a.n + T - 1) / T;
        (a.N > a.D ? tiles_cols : tiles_rows) += tr * (tr + 1) / 2;
      }
      auto splits_for = [](int tiles, int k) {
        const int ksteps = (k + BK - 1) / BK;
        return std::max(1, std::min(768 / std::max(1, tiles), ksteps / 4));
      };
      for (int i = 0; i < cnt; ++i) {
        const SimpleArgs& a = g.a[i];
        for (int r0 = 0; r0 < a.n; r0 += T) {
          GemmDesc d;
          d.lda = d.ldb = a.ld;
          d.C = a.buf[1] + (size_t)r0 * a.np + r0; d.ldc = a.np;
          d.M = std::min(T, a.n - r0);
          d.N = a.n - r0;
          if (a.N > a.D) {   // X^T X: the sum runs over the rows; operands start at column r0
            d.A = d.B = a.M + r0;
            d.K = a.N;
            d.splits = splits_for(tiles_cols, d.K);
            cols.push_back(d);
          } else {           // X X^T: the sum runs over the columns; operands start at row r0
            d.A = d.B = a.M + (size_t)r0 * a.ld;
            d.K = a.D;
            d.splits = splits_for(tiles_rows, d.K);
            rows.push_back(d);
          }
        }
      }
      if (!rows.empty())
        HIP_TRY((launch_gemm_group<T, T, BK, 2, 2, true, true, EPI_ATOMIC_F64, false, 0, true>(rows.data(),
                                                                                             (int)rows.size(), s)));
      if (!cols.empty())
        HIP_TRY((launch_gemm_group<T, T, BK, 2, 2, false, false, EPI_ATOMIC_F64, false, 0, true>(cols.data(),
                                                                                               (int)cols.size(), s)));
    }
    {
      // G = beta I + Gram / (N-1), then its inverse, one launch per pivot block
      ProfScope prof(NGSGD_PROF_SIMPLE_INVERSE, s);
      hipLaunchKernelGGL(simple_prepare_kernel, dim3(nblk_max, nblk_max, cnt), dim3(256), 0, s, g);
      LAUNCH_CHECK();
      const int wg = (nblk_max + 1) / 2;
      for (int k = 0; k < nblk_max; ++k) {
        hipLaunchKernelGGL(simple_sweep_kernel, dim3(wg + 1, wg, cnt), dim3(256), 0, s, g, k);   // + look-ahead column
        LAUNCH_CHECK();
      }
    }
    {
      // Q = G^{-1} X (row space) or X G^{-1} (column space), per-row factors, gamma
      ProfScope prof(NGSGD_PROF_SIMPLE_APPLY, s);
      std::vector<GemmDesc> rows, cols;
      for (int i = 0; i < cnt; ++i) {
        const SimpleArgs& a = g.a[i];
        GemmDesc d;
        d.C = a.Q; d.ldc = a.ldq;
        d.M = a.N; d.N = a.D; d.K = a.n;
        if (a.N > a.D) {
          d.A = a.M; d.lda = a.ld;         // X, N x D
          d.B = a.ginv; d.ldb = a.np;      // G^{-1} is symmetric: row d of it is column d
          cols.push_back(d);
        } else {
          d.A = a.ginv; d.lda = a.np;      // G^{-1}, N x N
          d.B = a.M; d.ldb = a.ld;         // X stored K x N
          rows.push_back(d);
        }
      }
      if (!rows.empty())
        HIP_TRY((launch_layer_tile<true, false, kBwdAccChunk>(pick_layer_tile(rows.data(), (int)rows.size()),
                                                             rows.data(), (int)rows.size(), s)));
      if (!cols.empty())
        HIP_TRY((launch_layer_tile<true, true, 0>(pick_layer_tile(cols.data(), (int)cols.size()), cols.data(),
                                                  (int)cols.size(), s)));
      hipLaunchKernelGGL(simple_rows_kernel, dim3(n_max, cnt), dim3(256), 0, s, g);
      LAUNCH_CHECK();
      hipLaunchKernelGGL(simple_gamma_kernel, dim3(cnt), dim3(256), 0, s, g);
      LAUNCH_CHECK();
      if (scale_output)
        for (int i = 0; i < cnt; ++i) {
          const SimpleArgs& a = g.a[i];
          hipLaunchKernelGGL(scale_rows_kernel, dim3((a.D + 1023) / 1024, a.N), dim3(256), 0, s, a.M, a.ld, a.N, a.D,
                             a.gamma);
          LAUNCH_CHECK();
        }
    }
    done += cnt;
  }
  return NGSGD_OK;
}

}  // namespace

extern "C" int ngsgd_simple_workspace_bytes(int32_t max_rows, int32_t dim, size_t* out_bytes) {
  if (out_bytes == nullptr || max_rows < 2 || dim < 1) return NGSGD_EINVAL;
  SimpleWork w;
  Carver c(nullptr);
  simple_layout(w, max_rows, dim, true, c);
  (void)c.take<double>(1);   // gamma
  *out_bytes = align_up(c.off, 256);
  return NGSGD_OK;
}

extern "C" int ngsgd_precondition_simple(float* dev_M, int32_t N, int32_t D, int32_t ld, float alpha, float epsilon,
                                         void* dev_workspace, size_t workspace_bytes, float* dev_gamma,
                                         float* dev_rownorm2, void* hip_stream) {
  if (dev_M == nullptr || dev_workspace == nullptr || (reinterpret_cast<uintptr_t>(dev_workspace) & 255u))
    return NGSGD_EINVAL;
  size_t need = 0;
  NG_TRY(ngsgd_simple_workspace_bytes(N, D, &need));
  if (workspace_bytes < need) return NGSGD_ENOMEM;
  SimpleCall c;
  Carver carve(dev_workspace);
  simple_layout(c.w, N, D, true, carve);
  c.gamma = carve.take<double>(1);
  c.M = dev_M; c.ld = ld; c.N = N; c.D = D;
  c.alpha = alpha; c.epsilon = epsilon;
  c.prow = c.w.prow;
  c.gamma_out = dev_gamma;
  c.rownorm2_out = dev_rownorm2;
  std::vector<SimpleCall> calls(1, c);
  return simple_many(calls, true, static_cast<hipStream_t>(hip_stream));
}

// ---- the simple method without a workspace argument ------------------------------------------------------
// Scratch of ngsgd_precondition_simple_static: a fixed array in the library's device image instead of memory the
// caller brings, for callers that cannot allocate.  Every GPU holds its own copy at its own address; in host
// code the array's name is only a handle for hipGetSymbolAddress, the address it returns is what kernels get.
static __device__ __align__(256) unsigned char scratch[NGSGD_SIMPLE_STATIC_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, looked up once per device.
int static_scratch(void** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return NGSGD_EUNSUPPORTED;
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (ptr == nullptr || (reinterpret_cast<uintptr_t>(ptr) & 255u)) return NGSGD_EHIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return NGSGD_OK;
}
}  // namespace

extern "C" int ngsgd_precondition_simple_static(float* dev_M, int32_t N, int32_t D, int32_t ld, float alpha,
                                                float epsilon, float* dev_gamma, float* dev_rownorm2,
                                                void* hip_stream) {
  if (dev_M == nullptr) return NGSGD_EINVAL;
  size_t need = 0;
  NG_TRY(ngsgd_simple_workspace_bytes(N, D, &need));
  if (need > (size_t)NGSGD_SIMPLE_STATIC_BYTES) return NGSGD_ENOMEM;   // the matrix is too large for the fixed scratch
  void* ptr = nullptr;
  NG_TRY(static_scratch(&ptr));
  // the scratch keeps the previous call's contents: the kernels clear what they accumulate into (the Gram
  // matrix) and write every other buffer before reading it, exactly as with a caller's reused workspace
  return ngsgd_precondition_simple(dev_M, N, D, ld, alpha, epsilon, ptr, (size_t)NGSGD_SIMPLE_STATIC_BYTES, dev_gamma,
                                   dev_rownorm2, hip_stream);
}

extern "C" int ngsgd_precond_workspace_bytes(int32_t dim, int32_t rank, int32_t max_batch, size_t* out_bytes) {
  if (out_bytes == nullptr) return NGSGD_EINVAL;
  NG_TRY(precond_check_config(dim, rank, max_batch, 4.f, 2000.f, 1e-10f, 4, 10));
  ngsgd_precond p;
  p.dim = dim; p.rank = rank; p.max_batch = max_batch;
  Carver c(nullptr);
  precond_layout(p, c);
  *out_bytes = align_up(c.off, 256);
  return NGSGD_OK;
}

extern "C" int ngsgd_precond_create(int32_t dim, int32_t rank, int32_t max_batch, float alpha,
                                    float num_samples_history, float epsilon, int32_t update_period,
                                    int32_t always_update_first, void* dev_workspace, size_t workspace_bytes,
                                    ngsgd_precond** out) {
  if (out == nullptr || dev_workspace == nullptr) return NGSGD_EINVAL;
  if (reinterpret_cast<uintptr_t>(dev_workspace) & 255u) return NGSGD_EINVAL;
  NG_TRY(precond_check_config(dim, rank, max_batch, alpha, num_samples_history, epsilon, update_period,
                              always_update_first));
  size_t need = 0;
  NG_TRY(ngsgd_precond_workspace_bytes(dim, rank, max_batch, &need));
  if (workspace_bytes < need) return NGSGD_ENOMEM;
  ngsgd_precond* p = new (std::nothrow) ngsgd_precond();
  if (p == nullptr) return NGSGD_ENOMEM;
  precond_configure(*p, dim, rank, max_batch, alpha, num_samples_history, epsilon, update_period,
                    always_update_first);
  Carver c(dev_workspace);
  precond_layout(*p, c);
  hipError_t e = hipMemset(dev_workspace, 0, need);
  if (e == hipSuccess) {
    PrecondScalars init;
    std::memset(&init, 0, sizeof(init));
    init.gamma = 1.0;
    e = hipMemcpy(p->st, &init, sizeof(init), hipMemcpyHostToDevice);
  }
  if (e != hipSuccess) {
    g_last_hip_error = (int)e;
    delete p;
    return NGSGD_EHIP;
  }
  *out = p;
  return NGSGD_OK;
}

extern "C" int ngsgd_precond_destroy(ngsgd_precond* p) {
  if (p == nullptr || p->owned_by_net) return NGSGD_EINVAL;
  delete p;
  return NGSGD_OK;
}

extern "C" int ngsgd_precond_reset(ngsgd_precond* p) {
  if (p == nullptr) return NGSGD_EINVAL;
  p->t = 0;
  return NGSGD_OK;
}

extern "C" int ngsgd_precondition(ngsgd_precond* p, float* dev_M, int32_t N, int32_t ld, float* dev_gamma,
                                  float* dev_rownorm2, void* hip_stream) {
  if (p == nullptr || dev_M == nullptr) return NGSGD_EINVAL;
  std::vector<PrecondCall> calls(1);
  calls[0] = PrecondCall{p, dev_M, ld, N, dev_gamma, dev_rownorm2};
  NG_TRY(join_side(p->sync, static_cast<hipStream_t>(hip_stream)));
  return precondition_many(calls, true, static_cast<hipStream_t>(hip_stream));
}

extern "C" int ngsgd_precond_get_state(const ngsgd_precond* p, float* dev_W, double* dev_d, double* dev_rho,
                                       int64_t* t_host, void* hip_stream) {
  if (p == nullptr) return NGSGD_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  NG_TRY(join_side(p->sync, s));
  if (t_host != nullptr) *t_host = p->t;
  if (p->rank == 0) {
    if (dev_rho != nullptr) HIP_TRY(hipMemsetAsync(dev_rho, 0, sizeof(double), s));
    return NGSGD_OK;
  }
  if (dev_W != nullptr)
    HIP_TRY(hipMemcpy2DAsync(dev_W, (size_t)p->dim * sizeof(float), p->W, (size_t)p->ldw * sizeof(float),
                             (size_t)p->dim * sizeof(float), p->rank, hipMemcpyDeviceToDevice, s));
  if (dev_d != nullptr)
    HIP_TRY(hipMemcpyAsync(dev_d, p->st->d, (size_t)p->rank * sizeof(double), hipMemcpyDeviceToDevice, s));
  if (dev_rho != nullptr)
    HIP_TRY(hipMemcpyAsync(dev_rho, &p->st->rho, sizeof(double), hipMemcpyDeviceToDevice, s));
  return NGSGD_OK;
}

extern "C" int ngsgd_precond_diagnostics(const ngsgd_precond* p, int32_t* flags_host, int32_t* sweeps_host,
                                         void* hip_stream) {
  if (p == nullptr) return NGSGD_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  NG_TRY(join_side(p->sync, s));
  int v[2] = {0, 0};
  if (p->rank > 0) {
    HIP_TRY(hipMemcpyAsync(v, &p->st->flags, sizeof(v), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
  }
  if (flags_host != nullptr) *flags_host = v[0];
  if (sweeps_host != nullptr) *sweeps_host = v[1];
  return NGSGD_OK;
}

extern "C" int ngsgd_precond_set_state(ngsgd_precond* p, const double* dev_R, const double* dev_d, double rho,
                                       int64_t t, void* hip_stream) {
  if (p == nullptr || t < 1 || !(rho > 0.0)) return NGSGD_EINVAL;
  if (p->rank == 0) {
    p->t = t;
    return NGSGD_OK;
  }
  if (dev_R == nullptr || dev_d == nullptr) return NGSGD_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  NG_TRY(join_side(p->sync, s));
  hipLaunchKernelGGL(set_state_kernel, dim3(p->rank), dim3(256), 0, s, dev_R, dev_d, rho, p->alpha, p->rank, p->dim,
                     p->W, p->ldw, p->st);
  LAUNCH_CHECK();
  p->t = t;
  return NGSGD_OK;
}

// ---------------------------------------------------------------------------------------------------
// network
struct ngsgd_layer {
  int din = 0, dout = 0, in1 = 0;   // in1 = din + 1 (bias input)
  int ldw = 0, ldx = 0, lda = 0;
  int nonlin = -1;                  // nonlinearity after this layer, -1 for the last
  int groups = 0;                   // p-norm output dimension
  float* W = nullptr;               // dout x ldw
  float* Xin = nullptr;             // max_batch x ldx, [input, 1]
  float* A = nullptr;               // max_batch x lda, affine output, later O_l
  float* sigma = nullptr;           // max_batch renorm divisors
  double* mc_scale = nullptr;       // max-change scale of the latest step
  ngsgd_precond pin, pout;
  SimpleWork sin, sout;             // scratch of the simple method (only laid out when it is selected)
};

struct ngsgd_net {
  int n_layers = 0;
  int max_batch = 0;
  int pnorm_group = 10;
  int renorm = 0;
  double max_change_per_sample = 0.0;
  int method = NGSGD_METHOD_ONLINE;
  double alpha = 4.0, simple_epsilon = 1e-20;
  std::vector<ngsgd_layer> layers;
  float* params = nullptr;
  size_t n_params_padded = 0;
  float* dX = nullptr;
  int lddx = 0;
  double* rowobj = nullptr;
  double* logprob = nullptr;
  int last_N = 0;
  float last_lr = 0.f;
  SideSync side[kSideStreams];
  int n_side = kSideStreams;   // streams in use
  // ordering between the stream that steps this replica and a stream that averages it with others
  hipEvent_t step_done = nullptr;   // recorded by an averaging call on the stream of the latest step (an event per
                                    // step would cost every step a marker packet on its critical stream)
  hipStream_t step_stream = nullptr;
  bool stepped = false;
  hipEvent_t avg_done = nullptr;    // recorded behind an averaging kernel that rewrote the weights
  bool avg_pending = false;
};

namespace {

// Side stream of the output-side instance of layer l when n_side streams are in use: the last layer's derivatives
// exist after the log-softmax (group 0, with all input sides); the others appear in descending layer order during
// the backward pass, two layers per group, everything below in the last group.  With one stream there is one group.
int output_side_group(int l, int n_layers, int n_side) {
  if (n_side <= 1 || l == n_layers - 1) return 0;
  return std::min(n_side - 1, 1 + (n_layers - 2 - l) / 2);
}

int net_check_config(const ngsgd_config* cfg) {
  if (cfg == nullptr || cfg->dims == nullptr || cfg->n_layers < 1 || cfg->n_layers > NGSGD_MAX_LAYERS)
    return NGSGD_EINVAL;
  if (cfg->n_layers > 1 && cfg->nonlin == nullptr) return NGSGD_EINVAL;
  if (cfg->max_batch < 1 || cfg->pnorm_group < 1) return NGSGD_EINVAL;
  if (cfg->dims[0] < 1 || (cfg->dims[0] & 3)) return NGSGD_EINVAL;
  if (!(cfg->max_change_per_sample >= 0.f)) return NGSGD_EINVAL;
  if (cfg->method != NGSGD_METHOD_ONLINE && cfg->method != NGSGD_METHOD_SIMPLE) return NGSGD_EINVAL;
  const bool simple = cfg->method == NGSGD_METHOD_SIMPLE;
  if (cfg->side_streams < 0 || cfg->side_streams > kSideStreams) return NGSGD_EINVAL;
  if (simple && (cfg->max_batch < 2 || !(cfg->alpha > 0.f) || !(cfg->simple_epsilon > 0.f))) return NGSGD_EINVAL;
  int din = cfg->dims[0];
  for (int l = 0; l < cfg->n_layers; ++l) {
    const int dout = cfg->dims[l + 1];
    if (dout < 1) return NGSGD_EINVAL;
    // the simple method keeps no factors: the ranks are not used
    NG_TRY(precond_check_config(din + 1, simple ? 0 : cfg->rank_in, cfg->max_batch, cfg->alpha,
                                cfg->num_samples_history, cfg->epsilon, cfg->update_period, cfg->always_update_first));
    NG_TRY(precond_check_config(dout, simple ? 0 : cfg->rank_out, cfg->max_batch, cfg->alpha,
                                cfg->num_samples_history, cfg->epsilon, cfg->update_period, cfg->always_update_first));
    if (l < cfg->n_layers - 1) {
      if (cfg->nonlin[l] == NGSGD_PNORM) {
        if (dout % cfg->pnorm_group || dout / cfg->pnorm_group > kPnormMaxGroupsLds) return NGSGD_EINVAL;
        din = dout / cfg->pnorm_group;
      } else if (cfg->nonlin[l] == NGSGD_TANH) {
        din = dout;
      } else {
        return NGSGD_EINVAL;
      }
    }
  }
  return NGSGD_OK;
}

void net_layout(ngsgd_net& net, const ngsgd_config* cfg, Carver& c) {
  net.n_layers = cfg->n_layers;
  net.max_batch = cfg->max_batch;
  net.pnorm_group = cfg->pnorm_group;
  net.renorm = cfg->renorm ? 1 : 0;
  net.max_change_per_sample = cfg->max_change_per_sample;
  net.method = cfg->method;
  net.alpha = cfg->alpha;
  net.simple_epsilon = cfg->simple_epsilon;
  net.n_side = cfg->side_streams > 0 ? cfg->side_streams : kDefaultSideStreams;
  const bool simple = cfg->method == NGSGD_METHOD_SIMPLE;
  net.layers.assign(cfg->n_layers, ngsgd_layer());
  int din = cfg->dims[0];
  size_t n_params = 0;
  int max_ldx = 0;
  for (int l = 0; l < cfg->n_layers; ++l) {
    ngsgd_layer& L = net.layers[l];
    L.din = din;
    L.dout = cfg->dims[l + 1];
    L.in1 = din + 1;
    L.ldw = pad32(L.in1);
    L.ldx = pad32(L.in1);
    L.lda = pad32(L.dout);
    L.nonlin = l < cfg->n_layers - 1 ? cfg->nonlin[l] : -1;
    L.groups = L.nonlin == NGSGD_PNORM ? L.dout / cfg->pnorm_group : L.dout;
    n_params += (size_t)L.dout * L.ldw;
    max_ldx = std::max(max_ldx, L.ldx);
    din = L.groups;
  }
  net.n_params_padded = n_params;
  net.params = c.take<float>(n_params);
  size_t off = 0;
  for (auto& L : net.layers) {
    L.W = net.params ? net.params + off : nullptr;
    off += (size_t)L.dout * L.ldw;
  }
  net.lddx = max_ldx;
  net.dX = c.take<float>((size_t)kMaxBwdSplits * net.max_batch * net.lddx);
  net.rowobj = c.take<double>(net.max_batch);
  net.logprob = c.take<double>(1);
  for (auto& L : net.layers) {
    L.Xin = c.take<float>((size_t)net.max_batch * L.ldx);
    L.A = c.take<float>((size_t)net.max_batch * L.lda);
    L.sigma = c.take<float>(net.max_batch);
    L.mc_scale = c.take<double>(1);
    precond_configure(L.pin, L.in1, simple ? 0 : cfg->rank_in, cfg->max_batch, cfg->alpha, cfg->num_samples_history,
                      cfg->epsilon, cfg->update_period, cfg->always_update_first);
    precond_configure(L.pout, L.dout, simple ? 0 : cfg->rank_out, cfg->max_batch, cfg->alpha,
                      cfg->num_samples_history, cfg->epsilon, cfg->update_period, cfg->always_update_first);
    L.pin.owned_by_net = L.pout.owned_by_net = true;
    L.pin.sync = &net.side[0];
    L.pout.sync = &net.side[output_side_group((int)(&L - net.layers.data()), cfg->n_layers, net.n_side)];
    precond_layout(L.pin, c);
    precond_layout(L.pout, c);
    if (simple) {   // gamma and the row norms go where the online method leaves them (st->gamma, prow)
      simple_layout(L.sin, cfg->max_batch, L.in1, false, c);
      simple_layout(L.sout, cfg->max_batch, L.dout, false, c);
    }
  }
}

int copy2d(const float* src, int lds_, float* dst, int ldd, int rows, int cols, float scale, const double* scale_dev,
           hipStream_t s) {
  hipLaunchKernelGGL(copy2d_kernel, dim3((cols + 1023) / 1024, rows), dim3(256), 0, s, src, lds_, dst, ldd, rows, cols,
                     scale, scale_dev);
  LAUNCH_CHECK();
  return NGSGD_OK;
}

// Orders stream s behind an averaging kernel that rewrote this replica's weights on another stream.  The wait is
// dropped once the replica's own stepping stream has taken it.
int order_after_average(ngsgd_net* net, hipStream_t s, bool stepping_stream) {
  if (net->avg_pending) {
    HIP_TRY(hipStreamWaitEvent(s, net->avg_done, 0));
    if (stepping_stream) net->avg_pending = false;
  }
  return NGSGD_OK;
}

GemmDesc update_desc(const ngsgd_layer& L, int N, float alpha, float beta, float* C, int ldc) {
  GemmDesc g;
  g.A = L.A; g.lda = L.lda;          // O_l stored N x dout: A^T
  g.B = L.Xin; g.ldb = L.ldx;        // Xbar_l stored N x in1
  g.C = C; g.ldc = ldc;
  g.M = L.dout; g.N = L.in1; g.K = N;
  g.alpha = alpha; g.beta = beta;
  g.alpha_dev[0] = &L.pout.st->gamma;
  g.alpha_dev[1] = &L.pin.st->gamma;
  g.alpha_dev[2] = L.mc_scale;
  return g;
}

}  // namespace

extern "C" int ngsgd_workspace_bytes(const ngsgd_config* cfg, size_t* out_bytes) {
  if (out_bytes == nullptr) return NGSGD_EINVAL;
  NG_TRY(net_check_config(cfg));
  ngsgd_net net;
  Carver c(nullptr);
  net_layout(net, cfg, c);
  *out_bytes = align_up(c.off, 256);
  return NGSGD_OK;
}

extern "C" int ngsgd_create(const ngsgd_config* cfg, void* dev_workspace, size_t workspace_bytes, ngsgd_net** out) {
  if (out == nullptr || dev_workspace == nullptr) return NGSGD_EINVAL;
  if (reinterpret_cast<uintptr_t>(dev_workspace) & 255u) return NGSGD_EINVAL;
  size_t need = 0;
  NG_TRY(ngsgd_workspace_bytes(cfg, &need));
  if (workspace_bytes < need) return NGSGD_ENOMEM;
  ngsgd_net* net = new (std::nothrow) ngsgd_net();
  if (net == nullptr) return NGSGD_ENOMEM;
  Carver c(dev_workspace);
  net_layout(*net, cfg, c);
  hipError_t e = hipMemset(dev_workspace, 0, need);
  PrecondScalars init;
  std::memset(&init, 0, sizeof(init));
  init.gamma = 1.0;
  const double one = 1.0;
  for (auto& L : net->layers) {
    if (e == hipSuccess) e = hipMemcpy(L.pin.st, &init, sizeof(init), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(L.pout.st, &init, sizeof(init), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(L.mc_scale, &one, sizeof(one), hipMemcpyHostToDevice);
  }
  // second stream for the factor updates: default priority, does not synchronise with the NULL stream
  if (e == hipSuccess) e = hipEventCreateWithFlags(&net->step_done, hipEventDisableTiming);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&net->avg_done, hipEventDisableTiming);
  for (int k = 0; k < net->n_side; ++k) {
    SideSync& sd = net->side[k];
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&sd.stream, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&sd.inputs_ready, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&sd.hj_done, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&sd.outputs_done, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&sd.done, hipEventDisableTiming);
  }
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    g_last_hip_error = (int)e;
    ngsgd_destroy(net);
    return NGSGD_EHIP;
  }
  *out = net;
  return NGSGD_OK;
}

extern "C" int ngsgd_destroy(ngsgd_net* net) {
  if (net == nullptr) return NGSGD_EINVAL;
  for (SideSync& sd : net->side) {
    if (sd.stream != nullptr) {
      (void)hipStreamSynchronize(sd.stream);
      (void)hipStreamDestroy(sd.stream);
    }
    for (hipEvent_t ev : {sd.inputs_ready, sd.hj_done, sd.outputs_done, sd.done})
      if (ev != nullptr) (void)hipEventDestroy(ev);
  }
  for (hipEvent_t ev : {net->step_done, net->avg_done})
    if (ev != nullptr) (void)hipEventDestroy(ev);
  delete net;
  return NGSGD_OK;
}

extern "C" int ngsgd_step(ngsgd_net* net, const float* dev_x, const int32_t* dev_labels, int32_t N, float lr,
                          double* dev_logprob_sum, void* hip_stream) {
  if (net == nullptr || dev_x == nullptr || dev_labels == nullptr) return NGSGD_EINVAL;
  if (N < 1 || N > net->max_batch || !aligned16(dev_x)) return NGSGD_EINVAL;
  if (net->method == NGSGD_METHOD_SIMPLE && N < 2) return NGSGD_EINVAL;   // nothing to hold out
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int nl = net->n_layers;
  auto& Ls = net->layers;
  for (SideSync& sd : net->side) sd.owner = s;
  NG_TRY(order_after_average(net, s, true));
  for (auto& L : Ls) {   // argument errors must leave the state untouched: check before any launch
    if (L.pin.rank > 0 && L.pin.t == 0 && N <= L.pin.rank) return NGSGD_EINVAL;
    if (L.pout.rank > 0 && L.pout.t == 0 && N <= L.pout.rank) return NGSGD_EINVAL;
  }

  // forward (Sec. 2): A_l = [X_l, 1] W_l^T, nonlinearity, log-softmax; the objective is cleared by the first
  // kernel of the step and accumulated by the log-softmax kernel
  double* const objective = dev_logprob_sum != nullptr ? dev_logprob_sum : net->logprob;
  {
    ProfScope prof(NGSGD_PROF_ELEMENTWISE, s);
    hipLaunchKernelGGL(copy_append_ones_kernel, dim3((Ls[0].ldx + 255) / 256, N), dim3(256), 0, s, dev_x, Ls[0].din,
                       Ls[0].Xin, Ls[0].ldx, N, Ls[0].din, objective);
    LAUNCH_CHECK();
  }
  for (int l = 0; l < nl; ++l) {
    ngsgd_layer& L = Ls[l];
    GemmDesc g;
    g.A = L.Xin; g.lda = L.ldx;
    g.B = L.W; g.ldb = L.ldw;
    g.C = L.A; g.ldc = L.lda;
    g.M = N; g.N = L.dout; g.K = L.in1;
    NG_TRY(launch_layer_gemms(GEMM_FWD, &g, 1, s));
    if (l < nl - 1) {
      ProfScope prof(NGSGD_PROF_ELEMENTWISE, s);
      ngsgd_layer& Nx = Ls[l + 1];
      if (L.nonlin == NGSGD_TANH) {
        hipLaunchKernelGGL(tanh_forward_kernel, dim3((Nx.ldx + 1023) / 1024, N), dim3(256), 0, s, L.A, L.lda, Nx.Xin,
                           Nx.ldx, N, L.dout);
      } else {
        if (L.dout >= kWideRow) {
          hipLaunchKernelGGL(pnorm_forward_kernel<512>, dim3(N), dim3(512), 0, s, L.A, L.lda, Nx.Xin, Nx.ldx,
                             L.sigma, N, L.groups, net->pnorm_group, net->renorm);
        } else {
          hipLaunchKernelGGL(pnorm_forward_kernel<256>, dim3(N), dim3(256), 0, s, L.A, L.lda, Nx.Xin, Nx.ldx,
                             L.sigma, N, L.groups, net->pnorm_group, net->renorm);
        }
      }
      LAUNCH_CHECK();
    }
  }
  ngsgd_layer& last = Ls[nl - 1];
  {
    ProfScope prof(NGSGD_PROF_ELEMENTWISE, s);
    if (last.dout >= kWideRow) {
      hipLaunchKernelGGL(softmax_xent_kernel<512>, dim3(N), dim3(512), 0, s, last.A, last.lda, dev_labels, N,
                         last.dout, net->rowobj, objective);
    } else {
      hipLaunchKernelGGL(softmax_xent_kernel<256>, dim3(N), dim3(256), 0, s, last.A, last.lda, dev_labels, N,
                         last.dout, net->rowobj, objective);
    }
    LAUNCH_CHECK();
  }

  // On a step whose factors are all due for an update (and none needs initialising) the products H, J and the
  // R x R work of each group of instances start on the group's side stream as soon as the group's matrices
  // exist, next to the backward pass; W_t is replaced only after Xhat has read it (the second half of each group's
  // update is enqueued at the end of the step).
  bool early = net->method == NGSGD_METHOD_ONLINE;
  for (auto& L : Ls)
    for (const ngsgd_precond* p : {&L.pin, &L.pout})
      if (p->rank > 0 && (p->t == 0 || !factor_due(*p))) early = false;
  std::vector<PrecondCall> early_calls[kSideStreams];
  int ready_layer[kSideStreams];   // a group starts once the derivatives of this layer (its lowest) exist
  for (int& r : ready_layer) r = nl - 1;
  if (early) {
    NG_TRY(ensure_kernel_attributes());
    for (int l = 0; l < nl; ++l) {
      ngsgd_layer& L = Ls[l];
      const int k = output_side_group(l, nl, net->n_side);
      ready_layer[k] = std::min(ready_layer[k], l);
      if (L.pout.rank > 0) early_calls[k].push_back(PrecondCall{&L.pout, L.A, L.lda, N, nullptr, nullptr});
      if (L.pin.rank > 0) early_calls[0].push_back(PrecondCall{&L.pin, L.Xin, L.ldx, N, nullptr, nullptr});
    }
  }
  auto early_start = [&](const int k) -> int {
    if (!early || early_calls[k].empty()) return NGSGD_OK;
    SideSync& sd = net->side[k];
    HIP_TRY(hipEventRecord(sd.inputs_ready, s));
    HIP_TRY(hipStreamWaitEvent(sd.stream, sd.inputs_ready, 0));
    NG_TRY(clear_accumulators(early_calls[k], sd.stream));
    NG_TRY(launch_h_products(early_calls[k], sd.stream));
    NG_TRY(launch_j_products(early_calls[k], sd.stream));
    HIP_TRY(hipEventRecord(sd.hj_done, sd.stream));
    return factor_begin(early_calls[k], sd.stream);
  };
  for (int k = 0; k < kSideStreams; ++k)
    if (ready_layer[k] == nl - 1) NG_TRY(early_start(k));   // (empty groups return at once)

  // backward on the unmodified derivatives (App. C.3, last paragraph)
  for (int l = nl - 1; l >= 1; --l) {
    ngsgd_layer& L = Ls[l];
    ngsgd_layer& P = Ls[l - 1];
    GemmDesc g;
    g.A = L.A; g.lda = L.lda;           // O_l, N x dout
    g.B = L.W; g.ldb = L.ldw;           // W_l as dout x din (bias column dropped)
    g.C = net->dX; g.ldc = net->lddx;
    g.M = N; g.N = L.din; g.K = L.dout;
    // few output tiles and a long K: split K into slabs that the nonlinearity's backward kernel sums
    const size_t slab = (size_t)net->max_batch * net->lddx;
    g.c_split_stride = (long long)slab;
    const int tiles = ((N + 63) / 64) * ((L.din + 63) / 64);
    g.splits = std::min(kMaxBwdSplits, choose_splits(tiles, (L.dout + LBK - 1) / LBK));
    const int n_slabs = planned_splits<64, 64, LBK>(g);   // depends on the K-block only, not on the tile shape
    NG_TRY(launch_layer_gemms(GEMM_BWD, &g, 1, s));
    ProfScope prof(NGSGD_PROF_ELEMENTWISE, s);
    if (P.nonlin == NGSGD_TANH) {
      hipLaunchKernelGGL(tanh_backward_kernel, dim3((P.dout + 1023) / 1024, N), dim3(256), 0, s, net->dX, net->lddx,
                         n_slabs, slab, L.Xin, L.ldx, P.A, P.lda, N, P.dout);
    } else {
      if (P.dout >= kWideRow) {
        hipLaunchKernelGGL(pnorm_backward_kernel<512>, dim3(N), dim3(512), 0, s, net->dX, net->lddx, n_slabs, slab,
                           L.Xin, L.ldx, P.sigma, P.A, P.lda, N, P.groups, net->pnorm_group, net->renorm);
      } else {
        hipLaunchKernelGGL(pnorm_backward_kernel<256>, dim3(N), dim3(256), 0, s, net->dX, net->lddx, n_slabs, slab,
                           L.Xin, L.ldx, P.sigma, P.A, P.lda, N, P.groups, net->pnorm_group, net->renorm);
      }
    }
    LAUNCH_CHECK();
    // the derivatives of layer l - 1 exist now: start the group of which it is the lowest layer
    for (int k = 0; k < kSideStreams; ++k)
      if (ready_layer[k] == l - 1) NG_TRY(early_start(k));
  }

  // maximum parameter change (App. C.3), then W_l += lr a_l gamma_o gamma_x Ohat_l^T Xhat_l  (Sec. 4.6) for the
  // listed layers, once both of their matrices are preconditioned
  auto update_layers = [&](const std::vector<int>& layers) -> int {
    if (layers.empty()) return NGSGD_OK;
    if (net->max_change_per_sample > 0.0) {
      MaxChangeGroup g;
      g.count = (int)layers.size();
      g.lr = lr;
      g.max_change_per_sample = net->max_change_per_sample;
      for (size_t i = 0; i < layers.size(); ++i) {
        ngsgd_layer& L = Ls[layers[i]];
        MaxChangeArgs& a = g.a[i];
        a.prow_o = L.pout.prow;
        a.prow_x = L.pin.prow;
        a.gamma_o = &L.pout.st->gamma;
        a.gamma_x = &L.pin.st->gamma;
        a.scale_out = L.mc_scale;
        a.N = N;
      }
      ProfScope prof(NGSGD_PROF_ELEMENTWISE, s);
      hipLaunchKernelGGL(max_change_kernel, dim3(g.count), dim3(256), 0, s, g);
      LAUNCH_CHECK();
    }
    std::vector<GemmDesc> upd;
    for (const int l : layers) upd.push_back(update_desc(Ls[l], N, lr, 1.f, Ls[l].W, Ls[l].ldw));
    return launch_layer_gemms(GEMM_UPD, upd.data(), (int)upd.size(), s);
  };
  std::vector<int> all_layers;
  for (int l = 0; l < nl; ++l) all_layers.push_back(l);

  // natural gradient: both matrices of every layer (Sec. 4.6; 2I instances), grouped calls; the factor updates
  // overlap the rest of this step and the next step's forward and backward passes on the side streams
  if (net->method == NGSGD_METHOD_SIMPLE) {
    // App. A instead: the factors come from the other rows of this minibatch, no state
    std::vector<SimpleCall> calls;
    for (auto& L : Ls) {
      calls.push_back(SimpleCall{L.A, L.lda, N, L.dout, net->alpha, net->simple_epsilon, L.sout, L.pout.prow,
                                 &L.pout.st->gamma, nullptr, nullptr});
      calls.push_back(SimpleCall{L.Xin, L.ldx, N, L.in1, net->alpha, net->simple_epsilon, L.sin, L.pin.prow,
                                 &L.pin.st->gamma, nullptr, nullptr});
    }
    NG_TRY(simple_many(calls, false, s));
    NG_TRY(update_layers(all_layers));
  } else if (early) {
    std::vector<PrecondCall> calls;
    for (auto& L : Ls) {
      calls.push_back(PrecondCall{&L.pout, L.A, L.lda, N, nullptr, nullptr});
      calls.push_back(PrecondCall{&L.pin, L.Xin, L.ldx, N, nullptr, nullptr});
    }
    // Xhat and gamma behind every group's H and J; the second half of each group's factor update is enqueued
    // after the rest of this step so that the caller's stream is never short of work
    // (the group whose matrices appeared last is still busy with H and J when the backward pass ends: the Xhat
    // products of the other groups go first)
    std::vector<PrecondCall> due;
    for (int k = 0; k < kSideStreams; ++k) {
      if (early_calls[k].empty()) continue;
      HIP_TRY(hipStreamWaitEvent(s, net->side[k].hj_done, 0));
      NG_TRY(precond_apply(early_calls[k], false, s, due, true, true, false));
    }
    NG_TRY(precond_apply(calls, false, s, due, true, false, true));
    for (int k = 0; k < kSideStreams; ++k)
      if (!early_calls[k].empty()) HIP_TRY(hipEventRecord(net->side[k].outputs_done, s));
    for (auto& c : calls) c.p->t += 1;
    NG_TRY(update_layers(all_layers));
    for (int k = 0; k < kSideStreams; ++k) {
      if (early_calls[k].empty()) continue;
      SideSync& sd = net->side[k];
      HIP_TRY(hipStreamWaitEvent(sd.stream, sd.outputs_done, 0));
      NG_TRY(factor_finish(early_calls[k], sd.stream));
      HIP_TRY(hipEventRecord(sd.done, sd.stream));
      sd.pending = true;
    }
  } else {
    // No factor is due, or the first call of an instance (initialisation): everything on the caller's stream.
    // On the step after an update the group that started last may still be running: the layers that do not
    // depend on it are preconditioned and updated first, the others behind them.
    SideSync* const last_side = &net->side[net->n_side - 1];
    std::vector<PrecondCall> calls[2];
    std::vector<int> layers[2];
    const bool split = net->n_side > 1 && last_side->pending;
    for (int l = 0; l < nl; ++l) {
      ngsgd_layer& L = Ls[l];
      const int late = split && L.pout.sync == last_side ? 1 : 0;
      calls[late].push_back(PrecondCall{&L.pout, L.A, L.lda, N, nullptr, nullptr});
      calls[0].push_back(PrecondCall{&L.pin, L.Xin, L.ldx, N, nullptr, nullptr});
      layers[late].push_back(l);
    }
    for (SideSync& sd : net->side)
      if (!split || &sd != last_side) NG_TRY(join_side(&sd, s));
    NG_TRY(precondition_many(calls[0], false, s));
    NG_TRY(update_layers(layers[0]));
    if (split) {
      NG_TRY(join_side(last_side, s));
      if (!calls[1].empty()) NG_TRY(precondition_many(calls[1], false, s));
      NG_TRY(update_layers(layers[1]));
    }
  }
  net->last_N = N;
  net->last_lr = lr;
  net->step_stream = s;   // an averaging call on another stream orders itself behind this stream's work so far
  net->stepped = true;
  return NGSGD_OK;
}

extern "C" int ngsgd_join(ngsgd_net* net, void* hip_stream) {
  if (net == nullptr) return NGSGD_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  for (SideSync& sd : net->side) NG_TRY(join_side(&sd, s));
  return NGSGD_OK;
}

extern "C" int ngsgd_average(ngsgd_net* const* nets, int32_t n, int32_t reset_preconditioners, void* hip_stream) {
  if (nets == nullptr || n < 1 || n > kMaxReplicas) return NGSGD_EINVAL;
  for (int i = 0; i < n; ++i) {
    if (nets[i] == nullptr) return NGSGD_EINVAL;
    if (nets[i]->n_params_padded != nets[0]->n_params_padded || nets[i]->n_layers != nets[0]->n_layers)
      return NGSGD_EINVAL;
    for (int l = 0; l < nets[0]->n_layers; ++l)
      if (nets[i]->layers[l].dout != nets[0]->layers[l].dout || nets[i]->layers[l].din != nets[0]->layers[l].din)
        return NGSGD_EINVAL;
  }
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  for (int i = 0; i < n; ++i) {
    // behind the replica's latest step (whatever stream it ran on), its factor updates and an earlier averaging
    if (nets[i]->stepped && nets[i]->step_stream != s) {
      HIP_TRY(hipEventRecord(nets[i]->step_done, nets[i]->step_stream));
      HIP_TRY(hipStreamWaitEvent(s, nets[i]->step_done, 0));
    }
    NG_TRY(order_after_average(nets[i], s, false));
    for (SideSync& sd : nets[i]->side) NG_TRY(join_side(&sd, s));
  }
  AverageArgs a;
  a.n = n;
  a.count = nets[0]->n_params_padded;
  for (int i = 0; i < n; ++i) a.params[i] = nets[i]->params;
  size_t blocks = (a.count + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(average_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a);
  LAUNCH_CHECK();
  for (int i = 0; i < n; ++i) {   // the replicas' next steps (on their own streams) wait for the new weights
    HIP_TRY(hipEventRecord(nets[i]->avg_done, s));
    nets[i]->avg_pending = true;
  }
  if (reset_preconditioners)
    for (int i = 0; i < n; ++i)
      for (auto& L : nets[i]->layers) L.pin.t = L.pout.t = 0;
  return NGSGD_OK;
}

extern "C" int ngsgd_get_params(const ngsgd_net* net, int32_t layer, float* dev_out, void* hip_stream) {
  if (net == nullptr || dev_out == nullptr || layer < 0 || layer >= net->n_layers) return NGSGD_EINVAL;
  const ngsgd_layer& L = net->layers[layer];
  NG_TRY(order_after_average(const_cast<ngsgd_net*>(net), static_cast<hipStream_t>(hip_stream), false));
  return copy2d(L.W, L.ldw, dev_out, L.in1, L.dout, L.in1, 1.f, nullptr, static_cast<hipStream_t>(hip_stream));
}

extern "C" int ngsgd_set_params(ngsgd_net* net, int32_t layer, const float* dev_in, void* hip_stream) {
  if (net == nullptr || dev_in == nullptr || layer < 0 || layer >= net->n_layers) return NGSGD_EINVAL;
  ngsgd_layer& L = net->layers[layer];
  NG_TRY(order_after_average(net, static_cast<hipStream_t>(hip_stream), false));
  return copy2d(dev_in, L.in1, L.W, L.ldw, L.dout, L.in1, 1.f, nullptr, static_cast<hipStream_t>(hip_stream));
}

extern "C" int ngsgd_net_precond(ngsgd_net* net, int32_t layer, int32_t side, ngsgd_precond** out) {
  if (net == nullptr || out == nullptr || layer < 0 || layer >= net->n_layers) return NGSGD_EINVAL;
  if (side != NGSGD_SIDE_INPUT && side != NGSGD_SIDE_OUTPUT) return NGSGD_EINVAL;
  ngsgd_layer& L = net->layers[layer];
  ngsgd_precond* p = side == NGSGD_SIDE_INPUT ? &L.pin : &L.pout;
  *out = p->rank > 0 ? p : nullptr;
  return NGSGD_OK;
}

extern "C" int ngsgd_last_preconditioned(ngsgd_net* net, int32_t layer, int32_t side, float* dev_out,
                                         void* hip_stream) {
  if (net == nullptr || dev_out == nullptr || layer < 0 || layer >= net->n_layers || net->last_N < 1)
    return NGSGD_EINVAL;
  if (side != NGSGD_SIDE_INPUT && side != NGSGD_SIDE_OUTPUT) return NGSGD_EINVAL;
  ngsgd_layer& L = net->layers[layer];
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (side == NGSGD_SIDE_INPUT)
    return copy2d(L.Xin, L.ldx, dev_out, L.in1, net->last_N, L.in1, 1.f, &L.pin.st->gamma, s);
  return copy2d(L.A, L.lda, dev_out, L.dout, net->last_N, L.dout, 1.f, &L.pout.st->gamma, s);
}

extern "C" int ngsgd_last_gradient(ngsgd_net* net, int32_t layer, float* dev_out, void* hip_stream) {
  if (net == nullptr || dev_out == nullptr || layer < 0 || layer >= net->n_layers || net->last_N < 1)
    return NGSGD_EINVAL;
  ngsgd_layer& L = net->layers[layer];
  GemmDesc g = update_desc(L, net->last_N, 1.f, 0.f, dev_out, L.in1);
  return launch_layer_gemms(GEMM_UPD, &g, 1, static_cast<hipStream_t>(hip_stream));
}

extern "C" int ngsgd_last_max_change_scale(ngsgd_net* net, int32_t layer, double* dev_out, void* hip_stream) {
  if (net == nullptr || dev_out == nullptr || layer < 0 || layer >= net->n_layers) return NGSGD_EINVAL;
  HIP_TRY(hipMemcpyAsync(dev_out, net->layers[layer].mc_scale, sizeof(double), hipMemcpyDeviceToDevice,
                         static_cast<hipStream_t>(hip_stream)));
  return NGSGD_OK;
}

extern "C" const char* ngsgd_strerror(int code) {
  switch (code) {
    case NGSGD_OK: return "ok";
    case NGSGD_EINVAL: return "invalid argument";
    case NGSGD_ENOMEM: return "workspace too small";
    case NGSGD_EHIP: return "HIP runtime error";
    case NGSGD_EUNSUPPORTED: return "unsupported";
    default: return "unknown error";
  }
}

extern "C" int ngsgd_profile_enable(int32_t on) {
  g_prof.on = on != 0;
  g_prof.used = 0;
  g_prof.dropped = 0;
  g_prof.recs.clear();
  return NGSGD_OK;
}

extern "C" int ngsgd_profile_read(double* ms_out, int64_t* launches_out, int32_t n_categories) {
  if (ms_out == nullptr || launches_out == nullptr || n_categories < NGSGD_PROF_CATEGORIES) return NGSGD_EINVAL;
  for (int i = 0; i < n_categories; ++i) {
    ms_out[i] = 0.0;
    launches_out[i] = 0;
  }
  for (const auto& r : g_prof.recs) {
    HIP_TRY(hipEventSynchronize(g_prof.pool[r.e0 + 1]));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, g_prof.pool[r.e0], g_prof.pool[r.e0 + 1]));
    ms_out[r.cat] += (double)ms;
    launches_out[r.cat] += 1;
  }
  const bool complete = g_prof.dropped == 0;
  g_prof.used = 0;
  g_prof.dropped = 0;
  g_prof.recs.clear();
  return complete ? NGSGD_OK : NGSGD_ENOMEM;   // the sums miss the groups that did not fit
}

extern "C" int ngsgd_set_wait_limit_us(int64_t microseconds) {
  if (microseconds < 0) return NGSGD_EINVAL;
  g_fused_wait_us.store((long long)microseconds);
  return NGSGD_OK;
}

extern "C" int ngsgd_last_hip_error(void) { return g_last_hip_error; }
extern "C" int ngsgd_version(void) { return 100; }
