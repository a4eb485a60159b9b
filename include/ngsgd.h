/*
 * ngsgd.h - C ABI of the MI355X NG-SGD minibatch-step library (libngsgd.so).
 *
 * One worker's natural-gradient SGD step from "Parallel training of DNNs with
 * Natural Gradient and Parameter Averaging" (Povey, Zhang, Khudanpur):
 * forward, objective, backward, online natural-gradient preconditioning of
 * both matrices that enter each layer's update, the rank-N update itself, and
 * on-device parameter averaging across replicas held on the same GPU.
 *
 * General conventions
 *   - All `dev_*` pointers are DEVICE pointers (HIP global memory on the
 *     current device).  Everything else is host memory.
 *   - Matrices are row-major fp32.  A leading dimension `ld` counts floats
 *     between consecutive rows; it must be a multiple of 4 and the base
 *     pointer 16-byte aligned.
 *   - The library allocates no device memory.  Every handle lives in a device
 *     workspace the caller allocates (size from the *_workspace_bytes call,
 *     256-byte aligned) and keeps alive until *_destroy.  Inputs and outputs
 *     stay caller-owned.
 *   - All work is enqueued on the HIP stream passed as `hip_stream` (a
 *     hipStream_t cast to void*; NULL is the default stream) and the calls
 *     return without waiting for it.  Scalars results are written to device
 *     memory.  Calls on the same handle must be issued in order on one stream.
 *     Handles are not thread-safe.
 *   - A network also owns up to three internal streams (default priority;
 *     ngsgd_config.side_streams): the factor updates of its preconditioners
 *     run there, each group of factors starting as soon as its matrix exists,
 *     so that they overlap the rest of the step and the following minibatch.
 *     Every call on the handle
 *     orders itself after whatever it depends on; a caller that wants the
 *     stream it passed to cover all of a step's work (to time it, or to read
 *     the handle's device memory directly) calls ngsgd_join first.
 *   - Every function returns NGSGD_OK (0) or a negative NGSGD_E* code.  After
 *     an error the handle's state is unchanged when the error is an argument
 *     error, and unspecified for NGSGD_EHIP.
 */
#ifndef NGSGD_H_
#define NGSGD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NGSGD_OK 0
#define NGSGD_EINVAL (-1)    /* bad argument: NULL, size, alignment, rank >= dim, N > max_batch ... */
#define NGSGD_ENOMEM (-2)    /* workspace too small */
#define NGSGD_EHIP (-3)      /* a HIP runtime call failed; see ngsgd_last_hip_error() */
#define NGSGD_EUNSUPPORTED (-4)

#define NGSGD_TANH 0
#define NGSGD_PNORM 1

#define NGSGD_MAX_LAYERS 16
#define NGSGD_MAX_RANK 96    /* the R x R update runs in one workgroup's LDS */

#define NGSGD_METHOD_ONLINE 0 /* Fisher factors from previous minibatches, App. B (the default)   */
#define NGSGD_METHOD_SIMPLE 1 /* Fisher factors from the other rows of the minibatch, App. A    */

#define NGSGD_SIDE_INPUT 0   /* preconditioner of the layer-input matrix [X_l, 1]   */
#define NGSGD_SIDE_OUTPUT 1  /* preconditioner of the output-derivative matrix O_l  */

typedef struct ngsgd_net ngsgd_net;          /* one replica: weights + 2I preconditioners */
typedef struct ngsgd_precond ngsgd_precond;  /* one instance of the online method         */

/* Network description (host memory, copied by ngsgd_create).
 * dims[0] is the input dimension, dims[1..n_layers] the output dimension of each affine layer;
 * nonlin[l] (l < n_layers-1) follows affine layer l, the last affine layer feeds a log-softmax.
 * A p-norm layer (p = 2) maps groups of `pnorm_group` adjacent outputs to their 2-norm, so the
 * next layer's input dimension is dims[l+1] / pnorm_group (must divide).  Each affine layer keeps
 * its bias as the last column of its weight matrix: W_l is dims[l+1] x (in_dim_l + 1)
 * (Sec. 4.4 of the paper).  Defaults of App. B.4/B.5: rank_in 20, rank_out 80, alpha 4,
 * num_samples_history 2000, epsilon 1e-10, update_period 4, always_update_first 10. */
typedef struct {
  int32_t n_layers;
  const int32_t* dims;
  const int32_t* nonlin;
  int32_t pnorm_group;
  int32_t max_batch;              /* largest minibatch a step will be given            */
  int32_t rank_in, rank_out;      /* 0 disables preconditioning on that side           */
  float alpha;                    /* identity smoothing, Sec. 4.8                      */
  float num_samples_history;      /* S in eta = 1 - exp(-N/S), App. B.4                */
  float epsilon;                  /* floor on rho and D, App. B.2-B.3                  */
  int32_t update_period;          /* J: factors updated when t < always_update_first   */
  int32_t always_update_first;    /*    or J divides t, App. B.4                       */
  int32_t renorm;                 /* 1: rows leave each p-norm layer with unit rms     */
  float max_change_per_sample;    /* App. C.3; 0 disables the limit (paper: 0.075)     */
  int32_t method;                 /* NGSGD_METHOD_ONLINE (App. B) or _SIMPLE (App. A)  */
  float simple_epsilon;           /* floor on tr(X^T X) in beta, App. A.2 (1e-20)      */
  int32_t side_streams;           /* internal streams for the factor updates: 0 = default
                                   * (2), else 1..3.  Two: the last layer's derivatives and
                                   * the layer inputs start after the forward pass, the
                                   * other derivatives after the backward pass (shortest
                                   * single-network step); three start the upper hidden
                                   * layers in the middle of the backward pass; one is
                                   * better when many networks share the GPU, which has
                                   * few hardware queues per process                      */
} ngsgd_config;

/* ---- one preconditioner instance (App. B) ------------------------------------------------- */

/* Device workspace needed by one instance for matrices of up to max_batch rows. */
int ngsgd_precond_workspace_bytes(int32_t dim, int32_t rank, int32_t max_batch, size_t* out_bytes);

/* Creates an instance in `dev_workspace`.  Requires 0 <= rank <= NGSGD_MAX_RANK, rank < dim.
 * The state (W_t = E_t^{1/2} R_t, D_t, rho_t) is built from the first matrix it is given
 * (App. B.3.2), which therefore needs more than `rank` rows. */
int ngsgd_precond_create(int32_t dim, int32_t rank, int32_t max_batch, float alpha,
                         float num_samples_history, float epsilon, int32_t update_period,
                         int32_t always_update_first, void* dev_workspace, size_t workspace_bytes,
                         ngsgd_precond** out);
int ngsgd_precond_destroy(ngsgd_precond* p);

/* Forgets the state: the next call re-initialises from its input, as a new process does. */
int ngsgd_precond_reset(ngsgd_precond* p);

/* The online natural-gradient call of Sec. 4.6 / App. B.5: overwrites the N x dim matrix dev_M
 * (leading dimension ld) with gamma_t * M * G_t^{-1}, which has the Frobenius norm of M, using
 * the factor estimated from the previous calls; then, when t < always_update_first or
 * update_period divides t, updates the factor with M.  t counts calls since creation / reset.
 *   dev_gamma     (optional, 1 float)  receives gamma_t (eq. gammat)
 *   dev_rownorm2  (optional, N floats) receives the squared 2-norm of each output row
 * Requires N <= max_batch; on the first call after creation/reset also N > rank. */
int ngsgd_precondition(ngsgd_precond* p, float* dev_M, int32_t N, int32_t ld, float* dev_gamma,
                       float* dev_rownorm2, void* hip_stream);

/* Copies the state out: dev_W (rank x dim floats, dense), dev_d (rank doubles, diag D_t),
 * dev_rho (1 double); *t_host receives the call counter.  Any pointer may be NULL. */
int ngsgd_precond_get_state(const ngsgd_precond* p, float* dev_W, double* dev_d, double* dev_rho,
                            int64_t* t_host, void* hip_stream);

/* Diagnostics of the latest factor update, copied to HOST memory after waiting for the stream:
 * flags (bit 0: orthogonality check still pending, 1: an eigenvalue of Z_t was floored, 2: the factor was
 * re-orthogonalised (App. B.3.1), 3: the eigen-solver hit its sweep limit) and the Jacobi sweeps it used. */
int ngsgd_precond_diagnostics(const ngsgd_precond* p, int32_t* flags_host, int32_t* sweeps_host,
                              void* hip_stream);

/* Installs a state given in the definitional form of App. B.1: dev_R (rank x dim doubles, dense,
 * orthonormal rows), dev_d (rank doubles > 0), rho > 0, and the call counter t >= 1.
 * W_t = E_t^{1/2} R_t is formed on the device (eq. beta2, etii, wt:def). */
int ngsgd_precond_set_state(ngsgd_precond* p, const double* dev_R, const double* dev_d, double rho,
                            int64_t t, void* hip_stream);

/* ---- the simple method (App. A), stateless ---------------------------------------------------- */

/* Device workspace for matrices of up to max_rows rows and dim columns. */
int ngsgd_simple_workspace_bytes(int32_t max_rows, int32_t dim, size_t* out_bytes);

/* Overwrites the N x D matrix dev_M (leading dimension ld, a multiple of 4, 16-byte aligned rows)
 * with gamma * Xhat, where row i of Xhat is (beta I + F_i)^{-1} x_i, F_i = sum_{j != i} x_j x_j^T / (N-1)
 * is estimated from the other rows, beta = alpha max(tr(X^T X), epsilon) / (N D), and gamma restores
 * the Frobenius norm of the input (App. A.2).  Computed as in App. A.3: one inverse of size
 * min(N, D) (column space if N > D, row space otherwise) and a scalar correction per row.
 *   dev_workspace  caller-owned scratch of at least ngsgd_simple_workspace_bytes(N, D) bytes,
 *                  256-byte aligned; holds nothing between calls
 *   dev_gamma      (optional, 1 float)  receives gamma
 *   dev_rownorm2   (optional, N floats) receives the squared 2-norm of each output row
 * Requires N >= 2.  Returns NGSGD_EINVAL / NGSGD_ENOMEM before anything is enqueued. */
int ngsgd_precondition_simple(float* dev_M, int32_t N, int32_t D, int32_t ld, float alpha, float epsilon,
                              void* dev_workspace, size_t workspace_bytes, float* dev_gamma,
                              float* dev_rownorm2, void* hip_stream);

/* The same call for callers that cannot allocate device memory or bring a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the scratch is a fixed array of
 * NGSGD_SIMPLE_STATIC_BYTES in the library's device image, one copy per GPU, held until the process
 * ends.  Allocates nothing, on the device or through any library.  Same arguments, results and
 * errors as ngsgd_precondition_simple; in addition NGSGD_ENOMEM when
 * ngsgd_simple_workspace_bytes(N, D) exceeds NGSGD_SIMPLE_STATIC_BYTES (16 MiB: up to 512 x 5000, or
 * any shape whose scratch fits), before anything is enqueued.  All calls on one GPU share the array:
 * calls that overlap in time on the same GPU (different streams, different threads) race; issue them
 * on one stream or order them yourself.  Must be called with the target device current. */
#define NGSGD_SIMPLE_STATIC_BYTES (16 * 1024 * 1024)
int ngsgd_precondition_simple_static(float* dev_M, int32_t N, int32_t D, int32_t ld, float alpha,
                                     float epsilon, float* dev_gamma, float* dev_rownorm2,
                                     void* hip_stream);

/* ---- one replica of the network -------------------------------------------------------------- */

int ngsgd_workspace_bytes(const ngsgd_config* cfg, size_t* out_bytes);

/* Creates a replica in `dev_workspace`; all weights start at zero (set them with
 * ngsgd_set_params; App. C.7 describes the initialisation the paper uses).  Synchronises the
 * device once. */
int ngsgd_create(const ngsgd_config* cfg, void* dev_workspace, size_t workspace_bytes,
                 ngsgd_net** out);
int ngsgd_destroy(ngsgd_net* net);

/* One NG-SGD minibatch step (Sec. 2, 4.5-4.7): maximises sum_i log p(y_i | x_i) by
 * W_l += lr * a_l * Obar_l^T Xbar_l for every layer, gradients summed over the minibatch.
 *   dev_x       N x dims[0] features, dense (ld = dims[0], which must be a multiple of 4)
 *   dev_labels  N class indices in [0, dims[n_layers])
 *   dev_logprob_sum (optional, 1 double) receives sum_i log p(y_i | x_i) evaluated before the update */
int ngsgd_step(ngsgd_net* net, const float* dev_x, const int32_t* dev_labels, int32_t N, float lr,
               double* dev_logprob_sum, void* hip_stream);

/* Makes hip_stream wait for what the network still has in flight on its internal streams (the latest
 * factor updates); enqueues nothing else. */
int ngsgd_join(ngsgd_net* net, void* hip_stream);

/* Parameter averaging of Sec. 3.1: every replica's weights are replaced by the arithmetic mean over
 * the n replicas (same configuration, same device).  With reset_preconditioners != 0 all their
 * preconditioners are reset, as the paper's re-spawned processes do (App. B.3.2).
 * The replicas may have been stepped on other streams than hip_stream: the averaging kernel waits (on
 * the device) for each replica's latest ngsgd_step and factor updates, and each replica's next call
 * waits for the averaged weights, so the caller needs no synchronisation of its own.  (The call records an
 * event on the stream of each replica's latest ngsgd_step: those streams must still exist, and no other
 * host thread may be enqueuing a step of these replicas during the call.) */
int ngsgd_average(ngsgd_net* const* nets, int32_t n, int32_t reset_preconditioners, void* hip_stream);

/* Weights of one layer as a dense dims[layer+1] x (in_dim+1) row-major matrix, bias last. */
int ngsgd_get_params(const ngsgd_net* net, int32_t layer, float* dev_out, void* hip_stream);
int ngsgd_set_params(ngsgd_net* net, int32_t layer, const float* dev_in, void* hip_stream);

/* Borrowed handle of a layer's preconditioner (side = NGSGD_SIDE_INPUT / NGSGD_SIDE_OUTPUT);
 * owned by the net, valid until ngsgd_destroy.  NULL result when that side's rank is 0. */
int ngsgd_net_precond(ngsgd_net* net, int32_t layer, int32_t side, ngsgd_precond** out);

/* Inspection of the latest step, for parity checks.  All outputs are dense row-major copies.
 *   ngsgd_last_preconditioned: the N x dim matrix Obar_l or Xbar_l (already rescaled by gamma)
 *   ngsgd_last_gradient:       a_l * Obar_l^T Xbar_l, dims[layer+1] x (in_dim+1), without lr
 *   ngsgd_last_max_change_scale: a_l of App. C.3 as one double (1 when the limit is disabled) */
int ngsgd_last_preconditioned(ngsgd_net* net, int32_t layer, int32_t side, float* dev_out,
                              void* hip_stream);
int ngsgd_last_gradient(ngsgd_net* net, int32_t layer, float* dev_out, void* hip_stream);
int ngsgd_last_max_change_scale(ngsgd_net* net, int32_t layer, double* dev_out, void* hip_stream);

/* ---- timing of kernel groups (for benchmarks) ------------------------------------------------
 * While enabled, every launch group of the categories below is bracketed by a pair of HIP events
 * recorded on the launch stream.  ngsgd_profile_read waits for the recorded events, adds the elapsed
 * milliseconds and the number of bracketed groups per category into ms_out / launches_out (arrays of
 * n_categories >= NGSGD_PROF_CATEGORIES entries, host memory) and clears the record.  Process-wide,
 * not thread-safe; at most 32768 groups are kept between reads: if more were launched the call still
 * fills the arrays with what was kept and returns NGSGD_ENOMEM. */
#define NGSGD_PROF_GEMM_FWD 0        /* A_l = [X_l, 1] W_l^T                                     */
#define NGSGD_PROF_GEMM_BWD 1        /* dX_l = O_l W_l                                           */
#define NGSGD_PROF_GEMM_UPD 2        /* W_l += lr Obar_l^T Xbar_l (one grouped launch per step)  */
#define NGSGD_PROF_PRECOND_H 3       /* H = X W^T and tr(X X^T)                                  */
#define NGSGD_PROF_PRECOND_J 4       /* J = H^T X                                                */
#define NGSGD_PROF_PRECOND_XHAT 5    /* Xhat = X - H W and row norms                             */
#define NGSGD_PROF_PRECOND_KL 6      /* K = J J^T, L = H^T H                                     */
#define NGSGD_PROF_PRECOND_SMALL 7   /* R x R update: Z_t, eigen-decomposition, A_t              */
#define NGSGD_PROF_PRECOND_WNEW 8    /* W_{t+1} = A_t B_t                                        */
#define NGSGD_PROF_ELEMENTWISE 9     /* nonlinearities, log-softmax, max-change                  */
#define NGSGD_PROF_PRECOND_MISC 10   /* clears, gamma, B_t, orthogonality check, rescale         */
#define NGSGD_PROF_INIT 11           /* state initialisation from the first minibatch            */
#define NGSGD_PROF_SIMPLE_GRAM 12    /* simple method: X^T X or X X^T                            */
#define NGSGD_PROF_SIMPLE_INVERSE 13 /* simple method: (beta I + Gram / (N-1))^{-1}              */
#define NGSGD_PROF_SIMPLE_APPLY 14   /* simple method: Q, per-row factors, gamma                 */
#define NGSGD_PROF_PRECOND_FUSED 15  /* H, Xhat and row norms in one pass (calls without factor update) */
#define NGSGD_PROF_CATEGORIES 16
int ngsgd_profile_enable(int32_t on);
int ngsgd_profile_read(double* ms_out, int64_t* launches_out, int32_t n_categories);

/* ---- diagnostics -------------------------------------------------------------------------- */
const char* ngsgd_strerror(int code);
/* The fused apply kernel (Xhat = X - (X W^T) W in one pass, used by calls that do not update their
 * factor) lets the workgroups that share a block of rows wait for each other's part of X W^T.  The wait
 * is bounded: after this many microseconds (default 2000) a workgroup stops waiting and leaves its part
 * of the matrix to the (slow) completion step of the following kernel, so the kernel ends whatever else
 * occupies the GPU.  0 makes every workgroup take that route at once unless its partners have already
 * finished (used by the tests of that route).  Process-wide. */
int ngsgd_set_wait_limit_us(int64_t microseconds);
/* hipError_t value of the most recent failed HIP call on this thread (0 if none). */
int ngsgd_last_hip_error(void);
/* Library version: major * 10000 + minor * 100 + patch. */
int ngsgd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* NGSGD_H_ */
