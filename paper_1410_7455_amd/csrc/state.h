// Device-resident state of one online natural-gradient instance and shared limits.
#pragma once

#include <stdint.h>

namespace ngsgd {

constexpr int kMaxRank = 96;        // NGSGD_MAX_RANK
constexpr int kMaxInstances = 32;   // instances handled by one grouped launch (2 * NGSGD_MAX_LAYERS)
constexpr int kMaxReplicas = 64;    // replicas averaged by one call

// flags
constexpr int kFlagOrthCheck = 1;   // App. B.3.1: C_t was floored or ill-conditioned, check R R^T
constexpr int kFlagFloored = 2;     // some eigenvalue of Z_t was floored
constexpr int kFlagReorth = 4;      // the latest update re-orthogonalised W
constexpr int kFlagNoConverge = 8;  // Jacobi hit its sweep limit

// Scalars of the factorisation F_t = R_t^T D_t R_t + rho_t I (eq. low:rank), kept in fp64 on the device.
struct PrecondScalars {
  double rho;             // rho_t
  double beta;            // beta_t (eq. beta2) for the current d, rho
  double gamma;           // gamma_t of the latest call (eq. gammat)
  double tr_M;            // tr(X X^T) of the latest call
  double tr_Mhat;         // tr(Xhat Xhat^T) of the latest call
  double trace_S0;        // tr(S_0), initialisation only
  int flags;
  int sweeps;             // Jacobi sweeps used by the latest update
  double d[kMaxRank];     // diag(D_t)
  double e[kMaxRank];     // diag(E_t) (eq. etii) for the current d, rho
};

}  // namespace ngsgd
