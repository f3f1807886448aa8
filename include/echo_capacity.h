/* Capacity and dissemination arithmetic of the rollout pool (host only, no GPU): how much rollout throughput keeps a
 * learner busy, which workers to activate for it, what staleness that implies, and how workers are ranked and
 * chained for snapshot forwarding.  Plain doubles in, plain values out; nothing is allocated, no state is kept;
 * arrays are the caller's (host).  Functions return a negative value (or NaN for doubles) on invalid arguments. */
#ifndef ECHO_CAPACITY_H
#define ECHO_CAPACITY_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Aggregate throughput (rollouts/s) that lets generation and dissemination of one publication period of kappa
 * learner steps fit into it (Sec. 3.3, Eq. 2): kappa*R / (kappa*T_train - T_bcast).  R rollouts per learner step,
 * times in seconds.  NaN unless kappa >= 1, R > 0 and kappa*T_train > T_bcast >= 0. */
double echo_mu_min(double kappa, double R, double T_train, double T_bcast);

/* Overlap condition (Sec. 3.3, Eq. 1): 1 if kappa*T_train >= T_bcast + kappa*R/mu_pool, 0 if not, -1 on invalid
 * arguments (mu_pool must be positive). */
int32_t echo_overlap_holds(double kappa, double R, double T_train, double T_bcast, double mu_pool);

/* Conservative staleness bound (Sec. 3.3; App. "Worst-Case Staleness Bound under Overlap"): kappa + ceil((T_bcast + R/mu_pool)/T_train) - 1. */
int32_t echo_staleness_bound(int32_t kappa, double R, double T_train, double T_bcast, double mu_pool);

/* Greedy activation (Sec. 3.4): rank the n workers by unit throughput cost rho_i = cost_i / mu_i ascending (equal
 * rho: lower index first) and activate the shortest prefix whose cumulative throughput reaches mu_target.
 *   mu, cost    host [n], mu_i > 0 (rollouts/s), cost_i >= 0 ($/h); available host [n] of 0/1 or NULL (all 1):
 *               unavailable workers are skipped (Eq. 4's availability bit)
 *   out_active  host [n] of 0/1; out_mu / out_cost (nullable) receive the activated totals
 * Returns the number of activated workers; if even the whole pool falls short, everything available is activated
 * and the return value is -(count) - 1. */
int32_t echo_greedy_activate(const double *mu, const double *cost, const int32_t *available, int32_t n, double mu_target,
                             int32_t *out_active, double *out_mu, double *out_cost);

/* Peer score of a forwarding candidate (App. "Forwarding-Chain Construction in Peer-Assisted Broadcast", worker scoring):
 * Decay * (0.5 Speed + 0.35 Success + 0.15 Stability) with
 *   Speed = 100 (log10(avg_speed) - 3) / 5     (avg_speed in bit/s: 100 at 100 Mbit/s; not clipped)
 *   Success = 100 success_rate                 Stability = 0 if consecutive_failures > 3, else 100 min(succ_count/10, 1)
 *   Decay = 1 - min(elapsed_s / 600, 0.3). */
double echo_peer_score(double avg_speed, double success_rate, int32_t consecutive_failures, int32_t succ_count, double elapsed_s);

/* Number of forwarding chains floor(B0 / Bw) for a learner uplink budget B0 and a per-worker forwarding bandwidth Bw
 * (same unit), at least 1. */
int32_t echo_n_chains(double B0, double Bw);

/* Chain assembly: workers ranked by score descending (equal scores: lower index first); the top n_chains are the
 * first hops of chains 0..n_chains-1, the others are appended to the chain tails round-robin in rank order.
 *   out_chain host [n]: chain of worker i; out_hop host [n]: its position in the chain (0 = fed by the learner). */
int32_t echo_chain_assign(const double *score, int32_t n, int32_t n_chains, int32_t *out_chain, int32_t *out_hop);

#ifdef __cplusplus
}
#endif
#endif
