// Host-only arithmetic of include/echo_capacity.h (no device code in this file).
#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

#include "../../include/echo_capacity.h"

namespace {
bool finite_pos(double x) { return std::isfinite(x) && x > 0; }
}  // namespace

extern "C" {

double echo_mu_min(double kappa, double R, double T_train, double T_bcast) {
  if (!(kappa >= 1) || !finite_pos(R) || !finite_pos(T_train) || !(T_bcast >= 0) || !(kappa * T_train > T_bcast)) return NAN;
  return kappa * R / (kappa * T_train - T_bcast);
}

int32_t echo_overlap_holds(double kappa, double R, double T_train, double T_bcast, double mu_pool) {
  if (!(kappa >= 1) || !finite_pos(R) || !finite_pos(T_train) || !(T_bcast >= 0) || !finite_pos(mu_pool)) return -1;
  return kappa * T_train >= T_bcast + kappa * R / mu_pool ? 1 : 0;
}

int32_t echo_staleness_bound(int32_t kappa, double R, double T_train, double T_bcast, double mu_pool) {
  if (kappa < 1 || !finite_pos(R) || !finite_pos(T_train) || !(T_bcast >= 0) || !finite_pos(mu_pool)) return -1;
  return kappa + (int32_t)std::ceil((T_bcast + R / mu_pool) / T_train) - 1;
}

int32_t echo_greedy_activate(const double *mu, const double *cost, const int32_t *available, int32_t n, double mu_target,
                             int32_t *out_active, double *out_mu, double *out_cost) {
  if (!mu || !cost || !out_active || n < 0 || !std::isfinite(mu_target)) return INT32_MIN;
  for (int i = 0; i < n; ++i)
    if (!finite_pos(mu[i]) || !(cost[i] >= 0) || !std::isfinite(cost[i])) return INT32_MIN;
  std::vector<int> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return cost[a] / mu[a] < cost[b] / mu[b]; });
  std::fill(out_active, out_active + n, 0);
  double got = 0, paid = 0;
  int count = 0;
  for (int k = 0; k < n && got < mu_target; ++k) {
    int i = order[k];
    if (available && !available[i]) continue;
    out_active[i] = 1;
    got += mu[i];
    paid += cost[i];
    ++count;
  }
  if (out_mu) *out_mu = got;
  if (out_cost) *out_cost = paid;
  return got >= mu_target ? count : -count - 1;
}

double echo_peer_score(double avg_speed, double success_rate, int32_t consecutive_failures, int32_t succ_count, double elapsed_s) {
  if (!finite_pos(avg_speed) || !(success_rate >= 0 && success_rate <= 1) || consecutive_failures < 0 || succ_count < 0 || !(elapsed_s >= 0))
    return NAN;
  double speed = 100.0 * (std::log10(avg_speed) - 3.0) / 5.0;
  double success = 100.0 * success_rate;
  double stability = consecutive_failures > 3 ? 0.0 : 100.0 * std::min(succ_count / 10.0, 1.0);
  double decay = 1.0 - std::min(elapsed_s / 600.0, 0.3);
  return decay * (0.5 * speed + 0.35 * success + 0.15 * stability);
}

int32_t echo_n_chains(double B0, double Bw) {
  if (!finite_pos(B0) || !finite_pos(Bw)) return -1;
  double q = std::floor(B0 / Bw);
  return q < 1 ? 1 : q > 2147483647.0 ? INT32_MAX : (int32_t)q;
}

int32_t echo_chain_assign(const double *score, int32_t n, int32_t n_chains, int32_t *out_chain, int32_t *out_hop) {
  if (!score || !out_chain || !out_hop || n < 0 || n_chains < 1) return -1;
  std::vector<int> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return score[a] > score[b]; });
  for (int k = 0; k < n; ++k) {
    out_chain[order[k]] = k % n_chains;
    out_hop[order[k]] = k / n_chains;
  }
  return 0;
}

}  // extern "C"
