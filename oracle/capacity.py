"""Oracle for the pool-capacity and dissemination arithmetic (test infrastructure: only tests may import it).

Every function is the paper's formula or rule written out in plain Python floats (fp64), one statement per
term, with the passage it follows; nothing here is shared with the library's implementation."""
import math


def mu_min(kappa, R, T_train, T_bcast):
    """Sec. 3.3, Eq. (2): the pool throughput at which Eq. (1) holds with equality."""
    period = kappa * T_train                      # one publication period
    left_for_generation = period - T_bcast        # what dissemination leaves of it
    return (kappa * R) / left_for_generation


def overlap_holds(kappa, R, T_train, T_bcast, mu_pool):
    """Sec. 3.3, Eq. (1)."""
    generation_time = (kappa * R) / mu_pool
    return kappa * T_train >= T_bcast + generation_time


def staleness_bound(kappa, R, T_train, T_bcast, mu_pool):
    """Sec. 3.3 / App. "Worst-Case Staleness Bound under Overlap": steps until R rollouts of a new snapshot exist, on top of kappa."""
    seconds_until_R = T_bcast + R / mu_pool
    return kappa + math.ceil(seconds_until_R / T_train) - 1


def greedy_activate(mu, cost, mu_target, available=None):
    """Sec. 3.4: workers by increasing rho = c / mu (equal rho: lower index first), cheapest prefix reaching the
    target; unavailable workers (Eq. 4's a_i = 0) are passed over.  Returns (active flags, throughput, cost, reached)."""
    n = len(mu)
    ranked = sorted(range(n), key=lambda i: (cost[i] / mu[i], i))
    active = [0] * n
    got = 0.0
    paid = 0.0
    for i in ranked:
        if got >= mu_target:
            break
        if available is not None and not available[i]:
            continue
        active[i] = 1
        got += mu[i]
        paid += cost[i]
    return active, got, paid, got >= mu_target


def peer_score(avg_speed, success_rate, consecutive_failures, succ_count, elapsed_s):
    """App. "Forwarding-Chain Construction in Peer-Assisted Broadcast", worker scoring."""
    speed = 100.0 * (math.log10(avg_speed) - 3.0) / 5.0
    success = 100.0 * success_rate
    if consecutive_failures > 3:
        stability = 0.0
    else:
        stability = 100.0 * min(succ_count / 10.0, 1.0)
    decay = 1.0 - min(elapsed_s / 600.0, 0.3)
    return decay * (0.5 * speed + 0.35 * success + 0.15 * stability)


def n_chains(B0, Bw):
    """App. "Forwarding-Chain Construction in Peer-Assisted Broadcast": floor(B0 / Bw) parallel chains (at least one)."""
    return max(1, math.floor(B0 / Bw))


def chain_assign(score, chains):
    """Chain assembly: the top `chains` workers are first hops, the rest go to the chain tails round-robin in rank
    order.  Returns (chain of worker i, hop of worker i)."""
    n = len(score)
    ranked = sorted(range(n), key=lambda i: (-score[i], i))
    chain = [0] * n
    hop = [0] * n
    tails = [0] * chains
    for k, i in enumerate(ranked):
        c = k % chains
        chain[i] = c
        hop[i] = tails[c]
        tails[c] += 1
    return chain, hop
