"""Pins for the oracle of the pool-capacity and dissemination arithmetic (CPU only): the paper's own statements
about its formulas, hand-worked rankings, brute force over small pools."""
import itertools
import math
import random

import pytest

from oracle import capacity as cap


def test_mu_min_is_where_the_overlap_condition_turns():
    rng = random.Random(0)
    for _ in range(200):
        kappa = rng.randint(1, 10)
        R, T = rng.uniform(1, 5000), rng.uniform(1, 3000)
        Tb = rng.uniform(0, 0.99 * kappa * T)
        m = cap.mu_min(kappa, R, T, Tb)
        assert cap.overlap_holds(kappa, R, T, Tb, m * (1 + 1e-9))
        assert not cap.overlap_holds(kappa, R, T, Tb, m * (1 - 1e-9))
    # no dissemination delay: the pool only has to produce R rollouts per learner step
    assert cap.mu_min(3, 2048, 1500.0, 0.0) == pytest.approx(2048 / 1500.0, rel=1e-15)
    # a delay of half the publication period doubles the requirement
    assert cap.mu_min(2, 100.0, 10.0, 10.0) == pytest.approx(2 * 100.0 / 10.0, rel=1e-15)


def test_staleness_bound_is_at_most_kappa_plus_one_under_the_overlap_condition():
    """The paper's claim for its settings: with the overlap condition and T_bcast < T_train the ceiling term is
    at most 2, hence kappa = S - 1 suffices (its example: S = 3, kappa = 2)."""
    rng = random.Random(1)
    seen = set()
    for _ in range(2000):
        kappa = rng.randint(1, 8)
        R, T = rng.uniform(1, 5000), rng.uniform(1, 3000)
        Tb = rng.uniform(0, 0.999 * T)
        mu = cap.mu_min(kappa, R, T, Tb) * rng.uniform(1.0, 3.0)
        b = cap.staleness_bound(kappa, R, T, Tb, mu)
        assert kappa <= b <= kappa + 1
        seen.add(b - kappa)
    assert seen == {0, 1}
    assert cap.staleness_bound(2, 2048, 1500.0, 300.0, 2048 / 1200.0) == 2      # 300 + 1200 s = exactly one step
    assert cap.staleness_bound(2, 2048, 1500.0, 301.0, 2048 / 1200.0) == 3
    # a starved pool is not covered by the claim: ten steps to collect R rollouts
    assert cap.staleness_bound(2, 1000.0, 100.0, 0.0, 1.0) == 2 + 10 - 1


def test_peer_score_components():
    # the speed term saturates at 100 when the measured rate reaches 100 Mbit/s (the paper's per-worker cap)
    assert cap.peer_score(1e8, 1.0, 0, 10, 0.0) == pytest.approx(100.0, abs=1e-12)
    assert cap.peer_score(1e3, 0.0, 4, 10, 0.0) == pytest.approx(0.0, abs=1e-12)          # 1 kbit/s, no success, unstable
    assert cap.peer_score(1e8, 0.0, 0, 0, 0.0) == pytest.approx(50.0, abs=1e-12)          # weights 0.5 / 0.35 / 0.15
    assert cap.peer_score(1e3, 1.0, 4, 0, 0.0) == pytest.approx(35.0, abs=1e-12)
    assert cap.peer_score(1e3, 0.0, 3, 10, 0.0) == pytest.approx(15.0, abs=1e-12)         # three failures still count as stable
    assert cap.peer_score(1e3, 0.0, 4, 10, 0.0) == pytest.approx(0.0, abs=1e-12)          # more than three do not
    assert cap.peer_score(1e3, 0.0, 0, 5, 0.0) == pytest.approx(7.5, abs=1e-12)           # five of ten successes
    assert cap.peer_score(1e3, 0.0, 0, 50, 0.0) == pytest.approx(15.0, abs=1e-12)
    # decay: linear over ten minutes, never below 0.7
    full = cap.peer_score(1e8, 1.0, 0, 10, 0.0)
    assert cap.peer_score(1e8, 1.0, 0, 10, 60.0) == pytest.approx(0.9 * full, rel=1e-12)
    assert cap.peer_score(1e8, 1.0, 0, 10, 180.0) == pytest.approx(0.7 * full, rel=1e-12)
    assert cap.peer_score(1e8, 1.0, 0, 10, 1e6) == pytest.approx(0.7 * full, rel=1e-12)
    # each decade of speed is worth 20 points of the speed term
    assert cap.peer_score(1e7, 0.0, 4, 0, 0.0) - cap.peer_score(1e6, 0.0, 4, 0, 0.0) == pytest.approx(10.0, abs=1e-12)


def stated_values():
    import os
    rows = []
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "paper_stated_values.txt")):
        line = line.split("#")[0].split()
        if line:
            rows.append((line[0], [float(x) for x in line[1:-1]], float(line[-1])))
    return rows


def test_values_the_paper_states():
    seen = set()
    for name, args, want in stated_values():
        seen.add(name)
        if name == "n_chains":
            assert cap.n_chains(*args) == want
        elif name == "speed_term":      # the score with nothing but the speed term, undecayed: 0.5 * Speed
            assert cap.peer_score(args[0], 0.0, 4, 0, 0.0) == pytest.approx(0.5 * want, abs=1e-12)
        elif name == "stale_bound":
            assert cap.staleness_bound(int(args[0]), *args[1:]) == want
    assert seen == {"n_chains", "speed_term", "stale_bound"}


def test_chains():
    assert [cap.n_chains(b, 100.0) for b in (300.0, 600.0, 700.0, 800.0)] == [3, 6, 7, 8]   # the paper's uplink budgets
    assert cap.n_chains(250.0, 100.0) == 2 and cap.n_chains(50.0, 100.0) == 1
    chain, hop = cap.chain_assign([5.0, 9.0, 1.0, 7.0, 3.0], 2)
    assert chain == [0, 0, 0, 1, 1] and hop == [1, 0, 2, 0, 1]
    chain, hop = cap.chain_assign([1.0, 1.0, 1.0], 5)            # fewer workers than chains: all are first hops
    assert chain == [0, 1, 2] and hop == [0, 0, 0]
    # every chain is a path: hops 0..len-1 once each, chain lengths differ by at most one, better scores sit nearer the learner
    rng = random.Random(2)
    score = [rng.random() for _ in range(23)]
    chain, hop = cap.chain_assign(score, 4)
    for c in range(4):
        members = sorted((hop[i], i) for i in range(23) if chain[i] == c)
        assert [h for h, _ in members] == list(range(len(members))) and len(members) in (5, 6)
        assert all(score[a] >= score[b] for (_, a), (_, b) in zip(members, members[1:]))


def test_greedy_activation_against_brute_force():
    rng = random.Random(3)
    for trial in range(300):
        n = rng.randint(1, 9)
        mu = [rng.uniform(0.1, 5.0) for _ in range(n)]
        cost = [rng.uniform(0.1, 5.0) for _ in range(n)]
        target = rng.uniform(0.0, 1.2 * sum(mu))
        active, got, paid, reached = cap.greedy_activate(mu, cost, target)
        assert got == pytest.approx(sum(m for m, a in zip(mu, active) if a))
        assert paid == pytest.approx(sum(c for c, a in zip(cost, active) if a))
        assert reached == (sum(mu) >= target)
        # a prefix of the rho order: nobody outside is cheaper per rollout than somebody inside
        rho = [c / m for c, m in zip(cost, mu)]
        inside = [rho[i] for i in range(n) if active[i]]
        outside = [rho[i] for i in range(n) if not active[i]]
        assert not inside or not outside or max(inside) <= min(outside)
        if reached and inside:
            # shortest such prefix: without its last (most expensive per rollout) member the target is missed
            last = max((i for i in range(n) if active[i]), key=lambda i: (rho[i], i))
            assert got - mu[last] < target
            # the knapsack optimum (Eq. 3) by brute force: the greedy pays at most one worker more than it
            best = min(sum(cost[i] for i in s) for k in range(n + 1) for s in itertools.combinations(range(n), k)
                       if sum(mu[i] for i in s) >= target)
            assert best - 1e-12 <= paid <= best + max(cost) + 1e-12
    # equal throughputs: the greedy prefix is the optimum
    active, got, paid, reached = cap.greedy_activate([1.0] * 5, [4.0, 1.0, 3.0, 2.0, 5.0], 2.5)
    assert active == [0, 1, 1, 1, 0] and paid == 6.0 and reached
    # equal rho: lower index first; an unavailable worker is passed over
    assert cap.greedy_activate([1.0, 1.0, 1.0], [2.0, 2.0, 2.0], 1.5)[0] == [1, 1, 0]
    assert cap.greedy_activate([1.0, 1.0, 1.0], [2.0, 2.0, 2.0], 1.5, available=[0, 1, 1])[0] == [0, 1, 1]
    assert cap.greedy_activate([1.0, 2.0], [1.0, 1.0], 10.0) == ([1, 1], 3.0, 2.0, False)
    assert cap.greedy_activate([1.0, 2.0], [1.0, 1.0], 0.0) == ([0, 0], 0.0, 0.0, True)
