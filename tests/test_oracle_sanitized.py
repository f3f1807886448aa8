"""The oracle's pins once more under AddressSanitizer + UndefinedBehaviorSanitizer (host code only): the fp64 oracle
and its fp32 sibling are rebuilt with -fsanitize=address,undefined and the pin tests run in a child process with the
sanitizer runtime preloaded; any out-of-bounds access, use after free or undefined operation ends the child with a
report.  The library's host-only capacity arithmetic is rebuilt the same way and driven against its oracle."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CAPACITY_DRIVER = r"""
import ctypes as C, math, random, sys
sys.path.insert(0, %(root)r)
from oracle import capacity as cap
L = C.CDLL(%(lib)r)
L.echo_mu_min.restype = C.c_double; L.echo_mu_min.argtypes = [C.c_double] * 4
L.echo_staleness_bound.restype = C.c_int32; L.echo_staleness_bound.argtypes = [C.c_int32] + [C.c_double] * 4
L.echo_peer_score.restype = C.c_double; L.echo_peer_score.argtypes = [C.c_double, C.c_double, C.c_int32, C.c_int32, C.c_double]
L.echo_n_chains.restype = C.c_int32; L.echo_n_chains.argtypes = [C.c_double, C.c_double]
L.echo_chain_assign.restype = C.c_int32; L.echo_chain_assign.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
L.echo_greedy_activate.restype = C.c_int32
L.echo_greedy_activate.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_double, C.c_void_p, C.c_void_p, C.c_void_p]
rng = random.Random(3)
for _ in range(200):
    k = rng.randint(1, 9); R, T = rng.uniform(1, 5000), rng.uniform(1, 3000); Tb = rng.uniform(0, 0.99 * k * T); mu = rng.uniform(0.01, 50)
    assert abs(L.echo_mu_min(k, R, T, Tb) - cap.mu_min(k, R, T, Tb)) <= 1e-12 * cap.mu_min(k, R, T, Tb)
    assert L.echo_staleness_bound(k, R, T, Tb, mu) == cap.staleness_bound(k, R, T, Tb, mu)
assert L.echo_n_chains(1e12, 1.0) == 2 ** 31 - 1 and L.echo_n_chains(0.0, 100.0) == -1
for n, chains in ((0, 1), (1, 3), (23, 4), (64, 8), (10, 10), (5, 64)):
    score = (C.c_double * max(n, 1))(*[round(rng.random(), 1) for _ in range(n)])
    chain, hop = (C.c_int32 * max(n, 1))(), (C.c_int32 * max(n, 1))()
    assert L.echo_chain_assign(score, n, chains, chain, hop) == 0
    want_chain, want_hop = cap.chain_assign(list(score)[:n], chains)
    assert list(chain)[:n] == want_chain and list(hop)[:n] == want_hop
for n in (0, 1, 7, 200):
    mu = (C.c_double * max(n, 1))(*[rng.uniform(0.1, 5) for _ in range(n)])
    cost = (C.c_double * max(n, 1))(*[rng.uniform(0.1, 3) for _ in range(n)])
    act = (C.c_int32 * max(n, 1))()
    got, paid = C.c_double(), C.c_double()
    L.echo_greedy_activate(mu, cost, None, n, 0.4 * sum(list(mu)[:n]), act, C.byref(got), C.byref(paid))
print("capacity ok")
"""


def test_oracle_pins_and_capacity_arithmetic_under_asan_and_ubsan(tmp_path):
    from oracle import build as ob
    libs = ob.build_sanitized()
    env = dict(os.environ, LD_PRELOAD=ob.asan_runtime(), ORACLE_SANITIZE="1", OMP_NUM_THREADS="4",
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:exitcode=97", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    pins = ["tests/test_oracle_model.py", "tests/test_oracle_primitives.py", "tests/test_oracle_rng_sampler.py",
            "tests/test_oracle_top_p.py", "tests/test_oracle_grpo.py"]
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *pins], cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail
    drv = tmp_path / "cap_driver.py"
    drv.write_text(CAPACITY_DRIVER % {"root": ROOT, "lib": libs["capacity"]})
    r = subprocess.run([sys.executable, str(drv)], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "capacity ok" in r.stdout, (r.stdout + r.stderr)[-3000:]
