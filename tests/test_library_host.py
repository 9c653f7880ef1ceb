"""Host-side checks of the C-ABI library that need no GPU: it loads, exports what the header declares, and its
CPU scheduler agrees with the oracle's exhaustive search and with the oracle's Algorithm 2, bit for bit."""
import math
import os
import re

import numpy as np
import pytest

from paper_2502_11058_amd import binding as B
from paper_2502_11058_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = []
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names += re.findall(r"\b(ddp_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_library_loads_and_exports_every_declared_symbol():
    lib = B.lib()
    declared = _declared_functions()
    assert len(declared) >= 15
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(B.EXPORTS) == declared


def test_missing_library_fails_loudly_no_fallback():
    # the product path has no CPU fallback: without the built library every entry point raises
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = ("from paper_2502_11058_amd import binding as B\n"
            "try:\n    B.ddp_schedule('enp', 4, 2, None, None, None)\nexcept FileNotFoundError as e:\n    print('missing:', e)\n")
    env = dict(os.environ, DREAMDDP_LIB="/nonexistent/libdreamddp.so", PYTHONPATH=root)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "missing: /nonexistent/libdreamddp.so is missing" in r.stdout, r.stdout + r.stderr


def test_create_without_gpu_fails_cleanly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(B.DdpError) as e:
        B.Context(0)
    assert e.value.code in (1, 5)


def _sets(policy, L, H, bp=None, comm=None):
    slot, sp, sl, cost = B.ddp_schedule(policy, L, H, None, bp, comm)
    return B.sets_from_csr(sp, sl), slot, cost


def test_opt_equals_brute_force_small(oracle):
    rng = np.random.default_rng(10)
    for _ in range(1500):
        L, H = int(rng.integers(1, 7)), int(rng.integers(1, 4))
        bp = rng.integers(0, 12, L)
        comm = rng.integers(0, 25, L)
        sizes, cost, _ = oracle.sched_brute(bp, comm, H)
        sets, slot, c = _sets("opt", L, H, bp, comm)
        assert sets == oracle.sets_from_sizes(L, sizes) and c == cost
        for s, S in enumerate(sets):
            assert all(slot[l] == s for l in S)


def test_opt_equals_brute_force_larger(oracle):
    rng = np.random.default_rng(11)
    for _ in range(60):
        L, H = int(rng.integers(7, 13)), int(rng.integers(2, 6))
        bp = rng.integers(1, 1000, L)
        comm = rng.integers(1, 4000, L)
        sizes, cost, n = oracle.sched_brute(bp, comm, H)
        assert n == math.comb(L + H - 1, H - 1)
        sets, _, c = _sets("opt", L, H, bp, comm)
        assert sets == oracle.sets_from_sizes(L, sizes) and c == cost


def test_alg2_equals_oracle_alg2(oracle):
    rng = np.random.default_rng(12)
    for _ in range(1500):
        L, H = int(rng.integers(1, 14)), int(rng.integers(1, 7))
        bp = rng.integers(0, 30, L)
        comm = rng.integers(0, 60, L)
        sizes, cost, omega = oracle.sched_alg2(bp, comm, H)
        sets, _, c = _sets("alg2", L, H, bp, comm)
        assert sets == oracle.sets_from_sizes(L, sizes) and c == cost
        assert B.ddp_schedule_alg2_solutions(bp, comm, H) == len(omega)
        assert c >= _sets("opt", L, H, bp, comm)[2]


def _branching_instance(L):
    """Backward 1 per layer, communication alternating 0 / huge: every second layer leaves both of Algorithm 2's
    branches open, so its solution set grows like the Fibonacci numbers."""
    return np.ones(L, dtype=np.int64), np.array([0 if i % 2 == 0 else 10 ** 6 for i in range(L)], dtype=np.int64)


def test_alg2_on_a_branching_instance_equals_oracle(oracle):
    bp, comm = _branching_instance(40)
    sizes, cost, omega = oracle.sched_alg2(bp, comm, 20)
    assert len(omega) == 6765                                            # F(20)
    sets, _, c = _sets("alg2", 40, 20, bp, comm)
    assert sets == oracle.sets_from_sizes(40, sizes) and c == cost
    assert B.ddp_schedule_alg2_solutions(bp, comm, 20) == len(omega)


def test_alg2_search_is_bounded():
    # L = 128, H = 64 on the same pattern would visit ~1e13 solutions: the library gives up after a fixed number of
    # steps with DDP_ESCHED and names the exact policy, which solves the instance at once
    import time
    bp, comm = _branching_instance(128)
    t0 = time.perf_counter()
    for call in (lambda: _sets("alg2", 128, 64, bp, comm), lambda: B.ddp_schedule_alg2_solutions(bp, comm, 64)):
        with pytest.raises(B.DdpError) as e:
            call()
        assert e.value.code == 6 and "DDP_SCHED_OPT" in str(e.value)
    assert time.perf_counter() - t0 < 30.0
    sets, _, c = _sets("opt", 128, 64, bp, comm)
    assert sorted(l for S in sets for l in S) == list(range(128)) and c > 0


def test_counter_example_of_optimal_hiding():
    bp, comm = [1, 1, 8, 1, 2], [2, 5, 2, 1, 9]
    assert _sets("alg2", 5, 2, bp, comm)[0::2] == ([[4, 3, 2], [1, 0]], 33)
    assert _sets("opt", 5, 2, bp, comm)[0::2] == ([[4], [3, 2, 1, 0]], 26)


@pytest.mark.parametrize("name", ["gpt2_small", "tinyllama_1b", "llama2_7b", "llama3_8b", "small_llama"])
def test_workload_schedules_match_oracle(oracle, name):
    w = W.get(name)
    fp, bp, comm = W.synthetic_times(w)
    L, H = w.n_layers, w.period
    for policy in ("enp", "round_robin", "full", "every", "alg2") + (("opt",) if math.comb(L + H - 1, H - 1) < 3e7 else ()):
        sets, slot, cost = _sets(policy, L, H, bp, comm)
        assert sets == oracle.schedule(policy, L, H, bp, comm), policy
        if policy in ("enp", "full", "opt", "alg2"):
            assert cost == oracle.sched_cost(bp, comm, [len(S) for S in sets])


def test_schedule_cost_entry_point(oracle):
    rng = np.random.default_rng(13)
    for _ in range(200):
        L, H = int(rng.integers(1, 9)), int(rng.integers(1, 5))
        bp = rng.integers(0, 30, L)
        comm = rng.integers(0, 60, L)
        cuts = sorted(rng.integers(0, L + 1, H - 1).tolist())
        edges = [0] + cuts + [L]
        sizes = [edges[i + 1] - edges[i] for i in range(H)]
        sets = oracle.sets_from_sizes(L, sizes)
        sp = np.cumsum([0] + sizes)
        sl = [l for S in sets for l in S]
        assert B.ddp_schedule_cost(bp, comm, sp, sl or [0]) == oracle.sched_cost(bp, comm, sizes)
    with pytest.raises(B.DdpError) as e:
        B.ddp_schedule_cost([1, 1], [1, 1], [0, 1, 2], [0, 1])       # not in BP order
    assert e.value.code == 6


def test_schedule_argument_errors():
    for args in [("opt", 0, 2, None, [1], [1]), ("opt", 2, 0, None, [1, 1], [1, 1]), ("opt", 2, 2, None, None, None),
                 ("opt", 2, 2, None, [1, -1], [1, 1]), ("alg2", 2, 2, None, [2 ** 62, 2 ** 62], [1, 1])]:
        with pytest.raises(B.DdpError) as e:
            B.ddp_schedule(*args)
        assert e.value.code == 1 and len(str(e.value)) > 10
    with pytest.raises(B.DdpError):
        B.ddp_schedule(17, 2, 2, None, [1, 1], [1, 1])


def test_fill_bubbles_equals_oracle(oracle):
    rng = np.random.default_rng(20)
    for _ in range(800):
        L, H = int(rng.integers(1, 12)), int(rng.integers(1, 6))
        bp = rng.integers(0, 30, L)
        comm = rng.integers(0, 30, L)
        cuts = sorted(rng.integers(0, L + 1, H - 1).tolist())
        edges = [0] + cuts + [L]
        sizes = [edges[i + 1] - edges[i] for i in range(H)]
        sp, sl = B.csr_from_sets(oracle.sets_from_sizes(L, sizes))
        osp, osl, extra = B.ddp_schedule_fill_bubbles(bp, comm, sp, sl)
        e_ref, sets_ref = oracle.fill_bubbles(bp, comm, sizes)
        assert extra.tolist() == e_ref and B.sets_from_csr(osp, osl) == sets_ref
    with pytest.raises(B.DdpError) as e:
        B.ddp_schedule_fill_bubbles([1, 1], [1, 1], [0, 1, 2], [0, 1])
    assert e.value.code == 6


def test_time_model_equals_oracle(oracle):
    rng = np.random.default_rng(21)
    for _ in range(800):
        L, H = int(rng.integers(1, 12)), int(rng.integers(1, 6))
        fp = rng.integers(0, 10, L)
        bp = rng.integers(0, 30, L)
        comm = rng.integers(0, 60, L)
        # arbitrary subsets in BP order, not only cuts
        sets = [sorted(rng.choice(L, int(rng.integers(0, L + 1)), replace=False).tolist(), reverse=True) for _ in range(H)]
        sp, sl = B.csr_from_sets(sets)
        it, ex, period = B.ddp_schedule_time_model(fp, bp, comm, sp, sl)
        it_ref, ex_ref, per_ref = oracle.time_model(fp, bp, comm, sets)
        assert it.tolist() == it_ref and ex.tolist() == ex_ref and period == per_ref
    with pytest.raises(B.DdpError) as e:
        B.ddp_schedule_time_model(None, [1, 1], [1, 1], [0, 2], [0, 1])          # ascending ids
    assert e.value.code == 6


@pytest.mark.parametrize("name", ["gpt2_small", "tinyllama_1b", "llama2_7b", "llama3_8b"])
def test_filled_workload_schedules(oracle, name):
    w = W.get(name)
    fp, bp, comm = W.synthetic_times(w)
    L, H = w.n_layers, w.period
    for policy in ("enp", "opt", "alg2"):
        _, sp, sl, _ = B.ddp_schedule(policy, L, H, fp, bp, comm)
        osp, osl, extra = B.ddp_schedule_fill_bubbles(bp, comm, sp, sl)
        sizes = [int(sp[i + 1] - sp[i]) for i in range(H)]
        assert (extra.tolist(), B.sets_from_csr(osp, osl)) == oracle.fill_bubbles(bp, comm, sizes)
        it0, ex0, per0 = B.ddp_schedule_time_model(fp, bp, comm, sp, sl)
        it1, ex1, per1 = B.ddp_schedule_time_model(fp, bp, comm, osp, osl)
        assert (it1.tolist(), ex1.tolist(), per1) == oracle.time_model(fp, bp, comm, B.sets_from_csr(osp, osl))


def test_header_is_plain_c_and_the_library_links_from_c(tmp_path):
    """include/dreamddp.h compiles as strict C99 and a C program linked against the shared library calls the scheduler."""
    import shutil
    import subprocess
    if not shutil.which("gcc"):
        pytest.skip("no C compiler")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    libdir = os.path.dirname(B.LIB_PATH)
    exe = str(tmp_path / "schedule_from_c")
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I" + os.path.join(root, "include"),
           os.path.join(root, "tests", "c_abi", "schedule_from_c.c"), "-L" + libdir, "-ldreamddp", "-Wl,-rpath," + libdir,
           "-Wl,--allow-shlib-undefined", "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    env = dict(os.environ, LD_LIBRARY_PATH=os.pathsep.join(filter(None, ["/opt/rocm/lib", os.environ.get("LD_LIBRARY_PATH", "")])))
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    lines = r.stdout.strip().splitlines()
    assert lines[0] == "policy 5 cost 33 sets 4 3 2 | 1 0 period 33"
    assert lines[1] == "policy 4 cost 26 sets 4 | 3 2 1 0 period 33"       # Eq. (7) charges each communication from its own layer's BP on
    assert lines[2].startswith("error: ddp_schedule")
