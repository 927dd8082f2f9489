"""CPU checks of the helpers the GPU parity tests rely on (no GPU, no HIP library)."""
import numpy as np

from gpu_util import check_selection, drift_bounds, topb_sum_bounds


def _topb_sum(row, bt):
    order = np.argsort(-row, kind="stable")
    return int(order[:bt].sum())


def test_topb_sum_bounds_hold_for_any_perturbation_inside_the_tolerance():
    r = np.random.default_rng(3)
    P, bt = 4000, 300
    ref = np.exp(r.standard_normal(P))
    tol = 2e-3 * ref
    lo, hi, amb = topb_sum_bounds(ref, tol, bt)
    assert lo <= _topb_sum(ref, bt) <= hi and amb >= 2
    for _ in range(200):
        got = ref + tol * r.uniform(-1, 1, P)
        assert lo <= _topb_sum(got, bt) <= hi
    # adversarial corners: push the undecided entries up from the left / from the right
    order = np.argsort(-ref, kind="stable")
    tau = ref[order[bt - 1]]
    near = np.abs(ref - tau) <= 2 * 2e-3 * tau
    for sign in (+1, -1):
        got = ref.copy()
        pos = np.arange(P)
        left = pos < np.median(pos[near])
        got[near & left] += sign * tol[near & left]
        got[near & ~left] -= sign * tol[near & ~left]
        assert lo <= _topb_sum(got, bt) <= hi


def test_topb_sum_bounds_exact_without_tolerance_and_with_full_budget():
    r = np.random.default_rng(4)
    ref = r.random(1000)
    lo, hi, amb = topb_sum_bounds(ref, np.zeros_like(ref), 100)
    assert lo == hi == _topb_sum(ref, 100) and amb == 0
    lo, hi, amb = topb_sum_bounds(ref, np.zeros_like(ref), 5000)
    assert lo == hi == 1000 * 999 // 2 and amb == 0


def test_drift_bounds_contain_the_exact_statistic():
    r = np.random.default_rng(5)
    W, P, B = 6, 3000, 200
    Ig = np.exp(r.standard_normal((W, P)))
    tol = 1e-3 * Ig
    (fl, fh), (rl, rh) = drift_bounds(Ig, tol, B, W)
    df = np.mean([_topb_sum(Ig[i], B) / B for i in range(3)])
    dr = np.mean([_topb_sum(Ig[i], B) / B for i in range(3, 6)])
    assert fl <= df <= fh and rl <= dr <= rh
    assert fh - fl < 0.05 * P and rh - rl < 0.05 * P


def test_check_selection_accepts_near_ties_only():
    P, W, B = 50, 2, 12
    fin = np.linspace(1.0, 2.0, P)
    idx = np.concatenate([np.arange(P - 10, P), [P, P + 1]])
    assert check_selection(idx, fin, W, B, 1e-3) == 0
    bad = idx.copy()
    bad[0] = 3                                   # far below the threshold
    try:
        check_selection(np.concatenate([np.sort(bad[:10]), [P, P + 1]]), fin, W, B, 1e-3)
    except AssertionError:
        pass
    else:
        raise AssertionError("a far-off index was accepted")
    fin2 = fin.copy()
    fin2[P - 11] = fin2[P - 10] * (1 - 1e-5)     # a near-tie just below the threshold
    swap = np.concatenate([[P - 11], np.arange(P - 9, P), [P, P + 1]])
    assert check_selection(swap, fin2, W, B, 1e-3) == 2


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N above 1 exits with a message instead of timing anything."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="2")
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py")], capture_output=True, text=True, timeout=120,
                       env=env)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_product_and_oracle_do_not_know_each_other():
    """No source of the package mentions the oracle, no source of the oracle mentions the package
    (the two share no code; only tests, the smoke check and the benchmark's CPU leg use both)."""
    import os
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

    def sources(top, exts):
        for d, _, files in os.walk(os.path.join(root, top)):
            if "_build" in d or "__pycache__" in d:
                continue
            for f in files:
                if f.endswith(exts):
                    yield os.path.join(d, f)

    for path in sources("paper_2605_08840_amd", (".py", ".hip", ".hpp", ".h")):
        text = open(path).read()
        assert not re.search(r"\boracle\b", text), path
    for path in list(sources("oracle", (".py", ".c", ".h"))):
        text = open(path).read()
        assert "paper_2605_08840_amd" not in text and "librestkv.so" not in text and "restkv.h" not in text, path
    assert not re.search(r"\boracle\b", open(os.path.join(root, "include", "restkv.h")).read())
