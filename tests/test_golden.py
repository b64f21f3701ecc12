"""The oracle reproduces its frozen toy-workload results (a regression value;
see tests/golden/make_golden.py for what it is and is not)."""
import importlib.util
import json
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def test_toy_oracle_regression():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    with open(os.path.join(HERE, "golden", "toy_oracle.json")) as f:
        want = json.load(f)
    got = json.loads(json.dumps(mod.compute()))
    assert got == want
    T, k = 512, 2
    n_exact, n_hit, n_cover, n_top1 = want["score_k2_vs_ref"]
    assert n_exact == n_cover <= T and n_exact <= n_top1 <= T and n_hit <= T * k
    assert want["score_k3_vs_ref"][2] >= n_cover       # a wider prediction covers at least as often
    assert sum(want["counts"]) == T * k
