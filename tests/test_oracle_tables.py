"""End-to-end pins of the oracle's encoder + decoder: the statistics the paper
prints for synthetic Gaussian keys at d = 128 (no dataset needed).  A dropped
term, a wrong sign or index anywhere in rotation, octahedral map, rounding,
codebooks or reconstruction moves these numbers by far more than the
tolerance."""
import numpy as np
import pytest

import oracle
from paper_2605_21226_amd import synth

D = 128


def _metrics(plan, mode, seed, n, n_query):
    keys = synth.gaussian_keys(seed, n, D)
    s = synth.sign_vectors(seed, 1, D)[0]
    k_hat = oracle.reconstruct(plan, oracle.encode(plan, keys, s, mode=mode), s)
    per_key = np.mean((k_hat - keys) ** 2, axis=1)
    cos = np.sum(k_hat * keys, axis=1) / (np.linalg.norm(k_hat, axis=1) * np.linalg.norm(keys, axis=1))
    q = synth.gaussian_queries(seed, n_query, D)
    ip = np.mean(np.abs(q @ keys.T - q @ k_hat.T))
    return dict(mse=float(np.mean(per_key)), cos=float(np.mean(cos)), tail95=float(np.percentile(per_key, 95)), ip=float(ip))


def _avg(plan, mode, seeds, n, n_query):
    ms = [_metrics(plan, mode, seed, n, n_query) for seed in seeds]
    return {k: float(np.mean([m[k] for m in ms])) for k in ms[0]}


def _close(got, printed, rel, digits):
    """within rel of the printed value, plus half a unit of its last printed digit"""
    return abs(got - printed) <= rel * abs(printed) + 0.5 * 10.0 ** (-digits)


def test_bit_split_diagonal_table(golden):
    """App. D: MSE and 1 - cos for 13 (b_dir, b_nrm) pairs, n = 8192, 4 seeds, local 3x3."""
    for b_dir, b_nrm, mse, omc in golden("bit_split_diagonal.txt"):
        plan = oracle.make_plan_pair(D, int(b_dir), int(b_nrm))
        m = _avg(plan, oracle.MODE_LOCAL_3X3, range(4), 8192, 4)
        assert _close(m["mse"], float(mse), 0.015, 4), (b_dir, b_nrm, m)
        assert _close(1 - m["cos"], float(omc), 0.015, 4), (b_dir, b_nrm, m)


def test_implemented_split_is_the_diagonal_minimum(golden):
    """Sec. 3.3: (b+1, b-1) has the lowest MSE of the diagonal through (b, b)."""
    for b in (2, 3, 4):
        mse = {}
        for delta in (-1, 0, 1, 2):
            if b - delta < 1:
                continue
            plan = oracle.make_plan_pair(D, b + delta, b - delta)
            mse[delta] = _metrics(plan, oracle.MODE_LOCAL_3X3, 0, 2048, 4)["mse"]
        assert min(mse, key=mse.get) == 1, (b, mse)


@pytest.mark.parametrize("b", [1, 2, 3, 4])
def test_rounding_ablation_table(golden, b):
    """App. E: scalar vs local 3x3 vs local 2x2 rounding at matched bits, n = 4096, 64 queries, 5 seeds.
    The printed "scalar" rows are three independent nearest-centroid rounds (Sec. 3.5); local 2x2 is read
    as the seed cell and its upper neighbour per axis (App. E does not define it; the bracketing pair of
    centroids would reproduce the 3x3 rows instead)."""
    rows = {r[1]: [float(x) for x in r[2:]] for r in golden("rounding_ablation.txt") if int(r[0]) == b}
    plan = oracle.make_plan(D, b)
    for name, mode in (("scalar", oracle.MODE_INDEPENDENT), ("local_3x3", oracle.MODE_LOCAL_3X3),
                       ("local_2x2", oracle.MODE_LOCAL_2X2)):
        cos, mse, tail95, ip = rows[name]
        m = _avg(plan, mode, range(5), 4096, 64)
        assert _close(m["cos"], cos, 0.002, 3), (b, name, m)
        assert _close(m["mse"], mse, 0.015, 4), (b, name, m)
        assert _close(m["tail95"], tail95, 0.02, 4), (b, name, m)
        assert _close(m["ip"], ip, 0.03, 3), (b, name, m)
    # "full" prints the same row as local_3x3: same records on a subsample
    keys = synth.gaussian_keys(99, 256, D)
    s = synth.sign_vectors(99, 1, D)[0]
    assert np.array_equal(oracle.encode(plan, keys, s, mode=oracle.MODE_LOCAL_3X3),
                          oracle.encode(plan, keys, s, mode=oracle.MODE_FULL))


def test_synthetic_fidelity_table(golden):
    """Sec. 4.1 table, OCTOPUS rows (n = 1024, 16 queries; 16 of the 64 seeds here)."""
    for b, cos, mse, ip in golden("synthetic_fidelity.txt"):
        plan = oracle.make_plan(D, int(b))
        m = _avg(plan, oracle.MODE_INDEPENDENT, range(16), 1024, 16)
        assert _close(m["cos"], float(cos), 0.002, 4), (b, m)
        assert _close(m["mse"], float(mse), 0.02, 4), (b, m)
        assert _close(m["ip"], float(ip), 0.03, 3), (b, m)
