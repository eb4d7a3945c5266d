"""Latency model (Experiments, table "Latency calculation"; Eq. 9) and sender-queue order
(Algorithm 2): the oracle's restatement pinned to the numbers the paper prints, and the
library's host-side functions against the oracle.  No GPU needed."""
import math
import os

import numpy as np
import pytest

import paper_2505_21594_amd as ee
from oracle import latency as lo

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "latency_worked_example.txt")


def _gold():
    kv, c_rows, proj = {}, [], []
    for line in open(GOLD):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "c_row":
            c_rows.append(tuple(float(x) for x in t[1:]))
        elif t[0] == "proj_2x":
            proj.append((int(t[1]), float(t[2])))
        else:
            kv[t[0]] = float(t[1])
    return kv, c_rows, proj


def test_oracle_reproduces_the_papers_worked_example():
    g, _, _ = _gold()
    gamma, T_p = int(g["gamma"]), g["gamma_Tp_ms"] / g["gamma"]
    per_round = 2 * g["Tc_ms"] + g["gamma_Tp_ms"] + g["Tq_ms"]
    assert per_round == g["round_ms"]
    n = 200
    sd = lo.latency_sd(n, g["tau"], gamma, T_p, g["Tq_ms"], g["Tc_ms"]) / n
    assert round(sd, 2) == g["sd_ms_per_token"]
    # the printed AR and FSD figures are the SD figure scaled by the printed speed-ups
    assert abs(g["ar_ms_per_token"] / g["sd_ms_per_token"] - g["speedup_ar_sd"]) < 0.005
    assert abs(g["sd_ms_per_token"] / g["fsd_ms_per_token"] - g["speedup_sd_fsd"]) < 0.005
    # the FSD formula reaches the printed figure for a synchronisation latency between 0 and the
    # drafting time it replaces (the paper does not print T_r)
    r = g["cache_miss_rate"]
    f0 = lo.latency_fsd(n, g["tau"], gamma, T_p, g["Tq_ms"], g["Tc_ms"], r, 0.0) / n
    f1 = lo.latency_fsd(n, g["tau"], gamma, T_p, g["Tq_ms"], g["Tc_ms"], r, g["gamma_Tp_ms"]) / n
    assert f0 < g["fsd_ms_per_token"] < f1
    assert abs(f1 - sd) < 1e-9                     # T_r = gamma T_p: no gain left


def test_oracle_latency_ratio_matches_the_system_metrics_table():
    _, c_rows, _ = _gold()
    assert len(c_rows) == 6
    for gTp, Tq, c_printed in c_rows:
        assert round(gTp / 4 / Tq, 2) == c_printed


def test_oracle_projection_matches_the_papers_statements():
    g, _, proj = _gold()
    c = g["proj_c"]
    for gamma, r_max in proj:
        # at the printed miss rate the projected speed-up is 2x to within the paper's rounding ("about")
        assert abs(lo.projected_speedup(gamma, c, r_max) - 2.0) < 0.08
        assert lo.projected_speedup(gamma, c, r_max - 0.05) > 2.0 > lo.projected_speedup(gamma, c, r_max + 0.05)
    # Eq. 9 is the ratio of the two table rows when communication and synchronisation are free
    for gamma, cc, r in ((4, 0.14, 0.4), (7, 0.3, 0.25), (10, 0.65, 0.1)):
        sd = lo.latency_sd(200, 3.0, gamma, cc * 500.0, 500.0, 0.0)
        fsd = lo.latency_fsd(200, 3.0, gamma, cc * 500.0, 500.0, 0.0, r, 0.0)
        assert abs(sd / fsd - lo.projected_speedup(gamma, cc, r)) < 1e-12
    assert lo.projected_speedup(4, 0.3, 1.0) == 1.0            # every round misses: nothing gained
    assert lo.projected_speedup(4, 0.3, 0.0) == 4 * 0.3 + 1.0  # every round hits: drafting is hidden


def test_oracle_special_cases():
    assert lo.latency_ar(1, 17.0, 0.0) == 17.0
    assert lo.latency_ar(10, 5.0, 3.0) == 56.0
    # one token per round and a free draft model: SD = AR plus one network round trip per token
    assert lo.latency_sd(10, 1.0, 4, 0.0, 5.0, 3.0) == 10 * (6.0 + 5.0)
    # r = 1 turns FSD into SD whatever T_r is
    assert lo.latency_fsd(50, 2.5, 4, 7.0, 90.0, 11.0, 1.0, 123.0) == lo.latency_sd(50, 2.5, 4, 7.0, 90.0, 11.0)


def test_oracle_sender_order():
    conf = [[0.9, 0.1, 0.99], [0.5, 0.95, 0.2], [0.7, 0.7, 0.7], [0.95, 0.3, 0.1]]
    acc = [1, 1, 2, 0]                      # scores: 0.9, 0.95, 0.7, 0.95
    order, scores = lo.sender_order(conf, acc)
    assert order == [1, 3, 0, 2] and scores == [0.95, 0.95, 0.9, 0.7]
    assert lo.exit_score([0.2, 0.8, 0.9], 0) == 0.2   # rows past the exit's own accept length do not count


@pytest.mark.parametrize("seed", range(5))
def test_library_latency_model_matches_the_oracle(seed):
    rng = np.random.default_rng(seed)
    T_p, T_q, T_c, T_r = rng.uniform(1, 400), rng.uniform(1, 700), rng.uniform(0, 120), rng.uniform(0, 200)
    tau, r, gamma, n = rng.uniform(1, 9), rng.uniform(0, 1), int(rng.integers(1, 11)), int(rng.integers(1, 500))
    got = ee.ee_latency_model(T_p, T_q, T_c, tau, gamma, n, r, T_r)
    exp = {"ar_ms": lo.latency_ar(n, T_q, T_c), "sd_ms": lo.latency_sd(n, tau, gamma, T_p, T_q, T_c),
           "fsd_ms": lo.latency_fsd(n, tau, gamma, T_p, T_q, T_c, r, T_r)}
    for k, v in exp.items():
        assert math.isclose(got[k], v, rel_tol=1e-12), k
        assert math.isclose(got[k + "_per_token"], v / n, rel_tol=1e-12)
    assert math.isclose(got["speedup_ar_to_sd"], exp["ar_ms"] / exp["sd_ms"], rel_tol=1e-12)
    assert math.isclose(got["speedup_sd_to_fsd"], exp["sd_ms"] / exp["fsd_ms"], rel_tol=1e-12)
    assert math.isclose(got["c"], T_p / T_q, rel_tol=1e-12)
    assert math.isclose(got["projected_sd_to_fsd"], lo.projected_speedup(gamma, T_p / T_q, r), rel_tol=1e-12)


def test_library_latency_model_worked_example_and_errors():
    g, _, _ = _gold()
    got = ee.ee_latency_model(g["gamma_Tp_ms"] / 4, g["Tq_ms"], g["Tc_ms"], g["tau"], 4, 200)
    assert round(got["sd_ms_per_token"], 2) == g["sd_ms_per_token"]
    for bad in (dict(tau=0.0), dict(T_q=0.0), dict(n=0), dict(gamma=0), dict(r=1.5), dict(T_c=-1.0)):
        kw = dict(T_p=10.0, T_q=100.0, T_c=5.0, tau=2.0, gamma=4, n=10, r=0.5, T_r=1.0)
        kw.update(bad)
        with pytest.raises(ee.EEError) as e:
            ee.ee_latency_model(**kw)
        assert e.value.code == ee.EE_EINVAL
