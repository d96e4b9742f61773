"""The queueing calculator against the numbers the paper prints and its own algebra."""
import math
import os

import pytest

from paper_2605_08581_amd import queueing as Q


@pytest.fixture(scope="module")
def g():
    vals = {}
    path = os.path.join(os.path.dirname(__file__), "golden", "queueing_numbers.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        k, v, tol = line.split()
        vals[k] = (float(v), float(tol))
    return vals


def test_calibrated_prefill_throughput_matches_the_printed_value(g):
    R = Q.calibrate_prefill_throughput(g["calib_mu"][0], g["calib_M"][0], g["calib_L"][0], g["calib_h"][0])
    assert abs(R - g["calib_R_pf"][0]) <= g["calib_R_pf"][1]
    assert abs(Q.service_rate(g["calib_M"][0], g["calib_L"][0], g["calib_h"][0], R) - g["calib_mu"][0]) < 1e-9
    waves = g["calib_mu"][0] / g["calib_M"][0]
    assert abs(waves - g["calib_waves_per_s"][0]) <= g["calib_waves_per_s"][1]
    assert abs(1.0 / Q.wave_service_time(g["calib_L"][0], g["calib_h"][0], R) - waves) < 1e-9


@pytest.mark.parametrize("tag", ["x4", "x13"])
def test_crossover_matches_the_printed_intervals(g, tag):
    mu, M = g[tag + "_mu"][0], g[tag + "_M"][0]
    for key, c2 in (("_lambda_c2_1", 1.0), ("_lambda_lo", g["c2_hi"][0]), ("_lambda_hi", g["c2_lo"][0])):
        want, tol = g[tag + key]
        assert abs(Q.crossover_rate(mu, M, c2) - want) <= tol, (tag, key)


def test_crossover_is_where_queueing_wait_equals_wave_duration():
    mu, M, c2 = 37.0, 12.0, 2.5
    lam = Q.crossover_rate(mu, M, c2)
    assert math.isclose(Q.admission_wait(lam, mu, c2), M / mu, rel_tol=1e-12)
    assert math.isclose(Q.crossover_rate(mu, 1.0, 1.0), mu / 2)          # unbatched M/M/1 knee
    assert Q.crossover_rate(mu, 1e9, c2) == pytest.approx(mu, rel=1e-6)   # large waves: the ceiling
    assert Q.admission_wait(mu, mu, c2) == float("inf")
    assert math.isclose(Q.admission_wait(0.0, mu, c2, dt_win=0.2), 0.1)


def test_theorem_one_algebra():
    M, R, L, h_lru, dh = 20.0, 700.0, 900.0, 0.2, 0.15
    mu_lru = Q.service_rate(M, L, h_lru, R)
    mu_prism = Q.service_rate(M, L, h_lru + dh, R)
    assert math.isclose(mu_prism - mu_lru, Q.service_gap(mu_lru, h_lru + dh, h_lru), rel_tol=1e-12)
    assert math.isclose(mu_prism - mu_lru, Q.stability_expansion(M, R, L, h_lru, dh), rel_tol=1e-12)
    assert Q.service_gap(mu_lru, h_lru, h_lru) == 0.0
    assert math.isclose(Q.service_ratio(M, R, L, h_lru + dh, M, R, L, h_lru), mu_prism / mu_lru, rel_tol=1e-12)
    assert math.isclose(Q.service_ratio(2 * M, R, L, h_lru, M, 2 * R, 2 * L, h_lru), 2.0)   # 2 * (1/2) * 2
    assert math.isclose(Q.full_prompt_gap(0.2, 660.0, 768.0), 0.2 * 660 / 768)
    assert math.isclose(Q.effective_prefill_throughput(600.0, 10.0, 32.0, 6400.0), 600.0 * 0.95)


def test_attention_only_knee_on_fixed_inputs():
    """Worked by hand: a 0.5 ms layer call, 40 layers -> 20 ms per wave; 10
    requests per wave -> mu = 500 requests/s; L (1 - h) = 600 uncached tokens per
    request -> R = 30 000 tokens/s per request; Eq. 15 with c2 = 1: 500 * 20 / 22."""
    k = Q.attention_only_knee(0.5e-3, 40, M=10.0, L=800.0, h=0.25, c2=1.0)
    assert k["wave_s"] == pytest.approx(0.02, rel=1e-12)
    assert k["mu_requests_per_s"] == pytest.approx(500.0, rel=1e-12)
    assert k["R_attn_tokens_per_s_per_request"] == pytest.approx(30000.0, rel=1e-12)
    assert k["lambda_star_requests_per_s"] == pytest.approx(454.5454545454545, rel=1e-12)
    assert k["scope"].startswith("attention-only")
    # the printed line of the replay's --knee leg carries exactly these numbers
    from paper_2605_08581_amd import replay
    line = replay.knee_line({"gpu_ms_per_wave": 0.5, "mean_wave_size": 10.0, "hit_rate": 0.25,
                             "prompt_tokens": 8000, "requests": 10}, n_layers=40)
    assert "attention-only" in line and "mu=500.0" in line and "lambda*=454.5" in line and "R_attn=30000" in line
