"""Pins of the oracle's calibrated Thompson-sampling controller (Section 3.3 "TS with
Calibration", Eq. 5-8, Algorithm 3, Appendix B) against things other than itself.  CPU only."""
import math

import numpy as np
import pytest
import scipy.special
import scipy.stats
import torch

import synth_inputs as si
from oracle import eesd_oracle as orc


@pytest.mark.parametrize("sm,ss,n,theta_m,theta_hat", [(0.2, 0.5, 0, 0.7, 0.3), (0.2, 0.5, 1, 0.7, 0.3), (0.4, 0.3, 7, 0.55, 0.81),
                                                       (0.05, 1.0, 40, 0.9, 0.2)])
def test_posterior_is_the_normal_normal_bayes_update(sm, ss, n, theta_m, theta_hat):
    """Numerical Bayes on a grid: prior N(theta_M, sigma_M^2) on mu, n observations with variance
    sigma_S^2 and sample mean theta_hat (only the mean matters for a normal likelihood)."""
    c = orc.CaliTS(sm, ss, theta_hat)
    c.n = n
    mu, var = c.posterior(theta_m)
    grid = np.linspace(-6.0, 7.0, 400001)
    rng = np.random.default_rng(3)
    obs = rng.normal(0.0, 1.0, n)
    obs = obs - obs.mean() + theta_hat if n else obs           # any sample with that mean
    logp = -0.5 * ((grid - theta_m) / sm) ** 2
    for x in obs:
        logp += -0.5 * ((x - grid) / ss) ** 2
    w = np.exp(logp - logp.max())
    w /= w.sum()
    m_num = float((w * grid).sum())
    v_num = float((w * (grid - m_num) ** 2).sum())
    assert abs(mu - m_num) < 1e-6
    assert abs(var - v_num) < 1e-6 * max(1.0, v_num) + 1e-9
    # Eq. 7 in its printed (precision) form
    assert abs(1.0 / var - (1.0 / sm ** 2 + n / ss ** 2)) < 1e-9 / var


def test_posterior_limits_stated_by_the_paper():
    c = orc.CaliTS(0.3, 0.6, 0.25)
    assert c.posterior(0.8) == (0.8, 0.3 ** 2)                 # no verification yet: the model's score
    c.n = 10 ** 9
    mu, var = c.posterior(0.8)
    assert abs(mu - 0.25) < 1e-8 and var < 1e-9                # many verifications: the observed mean


def test_normal_draws_follow_the_normal_law():
    z = np.array([orc.normal_draw(5, r, s) for r in range(1, 401) for s in range(1, 11)])
    assert scipy.stats.kstest(z, "norm").pvalue > 0.01
    assert abs(z.mean()) < 0.06 and abs(z.std() - 1.0) < 0.05
    # the same counters give the same variate; different slots differ
    assert orc.normal_draw(5, 1, 1) == orc.normal_draw(5, 1, 1) != orc.normal_draw(5, 1, 2)


def test_decide_is_bernoulli_of_the_clipped_draw():
    c = orc.CaliTS(1e-9, 1.0, 0.5, seed=9)      # sigma_M ~ 0: theta is the model's score
    for p in (0.0, 0.2, 0.9, 1.0, 1.7, -0.4):
        chis = [c.decide(p, r, 1)[1] for r in range(1, 4001)]
        want = min(1.0, max(0.0, p))
        assert abs(np.mean(chis) - want) < 0.03


def test_predictor_is_class_one_of_a_two_class_softmax():
    shape = si.TINY
    cw = si.cali_to_numpy(si.make_cali_weights(shape, 3))
    d = shape["d_model"]
    rng = np.random.default_rng(0)
    seen = []
    for i in (1, 2, 10, 11, 25):
        h_t, h_d = rng.normal(0, 0.3, d), rng.normal(0, 0.3, d)
        got = orc.cali_theta_m(cw, h_t, h_d, i)
        Wi = torch.from_numpy(cw["w"][min(i, 10) - 1]).double()
        lin = torch.nn.functional.linear(torch.from_numpy(np.concatenate([(Wi @ torch.from_numpy(h_t)).numpy(), h_d])),
                                         torch.from_numpy(cw["wp"]).double())
        want = float(scipy.special.softmax(lin.numpy())[1])
        assert abs(got - want) < 1e-12
        seen.append(got)
    assert max(seen) - min(seen) > 0.05          # the synthetic predictor is not stuck at 1/2
    assert orc.cali_theta_m(cw, h_t, h_d, 10) == orc.cali_theta_m(cw, h_t, h_d, 37)   # i = min(i, 10)


def test_running_mean_is_the_mean_of_what_the_target_judged():
    c = orc.CaliTS(0.2, 0.5, 0.6)
    obs = [0.6]                                   # theta_hat_0 counts as one observation
    for a, K in [(0, 3), (2, 2), (1, 4), (0, 1), (5, 5), (3, 7)]:
        c.update(a, K)
        obs += [1.0] * a + ([0.0] if a < K else [])
        assert abs(c.theta_hat - np.mean(obs)) < 1e-12
    assert c.n == 6
    # the printed form: |Q_v| successes for |Q_v| observations
    p = orc.CaliTS(0.2, 0.5, 0.6, update="printed")
    t, th = 0, 0.6
    for a, K in [(0, 3), (2, 2), (1, 4)]:
        p.update(a, K)
        t += a
        th = (th * (t - a + 1) + a) / (t + 1)
        assert abs(p.theta_hat - th) < 1e-12


def test_cali_generation_is_lossless_and_uses_the_predictor():
    w = si.weights_to_numpy(si.make_weights(si.TINY, seed=0, correlated_draft=0.05))
    cw = si.cali_to_numpy(si.make_cali_weights(si.TINY, 1))
    prompt = si.make_prompt(20, 512, 0)
    ar = orc.OracleEESD(w, 128, 0.0).ar_generate(prompt, 48)
    o = orc.OracleEESD(w, 128, 0.0, seed=4, k_cap=6)
    trace = []
    cali = orc.CaliTS(0.2, 0.5, 0.5, seed=4)
    assert o.generate_cali(prompt, 48, cw, cali, trace=trace) == ar
    ks = [r["K"] for r in trace]
    assert len(set(ks)) > 1                        # the controller really varied K
    for r in trace:     # drafting stopped on chi = 0 after K scores, or at the cap after K - 1 scores that all said "go on"
        chis = [c for _, _, c in r["scores"]]
        assert (len(chis) == r["K"] and not chis[-1] and all(chis[:-1])) or (len(chis) == r["K"] - 1 and all(chis))
    assert cali.n == len(trace)
    # the hidden state handed to the predictor is the target's at the last verified position:
    # the last position of the committed text, whose output is the round's pending token
    ref = orc.OracleEESD(w, 128, 0.0)
    ref.target_forward(list(prompt) + ar, 0)
    for r in trace:
        assert np.max(np.abs(r["h_t"] - ref.h_target_rows[r["base"] - 1])) < 1e-10
    assert any(r["a"] > 0 for r in trace)
