"""The calibrated controller (Section 3.3 "TS with Calibration", Eq. 5-8, Algorithm 3) on the GPU
against the oracle: the predictor's score per draft step under teacher forcing, the observations
it accumulates, and whole generations."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import eesd_oracle as orc
from gpu_common import make_pair, require_gpu, tol_of, top2_gap

pytestmark = pytest.mark.gpu

SHAPES = {"tiny_fp32": si.TINY, "gqa_bf16": si.TINY_GQA_BF16}


def _cali_pair(shape, seed, device="cuda"):
    cw = si.make_cali_weights(shape, seed)
    return si.cali_to_numpy(cw), {k: v.to(device).contiguous() for k, v in cw.items()}


@pytest.mark.parametrize("name,tiled", [("tiny_fp32", 0), ("gqa_bf16", 0), ("gqa_bf16", 1)])
@pytest.mark.parametrize("temp", [0.0, 1.0])
def test_predictor_scores_match_oracle_under_teacher_forcing(name, temp, tiled):
    require_gpu()
    import paper_2406_03853_amd as pk
    shape = SHAPES[name]
    tol = tol_of(shape)
    o, g = make_pair(shape, 3, 160, temp, k_cap=12, gamma=0.05, weight_layout=tiled)
    cw_np, cw_gpu = _cali_pair(shape, 1)
    if tiled:
        cw_gpu = pk.pack_calibration(cw_gpu)
    g.set_calibration(cw_gpu, 0.2, 0.5, 0.5)
    cali = orc.CaliTS(0.2, 0.5, 0.5)
    prompt = si.make_prompt(21, shape["vocab"], 1)
    t_ref = o.prefill(prompt)
    g.prefill(prompt)
    g.force_pending(t_ref)
    h_t = o.h_target_rows[-1]
    seen = []
    for K in (3, 12, 1, 5):          # 12 > the ten matrices: the last one is reused
        for k in range(1, K + 1):
            d = o.draft_step()
            g.force_drafts([d])
            g.draft_step(sync=False)
            want = orc.cali_theta_m(cw_np, h_t, o.h_draft, k)
            got = g.cali_score()
            assert abs(got - want) < tol, (K, k, got, want)
            seen.append(want)
        o.verify()
        g.verify()
        a, y = o.accept()
        g.accept()
        h_t = o.h_target_rows[a]
        cali.update(a, K)
        o.rollback(a, y)
        g.rollback_forced(a, y)
        th, w, n = g.cali_state()
        assert (th, w, n) == (cali.theta_hat, cali.weight, cali.n)
    assert max(seen) - min(seen) > 0.05


def _cali_generation_case(name, seed, first):
    """One generation under the calibrated controller on both sides; returns whether every decision of the run sat
    outside the score tolerance (then the K sequence and the posterior must be the oracle's, and that was asserted)."""
    import paper_2406_03853_amd as pk
    shape = SHAPES[name]
    tol = tol_of(shape)
    o, g = make_pair(shape, 7, 192, 0.0, k_cap=6, gamma=0.05, ts_mode=pk.TS_CALI, seed=seed)
    cw_np, cw_gpu = _cali_pair(shape, 2)
    prompt = si.make_prompt(24, shape["vocab"], 0)
    if first:
        with pytest.raises(pk.EesdError):
            g.generate(prompt, 8)                      # no predictor installed
    g.set_calibration(cw_gpu, 0.2, 0.5, 0.5)
    cali = orc.CaliTS(0.2, 0.5, 0.5, seed=seed)
    n_new = 40
    trace = []
    want = o.generate_cali(prompt, n_new, cw_np, cali, trace=trace)
    got, st = g.generate(prompt, n_new)
    # greedy: the text is the auto-regressive one whatever the controller does, up to near-ties
    ref = orc.OracleEESD(o.w, 192, 0.0)
    logits = ref.target_forward(list(prompt) + want[:-1], 0)[len(prompt) - 1:]
    safe_len = next((i for i in range(n_new) if top2_gap(logits[i]) <= 2 * tol), n_new)
    assert got[:safe_len] == want[:safe_len]
    # the K sequence is the oracle's as long as no decision sat inside the score tolerance
    margins = [abs(theta - orc.uniform(seed, orc.STREAM_TS_CHI, r + 1, k + 1)) for r, rec in enumerate(trace)
               for k, (_, theta, _) in enumerate(rec["scores"])]
    safe = safe_len == n_new and min(margins) > 0.3 * tol + 1e-3
    if safe:
        assert (st.rounds, st.drafted, st.accepted) == (o.stats.rounds, o.stats.drafted, o.stats.accepted)
        assert g.cali_state() == (cali.theta_hat, cali.weight, cali.n)
    assert len({rec["K"] for rec in trace}) > 1
    return safe


@pytest.mark.parametrize("name", list(SHAPES))
def test_cali_generation_matches_oracle(name):
    """Whole generations under the calibrated controller.  Rounds, drafts, acceptances and the posterior can only be
    compared for a run none of whose decisions sits inside the tolerance of the scores and none of whose greedy tokens
    is a near-tie; whether that holds is decided from the ORACLE's margins.  For the fp32 model such a run exists and
    the comparison is unconditional.  For the bf16 model it cannot be: with random weights every greedy stream meets
    a top-2 gap below twice the bf16 tolerance within a few tokens (a CPU search over 5 weight seeds x 3 prompts found
    no stream that gets past 6), so there the text is compared up to the first near-tie and the controller's
    decisions are covered unconditionally by the teacher-forced test above (scores within tolerance and an identical
    posterior after every round, both weight layouts)."""
    require_gpu()
    safe = _cali_generation_case(name, 4, True)
    if name == "tiny_fp32":
        assert safe


def test_cali_with_tree_and_argument_checks():
    require_gpu()
    import paper_2406_03853_amd as pk
    shape = si.TINY
    o, g = make_pair(shape, 9, 128, 0.0, k_cap=5, gamma=0.05, ts_mode=pk.TS_CALI, tree_width=3)
    cw_np, cw_gpu = _cali_pair(shape, 3)
    with pytest.raises(pk.EesdError):
        g.cali_score()
    with pytest.raises(pk.EesdError):
        g.set_calibration(cw_gpu, 0.0, 0.5, 0.5)
    g.set_calibration(cw_gpu, 0.3, 0.4, 0.6, update=1)
    prompt = si.make_prompt(16, shape["vocab"], 2)
    got, st = g.generate(prompt, 32)
    ar = orc.OracleEESD(o.w, 128, 0.0).ar_generate(prompt, 32)
    ref = orc.OracleEESD(o.w, 128, 0.0)
    logits = ref.target_forward(list(prompt) + ar[:-1], 0)[len(prompt) - 1:]
    safe_len = next((i for i in range(32) if top2_gap(logits[i]) <= 2e-4), 32)
    assert got[:safe_len] == ar[:safe_len]
    assert g.cali_state()[2] == st.rounds
