"""Candidate-tree verification (Section 4.3, tree-attention table) against the oracle, which
evaluates every root path on its own: node logits under the tree mask, the accepted path, the
caches after the accepted nodes moved into place, and whole generations."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import eesd_oracle as orc
from gpu_common import make_pair, rel_err, require_gpu, tol_of, top2_gap

pytestmark = pytest.mark.gpu

SHAPES = {"tiny_fp32": si.TINY, "gqa_bf16": si.TINY_GQA_BF16}


def _check_caches(o, g, n, tol):
    for cache in range(o.L + 1):
        ref = o.kv[cache] if cache < o.L else o.ee_kv
        k, v = g.kv(cache, n)
        assert rel_err(k, ref.k[:n]) < tol, ("K", cache)
        assert rel_err(v, ref.v[:n]) < tol, ("V", cache)


def _row(i, j, width):
    return 1 + (i - 1) * width + j


@pytest.mark.parametrize("width", [2, 4])
def test_tree_top_candidates_on_long_rows_with_ties(width):
    """A vocabulary of several entries per thread and logits stored as bf16, so that equal values are common: the
    candidates are the largest entries of the GPU's own row, equal values by lowest index."""
    require_gpu()
    shape = dict(si.TINY_GQA_BF16, vocab=9024, name="tiny_gqa_bf16_v9024")
    steps = min(4, 15 // width)                      # a verify block holds 1 + K width <= 16 rows
    o, g = make_pair(shape, 6, 96, 0.0, k_cap=steps, tree_width=width, logits_bf16=1)
    g.prefill(si.make_prompt(12, shape["vocab"], 3))
    ties = 0
    for i in range(steps):
        g.draft_step()
        lg = np.asarray(g.draft_logits(i), np.float64)
        want = sorted(range(len(lg)), key=lambda t: (-lg[t], t))[:width]
        assert g.tree_tokens(1 + (i + 1) * width)[1 + i * width:] == want == orc.top_candidates(lg, width)
        ties += len(set(lg[want])) < width or np.sum(lg == lg[want[-1]]) > 1
    assert ties > 0


@pytest.mark.parametrize("name", list(SHAPES))
@pytest.mark.parametrize("width", [2, 3])
def test_teacher_forced_tree_rounds_match_oracle(name, width):
    require_gpu()
    shape = SHAPES[name]
    tol = tol_of(shape)
    k_cap = (16 - 1) // width
    o, g = make_pair(shape, 3, 160, 0.0, k_cap=k_cap, gamma=0.05, tree_width=width, kv_page=16)
    prompt = si.make_prompt(29, shape["vocab"], 1)     # the block straddles a page boundary in some rounds
    t_ref = o.prefill(prompt)
    g.prefill(prompt)
    g.force_pending(t_ref)
    leaf = full = 0
    for K in [2, k_cap, 1, 3, k_cap, 2, 4][: 7 if width == 2 else 6]:
        K = min(K, k_cap)
        base = o.kv_len
        kids = [o.draft_step_tree() for _ in range(K)]
        g.force_drafts([t for k in kids for t in k])
        for i in range(K):
            g.draft_step(sync=(i == K - 1))
        for i in range(K):
            assert rel_err(g.draft_logits(i), o.q_logits[i]) < tol, ("draft logits", K, i)
        assert g.tree_tokens(1 + K * width)[1:] == [t for k in kids for t in k]
        a_ref, y_ref, branch = o.verify_accept_tree()
        g.verify()
        assert rel_err(g.verify_logits(0), o.tree_logits[()]) < tol
        for i in range(1, K + 1):
            for j in range(width):
                assert rel_err(g.verify_logits(_row(i, j, width)), o.tree_logits[(i, j)]) < tol, ("node logits", K, i, j)
        a_gpu, y_gpu = g.accept()
        visited = [o.tree_logits[()]] + [o.tree_logits[(i + 1, branch[i])] for i in range(a_ref)]
        if all(top2_gap(r) > 2 * tol for r in visited):
            assert (a_gpu, y_gpu) == (a_ref, y_ref), (K, a_gpu, y_gpu, a_ref, y_ref)
            assert g.accepted_tokens() == [kids[i][branch[i]] for i in range(a_ref)]
            leaf += a_ref > 0 and branch[-1] != 0
            full += a_ref == K
            o.rollback_tree(a_ref, y_ref, branch)
            g.rollback_forced(a_ref, y_ref)
            assert g.kv_len() == o.kv_len == base + a_ref + 1
            _check_caches(o, g, o.kv_len, tol)
        else:   # a near-tie: keep the two sides on the same text without using the GPU's decision
            o.rollback_tree(0, y_ref, [])
            g.rollback_forced(0, y_ref)
    assert leaf + full > 0
    s = g.stats()
    assert (s.rounds, s.drafted, s.accepted) == (o.stats.rounds, o.stats.drafted, o.stats.accepted)


@pytest.mark.parametrize("width", [2, 3, 4])
def test_tree_top_candidates_are_the_draft_models_most_likely_tokens(width):
    require_gpu()
    shape = si.TINY
    o, g = make_pair(shape, 5, 96, 0.0, k_cap=3, tree_width=width)
    prompt = si.make_prompt(12, shape["vocab"], 2)
    g.prefill(prompt)
    g.force_pending(o.prefill(prompt))
    for i in range(3):
        kids = o.draft_step_tree()
        g.force_drafts(kids)          # the GPU proposes for itself below; forcing keeps the chains equal
        g.draft_step()
        lg = g.draft_logits(i)
        assert g.tree_tokens(1 + (i + 1) * width)[1 + i * width:] == kids
        assert orc.top_candidates(lg, width) == sorted(range(len(lg)), key=lambda t: (-float(lg[t]), t))[:width]
    # unforced: the candidates are the top entries of the GPU's own logits row
    o2, g2 = make_pair(shape, 5, 96, 0.0, k_cap=3, tree_width=width)
    g2.prefill(prompt)
    for i in range(3):
        g2.draft_step()
        assert g2.tree_tokens(1 + (i + 1) * width)[1 + i * width:] == orc.top_candidates(g2.draft_logits(i), width)


@pytest.mark.parametrize("name", list(SHAPES))
@pytest.mark.parametrize("width", [2, 3])
def test_tree_generation_matches_oracle_and_autoregressive_text(name, width):
    require_gpu()
    import paper_2406_03853_amd as pk
    shape = SHAPES[name]
    tol = tol_of(shape)
    k_cap = 4
    o, g = make_pair(shape, 7, 192, 0.0, k_cap=k_cap, gamma=0.05, tree_width=width, ts_mode=pk.TS_FIXED)
    prompt = si.make_prompt(24, shape["vocab"], 0)
    n_new = 40
    trace = []
    want = o.generate_tree(prompt, n_new, fixed_k=k_cap, trace=trace)
    ar = orc.OracleEESD(o.w, 192, 0.0).ar_generate(prompt, n_new)
    assert want == ar
    got, st = g.generate(prompt, n_new)
    # equal up to the first decision the tolerance could flip;
    safe_len = n_new
    # near-ties are found from the auto-regressive logits of the committed text
    ref = orc.OracleEESD(o.w, 192, 0.0)
    logits = ref.target_forward(list(prompt) + want[:-1], 0)[len(prompt) - 1:]
    for i in range(n_new):
        if top2_gap(logits[i]) <= 2 * tol:
            safe_len = i
            break
    assert got[:safe_len] == want[:safe_len]
    if safe_len == n_new:
        assert st.rounds == o.stats.rounds and st.accepted == o.stats.accepted
        assert st.accepted > 0


def test_tree_mode_argument_checks():
    require_gpu()
    import paper_2406_03853_amd as pk
    w = si.weights_to_device(si.make_weights(si.TINY, seed=1), "cuda")
    with pytest.raises(pk.EesdError):
        pk.EESD(w, 64, 1.0, k_cap=3, tree_width=2)        # sampling: the tree keeps top-1 matches only
    with pytest.raises(pk.EesdError):
        pk.EESD(w, 64, 0.0, k_cap=8, tree_width=2)        # 1 + 8 * 2 rows > 16
    with pytest.raises(pk.EesdError):
        pk.EESD(w, 64, 0.0, k_cap=2, tree_width=5)
    g = pk.EESD(w, 64, 0.0, k_cap=3, tree_width=3)
    g.prefill(si.make_prompt(5, 512, 0))
    g.draft_step()
    g.verify()
    a, y = g.accept()
    assert g.accepted_tokens() == g.accepted_tokens() and len(g.accepted_tokens()) == a
    with pytest.raises(pk.EesdError):
        g.rollback(a + 1)
    g.rollback(a)
    with pytest.raises(pk.EesdError):
        g.accepted_tokens()
