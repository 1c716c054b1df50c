"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU or the HIP library.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import eesd_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [l.split() for l in f if l.strip() and not l.startswith("#")]


# ---------------------------------------------------------------------------
# counter hash and uniforms
# ---------------------------------------------------------------------------

def test_splitmix64_published_vector():
    want = [int(r[0]) for r in _rows("splitmix64_seed1234567.txt")]
    state, got = 1234567, []
    for _ in want:
        got.append(orc.splitmix64(state))
        state = (state + 0x9E3779B97F4A7C15) & ((1 << 64) - 1)
    assert got == want


def test_uniform_grid_and_moments():
    us = np.array([orc.uniform(7, orc.STREAM_DRAFT, r, s) for r in range(200) for s in range(50)])
    assert us.min() >= 0.0 and us.max() < 1.0
    assert np.all(us * 2.0 ** 53 == np.floor(us * 2.0 ** 53))
    assert abs(us.mean() - 0.5) < 0.01 and abs(us.var() - 1 / 12) < 0.005
    # distinct streams / rounds / slots give distinct numbers
    assert len({orc.uniform(7, s, r, k) for s in (1, 2, 3, 4, 5) for r in range(4) for k in range(4)}) == 80


# ---------------------------------------------------------------------------
# building blocks against library routines and invariants
# ---------------------------------------------------------------------------

def test_rmsnorm_matches_library_and_invariants():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 96))
    g = 1.0 + 0.3 * rng.standard_normal(96)
    got = orc.rmsnorm(x, g, 1e-6)
    want = torch.nn.functional.rms_norm(torch.from_numpy(x), (96,), torch.from_numpy(g), 1e-6).numpy()
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
    # unit gain: mean square of the output is 1 (up to eps); scale invariant
    y = orc.rmsnorm(x, np.ones(96), 0.0)
    assert np.allclose(np.mean(y * y, axis=-1), 1.0, atol=1e-12)
    assert np.allclose(orc.rmsnorm(3.7 * x, g, 0.0), orc.rmsnorm(x, g, 0.0), atol=1e-12)
    # eps sits inside the square root, added to the mean square
    one = orc.rmsnorm(np.array([[2.0, 0.0, 0.0, 0.0]]), np.ones(4), 3.0)
    assert np.allclose(one[0, 0], 2.0 / math.sqrt(1.0 + 3.0))


def test_softmax_silu_match_library():
    rng = np.random.default_rng(1)
    z = rng.standard_normal((3, 50)) * 4
    assert np.allclose(orc.softmax(z), torch.softmax(torch.from_numpy(z), -1).numpy(), atol=1e-15)
    assert np.allclose(orc.silu(z), torch.nn.functional.silu(torch.from_numpy(z)).numpy(), atol=1e-14)
    assert np.allclose(orc.softmax(z + 1000.0), orc.softmax(z), atol=1e-12)     # shift invariance, no overflow


def test_rope_complex_form_and_relative_position():
    rng = np.random.default_rng(2)
    hd, base = 16, 10000.0
    x = rng.standard_normal((4, 3, hd))
    pos = np.array([0, 1, 7, 300])
    y = orc.rope(x, pos, base)
    # pair (j, j+hd/2) is the complex number x_j + i x_{j+hd/2} multiplied by exp(i pos base^(-2j/hd))
    z = x[..., : hd // 2] + 1j * x[..., hd // 2:]
    w = np.exp(1j * pos[:, None, None] * base ** (-2.0 * np.arange(hd // 2) / hd)[None, None, :])
    zz = z * w
    assert np.allclose(y[..., : hd // 2], zz.real, atol=1e-12) and np.allclose(y[..., hd // 2:], zz.imag, atol=1e-12)
    assert np.allclose(y[0], x[0])                                            # position 0 is the identity
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1))  # a rotation
    # q_m . k_n depends on m - n only
    q, k = rng.standard_normal((1, 1, hd)), rng.standard_normal((1, 1, hd))
    def dot(m, n):
        return float(np.sum(orc.rope(q, np.array([m]), base) * orc.rope(k, np.array([n]), base)))
    assert abs(dot(5, 2) - dot(105, 102)) < 1e-10 and abs(dot(5, 2) - dot(6, 2)) > 1e-6


# ---------------------------------------------------------------------------
# the decoder against an independent library implementation of the LLaMA decoder
# ---------------------------------------------------------------------------

def _hf_model(shape, layers, norm, head, emb):
    from transformers import LlamaConfig, LlamaForCausalLM
    H, Hkv, hd, f = shape["n_heads"], shape["n_kv_heads"], shape["head_dim"], shape["d_ff"]
    cfg = LlamaConfig(hidden_size=shape["d_model"], intermediate_size=f, num_hidden_layers=len(layers),
                      num_attention_heads=H, num_key_value_heads=Hkv, head_dim=hd, vocab_size=shape["vocab"],
                      rms_norm_eps=shape["rms_eps"], rope_theta=shape["rope_base"], tie_word_embeddings=False,
                      attention_bias=False, mlp_bias=False, max_position_embeddings=1024,
                      attn_implementation="eager")
    m = LlamaForCausalLM(cfg).double().eval()
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    sd = {"model.embed_tokens.weight": t(emb), "model.norm.weight": t(norm), "lm_head.weight": t(head)}
    for l, w in enumerate(layers):
        p = f"model.layers.{l}."
        sd[p + "self_attn.q_proj.weight"] = t(w["wqkv"][: H * hd])
        sd[p + "self_attn.k_proj.weight"] = t(w["wqkv"][H * hd: (H + Hkv) * hd])
        sd[p + "self_attn.v_proj.weight"] = t(w["wqkv"][(H + Hkv) * hd:])
        sd[p + "self_attn.o_proj.weight"] = t(w["wo"])
        sd[p + "mlp.gate_proj.weight"] = t(w["w_gate_up"][:f])
        sd[p + "mlp.up_proj.weight"] = t(w["w_gate_up"][f:])
        sd[p + "mlp.down_proj.weight"] = t(w["w_down"])
        sd[p + "input_layernorm.weight"] = t(w["attn_norm"])
        sd[p + "post_attention_layernorm.weight"] = t(w["ffn_norm"])
    missing, unexpected = m.load_state_dict(sd, strict=False)
    assert not unexpected and all("rotary" in k or "inv_freq" in k for k in missing), (missing, unexpected)
    return m


@pytest.mark.parametrize("shape", [si.TINY, si.reduced_depth(si.TINY_GQA_BF16, 2, 1)], ids=["mha", "gqa"])
def test_target_and_draft_forward_match_library_llama(shape):
    shape = dict(shape, vocab=128)
    w = si.weights_to_numpy(si.make_weights(shape, seed=3, std=0.08, norm_gain_jitter=0.2))
    toks = si.make_prompt(11, shape["vocab"], 5)
    o = orc.OracleEESD(w, max_seq=32, temperature=0.0)
    got = o.target_forward(toks, 0)
    hf = _hf_model(shape, w["layers"], w["final_norm"], w["lm_head"], w["tok_emb"])
    with torch.no_grad():
        want = hf(torch.from_numpy(toks.astype(np.int64))[None]).logits[0].numpy()
    # the library builds its rotary cos/sin tables in fp32, hence 1e-5 and not 1e-12;
    # a structural mistake (pairing, sign, head mapping, eps placement) is an O(1) error
    assert np.max(np.abs(got - want)) < 1e-5 * max(1.0, np.max(np.abs(want)))
    # draft model (Eq. 1) = first N layers + the early-exit layer + its norm + its head
    N = shape["n_draft_layers"]
    hf_d = _hf_model(shape, w["layers"][:N] + [w["ee_layer"]], w["ee_norm"], w["ee_head"], w["tok_emb"])
    with torch.no_grad():
        want_d = hf_d(torch.from_numpy(toks.astype(np.int64))[None]).logits[0].numpy()
    o2 = orc.OracleEESD(w, max_seq=32, temperature=0.0)
    got_d = np.stack([o2.draft_forward(int(t), i) for i, t in enumerate(toks)])
    assert np.max(np.abs(got_d - want_d)) < 1e-5 * max(1.0, np.max(np.abs(want_d)))


# ---------------------------------------------------------------------------
# P3 / P4 / P5: block verify == sequential; rollback == never drafted; shared first-N cache
# ---------------------------------------------------------------------------

@pytest.fixture(scope="module")
def tiny_np():
    return si.weights_to_numpy(si.make_weights(si.TINY, seed=0, norm_gain_jitter=0.1))


def _caches(o, n):
    return [np.concatenate([c.k[:n].ravel(), c.v[:n].ravel()]) for c in o.kv + [o.ee_kv]]


def test_block_verify_equals_sequential_single_token_forwards(tiny_np):
    prompt = si.make_prompt(9, 512, 1)
    block = si.make_prompt(6, 512, 2)
    a = orc.OracleEESD(tiny_np, 64, 1.0)
    a.target_forward(prompt, 0)
    la = a.target_forward(block, len(prompt))
    b = orc.OracleEESD(tiny_np, 64, 1.0)
    b.target_forward(prompt, 0)
    lb = np.stack([b.target_forward([int(t)], len(prompt) + i)[0] for i, t in enumerate(block)])
    assert np.max(np.abs(la - lb)) < 1e-11
    for ca, cb in zip(_caches(a, 15), _caches(b, 15)):
        assert np.max(np.abs(ca - cb)) < 1e-12


def test_shared_first_n_cache_rows_equal_what_verify_writes(tiny_np):
    o = orc.OracleEESD(tiny_np, 64, 1.0, seed=4)
    o.prefill(si.make_prompt(8, 512, 3))
    for _ in range(3):
        o.draft_step()
    N = o.N
    before = [(o.kv[l].k[8:11].copy(), o.kv[l].v[8:11].copy()) for l in range(N)]
    ee_before = (o.ee_kv.k[8:11].copy(), o.ee_kv.v[8:11].copy())
    o.verify()
    for l in range(N):
        assert np.max(np.abs(before[l][0] - o.kv[l].k[8:11])) < 1e-12
        assert np.max(np.abs(before[l][1] - o.kv[l].v[8:11])) < 1e-12
    assert np.max(np.abs(ee_before[0] - o.ee_kv.k[8:11])) < 1e-12
    assert np.max(np.abs(ee_before[1] - o.ee_kv.v[8:11])) < 1e-12


@pytest.mark.parametrize("temp", [0.0, 1.0])
def test_rollback_equals_never_drafted(tiny_np, temp):
    prompt = si.make_prompt(10, 512, 6)
    o = orc.OracleEESD(tiny_np, 128, temp, seed=11, k_cap=5)
    committed = list(prompt) + [o.prefill(prompt)]
    accepted = 0
    for rnd in range(5):
        for _ in range(1 + rnd % 4):
            o.draft_step()
        o.verify()
        a, y = o.accept()
        committed += o.drafts[:a] + [y]
        accepted += a
        o.rollback(a, y)
    if temp > 0:
        assert accepted > 0            # rounds with a > 0 and with rejected drafts both occurred
    # a fresh model that is simply fed the committed tokens
    ref = orc.OracleEESD(tiny_np, 128, temp, seed=11)
    n = o.kv_len
    assert n == len(committed) - 1 and committed[n] == o.pending
    ref.target_forward(committed[:n], 0)
    for ca, cb in zip(_caches(o, n), _caches(ref, n)):
        assert np.max(np.abs(ca - cb)) < 1e-11


# ---------------------------------------------------------------------------
# P2: greedy speculative decoding == greedy auto-regressive decoding
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("gamma", [None, 0.05])
def test_greedy_eesd_equals_greedy_autoregressive(gamma):
    w = si.weights_to_numpy(si.make_weights(si.TINY, seed=0, correlated_draft=gamma))
    prompt = si.make_prompt(32, 512, 0)
    ar = orc.OracleEESD(w, 128, 0.0).ar_generate(prompt, 64)
    for kw in (dict(fixed_k=5), dict(fixed_k=1), dict(k_schedule=[1 + (i * 7) % 5 for i in range(64)]), dict()):
        o = orc.OracleEESD(w, 128, 0.0, seed=2, k_cap=5)
        out = o.generate(prompt, 64, **kw)
        assert out == ar
        if gamma is not None and kw.get("fixed_k") == 5:
            assert o.stats.accepted > 10          # the accept path was really taken
    assert len(ar) == 64


# ---------------------------------------------------------------------------
# P7: special cases of the accept rule
# ---------------------------------------------------------------------------

def test_accept_special_cases():
    p = si.make_prob_rows(4, 40, 3)
    drafts = [5, 17, 2]
    # q == p: every draft is accepted whatever the uniforms (u < 1), bonus token from the last row
    for s in range(20):
        u = si.make_uniforms(4, s)
        a, y = orc.decide_accept(p, p[:3].copy(), drafts, u[:3], u[3], greedy=False)
        assert a == 3 and y == orc.decide_sample(p[3], u[3])
    # p(d) == 0: never accepted; resampled token has p > q there
    q = si.make_prob_rows(3, 40, 8)
    p2 = p.copy(); p2[0, 5] = 0.0
    a, y = orc.decide_accept(p2, q, drafts, [0.0, 0.0, 0.0], 0.3, greedy=False)
    assert a == 0 and p2[0, y] > q[0, y]
    # u = 0 accepts anything with p > 0
    q3 = si.make_prob_rows(3, 40, 9)
    a, _ = orc.decide_accept(p, q3, drafts, [0.0, 0.0, 0.0], 0.5, greedy=False)
    assert a == 3
    # greedy: one-hot draft different from the target's top-1 => a = 0 and y = target top-1
    pl = si.make_logit_rows(3, 40, 1)
    top = int(np.argmax(pl[0]))
    a, y = orc.decide_accept(pl, None, [(top + 1) % 40, 0], None, None, greedy=True)
    assert (a, y) == (0, top)
    a, y = orc.decide_accept(pl, None, [top, int(np.argmax(pl[1]))], None, None, greedy=True)
    assert (a, y) == (2, int(np.argmax(pl[2])))
    # ties: lowest index
    assert orc.argmax_lowest(np.array([1.0, 3.0, 3.0, 2.0], np.float32)) == 1


def test_decide_sample_inverse_cdf():
    r = np.array([0.0, 0.25, 0.0, 0.5, 0.25, 0.0], np.float32)
    assert [orc.decide_sample(r, u) for u in (0.0, 0.2499, 0.25, 0.74, 0.75, 0.999999)] == [1, 1, 3, 3, 4, 4]
    assert orc.decide_sample(np.zeros(4, np.float32), 0.5) == -1
    assert orc.decide_sample(4.0 * r, 0.74) == 3            # weights need not be normalised
    # frequencies follow the weights
    us = si.make_uniforms(20000, 1)
    cnt = np.bincount([orc.decide_sample(r, u) for u in us], minlength=6) / 20000
    assert np.allclose(cnt, r, atol=0.012)


# ---------------------------------------------------------------------------
# P1: exact enumeration - the committed tokens follow the target's distribution
# ---------------------------------------------------------------------------

def _table(rows):
    rows = [np.array(r, np.float32) for r in rows]
    def f(prefix):
        h = 0
        for t in prefix:
            h = (h * 7 + t + 3) % 1009
        return rows[(h + len(prefix)) % len(rows)]
    return f


def _enumerate_output_distribution(p_of, q_of, k_of, V, L, grid):
    """Exact distribution of the first L committed tokens, by running the oracle's
    round on every cell of a uniform grid fine enough that each cell lies on one
    side of every threshold the round compares a uniform with."""
    mids = [(i + 0.5) / grid for i in range(grid)]
    memo = {}
    def dist(prefix):
        if len(prefix) >= L:
            return {prefix[:L]: Fraction(1)}
        if prefix in memo:
            return memo[prefix]
        K = k_of(prefix)
        counts = {}
        for us in itertools.product(mids, repeat=2 * K + 1):
            c = orc.abstract_round(prefix, K, q_of, p_of, us[:K], us[K:2 * K], us[2 * K])
            counts[c] = counts.get(c, 0) + 1
        out = {}
        for c, n in counts.items():
            for seq, pr in dist(prefix + c).items():
                out[seq] = out.get(seq, Fraction(0)) + Fraction(n, grid ** (2 * K + 1)) * pr
        memo[prefix] = out
        return out
    return dist(())


def _ar_distribution(p_of, V, L):
    out = {}
    for seq in itertools.product(range(V), repeat=L):
        pr = Fraction(1)
        for i, t in enumerate(seq):
            pr *= Fraction(float(p_of(seq[:i])[t]))
        if pr:
            out[seq] = pr
    return out


def test_exact_enumeration_quarter_grid_single_draft():
    # probabilities are multiples of 1/4, so p/q and the residual CDF have thresholds on the 1/12 grid
    P = [[.25, .25, .5], [.5, .25, .25], [0, .75, .25], [.25, .5, .25], [.5, 0, .5]]
    Q = [[.5, .25, .25], [.25, .75, 0], [.25, .25, .5], [0, .5, .5], [.75, .25, 0], [.25, .5, .25]]
    p_of, q_of = _table(P), _table(Q)
    got = _enumerate_output_distribution(p_of, q_of, lambda pre: 1, 3, 3, 12)
    want = _ar_distribution(p_of, 3, 3)
    assert got == want and sum(got.values()) == 1


@pytest.mark.parametrize("policy", ["k2", "k3", "mixed"])
def test_exact_enumeration_half_grid_multi_draft(policy):
    # probabilities are multiples of 1/2: every threshold is a multiple of 1/2, a grid of 4 is exact
    P = [[.5, .5, 0, 0], [0, .5, .5, 0], [.5, 0, 0, .5], [0, 0, .5, .5], [1, 0, 0, 0], [0, .5, 0, .5]]
    Q = [[.5, 0, .5, 0], [.5, .5, 0, 0], [0, 1, 0, 0], [0, .5, .5, 0], [.5, 0, 0, .5], [0, 0, .5, .5], [0, .5, 0, .5]]
    p_of, q_of = _table(P), _table(Q)
    k_of = {"k2": lambda pre: 2, "k3": lambda pre: 3 if len(pre) == 0 else 1,
            "mixed": lambda pre: 1 + (sum(pre) + len(pre)) % 2}[policy]
    got = _enumerate_output_distribution(p_of, q_of, k_of, 4, 4, 4)
    want = _ar_distribution(p_of, 4, 4)
    assert got == want and sum(got.values()) == 1


# ---------------------------------------------------------------------------
# P6: Beta posterior controller
# ---------------------------------------------------------------------------

def test_beta_update_hand_computed():
    for mode, K, a, want in [("prose", 4, 2, (3, 2)), ("literal", 4, 2, (3, 3)), ("prose", 4, 4, (5, 1)),
                             ("literal", 4, 4, (5, 1)), ("prose", 4, 0, (1, 2)), ("literal", 4, 3, (4, 2)),
                             ("literal", 1, 0, (1, 2))]:
        ts = orc.BetaTS(1, 1, 0, mode)
        ts.update(a, K)
        assert (ts.alpha, ts.beta) == want, (mode, K, a)


def test_beta_order_statistic_is_beta_distributed():
    from scipy import stats
    for a, b in [(1, 1), (3, 2), (2, 7), (10, 4)]:
        xs = [orc.beta_draw_int(a, b, 99, r, 1) for r in range(3000)]
        assert stats.kstest(xs, stats.beta(a, b).cdf).pvalue > 1e-3
        assert abs(np.mean(xs) - a / (a + b)) < 0.02


def test_k_is_truncated_geometric_with_continue_probability_alpha_over_alpha_plus_beta():
    from scipy import stats
    a, b, cap, n = 3, 2, 6, 20000
    ts = orc.BetaTS(a, b, seed=5)
    ks = np.array([ts.draw_k(r, cap) for r in range(n)])
    c = a / (a + b)                       # marginal P(chi = 1) under the posterior (conjugacy)
    want = np.array([c ** (k - 1) * (1 - c) for k in range(1, cap)] + [c ** (cap - 1)])
    got = np.bincount(ks, minlength=cap + 1)[1:]
    assert stats.chisquare(got, want * n).pvalue > 1e-3
    assert ts.draw_k(0, 1) == 1 and all(1 <= k <= cap for k in ks)


# ---------------------------------------------------------------------------
# P8: statistics of Section 4.1 / Appendix D against the printed rows
# ---------------------------------------------------------------------------

def test_harmonic_mean_reproduces_printed_rows_within_rounding():
    for v, r, hm in [(float(a), float(b), float(c)) for a, b, c in _rows("paper_hm_rows.txt")]:
        lo = orc.harmonic_mean_pct(v - 0.005, r - 0.005)
        hi = orc.harmonic_mean_pct(v + 0.005, r + 0.005)
        assert lo - 0.01 <= hm <= hi + 0.01, (v, r, hm, lo, hi)


def test_speedup_closed_form_is_the_time_model():
    for v, r, td, tt in [(0.52, 0.68, 7.5, 122.0), (0.3, 0.2, 0.74, 4.6), (0.9, 0.7, 30.0, 100.0)]:
        L = 512
        T = orc.predicted_time(L, v, r, td, tt)
        assert abs(L * tt / T - orc.predicted_speedup(v, r, td / tt)) < 1e-12
    # draft tokens for free and all accepted: every round of K drafts yields K+1 tokens
    assert abs(orc.predicted_speedup(1.0, 0.75, 0.0) - 4.0) < 1e-12


def test_stats_counters(tiny_np):
    o = orc.OracleEESD(tiny_np, 128, 1.0, seed=1, k_cap=5)
    out = o.generate(si.make_prompt(8, 512, 0), 30, fixed_k=3)
    s = o.stats
    assert len(out) == 30 and s.generated == 30 and s.drafted <= 3 * s.rounds
    assert 0 <= s.accepted <= s.drafted and abs(s.v_d - s.accepted / s.drafted) < 1e-15


def test_stats_hand_computed_rounds(tiny_np):
    """Appendix D on a hand-made run: three rounds with K = 3, 2, 4 drafts and a = 1, 2, 0 accepted, the
    first token from prefill: N_all_draft = 9, N_right = 3, L = 1 + (2 + 3 + 1) = 7, so v_d = 3/9,
    r_d = 3/7 and HM = 2 (1/3)(3/7) / (1/3 + 3/7) = 3/8."""
    o = orc.OracleEESD(tiny_np, 64, 1.0)
    n_out = 1
    for K, a in ((3, 1), (2, 2), (4, 0)):
        o.drafts = [0] * K
        o.rollback(a, 0)
        n_out += a + 1
    o.stats.generated = n_out
    s = o.stats
    assert (s.rounds, s.drafted, s.accepted, s.generated) == (3, 9, 3, 7)
    assert abs(s.v_d - 3 / 9) < 1e-15 and abs(s.r_d - 3 / 7) < 1e-15
    assert abs(orc.harmonic_mean_pct(s.v_d, s.r_d) - 37.5) < 1e-12
    # r_d is not v_d: a dropped "generated" (or the draft count in its place) fails here
    assert abs(s.r_d - s.v_d) > 0.09


def test_shapes_reproduce_printed_trainable_parameter_counts():
    """Section 3.1: the early-exit layer and its head are initialised from the target's last layer and LM
    head, so they have a decoder layer's and a full head's shape; their sizes must give the trainable
    parameters the main results table prints, and ten d x d matrices plus the 2 x 2d projection of
    Eq. 5 the predictor's."""
    shapes = {s["name"]: s for s in (si.LLAMA70B, si.LLAMA13B)}
    unit = {"B": 1e9, "M": 1e6}
    rows = _rows("paper_param_counts.txt")
    assert len(rows) == 2
    for name, trainable, tu, predictor, pu in rows:
        sh = shapes[name]
        d = sh["d_model"]
        n_train = si.layer_param_count(sh) + sh["vocab"] * d + d          # layer (with its two norms) + final norm + head
        n_pred = 10 * d * d + 2 * 2 * d
        digits = len(trainable.split(".")[1]) if "." in trainable else 0
        assert round(n_train / unit[tu], digits) == float(trainable), (name, n_train)
        digits = len(predictor.split(".")[1]) if "." in predictor else 0
        assert round(n_pred / unit[pu], digits) == float(predictor), (name, n_pred)
        cw = si.make_cali_weights(si.reduced_depth(dict(sh, d_model=64), 2, 1), 0)
        assert tuple(cw["w"].shape) == (10, 64, 64) and tuple(cw["wp"].shape) == (2, 128)
    # the weight container really has those shapes (checked on a narrow model of the same family)
    small = dict(si.LLAMA70B, d_model=256, n_heads=8, n_kv_heads=2, head_dim=32, d_ff=512, vocab=640, n_layers=2, n_draft_layers=1, dtype="f32")
    w = si.make_weights(small, seed=0)
    n = sum(int(w["ee_layer"][k].numel()) for k in si.LAYER_KEYS) + int(w["ee_head"].numel()) + int(w["ee_norm"].numel())
    assert n == si.layer_param_count(small) + small["vocab"] * small["d_model"] + small["d_model"]
