"""Pins of the oracle's candidate-tree decoding (Section 4.3, tree-attention table) against things
other than itself: brute force over all root paths, the auto-regressive continuation, and
from-scratch forwards of every path.  CPU only."""
import itertools

import numpy as np
import pytest

import synth_inputs as si
from oracle import eesd_oracle as orc


@pytest.fixture(scope="module")
def tiny_corr():
    return si.weights_to_numpy(si.make_weights(si.TINY, seed=0, correlated_draft=0.05))


def test_top_candidates_order_and_ties():
    row = np.array([0.5, 2.0, -1.0, 2.0, 0.5, 3.0, 0.5], np.float32)
    assert orc.top_candidates(row, 4) == [5, 1, 3, 0]
    assert orc.top_candidates(row, 7) == [5, 1, 3, 0, 4, 6, 2]
    rng = np.random.default_rng(1)
    for _ in range(20):
        r = rng.integers(0, 6, 50).astype(np.float32)          # many equal values
        want = sorted(range(50), key=lambda t: (-float(r[t]), t))[:5]
        assert orc.top_candidates(r, 5) == want
    assert orc.top_candidates(row, 1) == [orc.argmax_lowest(row)]


def _all_root_paths(children):
    """Every root path of the candidate tree: chain prefixes, each optionally ending in a leaf."""
    paths = [()]
    chain = ()
    for kids in children:
        for t in kids[1:]:
            paths.append(chain + (t,))
        chain = chain + (kids[0],)
        paths.append(chain)
    return paths


@pytest.mark.parametrize("width", [2, 3, 4])
def test_tree_walk_commits_the_longest_path_the_target_itself_would_take(width):
    """Brute force: over all root paths of the tree, the walk must accept the longest one that is
    a prefix of the target's own greedy continuation, and continue with the target's next token."""
    rng = np.random.default_rng(width)
    V = 5
    seen_leaf = seen_full = seen_zero = 0
    for trial in range(400):
        K = int(rng.integers(1, 5))
        children = [list(rng.choice(V, size=width, replace=False)) for _ in range(K)]
        table = {}

        def top_of(path):
            if path not in table:
                table[path] = int(rng.integers(0, V))
            return table[path]

        a, y, branch = orc.tree_walk(children, top_of)
        # the target's own continuation, K + 1 tokens
        cont = []
        for _ in range(K + 1):
            cont.append(top_of(tuple(cont)))
        best = max((p for p in _all_root_paths(children) if tuple(cont[:len(p)]) == p), key=len)
        assert a == len(best)
        assert [children[i][branch[i]] for i in range(a)] == list(best)
        assert y == cont[a]
        seen_leaf += a > 0 and branch[-1] != 0
        seen_full += a == K
        seen_zero += a == 0
    assert seen_leaf and seen_full and seen_zero


@pytest.mark.parametrize("width", [2, 3])
def test_tree_generation_equals_greedy_autoregressive_and_accepts_more(tiny_corr, width):
    prompt = si.make_prompt(24, 512, 0)
    ar = orc.OracleEESD(tiny_corr, 128, 0.0).ar_generate(prompt, 48)
    chain = orc.OracleEESD(tiny_corr, 128, 0.0, seed=2, k_cap=4)
    assert chain.generate(prompt, 48, fixed_k=4) == ar
    for kw in (dict(fixed_k=4), dict(fixed_k=1), dict(k_schedule=[1 + (i * 3) % 4 for i in range(48)]), dict()):
        t = orc.OracleEESDTree(tiny_corr, 128, width, seed=2, k_cap=4)
        trace = []
        assert t.generate_tree(prompt, 48, trace=trace, **kw) == ar
        if kw.get("fixed_k") == 4:
            assert t.stats.rounds <= chain.stats.rounds            # never fewer tokens per round than the chain
            assert any(r["a"] and r["branch"][-1] != 0 for r in trace)   # a leaf was accepted somewhere
            assert any(r["a"] == r["K"] for r in trace)


def test_node_logits_equal_from_scratch_forwards_of_every_path(tiny_corr):
    prompt = si.make_prompt(7, 512, 5)
    t = orc.OracleEESDTree(tiny_corr, 64, 3, seed=1, k_cap=3)
    t.prefill(prompt)
    for _ in range(3):
        t.draft_step_tree()
    rows = t.node_logits()
    chain = [k[0] for k in t.children]
    for key, got in rows.items():
        if key == ():
            path = []
        else:
            i, j = key
            path = chain[:i - 1] + [t.children[i - 1][j]]
        ref = orc.OracleEESD(tiny_corr, 64, 0.0)
        want = ref.target_forward(list(prompt) + [t.pending] + path, 0)[-1]
        assert np.max(np.abs(got - want)) < 1e-10, key
    assert len(rows) == 1 + 3 * 3


def test_tree_rollback_leaves_the_caches_of_the_committed_text(tiny_corr):
    prompt = si.make_prompt(9, 512, 8)
    t = orc.OracleEESDTree(tiny_corr, 128, 3, seed=3, k_cap=4)
    committed = list(prompt) + [t.prefill(prompt)]
    leaf = 0
    for rnd in range(8):
        for _ in range(1 + rnd % 4):
            t.draft_step_tree()
        a, y, branch = t.verify_accept_tree()
        leaf += a > 0 and branch[-1] != 0
        committed += t.rollback_tree(a, y, branch) + [y]
    assert leaf > 0
    n = t.kv_len
    assert n == len(committed) - 1 and committed[n] == t.pending
    ref = orc.OracleEESD(tiny_corr, 128, 0.0)
    ref.target_forward(committed[:n], 0)
    for c_t, c_r in zip(t.kv + [t.ee_kv], ref.kv + [ref.ee_kv]):
        assert np.max(np.abs(c_t.k[:n] - c_r.k[:n])) < 1e-11
        assert np.max(np.abs(c_t.v[:n] - c_r.v[:n])) < 1e-11
