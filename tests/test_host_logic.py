"""Host-side logic of the library against the oracle, without a GPU: the counter-based uniforms,
the Beta-posterior controller of Section 3.3 / Algorithm 2 (bit-exact for integer posteriors) and
the posterior update of Eq. 3-4 in both readings."""
import numpy as np
import pytest

import paper_2406_03853_amd as pk
from oracle import eesd_oracle as orc


def test_uniforms_are_bit_identical_to_the_oracles():
    for seed in (0, 1, 0xDEADBEEFCAFE, 2 ** 63 + 5):
        for stream in (1, 2, 3, 4, 5):
            for rnd in (0, 1, 77, 65535, 2 ** 20 + 3):
                for slot, sub in ((0, 0), (3, 0), (15, 1), (200, 4097)):
                    assert pk.host_uniform(seed, stream, rnd, slot, sub) == orc.uniform(seed, stream, rnd, slot, sub)


def test_draft_length_draws_are_bit_identical_for_integer_posteriors():
    for a, b in ((1, 1), (3, 2), (2, 9), (40, 17), (1, 300)):
        for seed in (0, 9):
            ts = orc.BetaTS(a, b, seed)
            for rnd in range(1, 120):
                for k_max in (1, 2, 5, 10):
                    assert pk.host_draw_k(a, b, seed, rnd, k_max) == ts.draw_k(rnd, k_max), (a, b, seed, rnd, k_max)


def test_posterior_update_matches_both_readings():
    for mode, reading in (("prose", 0), ("literal", 1)):
        for K in range(1, 8):
            for a in range(0, K + 1):
                ts = orc.BetaTS(2, 3, 0, mode)
                ts.update(a, K)
                assert pk.host_ts_update(2.0, 3.0, a, K, reading) == (ts.alpha, ts.beta)
    with pytest.raises(pk.EesdError):
        pk.host_ts_update(1.0, 1.0, 5, 4, 0)


def test_non_integer_posterior_keeps_the_law_of_k():
    from scipy import stats
    a, b, cap, n = 2.5, 1.5, 6, 4000
    ks = np.array([pk.host_draw_k(a, b, 3, rnd, cap) for rnd in range(n)])
    c = a / (a + b)
    want = np.array([c ** (k - 1) * (1 - c) for k in range(1, cap)] + [c ** (cap - 1)])
    got = np.bincount(ks, minlength=cap + 1)[1:]
    assert stats.chisquare(got, want * n).pvalue > 1e-3
    with pytest.raises(pk.EesdError):
        pk.host_draw_k(0.0, 1.0, 0, 0, 4)


def test_calibrated_controller_decisions_match_the_oracle():
    """Section 3.3 Eq. 6-7, Algorithm 3 steps 9-12 on the host: same posterior, same normal variate
    (both sides call the C library's log / cos / sqrt), same decision."""
    flips = 0
    for sm, ss in ((0.2, 0.5), (0.05, 1.0), (0.7, 0.1)):
        for seed in (0, 123456789):
            c = orc.CaliTS(sm, ss, 0.4, seed=seed)
            for n in (0, 1, 5, 60):
                c.n = n
                for rnd in range(1, 40):
                    for slot in (1, 2, 9):
                        theta_m = 0.05 + 0.9 * orc.uniform(7, 1, rnd, slot)
                        want_theta, want_chi = c.decide(theta_m, rnd, slot)
                        theta, chi = pk.host_cali_decide(sm, ss, c.theta_hat, n, theta_m, seed, rnd, slot)
                        assert abs(theta - want_theta) <= 1e-15 * max(1.0, abs(want_theta))
                        if abs(want_theta - orc.uniform(seed, orc.STREAM_TS_CHI, rnd, slot)) > 1e-12:
                            assert chi == want_chi
                        flips += chi
    assert 0 < flips


def test_calibrated_controller_update_matches_both_readings():
    for mode, reading in (("judged", 0), ("printed", 1)):
        c = orc.CaliTS(0.2, 0.5, 0.35, update=mode)
        th, w, n = 0.35, 1.0, 0
        for a, K in [(0, 3), (2, 2), (1, 4), (0, 1), (5, 5), (3, 7), (0, 2)]:
            c.update(a, K)
            th, w, n = pk.host_cali_update(th, w, n, a, K, reading)
            assert (th, w, n) == (c.theta_hat, c.weight, c.n)
    with pytest.raises(pk.EesdError):
        pk.host_cali_update(0.5, 1.0, 0, 3, 2, 0)


def test_operand_order_layouts_are_permutations_with_the_mfma_lane_order():
    """The operand-order layouts of the KV cache and of a prefill block's activation rows: every element has its own
    place (a permutation of the block), and the places are those of the MFMA operands - lane l = 16 g + i of a 1 KB
    block owns 16 contiguous bytes at 16 l."""
    import paper_2406_03853_amd as pk
    for hd in (64, 128):
        page = 64
        ks = np.array([[pk.host_layout_offset(0, s, c, hd) for c in range(hd)] for s in range(page)])
        vs = np.array([[pk.host_layout_offset(1, s, c, hd) for c in range(hd)] for s in range(page)])
        for off in (ks, vs):
            assert sorted(off.ravel().tolist()) == list(range(page * hd))
        for step in range(page // 32):
            for r in range(32):
                s = step * 32 + r
                tile, i = (r >> 2) & 1, ((r >> 3) << 2) | (r & 3)          # tile A: slots 8a+b, tile B: 8a+4+b; row 4a+b
                for c in range(hd):
                    q, g, e = c // 32, (c % 32) // 8, c % 8
                    assert ks[s, c] == ((((step * 2 + tile) * (hd // 32) + q) * 64) + 16 * g + i) * 8 + e
                    dt, ci = c // 16, c % 16
                    assert vs[s, c] == (((step * (hd // 16) + dt) * 64) + 16 * ((r >> 3) & 3) + ci) * 8 + (s & 7)
    steps = 5
    act = np.array([[pk.host_layout_offset(2, m, c, steps) for c in range(32 * steps)] for m in range(48)])
    assert sorted(act.ravel().tolist()) == list(range(48 * 32 * steps))
    for m in range(48):
        for c in range(32 * steps):
            assert act[m, c] == ((((m // 16) * steps + c // 32) * 64) + ((c % 32) // 8) * 16 + m % 16) * 8 + c % 8
    assert pk.host_layout_offset(0, 0, 0, 48) == -1 and pk.host_layout_offset(7, 0, 0, 64) == -1


def test_row_groups_partition_a_matrix_in_units_of_four_rows():
    """Tile-major weights: matrices with more tiles than CUs but fewer than four per CU are dealt to one row group per
    CU in units of 4 rows - consecutive, covering every row once, the first groups one unit larger; the others keep
    one 16-row tile per group."""
    import paper_2406_03853_amd as pk
    n_cu = 256
    for rows, want_groups in ((5120, 256), (8192, 256), (10240, 256), (15360, 256), (4608, 256), (4096, 256), (1024, 64), (27648, 1728), (32000, 2000)):
        groups = pk.host_layout_offset(5, 0, rows, n_cu)
        assert groups == want_groups
        geo = [(pk.host_layout_offset(3, g, rows, n_cu), pk.host_layout_offset(4, g, rows, n_cu)) for g in range(groups)]
        assert geo[0][0] == 0 and geo[-1][0] + geo[-1][1] == rows
        assert all(geo[g][0] + geo[g][1] == geo[g + 1][0] for g in range(groups - 1))
        sizes = [r for _, r in geo]
        assert all(r % 4 == 0 and r > 0 for r in sizes) and max(sizes) - min(sizes) in (0, 4)
        assert sizes == sorted(sizes, reverse=True)
        if groups == rows // 16:
            assert set(sizes) == {16}
    assert pk.host_layout_offset(3, 256, 5120, n_cu) == -1 and pk.host_layout_offset(5, 0, 5000, n_cu) == -1
