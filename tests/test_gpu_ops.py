"""Stand-alone kernels against the oracle: the weight-streaming product, softmax + sampling,
and the accept / resample decision (bit-exact on identical probability rows and uniforms)."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import eesd_oracle as orc
from gpu_common import TOL_BF16, TOL_F32, rel_err, require_gpu

pytestmark = pytest.mark.gpu


def _pk():
    import paper_2406_03853_amd as pk
    return pk


def _gemm_case(M, out, inn, dtype, path, seed):
    pk = _pk()
    g = torch.Generator().manual_seed(seed)
    W = (torch.randn(out, inn, generator=g) * 0.05).to(dtype)
    X = torch.randn(M, inn, generator=g)
    Y = torch.full((M, out), float("nan"), device="cuda")
    pk.op_gemm(W.cuda(), X.cuda(), Y, path)
    torch.cuda.synchronize()
    want = X.double().numpy() @ W.double().numpy().T
    return rel_err(Y.cpu().numpy(), want)


@pytest.mark.parametrize("M", [1, 2, 3, 5, 8, 11, 16])
@pytest.mark.parametrize("out,inn", [(512, 256), (256, 688), (1376, 256)])
def test_gemm_valu_fp32(M, out, inn):
    require_gpu()
    assert _gemm_case(M, out, inn, torch.float32, _pk().GEMM_VALU, 1) < TOL_F32


@pytest.mark.parametrize("M", [1, 2, 4])
@pytest.mark.parametrize("out,inn", [(1024, 512), (5120, 5120), (320, 13824), (32000, 1024)])
def test_gemm_valu_bf16(M, out, inn):
    require_gpu()
    if M * inn * 4 > 140 * 1024:
        pytest.skip("activations do not fit in LDS for this family")
    assert _gemm_case(M, out, inn, torch.bfloat16, _pk().GEMM_VALU, 2) < TOL_F32   # fp32 activations: tight


@pytest.mark.parametrize("M", [1, 2, 5, 11, 16])
@pytest.mark.parametrize("out,inn", [(1024, 512), (5120, 5120), (160, 13824), (32000, 1024), (80, 128)])
def test_gemm_mfma_bf16(M, out, inn):
    require_gpu()
    assert _gemm_case(M, out, inn, torch.bfloat16, _pk().GEMM_MFMA, 3) < TOL_BF16


@pytest.mark.parametrize("M", [1, 7, 16, 17, 40, 64, 100, 128])
@pytest.mark.parametrize("out,inn", [(1024, 512), (5120, 5120), (320, 13824), (32000, 1024), (64, 256)])
def test_gemm_tile_kernel_bf16(M, out, inn):
    """The LDS-shared tile kernel: prefill blocks (M > 16) and, forced, verify-sized blocks."""
    require_gpu()
    pk = _pk()
    try:
        pk.set_tunable("mfma_tile", 1)
        assert _gemm_case(M, out, inn, torch.bfloat16, pk.GEMM_MFMA, 6) < TOL_BF16
    finally:
        pk.set_tunable("mfma_tile", 0)


@pytest.mark.parametrize("kc,nwt", [(512, 4), (0, 8), (512, 8)])
@pytest.mark.parametrize("M", [2, 11, 16])
def test_gemm_tile_kernel_chunk_and_workgroup_shapes(kc, nwt, M):
    require_gpu()
    pk = _pk()
    try:
        pk.set_tunable("mfma_tile", 1)
        pk.set_tunable("tile_kc", kc)
        pk.set_tunable("tile_nwt", nwt)
        assert _gemm_case(M, 2048, 1536, torch.bfloat16, pk.GEMM_MFMA, 8) < TOL_BF16
        assert _gemm_case(M, 27648, 512, torch.bfloat16, pk.GEMM_MFMA, 9) < TOL_BF16
    finally:
        for k in ("mfma_tile", "tile_kc", "tile_nwt"):
            pk.set_tunable(k, 0)


@pytest.mark.parametrize("M", [65, 128])
def test_gemm_tile_kernel_prefill_chunk_256(M):
    require_gpu()
    pk = _pk()
    try:
        pk.set_tunable("pf_kc", 256)
        assert _gemm_case(M, 2048, 1536, torch.bfloat16, pk.GEMM_MFMA, 10) < TOL_BF16
    finally:
        pk.set_tunable("pf_kc", 0)


@pytest.mark.parametrize("M", [1, 5, 11, 16, 40, 128])
@pytest.mark.parametrize("out,inn", [(1024, 512), (5120, 5120), (320, 13824), (32000, 1024), (64, 256)])
def test_gemm_tiled_weight_layout_equals_row_major(M, out, inn):
    """The tile-major weight layout (one contiguous 1 KB read per MFMA operand): the same product as
    from the row-major matrix up to the order in which the waves' partial sums are added."""
    require_gpu()
    pk = _pk()
    g = torch.Generator(device="cpu").manual_seed(out + inn + M)
    W = (torch.randn(out, inn, generator=g) * 0.05).to(torch.bfloat16).cuda()
    X = torch.randn(M, inn, generator=g).cuda()
    Y0 = torch.empty(M, out, device="cuda")
    Y1 = torch.empty(M, out, device="cuda")
    Wp = pk.pack_weight(W)
    assert Wp.shape == W.shape and not torch.equal(Wp, W)
    for tile in (0, 1):
        try:
            pk.set_tunable("mfma_tile", tile)
            pk.op_gemm(W, X, Y0, pk.GEMM_MFMA)
            pk.op_gemm(Wp, X, Y1, pk.GEMM_MFMA, weight_layout=pk.WEIGHTS_TILED)
            torch.cuda.synchronize()
            assert float((Y0 - Y1).abs().max()) <= 2e-5 * float(Y0.abs().max())
        finally:
            pk.set_tunable("mfma_tile", 0)
    ref = X.double().cpu().numpy() @ W.double().cpu().numpy().T
    assert np.max(np.abs(Y1.cpu().numpy() - ref)) / np.max(np.abs(ref)) < TOL_BF16


@pytest.mark.parametrize("M", [17, 100, 256, 300, 512])
@pytest.mark.parametrize("out,inn", [(1024, 512), (8192, 2048), (10240, 1024), (15360, 1024), (5120, 13824), (4608, 512), (27648, 512)])
def test_prefill_gemm_on_tile_major_weights(M, out, inn):
    """Blocks of more than 16 rows on tile-major weights (the prefill GEMM: weight operands shared through LDS,
    the block's rows read in operand order).  On a 256-CU device the shapes give one tile per row group (1024,
    27648), groups of 2 tiles (8192), 3 (10240: 40 rows), 4 (15360: 60 rows), of 20 rows (5120: a whole tile
    and a quarter, the quarters of two groups gathered in one tile slot) and of 20 and 16 rows mixed (4608); the row counts give 1, 2 and 4 token blocks per wave, idle waves, and a ragged last block."""
    require_gpu()
    pk = _pk()
    g = torch.Generator(device="cpu").manual_seed(out + inn + M)
    W = (torch.randn(out, inn, generator=g) * 0.05).to(torch.bfloat16)
    X = torch.randn(M, inn, generator=g)
    Y = torch.full((M, out), float("nan"), device="cuda")
    pk.op_gemm(pk.pack_weight(W.cuda()), X.cuda(), Y, pk.GEMM_MFMA, weight_layout=pk.WEIGHTS_TILED)
    torch.cuda.synchronize()
    ref = X.double().numpy() @ W.double().numpy().T
    assert rel_err(Y.cpu().numpy(), ref) < TOL_BF16
    # against the rows as the kernel sees them (rounded to bf16): only the order of the fp32 sums differs
    ref16 = X.to(torch.bfloat16).double().numpy() @ W.double().numpy().T
    assert rel_err(Y.cpu().numpy(), ref16) < 1e-5
    if M <= 128:
        # the kernel that row-major weights (and pf_rows = 128) take for such blocks agrees
        Y0 = torch.empty(M, out, device="cuda")
        try:
            pk.set_tunable("pf_rows", 128)
            pk.op_gemm(pk.pack_weight(W.cuda()), X.cuda(), Y0, pk.GEMM_MFMA, weight_layout=pk.WEIGHTS_TILED)
            torch.cuda.synchronize()
        finally:
            pk.set_tunable("pf_rows", 0)
        assert float((Y0 - Y).abs().max()) <= 2e-5 * float(Y.abs().max())
    if out in (5120, 4608):
        # a tile slot per tail instead of the gathered one: the same sums in the same order
        Y0 = torch.empty(M, out, device="cuda")
        try:
            pk.set_tunable("pf_merge", 0)
            pk.op_gemm(pk.pack_weight(W.cuda()), X.cuda(), Y0, pk.GEMM_MFMA, weight_layout=pk.WEIGHTS_TILED)
            torch.cuda.synchronize()
        finally:
            pk.set_tunable("pf_merge", -1)
        assert torch.equal(Y0, Y)


def test_pack_weight_is_a_permutation_of_16_byte_pieces():
    require_gpu()
    pk = _pk()
    out, inn, hd = 512, 256, 128
    W = torch.arange(out * inn, dtype=torch.float32).remainder(65521).to(torch.bfloat16).reshape(out, inn).cuda()
    for kind, hdim in ((pk.PACK_PLAIN, 0), (pk.PACK_GATE_UP, 0), (pk.PACK_QKV, hd)):
        P = pk.pack_weight(W, kind, hdim).cpu().view(torch.int16).numpy().reshape(out // 16, inn // 32, 4, 16, 8)   # [tile][q][g][i][8]
        Wn = W.cpu().view(torch.int16).numpy()
        for tile in (0, 1, out // 16 - 1):
            for i in (0, 7, 8, 15):
                if kind == pk.PACK_PLAIN:
                    row = tile * 16 + i
                elif kind == pk.PACK_GATE_UP:
                    row = (0 if i < 8 else out // 2) + tile * 8 + (i & 7)
                else:
                    head, part = divmod(tile, hd // 16)
                    row = head * hd + (0 if i < 8 else hd // 2) + part * 8 + (i & 7)
                for q in (0, inn // 32 - 1):
                    for g in range(4):
                        assert (P[tile, q, g, i] == Wn[row, q * 32 + g * 8: q * 32 + g * 8 + 8]).all(), (kind, tile, i, q, g)
    with pytest.raises(pk.EesdError):
        pk.pack_weight(W[:, :96].contiguous())        # columns not a multiple of 128


@pytest.mark.parametrize("nw", [1, 2, 4, 16])
def test_gemm_mfma_launch_shapes(nw):
    require_gpu()
    pk = _pk()
    try:
        pk.set_tunable("mfma_nw", nw)
        assert _gemm_case(7, 2048, 2048, torch.bfloat16, pk.GEMM_MFMA, 4) < TOL_BF16
        assert _gemm_case(16, 176, 1280, torch.bfloat16, pk.GEMM_MFMA, 5) < TOL_BF16
    finally:
        pk.set_tunable("mfma_nw", 0)


@pytest.mark.parametrize("spread", [0, 1])                  # one workgroup / three kernels over 64 workgroups
@pytest.mark.parametrize("V", [512, 1000, 32000, 50257, 65536])   # 50257 is too long for the LDS-resident row
def test_softmax_sample_bit_exact_tokens(V, spread):
    require_gpu()
    pk = _pk()
    pk.set_tunable("smp_spread", spread)
    try:
        _softmax_sample_case(pk, V)
    finally:
        pk.set_tunable("smp_spread", -1)


def test_softmax_sample_edge_uniforms_and_one_hot_rows():
    """Uniforms at both ends of [0, 1) and rows whose whole mass sits on one entry (first, last, in the ragged tail of
    the last chunk), in both kernels: the token is the rule's on the GPU's own row."""
    require_gpu()
    pk = _pk()
    V = 32000
    try:
        for spread in (0, 1):
            pk.set_tunable("smp_spread", spread)
            for hot in (0, 31, 16383, 31743, 31999):
                row = np.full(V, -200.0, np.float32)
                row[hot] = 5.0
                for u in (0.0, 0.5, np.nextafter(1.0, 0.0)):
                    probs = torch.zeros(V, device="cuda")
                    tok = pk.op_softmax_sample(torch.from_numpy(row).cuda(), probs, 1.0, float(u))
                    assert tok == hot == orc.decide_sample(probs.cpu().numpy(), float(u)), (spread, hot, u)
            row = si.make_logit_rows(1, V, seed=5)[0]
            for u in (0.0, np.nextafter(1.0, 0.0)):
                probs = torch.zeros(V, device="cuda")
                tok = pk.op_softmax_sample(torch.from_numpy(row).cuda(), probs, 1.0, float(u))
                assert tok == orc.decide_sample(probs.cpu().numpy(), float(u)), (spread, u)
    finally:
        pk.set_tunable("smp_spread", -1)


def _softmax_sample_case(pk, V):
    logits = si.make_logit_rows(24, V, seed=V)
    us = si.make_uniforms(24, seed=V + 1)
    for i in range(24):
        T = [1.0, 0.7, 0.0][i % 3]
        lg = torch.from_numpy(logits[i]).cuda()
        probs = torch.zeros(V, device="cuda")
        tok = pk.op_softmax_sample(lg, probs, T, float(us[i]))
        if T == 0.0:
            assert tok == orc.argmax_lowest(logits[i])
            continue
        p_gpu = probs.cpu().numpy()
        p_ref = orc.softmax(logits[i].astype(np.float64) / T)
        assert np.max(np.abs(p_gpu - p_ref)) < 2e-6 * np.max(p_ref)
        # the decision is defined on the fp32 row: same row + same uniform => same token
        assert tok == orc.decide_sample(p_gpu, float(us[i]))


def test_argmax_ties_lowest_index():
    require_gpu()
    pk = _pk()
    row = np.zeros(5000, np.float32)
    row[[4100, 77, 2500]] = 3.0
    assert pk.op_softmax_sample(torch.from_numpy(row).cuda(), None, 0.0, 0.0) == 77


@pytest.mark.parametrize("V", [512, 32000, 50257])
@pytest.mark.parametrize("K", [0, 1, 3, 10, 15])
def test_accept_decision_bit_exact(V, K):
    require_gpu()
    pk = _pk()
    mism = 0
    for s in range(12):
        p = si.make_prob_rows(K + 1, V, seed=100 * K + s, zero_frac=0.1 if s % 3 == 0 else 0.0)
        # q close to p so that accept / reject both occur along the block
        q = p[:K] * np.exp(0.6 * np.random.default_rng(s).standard_normal((K, V))).astype(np.float32) if K else np.zeros((0, V), np.float32)
        if K:
            q = (q / q.sum(axis=1, keepdims=True)).astype(np.float32)
        drafts = np.array([orc.decide_sample(q[i], u) for i, u in enumerate(si.make_uniforms(K, seed=7 * s))], np.int32)
        us = si.make_uniforms(K + 1, seed=31 * s + K)
        want = orc.decide_accept(p, q if K else None, drafts, us[:K], us[K], greedy=False)
        qd = torch.from_numpy(q).cuda() if K else None
        got = pk.op_accept(torch.from_numpy(p).cuda(), qd, torch.from_numpy(drafts).cuda(), us, greedy=False)
        assert got == want, (s, got, want)
        mism += want[0] < K
    if K >= 3:
        assert 0 < mism      # rejections did happen


def test_accept_special_rows():
    require_gpu()
    pk = _pk()
    V = 2048
    p = si.make_prob_rows(4, V, seed=5)
    drafts = torch.tensor([3, 900, 2047], dtype=torch.int32, device="cuda")
    # q == p: all accepted, bonus from the last row
    us = si.make_uniforms(4, 9)
    a, y = pk.op_accept(torch.from_numpy(p).cuda(), torch.from_numpy(p[:3].copy()).cuda(), drafts, us, greedy=False)
    assert (a, y) == (3, orc.decide_sample(p[3], us[3]))
    # greedy on logits
    lg = si.make_logit_rows(4, V, seed=6)
    tops = lg.argmax(axis=1)
    d = torch.tensor([tops[0], tops[1], (tops[2] + 1) % V], dtype=torch.int32, device="cuda")
    assert pk.op_accept(torch.from_numpy(lg).cuda(), None, d, None, greedy=True) == (2, int(tops[2]))
    assert pk.op_accept(torch.from_numpy(lg).cuda(), None, d, None, greedy=True) == orc.decide_accept(lg, None, d.cpu().numpy(), None, None, True)


@pytest.mark.parametrize("spread", [0, 1])       # one workgroup walking the rows / all rows at once over 64 workgroups each
@pytest.mark.parametrize("K", [0, 1, 3, 7, 15])
@pytest.mark.parametrize("bf16", [1, 0])
def test_accept_on_logit_rows_bit_exact(K, bf16, spread):
    require_gpu()
    pk = _pk()
    pk.set_tunable("smp_spread", spread)
    try:
        _accept_on_logit_rows_case(pk, K, bf16, 32000 if K != 3 else 50257, spread)
    finally:
        pk.set_tunable("smp_spread", -1)


@pytest.mark.parametrize("V", [4095, 4096, 65536, 65537])
def test_sampling_tails_at_the_vocabulary_limits_of_the_spread_kernels(V):
    """With the built-in choice the spread kernels take vocabularies of 4096 .. 65536 entries and the one-workgroup
    kernels the rest: the rule's token on the kernel's own rows on both sides of both limits, ragged last chunks
    included (65536 fills all 64 chunks of 1024 exactly)."""
    require_gpu()
    pk = _pk()
    _accept_on_logit_rows_case(pk, 2, 0, V, int(4096 <= V <= 65536), n_seeds=2)
    logits = si.make_logit_rows(3, V, seed=V)
    us = si.make_uniforms(3, seed=V + 1)
    for i in range(3):
        probs = torch.zeros(V, device="cuda")
        tok = pk.op_softmax_sample(torch.from_numpy(logits[i]).cuda(), probs, 1.0, float(us[i]))
        p_gpu = probs.cpu().numpy()
        assert np.max(np.abs(p_gpu - orc.softmax(logits[i].astype(np.float64)))) < 2e-6 * p_gpu.max()
        assert tok == orc.decide_sample(p_gpu, float(us[i]))


def test_accept_on_logit_rows_rejected_with_an_empty_residual():
    """A draft whose entry has probability 0 under both models is rejected (u * 0 < 0 is false); with q equal to the
    kernel's own p row entry by entry the residual max(0, p - q) sums to 0 and the next token is drawn from p itself."""
    require_gpu()
    pk = _pk()
    V = 32000
    try:
        for spread in (0, 1):
            pk.set_tunable("smp_spread", spread)
            lg32 = si.make_logit_rows(2, V, seed=77)
            lg32[0, 1234] = -300.0
            lg = torch.from_numpy(lg32).cuda()
            us = np.array([0.3, 0.61])
            p_rows = torch.zeros((2, V), device="cuda")
            dd = torch.tensor([1234], dtype=torch.int32, device="cuda")
            pk.op_accept_logits(lg, p_rows, torch.zeros((1, V), device="cuda"), dd, us, 1.0)      # first call: the kernel's p rows
            q = p_rows[:1].clone()
            assert float(q[0, 1234]) == 0.0
            a, y = pk.op_accept_logits(lg, p_rows, q, dd, us, 1.0)
            p_gpu = p_rows.cpu().numpy()
            assert (a, y) == (0, orc.decide_sample(p_gpu[0], us[1])) == orc.decide_accept(p_gpu, q.cpu().numpy(), [1234], us[:1], us[1], greedy=False)
    finally:
        pk.set_tunable("smp_spread", -1)


def _accept_on_logit_rows_case(pk, K, bf16, V, spread, n_seeds=6):
    """The verification tail on 32000-way logit rows stored as bf16 (and as fp32): the bf16 values are the INPUT of
    both sides.  The probability rows the kernel leaves equal the fp64 softmax of those logits to fp32 rounding, and
    the decision is exactly the oracle's rule on the kernel's own rows with the same uniforms.  Greedy: argmax over
    exactly representable values, so the oracle's rule on the widened logits must agree with no row read back."""
    rej = 0
    for s in range(n_seeds):
        lg32 = si.make_logit_rows(K + 1, V, seed=1000 * K + s)
        lg = torch.from_numpy(lg32).cuda()
        if bf16:
            lg = lg.to(torch.bfloat16)
        lg_in = lg.float().cpu().numpy()                 # what both sides are given
        T = [1.0, 0.8][s % 2]
        p_ref = orc.softmax(lg_in.astype(np.float64) / T)
        # q close to p so that accept / reject both occur along the block
        q = (p_ref[:K] * np.exp(0.6 * np.random.default_rng(s).standard_normal((K, V)))) if K else np.zeros((0, V))
        if K:
            q = (q / q.sum(axis=1, keepdims=True)).astype(np.float32)
        drafts = np.array([orc.decide_sample(q[i], u) for i, u in enumerate(si.make_uniforms(K, seed=7 * s))], np.int32)
        us = si.make_uniforms(K + 1, seed=31 * s + K)
        p_rows = torch.full((K + 1, V), float("nan"), device="cuda")
        qd = torch.from_numpy(np.ascontiguousarray(q, np.float32)).cuda() if K else None
        dd = torch.from_numpy(drafts).cuda()
        a, y = pk.op_accept_logits(lg, p_rows, qd, dd, us, T)
        p_gpu = p_rows.cpu().numpy()
        n_rows = K + 1 if spread else a + 1              # the one-workgroup walk stops after row a
        assert np.isfinite(p_gpu[:n_rows]).all()
        assert np.max(np.abs(p_gpu[:n_rows] - p_ref[:n_rows])) < 2e-6 * np.max(p_ref)
        assert orc.decide_accept(p_gpu, q.astype(np.float32) if K else None, drafts, us[:K], us[K], greedy=False) == (a, y), (s, a, y)
        rej += a < K
        # greedy on the same logits
        tops = lg_in.argmax(axis=1)
        dg = tops[:K].astype(np.int32).copy()
        if K >= 2:
            dg[K // 2] = (dg[K // 2] + 1) % V              # first mismatch in the middle of the block
        got = pk.op_accept_logits(lg, None, None, torch.from_numpy(dg).cuda(), None, 0.0)
        assert got == orc.decide_accept(lg_in, None, dg, None, None, True)
        assert got[0] == (K // 2 if K >= 2 else K)
    if K >= 3:
        assert rej > 0


def test_round_with_bf16_logits_matches_oracle():
    """A context whose LM heads store bf16 logits (the 70B verify micro-benchmark's setting): logits within the bf16
    tolerance of the oracle's, and the round's decisions exactly the rule on the GPU's own probability rows."""
    require_gpu()
    pk = _pk()
    from gpu_common import make_pair, rel_err
    shape = si.TINY_GQA_BF16
    V = shape["vocab"]
    o, g = make_pair(shape, 13, 96, 1.0, k_cap=5, seed=3, logits_bf16=1, weight_layout=1)
    prompt = si.make_prompt(19, V, 2)
    o.prefill(prompt)
    t = g.prefill(prompt)
    assert orc.decide_sample(g.verify_probs(0), orc.uniform(3, orc.STREAM_RESAMPLE, 0)) == t
    o.pending = t
    for K in (4, 2, 5, 0):
        ds = []
        for i in range(K):
            d = g.draft_step()
            assert orc.decide_sample(g.draft_probs(i), orc.uniform(3, orc.STREAM_DRAFT, o.rnd, i)) == d
            o.draft_step(force_token=d)
            got = g.draft_logits(i)
            assert np.array_equal(got, torch.from_numpy(got).to(torch.bfloat16).float().numpy())     # bf16 values
            assert rel_err(got, o.q_logits[i]) < TOL_BF16
            ds.append(d)
        pl = o.verify()
        g.verify()
        a, y = g.accept()
        p = np.full((K + 1, V), np.nan, np.float32)
        for i in range(a + 1):
            p[i] = g.verify_probs(i)
        q = np.stack([g.draft_probs(i) for i in range(K)]) if K else None
        us = [orc.uniform(3, orc.STREAM_ACCEPT, o.rnd, i) for i in range(K)]
        assert orc.decide_accept(p, q, ds, us, orc.uniform(3, orc.STREAM_RESAMPLE, o.rnd), False) == (a, y)
        for i in range(K + 1):
            assert rel_err(g.verify_logits(i), pl[i]) < TOL_BF16
        o.rollback(a, y)
        g.rollback(a)
