"""Helpers of the GPU parity tests (HIP library vs CPU oracle on the same seeded inputs)."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import eesd_oracle as orc

TOL_F32 = 1e-4   # max-abs error relative to the largest reference magnitude, fp32 path
TOL_BF16 = 3e-2  # same, bf16 path


def require_gpu():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    return float(np.max(np.abs(np.asarray(got, np.float64) - want)) / max(1e-30, np.max(np.abs(want))))


def tol_of(shape: dict) -> float:
    return TOL_BF16 if shape["dtype"] == "bf16" else TOL_F32


def make_pair(shape, wseed, max_seq, temperature, k_cap=5, jitter=0.1, gamma=None, gen_device="cpu", **kw):
    """The same weights for the oracle (numpy, CPU) and the library (torch, GPU).
    gen_device="cuda" draws big models on the GPU and copies them to the host for the oracle."""
    import paper_2406_03853_amd as pk
    w = si.make_weights(shape, seed=wseed, norm_gain_jitter=jitter, correlated_draft=gamma, device=gen_device)
    if kw.get("tree_width", 0) >= 2:
        o = orc.OracleEESDTree(si.weights_to_numpy(w), max_seq, kw["tree_width"], seed=kw.get("seed", 0), k_cap=k_cap,
                               ts_update="literal" if kw.get("ts_update", 0) else "prose")
    else:
        o = orc.OracleEESD(si.weights_to_numpy(w), max_seq, temperature, seed=kw.get("seed", 0), k_cap=k_cap,
                           ts_update="literal" if kw.get("ts_update", 0) else "prose")
    wd = si.weights_to_device(w, "cuda")
    if kw.get("weight_layout", 0) == pk.WEIGHTS_TILED:
        wd = pk.pack_weights(wd)
    g = pk.EESD(wd, max_seq, temperature, k_cap=k_cap, **kw)
    return o, g


def sample_margin(r32: np.ndarray, u: float) -> float:
    """Distance of u from the nearest inverse-CDF threshold, relative to the total."""
    c = np.cumsum(r32.astype(np.float64))
    if not c[-1] > 0:
        return 0.0
    return float(np.min(np.abs(c / c[-1] - u)))


def top2_gap(logits: np.ndarray) -> float:
    s = np.sort(np.asarray(logits, np.float64))
    return float((s[-1] - s[-2]) / max(1e-30, np.max(np.abs(s))))
