"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke run.

This module only *makes data*: model shapes, random weight tensors, random
prompts and random probability rows.  It contains none of the decoding
method's arithmetic and imports neither the CPU oracle nor the HIP library,
so both sides can be fed from it without sharing any code of the method.

The shapes are the LLaMA-style decoder shapes the evaluation is quoted on
(a tiny fp32 model, a 13B-shaped and a 70B-shaped bf16 model), with weights
drawn i.i.d. from N(0, 0.02^2) and prompts drawn uniformly over the
vocabulary.  They stand in for the trained checkpoints and the text
benchmarks of the paper's evaluation (Section 4.1), which are not available.
"""
from __future__ import annotations

import copy
from typing import Dict, List, Optional

import numpy as np
import torch

# ---------------------------------------------------------------------------
# model shapes
# ---------------------------------------------------------------------------
# n_draft_layers is the paper's N (Section 3.1): the draft model is the first
# N decoder layers of the target plus one extra decoder layer and its own head.

TINY = dict(name="tiny", n_layers=4, n_draft_layers=1, d_model=256, n_heads=4,
            n_kv_heads=4, head_dim=64, d_ff=688, vocab=512, rms_eps=1e-6,
            rope_base=10000.0, dtype="fp32")

# a GQA variant of the tiny model (2 KV heads for 4 query heads), bf16
TINY_GQA_BF16 = dict(name="tiny_gqa_bf16", n_layers=3, n_draft_layers=1, d_model=512,
                     n_heads=4, n_kv_heads=2, head_dim=128, d_ff=1024, vocab=1024,
                     rms_eps=1e-6, rope_base=10000.0, dtype="bf16")

# a bf16 model with 64-wide heads (8 query heads on 2 KV heads)
TINY_HD64_BF16 = dict(name="tiny_hd64_bf16", n_layers=3, n_draft_layers=2, d_model=512,
                      n_heads=8, n_kv_heads=2, head_dim=64, d_ff=768, vocab=512,
                      rms_eps=1e-5, rope_base=10000.0, dtype="bf16")

LLAMA13B = dict(name="llama2-13b-shape", n_layers=40, n_draft_layers=5, d_model=5120,
                n_heads=40, n_kv_heads=40, head_dim=128, d_ff=13824, vocab=32000,
                rms_eps=1e-5, rope_base=10000.0, dtype="bf16")

LLAMA70B = dict(name="llama2-70b-shape", n_layers=80, n_draft_layers=10, d_model=8192,
                n_heads=64, n_kv_heads=8, head_dim=128, d_ff=28672, vocab=32000,
                rms_eps=1e-5, rope_base=10000.0, dtype="bf16")


def reduced_depth(shape: dict, n_layers: int, n_draft_layers: int) -> dict:
    """Same per-layer shape, fewer layers (used where a full-depth CPU run is too slow)."""
    s = copy.deepcopy(shape)
    s["n_layers"] = n_layers
    s["n_draft_layers"] = n_draft_layers
    s["name"] = f"{shape['name']}-L{n_layers}N{n_draft_layers}"
    return s


def layer_param_count(shape: dict) -> int:
    d, hd = shape["d_model"], shape["head_dim"]
    H, Hkv, f = shape["n_heads"], shape["n_kv_heads"], shape["d_ff"]
    return (H + 2 * Hkv) * hd * d + d * H * hd + 2 * f * d + d * f + 2 * d


def layer_bytes(shape: dict) -> int:
    return layer_param_count(shape) * (2 if shape["dtype"] == "bf16" else 4)


def head_bytes(shape: dict) -> int:
    return shape["vocab"] * shape["d_model"] * (2 if shape["dtype"] == "bf16" else 4)


def kv_bytes_per_token_layer(shape: dict) -> int:
    return 2 * shape["n_kv_heads"] * shape["head_dim"] * (2 if shape["dtype"] == "bf16" else 4)


# ---------------------------------------------------------------------------
# weights
# ---------------------------------------------------------------------------

def _torch_dtype(shape: dict) -> torch.dtype:
    return torch.bfloat16 if shape["dtype"] == "bf16" else torch.float32


def _randn(gen: torch.Generator, shape, std: float, dtype: torch.dtype, device) -> torch.Tensor:
    # drawn in fp32 then rounded once to the storage type: the rounded values
    # ARE the weights, for the oracle as well as for the GPU.
    rows = shape[0]
    out = torch.empty(shape, dtype=dtype, device=device)
    # chunked so a 32000 x 8192 head never needs a full fp32 temporary on a busy device
    step = max(1, (1 << 26) // max(1, int(np.prod(shape[1:]))))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        t = torch.randn((r1 - r0,) + tuple(shape[1:]), generator=gen, dtype=torch.float32, device=device)
        out[r0:r1] = (t * std).to(dtype)
    return out


def _gain(gen: torch.Generator, d: int, jitter: float, dtype: torch.dtype, device) -> torch.Tensor:
    g = torch.ones(d, dtype=torch.float32, device=device)
    if jitter > 0.0:
        g = g + jitter * torch.randn(d, generator=gen, dtype=torch.float32, device=device)
    return g.to(dtype)


def _make_layer(gen, shape: dict, std: float, jitter: float, dtype, device) -> Dict[str, torch.Tensor]:
    d, hd = shape["d_model"], shape["head_dim"]
    H, Hkv, f = shape["n_heads"], shape["n_kv_heads"], shape["d_ff"]
    return dict(
        attn_norm=_gain(gen, d, jitter, dtype, device),
        wqkv=_randn(gen, ((H + 2 * Hkv) * hd, d), std, dtype, device),   # rows: all q heads, all k heads, all v heads
        wo=_randn(gen, (d, H * hd), std, dtype, device),
        ffn_norm=_gain(gen, d, jitter, dtype, device),
        w_gate_up=_randn(gen, (2 * f, d), std, dtype, device),           # rows: gate (f), then up (f)
        w_down=_randn(gen, (d, f), std, dtype, device),
    )


def make_weights(shape: dict, seed: int, device="cpu", std: float = 0.02,
                 norm_gain_jitter: float = 0.0,
                 correlated_draft: Optional[float] = None) -> dict:
    """Random model weights.  Every matrix is row-major [out][in].

    correlated_draft=gamma builds a test-only model whose draft distribution is
    close to the target's: the output projections (wo, w_down) of the target
    layers past the first N and of the early-exit layer are scaled by gamma,
    and the early-exit norm/head are copies of the target's final norm/head.
    With random independent weights a greedy draft token is almost never
    accepted; this mode makes acceptance frequent so that accept paths with
    a > 0 are exercised.
    """
    dtype = _torch_dtype(shape)
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    d, V = shape["d_model"], shape["vocab"]
    w = dict(shape=dict(shape))
    w["tok_emb"] = _randn(gen, (V, d), std, dtype, device)
    w["layers"] = [_make_layer(gen, shape, std, norm_gain_jitter, dtype, device)
                   for _ in range(shape["n_layers"])]
    w["final_norm"] = _gain(gen, d, norm_gain_jitter, dtype, device)
    w["lm_head"] = _randn(gen, (V, d), std, dtype, device)
    w["ee_layer"] = _make_layer(gen, shape, std, norm_gain_jitter, dtype, device)
    w["ee_norm"] = _gain(gen, d, norm_gain_jitter, dtype, device)
    w["ee_head"] = _randn(gen, (V, d), std, dtype, device)
    if correlated_draft is not None:
        g = float(correlated_draft)
        for l in range(shape["n_draft_layers"], shape["n_layers"]):
            for k in ("wo", "w_down"):
                w["layers"][l][k] = (w["layers"][l][k].float() * g).to(dtype)
        for k in ("wo", "w_down"):
            w["ee_layer"][k] = (w["ee_layer"][k].float() * g).to(dtype)
        w["ee_norm"] = w["final_norm"].clone()
        w["ee_head"] = w["lm_head"].clone()
    return w


def make_cali_weights(shape: dict, seed: int, device="cpu", n_mats: int = 10, spread: float = 8.0) -> dict:
    """Random predictor of the calibrated controller: n_mats matrices [d][d] and one [2][2d]
    (both [out][in]) in the model's storage type, scaled so that scores spread over (0, 1)."""
    dtype = _torch_dtype(shape)
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed) + 7919)
    d = shape["d_model"]
    return dict(w=_randn(gen, (n_mats, d, d), 1.0 / d ** 0.5, dtype, device),
                wp=_randn(gen, (2, 2 * d), spread / (2 * d) ** 0.5, dtype, device))


def cali_to_numpy(cw: dict) -> dict:
    return {k: v.detach().to("cpu", torch.float32).numpy() for k, v in cw.items()}


LAYER_KEYS = ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")


def weights_to_numpy(w: dict) -> dict:
    """fp32 numpy copy of a weight dict (bf16 values widen exactly)."""
    def cv(t):
        return t.detach().to("cpu", torch.float32).numpy()
    out = dict(shape=dict(w["shape"]))
    for k in ("tok_emb", "final_norm", "lm_head", "ee_norm", "ee_head"):
        out[k] = cv(w[k])
    out["layers"] = [{k: cv(l[k]) for k in LAYER_KEYS} for l in w["layers"]]
    out["ee_layer"] = {k: cv(w["ee_layer"][k]) for k in LAYER_KEYS}
    return out


def weights_to_device(w: dict, device) -> dict:
    out = dict(shape=dict(w["shape"]))
    for k in ("tok_emb", "final_norm", "lm_head", "ee_norm", "ee_head"):
        out[k] = w[k].to(device).contiguous()
    out["layers"] = [{k: l[k].to(device).contiguous() for k in LAYER_KEYS} for l in w["layers"]]
    out["ee_layer"] = {k: w["ee_layer"][k].to(device).contiguous() for k in LAYER_KEYS}
    return out


# ---------------------------------------------------------------------------
# prompts, uniforms, probability rows
# ---------------------------------------------------------------------------

def make_prompt(n: int, vocab: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.integers(0, vocab, size=n, dtype=np.int32)


def make_uniforms(n: int, seed: int) -> np.ndarray:
    """n doubles in [0,1) on the 53-bit grid."""
    rng = np.random.default_rng(seed)
    return (rng.integers(0, 1 << 53, size=n, dtype=np.uint64).astype(np.float64)) * 2.0 ** -53


def make_logit_rows(rows: int, vocab: int, seed: int, std: float = 1.5) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((rows, vocab)) * std).astype(np.float32)


def make_prob_rows(rows: int, vocab: int, seed: int, peaked: float = 1.5,
                   zero_frac: float = 0.0) -> np.ndarray:
    """fp32 rows that are non-negative and sum to ~1 (sum differs from 1 by
    fp32 rounding, as the rows a softmax kernel writes do).  zero_frac sets a
    share of the entries to exactly 0."""
    rng = np.random.default_rng(seed)
    w = np.exp(rng.standard_normal((rows, vocab)) * peaked)
    if zero_frac > 0.0:
        w[rng.random((rows, vocab)) < zero_frac] = 0.0
        w[:, 0] += 1e-3  # never an all-zero row
    w = w / w.sum(axis=1, keepdims=True)
    return w.astype(np.float32)
