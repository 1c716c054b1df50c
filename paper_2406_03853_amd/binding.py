"""ctypes binding of libeesd.so: argument marshalling only.

The names follow include/eesd.h.  Nothing here computes: if the library is not
built the import of `lib()` raises, there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

DTYPE_F32, DTYPE_BF16 = 0, 1
TS_BETA, TS_FIXED, TS_SCHEDULE, TS_CALI = 0, 1, 2, 3
WEIGHTS_ROW_MAJOR, WEIGHTS_TILED = 0, 1
PACK_PLAIN, PACK_GATE_UP, PACK_QKV = 0, 1, 2
GEMM_AUTO, GEMM_VALU, GEMM_MFMA = 0, 1, 2
READ_DRAFT_LOGITS, READ_DRAFT_PROBS, READ_VERIFY_LOGITS, READ_KV_K, READ_KV_V, READ_TOKENS, READ_KV_LEN, READ_PAGE_TABLE, READ_TREE_TOKENS, READ_CALI_STATE, READ_VERIFY_PROBS, READ_LAUNCH_COUNTS = range(12)

_STATUS = {0: "EESD_OK", -1: "EESD_EINVAL", -2: "EESD_ENOMEM", -3: "EESD_ESTATE", -4: "EESD_ERANGE", -5: "EESD_EDEVICE"}


class EesdError(RuntimeError):
    def __init__(self, code: int, text: str = ""):
        super().__init__(f"{_STATUS.get(code, code)}: {text}")
        self.code = code


class _Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_draft_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ff", C.c_int32), ("vocab", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float), ("dtype", C.c_int32), ("max_seq", C.c_int32),
                ("kv_page", C.c_int32), ("k_cap", C.c_int32), ("temperature", C.c_float), ("seed", C.c_uint64),
                ("ts_alpha0", C.c_double), ("ts_beta0", C.c_double), ("ts_mode", C.c_int32), ("ts_update", C.c_int32),
                ("gemm_path", C.c_int32), ("tree_width", C.c_int32), ("verify_reuse", C.c_int32), ("weight_layout", C.c_int32),
                ("logits_bf16", C.c_int32)]


class _Calibration(C.Structure):
    _fields_ = [("w", C.c_void_p), ("wp", C.c_void_p), ("n_mats", C.c_int32), ("update", C.c_int32),
                ("sigma_m", C.c_double), ("sigma_s", C.c_double), ("theta_hat0", C.c_double)]


class _Layer(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")]


class _Weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("layers", C.POINTER(_Layer)), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("ee_layer", _Layer), ("ee_norm", C.c_void_p), ("ee_head", C.c_void_p)]


class _Stats(C.Structure):
    _fields_ = [("rounds", C.c_int64), ("drafted", C.c_int64), ("accepted", C.c_int64), ("generated", C.c_int64),
                ("v_d", C.c_double), ("r_d", C.c_double), ("hm", C.c_double), ("alpha", C.c_double), ("beta", C.c_double),
                ("ms_draft", C.c_double), ("ms_verify", C.c_double), ("ms_accept", C.c_double), ("ms_other", C.c_double)]


@dataclass
class Stats:
    rounds: int
    drafted: int
    accepted: int
    generated: int
    v_d: float
    r_d: float
    hm: float
    alpha: float
    beta: float
    ms_draft: float
    ms_verify: float
    ms_accept: float
    ms_other: float


def lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libeesd.so")


_LIB = None
EXPORTS = ["eesd_create", "eesd_destroy", "eesd_prefill", "eesd_draft_step", "eesd_verify", "eesd_accept", "eesd_accepted_tokens", "eesd_rollback",
           "eesd_generate", "eesd_get_stats", "eesd_last_error", "eesd_set_draft_schedule", "eesd_next_draft_len",
           "eesd_debug_read", "eesd_debug_force_drafts", "eesd_debug_force_pending", "eesd_debug_rollback", "eesd_debug_fill_cache",
           "eesd_host_uniform", "eesd_host_draw_k", "eesd_host_ts_update", "eesd_host_layout_offset", "eesd_set_calibration", "eesd_cali_score",
           "eesd_host_cali_decide", "eesd_host_cali_update", "eesd_debug_profile_begin", "eesd_debug_profile_end", "eesd_debug_copy", "eesd_set_tunable", "eesd_op_accept", "eesd_op_accept_logits", "eesd_op_softmax_sample", "eesd_op_gemm", "eesd_op_gemm_noalloc", "eesd_pack_weight"]


def lib() -> C.CDLL:
    """Loads libeesd.so (built by paper_2406_03853_amd/build.py).  Raises if it is missing."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is not built: run `python -m paper_2406_03853_amd.build`")
    L = C.CDLL(path)
    P, I32, VP = C.POINTER, C.c_int32, C.c_void_p
    L.eesd_create.argtypes = [P(_Config), P(_Weights), VP, P(VP)]
    L.eesd_destroy.argtypes = [VP]
    L.eesd_destroy.restype = None
    L.eesd_prefill.argtypes = [VP, P(I32), I32, P(I32)]
    L.eesd_draft_step.argtypes = [VP, P(I32)]
    L.eesd_verify.argtypes = [VP]
    L.eesd_accept.argtypes = [VP, P(C.c_double), P(I32), P(I32)]
    L.eesd_accepted_tokens.argtypes = [VP, P(I32), I32, P(I32)]
    L.eesd_rollback.argtypes = [VP, I32]
    L.eesd_generate.argtypes = [VP, P(I32), I32, I32, P(I32), P(I32), P(_Stats)]
    L.eesd_get_stats.argtypes = [VP, P(_Stats)]
    L.eesd_last_error.argtypes = [VP]
    L.eesd_last_error.restype = C.c_char_p
    L.eesd_set_draft_schedule.argtypes = [VP, P(I32), I32]
    L.eesd_next_draft_len.argtypes = [VP, I32, P(I32)]
    L.eesd_debug_read.argtypes = [VP, C.c_int, C.c_int, I32, VP, C.c_size_t]
    L.eesd_debug_force_drafts.argtypes = [VP, P(I32), I32]
    L.eesd_debug_force_pending.argtypes = [VP, I32]
    L.eesd_debug_rollback.argtypes = [VP, I32, I32]
    L.eesd_debug_fill_cache.argtypes = [VP, I32, I32]
    L.eesd_set_tunable.argtypes = [C.c_char_p, C.c_int]
    L.eesd_debug_profile_begin.argtypes = [VP, I32, I32, I32]
    L.eesd_debug_profile_end.argtypes = [VP, P(I32), P(C.c_double)]
    L.eesd_debug_copy.argtypes = [VP, VP, C.c_size_t, VP]
    L.eesd_host_uniform.argtypes = [C.c_uint64, I32, C.c_int64, I32, I32]
    L.eesd_host_uniform.restype = C.c_double
    L.eesd_host_layout_offset.argtypes = [I32, I32, I32, I32]
    L.eesd_host_layout_offset.restype = C.c_int64
    L.eesd_host_draw_k.argtypes = [C.c_double, C.c_double, C.c_uint64, C.c_int64, I32]
    L.eesd_host_ts_update.argtypes = [P(C.c_double), P(C.c_double), I32, I32, I32]
    L.eesd_set_calibration.argtypes = [VP, P(_Calibration)]
    L.eesd_cali_score.argtypes = [VP, P(C.c_float)]
    L.eesd_host_cali_decide.argtypes = [C.c_double, C.c_double, C.c_double, C.c_int64, C.c_double, C.c_uint64, C.c_int64, I32,
                                        P(C.c_double), P(I32)]
    L.eesd_host_cali_update.argtypes = [P(C.c_double), P(C.c_double), P(C.c_int64), I32, I32, I32]
    L.eesd_op_accept.argtypes = [VP, VP, VP, P(C.c_double), I32, I32, I32, VP, P(I32)]
    L.eesd_op_accept_logits.argtypes = [VP, I32, VP, VP, VP, P(C.c_double), I32, I32, C.c_float, VP, P(I32)]
    L.eesd_op_softmax_sample.argtypes = [VP, VP, I32, C.c_float, C.c_double, VP, P(I32)]
    L.eesd_op_gemm.argtypes = [VP, VP, VP, I32, I32, I32, I32, I32, I32, VP]
    L.eesd_op_gemm_noalloc.argtypes = [VP, VP, VP, I32, I32, I32, I32, VP]
    L.eesd_pack_weight.argtypes = [VP, VP, I32, I32, I32, I32, VP]
    for name in EXPORTS:
        if name not in ("eesd_destroy", "eesd_last_error", "eesd_host_uniform", "eesd_host_layout_offset"):
            getattr(L, name).restype = C.c_int
    _LIB = L
    return L


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _ptr(arr: np.ndarray, ct):
    return arr.ctypes.data_as(C.POINTER(ct))


def host_uniform(seed: int, stream: int, rnd: int, slot: int = 0, sub: int = 0) -> float:
    return lib().eesd_host_uniform(seed, stream, rnd, slot, sub)


def host_layout_offset(what: int, a: int, b: int, n: int) -> int:
    return lib().eesd_host_layout_offset(what, a, b, n)


def host_draw_k(alpha: float, beta: float, seed: int, rnd: int, k_max: int) -> int:
    k = lib().eesd_host_draw_k(alpha, beta, seed, rnd, k_max)
    if k < 1:
        raise EesdError(k, "eesd_host_draw_k")
    return k


def host_ts_update(alpha: float, beta: float, n_accepted: int, n_drafted: int, reading: int = 0):
    a, b = C.c_double(alpha), C.c_double(beta)
    rc = lib().eesd_host_ts_update(C.byref(a), C.byref(b), n_accepted, n_drafted, reading)
    if rc:
        raise EesdError(rc, "eesd_host_ts_update")
    return a.value, b.value


def host_cali_decide(sigma_m: float, sigma_s: float, theta_hat: float, n: int, theta_m: float, seed: int, rnd: int, slot: int):
    theta, chi = C.c_double(), C.c_int32()
    rc = lib().eesd_host_cali_decide(sigma_m, sigma_s, theta_hat, n, theta_m, seed, rnd, slot, C.byref(theta), C.byref(chi))
    if rc:
        raise EesdError(rc, "eesd_host_cali_decide")
    return theta.value, bool(chi.value)


def host_cali_update(theta_hat: float, weight: float, n: int, n_accepted: int, n_drafted: int, reading: int = 0):
    th, w, nn = C.c_double(theta_hat), C.c_double(weight), C.c_int64(n)
    rc = lib().eesd_host_cali_update(C.byref(th), C.byref(w), C.byref(nn), n_accepted, n_drafted, reading)
    if rc:
        raise EesdError(rc, "eesd_host_cali_update")
    return th.value, w.value, nn.value


def set_tunable(name: str, value: int) -> None:
    rc = lib().eesd_set_tunable(name.encode(), int(value))
    if rc:
        raise EesdError(rc, f"unknown tunable {name}")


class EESD:
    """One decoding context.  `weights` is the dict layout of synth_inputs.make_weights with
    torch tensors on the GPU; the tensors are borrowed by the library and kept alive here."""

    def __init__(self, weights: dict, max_seq: int, temperature: float, seed: int = 0, k_cap: int = 10,
                 kv_page: int = 16, alpha0: float = 1.0, beta0: float = 1.0, ts_mode: int = TS_BETA,
                 ts_update: int = 0, gemm_path: int = GEMM_AUTO, stream: int = 0, tree_width: int = 0, verify_reuse: int = 0, weight_layout: int = WEIGHTS_ROW_MAJOR,
                 logits_bf16: int = 0):
        sh = weights["shape"]
        self._keep = weights
        self.shape = sh
        self.vocab = sh["vocab"]
        cfg = _Config(sh["n_layers"], sh["n_draft_layers"], sh["d_model"], sh["n_heads"], sh["n_kv_heads"], sh["head_dim"],
                      sh["d_ff"], sh["vocab"], sh["rms_eps"], sh["rope_base"], DTYPE_BF16 if sh["dtype"] == "bf16" else DTYPE_F32,
                      max_seq, kv_page, k_cap, temperature, seed, alpha0, beta0, ts_mode, ts_update, gemm_path, tree_width, verify_reuse, weight_layout,
                      logits_bf16)

        def lw(d):
            return _Layer(*[d[k].data_ptr() for k in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")])
        self._layers = (_Layer * sh["n_layers"])(*[lw(l) for l in weights["layers"]])
        w = _Weights(weights["tok_emb"].data_ptr(), self._layers, weights["final_norm"].data_ptr(), weights["lm_head"].data_ptr(),
                     lw(weights["ee_layer"]), weights["ee_norm"].data_ptr(), weights["ee_head"].data_ptr())
        self._h = C.c_void_p()
        rc = lib().eesd_create(C.byref(cfg), C.byref(w), C.c_void_p(stream), C.byref(self._h))
        if rc:
            self._h = None
            raise EesdError(rc, "eesd_create")
        self.k_cap = k_cap
        self.tree_width = tree_width

    def close(self):
        if getattr(self, "_h", None):
            lib().eesd_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except TypeError:       # interpreter shutdown: the module's globals are already gone, the process frees the context
            pass

    def _ck(self, rc: int):
        if rc:
            raise EesdError(rc, lib().eesd_last_error(self._h).decode())

    # the calls of a round -------------------------------------------------------------------
    def prefill(self, prompt) -> int:
        p = _i32(prompt)
        tok = C.c_int32()
        self._ck(lib().eesd_prefill(self._h, _ptr(p, C.c_int32), len(p), C.byref(tok)))
        return tok.value

    def draft_step(self, sync: bool = True) -> Optional[int]:
        if not sync:
            self._ck(lib().eesd_draft_step(self._h, None))
            return None
        tok = C.c_int32()
        self._ck(lib().eesd_draft_step(self._h, C.byref(tok)))
        return tok.value

    def verify(self) -> None:
        self._ck(lib().eesd_verify(self._h))

    def accept(self, uniforms: Optional[Sequence[float]] = None):
        a, y = C.c_int32(), C.c_int32()
        if uniforms is None:
            self._ck(lib().eesd_accept(self._h, None, C.byref(a), C.byref(y)))
        else:
            u = np.ascontiguousarray(np.asarray(uniforms, dtype=np.float64))
            self._ck(lib().eesd_accept(self._h, _ptr(u, C.c_double), C.byref(a), C.byref(y)))
        return a.value, y.value

    def accepted_tokens(self) -> List[int]:
        toks = np.zeros(16, np.int32)
        n = C.c_int32()
        self._ck(lib().eesd_accepted_tokens(self._h, _ptr(toks, C.c_int32), 16, C.byref(n)))
        return toks[: n.value].tolist()

    def rollback(self, n_accepted: int) -> None:
        self._ck(lib().eesd_rollback(self._h, int(n_accepted)))

    def rollback_forced(self, n_accepted: int, pending: int) -> None:
        """Test hook (teacher forcing): keep any number of drafts and continue from a token of the caller's choice."""
        self._ck(lib().eesd_debug_rollback(self._h, int(n_accepted), int(pending)))

    def generate(self, prompt, max_new: int):
        p = _i32(prompt)
        out = np.zeros(max_new, np.int32)
        n = C.c_int32()
        st = _Stats()
        self._ck(lib().eesd_generate(self._h, _ptr(p, C.c_int32), len(p), max_new, _ptr(out, C.c_int32), C.byref(n), C.byref(st)))
        return out[: n.value].tolist(), Stats(*[getattr(st, f[0]) for f in _Stats._fields_])

    def stats(self) -> Stats:
        st = _Stats()
        self._ck(lib().eesd_get_stats(self._h, C.byref(st)))
        return Stats(*[getattr(st, f[0]) for f in _Stats._fields_])

    # controller ---------------------------------------------------------------------------------
    def set_draft_schedule(self, ks) -> None:
        k = _i32(ks)
        self._ck(lib().eesd_set_draft_schedule(self._h, _ptr(k, C.c_int32), len(k)))

    def set_calibration(self, cw: dict, sigma_m: float, sigma_s: float, theta_hat0: float, update: int = 0) -> None:
        """cw: {"w": [n_mats][d][d], "wp": [2][2d]} torch tensors on the GPU in the model's dtype (borrowed, kept alive here)."""
        self._cali_keep = cw
        cal = _Calibration(cw["w"].data_ptr(), cw["wp"].data_ptr(), int(cw["w"].shape[0]), update, sigma_m, sigma_s, theta_hat0)
        self._ck(lib().eesd_set_calibration(self._h, C.byref(cal)))

    def cali_score(self) -> float:
        th = C.c_float()
        self._ck(lib().eesd_cali_score(self._h, C.byref(th)))
        return th.value

    def cali_state(self):
        a = self._read(READ_CALI_STATE, 0, 0, np.empty(3, np.float64))
        return float(a[0]), float(a[1]), int(a[2])

    def next_draft_len(self, k_max: int) -> int:
        k = C.c_int32()
        self._ck(lib().eesd_next_draft_len(self._h, k_max, C.byref(k)))
        return k.value

    # hooks ---------------------------------------------------------------------------------------
    def force_drafts(self, toks) -> None:
        t = _i32(toks)
        self._ck(lib().eesd_debug_force_drafts(self._h, _ptr(t, C.c_int32), len(t)))

    def force_pending(self, tok: int) -> None:
        self._ck(lib().eesd_debug_force_pending(self._h, int(tok)))

    def fill_cache(self, n_tokens: int, pending: int = 1) -> None:
        self._ck(lib().eesd_debug_fill_cache(self._h, int(n_tokens), int(pending)))

    def profile_begin(self, family: int, epilogue_kind: int, in_dim: int = 0) -> None:
        self._ck(lib().eesd_debug_profile_begin(self._h, family, epilogue_kind, in_dim))

    def profile_end(self):
        n, ms = C.c_int32(), C.c_double()
        self._ck(lib().eesd_debug_profile_end(self._h, C.byref(n), C.byref(ms)))
        return n.value, ms.value

    def _read(self, what: int, index: int, n_tokens: int, arr: np.ndarray) -> np.ndarray:
        self._ck(lib().eesd_debug_read(self._h, what, index, n_tokens, arr.ctypes.data_as(C.c_void_p), arr.nbytes))
        return arr

    def draft_logits(self, slot: int) -> np.ndarray:
        return self._read(READ_DRAFT_LOGITS, slot, 0, np.empty(self.vocab, np.float32))

    def draft_probs(self, slot: int) -> np.ndarray:
        return self._read(READ_DRAFT_PROBS, slot, 0, np.empty(self.vocab, np.float32))

    def verify_logits(self, row: int) -> np.ndarray:
        return self._read(READ_VERIFY_LOGITS, row, 0, np.empty(self.vocab, np.float32))

    def verify_probs(self, row: int) -> np.ndarray:
        return self._read(READ_VERIFY_PROBS, row, 0, np.empty(self.vocab, np.float32))

    def launch_counts(self) -> np.ndarray:
        """[kernel][epilogue] launches: kernel 0 VALU, 1 per-tile, 2 per-group, 3 LDS-shared tiles, 4 prefill GEMM; epilogue 0 head, 1 residual, 2 SwiGLU, 3 QKV."""
        return self._read(READ_LAUNCH_COUNTS, 0, 0, np.empty(20, np.int32)).reshape(5, 4)

    def kv(self, cache: int, n_tokens: int):
        sh = self.shape
        k = self._read(READ_KV_K, cache, n_tokens, np.empty((n_tokens, sh["n_kv_heads"], sh["head_dim"]), np.float32))
        v = self._read(READ_KV_V, cache, n_tokens, np.empty((n_tokens, sh["n_kv_heads"], sh["head_dim"]), np.float32))
        return k, v

    def kv_len(self) -> int:
        return int(self._read(READ_KV_LEN, 0, 0, np.empty(1, np.int32))[0])

    def block_tokens(self, n: int) -> List[int]:
        return self._read(READ_TOKENS, 0, 0, np.empty(n, np.int32)).tolist()

    def tree_tokens(self, n: int) -> List[int]:
        return self._read(READ_TREE_TOKENS, 0, 0, np.empty(n, np.int32)).tolist()

    def page_table(self, n_pages: int) -> List[int]:
        return self._read(READ_PAGE_TABLE, 0, 0, np.empty(n_pages, np.int32)).tolist()


# stand-alone kernels: torch tensors on the GPU in, Python values out ------------------------------
def op_accept(p_rows, q_rows, drafts, uniforms, greedy: bool, stream: int = 0):
    K = int(drafts.numel())
    V = int(p_rows.shape[-1])
    res = np.zeros(2, np.int32)
    u = np.ascontiguousarray(np.asarray(uniforms if uniforms is not None else np.zeros(K + 1), dtype=np.float64))
    rc = lib().eesd_op_accept(p_rows.data_ptr(), q_rows.data_ptr() if q_rows is not None else None, drafts.data_ptr(),
                              _ptr(u, C.c_double), K, V, int(greedy), C.c_void_p(stream), _ptr(res, C.c_int32))
    if rc:
        raise EesdError(rc, "eesd_op_accept")
    return int(res[0]), int(res[1])


def op_accept_logits(p_logits, p_rows, q_rows, drafts, uniforms, temperature: float, stream: int = 0):
    """p_logits: [K+1][V] fp32 or bfloat16 torch tensor on the GPU; p_rows: fp32 [K+1][V] output (None when greedy)."""
    import torch
    K = int(drafts.numel())
    V = int(p_logits.shape[-1])
    res = np.zeros(2, np.int32)
    u = np.ascontiguousarray(np.asarray(uniforms if uniforms is not None else np.zeros(K + 1), dtype=np.float64))
    rc = lib().eesd_op_accept_logits(p_logits.data_ptr(), int(p_logits.dtype == torch.bfloat16), p_rows.data_ptr() if p_rows is not None else None,
                                     q_rows.data_ptr() if q_rows is not None else None, drafts.data_ptr(), _ptr(u, C.c_double), K, V,
                                     float(temperature), C.c_void_p(stream), _ptr(res, C.c_int32))
    if rc:
        raise EesdError(rc, "eesd_op_accept_logits")
    return int(res[0]), int(res[1])


def op_softmax_sample(logits, probs, temperature: float, u: float, stream: int = 0) -> int:
    tok = C.c_int32()
    rc = lib().eesd_op_softmax_sample(logits.data_ptr(), probs.data_ptr() if probs is not None else None, int(logits.numel()),
                                      float(temperature), float(u), C.c_void_p(stream), C.byref(tok))
    if rc:
        raise EesdError(rc, "eesd_op_softmax_sample")
    return tok.value


def calibration_copy(dst, src, stream: int = 0) -> None:
    rc = lib().eesd_debug_copy(dst.data_ptr(), src.data_ptr(), src.numel() * src.element_size(), C.c_void_p(stream))
    if rc:
        raise EesdError(rc, "eesd_debug_copy")


def op_gemm(W, X, Y, path: int = GEMM_AUTO, stream: int = 0, weight_layout: int = WEIGHTS_ROW_MAJOR) -> None:
    import torch
    M, inn = X.shape
    out = W.shape[0]
    dt = DTYPE_BF16 if W.dtype == torch.bfloat16 else DTYPE_F32
    rc = lib().eesd_op_gemm(W.data_ptr(), X.data_ptr(), Y.data_ptr(), M, out, inn, dt, path, weight_layout, C.c_void_p(stream))
    if rc:
        raise EesdError(rc, "eesd_op_gemm")


def op_gemm_noalloc(W, X, Y, stream: int = 0, weight_layout: int = WEIGHTS_ROW_MAJOR) -> None:
    M, inn = X.shape
    rc = lib().eesd_op_gemm_noalloc(W.data_ptr(), X.data_ptr(), Y.data_ptr(), M, W.shape[0], inn, weight_layout, C.c_void_p(stream))
    if rc:
        raise EesdError(rc, "eesd_op_gemm_noalloc")


def pack_weight(W, kind: int = PACK_PLAIN, head_dim: int = 0, stream: int = 0):
    """Tile-major copy of one bf16 matrix [out][in] (same shape and dtype; the library's kernel does the
    rearranging, torch only owns the new buffer)."""
    import torch
    assert W.dtype == torch.bfloat16 and W.is_contiguous() and W.dim() == 2
    dst = torch.empty_like(W)
    rc = lib().eesd_pack_weight(W.data_ptr(), dst.data_ptr(), W.shape[0], W.shape[1], kind, head_dim, C.c_void_p(stream))
    if rc:
        raise EesdError(rc, "eesd_pack_weight")
    return dst


def pack_weights(weights: dict) -> dict:
    """All matrices of a model dict in the tile-major layout (EESD(..., weight_layout=WEIGHTS_TILED)).
    Matrix by matrix, dropping this function's reference to each original as it goes, so a caller who
    gives up its own dict needs room for the model plus one matrix."""
    hd = weights["shape"]["head_dim"]
    out = dict(shape=dict(weights["shape"]), tok_emb=weights["tok_emb"], final_norm=weights["final_norm"], ee_norm=weights["ee_norm"])

    def layer(l):
        return dict(attn_norm=l["attn_norm"], ffn_norm=l["ffn_norm"], wqkv=pack_weight(l["wqkv"], PACK_QKV, hd), wo=pack_weight(l["wo"]),
                    w_gate_up=pack_weight(l["w_gate_up"], PACK_GATE_UP), w_down=pack_weight(l["w_down"]))
    out["layers"] = []
    layers = weights["layers"]
    for i in range(len(layers)):
        out["layers"].append(layer(layers[i]))
        layers[i] = None          # the caller's list gives the original up as well
    weights["layers"] = []
    out["ee_layer"] = layer(weights.pop("ee_layer"))
    out["lm_head"] = pack_weight(weights.pop("lm_head"))
    out["ee_head"] = pack_weight(weights.pop("ee_head"))
    return out


def pack_calibration(cw: dict) -> dict:
    import torch
    return dict(w=torch.stack([pack_weight(cw["w"][i].contiguous()) for i in range(cw["w"].shape[0])]), wp=cw["wp"])
