"""CPU oracle for Early-exiting Speculative Decoding (EESD).

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, fp64 numpy implementation
of what one EESD decoding round computes, written from the paper so that the
HIP library can be checked against it.  Nothing in the product path may
import it; it imports nothing from the product path.

What follows which passage of the paper:

* decoder layer / target forward ......... the LLaMA decoder the paper builds on
  (Section 3.1 names it and its RMSNorm; Section 4.1 lists the models)
* draft forward .......................... Section 3.1, Eq. 1: first-N layers of the
  target (shared weights and shared KV cache), one extra decoder layer, RMSNorm, head W
* drafting loop, verification, commit .... Algorithm 1 (steps 4-17)
* greedy acceptance ...................... footnote of Section 4.1 ("Evaluation stage")
* stochastic acceptance / resampling ..... the speculative-sampling rule of the works
  cited in Section 1 and Section 2 ("Efficient Decoding"); Abstract: the verified
  output keeps the distribution of auto-regressive decoding
* Beta posterior controller .............. Section 3.3 Eq. 2-4 and Algorithm 2 (Appendix A)
* v_d, r_d, harmonic mean, speed model ... Section 4.1 "Metrics", Appendix D
* calibrated controller .................. Section 3.3 "TS with Calibration", Eq. 5-8,
  Algorithm 3 and the posterior derived in Appendix B
* tree of draft candidates ............... Section 4.3 "Implement Tree Attention" and the
  caption of its table (a candidate is kept only if it is the target's top-1 token);
  the tree's shape is this file's reading, stated at OracleEESDTree

Pins (tests/test_oracle_*.py): exact enumeration of the output distribution
on a tiny vocabulary, greedy speculative == greedy auto-regressive, block
verification == sequential single-token forwards, rollback == never drafted,
the transformer against an independent library implementation of the LLaMA
decoder, closed forms of the Beta posterior, published vectors of the
counter hash; for the candidate tree (tests/test_oracle_tree_pins.py): brute force
over all root paths, equality with greedy auto-regressive decoding, from-scratch
forwards of every path, caches after rollback; for the calibrated controller
(tests/test_oracle_cali_pins.py): the posterior against numerical Bayes on a grid,
the normal variates against the normal law, the predictor against a library
two-class softmax, the running mean against a plain mean.  Per-seed sampled token streams at temperature 1 are fixed by
nothing but this file: "parity unpinned" by the paper for those.

Storage is float32 only where a value is *input data* (weights) or where the
method's decision is defined on fp32 probability rows (see decide_*); all
arithmetic is float64.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64

# ---------------------------------------------------------------------------
# counter-based uniforms
# ---------------------------------------------------------------------------
# Every random number the method draws is a pure function of
# (seed, stream, round, slot, sub): the splitmix64 output function applied to a
# 64-bit key.  Integer-only, so any implementation gives the same bits.

STREAM_DRAFT, STREAM_ACCEPT, STREAM_RESAMPLE, STREAM_TS_THETA, STREAM_TS_CHI = 1, 2, 3, 4, 5
_M64 = (1 << 64) - 1


def splitmix64(state: int) -> int:
    """One output of the splitmix64 generator whose state before the step is `state`."""
    z = (state + 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def uniform(seed: int, stream: int, rnd: int, slot: int = 0, sub: int = 0) -> float:
    """u in [0,1) on the 53-bit grid."""
    key = (seed ^ ((stream & 0xFF) << 56) ^ ((rnd & 0xFFFFFF) << 32) ^ ((slot & 0xFF) << 24) ^ (sub & 0xFFFFFF)) & _M64
    return (splitmix64(key) >> 11) * 2.0 ** -53


# ---------------------------------------------------------------------------
# O1: the decoder layer
# ---------------------------------------------------------------------------

def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """x_j * g_j / sqrt(mean_j x_j^2 + eps), row-wise."""
    x = x.astype(F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x * g.astype(F64) / np.sqrt(ms + eps)


def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary position embedding on x[m][heads][hd]; pairs are (j, j + hd/2),
    angle of pair j at position p is p * base^(-2j/hd)."""
    m, nh, hd = x.shape
    half = hd // 2
    j = np.arange(half, dtype=F64)
    inv = base ** (-2.0 * j / hd)
    ang = pos.astype(F64)[:, None] * inv[None, :]          # [m][half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def softmax(z: np.ndarray) -> np.ndarray:
    z = z.astype(F64)
    z = z - np.max(z, axis=-1, keepdims=True)
    e = np.exp(z)
    return e / np.sum(e, axis=-1, keepdims=True)


class KVCache:
    """Keys and values of one decoder layer: arrays [max_seq][n_kv_heads][hd]."""

    def __init__(self, max_seq: int, n_kv: int, hd: int):
        self.k = np.zeros((max_seq, n_kv, hd), F64)
        self.v = np.zeros((max_seq, n_kv, hd), F64)


def attention_kv_rows(x: np.ndarray, pos: np.ndarray, w: dict, sh: dict) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """q (rotated), k (rotated), v of the rows x at positions pos."""
    H, Hkv, hd = sh["n_heads"], sh["n_kv_heads"], sh["head_dim"]
    h = rmsnorm(x, w["attn_norm"], sh["rms_eps"])
    qkv = h @ w["wqkv"].astype(F64).T
    m = x.shape[0]
    q = qkv[:, : H * hd].reshape(m, H, hd)
    k = qkv[:, H * hd: (H + Hkv) * hd].reshape(m, Hkv, hd)
    v = qkv[:, (H + Hkv) * hd:].reshape(m, Hkv, hd)
    return rope(q, pos, sh["rope_base"]), rope(k, pos, sh["rope_base"]), v


def decoder_layer(x: np.ndarray, pos: np.ndarray, kv: KVCache, w: dict, sh: dict) -> np.ndarray:
    """One pre-norm LLaMA decoder layer on rows x[m][d] at absolute positions
    pos[m]; appends their keys/values to kv at those positions and attends
    causally over positions 0..pos[i]."""
    H, Hkv, hd = sh["n_heads"], sh["n_kv_heads"], sh["head_dim"]
    grp = H // Hkv
    x = x.astype(F64)
    q, k, v = attention_kv_rows(x, pos, w, sh)
    kv.k[pos] = k
    kv.v[pos] = v
    m = x.shape[0]
    att = np.zeros((m, H, hd), F64)
    for i in range(m):
        n = int(pos[i]) + 1
        for hq in range(H):
            hk = hq // grp
            sc = kv.k[:n, hk, :] @ q[i, hq] / math.sqrt(hd)
            att[i, hq] = softmax(sc) @ kv.v[:n, hk, :]
    x = x + att.reshape(m, H * hd) @ w["wo"].astype(F64).T
    h2 = rmsnorm(x, w["ffn_norm"], sh["rms_eps"])
    gu = h2 @ w["w_gate_up"].astype(F64).T
    f = sh["d_ff"]
    x = x + (silu(gu[:, :f]) * gu[:, f:]) @ w["w_down"].astype(F64).T
    return x


# ---------------------------------------------------------------------------
# decisions on probability rows
# ---------------------------------------------------------------------------
# The paper's experiments are greedy; for temperature > 0 the rule is the
# speculative-sampling one.  A decision (which token, accept or not) is an
# integer decided by floating point, so its arithmetic is fixed here: rows are
# fp32 probabilities, products and running sums are fp64.

def argmax_lowest(row: np.ndarray) -> int:
    return int(np.argmax(row))          # numpy returns the first maximum


def decide_sample(r: np.ndarray, u: float) -> int:
    """Inverse-CDF draw from the non-negative fp32 weights r (need not sum to 1):
    the smallest j with C_j > u*S, C the fp64 running sum, S its total.
    Returns -1 when S == 0."""
    c = np.cumsum(r.astype(np.float32).astype(F64))
    s = c[-1]
    if not s > 0.0:
        return -1
    hit = np.nonzero(c > F64(u) * s)[0]
    if hit.size:
        return int(hit[0])
    return int(np.nonzero(r > 0)[0][-1])


def decide_accept(p_rows: np.ndarray, q_rows: Optional[np.ndarray], drafts: Sequence[int],
                  u_acc: Sequence[float], u_res: float, greedy: bool) -> Tuple[int, int]:
    """Verification outcome of one round.

    p_rows[i] (i = 0..K) is the target's distribution for the token after verify
    row i, so p_rows[i] judges drafts[i]; q_rows[i] is the draft distribution
    drafts[i] was drawn from.  Returns (a, y): a = number of leading drafts
    accepted, y = the token the target contributes after them.
    Greedy: keep drafts while they equal the target's top-1; y = top-1 of row a.
    Stochastic: accept drafts[i] iff u*q < p (i.e. with probability min(1,p/q));
    on the first rejection y ~ norm(max(0, p - q)); if all K pass, y ~ p_rows[K].
    """
    K = len(drafts)
    a = 0
    if greedy:
        while a < K and argmax_lowest(p_rows[a]) == int(drafts[a]):
            a += 1
        return a, argmax_lowest(p_rows[a])
    p32 = p_rows.astype(np.float32)
    q32 = q_rows.astype(np.float32) if K else None      # K = 0: a plain target step, no draft rows
    while a < K:
        d = int(drafts[a])
        if F64(u_acc[a]) * F64(q32[a, d]) < F64(p32[a, d]):
            a += 1
        else:
            break
    if a < K:
        resid = np.maximum(np.float32(0.0), p32[a] - q32[a])   # one fp32 subtraction per entry
        y = decide_sample(resid, u_res)
        if y < 0:                                               # p == q entrywise: cannot be rejected in exact arithmetic
            y = decide_sample(p32[a], u_res)
    else:
        y = decide_sample(p32[K], u_res)
    return a, y


# ---------------------------------------------------------------------------
# Beta-posterior Thompson-sampling controller (Section 3.3, Algorithm 2)
# ---------------------------------------------------------------------------

def beta_draw_int(alpha: int, beta: int, seed: int, rnd: int, slot: int) -> float:
    """theta ~ Beta(alpha, beta) for positive integers: the alpha-th smallest of
    alpha+beta-1 independent uniforms (an order statistic), which needs only
    comparisons of exactly representable numbers."""
    n = alpha + beta - 1
    us = sorted(uniform(seed, STREAM_TS_THETA, rnd, slot, j) for j in range(n))
    return us[alpha - 1]


class BetaTS:
    """Posterior Beta(alpha, beta) over the probability theta that drafting should go on."""

    def __init__(self, alpha0: float = 1.0, beta0: float = 1.0, seed: int = 0, update: str = "prose"):
        self.alpha, self.beta, self.seed, self.update_mode = alpha0, beta0, seed, update

    def draw_k(self, rnd: int, k_max: int) -> int:
        """Algorithm 2, steps 5-14: draft, draw theta from the current posterior,
        draw chi ~ Bernoulli(theta), stop on chi = 0.  The posterior is that of
        the round's start for every draw, so K depends on nothing the drafts produce."""
        k = 0
        while True:
            k += 1
            if k >= k_max:
                return k_max
            a, b = self.alpha, self.beta
            if float(a).is_integer() and float(b).is_integer():
                theta = beta_draw_int(int(a), int(b), self.seed, rnd, k)
            else:
                raise ValueError("oracle controller draws Beta only for integer parameters")
            chi = uniform(self.seed, STREAM_TS_CHI, rnd, k) < theta
            if not chi:
                return k

    def update(self, n_accepted: int, n_drafted: int) -> None:
        """Eq. 3-4: alpha += r, beta += n - r, r successes out of n judged drafts.
        'prose' reading: the target judged the a accepted drafts and, if one was
        rejected, that one: r = a, n = min(a + 1, K).  'literal' reading takes
        |Q_v| = a + 1 in r = |Q_v| - 1, n = min(|Q_v| + 1, |Q_d|)."""
        a, K = n_accepted, n_drafted
        r = a
        n = min(a + 1, K) if self.update_mode == "prose" else max(r, min(a + 2, K))
        self.alpha += r
        self.beta += n - r


# ---------------------------------------------------------------------------
# Thompson sampling with calibration (Section 3.3 "TS with Calibration", Eq. 5-8, Algorithm 3)
# ---------------------------------------------------------------------------

def normal_draw(seed: int, rnd: int, slot: int) -> float:
    """Standard normal variate from two counter-based uniforms (Box-Muller, cosine branch).
    math.* are the C library's routines, which the library's host code calls too."""
    u1 = uniform(seed, STREAM_TS_THETA, rnd, slot, 0)
    u2 = uniform(seed, STREAM_TS_THETA, rnd, slot, 1)
    return math.sqrt(-2.0 * math.log(1.0 - u1)) * math.cos(2.0 * math.pi * u2)


def cali_theta_m(cw: dict, h_target: np.ndarray, h_draft: np.ndarray, i: int) -> float:
    """Eq. 5: theta_M = Sigmoid(W_p (W^i H_t^(T), H_{t+i}^(D))), i clipped to the number of W^i.
    W_p has two rows and was trained with cross-entropy on chi in {0, 1}: the score is the
    probability of class 1, i.e. the logistic function of the difference of the two outputs."""
    W = cw["w"][min(i, cw["w"].shape[0]) - 1].astype(F64)
    u = W @ h_target.astype(F64)
    z = cw["wp"].astype(F64) @ np.concatenate([u, h_draft.astype(F64)])
    return 1.0 / (1.0 + math.exp(-(float(z[1]) - float(z[0]))))


class CaliTS:
    """Gaussian posterior over theta: prior N(theta_M, sigma_M^2) from the predictor, n
    verifications whose sample mean theta_hat has variance sigma_S^2 each (Eq. 6-7)."""

    def __init__(self, sigma_m: float, sigma_s: float, theta_hat0: float, seed: int = 0, update: str = "judged"):
        self.sigma_m, self.sigma_s, self.seed, self.update_mode = float(sigma_m), float(sigma_s), seed, update
        self.theta_hat = float(theta_hat0)
        self.n = 0            # verifications so far
        self.weight = 1.0     # observations behind theta_hat; theta_hat0 counts as one (the "+1" of Eq. 8)

    def posterior(self, theta_m: float) -> Tuple[float, float]:
        sm2, ss2, n = self.sigma_m ** 2, self.sigma_s ** 2, self.n
        mu = ss2 / (n * sm2 + ss2) * theta_m + n * sm2 / (n * sm2 + ss2) * self.theta_hat
        var = sm2 * ss2 / (ss2 + n * sm2)
        return mu, var

    def decide(self, theta_m: float, rnd: int, slot: int) -> Tuple[float, bool]:
        """Algorithm 3, steps 9-12: theta ~ N(mu, sigma^2), chi ~ Bernoulli(theta) (theta <= 0
        never goes on, theta >= 1 always does)."""
        mu, var = self.posterior(theta_m)
        theta = mu + math.sqrt(var) * normal_draw(self.seed, rnd, slot)
        return theta, uniform(self.seed, STREAM_TS_CHI, rnd, slot) < theta

    def update(self, n_accepted: int, n_drafted: int) -> None:
        """Algorithm 3, steps 21-22.  theta_hat is the observed mean of chi.  Eq. 8 as printed adds
        |Q_v| successes for |Q_v| new observations, so it can only rise; 'judged' (default) counts
        what the target judged, as the Beta controller does: a successes out of min(a + 1, K)
        observations.  'printed' keeps the printed form with |Q_v| = a."""
        a, K = n_accepted, n_drafted
        self.n += 1
        new = min(a + 1, K) if self.update_mode == "judged" else a
        if new:
            self.theta_hat = (self.theta_hat * self.weight + a) / (self.weight + new)
            self.weight += new


# ---------------------------------------------------------------------------
# statistics (Section 4.1 "Metrics", Appendix D)
# ---------------------------------------------------------------------------

def harmonic_mean_pct(v_d: float, r_d: float) -> float:
    return 0.0 if v_d + r_d == 0 else 2.0 * v_d * r_d / (v_d + r_d) * 100.0


def predicted_time(L: int, v_d: float, r_d: float, t_draft: float, t_target: float) -> float:
    """Appendix D: time to produce L tokens given per-token draft and target times."""
    return r_d * L / v_d * t_draft + (1.0 - r_d) * L * t_target


def predicted_speedup(v_d: float, r_d: float, alpha: float) -> float:
    """Appendix D closed form with alpha = T_d / T_t."""
    return v_d / ((alpha - v_d) * r_d + v_d)


@dataclass
class Stats:
    rounds: int = 0
    drafted: int = 0        # N_all_draft
    accepted: int = 0       # N_right
    generated: int = 0      # L

    @property
    def v_d(self) -> float:
        return self.accepted / self.drafted if self.drafted else 0.0

    @property
    def r_d(self) -> float:
        return self.accepted / self.generated if self.generated else 0.0


# ---------------------------------------------------------------------------
# the model state and the calls of a round
# ---------------------------------------------------------------------------

class OracleEESD:
    """One sequence (batch 1).  Mirrors the call sequence of the library:
    prefill -> (draft_step)^K -> verify -> accept -> rollback -> ...

    weights: dict of fp32 numpy arrays, every matrix [out][in]:
      tok_emb, layers[l]{attn_norm,wqkv,wo,ffn_norm,w_gate_up,w_down}, final_norm,
      lm_head, ee_layer{...}, ee_norm, ee_head.
    """

    def __init__(self, weights: dict, max_seq: int, temperature: float, seed: int = 0,
                 k_cap: int = 10, alpha0: float = 1.0, beta0: float = 1.0, ts_update: str = "prose"):
        self.w = weights
        self.sh = sh = weights["shape"]
        self.L, self.N = sh["n_layers"], sh["n_draft_layers"]
        self.T = float(temperature)
        self.greedy = self.T == 0.0
        self.seed, self.k_cap, self.max_seq = seed, k_cap, max_seq
        # L target caches (the first N are also the draft model's) + the early-exit layer's own
        self.kv = [KVCache(max_seq, sh["n_kv_heads"], sh["head_dim"]) for _ in range(self.L)]
        self.ee_kv = KVCache(max_seq, sh["n_kv_heads"], sh["head_dim"])
        self.kv_len = 0
        self.pending: Optional[int] = None
        self.rnd = 0
        self.drafts: List[int] = []
        self.q_rows: List[np.ndarray] = []
        self.q_logits: List[np.ndarray] = []
        self.p_rows: Optional[np.ndarray] = None
        self.p_logits: Optional[np.ndarray] = None
        self.ts = BetaTS(alpha0, beta0, seed, ts_update)
        self.stats = Stats()

    # -- forwards ----------------------------------------------------------
    def _probs(self, logits: np.ndarray) -> np.ndarray:
        """softmax(logits / T), stored as the fp32 rows decisions are taken on."""
        return softmax(logits / self.T).astype(np.float32)

    def _ee_kv_fill(self, h_n: np.ndarray, pos: np.ndarray) -> None:
        # The early-exit layer's key/value at a position depend only on that
        # position's layer-N hidden state, so whoever computes that state for a
        # committed-or-candidate token also records them.
        _, k, v = attention_kv_rows(h_n, pos, self.w["ee_layer"], self.sh)
        self.ee_kv.k[pos] = k
        self.ee_kv.v[pos] = v

    def target_forward(self, tokens: Sequence[int], pos0: int) -> np.ndarray:
        """All L layers on the block `tokens` at positions pos0.. ; returns logits [m][V]."""
        pos = np.arange(pos0, pos0 + len(tokens))
        x = self.w["tok_emb"][np.asarray(tokens)].astype(F64)
        for l in range(self.L):
            x = decoder_layer(x, pos, self.kv[l], self.w["layers"][l], self.sh)
            if l + 1 == self.N:
                self._ee_kv_fill(x, pos)
        self.h_target_rows = x.copy()      # last-layer hidden states of the block (H^(T) of Eq. 5)
        h = rmsnorm(x, self.w["final_norm"], self.sh["rms_eps"])
        return h @ self.w["lm_head"].astype(F64).T

    def draft_forward(self, token: int, pos: int) -> np.ndarray:
        """Eq. 1: H^N from the first N layers (shared caches), the early-exit layer
        on top, RMSNorm, head W; returns draft logits [V]."""
        p = np.array([pos])
        x = self.w["tok_emb"][[token]].astype(F64)
        for l in range(self.N):
            x = decoder_layer(x, p, self.kv[l], self.w["layers"][l], self.sh)
        x = decoder_layer(x, p, self.ee_kv, self.w["ee_layer"], self.sh)
        self.h_draft = x[0].copy()         # last-layer hidden state of the draft model (H^(D) of Eq. 5)
        h = rmsnorm(x, self.w["ee_norm"], self.sh["rms_eps"])
        return (h @ self.w["ee_head"].astype(F64).T)[0]

    # -- the calls -----------------------------------------------------------
    def prefill(self, prompt: Sequence[int]) -> int:
        self.kv_len, self.rnd = 0, 0
        self.drafts, self.q_rows, self.q_logits = [], [], []
        logits = self.target_forward(prompt, 0)
        self.kv_len = len(prompt)
        self.prefill_logits = logits[-1]
        if self.greedy:
            tok = argmax_lowest(logits[-1].astype(np.float32))
        else:
            tok = decide_sample(self._probs(logits[-1]), uniform(self.seed, STREAM_RESAMPLE, 0))
        self.pending = tok
        self.rnd = 1
        return tok

    def draft_step(self, force_token: Optional[int] = None) -> int:
        """Algorithm 1 step 6: x_i from the draft model given everything so far."""
        i = len(self.drafts)
        tok_in = self.pending if i == 0 else self.drafts[-1]
        logits = self.draft_forward(tok_in, self.kv_len + i)
        self.q_logits.append(logits)
        if self.greedy:
            d = argmax_lowest(logits.astype(np.float32))
            self.q_rows.append(None)
        else:
            q = self._probs(logits)
            d = decide_sample(q, uniform(self.seed, STREAM_DRAFT, self.rnd, i))
            self.q_rows.append(q)
        if force_token is not None:
            d = int(force_token)
        self.drafts.append(d)
        return d

    def verify(self) -> np.ndarray:
        """Algorithm 1 step 15: one target forward over [pending, d_1..d_K]."""
        block = [self.pending] + self.drafts
        self.p_logits = self.target_forward(block, self.kv_len)
        self.p_rows = self.p_logits.astype(np.float32) if self.greedy else self._probs(self.p_logits)
        return self.p_logits

    def accept(self, u_acc: Optional[Sequence[float]] = None, u_res: Optional[float] = None) -> Tuple[int, int]:
        K = len(self.drafts)
        if u_acc is None:
            u_acc = [uniform(self.seed, STREAM_ACCEPT, self.rnd, i) for i in range(K)]
        if u_res is None:
            u_res = uniform(self.seed, STREAM_RESAMPLE, self.rnd)
        q = None if (self.greedy or K == 0) else np.stack(self.q_rows)
        self.last = decide_accept(self.p_rows, q, self.drafts, u_acc, u_res, self.greedy)
        return self.last

    def rollback(self, n_accepted: int, next_token: int) -> None:
        """Keep the accepted prefix: the caches of all L layers and of the early-exit
        layer are valid up to kv_len + a + 1 (the pending token and a drafts)."""
        K = len(self.drafts)
        self.kv_len += n_accepted + 1
        self.pending = int(next_token)
        self.ts.update(n_accepted, K)
        self.stats.rounds += 1
        self.stats.drafted += K
        self.stats.accepted += n_accepted
        self.drafts, self.q_rows, self.q_logits = [], [], []
        self.rnd += 1

    # -- the whole loop (Algorithm 1) --------------------------------------------
    def generate(self, prompt: Sequence[int], max_new: int, k_schedule: Optional[Sequence[int]] = None,
                 fixed_k: Optional[int] = None, trace: Optional[list] = None) -> List[int]:
        out = [self.prefill(prompt)]
        r = 0
        while len(out) < max_new:
            k_max = min(self.k_cap, max_new - len(out))
            if k_schedule is not None:
                K = min(int(k_schedule[r]), k_max)
            elif fixed_k is not None:
                K = min(fixed_k, k_max)
            else:
                K = self.ts.draw_k(self.rnd, k_max)
            for _ in range(K):
                self.draft_step()
            self.verify()
            a, y = self.accept()
            committed = self.drafts[:a] + [y]
            if trace is not None:
                trace.append(dict(K=K, a=a, y=y, drafts=list(self.drafts), q_logits=list(self.q_logits),
                                  p_logits=self.p_logits.copy(), base=self.kv_len))
            self.rollback(a, y)
            out.extend(committed)
            r += 1
        out = out[:max_new]
        self.stats.generated = len(out)
        return out

    def generate_cali(self, prompt: Sequence[int], max_new: int, cw: dict, cali: "CaliTS",
                      trace: Optional[list] = None) -> List[int]:
        """Algorithm 3: after every draft token the predictor scores the draft model's hidden
        state against the target's hidden state at the last verified position, and the
        calibrated posterior decides whether to draft on."""
        out = [self.prefill(prompt)]
        h_t = self.h_target_rows[-1]
        while len(out) < max_new:
            k_max = min(self.k_cap, max_new - len(out))
            k, scores = 0, []
            while True:
                self.draft_step()
                k += 1
                if k >= k_max:
                    break
                theta_m = cali_theta_m(cw, h_t, self.h_draft, k)
                theta, chi = cali.decide(theta_m, self.rnd, k)
                scores.append((theta_m, theta, chi))
                if not chi:
                    break
            self.verify()
            a, y = self.accept()
            if trace is not None:
                trace.append(dict(K=k, a=a, y=y, drafts=list(self.drafts), scores=scores, n=cali.n, theta_hat=cali.theta_hat,
                                  base=self.kv_len, h_t=h_t))
            h_t = self.h_target_rows[a]        # the position whose output is the next pending token
            committed = self.drafts[:a] + [y]
            cali.update(a, k)
            self.rollback(a, y)
            out.extend(committed)
        out = out[:max_new]
        self.stats.generated = len(out)
        return out

    def ar_generate(self, prompt: Sequence[int], max_new: int, uniforms: Optional[Sequence[float]] = None) -> List[int]:
        """Vanilla auto-regressive decoding with the target model only."""
        logits = self.target_forward(prompt, 0)[-1]
        pos = len(prompt)
        out = []
        for t in range(max_new):
            if self.greedy:
                tok = argmax_lowest(logits.astype(np.float32))
            else:
                tok = decide_sample(self._probs(logits), uniforms[t])
            out.append(tok)
            if t + 1 < max_new:
                logits = self.target_forward([tok], pos)[0]
                pos += 1
        return out


# ---------------------------------------------------------------------------
# tree of draft candidates (Section 4.3, "Implement Tree Attention")
# ---------------------------------------------------------------------------

def top_candidates(logits32: np.ndarray, c: int) -> List[int]:
    """The c highest entries of an fp32 row, highest first, equal values by lowest index."""
    order = np.lexsort((np.arange(logits32.shape[0]), -logits32.astype(np.float64)))
    return [int(t) for t in order[:c]]


def tree_walk(children: Sequence[Sequence[int]], top_of: Callable) -> Tuple[int, int, List[int]]:
    """Greedy acceptance over a tree of candidates.

    children[i] are the candidate tokens at depth i + 1; children[i][0] is the one the draft
    model went on from, the others are leaves.  top_of(path) is the target model's top-1 token
    after the committed text followed by `path` (a tuple of tokens).  A candidate is kept only
    if it IS the target's top-1 token (the caption of the tree-attention table), so the walk
    follows the target's own greedy continuation for as long as the tree contains it.
    Returns (a, y, branch): a accepted tokens, the next token y, and which child was taken at
    each accepted depth."""
    path: Tuple[int, ...] = ()
    branch: List[int] = []
    for kids in children:
        top = top_of(path)
        if top not in kids:
            return len(path), top, branch
        j = list(kids).index(top)
        path = path + (top,)
        branch.append(j)
        if j != 0:            # a leaf: nothing was drafted below it
            break
    return len(path), top_of(path), branch


class OracleEESDTree(OracleEESD):
    """EESD with several candidates per draft step, greedy decoding (temperature 0).

    Reading of Section 4.3 (the paper fixes neither the shape of the tree nor how it is
    grown): at every draft step the `width` most likely tokens of the draft distribution are
    candidates; the most likely one is extended by the next draft step, the others are leaves.
    The target model's output at a node is, by definition, its output on the committed text
    followed by the path to that node; this oracle evaluates exactly that, one path at a
    time, with no tree mask."""

    def __init__(self, weights: dict, max_seq: int, width: int, **kw):
        super().__init__(weights, max_seq, temperature=0.0, **kw)
        assert width >= 2
        self.width = width
        self.children: List[List[int]] = []

    def draft_step_tree(self, force: Optional[Sequence[int]] = None) -> List[int]:
        i = len(self.children)
        tok_in = self.pending if i == 0 else self.children[-1][0]
        logits = self.draft_forward(tok_in, self.kv_len + i)
        self.q_logits.append(logits)
        kids = top_candidates(logits.astype(np.float32), self.width)
        if force is not None:
            kids = [int(t) for t in force]
        self.children.append(kids)
        self.drafts.append(kids[0])
        return kids

    def node_logits(self) -> dict:
        """Target logits at every node: {(): row of the pending token, (i, j): child j at depth i}."""
        K = len(self.children)
        chain = [self.pending] + [kids[0] for kids in self.children]
        rows = {}
        # leaves, deepest first: a leaf at depth i overwrites cache position kv_len + i only,
        # which shallower nodes never look at
        full = self.target_forward(chain, self.kv_len)
        for i in range(K, 0, -1):
            for j in range(1, self.width):
                rows[(i, j)] = self.target_forward([self.children[i - 1][j]], self.kv_len + i)[0]
        full = self.target_forward(chain, self.kv_len)      # the chain's keys and values back in place
        rows[()] = full[0]
        for i in range(1, K + 1):
            rows[(i, 0)] = full[i]
        return rows

    def verify_accept_tree(self) -> Tuple[int, int, List[int]]:
        rows = self.node_logits()
        self.tree_logits = rows

        def top_of(path):
            if not path:
                return argmax_lowest(rows[()].astype(np.float32))
            i = len(path)
            j = self.children[i - 1].index(path[-1])
            return argmax_lowest(rows[(i, j)].astype(np.float32))

        self.last_tree = tree_walk(self.children, top_of)
        return self.last_tree

    def rollback_tree(self, a: int, y: int, branch: Sequence[int]) -> List[int]:
        """Commits the accepted path; returns its tokens.  The caches must hold the keys and
        values of the committed tokens: an accepted leaf is put where the chain token was."""
        K = len(self.children)
        toks = [self.children[i][branch[i]] for i in range(a)]
        if a and branch[a - 1] != 0:
            self.target_forward([toks[-1]], self.kv_len + a)
        self.kv_len += a + 1
        self.pending = int(y)
        self.ts.update(a, K)
        self.stats.rounds += 1
        self.stats.drafted += K
        self.stats.accepted += a
        self.children, self.drafts, self.q_rows, self.q_logits = [], [], [], []
        self.rnd += 1
        return toks

    def generate_tree(self, prompt: Sequence[int], max_new: int, fixed_k: Optional[int] = None,
                      k_schedule: Optional[Sequence[int]] = None, trace: Optional[list] = None) -> List[int]:
        out = [self.prefill(prompt)]
        r = 0
        while len(out) < max_new:
            k_max = min(self.k_cap, max_new - len(out))
            if k_schedule is not None:
                K = min(int(k_schedule[r]), k_max)
            elif fixed_k is not None:
                K = min(fixed_k, k_max)
            else:
                K = self.ts.draw_k(self.rnd, k_max)
            for _ in range(K):
                self.draft_step_tree()
            a, y, branch = self.verify_accept_tree()
            if trace is not None:
                trace.append(dict(K=K, a=a, y=y, branch=list(branch), children=[list(k) for k in self.children], base=self.kv_len))
            out.extend(self.rollback_tree(a, y, branch) + [y])
            r += 1
        out = out[:max_new]
        self.stats.generated = len(out)
        return out


# ---------------------------------------------------------------------------
# the round on abstract models (used to enumerate the output distribution)
# ---------------------------------------------------------------------------

def abstract_round(prefix: Tuple[int, ...], K: int, q_of: Callable, p_of: Callable,
                   u_draft: Sequence[float], u_acc: Sequence[float], u_res: float,
                   greedy: bool = False) -> Tuple[int, ...]:
    """One round of Algorithm 1 where the two models are given as functions
    prefix -> fp32 probability row.  Returns the tokens the round commits."""
    drafts, q_rows = [], []
    ctx = tuple(prefix)
    for i in range(K):
        q = q_of(ctx)
        d = argmax_lowest(q) if greedy else decide_sample(q, u_draft[i])
        drafts.append(d)
        q_rows.append(q)
        ctx = ctx + (d,)
    p_rows = np.stack([p_of(tuple(prefix) + tuple(drafts[:i])) for i in range(K + 1)])
    a, y = decide_accept(p_rows, np.stack(q_rows), drafts, u_acc, u_res, greedy)
    return tuple(drafts[:a]) + (y,)
