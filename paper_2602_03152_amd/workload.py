"""Seeded synthetic inputs for the FASA decode hot path.

This module only *draws inputs*: pre-RoPE Gaussian queries/keys/values, a random
dominant-FC list per KV head, a sparse set of salient tokens, the rotary position
encoding of the drawn vectors and the rounding to the storage dtype.  It holds none
of the method's own arithmetic (no scoring, no selection, no attention), so both the
CPU oracle's tests and the HIP path's tests/bench may feed from it.

The hot path consumes *post-RoPE* q and K (the paper's TIP/FAC stages, Sec. 4.1-4.2,
operate on the cached, already rotated keys), hence RoPE belongs to input synthesis.
Pairing convention: frequency chunk (FC) i is the rotation pair (dim i, dim i + d/2)
("rotate-half"), angular frequency theta_i = base^(-2 i / d), i = 0 .. d/2-1
(Sec. 3.1, FC definition; zero-based indices as in the I_dom definition of Sec. 4.1).

Storage: bf16 tensors are returned as numpy uint16 arrays holding the raw bf16 bit
patterns (round-to-nearest-even from float32); fp32 tensors as float32 arrays.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

SEED_BASE = 20260203 * 1000

# RNG stream ids (one independent PCG64 stream per tensor family)
_STREAM_Q, _STREAM_K, _STREAM_V, _STREAM_FC, _STREAM_SAL, _STREAM_APPEND = 0, 1, 2, 3, 4, 5


@dataclass(frozen=True)
class Workload:
    """Shape and recipe of one synthetic decode workload."""
    name: str
    config_id: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_fc: int            # F: dominant FCs per KV head (paper: N_tip)
    n_ctx: int           # N: cached tokens (paper: t)
    budget: int          # B: selected tokens per KV head (paper: N_fac)
    dtype: str           # "bf16" | "f32": storage type of q, K, V, Kp
    rope_base: float
    salient_frac: float
    fc_scale: float = 4.0

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    def scaled(self, **kw) -> "Workload":
        """Same recipe at another size (used for reduced parity cases)."""
        return replace(self, **kw)


def budget_fraction(n_ctx: int, frac: float = 0.189) -> int:
    """Token budget as a fixed share of the current context (long-CoT workload)."""
    return int(np.floor(frac * n_ctx))


WORKLOADS: Dict[int, Workload] = {
    0: Workload("tiny_1head_f32_n4096", 0, 1, 1, 1, 128, 16, 4096, 256, "f32", 1.0e4, 0.01),
    1: Workload("llama3_8b_layer_n32768_b2048", 1, 1, 32, 8, 128, 16, 32768, 2048, "bf16", 5.0e5, 0.01),
    2: Workload("batch16_n16384_b256", 2, 16, 32, 8, 128, 16, 16384, 256, "bf16", 5.0e5, 0.01),
    3: Workload("longcot_batch8_gqa7_n32768", 3, 8, 28, 4, 128, 16, 32768,
                budget_fraction(32768), "bf16", 1.0e6, 0.01),
    4: Workload("verylong_n131072_f32fc_b1024", 4, 1, 32, 8, 128, 32, 131072, 1024, "bf16", 5.0e5, 0.002),
}


def _rng(config_id: int, stream: int, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([SEED_BASE + 10 * config_id + stream, sub]))


# ----------------------------------------------------------------------------------
# dtype plumbing (no arithmetic of the method here)
# ----------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    x32 = np.asarray(x, dtype=np.float32)
    return f32_to_bf16_bits(x32) if dtype == "bf16" else np.ascontiguousarray(x32)


def storage_to_f64(x: np.ndarray) -> np.ndarray:
    """Exact widening of a storage array (uint16 bf16 bits or float32) to float64."""
    if x.dtype == np.uint16:
        return bf16_bits_to_f32(x).astype(np.float64)
    return x.astype(np.float64)


# ----------------------------------------------------------------------------------
# rotary position encoding of the drawn vectors (input synthesis)
# ----------------------------------------------------------------------------------
def rope_rotate_half(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotate `x[..., d]` at integer positions `pos` (broadcast over leading axes).

    FC i = (x[..., i], x[..., i + d/2]) is rotated by angle pos * base^(-2i/d):
        x'_i       = x_i cos - x_{i+d/2} sin
        x'_{i+d/2} = x_{i+d/2} cos + x_i sin
    Computed in float64.
    """
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    half = d // 2
    theta = np.float64(base) ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = np.asarray(pos, dtype=np.float64)[..., None] * theta
    c, s = np.cos(ang), np.sin(ang)
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def rotate_half_to_interleaved(x: np.ndarray) -> np.ndarray:
    """The same vectors in the other storage order of the rotation pairs: FC i moves from dims
    (i, i + d/2) to dims (2i, 2i+1), the indexing of Sec. 3.1.  A pure permutation of the last axis."""
    x = np.asarray(x)
    half = x.shape[-1] // 2
    out = np.empty_like(x)
    out[..., 0::2] = x[..., :half]
    out[..., 1::2] = x[..., half:]
    return out


def as_interleaved(x: dict) -> dict:
    """A drawn input set (make_inputs / make_append) with q and the keys re-stored interleaved.
    fc_idx keeps its meaning (FC numbers); V is untouched (its dim order carries no pairing)."""
    out = dict(x)
    for key in ("q", "K", "k_new", "q_pre"):
        if key in out:
            out[key] = rotate_half_to_interleaved(out[key])
    return out


def explicit_pairs(fc_idx: np.ndarray, d: int, interleaved: bool = False) -> np.ndarray:
    """[Hkv][F][2] int32: the two head dims of every listed FC, written out (input of the
    explicit-pair form of the dominant list)."""
    fc = np.asarray(fc_idx, dtype=np.int32)
    lo, hi = (2 * fc, 2 * fc + 1) if interleaved else (fc, fc + d // 2)
    return np.stack([lo, hi], axis=-1).astype(np.int32)


# ----------------------------------------------------------------------------------
# the recipe
# ----------------------------------------------------------------------------------
def draw_fc_idx(w: Workload) -> np.ndarray:
    """[Hkv][F] int32: F distinct FC indices in [0, d/2) per KV head, in draw order."""
    g = _rng(w.config_id, _STREAM_FC)
    half = w.head_dim // 2
    return np.stack([g.permutation(half)[: w.n_fc] for _ in range(w.n_kv_heads)]).astype(np.int32)


def _dom_dims(fc_idx_h: np.ndarray, d: int) -> np.ndarray:
    return np.concatenate([fc_idx_h, fc_idx_h + d // 2])


def draw_q_pre(w: Workload, fc_idx: np.ndarray, sub: int = 0) -> np.ndarray:
    """Pre-RoPE queries [Bt][Hq][d] float64; dominant FC dims of the head's KV group x fc_scale."""
    g = _rng(w.config_id, _STREAM_Q, sub)
    q = g.standard_normal((w.batch, w.n_q_heads, w.head_dim))
    for hq in range(w.n_q_heads):
        q[:, hq, _dom_dims(fc_idx[hq // w.group], w.head_dim)] *= w.fc_scale
    return q


def make_inputs(w: Workload, n_cap: Optional[int] = None) -> dict:
    """Draw one decode step's inputs.

    Returns a dict with
      q       [Bt][Hq][d]          storage dtype, post-RoPE at position N
      K, V    [Bt][Hkv][n_cap][d]  storage dtype, K post-RoPE at positions 0..N-1 (rows >= N zero)
      fc_idx  [Hkv][F] int32
      salient [Bt] list of int64 arrays (positions of the salient tokens)
      q_pre   [Bt][Hq][d] float64 (pre-RoPE queries, kept for the growing-cache recipe)
    """
    n, d = w.n_ctx, w.head_dim
    n_cap = n if n_cap is None else int(n_cap)
    assert n_cap >= n and d % 2 == 0 and w.n_q_heads % w.n_kv_heads == 0
    fc_idx = draw_fc_idx(w)
    q_pre = draw_q_pre(w, fc_idx)
    q_post = rope_rotate_half(q_pre, np.full((w.batch, w.n_q_heads), n), w.rope_base)

    st = np.uint16 if w.dtype == "bf16" else np.float32
    K = np.zeros((w.batch, w.n_kv_heads, n_cap, d), dtype=st)
    V = np.zeros((w.batch, w.n_kv_heads, n_cap, d), dtype=st)
    n_sal = int(round(w.salient_frac * n))
    pos = np.arange(n)
    salient = []
    for b in range(w.batch):
        gs = _rng(w.config_id, _STREAM_SAL, b)
        sal = np.sort(gs.choice(n, size=n_sal, replace=False)) if n_sal > 0 else np.zeros(0, np.int64)
        salient.append(sal)
        for h in range(w.n_kv_heads):
            gk = _rng(w.config_id, _STREAM_K, b * w.n_kv_heads + h)
            gv = _rng(w.config_id, _STREAM_V, b * w.n_kv_heads + h)
            k = gk.standard_normal((n, d), dtype=np.float32).astype(np.float64)
            k[:, _dom_dims(fc_idx[h], d)] *= w.fc_scale
            if n_sal > 0:
                q_dir = q_pre[b, h * w.group:(h + 1) * w.group].mean(axis=0)
                k[sal] += 0.5 * q_dir
            K[b, h, :n] = to_storage(rope_rotate_half(k, pos, w.rope_base), w.dtype)
            V[b, h, :n] = to_storage(gv.standard_normal((n, d), dtype=np.float32), w.dtype)
    return {
        "q": to_storage(q_post, w.dtype), "K": K, "V": V, "fc_idx": fc_idx,
        "salient": salient, "q_pre": q_pre, "n_cap": n_cap,
    }


def make_append(w: Workload, fc_idx: np.ndarray, step: int, n_before: int) -> dict:
    """Inputs of growing-cache step `step` (>= 1): one new K/V row per (b, h) that lands at
    position `n_before` (so the context becomes n_before + 1) and a fresh query at position
    n_before + 1.  Every 100th appended token is salient for the new query.
    """
    d = w.head_dim
    q_pre = draw_q_pre(w, fc_idx, sub=step)
    q_post = rope_rotate_half(q_pre, np.full((w.batch, w.n_q_heads), n_before + 1), w.rope_base)
    g = _rng(w.config_id, _STREAM_APPEND, step)
    k = g.standard_normal((w.batch, w.n_kv_heads, d))
    v = g.standard_normal((w.batch, w.n_kv_heads, d))
    for h in range(w.n_kv_heads):
        k[:, h, _dom_dims(fc_idx[h], d)] *= w.fc_scale
        if step % 100 == 0:
            k[:, h] += 0.5 * q_pre[:, h * w.group:(h + 1) * w.group].mean(axis=1)
    k_post = rope_rotate_half(k, np.full((w.batch, w.n_kv_heads), n_before), w.rope_base)
    return {"q": to_storage(q_post, w.dtype), "k_new": to_storage(k_post, w.dtype),
            "v_new": to_storage(v, w.dtype)}


# ----------------------------------------------------------------------------------
# analytic byte model of one decode step (Sec. 4.4, "Memory Movement Reduction")
# ----------------------------------------------------------------------------------
def algorithmic_bytes(w: Workload) -> dict:
    rows, e = w.batch * w.n_kv_heads, w.elem_bytes
    b_eff = min(w.budget, w.n_ctx)
    kp = rows * w.n_ctx * 2 * w.n_fc * e
    gather = rows * 2 * b_eff * w.head_dim * e
    inter = 2 * rows * w.n_ctx * 4 + 2 * rows * b_eff * 4
    dense = 2 * rows * w.n_ctx * w.head_dim * e
    return {"kp_read": kp, "kv_gather": gather, "alg": kp + gather,
            "alg_plus_intermediates": kp + gather + inter, "dense": dense}
