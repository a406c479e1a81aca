"""Plain, slow, float64 CPU oracle of the FASA decode step.  TEST INFRASTRUCTURE ONLY.

Every function restates one definition of the paper in numpy float64, with no blocking,
fusion or reordering beyond what the definition says.  Nothing here is imported by the
product path; nothing here imports the product path.

Tensor conventions (all "storage" arrays are numpy uint16 holding raw bf16 bits, or
float32; they are widened exactly to float64 before any arithmetic):
  q      [Bt][Hq][d]      post-RoPE query of the current step
  K, V   [Bt][Hkv][>=N][d]  cached post-RoPE keys / values, first N rows valid
  fc_idx [Hkv][F] int     dominant frequency chunks of each KV head (I_dom, Sec. 4.1)
FC i is the rotation pair (dim i, dim i + d/2) (rotate-half storage of the FC of
Sec. 3.1) unless a function is given another `pairing`: "interleaved" takes FC i as dims
(2i, 2i+1), the indexing Sec. 3.1 itself writes; "list" takes fc_idx as explicit dim pairs
[Hkv][F][2] (heads whose position encoding covers part of the dims, or none: Sec. 6).  GQA: query head hq belongs to KV head hq // G, G = Hq / Hkv; the paper is
silent on GQA, the reading taken is one score vector and one index set per KV head with
scores summed over the G query heads of the group.

Pins (tests/test_oracle_*.py): closed-form single-FC RoPE score (both pairings), hand-worked
fixture in tests/golden/ (all three pairings), F = d/2 equals the full dot product, brute-force top-k, F = d/2 with B = N
equals dense attention computed by torch's float64 scaled_dot_product_attention, convex
combination invariants of the attention output.  No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np


# ------------------------------------------------------------------------------------
# exact widening of storage to float64
# ------------------------------------------------------------------------------------
def widen(x: np.ndarray) -> np.ndarray:
    x = np.asarray(x)
    if x.dtype == np.uint16:  # raw bf16 bits: the upper half of a float32
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return x.astype(np.float64)


# ------------------------------------------------------------------------------------
# which two head dims an entry of a head's list names
# ------------------------------------------------------------------------------------
def fc_dims(fc_idx_h, d: int, pairing: str = "half") -> list:
    """[(lo, hi)] for every entry of one KV head's list.
    "half": FC i = (i, i + d/2); "interleaved": FC i = (2i, 2i+1) (Sec. 3.1 as written);
    "list": the entries are the pairs themselves."""
    if pairing == "half":
        return [(int(i), int(i) + d // 2) for i in fc_idx_h]
    if pairing == "interleaved":
        return [(2 * int(i), 2 * int(i) + 1) for i in fc_idx_h]
    if pairing == "list":
        return [(int(a), int(b)) for a, b in fc_idx_h]
    raise ValueError(pairing)


# ------------------------------------------------------------------------------------
# Sec. 3.1: rotary position encoding, FC i rotated by angle m * theta_i
# ------------------------------------------------------------------------------------
def rope_reference(x: np.ndarray, m: int, base: float, pairing: str = "half") -> np.ndarray:
    """Rotate one vector x[d] at position m, one 2x2 rotation matrix per FC (Sec. 3.1, FC
    definition: R_{m,theta_i} = [[cos, -sin], [sin, cos]], theta_i = base^(-2i/d), i from 0).
    FC i occupies dims (i, i + d/2), or (2i, 2i+1) for pairing "interleaved".  Written FC by FC
    on purpose (slow, obvious)."""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[0]
    out = np.empty(d, dtype=np.float64)
    for i, (lo, hi) in enumerate(fc_dims(range(d // 2), d, pairing)):
        theta = float(base) ** (-2.0 * i / d)
        c, s = np.cos(m * theta), np.sin(m * theta)
        R = np.array([[c, -s], [s, c]])
        out[[lo, hi]] = R @ x[[lo, hi]]
    return out


# ------------------------------------------------------------------------------------
# Alg. 2, "Split" + "UpdateCache" of the dominant key parts: the FC-major packed copy
# ------------------------------------------------------------------------------------
def pack_kcache(K: np.ndarray, fc_idx: np.ndarray, n_ctx: int, pairing: str = "half") -> np.ndarray:
    """Kp[b,h,f,n,:] = (K[b,h,n,lo_f], K[b,h,n,hi_f]), (lo_f, hi_f) the dims of list entry f
    ((i_f, i_f + d/2) by default); bit-exact copy, storage dtype kept."""
    Bt, Hkv, _, d = K.shape
    F = fc_idx.shape[1]
    Kp = np.zeros((Bt, Hkv, F, n_ctx, 2), dtype=K.dtype)
    for h in range(Hkv):
        for f, (lo, hi) in enumerate(fc_dims(fc_idx[h], d, pairing)):
            Kp[:, h, f, :, 0] = K[:, h, :n_ctx, lo]
            Kp[:, h, f, :, 1] = K[:, h, :n_ctx, hi]
    return Kp


# ------------------------------------------------------------------------------------
# Sec. 4.1, TIP: S_t = sum over dominant FCs of the single-FC scores (raw logits)
# ------------------------------------------------------------------------------------
def score(q: np.ndarray, K: np.ndarray, fc_idx: np.ndarray, n_ctx: int, pairing: str = "half"):
    """S[b,h,n] = sum_{g<G} sum_{f<F} ( q[b,hG+g,i_f] K[b,h,n,i_f] + q[b,hG+g,i_f+d/2] K[b,h,n,i_f+d/2] )
    (for another `pairing`: the two dims fc_dims names instead of i_f and i_f + d/2).

    Unscaled, no softmax (Sec. 3.3 calls these "raw score vectors"; Alg. 2 computes
    q^dom (K^dom)^T).  Also returns D[b,h,n] = the same sum over absolute values of the
    terms, which scales the forward-error bound of any floating-point evaluation order.
    """
    q64 = widen(q)
    Bt, Hq, d = q64.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    S = np.zeros((Bt, Hkv, n_ctx))
    D = np.zeros((Bt, Hkv, n_ctx))
    for b in range(Bt):
        for h in range(Hkv):
            for pair in fc_dims(fc_idx[h], d, pairing):
                for dim in pair:
                    k_col = widen(K[b, h, :n_ctx, dim])
                    for g in range(G):
                        S[b, h] += q64[b, h * G + g, dim] * k_col
                        D[b, h] += np.abs(q64[b, h * G + g, dim] * k_col)
    return S, D


# ------------------------------------------------------------------------------------
# Sec. 4.1: T_t = TopK-I(S_t, N_fac)
# ------------------------------------------------------------------------------------
def topk_indices(s_row: np.ndarray, budget: int) -> np.ndarray:
    """Indices of the min(budget, N) largest entries of one score row; equal scores are
    broken towards the lower index; returned sorted ascending (the set is what matters).
    The comparison is done on the values as given (float32 rows stay float32)."""
    n = s_row.shape[0]
    b = min(int(budget), n)
    order = np.argsort(-s_row, kind="stable")   # stable: among equals, lower index first
    return np.sort(order[:b]).astype(np.int64)


def topk(S: np.ndarray, budget: int, n_ctx: int) -> np.ndarray:
    """[Bt][Hkv][min(B,N)] int64."""
    Bt, Hkv = S.shape[:2]
    return np.stack([np.stack([topk_indices(S[b, h, :n_ctx], budget) for h in range(Hkv)])
                     for b in range(Bt)])


# ------------------------------------------------------------------------------------
# Sec. 4.2, FAC: gather the selected rows, exact softmax attention over them
# ------------------------------------------------------------------------------------
def sparse_attend(q: np.ndarray, K: np.ndarray, V: np.ndarray, T) -> np.ndarray:
    """O[b,hq] = softmax_j( q[b,hq] . K[b,h,T_j] / sqrt(d) ) V[b,h,T_j], h = hq // G.
    T[b][h] is any integer index sequence (order irrelevant).  float64 [Bt][Hq][d]."""
    q64 = widen(q)
    Bt, Hq, d = q64.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    O = np.zeros((Bt, Hq, d))
    for b in range(Bt):
        for h in range(Hkv):
            idx = np.asarray(T[b][h], dtype=np.int64)
            K_T = widen(K[b, h][idx])           # Gather(K, T)
            V_T = widen(V[b, h][idx])           # Gather(V, T)
            for g in range(G):
                logits = (K_T @ q64[b, h * G + g]) / np.sqrt(d)
                p = np.exp(logits - logits.max())
                p /= p.sum()
                O[b, h * G + g] = p @ V_T
    return O


def dense_attend(q: np.ndarray, K: np.ndarray, V: np.ndarray, n_ctx: int) -> np.ndarray:
    """Full-KV decode attention: FAC with T = all N tokens (the paper's FKV baseline)."""
    Bt, Hkv = K.shape[:2]
    T = [[np.arange(n_ctx) for _ in range(Hkv)] for _ in range(Bt)]
    return sparse_attend(q, K, V, T)


# ------------------------------------------------------------------------------------
# Alg. 2 (memory-optimised variant): Split / SelectTokens / Combine of the key cache
# ------------------------------------------------------------------------------------
def nondominant_dims(fc_idx_h: np.ndarray, d: int, pairing: str = "half") -> np.ndarray:
    """Head dims of one KV head that belong to no dominant FC, ascending."""
    dom = set()
    for lo, hi in fc_dims(fc_idx_h, d, pairing):
        dom.add(lo); dom.add(hi)
    return np.array([j for j in range(d) if j not in dom], dtype=np.int64)


def split_kcache(K: np.ndarray, fc_idx: np.ndarray, n_ctx: int, pairing: str = "half"):
    """Split(k, I_dom) for every cached key: (Kp, Knd).  Kp is the FC-major dominant copy kept on
    the device; Knd[b,h,n,:] holds the non-dominant dims of key n in ascending dim order (the part
    the memory-optimised variant keeps in host memory)."""
    Bt, Hkv, _, d = K.shape
    F = fc_idx.shape[1]
    Kp = pack_kcache(K, fc_idx, n_ctx, pairing)
    Knd = np.zeros((Bt, Hkv, n_ctx, d - 2 * F), dtype=K.dtype)
    for h in range(Hkv):
        Knd[:, h] = K[:, h, :n_ctx][:, :, nondominant_dims(fc_idx[h], d, pairing)]
    return Kp, Knd


def combine_selected(Kp: np.ndarray, Knd: np.ndarray, fc_idx: np.ndarray, T, pairing: str = "half") -> list:
    """SelectTokens + Combine: the full key rows of the selected tokens rebuilt from the two parts.
    Returns K_T[b][h] as arrays [len(T[b][h])][d], storage dtype (bit-exact copies)."""
    Bt, Hkv, F = Kp.shape[0], Kp.shape[1], Kp.shape[2]
    d = Knd.shape[-1] + 2 * F
    out = []
    for b in range(Bt):
        row = []
        for h in range(Hkv):
            idx = np.asarray(T[b][h], dtype=np.int64)
            k_t = np.zeros((len(idx), d), dtype=Kp.dtype)
            k_t[:, nondominant_dims(fc_idx[h], d, pairing)] = Knd[b, h][idx]
            for f, (lo, hi) in enumerate(fc_dims(fc_idx[h], d, pairing)):
                k_t[:, lo] = Kp[b, h, f, idx, 0]
                k_t[:, hi] = Kp[b, h, f, idx, 1]
            row.append(k_t)
        out.append(row)
    return out


def attend_on_rows(q: np.ndarray, K_T: list, V_T: list) -> np.ndarray:
    """FAC on already gathered rows (the last two lines of Alg. 2 before W_O)."""
    q64 = widen(q)
    Bt, Hq, d = q64.shape
    Hkv = len(K_T[0])
    G = Hq // Hkv
    O = np.zeros((Bt, Hq, d))
    for b in range(Bt):
        for h in range(Hkv):
            k64, v64 = widen(K_T[b][h]), widen(V_T[b][h])
            for g in range(G):
                logits = (k64 @ q64[b, h * G + g]) / np.sqrt(d)
                p = np.exp(logits - logits.max())
                p /= p.sum()
                O[b, h * G + g] = p @ v64
    return O


def offload_gpu_bytes(n_ctx: int, budget: int, d: int, d_dom: int, e: int) -> int:
    """Per layer and KV head, device-resident cache bytes of the memory-optimised variant
    (App. C, eq. memory_fasa_m): L*d_dom + b*d_nondom + b*d elements."""
    return (n_ctx * d_dom + budget * (d - d_dom) + budget * d) * e


# ------------------------------------------------------------------------------------
# Sec. 3.3 / Alg. 1: contextual agreement of single FCs, offline choice of the dominant set
# ------------------------------------------------------------------------------------
def contextual_agreement(q: np.ndarray, K: np.ndarray, n_ctx: int, top_k: int, score_dtype=np.float32,
                         pairing: str = "half") -> np.ndarray:
    """CA[b,h,i] = | TopK-I(alpha, K) & TopK-I(alpha^(i), K) | / K  (eq. ca_k), alpha = full-head raw
    scores, alpha^(i) = scores of FC i alone, both summed over the GQA group of KV head h (the same
    reading as for the online scores) and ranked in `score_dtype` with ties towards the lower index."""
    Bt, Hq, d = np.asarray(q).shape
    Hkv = K.shape[1]
    half = d // 2
    kk = min(int(top_k), n_ctx)
    all_fc = np.tile(np.arange(half), (Hkv, 1))
    S_full, _ = score(q, K, all_fc, n_ctx, pairing)
    T_full = topk(S_full.astype(score_dtype), kk, n_ctx)
    CA = np.zeros((Bt, Hkv, half))
    for i in range(half):
        S_i, _ = score(q, K, np.full((Hkv, 1), i), n_ctx, pairing)
        T_i = topk(S_i.astype(score_dtype), kk, n_ctx)
        for b in range(Bt):
            for h in range(Hkv):
                CA[b, h, i] = len(np.intersect1d(T_full[b, h], T_i[b, h])) / kk
    return CA


def dominant_fcs(ca_mean: np.ndarray, n_fc: int) -> np.ndarray:
    """I_dom[h] = the n_fc FCs with the largest mean CA (Alg. 1, stage 2); equal values towards the
    lower FC index; returned in descending order of CA.  ca_mean is [Hkv][d/2]."""
    return np.stack([np.argsort(-np.asarray(row, dtype=np.float64), kind="stable")[:n_fc] for row in ca_mean]).astype(np.int32)


# ------------------------------------------------------------------------------------
# the whole decode step: TIP -> TopK-I -> FAC
# ------------------------------------------------------------------------------------
def decode_step(q, K, V, fc_idx, n_ctx: int, budget: int, score_dtype=np.float32, pairing: str = "half"):
    """Returns (S float64, D, T, O).  The ranking is taken on S rounded to `score_dtype`
    (the precision the method's score vector is held in on the device: float32)."""
    S, D = score(q, K, fc_idx, n_ctx, pairing)
    T = topk(S.astype(score_dtype), budget, n_ctx)
    O = sparse_attend(q, K, V, T)
    return S, D, T, O
