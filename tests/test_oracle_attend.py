"""Pins of the oracle's FAC stage (Sec. 4.2) and of the whole step: reduction to dense attention
(library float64 SDPA), convex-combination invariants, closed-form two-token softmax."""
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import fasa_oracle as O
from paper_2602_03152_amd import workload as W

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "tiny_hand_worked.json")))


def _sig(x):
    return 1.0 / (1.0 + math.exp(-x))


def _small(seed=0, Bt=2, Hq=6, Hkv=2, d=16, N=41, dtype="bf16"):
    rng = np.random.default_rng(seed)
    q = W.to_storage(rng.standard_normal((Bt, Hq, d)), dtype)
    K = W.to_storage(rng.standard_normal((Bt, Hkv, N, d)), dtype)
    V = W.to_storage(rng.standard_normal((Bt, Hkv, N, d)), dtype)
    return q, K, V


def _sdpa_dense(q, K, V, n):
    q64 = torch.from_numpy(W.storage_to_f64(q)).unsqueeze(2)                 # [Bt][Hq][1][d]
    G = q.shape[1] // K.shape[1]
    K64 = torch.from_numpy(W.storage_to_f64(K[:, :, :n])).repeat_interleave(G, dim=1)
    V64 = torch.from_numpy(W.storage_to_f64(V[:, :, :n])).repeat_interleave(G, dim=1)
    return torch.nn.functional.scaled_dot_product_attention(q64, K64, V64).squeeze(2).numpy()


def test_hand_worked_attention():
    q = np.array(GOLD["q"], dtype=np.float32)[None]
    K = np.array(GOLD["K"], dtype=np.float32)[None, None]
    V = np.array(GOLD["V"], dtype=np.float32)[None, None]
    out = O.sparse_attend(q, K, V, [[GOLD["attend_T"]]])
    s0, s1 = _sig(GOLD["head0_logit_gap"]), _sig(GOLD["head1_logit_gap"])
    np.testing.assert_allclose(out[0, 0], [0.0, s0, 1 - s0, 0.0], rtol=0, atol=1e-15)
    np.testing.assert_allclose(out[0, 1], [0.0, 1 - s1, s1, 0.0], rtol=0, atol=1e-15)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_dense_attend_is_library_sdpa(dtype):
    q, K, V = _small(seed=1, dtype=dtype)
    n = 33
    np.testing.assert_allclose(O.dense_attend(q, K, V, n), _sdpa_dense(q, K, V, n), rtol=0, atol=1e-13)


def test_all_fcs_and_full_budget_is_dense_attention():
    """F = d/2 and B = N: the step degenerates to full-KV attention (FAC is exact softmax on T)."""
    q, K, V = _small(seed=2)
    N, d = K.shape[2], K.shape[3]
    fc = np.stack([np.random.default_rng(3).permutation(d // 2) for _ in range(K.shape[1])])
    for budget in (N, N + 5):
        S, D, T, out = O.decode_step(q, K, V, fc, N, budget)
        assert T.shape[-1] == N
        np.testing.assert_allclose(out, _sdpa_dense(q, K, V, N), rtol=0, atol=1e-13)


def test_output_is_a_convex_combination():
    q, K, V = _small(seed=4, dtype="f32")
    Bt, Hkv, N, d = K.shape
    T = [[np.array([3, 9, 0, 21, 40]) for _ in range(Hkv)] for _ in range(Bt)]
    c = np.linspace(-1, 1, d).astype(np.float32)
    Vc = np.broadcast_to(c, V.shape).copy()
    np.testing.assert_allclose(O.sparse_attend(q, K, Vc, T), np.broadcast_to(c, (Bt, q.shape[1], d)), rtol=0, atol=1e-15)
    # one selected token: the output is that value row
    T1 = [[np.array([h + 2 * b]) for h in range(Hkv)] for b in range(Bt)]
    out = O.sparse_attend(q, K, V, T1)
    G = q.shape[1] // Hkv
    for b in range(Bt):
        for hq in range(q.shape[1]):
            np.testing.assert_array_equal(out[b, hq], V[b, hq // G, (hq // G) + 2 * b].astype(np.float64))
    # zero query: uniform weights -> mean of the selected value rows
    out0 = O.sparse_attend(np.zeros_like(q), K, V, T)
    for b in range(Bt):
        for hq in range(q.shape[1]):
            np.testing.assert_allclose(out0[b, hq], V[b, hq // G, T[b][hq // G]].astype(np.float64).mean(0), atol=1e-15)


def test_order_of_the_index_set_is_irrelevant_and_positions_are_kept():
    q, K, V = _small(seed=5)
    Bt, Hkv = K.shape[:2]
    T = [[np.array([1, 8, 30, 17, 5, 22]) for _ in range(Hkv)] for _ in range(Bt)]
    Tp = [[t[::-1] for t in row] for row in T]
    np.testing.assert_allclose(O.sparse_attend(q, K, V, T), O.sparse_attend(q, K, V, Tp), rtol=0, atol=1e-14)
    # equals dense attention over a cache that holds exactly those rows (no re-rotation, rows used as cached)
    idx = np.sort(T[0][0])
    np.testing.assert_allclose(O.sparse_attend(q, K, V, T),
                               _sdpa_dense(q, K[:, :, idx], V[:, :, idx], len(idx)), rtol=0, atol=1e-13)


def test_shifting_all_logits_changes_nothing():
    """Adding the same constant to every selected logit leaves softmax unchanged: append a dim
    on which all keys are 1 and the query is large."""
    rng = np.random.default_rng(6)
    d, N = 8, 12
    q = rng.standard_normal((1, 1, d)).astype(np.float32)
    K = rng.standard_normal((1, 1, N, d)).astype(np.float32)
    V = rng.standard_normal((1, 1, N, d)).astype(np.float32)
    K[..., 0] = 1.0
    T = [[np.arange(0, N, 2)]]
    a = O.sparse_attend(q, K, V, T)
    q2 = q.copy(); q2[..., 0] += 7.0
    np.testing.assert_allclose(O.sparse_attend(q2, K, V, T), a, rtol=0, atol=1e-13)


def test_decode_step_ranks_in_float32():
    """The ranking is taken on float32 scores: two float64 scores that collapse to one float32
    value are a tie, resolved towards the lower index."""
    d = 4
    q = np.array([[[1.0, 0.0, 0.0, 0.0]]], dtype=np.float32)
    K = np.zeros((1, 1, 3, d), dtype=np.float32)
    K[0, 0, :, 0] = [1.0, 1.0 + 2.0 ** -23, 1.0]
    V = np.eye(3, d, dtype=np.float32)[None, None]
    S, D, T, out = O.decode_step(q, K, V, np.array([[0]]), 3, 1)
    assert T[0, 0].tolist() == [1]
    S, D, T, out = O.decode_step(q, K, V, np.array([[0]]), 3, 2)
    assert T[0, 0].tolist() == [0, 1]
