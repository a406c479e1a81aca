"""Pins of the oracle's TIP score and packed-copy definitions (Sec. 4.1; Alg. 2 Split/UpdateCache)."""
import json
import os

import numpy as np
import pytest

from oracle import fasa_oracle as O
from paper_2602_03152_amd import workload as W

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "tiny_hand_worked.json")))


def _gold_arrays():
    q = np.array(GOLD["q"], dtype=np.float32)[None]            # [1][2][4]
    K = np.array(GOLD["K"], dtype=np.float32)[None, None]      # [1][1][3][4]
    V = np.array(GOLD["V"], dtype=np.float32)[None, None]
    return q, K, V


def test_hand_worked_scores():
    q, K, _ = _gold_arrays()
    S1, D1 = O.score(q, K, np.array([[1]]), 3)
    np.testing.assert_array_equal(S1[0, 0], GOLD["S_fc1"])
    np.testing.assert_array_equal(D1[0, 0], GOLD["D_fc1"])
    S0, _ = O.score(q, K, np.array([[0]]), 3)
    np.testing.assert_array_equal(S0[0, 0], GOLD["S_fc0"])
    Sa, _ = O.score(q, K, np.array([[1, 0]]), 3)
    np.testing.assert_array_equal(Sa[0, 0], GOLD["S_all"])


def _small(seed=0, Bt=2, Hq=6, Hkv=2, d=16, N=37, dtype="bf16"):
    rng = np.random.default_rng(seed)
    q = W.to_storage(rng.standard_normal((Bt, Hq, d)), dtype)
    K = W.to_storage(rng.standard_normal((Bt, Hkv, N, d)), dtype)
    V = W.to_storage(rng.standard_normal((Bt, Hkv, N, d)), dtype)
    return q, K, V


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_all_fcs_equal_full_dot_product(dtype):
    """Sum over all d/2 FCs is the full attention logit (Sec. 4.1 decomposition), here summed
    over the GQA group; the right-hand side uses whole-vector einsum, no column selection."""
    q, K, _ = _small(dtype=dtype)
    Bt, Hq, d = q.shape
    Hkv, N = K.shape[1], K.shape[2]
    rng = np.random.default_rng(5)
    fc = np.stack([rng.permutation(d // 2) for _ in range(Hkv)])
    S, D = O.score(q, K, fc, N)
    q64 = W.storage_to_f64(q).reshape(Bt, Hkv, Hq // Hkv, d)
    K64 = W.storage_to_f64(K)
    full = np.einsum("bhgd,bhnd->bhn", q64, K64)
    np.testing.assert_allclose(S, full, rtol=0, atol=1e-12)
    assert np.all(D >= np.abs(S) - 1e-12)


def test_additive_over_disjoint_sets_and_order_free():
    q, K, _ = _small(seed=7)
    N = K.shape[2]
    a, b = np.array([[0, 3], [5, 1]]), np.array([[2, 7], [4, 6]])
    Sa, Da = O.score(q, K, a, N)
    Sb, Db = O.score(q, K, b, N)
    Sab, Dab = O.score(q, K, np.concatenate([a, b], axis=1), N)
    np.testing.assert_allclose(Sab, Sa + Sb, rtol=0, atol=1e-12)
    np.testing.assert_allclose(Dab, Da + Db, rtol=0, atol=1e-12)
    Sperm, _ = O.score(q, K, np.concatenate([b, a], axis=1)[:, ::-1], N)
    np.testing.assert_allclose(Sperm, Sab, rtol=0, atol=1e-12)


def test_gqa_sum_is_linear_in_the_query():
    """sum_g (q_g . k) = (sum_g q_g) . k : scoring a single summed query head gives the same S."""
    q, K, _ = _small(seed=8, dtype="f32")
    Bt, Hq, d = q.shape
    Hkv, N = K.shape[1], K.shape[2]
    fc = np.array([[1, 4, 6], [0, 2, 7]])
    S, _ = O.score(q, K, fc, N)
    qsum = q.astype(np.float64).reshape(Bt, Hkv, Hq // Hkv, d).sum(axis=2)
    # float64 "storage" is widened as is
    S1, _ = O.score(qsum, K, fc, N)
    np.testing.assert_allclose(S1, S, rtol=0, atol=1e-12)


def test_one_hot_keys_pick_query_entries():
    """Key n = e_j (unit vector): S[n] = sum_g q_g[j] if dim j belongs to a dominant FC, else 0."""
    d, Hq, Hkv = 8, 2, 1
    rng = np.random.default_rng(9)
    q = rng.standard_normal((1, Hq, d)).astype(np.float32)
    K = np.eye(d, dtype=np.float32)[None, None]
    fc = np.array([[2, 0]])
    S, _ = O.score(q, K, fc, d)
    expect = np.zeros(d)
    for j in (2, 6, 0, 4):
        expect[j] = q[0, :, j].astype(np.float64).sum()
    np.testing.assert_array_equal(S[0, 0], expect)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_pack_is_a_bit_exact_column_copy(dtype):
    q, K, _ = _small(seed=10, dtype=dtype)
    N, d = K.shape[2], K.shape[3]
    fc = np.array([[3, 0, 5], [7, 6, 1]])
    Kp = O.pack_kcache(K, fc, N - 2)
    assert Kp.dtype == K.dtype and Kp.shape == (2, 2, 3, N - 2, 2)
    for h in range(2):
        for f in range(3):
            np.testing.assert_array_equal(Kp[:, h, f, :, 0], K[:, h, :N - 2, fc[h, f]])
            np.testing.assert_array_equal(Kp[:, h, f, :, 1], K[:, h, :N - 2, fc[h, f] + d // 2])
    # scoring from the packed copy is the same contraction: q^dom (K^dom)^T (Alg. 2)
    S, _ = O.score(q, K, fc, N - 2)
    q64 = W.storage_to_f64(q)
    Kp64 = W.storage_to_f64(Kp)
    G = q.shape[1] // 2
    for h in range(2):
        qd = np.stack([q64[:, h * G:(h + 1) * G, fc[h]].sum(1), q64[:, h * G:(h + 1) * G, fc[h] + d // 2].sum(1)], -1)
        S2 = np.einsum("bfc,bfnc->bn", qd, Kp64[:, h])
        np.testing.assert_allclose(S2, S[:, h], rtol=0, atol=1e-12)
