"""Pins of the oracle's other pairings of head dims into frequency chunks: "interleaved" (FC i =
dims (2i, 2i+1), the indexing Sec. 3.1 writes) and "list" (explicit dim pairs; Sec. 6)."""
import json
import os

import numpy as np
import pytest

from oracle import fasa_oracle as O
from paper_2602_03152_amd import workload as W

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "tiny_hand_worked.json")))


def _gold():
    q = np.array(GOLD["q"], dtype=np.float32)[None]
    K = np.array(GOLD["K"], dtype=np.float32)[None, None]
    return q, K


def test_hand_worked_scores_interleaved_and_explicit_pair():
    q, K = _gold()
    S0, _ = O.score(q, K, np.array([[0]]), 3, "interleaved")
    np.testing.assert_array_equal(S0[0, 0], GOLD["S_il_fc0"])
    S1, _ = O.score(q, K, np.array([[1]]), 3, "interleaved")
    np.testing.assert_array_equal(S1[0, 0], GOLD["S_il_fc1"])
    Sa, _ = O.score(q, K, np.array([[1, 0]]), 3, "interleaved")
    np.testing.assert_array_equal(Sa[0, 0], GOLD["S_all"])
    Sp, _ = O.score(q, K, np.array([[[3, 0]]]), 3, "list")
    np.testing.assert_array_equal(Sp[0, 0], GOLD["S_pair_3_0"])


def _small(seed, Bt=2, Hq=6, Hkv=2, d=16, N=29, dtype="bf16"):
    rng = np.random.default_rng(seed)
    q = W.to_storage(rng.standard_normal((Bt, Hq, d)), dtype)
    K = W.to_storage(rng.standard_normal((Bt, Hkv, N, d)), dtype)
    return q, K


@pytest.mark.parametrize("pairing", ["interleaved", "list"])
def test_every_dim_listed_is_the_full_dot_product(pairing):
    """All d dims, in any pairing, add up to the whole-vector logit (einsum, no column selection)."""
    q, K = _small(1)
    Bt, Hq, d = q.shape
    Hkv, N = K.shape[1], K.shape[2]
    rng = np.random.default_rng(2)
    if pairing == "interleaved":
        fc = np.stack([rng.permutation(d // 2) for _ in range(Hkv)])
    else:
        fc = np.stack([rng.permutation(d).reshape(d // 2, 2) for _ in range(Hkv)])
    S, _ = O.score(q, K, fc, N, pairing)
    q64 = W.storage_to_f64(q).reshape(Bt, Hkv, Hq // Hkv, d)
    full = np.einsum("bhgd,bhnd->bhn", q64, W.storage_to_f64(K))
    np.testing.assert_allclose(S, full, rtol=0, atol=1e-12)


def test_one_hot_keys_pick_the_listed_dims():
    """Key n = e_n: S[n] = sum_g q_g[n] exactly when dim n is listed, else 0."""
    d = 8
    rng = np.random.default_rng(3)
    q = rng.standard_normal((1, 2, d)).astype(np.float32)
    K = np.eye(d, dtype=np.float32)[None, None]
    qs = q[0].astype(np.float64).sum(0)
    S, _ = O.score(q, K, np.array([[2, 0]]), d, "interleaved")        # dims 4, 5, 0, 1
    np.testing.assert_array_equal(S[0, 0], np.where(np.isin(np.arange(d), [4, 5, 0, 1]), qs, 0.0))
    S, _ = O.score(q, K, np.array([[[7, 2], [3, 6]]]), d, "list")
    np.testing.assert_array_equal(S[0, 0], np.where(np.isin(np.arange(d), [7, 2, 3, 6]), qs, 0.0))


def test_relabelled_storage_gives_the_same_scores():
    """Re-storing q and K interleaved and reading them with the interleaved pairing is a pure
    relabelling of dims: same scores as the rotate-half storage, FC numbers unchanged; the explicit
    pairs of either storage give them too."""
    q, K = _small(4)
    d, N = q.shape[2], K.shape[2]
    fc = np.array([[5, 0, 3], [1, 7, 2]])
    S, D = O.score(q, K, fc, N)
    qi, Ki = W.rotate_half_to_interleaved(q), W.rotate_half_to_interleaved(K)
    for args in [(qi, Ki, fc, N, "interleaved"),
                 (q, K, W.explicit_pairs(fc, d), N, "list"),
                 (qi, Ki, W.explicit_pairs(fc, d, interleaved=True), N, "list")]:
        S2, D2 = O.score(*args)
        np.testing.assert_array_equal(S2, S)
        np.testing.assert_array_equal(D2, D)


@pytest.mark.parametrize("i", [0, 9, 63])
def test_single_fc_closed_form_interleaved(i):
    """The closed form of a single-FC score (Sec. 3.3) with the pair stored at dims (2i, 2i+1)."""
    d, base, n_ctx, m = 128, 5.0e5, 5, 33
    a, b, c, dd = -0.5, 1.5, 0.25, 2.0
    theta = base ** (-2.0 * i / d)
    q_pre = np.zeros(d); q_pre[2 * i], q_pre[2 * i + 1] = a, b
    k_pre = np.zeros(d); k_pre[2 * i], k_pre[2 * i + 1] = c, dd
    q = O.rope_reference(q_pre, m, base, "interleaved").astype(np.float32)[None, None]
    K = np.stack([O.rope_reference(k_pre, n, base, "interleaved") for n in range(n_ctx)]).astype(np.float32)[None, None]
    expect = np.array([(a * c + b * dd) * np.cos((n - m) * theta) + (b * c - a * dd) * np.sin((n - m) * theta)
                       for n in range(n_ctx)])
    S, _ = O.score(q, K, np.array([[i]]), n_ctx, "interleaved")
    np.testing.assert_allclose(S[0, 0], expect, rtol=0, atol=2e-6)
    S_other, _ = O.score(q, K, np.array([[(i + 1) % (d // 2)]]), n_ctx, "interleaved")
    np.testing.assert_array_equal(S_other, 0.0)
    # the rotation itself: the generator's rotate-half routine on the re-stored vector
    np.testing.assert_allclose(O.rope_reference(q_pre, m, base, "interleaved"),
                               W.rotate_half_to_interleaved(W.rope_rotate_half(
                                   np.concatenate([q_pre[0::2], q_pre[1::2]]), np.array(m), base)),
                               rtol=0, atol=1e-12)


@pytest.mark.parametrize("pairing", ["interleaved", "list"])
def test_pack_and_split_are_bit_exact_column_copies(pairing):
    q, K = _small(5)
    N, d = K.shape[2], K.shape[3]
    if pairing == "interleaved":
        fc = np.array([[3, 0, 5], [7, 6, 1]])
        dims = np.stack([2 * fc, 2 * fc + 1], -1)
    else:
        fc = np.array([[[15, 0], [3, 8], [9, 1]], [[2, 4], [6, 5], [14, 7]]])
        dims = fc
    Kp, Knd = O.split_kcache(K, fc, N - 3, pairing)
    for h in range(2):
        for f in range(3):
            np.testing.assert_array_equal(Kp[:, h, f, :, 0], K[:, h, :N - 3, dims[h, f, 0]])
            np.testing.assert_array_equal(Kp[:, h, f, :, 1], K[:, h, :N - 3, dims[h, f, 1]])
        rest = [j for j in range(d) if j not in set(dims[h].reshape(-1).tolist())]
        np.testing.assert_array_equal(Knd[:, h], K[:, h, :N - 3][:, :, rest])
    # Combine(Split(k)) = k on any token list
    T = [[np.array([4, 0, 11]), np.array([7])], [np.array([1, 2]), np.array([25, 3, 9, 0])]]
    K_T = O.combine_selected(Kp, Knd, fc, T, pairing)
    for b in range(2):
        for h in range(2):
            np.testing.assert_array_equal(K_T[b][h], K[b, h][T[b][h]])
