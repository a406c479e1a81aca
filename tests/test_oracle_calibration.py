"""Pins of the oracle's contextual-agreement metric and dominant-FC choice (Sec. 3.3 eq. ca_k, Alg. 1)."""
import numpy as np
import pytest

from oracle import fasa_oracle as O
from paper_2602_03152_amd import workload as W


def test_ca_is_one_when_everything_is_selected_and_for_the_only_live_fc():
    rng = np.random.default_rng(0)
    d, N = 16, 40
    q = rng.standard_normal((1, 2, d)).astype(np.float32)
    K = rng.standard_normal((1, 1, N, d)).astype(np.float32)
    np.testing.assert_array_equal(O.contextual_agreement(q, K, N, N), 1.0)      # K = N: both sets are everything
    # keys that live in FC 3 only: the full-head score IS the FC-3 score
    K2 = np.zeros_like(K); K2[..., 3] = K[..., 3]; K2[..., 3 + d // 2] = K[..., 3 + d // 2]
    ca = O.contextual_agreement(q, K2, N, 7)
    assert ca[0, 0, 3] == 1.0
    # any other FC scores every token 0: its top-7 is tokens 0..6 (ties to the lower index)
    S3, _ = O.score(q, K2, np.array([[3]]), N)
    expect = len(np.intersect1d(O.topk_indices(S3[0, 0].astype(np.float32), 7), np.arange(7))) / 7
    assert ca[0, 0, 0] == expect == ca[0, 0, 5]


def test_ca_hand_example():
    """d = 4 (2 FCs), one head, 4 tokens, K = 2.  q = (1,1,1,1).
    keys: k0=(5,0,0,0) k1=(0,4,0,0) k2=(0,0,3,0) k3=(0,0,0,1) -> full scores (5,4,3,1), top-2 = {0,1};
    FC0 = dims (0,2): scores (5,0,3,0) -> {0,2}: CA = 1/2;  FC1 = dims (1,3): (0,4,0,1) -> {1,3}: CA = 1/2."""
    q = np.ones((1, 1, 4), dtype=np.float32)
    K = np.diag([5.0, 4.0, 3.0, 1.0]).astype(np.float32)[None, None]
    np.testing.assert_array_equal(O.contextual_agreement(q, K, 4, 2)[0, 0], [0.5, 0.5])
    K[0, 0, 2, 2] = 4.5           # full (5,4,4.5,1) -> {0,2}; FC0 (5,0,4.5,0) -> {0,2}: CA 1; FC1 (0,4,0,1) -> {1,3}: CA 0
    np.testing.assert_array_equal(O.contextual_agreement(q, K, 4, 2)[0, 0], [1.0, 0.0])


def test_dominant_fcs_is_a_stable_top_k():
    ca = np.array([[0.1, 0.9, 0.9, 0.3], [0.5, 0.5, 0.5, 0.7]])
    assert O.dominant_fcs(ca, 2).tolist() == [[1, 2], [3, 0]]
    assert O.dominant_fcs(ca, 4).tolist() == [[1, 2, 3, 0], [3, 0, 1, 2]]


def test_calibration_recovers_the_planted_dominant_fcs():
    """In the synthetic workload the dominant FCs carry 16x the energy of the others: averaged over a
    few queries, the F FCs with the highest contextual agreement are exactly the planted ones."""
    w = W.WORKLOADS[1].scaled(n_ctx=1024, budget=64, n_kv_heads=2, n_q_heads=8, n_fc=8, salient_frac=0.0)
    x = W.make_inputs(w)
    ca = np.zeros((w.n_kv_heads, w.head_dim // 2))
    for s in range(4):
        q = x["q"] if s == 0 else W.make_append(w, x["fc_idx"], step=s, n_before=w.n_ctx - 1)["q"]
        ca += O.contextual_agreement(q, x["K"], w.n_ctx, 128)[0]
    got = O.dominant_fcs(ca / 4, w.n_fc)
    for h in range(w.n_kv_heads):
        assert sorted(got[h].tolist()) == sorted(x["fc_idx"][h].tolist())
