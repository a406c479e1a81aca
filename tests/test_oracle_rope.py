"""Pins of the rotary encoding used to synthesise inputs (generator) and of the oracle's own
FC-by-FC rotation: relative-position identity (Sec. 3.1), closed-form single-FC score
(Sec. 3.3, single-FC scores), equivalence of rotate-half storage with the paper's
interleaved FC definition up to a fixed dim permutation."""
import numpy as np
import pytest

from oracle import fasa_oracle as O
from paper_2602_03152_amd import workload as W

BASES = [1.0e4, 5.0e5, 1.0e6]


@pytest.mark.parametrize("base", BASES)
def test_generator_rope_matches_fc_by_fc_rotation(base):
    rng = np.random.default_rng(1)
    d = 128
    for m in [0, 1, 7, 4095, 32768, 131071]:
        x = rng.standard_normal(d)
        a = W.rope_rotate_half(x, np.array(m), base)
        b = O.rope_reference(x, m, base)
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-9)  # angle ~1e5 rad: ulp(angle) ~ 1e-11


@pytest.mark.parametrize("base", BASES)
def test_relative_position_identity_full_and_per_fc(base):
    """(q R_m)(k R_n)^T depends on m - n only; the same holds FC by FC."""
    rng = np.random.default_rng(2)
    d = 64
    q, k = rng.standard_normal(d), rng.standard_normal(d)
    for delta in [0, 1, 5, 100, 3000]:
        ref_full, ref_fc = None, None
        for n in [0, 3, 250, 9000]:
            m = n + delta
            qm, kn = O.rope_reference(q, m, base), O.rope_reference(k, n, base)
            full = qm @ kn
            per_fc = qm[: d // 2] * kn[: d // 2] + qm[d // 2:] * kn[d // 2:]
            if ref_full is None:
                ref_full, ref_fc = full, per_fc
            assert abs(full - ref_full) < 1e-9 * (1 + abs(ref_full))
            np.testing.assert_allclose(per_fc, ref_fc, rtol=0, atol=1e-9)
            assert abs(per_fc.sum() - full) < 1e-10 * (1 + abs(full))


def test_position_zero_is_identity_and_pairs_keep_their_norm():
    rng = np.random.default_rng(3)
    d = 128
    x = rng.standard_normal(d)
    np.testing.assert_array_equal(O.rope_reference(x, 0, 1e4), x)
    np.testing.assert_array_equal(W.rope_rotate_half(x, np.array(0), 1e4), x)
    y = W.rope_rotate_half(x, np.array(12345), 5e5)
    np.testing.assert_allclose(y[:64] ** 2 + y[64:] ** 2, x[:64] ** 2 + x[64:] ** 2, rtol=1e-12)


@pytest.mark.parametrize("i", [0, 1, 17, 63])
def test_single_fc_score_closed_form(i):
    """A query/key pair that lives in FC i only: after rotation at m and n the TIP score with
    I_dom = {i} is (ac+bd) cos(phi) + (bc-ad) sin(phi), phi = (n-m) theta_i; it is also the full
    dot product, and the score of any other FC is zero."""
    d, base, n_ctx = 128, 5.0e5, 6
    a, b, c, dd = 0.75, -1.25, 2.0, 0.5
    theta = base ** (-2.0 * i / d)
    m = 40
    q_pre = np.zeros(d); q_pre[i], q_pre[i + d // 2] = a, b
    k_pre = np.zeros(d); k_pre[i], k_pre[i + d // 2] = c, dd
    q = O.rope_reference(q_pre, m, base).astype(np.float32)[None, None, :]
    K = np.stack([O.rope_reference(k_pre, n, base) for n in range(n_ctx)]).astype(np.float32)[None, None]
    expect = np.array([(a * c + b * dd) * np.cos((n - m) * theta) + (b * c - a * dd) * np.sin((n - m) * theta)
                       for n in range(n_ctx)])
    S, _ = O.score(q, K, np.array([[i]]), n_ctx)
    np.testing.assert_allclose(S[0, 0], expect, rtol=0, atol=2e-6)   # inputs were rounded to f32
    other = (i + 5) % (d // 2)
    S_other, _ = O.score(q, K, np.array([[other]]), n_ctx)
    np.testing.assert_array_equal(S_other, 0.0)
    S_all, _ = O.score(q, K, np.arange(d // 2)[None, :], n_ctx)
    np.testing.assert_allclose(S_all, S, rtol=0, atol=1e-12)


def test_rotate_half_equals_permuted_interleaved_definition():
    """The paper writes FC i as dims (2i, 2i+1).  With P: interleaved -> rotate-half storage,
    rotating in the interleaved layout and then permuting equals rotating the permuted vector
    with the rotate-half pairing, so scores and FC indices carry over unchanged."""
    rng = np.random.default_rng(4)
    d, base, m = 32, 1e4, 77
    x_il = rng.standard_normal(d)
    y_il = np.empty(d)
    for i in range(d // 2):           # the paper's block-diagonal rotation, interleaved dims
        th = base ** (-2.0 * i / d)
        c, s = np.cos(m * th), np.sin(m * th)
        y_il[2 * i] = c * x_il[2 * i] - s * x_il[2 * i + 1]
        y_il[2 * i + 1] = s * x_il[2 * i] + c * x_il[2 * i + 1]
    perm = np.concatenate([np.arange(0, d, 2), np.arange(1, d, 2)])   # rotate-half dim j <- interleaved perm[j]
    np.testing.assert_allclose(O.rope_reference(x_il[perm], m, base), y_il[perm], rtol=0, atol=1e-13)
