"""The synthetic-input recipe: determinism, shapes, bf16 rounding against torch's conversion,
and the analytic byte model (Sec. 4.4: the loaded fraction of the KV cache is F/d + B/N)."""
import numpy as np
import pytest
import torch

from paper_2602_03152_amd import workload as W


def test_bf16_rounding_is_nearest_even_like_torch():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 50,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40], np.float32)])
    ours = W.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(ours, ref)
    np.testing.assert_array_equal(W.bf16_bits_to_f32(ours), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


@pytest.mark.parametrize("cid,frac", [(0, 0.1875), (1, 0.1875), (2, 0.140625), (4, 0.2578125)])
def test_byte_model_fraction(cid, frac):
    w = W.WORKLOADS[cid]
    m = W.algorithmic_bytes(w)
    assert m["alg"] / m["dense"] == frac == w.n_fc / w.head_dim + w.budget / w.n_ctx


def test_byte_model_absolute_numbers():
    assert W.algorithmic_bytes(W.WORKLOADS[1])["alg"] == 25165824
    assert W.algorithmic_bytes(W.WORKLOADS[1])["alg_plus_intermediates"] == 27394048
    assert W.algorithmic_bytes(W.WORKLOADS[3])["alg"] == 168574976
    assert W.WORKLOADS[3].budget == 6193 and W.budget_fraction(33279) == 6289


def test_inputs_are_deterministic_and_shaped():
    w = W.WORKLOADS[1].scaled(n_ctx=300, budget=20)
    a, b = W.make_inputs(w, n_cap=320), W.make_inputs(w, n_cap=320)
    for k in ("q", "K", "V", "fc_idx"):
        np.testing.assert_array_equal(a[k], b[k])
    assert a["K"].shape == (1, 8, 320, 128) and a["K"].dtype == np.uint16
    assert a["q"].shape == (1, 32, 128) and a["fc_idx"].shape == (8, 16)
    assert np.all(a["K"][:, :, 300:] == 0)
    for h in range(8):
        assert len(set(a["fc_idx"][h].tolist())) == 16 and a["fc_idx"][h].max() < 64
    assert len(a["salient"][0]) == 3


def test_dominant_fcs_carry_more_energy_before_and_after_rotation():
    w = W.WORKLOADS[0].scaled(n_ctx=512, budget=16, salient_frac=0.0)
    x = W.make_inputs(w)
    K = x["K"][0, 0].astype(np.float64)
    pair_energy = K[:, :64] ** 2 + K[:, 64:] ** 2
    dom = np.zeros(64, bool); dom[x["fc_idx"][0]] = True
    assert pair_energy[:, dom].mean() > 10 * pair_energy[:, ~dom].mean()


def test_append_rows():
    w = W.WORKLOADS[3].scaled(batch=2, n_ctx=64, budget=12)
    x = W.make_inputs(w, n_cap=128)
    a = W.make_append(w, x["fc_idx"], step=1, n_before=64)
    assert a["k_new"].shape == (2, 4, 128) and a["q"].shape == (2, 28, 128) and a["k_new"].dtype == np.uint16
    b = W.make_append(w, x["fc_idx"], step=1, n_before=64)
    np.testing.assert_array_equal(a["k_new"], b["k_new"])
