"""GPU parity of the offline calibration (contextual agreement per FC, dominant-FC choice) against
the CPU oracle, and the whole method end to end: calibrate -> I_dom -> pack -> decode."""
import numpy as np
import pytest
import torch

from oracle import fasa_oracle as O
from paper_2602_03152_amd import workload as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fb():
    from paper_2602_03152_amd import binding
    return binding


def _device_scores(fb, w, x, q, fc_rows, pairing="half"):
    """float32 scores of the device for the dominant list fc_rows ([Hkv][F]) through the staged public
    calls (pack + fasa_score): what the calibration ranks, obtained without it."""
    from tests.gpu_util import to_dev
    n_cap = x["n_cap"]
    F = fc_rows.shape[1]
    tdt = torch.int16 if w.dtype == "bf16" else torch.float32
    shape = fb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, F, w.n_ctx, n_cap, 1, w.dtype, pairing=pairing)
    fc = to_dev(np.ascontiguousarray(fc_rows, dtype=np.int32))
    Kp = torch.zeros((w.batch, w.n_kv_heads, F, n_cap, 2), dtype=tdt, device="cuda")
    S = torch.zeros((w.batch, w.n_kv_heads, n_cap), dtype=torch.float32, device="cuda")
    fb.fasa_pack_kcache(shape, to_dev(x["K"]), fc, Kp, 0, w.n_ctx)
    fb.fasa_score(shape, to_dev(q), Kp, fc, S)
    torch.cuda.synchronize()
    return S.cpu().numpy()[:, :, :w.n_ctx]


def _exact_counts(fb, w, x, queries, top_k, pairing="half"):
    """Summed intersection sizes |TopK(full) & TopK(FC i)| that the oracle's ranking rule (stable top-K,
    ties to the lower index) gives on the DEVICE's own float32 scores: integer work, compared exactly."""
    half = w.head_dim // 2
    kk = min(top_k, w.n_ctx)
    cnt = np.zeros((w.batch, w.n_kv_heads, half), dtype=np.int64)
    for q in queries:
        T_full = O.topk(_device_scores(fb, w, x, q, np.tile(np.arange(half), (w.n_kv_heads, 1)), pairing), kk, w.n_ctx)
        for i in range(half):
            T_i = O.topk(_device_scores(fb, w, x, q, np.full((w.n_kv_heads, 1), i), pairing), kk, w.n_ctx)
            for b in range(w.batch):
                for h in range(w.n_kv_heads):
                    cnt[b, h, i] += len(np.intersect1d(T_full[b, h], T_i[b, h]))
    return cnt


def _calibrate(fb, w, x, queries, top_k, pairing="half"):
    from tests.gpu_util import to_dev
    half = w.head_dim // 2
    n_cap = x["n_cap"]
    tdt = torch.int16 if w.dtype == "bf16" else torch.float32
    shape = fb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, half, w.n_ctx, n_cap, top_k, w.dtype,
                          pairing=pairing)
    K = to_dev(x["K"])
    fc_all = torch.arange(half, dtype=torch.int32, device="cuda").repeat(w.n_kv_heads, 1).contiguous()
    Kp_all = torch.zeros((w.batch, w.n_kv_heads, half, n_cap, 2), dtype=tdt, device="cuda")
    fb.fasa_pack_kcache(shape, K, fc_all, Kp_all, 0, w.n_ctx)
    nbytes = fb.fasa_calibration_workspace_bytes(shape, top_k)
    cws = torch.full((nbytes,), 0x3C, dtype=torch.uint8, device="cuda")       # needs no preparation
    ca = torch.zeros((w.batch, w.n_kv_heads, half), dtype=torch.float32, device="cuda")
    for q in queries:
        fb.fasa_contextual_agreement(shape, to_dev(q), Kp_all, top_k, ca, cws, nbytes)
    torch.cuda.synchronize()
    return ca.cpu().numpy()


@pytest.mark.parametrize("name,kw,top_k", [
    ("bf16_g4", dict(cid=1, n_ctx=1024 + 5, budget=64, n_kv_heads=2, n_q_heads=8), 96),
    ("f32_g1", dict(cid=0, n_ctx=777, budget=64), 50),
    ("gqa7", dict(cid=3, batch=2, n_ctx=600, budget=64, n_kv_heads=2, n_q_heads=14), 64),
    ("k_ge_n", dict(cid=1, n_ctx=100, budget=64, n_kv_heads=1, n_q_heads=4), 500),
])
def test_contextual_agreement_matches_oracle(fb, name, kw, top_k):
    kw = dict(kw); cid = kw.pop("cid")
    w = W.WORKLOADS[cid].scaled(**kw)
    x = W.make_inputs(w, n_cap=(w.n_ctx + 63) // 64 * 64)
    q2 = W.make_append(w, x["fc_idx"], step=1, n_before=w.n_ctx - 1)["q"]
    print("calibration", name, flush=True)
    got = _calibrate(fb, w, x, [x["q"], q2], top_k)
    ref = O.contextual_agreement(x["q"], x["K"], w.n_ctx, top_k) + O.contextual_agreement(q2, x["K"], w.n_ctx, top_k)
    kk = min(top_k, w.n_ctx)
    cnt_got, cnt_ref = np.rint(got * kk).astype(int), np.rint(ref * kk).astype(int)     # summed intersection sizes
    assert np.abs(got * kk - cnt_got).max() < 1e-3
    # the parity bar: integer intersection counts, exact, on the scores the device itself computed
    np.testing.assert_array_equal(cnt_got, _exact_counts(fb, w, x, [x["q"], q2], top_k))
    # cross-check against the oracle's own float64-accumulated scores (rounded to float32 before ranking):
    # the two float32 values of a score differ in the last bits, which can move a token across the K-th
    # place of a ranking; not a parity bar, a bound on how much that can matter
    assert np.abs(cnt_got - cnt_ref).max() <= 4, int(np.abs(cnt_got - cnt_ref).max())
    print("  counts equal to the float64-score oracle's on %.1f %% of (head, FC) pairs"
          % (100 * (cnt_got == cnt_ref).mean()), flush=True)
    assert (cnt_got == cnt_ref).mean() > 0.9


def test_contextual_agreement_interleaved_storage(fb):
    """The same vectors stored with FC i at dims (2i, 2i+1): the agreement of FC i is what it was
    (the device's float32 scores are even bit-identical, the FC's two products being added in the
    same order), and it matches the oracle reading the interleaved storage."""
    w = W.WORKLOADS[1].scaled(n_ctx=900 + 7, budget=64, n_kv_heads=2, n_q_heads=8)
    x = W.make_inputs(w, n_cap=(w.n_ctx + 63) // 64 * 64)
    xi = W.as_interleaved(x)
    print("calibration interleaved", flush=True)
    got_half = _calibrate(fb, w, x, [x["q"]], 80)
    got = _calibrate(fb, w, xi, [xi["q"]], 80, pairing="interleaved")
    np.testing.assert_array_equal(got, got_half)
    ref = O.contextual_agreement(xi["q"], xi["K"], w.n_ctx, 80, pairing="interleaved")
    cnt_got, cnt_ref = np.rint(got * 80).astype(int), np.rint(ref * 80).astype(int)
    np.testing.assert_array_equal(cnt_got, _exact_counts(fb, w, xi, [xi["q"]], 80, pairing="interleaved"))
    assert np.abs(cnt_got - cnt_ref).max() <= 4          # cross-check, see above
    assert (cnt_got == cnt_ref).mean() > 0.9


def test_calibrate_then_decode_end_to_end(fb):
    """Alg. 1 then Alg. 2 on the device: the calibrated dominant set equals the planted one, and a
    decode step with it equals the oracle's step."""
    from tests.gpu_util import Device, to_host
    w = W.WORKLOADS[1].scaled(n_ctx=1024, budget=64, n_kv_heads=2, n_q_heads=8, n_fc=8, salient_frac=0.0)
    x = W.make_inputs(w)
    queries = [x["q"]] + [W.make_append(w, x["fc_idx"], step=s, n_before=w.n_ctx - 1)["q"] for s in range(1, 4)]
    ca = _calibrate(fb, w, x, queries, 128)[0] / len(queries)
    shape = fb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_fc, w.n_ctx, x["n_cap"], w.budget, w.dtype)
    fc = np.zeros((w.n_kv_heads, w.n_fc), dtype=np.int32)
    fb.fasa_select_dominant_fcs(shape, np.ascontiguousarray(ca, dtype=np.float32), fc)
    fb.fasa_validate_fc_idx(shape, fc)
    for h in range(w.n_kv_heads):
        assert sorted(fc[h].tolist()) == sorted(x["fc_idx"][h].tolist())
    x2 = dict(x); x2["fc_idx"] = fc
    d = Device(w, x2)
    d.pack()
    fb.fasa_decode_step(d.shape, d.q, d.K, d.V, d.Kp, d.fc_idx, None, None, d.S, d.T, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    S, D, T, out = O.decode_step(x["q"], x["K"], x["V"], fc, w.n_ctx, w.budget)
    np.testing.assert_array_equal(np.sort(to_host(d.T), -1), O.topk(to_host(d.S)[:, :, :w.n_ctx], w.budget, w.n_ctx))
    assert np.abs(to_host(d.O) - O.sparse_attend(x["q"], x["K"], x["V"], np.sort(to_host(d.T), -1))).max() <= 2e-3
