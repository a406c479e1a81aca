"""GPU parity of the memory-optimised variant (non-dominant key dims and values in pinned host
memory, fetched by the device over PCIe) against the CPU oracle and against the on-device variant."""
import numpy as np
import pytest
import torch

from oracle import fasa_oracle as O
from paper_2602_03152_amd import workload as W

pytestmark = pytest.mark.gpu
OUT_ATOL = 2e-3
SCORE_RTOL = 1e-5


@pytest.fixture(scope="module")
def fb():
    from paper_2602_03152_amd import binding
    return binding


def _pinned(shape, np_dtype):
    tdt = {np.dtype(np.uint16): torch.int16, np.dtype(np.float32): torch.float32}[np.dtype(np_dtype)]
    return torch.zeros(shape, dtype=tdt).pin_memory()


CASES = {
    "cfg1_ragged": dict(cid=1, n_ctx=3000 + 11, budget=300),
    "cfg3_gqa7": dict(cid=3, batch=2, n_ctx=2100, budget=W.budget_fraction(2100)),
    "cfg0_f32": dict(cid=0, n_ctx=2049, budget=130),
    "odd_f5": dict(cid=1, n_ctx=1500, budget=77, n_fc=5, n_kv_heads=2, n_q_heads=8),
    "all_fcs": dict(cid=1, n_ctx=900, budget=50, n_fc=64, n_kv_heads=2, n_q_heads=4),
    "budget_ge_n": dict(cid=1, n_ctx=333, budget=1000, n_kv_heads=2, n_q_heads=8),
}


@pytest.mark.parametrize("name,pairing", [(n, "half") for n in CASES] +
                         [("cfg1_ragged", "interleaved"), ("odd_f5", "interleaved"), ("cfg0_f32", "interleaved")])
def test_offload_step_matches_oracle_and_on_device_variant(fb, name, pairing):
    from tests.gpu_util import Device, to_host, to_dev
    kw = dict(CASES[name]); cid = kw.pop("cid")
    w = W.WORKLOADS[cid].scaled(**kw)
    n_cap = (w.n_ctx + 1 + 63) // 64 * 64
    x = W.make_inputs(w, n_cap=n_cap)
    if pairing == "interleaved":
        x = W.as_interleaved(x)         # the same vectors, FC i stored at dims (2i, 2i+1)
    print("offload", name, pairing, flush=True)
    d = Device(w, x, pairing=pairing)
    nd = w.head_dim - 2 * w.n_fc
    Knd = _pinned((w.batch, w.n_kv_heads, n_cap, max(nd, 1)), d.st)
    Vh = _pinned(x["V"].shape, d.st)
    Vh.copy_(torch.from_numpy(x["V"].view(np.int16) if d.st == np.uint16 else x["V"]))
    stage_bytes = fb.fasa_offload_stage_bytes(d.shape)
    stage = torch.full((stage_bytes,), 0x11, dtype=torch.uint8, device="cuda")

    # Split: dominant pairs to the device copy, the rest to host memory
    fb.fasa_offload_split_kcache(d.shape, d.K, d.fc_idx, d.Kp, Knd, 0, w.n_ctx)
    torch.cuda.synchronize()
    Kp_ref, Knd_ref = O.split_kcache(x["K"], x["fc_idx"], w.n_ctx, pairing)
    np.testing.assert_array_equal(to_host(d.Kp, d.st)[:, :, :, :w.n_ctx], Kp_ref)
    knd_host = Knd.numpy().view(d.st) if d.st == np.uint16 else Knd.numpy()
    if nd > 0:
        np.testing.assert_array_equal(knd_host[:, :, :w.n_ctx, :nd].reshape(Knd_ref.shape), Knd_ref)

    # one step; the device reads the selected rows straight from host memory
    fb.fasa_offload_decode_step(d.shape, d.q, d.Kp, d.fc_idx, Knd, Vh, None, None, d.S, d.T, d.O,
                                d.ws, d.ws_bytes, stage, stage_bytes)
    torch.cuda.synchronize()
    bsel = d.bsel
    T = to_host(d.T)
    S_ref, D_ref = O.score(x["q"], x["K"], x["fc_idx"], w.n_ctx, pairing)
    S = to_host(d.S)[:, :, :w.n_ctx].astype(np.float64)
    assert np.all(np.abs(S - S_ref) <= SCORE_RTOL * np.maximum(np.abs(S_ref), D_ref))
    np.testing.assert_array_equal(np.sort(T, -1), O.topk(to_host(d.S)[:, :, :w.n_ctx], w.budget, w.n_ctx))
    # staging holds Combine(...) = Gather(K, T) and Gather(V, T), bit for bit, in the order of T
    e = 2 if d.st == np.uint16 else 4
    rows = w.batch * w.n_kv_heads
    st_host = stage.cpu().numpy()
    half = rows * bsel * w.head_dim * e
    KT = st_host[:half].view(d.st).reshape(w.batch, w.n_kv_heads, bsel, w.head_dim)
    VT = st_host[half:2 * half].view(d.st).reshape(w.batch, w.n_kv_heads, bsel, w.head_dim)
    K_T_ref = O.combine_selected(Kp_ref, Knd_ref, x["fc_idx"], T, pairing)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            np.testing.assert_array_equal(KT[b, h], K_T_ref[b][h])
            np.testing.assert_array_equal(KT[b, h], x["K"][b, h][T[b, h]])
            np.testing.assert_array_equal(VT[b, h], x["V"][b, h][T[b, h]])
    V_T_ref = [[x["V"][b, h][T[b, h]] for h in range(w.n_kv_heads)] for b in range(w.batch)]
    out_ref = O.attend_on_rows(x["q"], K_T_ref, V_T_ref)
    out = to_host(d.O).copy()
    assert np.abs(out - out_ref).max() <= OUT_ATOL
    # the on-device variant on the same cache gives the same set and the same output
    fb.fasa_decode_step(d.shape, d.q, d.K, d.V, d.Kp, d.fc_idx, None, None, d.S, d.T, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(np.sort(to_host(d.T), -1), np.sort(T, -1))
    assert np.abs(to_host(d.O) - out).max() <= 2e-5


def test_offload_growing_cache(fb):
    """Appends go to both homes: dominant pairs to the device copy, the rest and the value row to host."""
    from tests.gpu_util import Device, to_host, to_dev
    w = W.WORKLOADS[3].scaled(batch=2, n_ctx=1500, budget=W.budget_fraction(1500))
    steps = 4
    n_cap = 1536
    x = W.make_inputs(w, n_cap=n_cap)
    K, V = x["K"].copy(), x["V"].copy()
    d = Device(w, x)
    nd = w.head_dim - 2 * w.n_fc
    Knd = _pinned((w.batch, w.n_kv_heads, n_cap, nd), d.st)
    Vh = _pinned(x["V"].shape, d.st)
    Vh.copy_(torch.from_numpy(x["V"].view(np.int16)))
    d.T = torch.full((w.batch, w.n_kv_heads, W.budget_fraction(1500 + steps)), -1, dtype=torch.int32, device="cuda")
    shapes = [d.make_shape(n_ctx=1500 + s, budget=W.budget_fraction(1500 + s)) for s in range(steps + 1)]
    d.ws_bytes = max(fb.fasa_workspace_bytes(sh) for sh in shapes)
    d.ws = torch.full((d.ws_bytes,), 0x77, dtype=torch.uint8, device="cuda")
    fb.fasa_workspace_init(d.shape, d.ws, d.ws_bytes)
    stage_bytes = max(fb.fasa_offload_stage_bytes(sh) for sh in shapes)
    stage = torch.zeros((stage_bytes,), dtype=torch.uint8, device="cuda")
    fb.fasa_offload_split_kcache(d.shape, d.K, d.fc_idx, d.Kp, Knd, 0, w.n_ctx)
    n = w.n_ctx
    for s in range(1, steps + 1):
        a = W.make_append(w, x["fc_idx"], step=s, n_before=n)
        K[:, :, n] = a["k_new"]; V[:, :, n] = a["v_new"]
        n += 1
        b = W.budget_fraction(n)
        print("offload append step", s, "n", n, flush=True)
        fb.fasa_offload_decode_step(shapes[s], to_dev(a["q"]), d.Kp, d.fc_idx, Knd, Vh, to_dev(a["k_new"]),
                                    to_dev(a["v_new"]), d.S, d.T, d.O, d.ws, d.ws_bytes, stage, stage_bytes)
        torch.cuda.synchronize()
        Kp_ref, Knd_ref = O.split_kcache(K, x["fc_idx"], n)
        np.testing.assert_array_equal(to_host(d.Kp, np.uint16)[:, :, :, :n], Kp_ref)
        np.testing.assert_array_equal(Knd.numpy().view(np.uint16)[:, :, :n], Knd_ref)
        np.testing.assert_array_equal(Vh.numpy().view(np.uint16)[:, :, :n], V[:, :, :n])
        T = to_host(d.T).reshape(-1)[: w.batch * w.n_kv_heads * b].reshape(w.batch, w.n_kv_heads, b)
        S_ref, _ = O.score(a["q"], K, x["fc_idx"], n)
        np.testing.assert_array_equal(np.sort(T, -1), O.topk(to_host(d.S)[:, :, :n], b, n))
        ref = O.sparse_attend(a["q"], K, V, T)
        assert np.abs(to_host(d.O) - ref).max() <= OUT_ATOL
