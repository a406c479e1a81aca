"""fasa_decode_step_static (the entry point that allocates nothing: its workspace is an array inside
the library) against fasa_decode_step on a caller-owned workspace: two calls in a row through the
C ABI, the second on a smaller input whose workspace layout differs, so the second call finds the
first one's leftovers where its own counters live.  Collected last on purpose: its file name sorts
after every other test file."""
import numpy as np
import pytest
import torch

from paper_2602_03152_amd import workload as W

pytestmark = pytest.mark.gpu

OUT_ATOL = 2e-3


def _one_call(fb, w, seed_sub, append):
    from tests.gpu_util import Device, to_dev, to_host
    x = W.make_inputs(w, n_cap=(w.n_ctx + 63) // 64 * 64)
    k_new = v_new = None
    if append:   # the new row overwrites token n_ctx - 1 in K, V and the packed copy, on both paths alike
        app = W.make_append(w, x["fc_idx"], seed_sub + 1, w.n_ctx - 1)
        k_new, v_new, x["q"] = app["k_new"], app["v_new"], app["q"]
    out = []
    for static in (False, True):
        d = Device(w, x)
        d.pack()
        kd = None if k_new is None else to_dev(k_new)
        vd = None if v_new is None else to_dev(v_new)
        if static:
            fb.fasa_decode_step_static(d.shape, d.q, d.K, d.V, d.Kp, d.fc_idx, kd, vd, d.S, d.T, d.O)
        else:
            fb.fasa_decode_step(d.shape, d.q, d.K, d.V, d.Kp, d.fc_idx, kd, vd, d.S, d.T, d.O, d.ws, d.ws_bytes)
        torch.cuda.synchronize()
        out.append((to_host(d.S)[:, :, :w.n_ctx].copy(), np.sort(to_host(d.T), axis=-1), to_host(d.O).copy(),
                    to_host(d.Kp).copy(), to_host(d.K).copy(), to_host(d.V).copy()))
    (S0, T0, O0, Kp0, K0, V0), (S1, T1, O1, Kp1, K1, V1) = out
    assert np.array_equal(S0.view(np.uint32), S1.view(np.uint32)), "scores differ"
    assert np.array_equal(T0, T1), "index sets differ"
    assert np.array_equal(Kp0, Kp1) and np.array_equal(K0, K1) and np.array_equal(V0, V1), "caches differ"
    err = float(np.abs(O0.astype(np.float64) - O1.astype(np.float64)).max())
    assert err <= OUT_ATOL, err
    return err


def test_static_workspace_two_calls_second_smaller():
    from paper_2602_03152_amd import binding as fb
    big = W.WORKLOADS[1].scaled(n_ctx=9000 + 13, budget=700)            # 8 rows
    small = W.WORKLOADS[3].scaled(batch=1, n_ctx=2048 + 5, budget=150)  # 4 rows, GQA 7: another layout
    e1 = _one_call(fb, big, 0, append=False)
    e2 = _one_call(fb, small, 1, append=True)
    e3 = _one_call(fb, big, 2, append=True)       # and back to the larger layout
    print("static workspace: max |O_static - O_workspace| = %.2e, %.2e, %.2e" % (e1, e2, e3))


def test_static_workspace_rejects_oversize():
    from paper_2602_03152_amd import binding as fb
    s = fb.make_shape(64, 32, 8, 128, 16, 65536, 65536, 4096, "bf16")
    assert fb.fasa_workspace_bytes(s) > fb.FASA_STATIC_WS_BYTES
    with pytest.raises(fb.FasaError) as e:
        fb.fasa_decode_step_static(s, 16, 16, 16, 16, 16, None, None, 16, 16, 16)
    assert e.value.status == fb.FASA_EWORKSPACE
