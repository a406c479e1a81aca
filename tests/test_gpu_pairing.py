"""GPU parity of the other pairings of head dims into frequency chunks: FC i stored at dims
(2i, 2i+1) (the indexing of Sec. 3.1) and explicit dim pairs (the heads of Sec. 6), through every
entry point that reads the dominant list: packing, scoring, the fused steps with and without an
appended row, ragged and paged."""
import numpy as np
import pytest
import torch

from oracle import fasa_oracle as O
from paper_2602_03152_amd import workload as W
from tests.test_gpu_decode_step import compare_step, run_step

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fb():
    from paper_2602_03152_amd import binding
    return binding


def random_pairs(seed, n_kv_heads, n_fc, d):
    """[Hkv][F][2]: 2F distinct dims per head in random order (pairs that are no rotation pairs)."""
    rng = np.random.default_rng(seed)
    return np.stack([rng.permutation(d)[: 2 * n_fc].reshape(n_fc, 2) for _ in range(n_kv_heads)]).astype(np.int32)


def variant(w, x, pairing, seed=0):
    """(inputs, oracle pairing) of one drawn workload read through `pairing`:
    interleaved = the same vectors re-stored; pairs = the same storage, FCs written out as dim
    pairs; random = arbitrary dim pairs."""
    if pairing == "interleaved":
        return W.as_interleaved(x), "interleaved"
    y = dict(x)
    if pairing == "pairs":
        y["fc_idx"] = W.explicit_pairs(x["fc_idx"], w.head_dim)
    else:
        y["fc_idx"] = random_pairs(seed, w.n_kv_heads, w.n_fc, w.head_dim)
    return y, "list"


CASES = {
    "cfg1": dict(cid=1, n_ctx=5000 + 19, budget=313),
    "cfg3_gqa7": dict(cid=3, batch=2, n_ctx=4099, budget=W.budget_fraction(4099)),
    "cfg0_f32": dict(cid=0, n_ctx=2049, budget=65),
    "fc8": dict(cid=1, n_ctx=3000, budget=200, n_fc=8, n_kv_heads=2, n_q_heads=8),
    "fc5_generic": dict(cid=1, n_ctx=1500, budget=77, n_fc=5, n_kv_heads=2, n_q_heads=8),
    "fc40_generic_f32": dict(cid=0, n_ctx=1030, budget=100, n_fc=40),
    "fc64_all": dict(cid=1, n_ctx=2100, budget=200, n_fc=64, n_kv_heads=2, n_q_heads=4),
}


@pytest.mark.parametrize("pairing", ["interleaved", "pairs", "random"])
@pytest.mark.parametrize("name", list(CASES))
def test_pack_score_and_step(fb, name, pairing):
    from tests.gpu_util import Device, to_host
    kw = dict(CASES[name]); cid = kw.pop("cid")
    w = W.WORKLOADS[cid].scaled(**kw)
    x0 = W.make_inputs(w, n_cap=(w.n_ctx + 63) // 64 * 64)
    x, op = variant(w, x0, pairing, seed=len(name))
    print("pairing", name, pairing, flush=True)
    d = Device(w, x, pairing=op)
    fb.fasa_validate_fc_idx(d.shape, x["fc_idx"])
    d.pack()
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(d.Kp, d.st)[:, :, :, :w.n_ctx], O.pack_kcache(x["K"], x["fc_idx"], w.n_ctx, op))
    run_step(fb, w, x, d=d)
    n_diff, o_err = compare_step(w, x["q"], x["K"], x["V"], x["fc_idx"], d, w.n_ctx, w.budget, pairing=op)
    print("  set diff vs oracle:", n_diff, " max |O err|:", o_err, flush=True)
    if pairing != "random":
        # a relabelling of dims: the FC's two products are added in the same order, so the float32
        # scores and the selected set are those of the rotate-half run, bit for bit
        S, T = to_host(d.S).copy(), np.sort(to_host(d.T), -1)
        d0 = run_step(fb, w, x0)
        np.testing.assert_array_equal(to_host(d0.S)[:, :, :w.n_ctx], S[:, :, :w.n_ctx])
        np.testing.assert_array_equal(np.sort(to_host(d0.T), -1), T)


@pytest.mark.parametrize("pairing", ["interleaved", "random"])
@pytest.mark.parametrize("name,kw", [
    ("cfg1_tail", dict(cid=1, n_ctx=3000 + 1, budget=128)),          # the new token opens a 4-token group
    ("cfg3", dict(cid=3, batch=2, n_ctx=2048 + 4, budget=300)),
    ("f32", dict(cid=0, n_ctx=1026, budget=64)),
    ("generic_f", dict(cid=1, n_ctx=1500, budget=77, n_fc=5, n_kv_heads=2, n_q_heads=8)),
])
def test_step_with_appended_row(fb, name, kw, pairing):
    """The appended row reaches K, V and - through the listed dims - the packed copy and its own score."""
    from tests.gpu_util import Device, to_host
    kw = dict(kw); cid = kw.pop("cid")
    w = W.WORKLOADS[cid].scaled(**kw)
    n_cap = (w.n_ctx + 63) // 64 * 64
    wb = w.scaled(n_ctx=w.n_ctx - 1)
    x0 = W.make_inputs(wb, n_cap=n_cap)
    a0 = W.make_append(wb, x0["fc_idx"], step=1, n_before=wb.n_ctx)
    x, op = variant(w, x0, pairing, seed=7)
    a = W.as_interleaved(a0) if pairing == "interleaved" else a0
    print("pairing append", name, pairing, flush=True)
    d = Device(w, x, n_cap=n_cap, pairing=op)
    fb.fasa_pack_kcache(d.shape, d.K, d.fc_idx, d.Kp, 0, wb.n_ctx)
    run_step(fb, w, x, d=d, k_new=a["k_new"], v_new=a["v_new"], q=a["q"])
    K, V = x["K"].copy(), x["V"].copy()
    K[:, :, wb.n_ctx] = a["k_new"]; V[:, :, wb.n_ctx] = a["v_new"]
    np.testing.assert_array_equal(to_host(d.K, d.st), K)
    np.testing.assert_array_equal(to_host(d.V, d.st), V)
    np.testing.assert_array_equal(to_host(d.Kp, d.st)[:, :, :, :w.n_ctx], O.pack_kcache(K, x["fc_idx"], w.n_ctx, op))
    compare_step(w, a["q"], K, V, x["fc_idx"], d, w.n_ctx, w.budget, pairing=op)


def test_paged_ragged_step_with_explicit_pairs(fb):
    """Explicit dim pairs through the paged, ragged step with an appended row per sequence."""
    from tests.gpu_util import to_dev, to_host
    from tests.test_gpu_paged import PagedDevice, gather_from_pool
    w = W.WORKLOADS[2].scaled(batch=3, n_ctx=2100, budget=200)
    lens = np.array([2100, 517, 1290], np.int32)
    x0 = W.make_inputs(w, n_cap=2112)
    x, op = variant(w, x0, "random", seed=11)
    a = W.make_append(w, x0["fc_idx"], step=1, n_before=0)
    print("pairing paged ragged", flush=True)
    page, layout = 16, "token_major"
    d = PagedDevice(fb, w, x, page, layout, seed=5, pairing=op)
    fb.fasa_pack_kcache_paged(d.shape, d.paging, d.K, d.fc_idx, d.Kp, 0, w.n_ctx)
    n_ctx_seq = to_dev(lens)
    fb.fasa_decode_step_paged(d.shape, d.paging, to_dev(a["q"]), d.K, d.V, d.Kp, d.fc_idx, to_dev(a["k_new"]),
                              to_dev(a["v_new"]), n_ctx_seq, None, d.S, d.T, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    K = gather_from_pool(to_host(d.K, d.st), d.table_host, page, layout)
    V = gather_from_pool(to_host(d.V, d.st), d.table_host, page, layout)
    S, T, out = to_host(d.S), to_host(d.T), to_host(d.O)
    for b in range(w.batch):
        n = int(lens[b])
        Kb, Vb = x["K"][b:b + 1].copy(), x["V"][b:b + 1].copy()
        Kb[:, :, n - 1] = a["k_new"][b]; Vb[:, :, n - 1] = a["v_new"][b]
        np.testing.assert_array_equal(K[b, :, :n], Kb[0, :, :n])
        np.testing.assert_array_equal(V[b, :, :n], Vb[0, :, :n])
        S_ref, D_ref = O.score(a["q"][b:b + 1], Kb, x["fc_idx"], n, op)
        assert np.all(np.abs(S[b:b + 1, :, :n] - S_ref) <= 1e-5 * np.maximum(np.abs(S_ref), D_ref))
        bsel = min(w.budget, n)
        Tb = np.sort(T[b, :, :bsel], -1)
        np.testing.assert_array_equal(Tb, O.topk(S[b:b + 1, :, :n], w.budget, n)[0])
        ref = O.sparse_attend(a["q"][b:b + 1], Kb, Vb, Tb[None])
        assert np.abs(out[b:b + 1] - ref).max() <= 2e-3
