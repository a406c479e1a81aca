"""GPU parity, stage by stage, through the C ABI, against the CPU oracle on the same seeded inputs."""
import zlib

import numpy as np
import pytest
import torch

from oracle import fasa_oracle as O
from paper_2602_03152_amd import workload as W

pytestmark = pytest.mark.gpu

SCORE_RTOL = 1e-5   # |S_gpu - S_ref| <= 1e-5 * max(|S_ref|, D), D = sum of absolute terms
OUT_ATOL = 2e-3     # stated bar for bf16 inputs with float32 accumulation


@pytest.fixture(scope="module")
def fb():
    from paper_2602_03152_amd import binding
    return binding


def _dev(w, x, **kw):
    from tests.gpu_util import Device
    return Device(w, x, **kw)


def _case(cid, **kw):
    w = W.WORKLOADS[cid].scaled(**kw)
    n_cap = (w.n_ctx + 63) // 64 * 64
    return w, W.make_inputs(w, n_cap=n_cap)


CASES = {
    "cfg0_full": dict(cid=0),
    "cfg0_ragged": dict(cid=0, n_ctx=4096 - 37, budget=200),
    "cfg1_small_ragged": dict(cid=1, n_ctx=3000 + 21, budget=333),
    "cfg1_f1": dict(cid=1, n_ctx=1500, budget=64, n_fc=1),
    "cfg1_f64": dict(cid=1, n_ctx=2050, budget=64, n_fc=64, n_kv_heads=2, n_q_heads=8),
    "cfg2_small": dict(cid=2, batch=3, n_ctx=2111, budget=256),
    "cfg3_gqa7": dict(cid=3, batch=2, n_ctx=4099, budget=W.budget_fraction(4099)),
    "cfg4_f32fc": dict(cid=4, n_ctx=9001, budget=1024, salient_frac=0.002),
    "tiny_n1": dict(cid=1, n_ctx=1, budget=1, n_kv_heads=1, n_q_heads=4),
    "tiny_n5_f32": dict(cid=0, n_ctx=5, budget=3),
}


@pytest.fixture(scope="module", params=list(CASES))
def case(request):
    kw = dict(CASES[request.param])
    cid = kw.pop("cid")
    w, x = _case(cid, **kw)
    return request.param, w, x


def test_pack_is_bit_exact(fb, case):
    from tests.gpu_util import to_host
    name, w, x = case
    d = _dev(w, x)
    print("pack", name, flush=True)
    d.pack()
    torch.cuda.synchronize()
    ref = O.pack_kcache(x["K"], x["fc_idx"], w.n_ctx)
    got = to_host(d.Kp, d.st)
    np.testing.assert_array_equal(got[:, :, :, :w.n_ctx], ref)
    assert not got[:, :, :, w.n_ctx:].any()          # nothing written past n_end


def test_pack_append_range(fb, case):
    from tests.gpu_util import to_host
    name, w, x = case
    if w.n_ctx < 3:
        pytest.skip("needs 3 tokens")
    d = _dev(w, x)
    print("pack-append", name, flush=True)
    n = w.n_ctx
    d.pack(0, n - 2)
    d.pack(n - 2, n - 1)
    d.pack(n - 1, n)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(d.Kp, d.st)[:, :, :, :n], O.pack_kcache(x["K"], x["fc_idx"], n))


def test_score_matches_oracle(fb, case):
    from tests.gpu_util import to_host
    name, w, x = case
    d = _dev(w, x)
    print("score", name, flush=True)
    d.pack()
    fb.fasa_score(d.shape, d.q, d.Kp, d.fc_idx, d.S)
    torch.cuda.synchronize()
    S_ref, D_ref = O.score(x["q"], x["K"], x["fc_idx"], w.n_ctx)
    S = to_host(d.S)
    err = np.abs(S[:, :, :w.n_ctx].astype(np.float64) - S_ref)
    bound = SCORE_RTOL * np.maximum(np.abs(S_ref), D_ref)
    assert np.all(err <= bound), float((err / np.maximum(bound, 1e-300)).max())
    assert np.isnan(S[:, :, w.n_ctx:]).all()          # entries >= n_ctx untouched (poison kept)


def _check_topk_exact(fb, S_np, n_ctx, budget, n_cap=None):
    """fasa_topk on a given float32 score tensor equals the oracle's set on the same float32 values."""
    from tests.gpu_util import round_up
    Bt, Hkv, n_alloc = S_np.shape
    n_cap = n_alloc if n_cap is None else n_cap
    assert n_cap % 64 == 0 and n_alloc == n_cap
    shape = fb.make_shape(Bt, Hkv * 4, Hkv, 128, 16, n_ctx, n_cap, budget, "bf16")
    bsel = min(budget, n_ctx)
    S = torch.from_numpy(S_np).cuda()
    T = torch.full((Bt, Hkv, bsel), -7, dtype=torch.int32, device="cuda")
    nbytes = fb.fasa_workspace_bytes(shape)
    ws = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device="cuda")
    fb.fasa_workspace_init(shape, ws, nbytes)
    ref = O.topk(S_np, budget, n_ctx)
    for _ in range(2):          # the second call runs on the workspace as the first one left it
        T.fill_(-7)
        fb.fasa_topk(shape, S, T, ws, nbytes)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(np.sort(T.cpu().numpy(), axis=-1), ref)


TOPK_SHAPES = [  # (rows as Bt,Hkv), N, B
    ((1, 1), 4096, 256), ((1, 8), 32768 // 4 + 13, 2048 // 4), ((2, 3), 1000, 1), ((1, 2), 1000, 999),
    ((1, 2), 1000, 1000), ((1, 2), 1000, 5000), ((1, 1), 1, 1), ((1, 1), 63, 7), ((1, 1), 65, 64),
    ((3, 4), 2049, 100), ((1, 1), 20000, 6193 * 20000 // 32768),
    ((1, 2), 70001, 300), ((1, 8), 40000, 7000),      # several workgroups per row / chunked single workgroup
]


@pytest.mark.parametrize("rows,n,b", TOPK_SHAPES)
@pytest.mark.parametrize("dist", ["gauss", "dups", "zeros", "onebin", "allequal", "negative"])
def test_topk_exact_on_given_scores(fb, rows, n, b, dist):
    from tests.gpu_util import round_up
    print("topk", rows, n, b, dist, flush=True)
    rng = np.random.default_rng(zlib.crc32(repr((rows, n, b, dist)).encode()))
    n_cap = round_up(n, 64)
    S = np.full(rows + (n_cap,), np.nan, dtype=np.float32)
    if dist == "gauss":
        v = rng.standard_normal(rows + (n,)) * 180.0
    elif dist == "dups":
        v = np.round(rng.standard_normal(rows + (n,)) * 4) / 2      # few distinct values, many ties
    elif dist == "zeros":
        v = rng.standard_normal(rows + (n,))
        v[..., ::3] = 0.0
        v[..., 1::3] = -0.0
    elif dist == "onebin":
        v = 256.0 + rng.random(rows + (n,)) * 31.0                  # all keys share the top 12 bits
    elif dist == "allequal":
        v = np.full(rows + (n,), 3.25)
    else:
        v = -np.abs(rng.standard_normal(rows + (n,))) * 1e-3 - 1e-30
    S[..., :n] = v.astype(np.float32)
    _check_topk_exact(fb, S, n, b)


def test_topk_denormals_and_extremes(fb):
    n = 777
    v = np.zeros(832, dtype=np.float32)
    rng = np.random.default_rng(5)
    v[:n] = rng.choice(np.array([1e-45, -1e-45, 1e-40, -1e-40, 3.4e38, -3.4e38, np.inf, -np.inf, 0.0, -0.0, 1.0],
                                dtype=np.float32), size=n)
    for b in (1, 10, 300, 776):
        _check_topk_exact(fb, v[None, None, :].copy(), n, b)


def test_attend_matches_oracle_on_the_oracle_set(fb, case):
    from tests.gpu_util import to_host
    name, w, x = case
    d = _dev(w, x)
    print("attend", name, flush=True)
    S_ref, _ = O.score(x["q"], x["K"], x["fc_idx"], w.n_ctx)
    T_ref = O.topk(S_ref.astype(np.float32), w.budget, w.n_ctx)
    # hand the kernel the set in a scrambled order: the result may not depend on it
    rng = np.random.default_rng(1)
    T_scr = np.stack([np.stack([rng.permutation(T_ref[b, h]) for h in range(w.n_kv_heads)]) for b in range(w.batch)])
    d.T.copy_(torch.from_numpy(T_scr.astype(np.int32)))
    fb.fasa_sparse_attend(d.shape, d.q, d.K, d.V, d.T, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    ref = O.sparse_attend(x["q"], x["K"], x["V"], T_ref)
    err = np.abs(to_host(d.O).astype(np.float64) - ref).max()
    print("  max abs err", err, flush=True)
    assert err <= OUT_ATOL


def test_dense_attend_matches_oracle(fb, case):
    from tests.gpu_util import to_host
    name, w, x = case
    d = _dev(w, x)
    print("dense", name, flush=True)
    fb.fasa_dense_attend(d.shape, d.q, d.K, d.V, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    ref = O.dense_attend(x["q"], x["K"], x["V"], w.n_ctx)
    err = np.abs(to_host(d.O).astype(np.float64) - ref).max()
    print("  max abs err", err, flush=True)
    assert err <= OUT_ATOL


def test_attend_invariants_that_expose_dropped_or_doubled_rows(fb):
    """Zero query -> uniform weights -> the plain mean of the selected V rows (every row counts
    exactly once); constant V -> that constant; one selected token -> its V row."""
    from tests.gpu_util import to_host
    w, x = _case(3, batch=2, n_ctx=1237, budget=389)      # G = 7, ragged split tail
    rng = np.random.default_rng(3)
    T = np.stack([np.stack([rng.choice(w.n_ctx, size=w.budget, replace=False) for _ in range(w.n_kv_heads)])
                  for _ in range(w.batch)]).astype(np.int32)
    x0 = dict(x); x0["q"] = np.zeros_like(x["q"])
    d = _dev(w, x0)
    d.T.copy_(torch.from_numpy(T))
    fb.fasa_sparse_attend(d.shape, d.q, d.K, d.V, d.T, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    V64 = W.storage_to_f64(x["V"])
    G = w.group
    got = to_host(d.O).astype(np.float64)
    for b in range(w.batch):
        for hq in range(w.n_q_heads):
            np.testing.assert_allclose(got[b, hq], V64[b, hq // G, T[b, hq // G]].mean(0), rtol=0, atol=2e-6)
    # constant V
    c = W.to_storage(np.linspace(-2, 2, 128), w.dtype)
    xc = dict(x); xc["V"] = np.broadcast_to(c, x["V"].shape).copy()
    d = _dev(w, xc)
    d.T.copy_(torch.from_numpy(T))
    fb.fasa_sparse_attend(d.shape, d.q, d.K, d.V, d.T, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    np.testing.assert_allclose(to_host(d.O), np.broadcast_to(W.storage_to_f64(c), (w.batch, w.n_q_heads, 128)),
                               rtol=0, atol=1e-5)
    # budget 1
    w1 = w.scaled(budget=1)
    d = _dev(w1, x)
    T1 = T[:, :, :1].copy()
    d.T.copy_(torch.from_numpy(T1))
    fb.fasa_sparse_attend(d.shape, d.q, d.K, d.V, d.T, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    got = to_host(d.O)
    for b in range(w.batch):
        for hq in range(w.n_q_heads):
            np.testing.assert_array_equal(got[b, hq].astype(np.float64), V64[b, hq // G, T1[b, hq // G, 0]])


@pytest.mark.parametrize("G", [1, 2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_every_gqa_group_size(fb, G, dtype):
    """All template instances of the attention kernels (group sizes 1..8, both storage types), with a
    ragged list length, plus the fused step on the same shape."""
    from tests.gpu_util import to_host
    w = W.WORKLOADS[1].scaled(batch=2, n_kv_heads=3, n_q_heads=3 * G, n_ctx=1900 + G, budget=150 + 3 * G,
                              n_fc=5 + 4 * G, dtype=dtype)
    x = W.make_inputs(w, n_cap=(w.n_ctx + 63) // 64 * 64)
    d = _dev(w, x)
    d.pack()
    print("gqa", G, dtype, flush=True)
    fb.fasa_decode_step(d.shape, d.q, d.K, d.V, d.Kp, d.fc_idx, None, None, d.S, d.T, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    S_ref, D_ref = O.score(x["q"], x["K"], x["fc_idx"], w.n_ctx)
    S = to_host(d.S)[:, :, :w.n_ctx].astype(np.float64)
    assert np.all(np.abs(S - S_ref) <= SCORE_RTOL * np.maximum(np.abs(S_ref), D_ref))
    T = np.sort(to_host(d.T), -1)
    np.testing.assert_array_equal(T, O.topk(to_host(d.S)[:, :, :w.n_ctx], w.budget, w.n_ctx))   # same float32 scores
    ref = O.sparse_attend(x["q"], x["K"], x["V"], T)
    assert np.abs(to_host(d.O) - ref).max() <= OUT_ATOL
    fb.fasa_dense_attend(d.shape, d.q, d.K, d.V, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    assert np.abs(to_host(d.O) - O.dense_attend(x["q"], x["K"], x["V"], w.n_ctx)).max() <= OUT_ATOL


def test_strided_kv_cache(fb):
    """K and V living in a larger allocation (row pitch 160 elements, head/batch pitches padded)."""
    from tests.gpu_util import to_host, to_dev
    w, x = _case(1, n_ctx=700, budget=90, n_kv_heads=2, n_q_heads=8, batch=2)
    n_cap = 704
    sn, sh = 160, 704 * 160 + 64
    sb = 2 * sh + 128
    big = np.zeros((2 * sb,), dtype=np.uint16)
    bigv = np.zeros((2 * sb,), dtype=np.uint16)
    for b in range(2):
        for h in range(2):
            for arr, src in ((big, x["K"]), (bigv, x["V"])):
                view = arr[b * sb + h * sh: b * sb + h * sh + n_cap * sn].reshape(n_cap, sn)
                view[:, :128] = src[b, h]
    d = _dev(w, x)
    Kd, Vd = to_dev(big), to_dev(bigv)
    shape = fb.make_shape(2, 8, 2, 128, 16, 700, n_cap, 90, "bf16", sb, sh, sn)
    fb.fasa_pack_kcache(shape, Kd, d.fc_idx, d.Kp, 0, 700)
    nbytes = fb.fasa_workspace_bytes(shape)
    ws = torch.full((nbytes,), 0x33, dtype=torch.uint8, device="cuda")
    fb.fasa_workspace_init(shape, ws, nbytes)
    fb.fasa_decode_step(shape, d.q, Kd, Vd, d.Kp, d.fc_idx, None, None, d.S, d.T, d.O, ws, nbytes)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(d.Kp, np.uint16)[:, :, :, :700], O.pack_kcache(x["K"], x["fc_idx"], 700))
    T = np.sort(to_host(d.T), axis=-1)
    ref = O.sparse_attend(x["q"], x["K"], x["V"], T)
    assert np.abs(to_host(d.O) - ref).max() <= OUT_ATOL


def test_launch_plans_assume_this_device():
    """The launch plans and workspace sizes are computed on the host for a fixed number of compute units
    (fasa_workspace_bytes is a pure function): that number must be the device's."""
    import os
    import re
    src = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2602_03152_amd", "csrc",
                            "fasa_internal.h")).read()
    assumed = int(re.search(r"constexpr int kAssumedCUs = (\d+);", src).group(1))
    assert torch.cuda.get_device_properties(0).multi_processor_count == assumed
