"""GPU parity of the paged-cache entry points: K/V rows scattered over a pool of fixed-size blocks
behind a block table.  Paging is a storage layout, not arithmetic: the oracle runs on the logical
(contiguous) view of the same cache."""
import numpy as np
import pytest
import torch

from oracle import fasa_oracle as O
from paper_2602_03152_amd import workload as W
from tests.test_gpu_decode_step import compare_step
from tests.test_gpu_ragged import compare_ragged, i32_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fb():
    from paper_2602_03152_amd import binding
    return binding


def scatter_to_pool(K, V, page, layout, seed, spare=3):
    """Logical caches [B][Hkv][n_cap][D] -> (poolK, poolV, table, strides) with the blocks of every
    sequence at random pool positions and `spare` pool blocks that belong to nobody (poisoned)."""
    B, Hkv, n_cap, D = K.shape
    assert n_cap % page == 0
    nblk = n_cap // page
    n_pool = B * nblk + spare
    rng = np.random.default_rng(seed)
    table = rng.permutation(n_pool)[: B * nblk].reshape(B, nblk).astype(np.int32)
    poison = np.uint16(0x7FC1) if K.dtype == np.uint16 else np.float32(np.nan)
    if layout == "token_major":          # [block][token][head][dim]
        shp, strides = (n_pool, page, Hkv, D), dict(sb=page * Hkv * D, sn=Hkv * D, sh=D)
    else:                                # [block][head][token][dim]
        shp, strides = (n_pool, Hkv, page, D), dict(sb=Hkv * page * D, sh=page * D, sn=D)
    pk, pv = np.full(shp, poison, dtype=K.dtype), np.full(shp, poison, dtype=V.dtype)
    for b in range(B):
        for j in range(nblk):
            kb, vb = K[b, :, j * page:(j + 1) * page], V[b, :, j * page:(j + 1) * page]     # [Hkv][page][D]
            if layout == "token_major":
                pk[table[b, j]], pv[table[b, j]] = kb.transpose(1, 0, 2), vb.transpose(1, 0, 2)
            else:
                pk[table[b, j]], pv[table[b, j]] = kb, vb
    return pk, pv, table, strides


def gather_from_pool(pool, table, page, layout):
    """Inverse of scatter_to_pool: the logical view [B][Hkv][n_cap][D]."""
    B, nblk = table.shape
    blocks = pool[table.reshape(-1)]                       # [B*nblk][...]
    if layout == "token_major":
        blocks = blocks.transpose(0, 2, 1, 3)              # -> [.., head, token, dim]
    Hkv, D = blocks.shape[1], blocks.shape[3]
    return blocks.reshape(B, nblk, Hkv, page, D).transpose(0, 2, 1, 3, 4).reshape(B, Hkv, nblk * page, D)


class PagedDevice:
    def __init__(self, fb, w, x, page, layout, seed=7, pairing="half"):
        from tests.gpu_util import to_dev
        self.w, self.page, self.layout = w, page, layout
        self.n_cap = x["n_cap"]
        pk, pv, table, st = scatter_to_pool(x["K"], x["V"], page, layout, seed)
        self.table_host = table
        self.K, self.V, self.table = to_dev(pk), to_dev(pv), to_dev(table)
        self.q, self.fc_idx = to_dev(x["q"]), to_dev(x["fc_idx"])
        tdt = torch.int16 if w.dtype == "bf16" else torch.float32
        self.st = np.uint16 if w.dtype == "bf16" else np.float32
        self.shape = fb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_fc, w.n_ctx, self.n_cap,
                                   w.budget, w.dtype, kv_stride_b=st["sb"], kv_stride_h=st["sh"], kv_stride_n=st["sn"],
                                   pairing=pairing)
        self.paging = fb.make_paging(self.table, page, pk.shape[0])
        self.Kp = torch.zeros((w.batch, w.n_kv_heads, w.n_fc, self.n_cap, 2), dtype=tdt, device="cuda")
        self.S = torch.full((w.batch, w.n_kv_heads, self.n_cap), float("nan"), dtype=torch.float32, device="cuda")
        self.bsel = min(w.budget, w.n_ctx)
        self.T = torch.full((w.batch, w.n_kv_heads, self.bsel), -1, dtype=torch.int32, device="cuda")
        self.O = torch.full((w.batch, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.float32, device="cuda")
        self.ws_bytes = fb.fasa_workspace_bytes(self.shape)
        self.ws = torch.full((self.ws_bytes,), 0x5A, dtype=torch.uint8, device="cuda")
        fb.fasa_workspace_init(self.shape, self.ws, self.ws_bytes)


CASES = {
    "bf16_p16_token_major": dict(cid=1, page=16, layout="token_major", n_ctx=5000 + 19, budget=313),
    "bf16_p64_head_major": dict(cid=2, page=64, layout="head_major", batch=3, n_ctx=3001, budget=256),
    "bf16_p256_gqa7": dict(cid=3, page=256, layout="token_major", batch=2, n_ctx=4099, budget=775, cap=4352),
    "f32_p32": dict(cid=0, page=32, layout="head_major", n_ctx=2049, budget=65),
    "p1": dict(cid=1, page=1, layout="token_major", n_ctx=300, budget=40, n_kv_heads=2, n_q_heads=8),
    "budget_ge_n": dict(cid=1, page=16, layout="token_major", n_ctx=130, budget=4096, n_kv_heads=2, n_q_heads=8),
}


def _workload(c):
    c = dict(c)
    cid, page, layout, cap = c.pop("cid"), c.pop("page"), c.pop("layout"), c.pop("cap", None)
    w = W.WORKLOADS[cid].scaled(**c)
    n_cap = cap or (w.n_ctx + 63) // 64 * 64
    return w, W.make_inputs(w, n_cap=n_cap), page, layout


@pytest.mark.parametrize("name", list(CASES))
def test_paged_pack_and_step_match_oracle(fb, name):
    from tests.gpu_util import Device, to_host
    w, x, page, layout = _workload(CASES[name])
    print("paged", name, flush=True)
    d = PagedDevice(fb, w, x, page, layout)
    fb.fasa_pack_kcache_paged(d.shape, d.paging, d.K, d.fc_idx, d.Kp, 0, w.n_ctx)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(d.Kp, d.st)[:, :, :, :w.n_ctx], O.pack_kcache(x["K"], x["fc_idx"], w.n_ctx))
    fb.fasa_decode_step_paged(d.shape, d.paging, d.q, d.K, d.V, d.Kp, d.fc_idx, None, None, None, None,
                              d.S, d.T, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    n_diff, o_err = compare_step(w, x["q"], x["K"], x["V"], x["fc_idx"], d, w.n_ctx, w.budget)
    print("  set diff vs oracle:", n_diff, " max |O err|:", o_err, flush=True)
    # same cache stored contiguously, same kernels: identical scores and set
    e = Device(w, x)
    e.pack()
    fb.fasa_decode_step(e.shape, e.q, e.K, e.V, e.Kp, e.fc_idx, None, None, e.S, e.T, e.O, e.ws, e.ws_bytes)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(d.S)[:, :, :w.n_ctx], to_host(e.S)[:, :, :w.n_ctx])
    np.testing.assert_array_equal(np.sort(to_host(d.T), -1), np.sort(to_host(e.T), -1))
    assert float(np.abs(to_host(d.O) - to_host(e.O)).max()) <= 2e-5
    # a second call on the same workspace
    fb.fasa_decode_step_paged(d.shape, d.paging, d.q, d.K, d.V, d.Kp, d.fc_idx, None, None, None, None,
                              d.S, d.T, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(np.sort(to_host(d.T), -1), np.sort(to_host(e.T), -1))


def test_paged_ragged_append_lands_in_the_right_blocks(fb):
    """Mixed lengths on a paged cache, with an append: the new rows go to the pool slot the table
    names for position N_b - 1 (blocks of other sequences and spare blocks untouched), and every
    sequence equals the oracle on its own logical prefix."""
    from tests.gpu_util import to_dev, to_host
    lens = [3000, 517, 64, 1]
    page, layout = 16, "token_major"
    w = W.WORKLOADS[2].scaled(batch=len(lens), n_ctx=3008, budget=600)
    x = W.make_inputs(w, n_cap=3008)
    d = PagedDevice(fb, w, x, page, layout)
    fb.fasa_pack_kcache_paged(d.shape, d.paging, d.K, d.fc_idx, d.Kp, 0, w.n_ctx)
    a = W.make_append(w, x["fc_idx"], step=1, n_before=lens[0])
    K, V = x["K"].copy(), x["V"].copy()
    for b, n in enumerate(lens):
        K[b, :, n - 1], V[b, :, n - 1] = a["k_new"][b], a["v_new"][b]        # lands at position N_b - 1
    budgets = [max(1, W.budget_fraction(n)) for n in lens]
    fb.fasa_decode_step_paged(d.shape, d.paging, to_dev(a["q"]), d.K, d.V, d.Kp, d.fc_idx, to_dev(a["k_new"]),
                              to_dev(a["v_new"]), i32_dev(lens), i32_dev(budgets), d.S, d.T, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    pk, pv = to_host(d.K, d.st), to_host(d.V, d.st)
    ek, ev, _, _ = scatter_to_pool(K, V, page, layout, seed=7)                 # same seed: same table
    np.testing.assert_array_equal(pk, ek)                                       # incl. the poisoned spare blocks
    np.testing.assert_array_equal(pv, ev)
    np.testing.assert_array_equal(gather_from_pool(pk, d.table_host, page, layout), K)
    for b, n in enumerate(lens):
        np.testing.assert_array_equal(to_host(d.Kp, d.st)[b:b + 1, :, :, :n], O.pack_kcache(K[b:b + 1], x["fc_idx"], n))
    compare_ragged(w, a["q"], K, V, x["fc_idx"], d, lens, budgets, min(w.budget, w.n_ctx))


def test_stray_table_entries_are_clamped(fb):
    """The table is device data the host cannot validate: entries outside the pool are clamped into
    it, so the call stays inside the pool allocation (the result is then unspecified)."""
    w = W.WORKLOADS[1].scaled(n_ctx=500, budget=50, n_kv_heads=2, n_q_heads=8)
    x = W.make_inputs(w, n_cap=512)
    d = PagedDevice(fb, w, x, 16, "token_major")
    bad = d.table.clone()
    bad[0, 3] = -5
    bad[0, 7] = 10 ** 9
    paging = fb.make_paging(bad, 16, int(d.K.shape[0]))
    fb.fasa_pack_kcache_paged(d.shape, paging, d.K, d.fc_idx, d.Kp, 0, w.n_ctx)
    fb.fasa_decode_step_paged(d.shape, paging, d.q, d.K, d.V, d.Kp, d.fc_idx, None, None, None, None,
                              d.S, d.T, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    T = d.T.cpu().numpy()
    assert T.min() >= 0 and T.max() < w.n_ctx


def _random_paged_cases(n_cases, seed=20260203):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n_cases):
        G, hkv, batch = int(rng.integers(1, 9)), int(rng.choice([1, 2, 4, 8])), int(rng.integers(1, 5))
        n_max = int(rng.integers(130, 5000))
        budget = int(rng.integers(1, n_max + 1))
        out.append(dict(G=G, hkv=hkv, batch=batch, page=int(rng.choice([1, 8, 16, 64, 128])),
                        layout=str(rng.choice(["token_major", "head_major"])), n_max=n_max,
                        n_fc=int(rng.choice([8, 16, 24, 32, int(rng.integers(1, 65))])),
                        dtype="bf16" if rng.random() < 0.7 else "f32", budget=budget,
                        lens=[int(rng.integers(1, n_max + 1)) for _ in range(batch)],
                        buds=[int(rng.integers(1, budget + 1)) for _ in range(batch)]))
    return out


@pytest.mark.parametrize("case", range(12))
def test_random_ragged_paged_steps_with_append(fb, case):
    """Seeded sweep over group size, head count, page size, block layout, F, storage type, lengths and
    budgets: a ragged step with an append on a paged cache, every sequence against the oracle."""
    from tests.gpu_util import to_dev
    c = _random_paged_cases(12)[case]
    print("random paged", case, c, flush=True)
    w = W.WORKLOADS[1].scaled(batch=c["batch"], n_kv_heads=c["hkv"], n_q_heads=c["hkv"] * c["G"], n_fc=c["n_fc"],
                              n_ctx=c["n_max"], budget=c["budget"], dtype=c["dtype"])
    x = W.make_inputs(w, n_cap=(c["n_max"] + 127) // 128 * 128)
    d = PagedDevice(fb, w, x, c["page"], c["layout"], seed=case)
    fb.fasa_pack_kcache_paged(d.shape, d.paging, d.K, d.fc_idx, d.Kp, 0, c["n_max"])
    a = W.make_append(w, x["fc_idx"], step=1, n_before=c["lens"][0])
    K, V = x["K"].copy(), x["V"].copy()
    for b, n in enumerate(c["lens"]):
        K[b, :, n - 1], V[b, :, n - 1] = a["k_new"][b], a["v_new"][b]
    fb.fasa_decode_step_paged(d.shape, d.paging, to_dev(a["q"]), d.K, d.V, d.Kp, d.fc_idx, to_dev(a["k_new"]),
                              to_dev(a["v_new"]), i32_dev(c["lens"]), i32_dev(c["buds"]), d.S, d.T, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    compare_ragged(w, a["q"], K, V, x["fc_idx"], d, c["lens"], [min(b_, n) for b_, n in zip(c["buds"], c["lens"])],
                   min(c["budget"], c["n_max"]))
