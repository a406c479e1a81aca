"""GPU parity of the ragged decode step (per-sequence lengths and budgets read from device arrays)
against the CPU oracle run once per sequence, and of one captured HIP graph of it replayed over a
growing cache."""
import numpy as np
import pytest
import torch

from oracle import fasa_oracle as O
from paper_2602_03152_amd import workload as W
from tests.test_gpu_decode_step import SCORE_RTOL, OUT_ATOL, check_selection

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fb():
    from paper_2602_03152_amd import binding
    return binding


def i32_dev(v):
    return torch.tensor(list(v), dtype=torch.int32, device="cuda")


def compare_ragged(w, q, K, V, fc_idx, d, lens, budgets, pitch):
    """Every sequence against the oracle at its own (N_b, B_b); returns max |O err|."""
    from tests.gpu_util import to_host
    S_dev = to_host(d.S)
    T_dev = to_host(d.T).reshape(-1)[: w.batch * w.n_kv_heads * pitch].reshape(w.batch, w.n_kv_heads, pitch)
    O_dev = to_host(d.O).astype(np.float64)
    worst = 0.0
    for b in range(w.batch):
        n, bud = int(lens[b]), int(budgets[b])
        bsel = min(bud, n)
        S_ref, D_ref = O.score(q[b:b + 1], K[b:b + 1], fc_idx, n)
        S = S_dev[b:b + 1, :, :n].astype(np.float64)
        assert np.all(np.abs(S - S_ref) <= SCORE_RTOL * np.maximum(np.abs(S_ref), D_ref)), b
        T = T_dev[b:b + 1, :, :bsel]
        check_selection(S_ref, D_ref, T, bud, n)
        O_ref = O.sparse_attend(q[b:b + 1], K[b:b + 1], V[b:b + 1], T)
        err = float(np.abs(O_dev[b:b + 1] - O_ref).max())
        assert err <= OUT_ATOL, (b, err)
        worst = max(worst, err)
    return worst


CASES = {
    # lengths, budgets (None = the shape's), shape budget
    "bf16_mixed": dict(cid=2, lens=[3001, 1, 130, 2048], budgets=[256, 5, 300, 300], budget=300),
    "bf16_uniform_budget": dict(cid=2, lens=[2500, 64, 65, 4100], budgets=None, budget=200, n_max=4100),
    "f32_g1": dict(cid=0, lens=[2049], budgets=[65], budget=128, n_max=2500),
    "gqa7": dict(cid=3, lens=[4099, 3000], budgets=[775, 567], budget=800),
}


@pytest.mark.parametrize("name", list(CASES))
def test_ragged_step_matches_oracle_per_sequence(fb, name):
    from tests.gpu_util import Device, to_host
    c = CASES[name]
    lens = c["lens"]
    n_max = c.get("n_max", max(lens))
    w = W.WORKLOADS[c["cid"]].scaled(batch=len(lens), n_ctx=n_max, budget=c["budget"])
    x = W.make_inputs(w, n_cap=(n_max + 63) // 64 * 64)
    print("ragged", name, lens, c["budgets"], flush=True)
    d = Device(w, x)
    d.pack()
    n_dev = i32_dev(lens)
    b_dev = None if c["budgets"] is None else i32_dev(c["budgets"])
    fb.fasa_decode_step_ragged(d.shape, d.q, d.K, d.V, d.Kp, d.fc_idx, None, None, n_dev, b_dev,
                               d.S, d.T, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    budgets = [min(c["budget"], v) for v in (c["budgets"] or [c["budget"]] * len(lens))]
    pitch = min(w.budget, w.n_ctx)
    err = compare_ragged(w, x["q"], x["K"], x["V"], x["fc_idx"], d, lens, budgets, pitch)
    print("  max |O err|:", err, flush=True)
    # nothing is written beyond a sequence's own extent
    S, T = to_host(d.S), to_host(d.T)
    for b, n in enumerate(lens):
        assert np.isnan(S[b, :, n:]).all()
        assert (T[b, :, min(budgets[b], n):] == -1).all()
    # the workspace is left prepared: a second call gives the same sets
    T0 = [np.sort(T[b, :, :min(budgets[b], n)], -1) for b, n in enumerate(lens)]
    fb.fasa_decode_step_ragged(d.shape, d.q, d.K, d.V, d.Kp, d.fc_idx, None, None, n_dev, b_dev,
                               d.S, d.T, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    T = to_host(d.T)
    for b, n in enumerate(lens):
        np.testing.assert_array_equal(np.sort(T[b, :, :min(budgets[b], n)], -1), T0[b])


def test_ragged_with_equal_lengths_equals_uniform_call(fb):
    from tests.gpu_util import Device, to_host
    w = W.WORKLOADS[2].scaled(batch=3, n_ctx=5003, budget=400)
    x = W.make_inputs(w, n_cap=5056)
    d, e = Device(w, x), Device(w, x)
    d.pack(); e.pack()
    fb.fasa_decode_step(d.shape, d.q, d.K, d.V, d.Kp, d.fc_idx, None, None, d.S, d.T, d.O, d.ws, d.ws_bytes)
    fb.fasa_decode_step_ragged(e.shape, e.q, e.K, e.V, e.Kp, e.fc_idx, None, None, i32_dev([5003] * 3),
                               i32_dev([400] * 3), e.S, e.T, e.O, e.ws, e.ws_bytes)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(e.S)[:, :, :w.n_ctx], to_host(d.S)[:, :, :w.n_ctx])
    np.testing.assert_array_equal(np.sort(to_host(e.T), -1), np.sort(to_host(d.T), -1))
    assert float(np.abs(to_host(e.O) - to_host(d.O)).max()) <= 2e-5


def test_lengths_outside_the_shape_are_clamped(fb):
    """Lengths and budgets are device data the host cannot validate: the kernels clamp them into
    [1, upper bound], so stray values can never become stray addresses."""
    from tests.gpu_util import Device
    w = W.WORKLOADS[2].scaled(batch=4, n_ctx=1000, budget=100)
    x = W.make_inputs(w, n_cap=1024)
    d = Device(w, x)
    d.pack()
    fb.fasa_decode_step_ragged(d.shape, d.q, d.K, d.V, d.Kp, d.fc_idx, None, None,
                               i32_dev([0, -7, 10 ** 9, 1000]), i32_dev([0, 50, -1, 10 ** 9]),
                               d.S, d.T, d.O, d.ws, d.ws_bytes)
    torch.cuda.synchronize()
    compare_ragged(w, x["q"], x["K"], x["V"], x["fc_idx"], d, [1, 1, 1000, 1000], [1, 1, 1, 100], 100)


def test_one_graph_serves_a_growing_ragged_batch(fb):
    """One captured graph of the ragged step (append + score + select + attend), replayed with the
    lengths advanced on the device between replays; every replay is checked against the oracle,
    with eager work and synchronisations between replays."""
    from tests.gpu_util import Device, to_dev, to_host
    lens = [3000, 517, 64]
    steps = 5
    n_max = max(lens) + steps
    w = W.WORKLOADS[3].scaled(batch=len(lens), n_ctx=n_max, budget=600)
    x = W.make_inputs(w, n_cap=(n_max + 63) // 64 * 64)
    K, V = x["K"].copy(), x["V"].copy()
    d = Device(w, x)
    d.pack()
    n_dev = i32_dev(lens)
    b_dev = i32_dev([W.budget_fraction(n) for n in lens])
    # eager warm-up before the capture: re-appends each sequence's own last row (no change)
    k_last = np.stack([K[b, :, n - 1] for b, n in enumerate(lens)])
    v_last = np.stack([V[b, :, n - 1] for b, n in enumerate(lens)])
    q_buf, k_buf, v_buf = to_dev(x["q"]), to_dev(k_last), to_dev(v_last)

    def step():
        fb.fasa_decode_step_ragged(d.shape, q_buf, d.K, d.V, d.Kp, d.fc_idx, k_buf, v_buf, n_dev, b_dev,
                                   d.S, d.T, d.O, d.ws, d.ws_bytes)

    step()
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(d.K, np.uint16), K)
    compare_ragged(w, x["q"], K, V, x["fc_idx"], d, lens, [W.budget_fraction(n) for n in lens],
                   min(w.budget, w.n_ctx))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step()
    torch.cuda.synchronize()

    cur = list(lens)
    for s in range(1, steps + 1):
        a = W.make_append(w, x["fc_idx"], step=s, n_before=cur[0])
        for b in range(w.batch):
            K[b, :, cur[b]] = a["k_new"][b]; V[b, :, cur[b]] = a["v_new"][b]
            cur[b] += 1
        budgets = [W.budget_fraction(n) for n in cur]
        q_buf.copy_(to_dev(a["q"])); k_buf.copy_(to_dev(a["k_new"])); v_buf.copy_(to_dev(a["v_new"]))
        n_dev.add_(1)
        b_dev.copy_(i32_dev(budgets))
        print("graph replay", s, cur, budgets, flush=True)
        g.replay()
        torch.cuda.synchronize()
        for b in range(w.batch):
            np.testing.assert_array_equal(to_host(d.K, np.uint16)[b, :, :cur[b]], K[b, :, :cur[b]])
            np.testing.assert_array_equal(to_host(d.V, np.uint16)[b, :, :cur[b]], V[b, :, :cur[b]])
            np.testing.assert_array_equal(to_host(d.Kp, np.uint16)[b:b + 1, :, :, :cur[b]],
                                          O.pack_kcache(K[b:b + 1], x["fc_idx"], cur[b]))
        compare_ragged(w, a["q"], K, V, x["fc_idx"], d, cur, budgets, min(w.budget, w.n_ctx))
