#!/usr/bin/env python3
"""Benchmark of the FASA decode hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--no-cpu-baseline]

A "step" is one fasa_decode_step (scores + histogram, then selection and sparse attention in one
kernel) over one batch of synthetic, HBM-resident input shaped like the chosen workload (default: the
Llama-3-8B-shaped layer at 32k context, budget 2048, 16 dominant FCs).  The step rotates over R
independent buffer sets so that the bytes a step touches have left the 256 MB last-level cache before
their set comes round again.

Passes, all inside this process:
  timed      W warm-up + exactly K steps launched eagerly on one stream, bracketed by synchronize;
             `value` = microseconds per step, `step_roofline` = the step's algorithmic bytes over that
             time against the HBM peak.  The same steps as one captured HIP graph are timed too
             (`graph_us_per_step`), every replay checked against the eager result.
  kernels    the same K steps with the library's per-kernel timestamps on: average GPU execution time
             of every kernel of the path -> `kernels`; `roofline` describes the kernel that takes the
             longest.  `traffic` quotes the HBM bytes per launch measured with rocprofv3 counters
             (profiles/), only while the kernel sources are the ones they were measured on.
  baselines  the library's own full-KV decode kernel on the same buffers (`dense_baseline`) and the
             CPU oracle timed on the host cores (`cpu_baseline`).
  others     the remaining workload shapes, timed briefly (`other_workloads`).
Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X published HBM3E bandwidth
LLC_BYTES = 256 << 20         # last-level (memory-side) cache the rotation has to defeat

# HBM traffic per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, scaled by
# what the same counters read for a plain copy kernel of known size (see profiles/).  Keyed by
# (workload config id, kernel name); bytes per launch.  None = not measured yet.
MEASURED_TRAFFIC = {
    "source_hash": "edb18815d50a8b3a",   # source_hash() of the kernels the counters were taken on
    # profiles/decode_step_tiny_1head_f32_n4096_hbm_counters.txt  (read + written)
    (0, "fasa_dense_attend"): 4327810 + 39456,
    (0, "fasa_score_hist"): 601133 + 21632,
    (0, "fasa_select"): 135682 + 19860,
    (0, "fasa_sparse_attend"): 321111 + 2976,
    # profiles/decode_step_llama3_8b_layer_n32768_b2048_hbm_counters.txt  (read + written)
    (1, "fasa_dense_attend"): 135500293 + 2162944,
    (1, "fasa_score_hist"): 16890367 + 1323072,
    (1, "fasa_select_attend"): 10539073 + 1277719,
    # profiles/decode_step_batch16_n16384_b256_hbm_counters.txt  (read + written)
    (2, "fasa_dense_attend"): 1076170460 + 4558848,
    (2, "fasa_score_hist"): 134446381 + 10223337,
    (2, "fasa_select_attend"): 27812435 + 3344355,
    # profiles/decode_step_longcot_batch8_gqa7_n32768_hbm_counters.txt  (read + written)
    (3, "fasa_dense_attend"): 538972426 + 3879936,
    (3, "fasa_score_hist"): 67269630 + 5386022,
    (3, "fasa_select_attend"): 108590458 + 5034110,
    # profiles/decode_step_verylong_n131072_f32fc_b1024_hbm_counters.txt  (read + written)
    (4, "fasa_dense_attend"): 538112279 + 2162944,
    (4, "fasa_score_hist"): 134514100 + 4998817,
    (4, "fasa_select_attend"): 9948239 + 2300813,
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def growing(args, w, fb, W, np, torch):
    """Growing-cache decode loop (the long-CoT workload): every step appends one K/V row per (b, h) to
    the cache and to the packed copy inside fasa_decode_step, then scores, selects and attends over
    the new length.  All steps are enqueued on one stream; one synchronize at the end."""
    steps = args.growing
    n0 = w.n_ctx
    n_cap = (n0 + steps + 63) // 64 * 64
    x = W.make_inputs(w, n_cap=n_cap)
    dev = lambda a: torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()
    tdt = torch.int16 if w.dtype == "bf16" else torch.float32
    q0, K, V, fc = dev(x["q"]), dev(x["K"]), dev(x["V"]), dev(x["fc_idx"])
    mk = lambda n: fb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_fc, n, n_cap,
                                 W.budget_fraction(n), w.dtype)
    shapes = [mk(n0 + s) for s in range(steps + 1)]
    ws_bytes = max(fb.fasa_workspace_bytes(sh) for sh in shapes)
    ws = torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda")
    fb.fasa_workspace_init(shapes[0], ws, ws_bytes)
    Kp = torch.zeros((w.batch, w.n_kv_heads, w.n_fc, n_cap, 2), dtype=tdt, device="cuda")
    S = torch.zeros((w.batch, w.n_kv_heads, n_cap), dtype=torch.float32, device="cuda")
    T = torch.zeros((w.batch, w.n_kv_heads, W.budget_fraction(n0 + steps)), dtype=torch.int32, device="cuda")
    O = torch.zeros((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    fb.fasa_pack_kcache(shapes[0], K, fc, Kp, 0, n0)
    app = [W.make_append(w, x["fc_idx"], step=s, n_before=n0 + s - 1) for s in range(1, steps + 1)]
    qs = [q0] + [dev(a["q"]) for a in app]
    kn = [None] + [dev(a["k_new"]) for a in app]
    vn = [None] + [dev(a["v_new"]) for a in app]
    torch.cuda.synchronize()

    def run(first, last):
        for s in range(first, last + 1):
            fb.fasa_decode_step(shapes[s], qs[s], K, V, Kp, fc, kn[s], vn[s], S, T, O, ws, ws_bytes)

    run(0, min(args.warmup, steps))                   # warm-up re-appends the same rows: idempotent
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    ev[0].record(); run(0, 0); ev[1].record()
    run(1, steps - 1)
    ev[2].record(); run(steps, steps); ev[3].record()
    torch.cuda.synchronize()
    total_us = ev[0].elapsed_time(ev[3]) * 1e3
    per_step = total_us / (steps + 1)
    alg0 = W.algorithmic_bytes(w)["alg"]
    out = {
        "metric": "us_per_decode_step", "value": round(per_step, 3), "unit": "us", "n_gpus": 1,
        "steps": steps + 1, "warmup": args.warmup, "ms_per_step": round(per_step / 1e3, 6),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "accum_dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name + "_growing", "batch": w.batch, "n_q_heads": w.n_q_heads,
                   "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "n_ctx_first": n0, "n_ctx_last": n0 + steps,
                   "budget_first": W.budget_fraction(n0), "budget_last": W.budget_fraction(n0 + steps),
                   "n_fc": w.n_fc, "storage_dtype": w.dtype, "launch": "eager", "buffer_sets": 1},
        "first_step_us": round(ev[0].elapsed_time(ev[1]) * 1e3, 3),
        "last_step_us": round(ev[2].elapsed_time(ev[3]) * 1e3, 3),
        "hbm": {"alg_bytes_first_step": alg0, "step_gbps": round(alg0 / per_step / 1e3, 1),
                "step_frac_of_peak": round(alg0 / per_step / 1e3 / HBM_PEAK_GBPS, 4)},
        "roofline": None, "cpu_baseline": None,
    }
    print(json.dumps(out), flush=True)


def offload(args, w, fb, W, np, torch):
    """Memory-optimised variant: Kp on the device, non-dominant key dims and values in pinned host
    memory.  The step is PCIe-bound: rows * B * ((d - 2F) + d) * e bytes cross the link per step."""
    PCIE_PEAK_GBPS = 64.0                                  # PCIe Gen5 x16, one direction
    x = W.make_inputs(w)
    n_cap = x["n_cap"]
    rows, e = w.batch * w.n_kv_heads, w.elem_bytes
    bsel = min(w.budget, w.n_ctx)
    dev = lambda a: torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()
    tdt = torch.int16 if w.dtype == "bf16" else torch.float32
    shape = fb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_fc, w.n_ctx, n_cap, w.budget, w.dtype)
    q, K, fc = dev(x["q"]), dev(x["K"]), dev(x["fc_idx"])
    nd = w.head_dim - 2 * w.n_fc
    Knd = torch.zeros((w.batch, w.n_kv_heads, n_cap, nd), dtype=tdt).pin_memory()
    Vh = torch.from_numpy(x["V"].view(np.int16) if x["V"].dtype == np.uint16 else x["V"]).pin_memory()
    Kp = torch.zeros((w.batch, w.n_kv_heads, w.n_fc, n_cap, 2), dtype=tdt, device="cuda")
    S = torch.zeros((w.batch, w.n_kv_heads, n_cap), dtype=torch.float32, device="cuda")
    T = torch.zeros((w.batch, w.n_kv_heads, bsel), dtype=torch.int32, device="cuda")
    O = torch.zeros((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    ws_bytes = fb.fasa_workspace_bytes(shape)
    ws = torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda")
    fb.fasa_workspace_init(shape, ws, ws_bytes)
    stage_bytes = fb.fasa_offload_stage_bytes(shape)
    stage = torch.empty((stage_bytes,), dtype=torch.uint8, device="cuda")
    fb.fasa_offload_split_kcache(shape, K, fc, Kp, Knd, 0, w.n_ctx)
    torch.cuda.synchronize()
    del K                                                  # the full key cache does not stay on the device

    def step():
        fb.fasa_offload_decode_step(shape, q, Kp, fc, Knd, Vh, None, None, S, T, O, ws, ws_bytes, stage, stage_bytes)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(args.steps):
        step()
    b.record()
    torch.cuda.synchronize()
    us = a.elapsed_time(b) / args.steps * 1e3
    fb.fasa_profile_reset(); fb.fasa_profile_enable(True)
    for _ in range(args.steps):
        step()
    prof = fb.profile_summary()
    fb.fasa_profile_enable(False); fb.fasa_profile_reset()
    pcie_bytes = rows * bsel * (nd + w.head_dim) * e
    g_us = prof["fasa_offload_gather"][1] / prof["fasa_offload_gather"][0] * 1e3
    gpu_cache = rows * (w.n_ctx * 2 * w.n_fc + bsel * nd + bsel * w.head_dim) * e      # App. C memory model
    full_cache = rows * w.n_ctx * 2 * w.head_dim * e
    out = {
        "metric": "us_per_decode_step", "value": round(us, 3), "unit": "us", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(us / 1e3, 6), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "accum_dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name + "_offload", "batch": w.batch, "n_q_heads": w.n_q_heads,
                   "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "n_ctx": w.n_ctx, "budget": bsel,
                   "n_fc": w.n_fc, "storage_dtype": w.dtype, "launch": "eager", "buffer_sets": 1},
        "roofline": {"bound": "pcie", "kernel": "fasa_offload_gather", "achieved": round(pcie_bytes / g_us / 1e3, 2),
                     "peak": PCIE_PEAK_GBPS, "unit": "GB/s", "frac": round(pcie_bytes / g_us / 1e3 / PCIE_PEAK_GBPS, 4),
                     "traffic": None},
        "kernels": {k: {"launches": n, "avg_us": round(ms / n * 1e3, 3)} for k, (n, ms) in prof.items()},
        "pcie_bytes_per_step": pcie_bytes,
        "device_cache_bytes": gpu_cache, "full_cache_bytes": full_cache,
        "cache_reduction": round(full_cache / gpu_cache, 3),
        "cpu_baseline": None,
    }
    print(json.dumps(out), flush=True)


def calibrate(args, w, fb, W, np, torch):
    """Offline calibration on the device: contextual agreement of every FC of every KV head with the
    full head, one query sample per call, then the dominant-FC choice on the host.  Reports the time
    per sample (the dominant work: d/2 + 1 scoring passes over the cache and d/2 + 1 top-K selections
    per KV head) and whether the planted dominant FCs of the synthetic workload come out."""
    n_samples, top_k = args.calibrate, min(w.budget, w.n_ctx)
    half = w.head_dim // 2
    x = W.make_inputs(w)
    n_cap = x["n_cap"]
    dev = lambda a: torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()
    tdt = torch.int16 if w.dtype == "bf16" else torch.float32
    shape = fb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, half, w.n_ctx, n_cap, top_k, w.dtype)
    K = dev(x["K"])
    fc_all = torch.arange(half, dtype=torch.int32, device="cuda").repeat(w.n_kv_heads, 1).contiguous()
    Kp_all = torch.zeros((w.batch, w.n_kv_heads, half, n_cap, 2), dtype=tdt, device="cuda")
    fb.fasa_pack_kcache(shape, K, fc_all, Kp_all, 0, w.n_ctx)
    nbytes = fb.fasa_calibration_workspace_bytes(shape, top_k)
    cws = torch.empty((nbytes,), dtype=torch.uint8, device="cuda")
    ca = torch.zeros((w.batch, w.n_kv_heads, half), dtype=torch.float32, device="cuda")
    q_host = [x["q"]] + [W.make_append(w, x["fc_idx"], step=s, n_before=w.n_ctx - 1)["q"] for s in range(1, n_samples)]
    qs = [dev(q) for q in q_host]
    fb.fasa_contextual_agreement(shape, qs[0], Kp_all, top_k, ca, cws, nbytes)         # warm-up
    torch.cuda.synchronize()
    ca.zero_()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for q in qs:
        fb.fasa_contextual_agreement(shape, q, Kp_all, top_k, ca, cws, nbytes)
    b.record()
    torch.cuda.synchronize()
    us = a.elapsed_time(b) / n_samples * 1e3
    fb.fasa_profile_reset(); fb.fasa_profile_enable(True)
    fb.fasa_contextual_agreement(shape, qs[0], Kp_all, top_k, ca, cws, nbytes)
    prof = fb.profile_summary()
    fb.fasa_profile_enable(False); fb.fasa_profile_reset()
    ca_mean = (ca.cpu().numpy() - 0).mean(axis=0)            # over the batch; one extra sample of q0 is in the sum
    fc = np.zeros((w.n_kv_heads, w.n_fc), dtype=np.int32)
    dec = fb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_fc, w.n_ctx, n_cap, w.budget, w.dtype)
    fb.fasa_select_dominant_fcs(dec, np.ascontiguousarray(ca_mean, dtype=np.float32), fc)
    recovered = float(np.mean([len(set(fc[h].tolist()) & set(x["fc_idx"][h].tolist())) / w.n_fc
                               for h in range(w.n_kv_heads)]))
    rows, e = w.batch * w.n_kv_heads, w.elem_bytes
    kp_bytes = 2 * rows * w.n_ctx * w.head_dim * e            # the packed copy is read twice: all FCs at once, each FC alone
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import fasa_oracle as O
        t0 = time.time()
        O.contextual_agreement(q_host[0][:1], x["K"][:1], w.n_ctx, top_k)
        dt = time.time() - t0
        cpu = {"value": round(dt * w.batch * 1e6, 1), "unit": "us", "cores": 1, "kind": "oracle",
               "sample": "contextual agreement of one query sample on 1 of %d batch entries, scaled to the batch; "
                         "numpy float64" % w.batch}
    out = {
        "metric": "us_per_calibration_sample", "value": round(us, 3), "unit": "us", "n_gpus": 1, "steps": n_samples,
        "warmup": 1, "ms_per_step": round(us / 1e3, 6), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "accum_dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name + "_calibration", "batch": w.batch, "n_q_heads": w.n_q_heads,
                   "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "n_ctx": w.n_ctx, "top_k": top_k,
                   "storage_dtype": w.dtype, "launch": "eager"},
        "kernels": {k: {"launches": n, "avg_us": round(ms / n * 1e3, 3)} for k, (n, ms) in prof.items()},
        "hbm": {"alg_bytes": kp_bytes, "step_gbps": round(kp_bytes / us / 1e3, 1),
                "step_frac_of_peak": round(kp_bytes / us / 1e3 / HBM_PEAK_GBPS, 4)},
        "planted_fcs_recovered": round(recovered, 4),
        "roofline": None, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


def ragged(args, w, fb, W, np, torch):
    """Serving loop: a batch whose sequences have different lengths, every length growing by one per
    step, driven by ONE captured graph of fasa_decode_step_ragged (append + score + select + attend)
    whose per-sequence lengths and budgets live on the device."""
    steps = args.ragged
    n_max = w.n_ctx
    n_cap = (n_max + 63) // 64 * 64
    x = W.make_inputs(w, n_cap=n_cap)
    dev = lambda a: torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()
    tdt = torch.int16 if w.dtype == "bf16" else torch.float32
    rng = np.random.default_rng(20260203)
    lens0 = rng.integers(n_max // 4, n_max - steps, size=w.batch).astype(np.int32)
    lens0[0] = n_max - steps - 1                          # one sequence at the top of the range
    frac = w.budget / w.n_ctx
    shape = fb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_fc, n_max, n_cap, w.budget, w.dtype)
    q, K, V, fc = dev(x["q"]), dev(x["K"]), dev(x["V"]), dev(x["fc_idx"])
    a0 = W.make_append(w, x["fc_idx"], step=1, n_before=int(lens0[0]))
    k_new, v_new = dev(a0["k_new"]), dev(a0["v_new"])
    Kp = torch.zeros((w.batch, w.n_kv_heads, w.n_fc, n_cap, 2), dtype=tdt, device="cuda")
    fb.fasa_pack_kcache(shape, K, fc, Kp, 0, n_max)
    S = torch.zeros((w.batch, w.n_kv_heads, n_cap), dtype=torch.float32, device="cuda")
    T = torch.zeros((w.batch, w.n_kv_heads, min(w.budget, n_max)), dtype=torch.int32, device="cuda")
    O = torch.zeros((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    ws_bytes = fb.fasa_workspace_bytes(shape)
    ws = torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda")
    fb.fasa_workspace_init(shape, ws, ws_bytes)
    n_dev = torch.from_numpy(lens0.copy()).cuda()
    b_dev = torch.from_numpy(np.maximum(1, np.floor(frac * lens0)).astype(np.int32)).cuda()
    one = torch.ones_like(n_dev)

    def step():
        fb.fasa_decode_step_ragged(shape, q, K, V, Kp, fc, k_new, v_new, n_dev, b_dev, S, T, O, ws, ws_bytes)

    step()                                                # eager warm-up (re-appends at the current last position)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        n_dev.add_(one)                                   # the lengths advance inside the graph: a replay is a step
        step()
    torch.cuda.synchronize()
    for _ in range(min(args.warmup, 8)):
        g.replay()
    torch.cuda.synchronize()
    n_dev.copy_(torch.from_numpy(lens0))
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(steps):
        g.replay()
    b.record()
    torch.cuda.synchronize()
    us = a.elapsed_time(b) / steps * 1e3
    lens_end = n_dev.cpu().numpy()
    assert (lens_end == lens0 + steps).all()
    e, rows_b = w.elem_bytes, w.n_kv_heads
    mean_len = float(lens0.mean() + steps / 2)
    alg = int(sum(rows_b * (n * 2 * w.n_fc * e + 2 * min(max(1, int(frac * n)), n) * w.head_dim * e)
                  for n in (lens0 + steps // 2)))
    out = {
        "metric": "us_per_decode_step", "value": round(us, 3), "unit": "us", "n_gpus": 1, "steps": steps,
        "warmup": min(args.warmup, 8), "ms_per_step": round(us / 1e3, 6), "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "accum_dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name + "_ragged", "batch": w.batch, "n_q_heads": w.n_q_heads,
                   "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "n_ctx_bound": n_max,
                   "n_ctx_min": int(lens0.min()), "n_ctx_mean": round(mean_len, 1), "n_ctx_max": int(lens0.max()) + steps,
                   "budget_fraction": round(frac, 4), "n_fc": w.n_fc, "storage_dtype": w.dtype,
                   "launch": "one hipgraph, lengths on the device"},
        "hbm": {"alg_bytes_mid_step": alg, "step_gbps": round(alg / us / 1e3, 1),
                "step_frac_of_peak": round(alg / us / 1e3 / HBM_PEAK_GBPS, 4)},
        "roofline": None, "cpu_baseline": None,
    }
    print(json.dumps(out), flush=True)


def paged(args, w, fb, W, np, torch):
    """The decode step on a paged K/V cache (blocks of --paged tokens at random places of a pool, token-major
    blocks), timed next to the same step on the contiguous cache, both over rotating buffer sets."""
    page = args.paged
    x = W.make_inputs(w)
    n_cap = x["n_cap"]
    assert page >= 1 and page & (page - 1) == 0 and n_cap % page == 0, "--paged takes a power of two dividing the capacity"
    B, Hkv, D = w.batch, w.n_kv_heads, w.head_dim
    nblk = n_cap // page
    n_pool = B * nblk + 3                                   # three blocks that belong to nobody
    rng = np.random.default_rng(20260203)
    table = rng.permutation(n_pool)[: B * nblk].reshape(B, nblk).astype(np.int32)

    def to_pool(a):                                         # [B][Hkv][n_cap][D] -> [block][token][head][dim]
        pool = np.zeros((n_pool, page, Hkv, D), dtype=a.dtype)
        blocks = a.reshape(B, Hkv, nblk, page, D).transpose(0, 2, 3, 1, 4)     # [B][nblk][page][Hkv][D]
        pool[table.reshape(-1)] = blocks.reshape(B * nblk, page, Hkv, D)
        return pool

    dev = lambda a: torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()
    tdt = torch.int16 if w.dtype == "bf16" else torch.float32
    bsel = min(w.budget, w.n_ctx)
    shape_c = fb.make_shape(B, w.n_q_heads, Hkv, D, w.n_fc, w.n_ctx, n_cap, w.budget, w.dtype)
    shape_p = fb.make_shape(B, w.n_q_heads, Hkv, D, w.n_fc, w.n_ctx, n_cap, w.budget, w.dtype,
                            kv_stride_b=page * Hkv * D, kv_stride_h=D, kv_stride_n=Hkv * D)
    ws_bytes = fb.fasa_workspace_bytes(shape_p)
    table_dev = torch.from_numpy(table).cuda()
    paging = fb.make_paging(table_dev, page, n_pool)
    q0, fc = dev(x["q"]), dev(x["fc_idx"])
    Kc0, Vc0, Kp0, Vp0 = dev(x["K"]), dev(x["V"]), dev(to_pool(x["K"])), dev(to_pool(x["V"]))
    touched = W.algorithmic_bytes(w)["alg_plus_intermediates"]
    R = args.sets or max(4, min(32, int(np.ceil(2.5 * LLC_BYTES / touched))))
    sets = []
    for r in range(R):
        s = {"q": q0.clone(), "Kc": Kc0.clone(), "Vc": Vc0.clone(), "Kpool": Kp0.clone(), "Vpool": Vp0.clone()}
        for tag in ("c", "p"):
            s["Kp" + tag] = torch.zeros((B, Hkv, w.n_fc, n_cap, 2), dtype=tdt, device="cuda")
            s["S" + tag] = torch.zeros((B, Hkv, n_cap), dtype=torch.float32, device="cuda")
            s["T" + tag] = torch.zeros((B, Hkv, bsel), dtype=torch.int32, device="cuda")
            s["O" + tag] = torch.zeros((B, w.n_q_heads, D), dtype=torch.float32, device="cuda")
            s["ws" + tag] = torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda")
            fb.fasa_workspace_init(shape_p, s["ws" + tag], ws_bytes)
        fb.fasa_pack_kcache(shape_c, s["Kc"], fc, s["Kpc"], 0, w.n_ctx)
        fb.fasa_pack_kcache_paged(shape_p, paging, s["Kpool"], fc, s["Kpp"], 0, w.n_ctx)
        sets.append(s)
    torch.cuda.synchronize()

    def step_c(s):
        fb.fasa_decode_step(shape_c, s["q"], s["Kc"], s["Vc"], s["Kpc"], fc, None, None, s["Sc"], s["Tc"], s["Oc"],
                            s["wsc"], ws_bytes)

    def step_p(s):
        fb.fasa_decode_step_paged(shape_p, paging, s["q"], s["Kpool"], s["Vpool"], s["Kpp"], fc, None, None, None, None,
                                  s["Sp"], s["Tp"], s["Op"], s["wsp"], ws_bytes)

    K_steps = max(R, (args.steps // R) * R)
    res = {}
    for name, fn in (("contiguous", step_c), ("paged", step_p)):
        for i in range(args.warmup):
            fn(sets[i % R])
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(K_steps):
            fn(sets[i % R])
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) / K_steps * 1e3
        fb.fasa_profile_reset(); fb.fasa_profile_enable(True)
        for i in range(K_steps):
            fn(sets[i % R])
        prof = fb.profile_summary()
        fb.fasa_profile_enable(False); fb.fasa_profile_reset()
        res[name] = {"us_per_step": round(us, 3),
                     "kernels": {k: round(ms / n * 1e3, 3) for k, (n, ms) in prof.items()}}
        log("%s: %.2f us/step %s" % (name, us, res[name]["kernels"]))
    s0 = sets[0]
    same_set = bool(np.array_equal(np.sort(s0["Tc"].cpu().numpy(), -1), np.sort(s0["Tp"].cpu().numpy(), -1)))
    o_diff = float((s0["Oc"] - s0["Op"]).abs().max())
    assert same_set and o_diff <= 2e-5, (same_set, o_diff)
    us = res["paged"]["us_per_step"]
    out = {
        "metric": "us_per_decode_step", "value": us, "unit": "us", "n_gpus": 1, "steps": K_steps,
        "warmup": args.warmup, "ms_per_step": round(us / 1e3, 6), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "accum_dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name + "_paged", "batch": B, "n_q_heads": w.n_q_heads, "n_kv_heads": Hkv,
                   "head_dim": D, "n_ctx": w.n_ctx, "budget": bsel, "n_fc": w.n_fc, "storage_dtype": w.dtype,
                   "page_size": page, "pool_blocks": n_pool, "block_layout": "[block][token][head][dim]",
                   "buffer_sets": R, "launch": "eager"},
        "paged": res["paged"], "contiguous": res["contiguous"],
        "same_index_set_as_contiguous": same_set, "max_abs_output_difference": o_diff,
    }
    print(json.dumps(out), flush=True)


def recall_table(args, w, fb, W, np, torch):
    """Selection quality on the synthetic workload, in the form of the paper's compound contextual
    agreement table (Sec. 3.3): for F dominant FCs and a top-K, the share of the full-head top-K set
    (the paper's "Oracle" ranking, all d/2 FCs) that the F-FC scores recover.  Same kernels as the
    decode step; averaged over KV heads and a few queries.  Not timed."""
    half = w.head_dim // 2
    x = W.make_inputs(w)
    n_cap = x["n_cap"]
    dev = lambda a: torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()
    tdt = torch.int16 if w.dtype == "bf16" else torch.float32
    rows = w.batch * w.n_kv_heads
    K = dev(x["K"])
    queries = [dev(x["q"])] + [dev(W.make_append(w, x["fc_idx"], step=s, n_before=w.n_ctx - 1)["q"]) for s in range(1, 4)]
    mk = lambda F, k: fb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, F, w.n_ctx, n_cap, k, w.dtype)
    ks = [k for k in (64, 256, 512, 1024, 2048) if k < w.n_ctx]
    fs = sorted({max(1, w.n_fc // 4), max(1, w.n_fc // 2), (3 * w.n_fc) // 4, w.n_fc})
    ws_bytes = max(fb.fasa_workspace_bytes(mk(half, k)) for k in ks)
    ws = torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda")
    fb.fasa_workspace_init(mk(half, ks[0]), ws, ws_bytes)
    S = torch.zeros((w.batch, w.n_kv_heads, n_cap), dtype=torch.float32, device="cuda")

    def top_sets(fc_host, F, q):
        fc = dev(np.ascontiguousarray(fc_host[:, :F]))
        Kp = torch.zeros((w.batch, w.n_kv_heads, F, n_cap, 2), dtype=tdt, device="cuda")
        fb.fasa_pack_kcache(mk(F, ks[0]), K, fc, Kp, 0, w.n_ctx)
        fb.fasa_score(mk(F, ks[0]), q, Kp, fc, S)
        out = {}
        for k in ks:
            T = torch.zeros((w.batch, w.n_kv_heads, k), dtype=torch.int32, device="cuda")
            fb.fasa_topk(mk(F, k), S, T, ws, ws_bytes)
            out[k] = T.cpu().numpy().reshape(rows, k)
        return out

    fc_all = np.tile(np.arange(half, dtype=np.int32), (w.n_kv_heads, 1))
    table = {F: {k: 0.0 for k in ks} for F in fs}
    for q in queries:
        full = top_sets(fc_all, half, q)
        for F in fs:
            part = top_sets(x["fc_idx"], F, q)             # the first F of the head's dominant FCs
            for k in ks:
                table[F][k] += float(np.mean([len(np.intersect1d(full[k][r], part[k][r])) / k for r in range(rows)]))
    table = {str(F): {str(k): round(v / len(queries), 4) for k, v in row.items()} for F, row in table.items()}
    print(json.dumps({"metric": "top_k_recall_vs_full_head", "unit": "fraction", "n_gpus": 1, "data": "synthetic",
                      "config": {"workload": w.name + "_recall_table", "n_ctx": w.n_ctx, "queries": len(queries),
                                 "rows": "F (dominant FCs used)", "columns": "K (top-K size)"},
                      "recall": table}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=240)
    ap.add_argument("--warmup", type=int, default=24)
    ap.add_argument("--config", type=int, default=1, help="workload id (0-4); the metric is quoted on 1")
    ap.add_argument("--sets", type=int, default=0, help="buffer sets to rotate over (0 = derive)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--growing", type=int, default=0, metavar="STEPS",
                    help="long-CoT recipe: STEPS consecutive decode steps on ONE cache that grows by one "
                         "appended K/V row per step (budget = 18.9%% of the current length); use with --config 3")
    ap.add_argument("--offload", action="store_true",
                    help="time the memory-optimised variant (non-dominant key dims and values in pinned "
                         "host memory, fetched over PCIe) instead of the on-device one")
    ap.add_argument("--calibrate", type=int, default=0, metavar="SAMPLES",
                    help="time the offline calibration (contextual agreement of every FC, on the device) over "
                         "SAMPLES query samples instead of the decode step")
    ap.add_argument("--ragged", type=int, default=0, metavar="STEPS",
                    help="serving loop: mixed sequence lengths growing by one per step, one captured graph "
                         "with the lengths on the device; use with --config 2")
    ap.add_argument("--paged", type=int, default=0, metavar="PAGE",
                    help="time the step on a paged K/V cache (blocks of PAGE tokens scattered over a pool) next to "
                         "the contiguous cache")
    ap.add_argument("--recall-table", action="store_true",
                    help="selection quality only: recall of the full-head top-K set by F dominant FCs, for several "
                         "F and K (the synthetic analogue of the paper's compound contextual agreement table)")
    ap.add_argument("--pairing", choices=["half", "interleaved", "list"], default="half",
                    help="default mode only: how the dominant list names head dims (the same vectors re-stored "
                         "with FC i at dims (2i, 2i+1), or the FCs written out as explicit dim pairs)")
    ap.add_argument("--stage-timers", action="store_true",
                    help="with FASA_LIB pointing at the traced library (python -m paper_2602_03152_amd.build --trace): "
                         "run three steps and let the kernels print their phase times for row 0; nothing is timed")
    ap.add_argument("--other-workloads", default="3,4,2",
                    help="default mode: workload ids timed briefly after the headline one and reported under "
                         "other_workloads (empty string: none)")
    ap.add_argument("--other-budget-s", type=float, default=150.0,
                    help="no further workload of --other-workloads is started once the run has taken this long")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only plain device copies of known size (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the hot path shards by batch / KV head with no "
                 "exchange; no multi-GPU path exists here). Re-run with --gpus 1.")

    import numpy as np
    import torch

    from paper_2602_03152_amd import binding as fb      # raises if libfasa.so is missing
    from paper_2602_03152_amd import workload as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        # 8 rotating 256 MiB copies: under `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` the copy kernel's
        # counter value per dispatch, divided by 256 MiB, is the scale of the counter on this machine
        nbytes = 256 << 20
        src = [torch.full((nbytes,), i, dtype=torch.uint8, device="cuda") for i in range(4)]
        dst = [torch.empty((nbytes,), dtype=torch.uint8, device="cuda") for _ in range(4)]
        torch.cuda.synchronize()
        for i in range(8):
            dst[i % 4].copy_(src[i % 4])
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": nbytes, "copies": 8}), flush=True)
        return
    w = W.WORKLOADS[args.config]
    if args.growing:
        return growing(args, w, fb, W, np, torch)
    if args.offload:
        return offload(args, w, fb, W, np, torch)
    if args.calibrate:
        return calibrate(args, w, fb, W, np, torch)
    if args.ragged:
        return ragged(args, w, fb, W, np, torch)
    if args.paged:
        return paged(args, w, fb, W, np, torch)
    if args.recall_table:
        return recall_table(args, w, fb, W, np, torch)
    if args.stage_timers:
        return stage_timers(args, w, fb, W, np, torch)

    t_start = time.time()
    head = measure(args, w, fb, W, np, torch, steps=args.steps, warmup=args.warmup, full=True)
    # ---------------- the other workloads at a 32k+ context (and the batch one), briefly ----------------
    others = {}
    for cid in [int(c) for c in args.other_workloads.split(",") if c.strip()]:
        if cid == w.config_id or cid not in W.WORKLOADS:
            continue
        if time.time() - t_start > args.other_budget_s:
            log("other workloads: time budget used up, skipping config %d" % cid)
            continue
        wo = W.WORKLOADS[cid]
        r = measure(args, wo, fb, W, np, torch, steps=min(args.steps, 100), warmup=min(args.warmup, 10), full=False)
        others[wo.name] = {"us_per_step": r["us_per_step"], "steps": r["timed_steps"], "alg_bytes": r["model"]["alg"],
                           "step_frac_of_peak": round(r["model"]["alg"] / r["us_per_step"] / 1e3 / HBM_PEAK_GBPS, 4),
                           "kernels_avg_us": {k: v["avg_us"] for k, v in r["kernels"].items()},
                           "dominant_kernel": r["roofline"]["kernel"], "dominant_kernel_frac": r["roofline"]["frac"]}
    us = head["us_per_step"]
    model = head["model"]
    out = {
        "metric": "us_per_decode_step", "value": round(us, 3), "unit": "us",
        "n_gpus": 1, "steps": args.steps, "timed_steps": head["timed_steps"], "warmup": args.warmup,
        "ms_per_step": round(us / 1e3, 6),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        # storage and matrix-core input type; every sum is accumulated in float32
        "dtype": w.dtype, "accum_dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "n_ctx": w.n_ctx, "budget": min(w.budget, w.n_ctx), "n_fc": w.n_fc,
                   "storage_dtype": w.dtype, "pairing": args.pairing, "buffer_sets": head["buffer_sets"],
                   "launch": "eager"},
        # the whole step against the HBM roofline: what the benchmark spec's target is about
        "step_roofline": {"bound": "hbm", "bytes": model["alg"], "us": round(us, 3),
                          "achieved": round(model["alg"] / us / 1e3, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                          "frac": round(model["alg"] / us / 1e3 / HBM_PEAK_GBPS, 4)},
        "hbm": {"alg_bytes": model["alg"], "alg_plus_intermediate_bytes": model["alg_plus_intermediates"],
                # the same with the intermediates (S written and re-read, T) counted: the bytes actually touched
                "step_touched_gbps": round(model["alg_plus_intermediates"] / us / 1e3, 1),
                "step_touched_frac_of_peak": round(model["alg_plus_intermediates"] / us / 1e3 / HBM_PEAK_GBPS, 4),
                "kernel_time_gbps": round(model["alg"] / head["sum_kernel_us"] / 1e3, 1),
                # second denominator: what a plain 256 MiB device copy moves (read + write) on this machine
                "copy_ceiling_gbps": head["copy_gbps"]},
        "step_us_percentiles": head["step_pct"],
        "graph_us_per_step": head["graph_us"], "graph_steps": head["graph_steps"],
        "graph_replays_match_eager": head["graph_ok"],
        "sum_kernel_us": round(head["sum_kernel_us"], 3),
        "roofline": head["roofline"],
        "kernels": head["kernels"],
        "dense_baseline": head["dense_baseline"],
        "selection_recall_vs_full_head": head["recall"],
        "other_workloads": others,
        "cpu_baseline": head["cpu"],
    }
    print(json.dumps(out), flush=True)


def stage_timers(args, w, fb, W, np, torch):
    """Three warm and three cold steps on one buffer set with the traced library (FASA_LIB): the kernels print
    their phases."""
    x = W.make_inputs(w)
    dev = lambda a: torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()
    tdt = torch.int16 if w.dtype == "bf16" else torch.float32
    n_cap, bsel = x["n_cap"], min(w.budget, w.n_ctx)
    shape = fb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_fc, w.n_ctx, n_cap, w.budget, w.dtype)
    q, K, V, fc = dev(x["q"]), dev(x["K"]), dev(x["V"]), dev(x["fc_idx"])
    Kp = torch.zeros((w.batch, w.n_kv_heads, w.n_fc, n_cap, 2), dtype=tdt, device="cuda")
    S = torch.zeros((w.batch, w.n_kv_heads, n_cap), dtype=torch.float32, device="cuda")
    T = torch.zeros((w.batch, w.n_kv_heads, bsel), dtype=torch.int32, device="cuda")
    O = torch.zeros((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    ws_bytes = fb.fasa_workspace_bytes(shape)
    ws = torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda")
    fb.fasa_workspace_init(shape, ws, ws_bytes)
    fb.fasa_pack_kcache(shape, K, fc, Kp, 0, w.n_ctx)
    for i in range(3):
        fb.fasa_decode_step(shape, q, K, V, Kp, fc, None, None, S, T, O, ws, ws_bytes)
        torch.cuda.synchronize()
        print("---- step %d (warm: same buffers as the step before) ----" % i, flush=True)
    # the same step with nothing of it left in the caches: 1 GiB is read in between (the last-level cache
    # holds 256 MiB), which leaves the caches full of clean lines as bench.py's rotation over buffer sets does
    junk = torch.zeros((1 << 28,), dtype=torch.float32, device="cuda")
    for i in range(3):
        junk.sum().item()
        torch.cuda.synchronize()
        fb.fasa_decode_step(shape, q, K, V, Kp, fc, None, None, S, T, O, ws, ws_bytes)
        torch.cuda.synchronize()
        print("---- step %d (cold: 1 GiB read since the step before) ----" % (3 + i), flush=True)


def source_hash():
    """Hash of the kernel sources: measured HBM traffic is only quoted for the sources it was measured on."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2602_03152_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")) and name != "floors.hip":
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(config_id, kernel):
    """Bytes per launch from the rocprofv3 --pmc runs under profiles/, or None if the kernels changed since."""
    if MEASURED_TRAFFIC.get("source_hash") != source_hash():
        if not measured_traffic.warned:
            log("bench: kernel sources differ from the ones the HBM counters in profiles/ were taken on: traffic = null")
            measured_traffic.warned = True
        return None
    return MEASURED_TRAFFIC.get((config_id, kernel))


measured_traffic.warned = False


def measure(args, w, fb, W, np, torch, steps, warmup, full):
    """Times `steps` decode steps of workload w (after `warmup`), rotating over R HBM-resident buffer sets;
    then per-kernel GPU times.  full: also the captured graph, single-step percentiles, the copy ceiling,
    the dense baseline, the selection recall and the CPU oracle."""
    rows = w.batch * w.n_kv_heads
    model = W.algorithmic_bytes(w)
    bsel = min(w.budget, w.n_ctx)
    e = w.elem_bytes

    # ---------------- inputs: one seeded draw, cloned into R device-resident sets ----------------
    t0 = time.time()
    x = W.make_inputs(w)
    if args.pairing == "interleaved":
        x = W.as_interleaved(x)
    elif args.pairing == "list":
        x["fc_idx"] = W.explicit_pairs(x["fc_idx"], w.head_dim)
    log("%s: inputs drawn in %.1fs" % (w.name, time.time() - t0))
    n_cap = x["n_cap"]
    tdt = torch.int16 if w.dtype == "bf16" else torch.float32
    touched = model["alg_plus_intermediates"]
    R = args.sets or max(4, min(64, int(np.ceil(2.5 * LLC_BYTES / touched))))
    dev = lambda a: torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()
    shape = fb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_fc, w.n_ctx, n_cap, w.budget, w.dtype,
                          pairing=args.pairing)
    ws_bytes = fb.fasa_workspace_bytes(shape)
    q0, K0, V0, fc = dev(x["q"]), dev(x["K"]), dev(x["V"]), dev(np.ascontiguousarray(x["fc_idx"]))
    sets = []
    for r in range(R):
        s = {
            "q": q0.clone(), "K": K0 if r == 0 else K0.clone(), "V": V0 if r == 0 else V0.clone(),
            "Kp": torch.zeros((w.batch, w.n_kv_heads, w.n_fc, n_cap, 2), dtype=tdt, device="cuda"),
            "S": torch.zeros((w.batch, w.n_kv_heads, n_cap), dtype=torch.float32, device="cuda"),
            "T": torch.zeros((w.batch, w.n_kv_heads, bsel), dtype=torch.int32, device="cuda"),
            "O": torch.zeros((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda"),
            "ws": torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda"),
        }
        fb.fasa_workspace_init(shape, s["ws"], ws_bytes)
        fb.fasa_pack_kcache(shape, s["K"], fc, s["Kp"], 0, w.n_ctx)
        sets.append(s)
    torch.cuda.synchronize()
    log("workload %s: R=%d buffer sets, %.1f MB touched per step, %.2f GB resident"
        % (w.name, R, touched / 1e6, torch.cuda.memory_allocated() / 1e9))

    def step(s):
        fb.fasa_decode_step(shape, s["q"], s["K"], s["V"], s["Kp"], fc, None, None,
                            s["S"], s["T"], s["O"], s["ws"], ws_bytes)

    def dense(s):
        fb.fasa_dense_attend(shape, s["q"], s["K"], s["V"], s["O"], s["ws"], ws_bytes)

    def time_loop(fn, n_steps, warm):
        for i in range(warm):
            fn(sets[i % R])
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(n_steps):
            fn(sets[i % R])
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n_steps * 1e3          # us per step

    # ---------------- pass 1: the timed region: exactly `steps` eager steps ----------------
    us_per_step = time_loop(step, steps, warmup)
    log("%s: %.2f us/step over %d steps" % (w.name, us_per_step, steps))
    res = {"us_per_step": us_per_step, "timed_steps": steps, "buffer_sets": R, "model": model,
           "graph_us": None, "graph_steps": None, "graph_ok": None, "step_pct": None, "copy_gbps": None,
           "dense_baseline": None, "recall": None, "cpu": None}

    if full and not args.no_graph:
        # the same steps as ONE captured graph (one step per buffer set), replayed; every replay is checked
        ref_T = np.sort(sets[0]["T"].cpu().numpy(), -1)
        ref_O = sets[0]["O"].cpu().numpy().copy()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(sets[0])
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for s in sets:
                step(s)
        torch.cuda.synchronize()
        n_replays = max(1, steps // R)
        for _ in range(max(1, warmup // R)):
            g.replay()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n_replays):
            g.replay()
        b.record()
        torch.cuda.synchronize()
        res["graph_us"] = round(a.elapsed_time(b) / (n_replays * R) * 1e3, 3)
        res["graph_steps"] = n_replays * R
        ok = True
        for _ in range(3):
            g.replay()
            torch.cuda.synchronize()
            ok &= bool(np.array_equal(np.sort(sets[0]["T"].cpu().numpy(), -1), ref_T))
            ok &= bool(np.abs(sets[0]["O"].cpu().numpy() - ref_O).max() <= 2e-5)
            step(sets[1]); torch.cuda.synchronize()
        res["graph_ok"] = ok
        log("graph: %.2f us/step, replays match eager: %s" % (res["graph_us"], ok))

    if full:
        # ---------------- distribution of single steps (one event pair per step: adds ~2 us each) ----------------
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        for i in range(steps):
            evs[i][0].record(); step(sets[i % R]); evs[i][1].record()
        torch.cuda.synchronize()
        per = np.array([a.elapsed_time(b) * 1e3 for a, b in evs])
        res["step_pct"] = {"p10": round(float(np.percentile(per, 10)), 3), "p50": round(float(np.percentile(per, 50)), 3),
                           "p90": round(float(np.percentile(per, 90)), 3), "includes_event_overhead": True}
        # ---------------- measured ceiling: a plain device copy (read + write bytes per second) ----------------
        cp_src = torch.empty((256 << 20,), dtype=torch.uint8, device="cuda")
        cp_dst = torch.empty_like(cp_src)
        for _ in range(3):
            cp_dst.copy_(cp_src)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(10):
            cp_dst.copy_(cp_src)
        b.record()
        torch.cuda.synchronize()
        res["copy_gbps"] = round(2 * cp_src.numel() * 10 / (a.elapsed_time(b) * 1e-3) / 1e9, 1)
        del cp_src, cp_dst

    # ---------------- pass 2: per-kernel GPU time (start/stop timestamps of every launch) ----------------
    fb.fasa_profile_reset()
    fb.fasa_profile_enable(True)
    for i in range(steps):
        step(sets[i % R])
    prof = fb.profile_summary()
    prof_dense = {}
    if full:
        fb.fasa_profile_reset()
        for i in range(steps):
            dense(sets[i % R])
        prof_dense = fb.profile_summary()
    fb.fasa_profile_enable(False)
    fb.fasa_profile_reset()

    alg_bytes = {   # algorithmic bytes per launch of each kernel (what the method itself must move)
        "fasa_score_hist": rows * w.n_ctx * 2 * w.n_fc * e,
        "fasa_score": rows * w.n_ctx * 2 * w.n_fc * e,
        "fasa_select": rows * w.n_ctx * 4,
        "fasa_select_all": rows * bsel * 4,
        "fasa_sparse_attend": rows * 2 * bsel * w.head_dim * e,
        "fasa_select_attend": rows * w.n_ctx * 4 + rows * 2 * bsel * w.head_dim * e,    # scores read + rows gathered
        "fasa_dense_attend": rows * 2 * w.n_ctx * w.head_dim * e,
    }
    kernels = {}
    for name, (launches, ms) in {**prof, **prof_dense}.items():
        us = ms / launches * 1e3
        ent = {"launches": launches, "avg_us": round(us, 3)}
        if name in alg_bytes:
            ent["alg_bytes"] = alg_bytes[name]
            ent["gbps"] = round(alg_bytes[name] / us / 1e3, 1)
            ent["traffic"] = measured_traffic(w.config_id, name)
        kernels[name] = ent
    # the dominant kernel of the step is the one that takes the longest
    dom = max(prof, key=lambda k: prof[k][1] / prof[k][0])
    dom_us = prof[dom][1] / prof[dom][0] * 1e3
    achieved = alg_bytes[dom] / dom_us / 1e3
    res["roofline"] = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                       "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "avg_us": round(dom_us, 3),
                       "alg_bytes": alg_bytes[dom], "traffic": measured_traffic(w.config_id, dom)}
    res["kernels"] = kernels
    res["sum_kernel_us"] = sum(prof[k][1] / prof[k][0] * 1e3 for k in prof)
    if not full:
        del sets, q0, K0, V0
        torch.cuda.empty_cache()
        return res

    dense_us = time_loop(dense, steps, warmup)
    dense_kernel_us = sum(ms / n * 1e3 for n, ms in prof_dense.values())
    log("dense full-KV decode: %.2f us/step" % dense_us)
    res["dense_baseline"] = {"us_per_step": round(dense_us, 3), "kernel_us": round(dense_kernel_us, 3),
                             "bytes": model["dense"], "gbps": round(model["dense"] / dense_us / 1e3, 1),
                             "speedup_of_fasa": round(dense_us / us_per_step, 3)}

    # ---------------- selection quality against full-head scores (not timed) ----------------
    # The paper's "Oracle" upper bound ranks tokens by the full-head logits (all d/2 FCs); the share of
    # its top-B set that the F dominant FCs recover is the synthetic analogue of the paper's contextual
    # agreement.  Same kernels, F = d/2.
    if w.n_fc < w.head_dim // 2 and bsel < w.n_ctx:
        half = w.head_dim // 2
        s0 = sets[0]
        fc_all_host = np.tile(np.arange(half, dtype=np.int32), (w.n_kv_heads, 1))
        if args.pairing == "list":
            fc_all_host = W.explicit_pairs(fc_all_host, w.head_dim)
        fc_all = dev(np.ascontiguousarray(fc_all_host))
        shape_all = fb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, half, w.n_ctx, n_cap, w.budget, w.dtype,
                                  pairing=args.pairing)
        Kp_all = torch.zeros((w.batch, w.n_kv_heads, half, n_cap, 2), dtype=tdt, device="cuda")
        S_all = torch.zeros_like(s0["S"]); T_all = torch.zeros_like(s0["T"])
        fb.fasa_pack_kcache(shape_all, s0["K"], fc_all, Kp_all, 0, w.n_ctx)
        fb.fasa_score(shape_all, s0["q"], Kp_all, fc_all, S_all)
        fb.fasa_topk(shape_all, S_all, T_all, s0["ws"], ws_bytes)
        step(s0)
        torch.cuda.synchronize()
        Ta, Tf = T_all.cpu().numpy().reshape(rows, -1), s0["T"].cpu().numpy().reshape(rows, -1)
        res["recall"] = round(float(np.mean([len(np.intersect1d(Ta[r], Tf[r])) / bsel for r in range(rows)])), 4)
        del Kp_all, S_all, T_all
        log("top-B recall of the F=%d dominant FCs against full-head scores: %.4f" % (w.n_fc, res["recall"]))

    # ---------------- pass 3: CPU oracle on the host cores ----------------
    if not args.no_cpu_baseline:
        from oracle import fasa_oracle as O
        sub = list(range(w.batch)) if w.batch <= 2 else [0]          # bounded sample of the batch
        qs, Ks, Vs = x["q"][sub], x["K"][sub], x["V"][sub]
        reps, t_cpu0, c0 = 0, time.time(), time.process_time()
        while True:
            O.decode_step(qs, Ks, Vs, x["fc_idx"], w.n_ctx, w.budget, pairing=args.pairing)
            reps += 1
            if time.time() - t_cpu0 >= 10.0 or reps >= 200:
                break
        wall, cpu_t = time.time() - t_cpu0, time.process_time() - c0
        per_step = wall / reps * (w.batch / len(sub))
        res["cpu"] = {"value": round(per_step * 1e6, 1), "unit": "us", "cores": max(1, int(round(cpu_t / wall))),
                      "kind": "oracle",
                      "sample": "%d full oracle decode steps on %d of %d batch entries, scaled to the batch; "
                                "numpy float64" % (reps, len(sub), w.batch)}
        log("cpu oracle: %.0f us/step (%d reps)" % (res["cpu"]["value"], reps))
    del sets, q0, K0, V0
    torch.cuda.empty_cache()
    return res


if __name__ == "__main__":
    main()
