"""Plumbing for the GPU parity tests: upload seeded inputs, allocate outputs, call the C ABI
through the binding, bring results back as numpy.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from paper_2602_03152_amd import binding as fb


def round_up(x, m):
    return (x + m - 1) // m * m


def to_dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_host(t: torch.Tensor, like: np.dtype = None) -> np.ndarray:
    a = t.detach().cpu().numpy()
    if like is not None and np.dtype(like) == np.uint16:
        a = a.view(np.uint16)
    return a


class Device:
    """Device-side buffers of one workload (inputs from the generator, outputs zero/garbage filled)."""

    def __init__(self, w, x, n_cap=None, poison=True, pairing="half"):
        self.w = w
        self.pairing = pairing      # how x["fc_idx"] names head dims ("half" | "interleaved" | "list")
        self.n_cap = x["n_cap"] if n_cap is None else n_cap
        assert self.n_cap % 64 == 0
        self.st = np.uint16 if w.dtype == "bf16" else np.float32
        tdt = torch.int16 if w.dtype == "bf16" else torch.float32
        self.q = to_dev(x["q"])
        self.K = to_dev(x["K"])
        self.V = to_dev(x["V"])
        self.fc_idx = to_dev(x["fc_idx"])
        rows = w.batch * w.n_kv_heads
        self.Kp = torch.zeros((w.batch, w.n_kv_heads, w.n_fc, self.n_cap, 2), dtype=tdt, device="cuda")
        self.S = torch.full((w.batch, w.n_kv_heads, self.n_cap), float("nan") if poison else 0.0,
                            dtype=torch.float32, device="cuda")
        self.bsel = min(w.budget, w.n_ctx)
        self.T = torch.full((w.batch, w.n_kv_heads, self.bsel), -1, dtype=torch.int32, device="cuda")
        self.O = torch.full((w.batch, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.float32, device="cuda")
        self.shape = self.make_shape()
        self.ws_bytes = fb.fasa_workspace_bytes(self.shape)
        assert self.ws_bytes > 0
        # poisoned, then prepared by the library itself: it may not rely on the allocator's zeros
        self.ws = torch.full((self.ws_bytes,), 0x5A, dtype=torch.uint8, device="cuda")
        fb.fasa_workspace_init(self.shape, self.ws, self.ws_bytes)

    def make_shape(self, n_ctx=None, budget=None):
        w = self.w
        return fb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_fc,
                             w.n_ctx if n_ctx is None else n_ctx, self.n_cap,
                             w.budget if budget is None else budget, w.dtype, pairing=self.pairing)

    def pack(self, n_begin=0, n_end=None):
        fb.fasa_pack_kcache(self.shape, self.K, self.fc_idx, self.Kp, n_begin,
                            self.w.n_ctx if n_end is None else n_end)


def sets_from_T(T: np.ndarray):
    return [[T[b, h] for h in range(T.shape[1])] for b in range(T.shape[0])]
