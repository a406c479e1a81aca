"""ctypes binding of libfasa.so: argument marshalling only, same names as include/fasa.h.

Device buffers are torch tensors (torch is used for HBM allocation and streams, nothing else);
bf16 tensors may be passed as torch.bfloat16 or as int16/uint16 bit patterns.  Every function
raises FasaError on a non-zero status.  Importing this module fails loudly if the library has not
been built (python -m paper_2602_03152_amd.build): there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

# torch first: it brings its own HIP runtime (libamdhip64.so.7); libfasa.so asks for the same
# soname and must bind to the copy torch's allocator and streams live in, not to a second one.
import torch  # noqa: F401

# FASA_LIB names another build of the same library (the traced one of build.py --trace); default: in-tree
_LIB_PATH = os.environ.get("FASA_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libfasa.so")

FASA_OK, FASA_EINVAL, FASA_EUNSUPPORTED, FASA_EWORKSPACE, FASA_EHIP = 0, -1, -2, -3, -4
FASA_BF16, FASA_F32 = 0, 1
FASA_PAIR_ROTATE_HALF, FASA_PAIR_INTERLEAVED, FASA_PAIR_LIST = 0, 1, 2

EXPORTS = [
    "fasa_workspace_bytes", "fasa_workspace_init", "fasa_validate_fc_idx", "fasa_pack_kcache", "fasa_score", "fasa_topk",
    "fasa_sparse_attend", "fasa_dense_attend", "fasa_decode_step", "fasa_decode_step_static", "fasa_decode_step_ragged",
    "fasa_pack_kcache_paged", "fasa_decode_step_paged",
    "fasa_offload_stage_bytes",
    "fasa_offload_split_kcache", "fasa_offload_decode_step", "fasa_calibration_workspace_bytes",
    "fasa_contextual_agreement", "fasa_select_dominant_fcs", "fasa_strerror",
    "fasa_last_hip_error", "fasa_version", "fasa_profile_enable", "fasa_profile_reset",
    "fasa_profile_collect", "fasa_profile_entry",
]


class FasaShape(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("n_fc", C.c_int32), ("n_ctx", C.c_int32), ("n_cap", C.c_int32), ("budget", C.c_int32),
        ("dtype", C.c_int32), ("pairing", C.c_int32),
        ("kv_stride_b", C.c_int64), ("kv_stride_h", C.c_int64), ("kv_stride_n", C.c_int64),
    ]


class FasaPaging(C.Structure):
    _fields_ = [("block_table", C.c_void_p), ("max_blocks", C.c_int32), ("page_size", C.c_int32),
                ("n_pool_blocks", C.c_int32), ("reserved", C.c_int32)]


class FasaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib.fasa_strerror(status).decode()
        if status == FASA_EHIP:
            msg += " [hipError %d]" % _lib.fasa_last_hip_error()
        super().__init__("%s: %s (%d)" % (where, msg, status))


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libfasa.so is not built; run `python -m paper_2602_03152_amd.build` "
                          "(expected at %s)" % _LIB_PATH)
    lib = C.CDLL(_LIB_PATH)
    P, I32, SZ = C.c_void_p, C.c_int32, C.c_size_t
    SP = C.POINTER(FasaShape)
    lib.fasa_workspace_bytes.argtypes = [SP]; lib.fasa_workspace_bytes.restype = SZ
    lib.fasa_workspace_init.argtypes = [SP, P, SZ, P]; lib.fasa_workspace_init.restype = C.c_int
    lib.fasa_validate_fc_idx.argtypes = [SP, P]; lib.fasa_validate_fc_idx.restype = C.c_int
    lib.fasa_pack_kcache.argtypes = [SP, P, P, P, I32, I32, P]; lib.fasa_pack_kcache.restype = C.c_int
    lib.fasa_score.argtypes = [SP, P, P, P, P, P]; lib.fasa_score.restype = C.c_int
    lib.fasa_topk.argtypes = [SP, P, P, P, SZ, P]; lib.fasa_topk.restype = C.c_int
    lib.fasa_sparse_attend.argtypes = [SP, P, P, P, P, P, P, SZ, P]; lib.fasa_sparse_attend.restype = C.c_int
    lib.fasa_dense_attend.argtypes = [SP, P, P, P, P, P, SZ, P]; lib.fasa_dense_attend.restype = C.c_int
    lib.fasa_decode_step.argtypes = [SP, P, P, P, P, P, P, P, P, P, P, P, SZ, P]
    lib.fasa_decode_step.restype = C.c_int
    lib.fasa_decode_step_static.argtypes = [SP, P, P, P, P, P, P, P, P, P, P, P]
    lib.fasa_decode_step_static.restype = C.c_int
    lib.fasa_decode_step_ragged.argtypes = [SP, P, P, P, P, P, P, P, P, P, P, P, P, P, SZ, P]
    lib.fasa_decode_step_ragged.restype = C.c_int
    PP = C.POINTER(FasaPaging)
    lib.fasa_pack_kcache_paged.argtypes = [SP, PP, P, P, P, I32, I32, P]
    lib.fasa_pack_kcache_paged.restype = C.c_int
    lib.fasa_decode_step_paged.argtypes = [SP, PP, P, P, P, P, P, P, P, P, P, P, P, P, P, SZ, P]
    lib.fasa_decode_step_paged.restype = C.c_int
    lib.fasa_offload_stage_bytes.argtypes = [SP]; lib.fasa_offload_stage_bytes.restype = SZ
    lib.fasa_offload_split_kcache.argtypes = [SP, P, P, P, P, I32, I32, P]
    lib.fasa_offload_split_kcache.restype = C.c_int
    lib.fasa_offload_decode_step.argtypes = [SP, P, P, P, P, P, P, P, P, P, P, P, SZ, P, SZ, P]
    lib.fasa_offload_decode_step.restype = C.c_int
    lib.fasa_calibration_workspace_bytes.argtypes = [SP, I32]; lib.fasa_calibration_workspace_bytes.restype = SZ
    lib.fasa_contextual_agreement.argtypes = [SP, P, P, I32, P, P, SZ, P]
    lib.fasa_contextual_agreement.restype = C.c_int
    lib.fasa_select_dominant_fcs.argtypes = [SP, P, P]; lib.fasa_select_dominant_fcs.restype = C.c_int
    lib.fasa_strerror.argtypes = [C.c_int]; lib.fasa_strerror.restype = C.c_char_p
    lib.fasa_last_hip_error.argtypes = []; lib.fasa_last_hip_error.restype = C.c_int
    lib.fasa_version.argtypes = []; lib.fasa_version.restype = C.c_int
    lib.fasa_profile_enable.argtypes = [C.c_int]; lib.fasa_profile_enable.restype = C.c_int
    lib.fasa_profile_reset.argtypes = []; lib.fasa_profile_reset.restype = C.c_int
    lib.fasa_profile_collect.argtypes = []; lib.fasa_profile_collect.restype = C.c_int
    lib.fasa_profile_entry.argtypes = [C.c_int, C.c_char_p, SZ, C.POINTER(C.c_int64), C.POINTER(C.c_double)]
    lib.fasa_profile_entry.restype = C.c_int
    return lib


_lib = _load()
lib = _lib   # raw handle, for tests of the C ABI itself


def make_shape(batch, n_q_heads, n_kv_heads, head_dim, n_fc, n_ctx, n_cap, budget, dtype,
               kv_stride_b=None, kv_stride_h=None, kv_stride_n=None, pairing=0) -> FasaShape:
    """Shape struct; K/V strides default to a contiguous [batch][n_kv_heads][n_cap][head_dim] cache.
    pairing: FASA_PAIR_* or "half" | "interleaved" | "list"."""
    sn = head_dim if kv_stride_n is None else kv_stride_n
    sh = n_cap * sn if kv_stride_h is None else kv_stride_h
    sb = n_kv_heads * sh if kv_stride_b is None else kv_stride_b
    code = {"bf16": FASA_BF16, "f32": FASA_F32, FASA_BF16: FASA_BF16, FASA_F32: FASA_F32}[dtype]
    pair = {"half": FASA_PAIR_ROTATE_HALF, "interleaved": FASA_PAIR_INTERLEAVED, "list": FASA_PAIR_LIST}.get(pairing, pairing)
    return FasaShape(batch, n_q_heads, n_kv_heads, head_dim, n_fc, n_ctx, n_cap, budget, code, int(pair), sb, sh, sn)


def _ptr(x) -> Optional[int]:
    """Raw address of a torch tensor / numpy array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if hasattr(x, "ctypes"):
        return x.ctypes.data
    raise TypeError("cannot take the address of %r" % type(x))


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if hasattr(stream, "cuda_stream"):
        return stream.cuda_stream
    return int(stream)


def _check(status: int, where: str):
    if status != FASA_OK:
        raise FasaError(status, where)


def fasa_workspace_bytes(shape: FasaShape) -> int:
    return int(_lib.fasa_workspace_bytes(C.byref(shape)))


def fasa_workspace_init(shape: FasaShape, ws, ws_bytes: int, stream=None) -> None:
    _check(_lib.fasa_workspace_init(C.byref(shape), _ptr(ws), ws_bytes, _stream(stream)), "fasa_workspace_init")


def fasa_validate_fc_idx(shape: FasaShape, fc_idx_host) -> None:
    _check(_lib.fasa_validate_fc_idx(C.byref(shape), _ptr(fc_idx_host)), "fasa_validate_fc_idx")


def fasa_pack_kcache(shape, K, fc_idx, Kp, n_begin: int, n_end: int, stream=None) -> None:
    _check(_lib.fasa_pack_kcache(C.byref(shape), _ptr(K), _ptr(fc_idx), _ptr(Kp), n_begin, n_end,
                                 _stream(stream)), "fasa_pack_kcache")


def fasa_score(shape, q, Kp, fc_idx, S, stream=None) -> None:
    _check(_lib.fasa_score(C.byref(shape), _ptr(q), _ptr(Kp), _ptr(fc_idx), _ptr(S), _stream(stream)),
           "fasa_score")


def fasa_topk(shape, S, T, ws, ws_bytes: int, stream=None) -> None:
    _check(_lib.fasa_topk(C.byref(shape), _ptr(S), _ptr(T), _ptr(ws), ws_bytes, _stream(stream)), "fasa_topk")


def fasa_sparse_attend(shape, q, K, V, T, O, ws, ws_bytes: int, stream=None) -> None:
    _check(_lib.fasa_sparse_attend(C.byref(shape), _ptr(q), _ptr(K), _ptr(V), _ptr(T), _ptr(O), _ptr(ws),
                                   ws_bytes, _stream(stream)), "fasa_sparse_attend")


def fasa_dense_attend(shape, q, K, V, O, ws, ws_bytes: int, stream=None) -> None:
    _check(_lib.fasa_dense_attend(C.byref(shape), _ptr(q), _ptr(K), _ptr(V), _ptr(O), _ptr(ws), ws_bytes,
                                  _stream(stream)), "fasa_dense_attend")


def fasa_decode_step(shape, q, K, V, Kp, fc_idx, k_new, v_new, S, T, O, ws, ws_bytes: int, stream=None) -> None:
    _check(_lib.fasa_decode_step(C.byref(shape), _ptr(q), _ptr(K), _ptr(V), _ptr(Kp), _ptr(fc_idx),
                                 _ptr(k_new), _ptr(v_new), _ptr(S), _ptr(T), _ptr(O), _ptr(ws), ws_bytes,
                                 _stream(stream)), "fasa_decode_step")


FASA_STATIC_WS_BYTES = 32 << 20


def fasa_decode_step_static(shape, q, K, V, Kp, fc_idx, k_new, v_new, S, T, O, stream=None) -> None:
    _check(_lib.fasa_decode_step_static(C.byref(shape), _ptr(q), _ptr(K), _ptr(V), _ptr(Kp), _ptr(fc_idx),
                                        _ptr(k_new), _ptr(v_new), _ptr(S), _ptr(T), _ptr(O), _stream(stream)),
           "fasa_decode_step_static")


def fasa_decode_step_ragged(shape, q, K, V, Kp, fc_idx, k_new, v_new, n_ctx_seq, budget_seq, S, T, O, ws,
                            ws_bytes: int, stream=None) -> None:
    _check(_lib.fasa_decode_step_ragged(C.byref(shape), _ptr(q), _ptr(K), _ptr(V), _ptr(Kp), _ptr(fc_idx),
                                        _ptr(k_new), _ptr(v_new), _ptr(n_ctx_seq), _ptr(budget_seq),
                                        _ptr(S), _ptr(T), _ptr(O), _ptr(ws), ws_bytes, _stream(stream)),
           "fasa_decode_step_ragged")


def make_paging(block_table, page_size: int, n_pool_blocks: int) -> FasaPaging:
    """Paging struct for a DEVICE int32 block table [batch][max_blocks] (the tensor must outlive the call)."""
    return FasaPaging(_ptr(block_table), int(block_table.shape[1]), int(page_size), int(n_pool_blocks), 0)


def fasa_pack_kcache_paged(shape, paging, K, fc_idx, Kp, n_begin: int, n_end: int, stream=None) -> None:
    _check(_lib.fasa_pack_kcache_paged(C.byref(shape), C.byref(paging), _ptr(K), _ptr(fc_idx), _ptr(Kp), n_begin,
                                       n_end, _stream(stream)), "fasa_pack_kcache_paged")


def fasa_decode_step_paged(shape, paging, q, K, V, Kp, fc_idx, k_new, v_new, n_ctx_seq, budget_seq, S, T, O, ws,
                           ws_bytes: int, stream=None) -> None:
    _check(_lib.fasa_decode_step_paged(C.byref(shape), C.byref(paging), _ptr(q), _ptr(K), _ptr(V), _ptr(Kp),
                                       _ptr(fc_idx), _ptr(k_new), _ptr(v_new), _ptr(n_ctx_seq), _ptr(budget_seq),
                                       _ptr(S), _ptr(T), _ptr(O), _ptr(ws), ws_bytes, _stream(stream)),
           "fasa_decode_step_paged")


def fasa_offload_stage_bytes(shape: FasaShape) -> int:
    return int(_lib.fasa_offload_stage_bytes(C.byref(shape)))


def fasa_offload_split_kcache(shape, K, fc_idx, Kp, Knd_host, n_begin: int, n_end: int, stream=None) -> None:
    _check(_lib.fasa_offload_split_kcache(C.byref(shape), _ptr(K), _ptr(fc_idx), _ptr(Kp), _ptr(Knd_host),
                                          n_begin, n_end, _stream(stream)), "fasa_offload_split_kcache")


def fasa_offload_decode_step(shape, q, Kp, fc_idx, Knd_host, V_host, k_new, v_new, S, T, O, ws, ws_bytes: int,
                             stage, stage_bytes: int, stream=None) -> None:
    _check(_lib.fasa_offload_decode_step(C.byref(shape), _ptr(q), _ptr(Kp), _ptr(fc_idx), _ptr(Knd_host),
                                         _ptr(V_host), _ptr(k_new), _ptr(v_new), _ptr(S), _ptr(T), _ptr(O),
                                         _ptr(ws), ws_bytes, _ptr(stage), stage_bytes, _stream(stream)),
           "fasa_offload_decode_step")


def fasa_calibration_workspace_bytes(shape: FasaShape, top_k: int) -> int:
    return int(_lib.fasa_calibration_workspace_bytes(C.byref(shape), top_k))


def fasa_contextual_agreement(shape, q, Kp_all, top_k: int, CA_sum, cws, cws_bytes: int, stream=None) -> None:
    _check(_lib.fasa_contextual_agreement(C.byref(shape), _ptr(q), _ptr(Kp_all), top_k, _ptr(CA_sum), _ptr(cws),
                                          cws_bytes, _stream(stream)), "fasa_contextual_agreement")


def fasa_select_dominant_fcs(shape, ca_mean_host, fc_idx_host_out) -> None:
    _check(_lib.fasa_select_dominant_fcs(C.byref(shape), _ptr(ca_mean_host), _ptr(fc_idx_host_out)),
           "fasa_select_dominant_fcs")


def fasa_strerror(status: int) -> str:
    return _lib.fasa_strerror(status).decode()


def fasa_last_hip_error() -> int:
    return int(_lib.fasa_last_hip_error())


def fasa_version() -> int:
    return int(_lib.fasa_version())


def fasa_profile_enable(on: bool) -> None:
    _check(_lib.fasa_profile_enable(1 if on else 0), "fasa_profile_enable")


def fasa_profile_reset() -> None:
    _check(_lib.fasa_profile_reset(), "fasa_profile_reset")


def fasa_profile_collect() -> int:
    """Synchronises the device, folds the recorded launches; returns the number of kernels seen."""
    n = _lib.fasa_profile_collect()
    if n < 0:
        raise FasaError(n, "fasa_profile_collect")
    return int(n)


def fasa_profile_entry(i: int):
    """(kernel name, launches, total_ms) of entry i."""
    buf = C.create_string_buffer(128)
    launches, ms = C.c_int64(0), C.c_double(0.0)
    _check(_lib.fasa_profile_entry(i, buf, 128, C.byref(launches), C.byref(ms)), "fasa_profile_entry")
    return buf.value.decode(), int(launches.value), float(ms.value)


def profile_summary() -> dict:
    """{kernel name: (launches, total_ms)} since the last reset (convenience over the two calls above)."""
    out = {}
    for i in range(fasa_profile_collect()):
        name, launches, ms = fasa_profile_entry(i)
        out[name] = (launches, ms)
    return out
