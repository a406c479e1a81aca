"""The C-ABI library on a host without a GPU: it loads, exports every symbol the header declares,
and validates arguments before any HIP call (error codes, never a crash)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2602_03152_amd", "libfasa.so")

if not os.path.exists(LIB):   # build once if the tree is fresh (the GPU tests load what is built)
    from paper_2602_03152_amd import build as _build
    _build.build(verbose=False)

from paper_2602_03152_amd import binding as fb  # noqa: E402


def _declared():
    text = open(os.path.join(ROOT, "include", "fasa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fasa_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = _declared()
    assert len(names) >= 25 and "fasa_decode_step" in names and "fasa_pack_kcache" in names
    lib = C.CDLL(LIB)
    for n in names:
        assert hasattr(lib, n), n
        assert hasattr(fb, n), "binding lacks %s" % n
    assert sorted(fb.EXPORTS) == names


def _shape(**kw):
    base = dict(batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128, n_fc=16, n_ctx=1000, n_cap=1024,
                budget=100, dtype="bf16")
    base.update(kw)
    return fb.make_shape(**base)


def test_version_and_strerror():
    assert fb.fasa_version() >= 1000
    assert fb.fasa_strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -99):
        assert len(fb.fasa_strerror(code)) > 3


def test_workspace_bytes_is_pure_and_monotone():
    a = fb.fasa_workspace_bytes(_shape())
    assert a > 0 and a % 256 == 0 and a == fb.fasa_workspace_bytes(_shape())
    assert fb.fasa_workspace_bytes(_shape(n_cap=4096, n_ctx=4000)) > a
    assert fb.fasa_workspace_bytes(_shape(n_cap=1000)) == 0          # n_cap not a multiple of 64
    assert fb.fasa_workspace_bytes(_shape(n_ctx=2000)) == 0          # n_ctx > n_cap
    assert fb.fasa_workspace_bytes(_shape(budget=0)) == 0


def test_validate_fc_idx():
    s = _shape(n_fc=4)
    ok = np.tile(np.array([0, 63, 5, 17], np.int32), (8, 1))
    fb.fasa_validate_fc_idx(s, ok)
    for bad in ([0, 64, 5, 17], [0, -1, 5, 17], [5, 63, 5, 17]):
        arr = ok.copy(); arr[3] = bad
        with pytest.raises(fb.FasaError) as e:
            fb.fasa_validate_fc_idx(s, arr)
        assert e.value.status == fb.FASA_EINVAL
    with pytest.raises(fb.FasaError):
        fb.fasa_validate_fc_idx(s, None)


A = 0x10000   # a fake, 16-byte aligned "device pointer": validation must fail before it is touched


@pytest.mark.parametrize("kw,code", [
    (dict(batch=0), fb.FASA_EINVAL),
    (dict(n_q_heads=30), fb.FASA_EINVAL),              # not a multiple of n_kv_heads
    (dict(head_dim=127), fb.FASA_EINVAL),
    (dict(head_dim=64), fb.FASA_EUNSUPPORTED),
    (dict(n_q_heads=72), fb.FASA_EUNSUPPORTED),        # GQA group 9
    (dict(n_fc=0), fb.FASA_EINVAL),
    (dict(n_fc=65), fb.FASA_EINVAL),
    (dict(n_ctx=0), fb.FASA_EINVAL),
    (dict(n_ctx=1025), fb.FASA_EINVAL),
    (dict(budget=0), fb.FASA_EINVAL),
    (dict(n_cap=1000), fb.FASA_EINVAL),
    (dict(dtype=fb.FASA_F32, kv_stride_n=100), fb.FASA_EINVAL),
    (dict(kv_stride_n=132), fb.FASA_EINVAL),           # not a multiple of 8 elements
])
def test_decode_step_rejects_bad_shapes(kw, code):
    s = _shape(**kw)
    if "dtype" in kw and kw["dtype"] == fb.FASA_F32:
        pass
    rc = fb.lib.fasa_decode_step(C.byref(s), A, A, A, A, A, None, None, A, A, A, A, 1 << 40, None)
    assert rc == code


def test_pairing_field_is_validated():
    for bad in (3, -1, 1 << 20):
        s = _shape(); s.pairing = bad
        assert fb.lib.fasa_score(C.byref(s), A, A, A, A, None) == fb.FASA_EINVAL
        assert fb.fasa_workspace_bytes(s) == 0


def test_validate_explicit_pair_list():
    s = _shape(n_fc=3); s.pairing = fb.FASA_PAIR_LIST
    ok = np.tile(np.array([[0, 127], [64, 5], [17, 3]], np.int32), (8, 1, 1))
    fb.fasa_validate_fc_idx(s, ok)
    for bad in ([[0, 128], [64, 5], [17, 3]], [[0, -1], [64, 5], [17, 3]], [[0, 127], [64, 0], [17, 3]]):
        arr = ok.copy(); arr[5] = bad
        with pytest.raises(fb.FasaError) as e:
            fb.fasa_validate_fc_idx(s, arr)
        assert e.value.status == fb.FASA_EINVAL
    # FC numbers: the interleaved pairing takes the same lists as rotate-half
    s = _shape(n_fc=4); s.pairing = fb.FASA_PAIR_INTERLEAVED
    fb.fasa_validate_fc_idx(s, np.tile(np.array([0, 63, 5, 17], np.int32), (8, 1)))


def test_fc_number_entry_points_refuse_explicit_pairs():
    s = _shape(); s.pairing = fb.FASA_PAIR_LIST
    L = fb.lib
    assert fb.fasa_offload_stage_bytes(s) == 0
    assert L.fasa_offload_split_kcache(C.byref(s), A, A, A, A, 0, 10, None) == fb.FASA_EUNSUPPORTED
    assert L.fasa_offload_decode_step(C.byref(s), A, A, A, A, A, None, None, A, A, A, A, 1 << 40, A, 1 << 40,
                                      None) == fb.FASA_EUNSUPPORTED
    assert fb.fasa_calibration_workspace_bytes(s, 64) == 0
    assert L.fasa_contextual_agreement(C.byref(s), A, A, 64, A, A, 1 << 40, None) == fb.FASA_EUNSUPPORTED
    ca = np.zeros((8, 64), np.float32); out = np.zeros((8, 16), np.int32)
    assert L.fasa_select_dominant_fcs(C.byref(s), ca.ctypes.data, out.ctypes.data) == fb.FASA_EUNSUPPORTED


def test_null_and_misaligned_pointers():
    s = _shape()
    L = fb.lib
    assert L.fasa_score(C.byref(s), None, A, A, A, None) == fb.FASA_EINVAL
    assert L.fasa_score(C.byref(s), A, A + 4, A, A, None) == fb.FASA_EINVAL
    assert L.fasa_score(None, A, A, A, A, None) == fb.FASA_EINVAL
    assert L.fasa_pack_kcache(C.byref(s), A, A, None, 0, 10, None) == fb.FASA_EINVAL
    assert L.fasa_pack_kcache(C.byref(s), A, A, A, 10, 5, None) == fb.FASA_EINVAL
    assert L.fasa_pack_kcache(C.byref(s), A, A, A, 0, 1025, None) == fb.FASA_EINVAL
    assert L.fasa_pack_kcache(C.byref(s), A, A, A, 7, 7, None) == fb.FASA_OK      # empty range: nothing to do
    assert L.fasa_topk(C.byref(s), A, A + 8, A, 1 << 40, None) == fb.FASA_EINVAL
    assert L.fasa_topk(C.byref(s), A, A, None, 1 << 40, None) == fb.FASA_EINVAL
    assert L.fasa_sparse_attend(C.byref(s), A, A, A, None, A, A, 1 << 40, None) == fb.FASA_EINVAL
    assert L.fasa_dense_attend(C.byref(s), A, A, None, A, A, 1 << 40, None) == fb.FASA_EINVAL
    # k_new without v_new
    assert L.fasa_decode_step(C.byref(s), A, A, A, A, A, A, None, A, A, A, A, 1 << 40, None) == fb.FASA_EINVAL
    # ragged step: the length array is required, the budget array optional, both 4-byte aligned
    assert L.fasa_decode_step_ragged(C.byref(s), A, A, A, A, A, None, None, None, None, A, A, A, A, 1 << 40, None) == fb.FASA_EINVAL
    assert L.fasa_decode_step_ragged(C.byref(s), A, A, A, A, A, None, None, A + 2, None, A, A, A, A, 1 << 40, None) == fb.FASA_EINVAL
    assert L.fasa_decode_step_ragged(C.byref(s), A, A, A, A, A, None, None, A, A + 1, A, A, A, A, 1 << 40, None) == fb.FASA_EINVAL
    assert L.fasa_decode_step_ragged(C.byref(s), A, A, A, A, A, None, None, A, None, A, A, A, A, 0, None) == fb.FASA_EWORKSPACE


def test_paging_is_validated():
    s = _shape()
    L = fb.lib
    ok = fb.FasaPaging(A, 64, 16, 100, 0)
    call = lambda pg: L.fasa_decode_step_paged(C.byref(s), C.byref(pg), A, A, A, A, A, None, None, None, None,
                                               A, A, A, A, 0, None)
    assert call(ok) == fb.FASA_EWORKSPACE                                 # everything else is fine
    assert call(fb.FasaPaging(None, 64, 16, 100, 0)) == fb.FASA_EINVAL    # no table
    assert call(fb.FasaPaging(A + 2, 64, 16, 100, 0)) == fb.FASA_EINVAL   # misaligned table
    assert call(fb.FasaPaging(A, 64, 24, 100, 0)) == fb.FASA_EINVAL       # page size not a power of two
    assert call(fb.FasaPaging(A, 64, 0, 100, 0)) == fb.FASA_EINVAL
    assert call(fb.FasaPaging(A, 4, 16, 100, 0)) == fb.FASA_EINVAL        # table does not cover n_ctx
    assert call(fb.FasaPaging(A, 64, 16, 0, 0)) == fb.FASA_EINVAL         # empty pool
    assert call(fb.FasaPaging(A, 64, 16, 100, 1)) == fb.FASA_EINVAL       # reserved
    assert call(fb.FasaPaging(A, 64, 1024, 1 << 22, 0)) == fb.FASA_EUNSUPPORTED   # slots beyond 2^31
    assert L.fasa_decode_step_paged(C.byref(s), None, A, A, A, A, A, None, None, None, None, A, A, A, A, 1 << 40,
                                    None) == fb.FASA_EINVAL
    small = fb.FasaPaging(A, 4, 16, 100, 0)
    assert L.fasa_pack_kcache_paged(C.byref(s), C.byref(small), A, A, A, 0, 65, None) == fb.FASA_EINVAL  # table ends at 64
    assert L.fasa_pack_kcache_paged(C.byref(s), C.byref(ok), A, A, A, 5, 5, None) == fb.FASA_OK         # empty range


def test_workspace_too_small():
    s = _shape()
    need = fb.fasa_workspace_bytes(s)
    L = fb.lib
    assert L.fasa_topk(C.byref(s), A, A, A, need - 1, None) == fb.FASA_EWORKSPACE
    assert L.fasa_workspace_init(C.byref(s), A, need - 1, None) == fb.FASA_EWORKSPACE
    assert L.fasa_workspace_init(C.byref(s), None, need, None) == fb.FASA_EINVAL
    assert L.fasa_sparse_attend(C.byref(s), A, A, A, A, A, A, 16, None) == fb.FASA_EWORKSPACE
    assert L.fasa_decode_step(C.byref(s), A, A, A, A, A, None, None, A, A, A, A, 0, None) == fb.FASA_EWORKSPACE


def test_static_workspace_entry_point_refuses_before_any_hip_call():
    """fasa_decode_step_static: bad shapes, null pointers and shapes whose workspace exceeds the
    library's own array are refused on a host without a GPU (no HIP call is made before that)."""
    L = fb.lib
    assert fb.FASA_STATIC_WS_BYTES == 32 << 20
    text = open(os.path.join(ROOT, "include", "fasa.h")).read()
    assert re.search(r"#define\s+FASA_STATIC_WS_BYTES\s+\(32u\s*<<\s*20\)", text)
    big = _shape(batch=64, n_ctx=65536, n_cap=65536, budget=4096)
    assert fb.fasa_workspace_bytes(big) > fb.FASA_STATIC_WS_BYTES
    assert L.fasa_decode_step_static(C.byref(big), A, A, A, A, A, None, None, A, A, A, None) == fb.FASA_EWORKSPACE
    assert L.fasa_decode_step_static(C.byref(_shape(budget=0)), A, A, A, A, A, None, None, A, A, A, None) == fb.FASA_EINVAL
    assert L.fasa_decode_step_static(C.byref(_shape()), None, A, A, A, A, None, None, A, A, A, None) == fb.FASA_EINVAL
    assert L.fasa_decode_step_static(None, A, A, A, A, A, None, None, A, A, A, None) == fb.FASA_EINVAL


def test_binding_raises():
    s = _shape(budget=0)
    with pytest.raises(fb.FasaError) as e:
        fb.fasa_topk(s, A, A, A, 1 << 40, stream=0)
    assert e.value.status == fb.FASA_EINVAL and "invalid" in str(e.value)


def test_profile_api_without_launches():
    fb.fasa_profile_reset()
    fb.fasa_profile_enable(False)
    buf = C.create_string_buffer(8)
    assert fb.lib.fasa_profile_entry(0, buf, 8, None, None) == fb.FASA_EINVAL


def test_select_dominant_fcs_matches_the_oracle_rule():
    from oracle import fasa_oracle as O
    rng = np.random.default_rng(0)
    s = _shape(n_fc=16)
    ca = np.round(rng.random((8, 64)), 2).astype(np.float32)          # rounding creates ties
    out = np.zeros((8, 16), dtype=np.int32)
    fb.fasa_select_dominant_fcs(s, ca, out)
    np.testing.assert_array_equal(out, O.dominant_fcs(ca, 16))
    with pytest.raises(fb.FasaError):
        fb.fasa_select_dominant_fcs(s, None, out)


def test_calibration_and_offload_sizes_and_errors():
    s = _shape()
    assert fb.fasa_calibration_workspace_bytes(s, 64) > 64 * 8 * 1024 * 4
    assert fb.fasa_calibration_workspace_bytes(s, 0) == 0
    assert fb.fasa_calibration_workspace_bytes(_shape(batch=200), 64) == 0      # 200 * 8 * 64 virtual heads
    assert fb.fasa_offload_stage_bytes(s) == 2 * 8 * 100 * 128 * 2 + (-(2 * 8 * 100 * 128 * 2) % 256)
    L = fb.lib
    assert L.fasa_contextual_agreement(C.byref(s), A, A, 64, A, A, 16, None) == fb.FASA_EWORKSPACE
    assert L.fasa_contextual_agreement(C.byref(s), A, None, 64, A, A, 1 << 40, None) == fb.FASA_EINVAL
    assert L.fasa_offload_decode_step(C.byref(s), A, A, A, A, A, None, None, A, A, A, A, 1 << 40, A, 16, None) == fb.FASA_EWORKSPACE
    assert L.fasa_offload_decode_step(C.byref(s), A, A, A, None, A, None, None, A, A, A, A, 1 << 40, A, 1 << 40, None) == fb.FASA_EINVAL
    assert L.fasa_offload_split_kcache(C.byref(s), A, A, A, A, 5, 4, None) == fb.FASA_EINVAL


def test_header_is_plain_c_and_structs_match_the_binding(tmp_path):
    """include/fasa.h compiles as strict C99 and as C++, and the struct layouts the compiler sees are
    the ones the ctypes binding marshals."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None or shutil.which("g++") is None:
        pytest.skip("no host compiler")
    inc = os.path.join(ROOT, "include")
    src = tmp_path / "layout.c"
    fields_shape = [n for n, _ in fb.FasaShape._fields_]
    fields_paging = [n for n, _ in fb.FasaPaging._fields_]
    prints = ['printf("%zu\\n", sizeof(fasa_shape));', 'printf("%zu\\n", sizeof(fasa_paging));']
    prints += ['printf("%%zu\\n", offsetof(fasa_shape, %s));' % f for f in fields_shape]
    prints += ['printf("%%zu\\n", offsetof(fasa_paging, %s));' % f for f in fields_paging]
    src.write_text('#include <stddef.h>\n#include <stdio.h>\n#include "fasa.h"\nint main(void) {\n%s\nreturn 0; }\n'
                   % "\n".join(prints))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, str(src), "-o", str(exe)],
                   check=True)
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c++",
                    "-I", inc, str(src)], check=True)
    got = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    want = [C.sizeof(fb.FasaShape), C.sizeof(fb.FasaPaging)]
    want += [getattr(fb.FasaShape, f).offset for f in fields_shape]
    want += [getattr(fb.FasaPaging, f).offset for f in fields_paging]
    assert got == want
