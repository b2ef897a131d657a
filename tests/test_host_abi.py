"""CPU-side checks of the C-ABI library: it loads, exports every symbol include/atts.h declares,
and rejects bad arguments on the host before touching a device (no compute is launched here)."""
import ctypes
import os
import re

import pytest

import paper_2509_15148_amd as A
from paper_2509_15148_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "atts.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(atts_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert len(names) >= 18
    lib = ctypes.CDLL(A.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(A.EXPORTS)


def test_error_string_and_status_codes():
    with pytest.raises(A.AttsError) as e:
        A.Calib(0)
    assert e.value.code == A.ERR_INVALID_ARG and "capacity" in str(e.value)
    with pytest.raises(A.AttsError) as e:
        A.Calib((1 << 30) + 1)
    assert e.value.code == A.ERR_INVALID_ARG


def test_null_handles_are_rejected_on_the_host():
    lib = B._lib
    null = ctypes.c_void_p(0)
    n = ctypes.c_int64()
    assert lib.atts_calib_size(null, ctypes.byref(n)) == A.ERR_INVALID_ARG
    assert lib.atts_calibrate_online(null, null, ctypes.c_int64(4), null) == A.ERR_INVALID_ARG
    alphas = (ctypes.c_double * 1)(0.1)
    assert lib.atts_classify_ordinal(null, null, ctypes.c_int64(0), alphas, 1, null, null, null, null, null) \
        == A.ERR_INVALID_ARG
    out = ctypes.c_size_t()
    assert lib.atts_workspace_bytes(null, 4, 2, 3, ctypes.byref(out)) == A.ERR_INVALID_ARG
    assert lib.atts_score_drafts(null, null, 1, null, null, 1, 1, 0, null, null, null, ctypes.c_size_t(0), null) \
        == A.ERR_INVALID_ARG
    assert lib.atts_model_destroy(null) == 0
    assert lib.atts_calib_destroy(null) == 0


def test_model_description_is_validated_before_any_device_call():
    lib = B._lib
    handle = ctypes.c_void_p()
    w = B._Weights()

    def create(**kw):
        base = dict(n_layers=1, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=128, vocab=100, dtype=0,
                    rope_theta=1e4, rms_eps=1e-6)
        base.update(kw)
        d = B._ModelDesc(*[base[k] for k, _ in B._ModelDesc._fields_])
        return lib.atts_model_create(ctypes.byref(d), ctypes.byref(w), ctypes.byref(handle))

    assert create(dtype=7) == A.ERR_INVALID_ARG
    assert create(d_model=0) == A.ERR_INVALID_ARG
    assert create(n_kv_heads=3) == A.ERR_SHAPE
    assert create(head_dim=15) == A.ERR_SHAPE
    assert create(head_dim=512) == A.ERR_SHAPE
    assert create(d_model=66, dtype=1) == A.ERR_SHAPE          # 132-byte rows are not 16-byte multiples
    assert create() == A.ERR_INVALID_ARG                        # all weight pointers are NULL
    assert b"NULL" in lib.atts_last_error_string()
    assert not handle.value


def test_stage_entry_points_validate_arguments():
    lib = B._lib
    null = ctypes.c_void_p(0)
    out = ctypes.c_size_t()
    assert lib.atts_lmhead_workspace_bytes(0, 10, ctypes.byref(out)) == A.ERR_INVALID_ARG
    assert lib.atts_lmhead_workspace_bytes(256, 1024, ctypes.byref(out)) == 0 and out.value > 0
    assert lib.atts_lmhead_logprobs(9, null, null, null, 1, 8, 8, null, null, ctypes.c_size_t(0), null) == A.ERR_INVALID_ARG
    assert lib.atts_gemm_nt(1, null, null, null, 4, 4, 8, null) == A.ERR_INVALID_ARG
    assert lib.atts_attention_workspace_bytes(1, 100, 2, 128, ctypes.byref(out)) == 0
    assert out.value == 2 * 128 * 128 * 2                         # [n_kv, hd, 128 padded rows] bf16
    assert lib.atts_attention_workspace_bytes(0, 100, 2, 32, ctypes.byref(out)) == 0 and out.value == 0
    assert lib.atts_attention_shared_prefix(1, null, null, 4, 1, 4, 2, 1, 128, null, ctypes.c_size_t(0), null) \
        == A.ERR_INVALID_ARG


def test_classic_pipeline_and_import_validate_arguments():
    lib = B._lib
    null = ctypes.c_void_p(0)
    out = ctypes.c_size_t()
    i64, f64 = ctypes.c_int64, ctypes.c_double
    assert lib.atts_classic_workspace_bytes(i64(0), ctypes.byref(out)) == A.ERR_INVALID_ARG
    assert lib.atts_classic_workspace_bytes(i64(1000), ctypes.byref(out)) == 0 and out.value >= 2 * 1000 * 4
    assert out.value % 256 == 0
    assert lib.atts_classic_normalize(null, i64(3), 0, null, null) == A.ERR_INVALID_ARG          # m < 1
    assert lib.atts_classic_normalize(null, i64(3), 4, null, null) == A.ERR_INVALID_ARG          # NULL arrays
    assert lib.atts_classic_normalize(null, i64(0), 4, null, null) == 0                          # nothing to do
    one = ctypes.c_void_p(256)                                                                   # non-NULL, never dereferenced
    assert lib.atts_classic_threshold(one, i64(10), f64(1.5), one, one, ctypes.c_size_t(1 << 20), null) == A.ERR_INVALID_ARG
    assert lib.atts_classic_threshold(one, i64(10), f64(0.1), one, null, ctypes.c_size_t(0), null) == A.ERR_WORKSPACE
    assert lib.atts_classic_threshold(one, i64(10), f64(0.1), one, one, ctypes.c_size_t(16), null) == A.ERR_WORKSPACE
    assert lib.atts_classic_prediction_sets(null, i64(5), null, null, null) == A.ERR_INVALID_ARG
    assert lib.atts_classic_prediction_sets(null, i64(0), null, null, null) == 0
    assert lib.atts_calib_import(null, null, i64(0), null) == A.ERR_INVALID_ARG
