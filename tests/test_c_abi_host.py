"""Host-side checks of the C ABI: the library loads, exports every function the header
declares, and its pure-host entry points validate arguments.  No compute call is made."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "lychee.h")


@pytest.fixture(scope="module")
def lb():
    from paper_2602_04541_amd import binding
    return binding


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lychee_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_function_is_exported(lb):
    names = _declared_functions()
    assert "lychee_decode_attn" in names and "lychee_decode_step" in names
    lib = ctypes.CDLL(lb.LIB_PATH)
    for name in names:
        assert hasattr(lib, name), "%s is declared in lychee.h but not exported" % name
    assert sorted(lb.EXPORTS) == names


def test_shape_validation(lb):
    ok = lb.make_shape(1, 32, 8, 131072, 4096)
    assert lb.check_shape(ok) == lb.OK
    assert lb.check_shape(lb.make_shape(1, 32, 8, 131072, 4096, head_dim=64)) == lb.EUNSUPPORTED
    assert lb.check_shape(lb.make_shape(1, 64, 8, 1024, 16)) == lb.EUNSUPPORTED     # 8 q heads per KV head
    assert lb.check_shape(lb.make_shape(1, 30, 8, 1024, 16)) == lb.EINVAL           # not a multiple
    assert lb.check_shape(lb.make_shape(0, 32, 8, 1024, 16)) == lb.EINVAL
    assert lb.check_shape(lb.make_shape(257, 32, 8, 1024, 16)) == lb.EUNSUPPORTED
    assert lb.check_shape(lb.make_shape(1, 32, 8, 1024, 0)) == lb.EINVAL            # k < 1
    assert lb.check_shape(lb.make_shape(1, 32, 8, 0, 16)) == lb.EINVAL
    assert lb.check_shape(lb.make_shape(1, 32, 8, 1024, 16, strides=(8 * 1024 * 128, 1024 * 128, 64))) == lb.EINVAL
    assert lb.check_shape(lb.make_shape(1, 32, 8, 1024, 16, strides=(8 * 1024 * 132, 1024 * 132, 132))) == lb.EINVAL
    assert lb.check_shape(lb.make_shape(2, 32, 8, 1024, 16, strides=(0, 1024 * 128, 128))) == lb.EINVAL
    # token-major layout is fine
    assert lb.check_shape(lb.make_shape(2, 32, 8, 1024, 16, strides=(1024 * 8 * 128, 128, 8 * 128))) == lb.OK


def test_mask_validation(lb):
    s = lb.make_shape(1, 8, 2, 4096, 256)
    all_r = np.ones(8, np.uint8)
    mixed = np.array([1, 0, 0, 0, 1, 0, 0, 0], np.uint8)
    assert lb.check_shape(s, all_r, has_idx_in=False) == lb.OK
    assert lb.check_shape(s, mixed, has_idx_in=True) == lb.OK
    assert lb.check_shape(s, mixed, has_idx_in=False) == lb.EINVAL
    assert lb.check_shape(s, np.full(8, 2, np.uint8), has_idx_in=True) == lb.EINVAL


def test_workspace_size(lb):
    assert lb.workspace_bytes(lb.make_shape(1, 32, 8, 131072, 4096, head_dim=64)) == 0
    small = lb.workspace_bytes(lb.make_shape(1, 8, 2, 4096, 256))
    big = lb.workspace_bytes(lb.make_shape(1, 32, 8, 131072, 4096))
    assert 0 < small < big
    assert small % 256 == 0 and big % 256 == 0
    # selection scores alone need B * H_kv * L * 4 bytes
    assert big >= 8 * 131072 * 4
    assert big < 256 * 2 ** 20
    s = lb.make_shape(1, 32, 8, 131072, 4096)
    assert lb.step_workspace_bytes(s, 36) == 36 * big
    assert lb.step_workspace_bytes(s, 0) == 0 and lb.step_workspace_bytes(s, 1000) == 0


def test_error_strings(lb):
    assert lb.strerror(lb.OK) == "ok"
    for code in (lb.EINVAL, lb.EUNSUPPORTED, lb.EWORKSPACE, lb.EHIP):
        assert len(lb.strerror(code)) > 3
    assert "unknown" in lb.strerror(-99)


def test_calls_reject_null_context_without_touching_a_gpu(lb):
    lib = ctypes.CDLL(lb.LIB_PATH)
    s = lb.make_shape(1, 8, 2, 4096, 256)
    lib.lychee_set_option.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32]
    assert lib.lychee_set_option(None, lb.OPT_WG_PER_CU, 2) == lb.EINVAL
    lib.lychee_dense_decode_attn.argtypes = lb._lib.lychee_dense_decode_attn.argtypes
    assert lib.lychee_dense_decode_attn(None, ctypes.byref(s), None, None, None, None, None, None, 0, None) == lb.EINVAL
    lib.lychee_decode_attn_deferred.argtypes = lb._lib.lychee_decode_attn_deferred.argtypes
    assert lib.lychee_decode_attn_deferred(None, ctypes.byref(s), None, None, None, None, None, None, None, None,
                                           None, 0, None) == lb.EINVAL
    lib.lychee_select_flush.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    assert lib.lychee_select_flush(None, None) == lb.EINVAL


def test_create_fails_cleanly_without_a_gpu(lb):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(lb.LycheeError) as e:
        lb.Context(0)
    assert e.value.code == lb.EHIP


def test_ratio_rule_field_is_validated(lb):
    assert lb.check_shape(lb.make_shape(1, 8, 2, 4096, 256, keep_ppm=300000)) == lb.OK
    assert lb.check_shape(lb.make_shape(1, 8, 2, 4096, 256, keep_ppm=1000000)) == lb.OK
    assert lb.check_shape(lb.make_shape(1, 8, 2, 4096, 256, keep_ppm=1000001)) == lb.EINVAL
    assert lb.check_shape(lb.make_shape(1, 8, 2, 4096, 256, keep_ppm=-1)) == lb.EINVAL
    assert lb.check_shape(lb.make_shape(1, 8, 2, 4096, 256, block_size=64)) == lb.OK
    assert lb.check_shape(lb.make_shape(1, 8, 2, 4096, 256, block_size=1)) == lb.OK
    assert lb.check_shape(lb.make_shape(1, 8, 2, 4096, 256, block_size=32)) == lb.EUNSUPPORTED


def test_probability_rule_fields_are_validated(lb):
    ok = lb.make_shape(1, 8, 2, 4096, 256, prob_rule=lb.RULE_TOP_P, prob_param=0.9)
    assert lb.check_shape(ok) == lb.OK
    assert lb.check_shape(lb.make_shape(1, 8, 2, 4096, 256, prob_rule=lb.RULE_THRESHOLD, prob_param=1e-4)) == lb.OK
    assert lb.check_shape(lb.make_shape(1, 8, 2, 4096, 256, prob_rule=3, prob_param=0.5)) == lb.EINVAL
    assert lb.check_shape(lb.make_shape(1, 8, 2, 4096, 256, prob_rule=1, prob_param=0.0)) == lb.EINVAL
    assert lb.check_shape(lb.make_shape(1, 8, 2, 4096, 256, prob_rule=2, prob_param=1.5)) == lb.EINVAL
    assert lb.check_shape(lb.make_shape(1, 8, 2, 4096, 256, prob_rule=2, prob_param=0.5, block_size=64)) == lb.EUNSUPPORTED
    assert lb.check_shape(lb.make_shape(1, 8, 2, 4096, 256, prob_rule=2, prob_param=0.5, keep_ppm=1000)) == lb.EUNSUPPORTED
