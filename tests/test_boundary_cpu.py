"""The C-ABI library without a GPU: it loads, exports every symbol the header declares, and
rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

import paper_2510_02329_amd as sj
from paper_2510_02329_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sj.lib_path()):
        from paper_2510_02329_amd.build import build_library
        build_library(verbose=False)
    return sj.load_library()


def _declared():
    text = open(os.path.join(ROOT, "include", "sj.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sj_[a-z_0-9]+)\s*\(", text)) - {"sj_tensor_fn"})


def test_exports_every_declared_symbol(lib):
    names = _declared()
    assert "sj_verify_step" in names and "sj_model_load" in names and len(names) >= 17
    for n in names:
        assert hasattr(lib, n), n


def test_binding_has_the_same_names():
    for n in _declared():
        assert hasattr(sj, n), n


def _cfg(**kw):
    base = dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ffn=768, vocab=4096,
                dtype=0, rope_base=10000.0, rms_eps=1e-5, temperature=1.0, max_gamma=4)
    base.update(kw)
    return sj.SJConfig(**base)


@pytest.mark.parametrize("bad", [dict(dtype=7), dict(d_model=250), dict(head_dim=96), dict(n_kv_heads=3),
                                 dict(max_gamma=0), dict(max_gamma=64), dict(temperature=-1.0), dict(vocab=1000),
                                 dict(d_ffn=100), dict(rope_base=0.5)])
def test_bad_config_is_einval(lib, bad):
    with pytest.raises(sj.SJError) as e:
        sj.sj_model_load(_cfg(**bad), lambda name, layer: None)
    assert e.value.code == binding.SJ_EINVAL
    assert sj.sj_last_error()


def test_null_arguments_are_einval(lib):
    out = C.c_void_p()
    assert lib.sj_model_load(None, binding._TENSOR_FN(lambda *a: 0), None, C.byref(out)) == binding.SJ_EINVAL
    assert lib.sj_kv_create(None, 1, None, C.byref(out)) == binding.SJ_EINVAL
    assert lib.sj_kv_free(None) == binding.SJ_EINVAL
    assert lib.sj_model_free(None) == binding.SJ_EINVAL
    assert lib.sj_verify_step(None, None, 4, None, None, None, 0.5, None, None, None) == binding.SJ_EINVAL
    assert lib.sj_verify_head(None, None, 4, None, None, None, None, 0.5, None, None, None) == binding.SJ_EINVAL
    assert lib.sj_prefill(None, None, 0, None, 1, None) == binding.SJ_EINVAL
    assert lib.sj_kv_set(None, 0, None, None, 0, 0) == binding.SJ_EINVAL
    assert lib.sj_kv_state(None, None, None) == binding.SJ_EINVAL
    assert lib.sj_debug_fetch(None, 0, None, 0) == binding.SJ_EINVAL
    assert lib.sj_set_mode(None, 0) == binding.SJ_EINVAL
    assert lib.sj_model_weight_bytes(None) == 0
    assert b"gfx950" in lib.sj_version()


def test_load_without_gpu_fails_loudly(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(sj.SJError) as e:
        sj.sj_model_load(_cfg(), lambda name, layer: None)
    assert e.value.code in (binding.SJ_EHIP, binding.SJ_ENOMEM)
