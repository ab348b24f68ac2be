"""The C-ABI library loads and exports every function include/oxy.h declares.  No GPU,
no compute calls."""
import ctypes
import os
import re

from paper_2603_14371_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "oxy.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(oxy_[a-z_]+)\s*\(", text)))


def test_every_declared_function_is_exported_and_bound():
    names = _declared()
    assert "oxy_pool_create" in names and "oxy_prefix_append" in names
    assert "oxy_stream_append" in names and "oxy_mixed_attention" in names
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == names
    for name in names:
        assert callable(getattr(binding, name)), name
    assert binding.oxy_version() == 1


def test_signatures_carry_no_framework_types():
    text = open(os.path.join(ROOT, "include", "oxy.h")).read()
    assert "torch" not in text and "at::" not in text and "#include <hip" not in text


def test_invalid_configs_are_rejected_without_a_device():
    cfg = binding.make_config(2, 8, flags=binding.POOL_HOST_ONLY, head_dim=128)
    assert binding.oxy_kv_bytes(cfg) == 0
    try:
        binding.oxy_pool_create(cfg)
        assert False
    except binding.OxyError as e:
        assert e.code == binding.ERR_INVALID_ARG
    cfg = binding.make_config(2, 8)                # not host-only but no device buffers
    try:
        binding.oxy_pool_create(cfg)
        assert False
    except binding.OxyError as e:
        assert e.code == binding.ERR_INVALID_ARG
    cfg = binding.make_config(18, 8192)
    assert binding.oxy_kv_bytes(cfg) == 18 * 8192 * 16384
