"""The C-ABI library builds, loads and exports every symbol include/river.h declares
(no compute calls: this runs without a GPU)."""
import ctypes
import os
import re

from paper_2604_18396_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "river.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(river_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    if build.is_stale():
        build.build()
    lib = ctypes.CDLL(build.LIB)
    names = declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in river.h but not exported"
    assert sorted(binding.EXPORTS) == names          # the binding covers the whole header


def test_host_side_validation_needs_no_gpu():
    lib = binding.load()
    from paper_2604_18396_amd import configs
    c = binding.make_config(configs.TINY)
    n = lib.river_workspace_bytes(ctypes.byref(c))
    # at least the two caches
    assert n >= 2 * 4 * 64 * 128 * 4
    bad = binding.make_config(configs.TINY.with_(head_dim=48))
    assert lib.river_workspace_bytes(ctypes.byref(bad)) == 0
    bad = binding.make_config(configs.TINY.with_(river_group=24))
    assert lib.river_workspace_bytes(ctypes.byref(bad)) == 0
    assert lib.river_workspace_bytes(None) == 0
    # the one-launch mode is offered for bf16 only
    bad = binding.make_config(configs.TINY, exec_mode=binding.EXEC_PERSISTENT)
    assert lib.river_workspace_bytes(ctypes.byref(bad)) == 0
    ok = binding.make_config(configs.TINY.with_(dtype=configs.DTYPE_BF16), exec_mode=binding.EXEC_PERSISTENT)
    assert lib.river_workspace_bytes(ctypes.byref(ok)) > 0
    bad = binding.make_config(configs.TINY.with_(river_group=24))
    h = ctypes.c_void_p()
    assert lib.river_create(ctypes.byref(bad), None, None, None, 0, None, ctypes.byref(h)) == binding.RIVER_EINVAL
    assert b"river_group" in lib.river_last_error(None)
    assert lib.river_destroy(None) == 0
    assert lib.river_position(None) == binding.RIVER_EINVAL
    assert lib.river_decode_step(None, None, None, None, None, None) == binding.RIVER_EINVAL
    assert lib.river_quantize_w4(None, 1, 64, 64, 0, None, None, None, None) == binding.RIVER_EINVAL
