"""Boundary checks that need no GPU: the shared library loads, exports every function the header
declares, and rejects bad arguments on the host before anything is enqueued."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _header_functions():
    text = open(os.path.join(ROOT, "include", "icecache.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ice_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2604_10539_amd import binding
    names = _header_functions()
    assert len(names) >= 12 and "ice_build_index" in names and "ice_select_attend" in names
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), "libicecache.so does not export %s" % n
    assert sorted(binding.SYMBOLS) == names, "binding and header disagree on the entry points"


def test_host_side_argument_errors():
    import paper_2604_10539_amd as p
    from paper_2604_10539_amd import binding as b
    good = p.make_config(1, 8, 4, 4096)
    assert p.ice_workspace_bytes(good, 16, 64) > 0
    for cfg, ps, nc in [(p.make_config(1, 8, 4, 4096, head_dim=64), 16, 64), (p.make_config(1, 8, 3, 4096), 16, 64),
                        (good, 8, 64), (good, 16, 0), (p.make_config(0, 8, 4, 4096), 16, 64)]:
        assert p.ice_workspace_bytes(cfg, ps, nc) == 0
    fake = 0x10000000  # a 256-byte aligned address that is never dereferenced on these paths

    def status(fn, *a):
        with pytest.raises(p.IceError) as e:
            fn(*a)
        return e.value.status

    assert status(p.ice_create, p.make_config(1, 8, 4, 4096, head_dim=64), fake, 1 << 30) == b.ICE_ERR_UNSUPPORTED
    assert status(p.ice_create, p.make_config(1, 8, 5, 4096), fake, 1 << 30) == b.ICE_ERR_UNSUPPORTED
    assert status(p.ice_create, good, fake + 8, 1 << 30) == b.ICE_ERR_INVALID_ARG
    assert status(p.ice_create, good, 0, 1 << 30) == b.ICE_ERR_INVALID_ARG
    h = p.ice_create(good, fake, 1 << 20)
    try:
        assert status(p.ice_insert, h, fake, fake) == b.ICE_ERR_STATE
        assert status(p.ice_select, h, fake, 256, fake, fake) == b.ICE_ERR_STATE
        assert status(p.ice_attend, h, fake, fake, fake, 16, fake) == b.ICE_ERR_STATE
        assert status(p.ice_export_index, h) == b.ICE_ERR_STATE
        assert status(p.ice_build_index, h, 0, fake, 1024, 16, 64) == b.ICE_ERR_INVALID_ARG
        assert status(p.ice_build_index, h, fake + 2, fake, 1024, 16, 64) == b.ICE_ERR_INVALID_ARG
        assert status(p.ice_build_index, h, fake, fake, 1024, 24, 64) == b.ICE_ERR_UNSUPPORTED
        assert status(p.ice_build_index, h, fake, fake, 32, 16, 64) == b.ICE_ERR_SHAPE        # clusters > tokens
        assert status(p.ice_build_index, h, fake, fake, 8192, 16, 64) == b.ICE_ERR_SHAPE      # tokens > max_tokens
        assert status(p.ice_build_index, h, fake, fake, 1024, 16, 64) == b.ICE_ERR_CAPACITY   # 1 MiB workspace
        assert "workspace" in p.ice_last_error()
    finally:
        p.ice_destroy(h)
    assert status(p.ice_destroy, 0) == b.ICE_ERR_INVALID_ARG


def test_peak_microbenchmarks_reject_bad_arguments():
    import paper_2604_10539_amd as p
    from paper_2604_10539_amd import binding as b
    fake = 0x10000000
    for call in (lambda: b.lib().ice_debug_peak_read(None, 1 << 20, fake, None),
                 lambda: b.lib().ice_debug_peak_read(fake + 4, 1 << 20, fake, None),
                 lambda: b.lib().ice_debug_peak_read(fake, 8, fake, None),
                 lambda: b.lib().ice_debug_peak_mfma(None, 16, None, None),
                 lambda: b.lib().ice_debug_peak_mfma(fake, 0, None, None)):
        assert call() == b.ICE_ERR_INVALID_ARG


def test_product_package_never_touches_the_oracle():
    pkg = os.path.join(ROOT, "paper_2604_10539_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), "%s mentions the oracle" % f
