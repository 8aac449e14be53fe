"""The C-ABI library loads, exports every symbol include/radar.h declares, and its
host-side argument checks answer without touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2512_14069_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build_library(force=False)
    return binding.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "radar.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(radar_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2512_14069_amd import binding
    names = declared_functions()
    assert len(names) >= 12
    assert sorted(binding.EXPORTS) == names
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings_and_version(lib):
    from paper_2512_14069_amd import binding
    assert binding.radar_version() >= 100
    assert binding.status_string(0) == "ok"
    for code in (-1, -2, -3, -4, -99):
        assert binding.status_string(code)


def test_workspace_queries(lib):
    from paper_2512_14069_amd import binding as b
    d = b.expand_desc(10, 128256, 10, 0, 810)
    n = b.radar_draft_expand_workspace_bytes(d)
    assert n >= 4096 + 10 * 32 * 16 * 8 and n % 256 == 0
    a = b.accept_desc(1, 60, 128256, 59, 0, 1.0)
    assert b.radar_verify_accept_workspace_bytes(a) >= 4096 + 60 * 32 * 16
    assert b.radar_draft_rerank_workspace_bytes(810, 60) >= 0


def test_host_side_argument_checks_need_no_gpu(lib):
    """Validation happens before any kernel launch: bad descriptors come back as status codes."""
    from paper_2512_14069_amd import binding as b
    one = ctypes.c_void_p(256)      # never dereferenced: every case below is rejected first
    d = b.expand_desc(10, 128256, 10, 0, 50)                      # pool too small
    args = [one] * 12
    assert lib.radar_draft_expand(*args, ctypes.byref(d), one, 1 << 30, None) == -1
    d = b.expand_desc(10, 128256, 17, 0, 5000)                    # k above the compiled limit
    assert lib.radar_draft_expand(*args, ctypes.byref(d), one, 1 << 30, None) == -2
    d = b.expand_desc(10, 128256, 10, 0, 5000)
    assert lib.radar_draft_expand(*args, ctypes.byref(d), one, 16, None) == -3   # workspace too small
    assert lib.radar_draft_expand(*([None] + args[1:]), ctypes.byref(d), one, 1 << 30, None) == -1
    a = b.accept_desc(1, 65, 1000, 10, 0, 1.0)                    # T above 64
    assert lib.radar_verify_accept(*([one] * 8), ctypes.byref(a), one, 1 << 30, None) == -2
    a = b.accept_desc(1, 60, 1000, 59, 1, 0.0)                    # sampling needs temperature > 0
    assert lib.radar_verify_accept(*([one] * 8), ctypes.byref(a), one, 1 << 30, None) == -1
    a = b.accept_desc(1, 60, 1000, 59, 1, 1.0)                    # sampling needs uniforms
    assert lib.radar_verify_accept(one, one, one, one, None, one, one, one, ctypes.byref(a), one, 1 << 30, None) == -1
    assert lib.radar_draft_rerank(one, one, one, 5000, 10, 0, one, one, one, one, one, one, one, 256, None) == -2
    assert lib.radar_draft_rerank(one, one, one, 100, 64, 0, one, one, one, one, one, one, one, 256, None) == -2
    assert lib.radar_workspace_init(None, 4096, None) == -1
