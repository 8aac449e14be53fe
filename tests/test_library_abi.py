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


def test_host_side_checks_of_the_widened_entry_points(lib):
    """Prediction model, cycle state and draft-distribution verification: rejected before any launch."""
    from paper_2512_14069_amd import binding as b
    one = ctypes.c_void_p(256)

    def params(k=10, H=128, M=128, w_hh=256):
        pp = b.PolicyParams()
        for n in ("w_ih", "b_ih", "b_hh", "w1", "b1", "w2", "b2"):
            setattr(pp, n, 256)
        pp.w_hh, pp.k, pp.H, pp.M = w_hh, k, H, M
        return pp

    step = lambda pp, h=one, c=one, B=1: lib.radar_policy_step(one, h, c, ctypes.byref(pp), None, one, one, one, one, one, B, None)
    assert step(params(H=64)) == -2                                # only H = 128 is built
    assert step(params(M=129)) == -2
    assert step(params(k=17)) == -2
    assert step(params(k=0)) == -1
    assert step(params(w_hh=260)) == -1                            # w_hh rows are read 16 bytes per lane
    assert step(params(), h=one, c=None) == -1                     # h and c come together
    assert step(params(), h=ctypes.c_void_p(260)) == -1            # h is read 16 bytes per lane
    assert step(params(), B=-1) == -1
    assert step(params(), B=0) == 0                                # nothing to do, nothing launched

    io = b.PolicyIO()
    for n in ("h_out", "c_out", "logits", "probs", "action"):
        setattr(io, n, 256)
    d = b.expand_desc(10, 128256, 10, 0, 5000)
    fused = lambda pp, io_, desc: lib.radar_draft_expand_policy(*([one] * 12), ctypes.byref(desc), ctypes.byref(pp),
                                                                ctypes.byref(io_), one, 1 << 30, None)
    assert fused(params(k=8), io, d) == -1                         # the model must read exactly k confidences
    io_bad = b.PolicyIO()
    assert fused(params(), io_bad, d) == -1                        # outputs missing
    cyc = lambda desc, pp, io_, state: lib.radar_draft_expand_cycle(
        *([one] * 12), ctypes.byref(desc), None if pp is None else ctypes.byref(pp), None if io_ is None else ctypes.byref(io_),
        state, one, 1 << 30, None)
    assert cyc(d, None, None, None) == -1                          # no state
    assert cyc(d, None, io, one) == -1                             # io without a model
    assert cyc(b.expand_desc(10, 128256, 10, 4950, 5000), None, None, one) == -1   # the pool could overflow
    assert lib.radar_cycle_begin(None, None) == -1
    assert lib.radar_draft_rerank_cycle(one, one, one, None, 100, 10, 0, one, one, one, one, one, one, one, 256, None) == -1
    assert lib.radar_draft_rerank_cycle(one, one, one, one, 5000, 10, 0, one, one, one, one, one, one, one, 256, None) == -2

    q = lambda desc, q_rows=one: lib.radar_verify_accept_q(one, one, q_rows, one, one, one, one, one, one, one,
                                                           ctypes.byref(desc), one, 1 << 40, None)
    assert q(b.accept_q_desc(1, 65, 65, 1000, 10)) == -2            # T above 64
    assert q(b.accept_q_desc(1, 60, 60, 1 << 21, 10)) == -2         # vocabulary above the compiled limit
    assert q(b.accept_q_desc(1, 60, 30, 1000, 10), q_rows=None) == -1   # no row map and Tq != T
    assert q(b.accept_q_desc(1, 60, 60, 1000, 10, temperature=0.0)) == -1
    assert q(b.accept_q_desc(1, 60, 60, 1000, 10, draft_temperature=-1.0)) == -1
    assert q(b.accept_q_desc(600, 60, 60, 1000, 10)) == -2          # rows ride on one grid dimension
    small = b.accept_q_desc(1, 60, 60, 1000, 10)
    assert lib.radar_verify_accept_q(one, one, one, one, one, one, one, one, one, one, ctypes.byref(small), one, 16, None) == -3
    assert b.radar_verify_accept_q_workspace_bytes(small) >= 1000 * 4
