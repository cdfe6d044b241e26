"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching any device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "lnmod.h")

from paper_2605_17923_amd import lnmod, lnmod_tools  # noqa: E402


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(lnmod.LIBRARY):
        from paper_2605_17923_amd.build import build_library
        build_library()
    return lnmod.library()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lnmod_[a-z_0-9]+)\s*\(", text)))


def dynamic_symbols(path):
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", path], capture_output=True, text=True, check=True).stdout
    return sorted(line.split()[-1] for line in out.splitlines() if line.strip())


def test_header_symbols_are_exported(lib):
    names = declared_functions()
    assert set(names) == set(lnmod.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_operator_library_exports_the_operator_and_scheduler_entry_points_only(lib):
    """No measurement or tuning entry, no C++ symbol and no variable leaves liblnmod.so."""
    sched = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "lnmod_sched.h")).read(), flags=re.S)
    sched_names = set(re.findall(r"\b(lnmod_[a-z_0-9]+)\s*\(", sched))
    assert sched_names
    assert set(dynamic_symbols(lnmod.LIBRARY)) == set(declared_functions()) | sched_names


def test_binding_mirrors_every_entry_point():
    for n in declared_functions():
        assert callable(getattr(lnmod, n)), n


def test_status_strings(lib):
    seen = set()
    for code in range(6):
        s = lnmod.lnmod_status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 6
    assert lnmod.lnmod_status_string(99) == "unknown status"


A = 0x1000          # a 16-byte aligned fake address; validation never dereferences it


def fwd(x=A, shift=A, scale=A, B=2, S=4, D=64, eps=1e-6, y=A, mean=A, rstd=A, dtype=0, mod=0):
    return lnmod.lnmod_forward(x, shift, scale, B, S, D, eps, None, y, mean, rstd, dtype, mod)


def bwd(dy=A, x=A, scale=A, B=2, S=4, D=64, eps=1e-6, mean=A, rstd=A, dx=A, dshift=A, dscale=A,
        ws=A, ws_bytes=1 << 40, dtype=0, mod=0):
    return lnmod.lnmod_backward(dy, x, None, scale, B, S, D, eps, None, mean, rstd, dx, dshift,
                                dscale, ws, ws_bytes, dtype, mod)


def test_forward_rejects_bad_arguments(lib):
    assert fwd(x=None) == lnmod.LNMOD_EINVAL
    assert fwd(shift=None) == lnmod.LNMOD_EINVAL
    assert fwd(mean=None) == lnmod.LNMOD_EINVAL                      # one statistic alone
    assert fwd(rstd=None) == lnmod.LNMOD_EINVAL
    assert fwd(mean=None, rstd=None, y=A + 2) == lnmod.LNMOD_EALIGN   # neither: valid so far
    assert fwd(B=-1) == lnmod.LNMOD_EINVAL
    assert fwd(S=-1) == lnmod.LNMOD_EINVAL
    assert fwd(B=1 << 20, S=1 << 20) == lnmod.LNMOD_EINVAL          # 2^40 tokens
    assert fwd(eps=0.0) == lnmod.LNMOD_EINVAL
    assert fwd(eps=-1e-6) == lnmod.LNMOD_EINVAL
    assert fwd(eps=float("nan")) == lnmod.LNMOD_EINVAL
    assert fwd(eps=float("inf")) == lnmod.LNMOD_EINVAL
    assert fwd(dtype=2) == lnmod.LNMOD_EINVAL
    assert fwd(mod=2) == lnmod.LNMOD_EINVAL
    assert fwd(D=0) == lnmod.LNMOD_EUNSUPPORTED
    assert fwd(D=60) == lnmod.LNMOD_EUNSUPPORTED                    # bf16 needs a multiple of 8
    assert fwd(D=62, dtype=1) == lnmod.LNMOD_EUNSUPPORTED           # fp32 needs a multiple of 4
    assert fwd(D=8200) == lnmod.LNMOD_EUNSUPPORTED
    assert fwd(x=A + 8) == lnmod.LNMOD_EALIGN
    assert fwd(y=A + 2) == lnmod.LNMOD_EALIGN
    # nothing to do: fine, and nothing is enqueued
    assert fwd(B=0) == lnmod.LNMOD_OK
    assert fwd(S=0) == lnmod.LNMOD_OK
    assert fwd(S=0, x=None, y=None) == lnmod.LNMOD_OK


def test_backward_rejects_bad_arguments(lib):
    assert bwd(dy=None) == lnmod.LNMOD_EINVAL
    assert bwd(dscale=None) == lnmod.LNMOD_EINVAL
    assert bwd(rstd=None) == lnmod.LNMOD_EINVAL                      # one statistic alone
    assert bwd(mean=None) == lnmod.LNMOD_EINVAL
    # without both statistics the call is a valid "recompute" request: later checks still apply
    assert bwd(mean=None, rstd=None, ws=None) == lnmod.LNMOD_EWORKSPACE
    assert bwd(mean=None, rstd=None, dx=A + 4) == lnmod.LNMOD_EALIGN
    assert bwd(D=12) == lnmod.LNMOD_EUNSUPPORTED
    assert bwd(dx=A + 4) == lnmod.LNMOD_EALIGN
    assert bwd(ws=None) == lnmod.LNMOD_EWORKSPACE
    need = lnmod.lnmod_backward_workspace_bytes(2, 8, 64, 0)
    assert need > 0
    assert bwd(ws_bytes=need - 1) == lnmod.LNMOD_EWORKSPACE
    assert bwd(ws=A + 4, ws_bytes=need) == lnmod.LNMOD_EALIGN
    assert bwd(mod=3) == lnmod.LNMOD_EINVAL
    assert bwd(B=0) == lnmod.LNMOD_OK
    assert bwd(S=0, mod=1) == lnmod.LNMOD_OK


def test_varlen_rejects_bad_arguments(lib):
    f = lnmod.lnmod_forward_varlen
    assert f(A, A, A, None, 3, 10, 64, 1e-6, None, A, A, A, 0) == lnmod.LNMOD_EINVAL
    assert f(A, A, A, A, -1, 10, 64, 1e-6, None, A, A, A, 0) == lnmod.LNMOD_EINVAL
    assert f(A, A, A, A, 0, 10, 64, 1e-6, None, A, A, A, 0) == lnmod.LNMOD_EINVAL   # tokens, no segment
    assert f(A, A, A, A, 3, 1 << 31, 64, 1e-6, None, A, A, A, 0) == lnmod.LNMOD_EINVAL
    assert f(A, A, A, A, 3, 10, 65, 1e-6, None, A, A, A, 0) == lnmod.LNMOD_EUNSUPPORTED
    assert f(A, A, A, A, 3, 0, 64, 1e-6, None, A, A, A, 0) == lnmod.LNMOD_OK
    b = lnmod.lnmod_backward_varlen
    assert b(A, A, None, A, A, 3, 10, 64, 1e-6, None, A, A, A, A, A, None, 0, 0) == lnmod.LNMOD_EWORKSPACE
    assert b(A, A, None, A, None, 3, 10, 64, 1e-6, None, A, A, A, A, A, A, 1 << 40, 0) == lnmod.LNMOD_EINVAL


def test_workspace_query(lib):
    q = lnmod.lnmod_backward_workspace_bytes
    assert q(1, 75600, 5120, lnmod.LNMOD_PER_TOKEN) == 0
    assert q(-1, 10, 64, 0) == 0 and q(1, -1, 64, 0) == 0 and q(1, 10, 66, 0) == 0
    slot = 2 * 5120 * 4                       # one partial-sum slot: dshift and dscale rows in fp32
    n = q(1, 75600, 5120, 0)
    assert n % slot == 0 and n >= slot
    # the partial sums stay a small part of the backward's own traffic (6*D bytes per token)
    assert 2 * n <= 0.05 * 75600 * 6 * 5120
    m = q(24, 152880, 5120, 0)
    assert m % slot == 0 and m >= 24 * slot
    # 24 segments: the query covers the plan with the most slots (the backward that recomputes the
    # statistics runs two blocks per CU at this width, twice the slots of the plain backward)
    assert 2 * m <= 0.08 * 152880 * 6 * 5120
    # many short segments: at least one slot per segment, still bounded
    k = q(1000, 16000, 1536, 0)
    assert k >= 1000 * 2 * 1536 * 4
    assert q(1, 10, 5120, 0) <= n


def test_backward_static_validates_like_backward_and_refuses_what_does_not_fit(lib):
    E = lnmod

    def sb(dy=A, x=A, scale=A, B=2, S=4, D=64, eps=1e-6, mean=A, rstd=A, dx=A, dshift=A, dscale=A, dtype=0, mod=0):
        return lnmod.lnmod_backward_static(dy, x, None, scale, B, S, D, eps, None, mean, rstd, dx, dshift, dscale,
                                           dtype, mod)
    assert sb(dy=None) == E.LNMOD_EINVAL and sb(dx=None) == E.LNMOD_EINVAL and sb(dscale=None) == E.LNMOD_EINVAL
    assert sb(mean=None) == E.LNMOD_EINVAL and sb(eps=0.0) == E.LNMOD_EINVAL and sb(mod=2) == E.LNMOD_EINVAL
    assert sb(B=-1) == E.LNMOD_EINVAL and sb(B=1 << 40, S=1 << 40) == E.LNMOD_EINVAL
    assert sb(D=63) == E.LNMOD_EUNSUPPORTED and sb(D=8200) == E.LNMOD_EUNSUPPORTED
    assert sb(x=A + 4) == E.LNMOD_EALIGN and sb(dshift=A + 8) == E.LNMOD_EALIGN
    assert sb(B=0, S=0) == E.LNMOD_OK and sb(B=0, S=5) == E.LNMOD_OK
    # the headline problem needs 256 slots of 40 KB: it fits; 3000 samples at D = 8192 do not
    assert 256 * 2 * 5120 * 4 <= lnmod.LNMOD_STATIC_WORKSPACE_BYTES
    assert sb(B=3000, S=40, D=8192) == E.LNMOD_EWORKSPACE
    assert sb(B=3000, S=40, D=8192, mean=None, rstd=None) == E.LNMOD_EWORKSPACE
    header = open(HEADER).read()
    assert "#define LNMOD_STATIC_WORKSPACE_BYTES ((size_t)64 << 20)" in header


def gfwd(x=A, u=A, gate=A, shift=A, scale=A, cu=None, n=2, s=4, D=64, eps=1e-6, h=A, y=A, mean=A,
         rstd=A, dtype=0):
    return lnmod.lnmod_gated_forward(x, u, gate, shift, scale, cu, n, s, D, eps, None, h, y, mean,
                                     rstd, dtype)


def gbwd(dy=A, dh=A, h=A, u=A, gate=A, scale=A, cu=None, n=2, s=4, D=64, eps=1e-6, mean=A, rstd=A,
         dx=A, du=A, dgate=A, dshift=A, dscale=A, ws=A, ws_bytes=1 << 40, dtype=0):
    return lnmod.lnmod_gated_backward(dy, dh, h, u, gate, scale, cu, n, s, D, eps, None, mean, rstd,
                                      dx, du, dgate, dshift, dscale, ws, ws_bytes, dtype)


def test_gated_rejects_bad_arguments(lib):
    E = lnmod
    assert gfwd(u=None) == E.LNMOD_EINVAL and gfwd(gate=None) == E.LNMOD_EINVAL
    assert gfwd(h=None) == E.LNMOD_EINVAL and gfwd(mean=None) == E.LNMOD_EINVAL
    assert gfwd(eps=0.0) == E.LNMOD_EINVAL and gfwd(dtype=2) == E.LNMOD_EINVAL
    assert gfwd(n=-1) == E.LNMOD_EINVAL and gfwd(n=1 << 40, s=1 << 40) == E.LNMOD_EINVAL
    assert gfwd(D=63) == E.LNMOD_EUNSUPPORTED and gfwd(D=8200) == E.LNMOD_EUNSUPPORTED
    assert gfwd(D=68, dtype=0) == E.LNMOD_EUNSUPPORTED
    assert gfwd(u=A + 8) == E.LNMOD_EALIGN and gfwd(h=A + 2) == E.LNMOD_EALIGN
    assert gfwd(n=2, s=0) == E.LNMOD_OK and gfwd(n=0, s=0) == E.LNMOD_OK
    assert gfwd(cu=A, n=0, s=5) == E.LNMOD_EINVAL            # tokens that belong to no segment
    assert gbwd(dh=None) == E.LNMOD_EINVAL and gbwd(du=None) == E.LNMOD_EINVAL
    assert gbwd(dgate=None) == E.LNMOD_EINVAL and gbwd(eps=float("nan")) == E.LNMOD_EINVAL
    assert gbwd(D=12, dtype=0) == E.LNMOD_EUNSUPPORTED
    assert gbwd(dy=A + 4) == E.LNMOD_EALIGN and gbwd(du=A + 4) == E.LNMOD_EALIGN
    assert gbwd(ws=None) == E.LNMOD_EWORKSPACE and gbwd(ws_bytes=16) == E.LNMOD_EWORKSPACE
    assert gbwd(ws=A + 4) == E.LNMOD_EALIGN
    assert gbwd(n=0, s=0) == E.LNMOD_OK


def test_gated_workspace_query(lib):
    q = lnmod.lnmod_gated_backward_workspace_bytes
    assert q(-1, 10, 64) == 0 and q(1, -1, 64) == 0 and q(1, 10, 66) == 0
    slot = 3 * 5120 * 4                       # dshift, dscale and dgate rows in fp32
    n = q(1, 75600, 5120)
    assert n % slot == 0 and n >= slot
    assert 2 * n <= 0.05 * 75600 * 12 * 5120   # small beside the backward's own 12*D bytes per token
    m = q(24, 152880, 5120)
    assert m % slot == 0 and m >= 24 * slot


def test_qknorm_rejects_bad_arguments_and_sizes_workspace(lib):
    E = lnmod
    f = lambda q=A, k=A, wq=A, wk=A, N=10, D=64, eps=1e-6, qo=A, ko=A, rq=A, rk=A, dtype=0: \
        lnmod.lnmod_qknorm_forward(q, k, wq, wk, N, D, eps, None, qo, ko, rq, rk, dtype)
    assert f(k=None) == E.LNMOD_EINVAL and f(rk=None) == E.LNMOD_EINVAL and f(eps=-1.0) == E.LNMOD_EINVAL
    assert f(N=-1) == E.LNMOD_EINVAL and f(N=1 << 31) == E.LNMOD_EINVAL and f(dtype=5) == E.LNMOD_EINVAL
    assert f(D=12) == E.LNMOD_EUNSUPPORTED and f(D=8200) == E.LNMOD_EUNSUPPORTED
    assert f(wq=A + 8) == E.LNMOD_EALIGN and f(ko=A + 2) == E.LNMOD_EALIGN
    assert f(N=0) == E.LNMOD_OK
    b = lambda dqo=A, dko=A, q=A, k=A, wq=A, wk=A, N=10, D=64, eps=1e-6, rq=A, rk=A, dq=A, dk=A, dwq=A, \
        dwk=A, ws=A, wsb=1 << 40, dtype=0: lnmod.lnmod_qknorm_backward(
            dqo, dko, q, k, wq, wk, N, D, eps, None, rq, rk, dq, dk, dwq, dwk, ws, wsb, dtype)
    assert b(dko=None) == E.LNMOD_EINVAL and b(dwk=None) == E.LNMOD_EINVAL
    assert b(D=68) == E.LNMOD_EUNSUPPORTED and b(dq=A + 4) == E.LNMOD_EALIGN
    assert b(ws=None) == E.LNMOD_EWORKSPACE and b(wsb=8) == E.LNMOD_EWORKSPACE and b(ws=A + 4) == E.LNMOD_EALIGN
    wq = lnmod.lnmod_qknorm_backward_workspace_bytes
    assert wq(-1, 64) == 0 and wq(10, 66) == 0
    n = wq(75600, 5120)
    assert n % (2 * 5120 * 4) == 0 and 0 < 2 * n <= 0.05 * 2 * 75600 * 6 * 5120
    assert wq(1, 5120) == 2 * 5120 * 4


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(lnmod, "_lib", None)
    monkeypatch.setattr(lnmod, "LIBRARY", os.path.join(tmp_path, "nope.so"))
    with pytest.raises(RuntimeError, match="not built"):
        lnmod.lnmod_forward(A, A, A, 1, 1, 64, 1e-6, None, A, A, A, 0, 0)


# ---- the measurement library (include/lnmod_tools.h)

TOOLS_HEADER = os.path.join(ROOT, "include", "lnmod_tools.h")
T = lnmod_tools


@pytest.fixture(scope="module")
def tools(lib):
    return lnmod_tools.library()


def test_tools_header_symbols_are_exported(tools):
    text = re.sub(r"/\*.*?\*/", "", open(TOOLS_HEADER).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(lnmod_[a-z_0-9]+)\s*\(", text)))
    assert set(names) == set(lnmod_tools.EXPORTS)
    assert set(dynamic_symbols(lnmod_tools.LIBRARY)) == set(names)
    for n in names:
        assert hasattr(tools, n), n
        assert callable(getattr(lnmod_tools, n)), n


def test_copy_probe_and_comparators_reject_bad_arguments(tools):
    E = lnmod
    assert T.lnmod_copy(None, A, 64, None) == E.LNMOD_EINVAL
    assert T.lnmod_copy(A, A, 60, None) == E.LNMOD_EINVAL
    assert T.lnmod_copy(A + 4, A, 64, None) == E.LNMOD_EALIGN
    assert T.lnmod_copy(A, A, 0, None) == E.LNMOD_OK
    probe = T.lnmod_stream_probe
    assert probe([A, A, A, A, A], [A], 4096, None) == E.LNMOD_EINVAL           # no such mixture
    assert probe([A, A, A, A], [A], 4096, None) == E.LNMOD_EINVAL
    assert probe([A, None], [A], 4096, None) == E.LNMOD_EINVAL
    assert probe([A], [None], 4096, None, writes=0) == E.LNMOD_EINVAL
    assert probe([A], [A], 512, None, writes=0) == E.LNMOD_EINVAL             # out[0] must hold 1 KB
    assert probe([A, A], [A], 4100, None) == E.LNMOD_EINVAL
    assert probe([A, A], [A + 8], 4096, None) == E.LNMOD_EALIGN
    assert probe([A, A], [A], 4096, None, launch=(256, 9, 4)) == E.LNMOD_EINVAL
    assert probe([A, A], [A], 4096, None, launch=(256, 4, 3)) == E.LNMOD_EINVAL
    assert probe([A, A], [A], 4096, None, launch=(0, 4, 4)) == E.LNMOD_EINVAL
    assert probe([], [A], 0, None) == E.LNMOD_OK
    for nr, nw in T.PROBE_MIXTURES:
        assert probe([A] * nr, [A] * max(nw, 1), 0, None, writes=nw) == E.LNMOD_OK
    u = T.lnmod_unfused_forward
    assert u(A, A, A, 2, 4, 64, 1e-6, None, None, A, A, A, 0) == E.LNMOD_EINVAL
    assert u(A, A, A, 2, 4, 63, 1e-6, None, A, A, A, A, 0) == E.LNMOD_EUNSUPPORTED
    g = T.lnmod_gate_residual
    assert g(A, None, A, 2, 4, 64, None, A, 0) == E.LNMOD_EINVAL
    assert g(A, A, A, 2, 4, 60, None, A, 0) == E.LNMOD_EUNSUPPORTED
    assert g(A, A, A + 1, 2, 4, 64, None, A, 0) == E.LNMOD_EALIGN


def sfwd(shape, x=A, shift=A, scale=A, cu=None, B=2, S=4, D=64, eps=1e-6, y=A, mean=A, rstd=A, dtype=0, mod=0):
    return T.lnmod_forward_shaped(shape, x, shift, scale, cu, B, S, D, eps, None, y, mean, rstd, dtype, mod)


def sbwd(shape, dy=A, x=A, scale=A, cu=None, B=2, S=4, D=64, eps=1e-6, mean=A, rstd=A, dx=A, dshift=A, dscale=A,
         ws=A, ws_bytes=1 << 40, dtype=0, mod=0):
    return T.lnmod_backward_shaped(shape, dy, x, scale, cu, B, S, D, eps, None, mean, rstd, dx, dshift, dscale,
                                   ws, ws_bytes, dtype, mod)


def test_shaped_calls_validate_the_shape_and_then_like_the_operator_calls(tools):
    E = lnmod
    for bad in ((17, 1, 1, 1), (-1, 1, 1, 1), (0, 1, 1, 1), (1, 0, 1, 1), (1, 7, 1, 1), (1, 1, 0, 1), (1, 1, 3, 1),
                (1, 1, 1, 0), (1, 1, 1, 17), (1, 1, 1, 4, -1, 0), (1, 1, 1, 4, 257, 0), (1, 1, 1, 4, 8, 2), (1, 1, 1, 4, 0, 0, 3), (1, 1, 1, 4, 0, 0, -1)):
        assert sfwd(bad) == E.LNMOD_EINVAL, bad
        assert sbwd(bad) == E.LNMOD_EINVAL, bad
        assert T.lnmod_backward_workspace_bytes_shaped(bad, 1, 100, 64, 0) == 0
        assert T.lnmod_describe_launch(False, bad, 1, 100, False, 64, 0, 0) == ""
    ok = (1, 1, 1, 4)
    assert sfwd(ok, x=None) == E.LNMOD_EINVAL and sfwd(ok, D=63) == E.LNMOD_EUNSUPPORTED
    assert sfwd(ok, y=A + 4) == E.LNMOD_EALIGN and sfwd(ok, S=0) == E.LNMOD_OK
    assert sfwd(ok, cu=A, mod=1) == E.LNMOD_EINVAL                  # packed batches are per segment
    assert sbwd(ok, dx=None) == E.LNMOD_EINVAL and sbwd(ok, ws=None) == E.LNMOD_EWORKSPACE
    assert sbwd(ok, ws_bytes=16) == E.LNMOD_EWORKSPACE and sbwd(None, ws_bytes=16) == E.LNMOD_EWORKSPACE
    assert T.lnmod_backward_workspace_bytes_shaped(None, 1, 75600, 5120, 0) == \
        lnmod.lnmod_backward_workspace_bytes(1, 75600, 5120, 0)
    # the workspace follows the shape: twice the blocks per CU, twice the slots
    one = T.lnmod_backward_workspace_bytes_shaped((4, 3, 2, 1), 1, 75600, 5120, 0)
    two = T.lnmod_backward_workspace_bytes_shaped((4, 3, 2, 2), 1, 75600, 5120, 0)
    assert one == 256 * 2 * 5120 * 4 and two == 2 * one


def test_a_shape_that_does_not_cover_the_row_fails_before_any_launch(tools):
    small = (1, 1, 1, 4)                                           # 64 chunks: 512 bf16 features
    assert sfwd(small, D=520, B=1, S=8) == 5
    assert sfwd(small, D=520, B=1, S=8, mod=1) == 5
    assert sbwd(small, D=520, B=1, S=8) == 5
    assert sbwd(small, D=520, B=1, S=8, mean=None, rstd=None) == 5
    assert sbwd(small, D=520, B=1, S=8, mod=1, ws=None, ws_bytes=0) == 5


def test_table_shape_matches_the_documented_entries(tools):
    # bf16 D = 5120 (the headline width) and D = 1536, as the design notes list them
    get = T.lnmod_table_shape
    assert get(T.LNMOD_FAMILY_FORWARD, 5120, 0) == (0, (5, 2, 2, 1))
    assert get(T.LNMOD_FAMILY_BACKWARD, 5120, 0) == (0, (4, 3, 2, 1))
    assert get(T.LNMOD_FAMILY_BACKWARD_RECOMPUTE, 5120, 0) == (0, (4, 3, 1, 2))
    assert get(T.LNMOD_FAMILY_FORWARD, 1536, 0) == (0, (1, 3, 2, 4))
    assert get(T.LNMOD_FAMILY_FORWARD, 1536, 0, tokens=200000) == (0, (1, 3, 2, 3))
    assert get(T.LNMOD_FAMILY_GATED_FORWARD, 5120, 0) == (0, (4, 3, 1, 1))
    assert get(T.LNMOD_FAMILY_GATED_BACKWARD, 5120, 0) == (0, (8, 2, 1, 1))
    assert get(T.LNMOD_FAMILIES, 5120, 0)[0] == 1 and get(0, 5120, 2)[0] == 1
    assert get(0, 5124, 0)[0] == 2 and get(0, 8200, 1)[0] == 2
    # every family's entry covers its row, at every supported width and both types
    for fam in range(T.LNMOD_FAMILIES):
        for dtype, vec in ((0, 8), (1, 4)):
            for D in range(8, 8193, 8):
                st, (K, VPL, R, per_cu) = get(fam, D, dtype)
                assert st == 0
                assert K * VPL * 64 >= D // vec and R in (1, 2) and per_cu >= 1, (fam, dtype, D)


def test_describe_launch_names_the_kernels_of_the_headline_workload(tools):
    d = T.lnmod_describe_launch
    assert d(False, None, 1, 75600, False, 5120, 0, 0) == \
        "fwd_split_kernel<bf16_io, 2, 5, 2, true, 0, true> grid=256 block=320 clusters=1"
    assert d(True, None, 1, 75600, False, 5120, 0, 0) == \
        ("bwd_seg_kernel<bf16_io, 3, 4, 2, false, false, true, false> grid=256 block=256 clusters=1"
         " + bwd_reduce_kernel<4, 4> grid=160 block=1024 slots=256")
    assert "true, true>" in d(True, None, 1, 75600, False, 5120, 0, 0, recompute=True)
    assert d(True, None, 2, 32760, False, 5120, 0, 1).startswith("bwd_seg_kernel<bf16_io, 2, 5, 1, true, true, true, false>")
    assert "reduce" not in d(True, None, 2, 32760, False, 5120, 0, 1)
    assert d(False, (4, 3, 1, 2), 1, 75600, False, 5120, 0, 0).startswith("fwd_split_kernel<bf16_io, 3, 4, 1, false, 0, true> grid=512")
    assert d(False, (5, 2, 2, 1, 8, 1), 1, 75600, False, 5120, 0, 0).endswith("grid=256 block=320 clusters=8")
    assert d(True, (4, 3, 2, 1, 8, 1), 1, 75600, False, 5120, 0, 0).endswith("slots=256")
    assert d(False, None, 1, 0, False, 5120, 0, 0) == "" and d(False, None, 1, 10, False, 5121, 0, 0) == ""


def test_describe_launch_shows_which_forward_loop_a_batch_of_several_segments_gets(tools):
    d = T.lnmod_describe_launch
    # bf16 rows shared by three or more waves, and D = 1536: one loop over all rows (mode 4), the fewest
    # clusters (a power of two, 2 ... 32) that leave a block at most 32 segments
    assert d(False, None, 24, 152880, True, 5120, 0, 0) == \
        "fwd_split_kernel<bf16_io, 2, 5, 2, true, 4, true> grid=256 block=320 clusters=2"
    assert d(False, None, 96, 149760, True, 5120, 0, 0).endswith("4, true> grid=256 block=320 clusters=4")
    assert d(False, None, 480, 149760, True, 5120, 0, 0).endswith("clusters=16")
    assert d(False, None, 5000, 150000, True, 5120, 0, 0).endswith("clusters=32")
    assert d(False, None, 4, 32760, False, 5120, 0, 0).endswith("4, true> grid=256 block=320 clusters=2")
    assert d(False, None, 24, 152880, True, 1536, 0, 0) == \
        "fwd_split_kernel<bf16_io, 3, 1, 2, true, 4, true> grid=1024 block=64 clusters=2"
    # one segment, narrow bf16 rows and fp32: one loop per segment (mode 0)
    assert ", 0, true>" in d(False, None, 1, 152880, True, 5120, 0, 0)
    assert ", 0, true>" in d(False, None, 24, 152880, True, 2048, 0, 0)
    assert ", 0, true>" in d(False, None, 24, 152880, True, 5120, 1, 0)
    # shape[6] overrides the choice either way
    tab = (5, 2, 2, 1)
    assert ", 0, true>" in d(False, tab + (0, 0, 2), 24, 152880, True, 5120, 0, 0)
    assert ", 4, true>" in d(False, (2, 2, 1, 4, 0, 0, 1), 24, 152880, True, 2048, 0, 0)
    assert d(False, tab + (8, 1, 1), 24, 152880, True, 5120, 0, 0).endswith("4, true> grid=256 block=320 clusters=8")
