"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching any device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "lnmod.h")

from paper_2605_17923_amd import lnmod  # noqa: E402


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


def test_header_symbols_are_exported(lib):
    names = declared_functions()
    assert set(names) == set(lnmod.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


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


def test_copy_and_unfused_reject_bad_arguments(lib):
    assert lnmod.lnmod_copy(None, A, 64, None) == lnmod.LNMOD_EINVAL
    assert lnmod.lnmod_copy(A, A, 60, None) == lnmod.LNMOD_EINVAL
    assert lnmod.lnmod_copy(A + 4, A, 64, None) == lnmod.LNMOD_EALIGN
    assert lnmod.lnmod_copy(A, A, 0, None) == lnmod.LNMOD_OK
    probe = lnmod.lnmod_stream_probe
    assert probe(A, A, A, 4096, 0, None) == lnmod.LNMOD_EINVAL                 # no such mode
    assert probe(A, None, A, 4096, lnmod.LNMOD_PROBE_ADD, None) == lnmod.LNMOD_EINVAL
    assert probe(None, None, A, 4096, lnmod.LNMOD_PROBE_READ, None) == lnmod.LNMOD_EINVAL
    assert probe(A, None, A, 512, lnmod.LNMOD_PROBE_READ, None) == lnmod.LNMOD_EINVAL
    assert probe(None, None, None, 4096, lnmod.LNMOD_PROBE_WRITE, None) == lnmod.LNMOD_EINVAL
    assert probe(A, A, A, 4100, lnmod.LNMOD_PROBE_ADD, None) == lnmod.LNMOD_EINVAL
    assert probe(A, A, A + 8, 4096, lnmod.LNMOD_PROBE_ADD, None) == lnmod.LNMOD_EALIGN
    assert probe(None, None, None, 0, lnmod.LNMOD_PROBE_WRITE, None) == lnmod.LNMOD_OK
    u = lnmod.lnmod_unfused_forward
    assert u(A, A, A, 2, 4, 64, 1e-6, None, None, A, A, A, 0) == lnmod.LNMOD_EINVAL
    assert u(A, A, A, 2, 4, 63, 1e-6, None, A, A, A, A, 0) == lnmod.LNMOD_EUNSUPPORTED


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
    g = lnmod.lnmod_gate_residual
    assert g(A, None, A, 2, 4, 64, None, A, 0) == E.LNMOD_EINVAL
    assert g(A, A, A, 2, 4, 60, None, A, 0) == E.LNMOD_EUNSUPPORTED
    assert g(A, A, A + 1, 2, 4, 64, None, A, 0) == E.LNMOD_EALIGN


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


# ---- tuning interface (include/lnmod_tuning.h)

TUNING_HEADER = os.path.join(ROOT, "include", "lnmod_tuning.h")


def test_tuning_header_symbols_are_exported(lib):
    text = re.sub(r"/\*.*?\*/", "", open(TUNING_HEADER).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(lnmod_[a-z_0-9]+)\s*\(", text)))
    assert set(names) == set(lnmod.TUNING_EXPORTS)
    for n in names:
        assert hasattr(lib, n), n
        assert callable(getattr(lnmod, n)), n


def test_tuning_set_shape_validation(lib):
    ok = lnmod.lnmod_tuning_set_shape
    try:
        assert ok(-1, 1, 1, 1, 1) == 1 and ok(lnmod.LNMOD_TUNE_FAMILIES, 1, 1, 1, 1) == 1
        for bad in ((17, 1, 1, 1), (-1, 1, 1, 1), (1, 0, 1, 1), (1, 7, 1, 1), (1, 1, 0, 1), (1, 1, 3, 1),
                    (1, 1, 1, 0), (1, 1, 1, 17)):
            assert ok(lnmod.LNMOD_TUNE_FORWARD, *bad) == 1, bad
        assert ok(lnmod.LNMOD_TUNE_FORWARD, 4, 3, 1, 2) == 0
    finally:
        for fam in range(lnmod.LNMOD_TUNE_FAMILIES):
            assert ok(fam, 0, 0, 0, 0) == 0


def test_tuning_table_shape_matches_the_documented_entries(lib):
    # bf16 D = 5120 (the headline width) and D = 1536, as the design notes list them
    get = lnmod.lnmod_tuning_table_shape
    assert get(lnmod.LNMOD_TUNE_FORWARD, 5120, 0) == (0, (5, 2, 2, 1))
    assert get(lnmod.LNMOD_TUNE_BACKWARD, 5120, 0) == (0, (4, 3, 2, 1))
    assert get(lnmod.LNMOD_TUNE_BACKWARD_RECOMPUTE, 5120, 0) == (0, (4, 3, 1, 2))
    assert get(lnmod.LNMOD_TUNE_FORWARD, 1536, 0) == (0, (1, 3, 2, 4))
    assert get(lnmod.LNMOD_TUNE_GATED_FORWARD, 5120, 0) == (0, (4, 3, 1, 1))
    assert get(lnmod.LNMOD_TUNE_GATED_BACKWARD, 5120, 0) == (0, (8, 2, 1, 1))
    assert get(lnmod.LNMOD_TUNE_FAMILIES, 5120, 0)[0] == 1 and get(0, 5120, 2)[0] == 1
    assert get(0, 5124, 0)[0] == 2 and get(0, 8200, 1)[0] == 2
    # every family's entry covers its row, at every supported width and both types
    for fam in range(lnmod.LNMOD_TUNE_FAMILIES):
        for dtype, vec in ((0, 8), (1, 4)):
            for D in range(8, 8193, 8):
                st, (K, VPL, R, per_cu) = get(fam, D, dtype)
                assert st == 0
                assert K * VPL * 64 >= D // vec and R in (1, 2) and per_cu >= 1, (fam, dtype, D)


def test_override_that_does_not_cover_the_row_fails_before_any_launch(lib):
    try:
        for fam in range(lnmod.LNMOD_TUNE_FAMILIES):
            assert lnmod.lnmod_tuning_set_shape(fam, 1, 1, 1, 4) == 0      # 64 chunks: 512 bf16 features
        assert fwd(D=520, B=1, S=8) == 5
        assert fwd(D=520, B=1, S=8, mod=1) == 5
        assert bwd(D=520, B=1, S=8) == 5
        assert bwd(D=520, B=1, S=8, mean=None, rstd=None) == 5
        assert bwd(D=520, B=1, S=8, mod=1, ws=None, ws_bytes=0) == 5
    finally:
        for fam in range(lnmod.LNMOD_TUNE_FAMILIES):
            lnmod.lnmod_tuning_set_shape(fam, 0, 0, 0, 0)
