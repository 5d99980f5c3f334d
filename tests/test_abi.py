"""Host-side checks of the C ABI (no GPU needed): the library loads, exports every symbol that
include/llla.h declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2510_01450_amd as llla
from paper_2510_01450_amd.binding import _Strides

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # never dereferenced: every call below fails validation first


def _declared_symbols(header="llla.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(llla_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared_symbols()
    assert {"llla_forward", "llla_decode", "llla_forward_workspace_bytes", "llla_decode_workspace_bytes",
            "llla_status_string", "llla_version"} <= set(names)
    llla.lib()                                  # builds the library if the tree has none
    L = ctypes.CDLL(llla.lib_path())
    for name in names:
        assert hasattr(L, name), name


def test_measurement_aids_live_in_a_library_of_their_own():
    """The production library exports the method only; the profiling hooks and the MFMA probe exist in the
    measurement build, which also exports everything llla.h declares."""
    aids = _declared_symbols("llla_measure.h")
    assert set(aids) == {"llla_profile_enable", "llla_profile_last", "llla_probe_mfma_f16", "llla_probe_copy"}
    assert not set(aids) & set(_declared_symbols())
    llla.lib()
    P = ctypes.CDLL(llla.lib_path())
    for name in aids:
        assert not hasattr(P, name), name + " leaked into the production library"
    llla.measure_lib()
    M = ctypes.CDLL(llla.measure_lib_path())
    for name in aids + _declared_symbols():
        assert hasattr(M, name), name


def test_a_stale_library_is_detected():
    """The binding compares a hash of the sources with the stamp the build left beside the library."""
    from paper_2510_01450_amd import build
    llla.lib()
    assert build.is_current(build.LIB)
    stamp = build.stamp_path(build.LIB)
    good = open(stamp).read()
    try:
        open(stamp, "w").write("0" * 64 + "\n")
        assert not build.is_current(build.LIB)
    finally:
        open(stamp, "w").write(good)
    assert build.is_current(build.LIB)


def _fwd(Q=FAKE, K=FAKE, V=FAKE, O=FAKE, sq=None, B=1, H=1, n=64, d=64, din=0, dout=0, causal=1, lam=1e-2,
         scale=0.125, path=0, ws=0, wsb=0):
    s = _Strides(H * n * d, n * d, d) if sq is None else sq
    return llla.lib().llla_forward_path(Q, K, V, O, s, s, s, s, B, H, n, d, din, dout, causal, lam, scale, path,
                                        ws, wsb, 0)


def _dec(q=FAKE, K=FAKE, V=FAKE, o=FAKE, B=1, H=1, L=64, d=64, din=0, dout=0, lam=1e-2, scale=0.125, path=0,
         sk=None):
    s = _Strides(H * L * d, L * d, d) if sk is None else sk
    return llla.lib().llla_decode_path(q, K, V, o, s, s, 0, B, H, L, d, din, dout, lam, scale, path, 0, 0, 0)


@pytest.mark.parametrize("kw,code", [
    (dict(Q=0), 1), (dict(O=0), 1),
    (dict(n=0), 2), (dict(B=-1), 2), (dict(sq=_Strides(64 * 64, 64 * 64, 32)), 2), (dict(B=70000), 2),
    (dict(din=7), 3), (dict(dout=-1), 3),
    (dict(lam=0.0), 4), (dict(lam=-1.0), 4), (dict(lam=float("nan")), 4), (dict(lam=float("inf")), 4),
    (dict(scale=float("inf")), 4), (dict(path=9), 4),
    (dict(Q=FAKE + 4), 5), (dict(sq=_Strides(64 * 64, 64 * 64, 66)), 5),
    (dict(d=48), 7), (dict(d=256), 7),
])
def test_forward_rejects_bad_arguments(kw, code):
    assert _fwd(**kw) == code


def test_forward_ex_validation():
    """The scalar ridge is ignored (not validated) when a per-row ridge is given; misaligned extras are refused.
    FAKE pointers are never dereferenced: each call fails a later check (no workspace on the MFMA path is not
    reached with fp32 inputs, so the calls below stop at the checks named)."""
    s = _Strides(64 * 64, 64 * 64, 64)
    ex = llla.lib().llla_forward_ex
    # bad scalar lambda, no per-row ridge -> PARAM
    assert ex(FAKE, FAKE, FAKE, FAKE, s, s, s, s, 1, 1, 64, 64, 0, 0, 1, 0.0, None, 0.125, None, None, 0, 0, 0, 0) == 4
    # same scalar with a per-row ridge: passes that check and trips on the misaligned rho pointer instead
    assert ex(FAKE, FAKE, FAKE, FAKE, s, s, s, s, 1, 1, 64, 64, 0, 0, 1, 0.0, FAKE, 0.125, FAKE + 2, None, 0, 0, 0,
              0) == 5
    assert ex(FAKE, FAKE, FAKE, FAKE, s, s, s, s, 1, 1, 64, 64, 0, 0, 1, 0.0, FAKE + 1, 0.125, None, None, 0, 0, 0,
              0) == 5
    # bf16 + MFMA path without workspace -> WORKSPACE (reached only after the ridge checks passed)
    assert ex(FAKE, FAKE, FAKE, FAKE, s, s, s, s, 1, 1, 64, 64, 1, 0, 1, 0.0, FAKE, 0.125, None, None, 2, 0, 0, 0) == 6


def test_forward_cg_validation():
    s = _Strides(64 * 64, 64 * 64, 64)
    cg = llla.lib().llla_forward_cg

    def call(din=1, d=64, T=4, eps=0.0, lam=1e-2, rho=None, ws=0, wsb=0):
        return cg(FAKE, FAKE, FAKE, FAKE, s, s, s, s, 1, 1, 64, d, din, 0, lam, 0.125, T, eps, rho, None, None, ws, wsb, 0)

    assert call(T=-1) == 4 and call(T=5000) == 4 and call(eps=-1.0) == 4 and call(eps=float("nan")) == 4
    assert call(lam=0.0) == 4
    assert call(rho=FAKE + 2) == 5
    assert call(din=0) == 7            # fp32 inputs have no approximate mode
    assert call(d=32) == 6             # served on zero-padded copies: the workspace is what is missing
    assert call(d=32, din=0) == 7
    assert call() == 6                 # everything valid but no workspace
    assert llla.lib().llla_forward_cg_workspace_bytes(1, 1, 64, 64, 1) > llla.lib().llla_forward_workspace_bytes(1, 1, 64, 64, 1)
    assert llla.lib().llla_forward_cg_workspace_bytes(1, 1, 64, 64, 0) == 0


@pytest.mark.parametrize("kw,code", [
    (dict(q=0), 1), (dict(L=0), 2), (dict(din=5), 3), (dict(lam=0.0), 4), (dict(K=FAKE + 2), 5), (dict(d=20), 7),
    (dict(sk=_Strides(64 * 64, 64 * 64, 8)), 2),
])
def test_decode_rejects_bad_arguments(kw, code):
    assert _dec(**kw) == code


def test_status_strings_and_version():
    seen = {llla.status_string(c) for c in range(9)}
    assert len(seen) == 9 and "ok" in seen
    assert re.match(r"^\d+\.\d+\.\d+$", llla.version())


def test_workspace_queries_are_pure():
    import torch
    assert llla.forward_workspace_bytes(0, 1, 1, 64, torch.float32) == 0
    a = llla.forward_workspace_bytes(4, 16, 4096, 64, torch.bfloat16)
    assert a == llla.forward_workspace_bytes(4, 16, 4096, 64, torch.bfloat16)
    # Theta(B*H*n*d): far below one d x d matrix per query
    assert a < 4 * 16 * 4096 * 64 * 64


def test_product_has_no_cpu_fallback():
    import torch
    x = torch.zeros(1, 1, 8, 16)
    with pytest.raises(ValueError):
        llla.llla_forward(x, x, x, 1e-2, 0.25)


def _bwd(Q=FAKE, K=FAKE, V=FAKE, dO=FAKE, dQ=FAKE, dK=FAKE, dV=FAKE, dlam=None, s=None, B=1, H=1, n=64, d=64, din=0,
         lam=1e-2, lam_rows=None, scale=0.125, path=0, ws=0, wsb=0):
    s = _Strides(H * n * d, n * d, d) if s is None else s
    return llla.lib().llla_backward(Q, K, V, dO, s, s, s, s, dQ, dK, dV, dlam, B, H, n, d, din, lam, lam_rows, scale,
                                    path, ws, wsb, 0)


@pytest.mark.parametrize("kw,code", [
    (dict(dO=0), 1), (dict(dK=0), 1),
    (dict(n=0), 2), (dict(s=_Strides(64 * 64, 64 * 64, 32)), 2),
    (dict(din=5), 3),
    (dict(lam=0.0), 4), (dict(scale=float("nan")), 4), (dict(path=5), 4),
    (dict(path=2), 7), (dict(path=2, din=0, d=32), 7), (dict(path=2, din=1, d=32), 6),
    (dict(dQ=FAKE + 8), 5), (dict(dlam=FAKE + 2), 5), (dict(lam_rows=FAKE + 1), 5),
    (dict(), 6), (dict(ws=FAKE + 16, wsb=1 << 30), 6), (dict(ws=FAKE, wsb=16), 6),
    (dict(d=24), 7),
])
def test_backward_rejects_bad_arguments(kw, code):
    """Every call fails a host-side check before anything is launched (the last valid-looking one for lack of a
    workspace)."""
    assert _bwd(**kw) == code


def test_backward_workspace_size():
    assert llla.backward_workspace_bytes(2, 3, 100, 64, __import__("torch").bfloat16) >= 2 * 3 * 100 * (2 * 64 + 8) * 4
    assert llla.lib().llla_backward_workspace_bytes(1, 1, 0, 64, 0) == 0
    # a bad scalar ridge is ignored when a ridge per row is given: the call gets as far as the workspace check
    assert _bwd(lam=0.0, lam_rows=FAKE) == 6


def test_small_head_dimensions_dispatch_on_the_host():
    """d = 16 / 32: the workspace holds the zero-padded copies and the d = 64 workspace behind them; a forced
    matrix-core call is served (it fails for lack of a workspace, not as unsupported), for both dtypes."""
    L = llla.lib()
    for din in (0, 1):
        inner = L.llla_forward_workspace_bytes(2, 3, 500, 64, din)
        esz = 4 if din == 0 else 2
        for d in (16, 32):
            need = L.llla_forward_workspace_bytes(2, 3, 500, d, din)
            rows = 2 * 3 * 500
            assert need >= inner + rows * 64 * (3 * esz + 8)          # Q, K, V copies, O and rho rows
            assert _fwd(d=d, din=din, dout=din, path=2) == 6             # served: the workspace is what is missing
    # LLLA_PATH_AUTO, bf16, 64 rows, d = 32: the padded call (its workspace is checked, and missing)
    assert _fwd(d=32, din=1, n=64, path=0) == 6
    assert _bwd(d=32, din=1, n=64, path=0) == 6                          # backward: padded from 64 rows on at d = 32
    assert _bwd(d=16, din=1, n=64, path=2) == 6
    assert _bwd(d=16, din=0, n=64, path=2) == 7                          # no fp32 matrix-core backward
