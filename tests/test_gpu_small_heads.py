"""Head dimensions 16 and 32 on the matrix-core forward (the d = 64 kernels on zero-padded copies): element by element
against the fp64 oracle, through the C ABI, forced with path='mfma', and where 'auto' chooses them.  The gate is
the one of the other parity tests (tests/parity.py) with the head dimension the CALLER passed, d = 16 or 32: rows
below 4d, not below 4 * 64, get the wider bound."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2510_01450_amd as llla
import workloads
from parity import check

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(name, B, H, n, d, dtype, values=None, index=0):
    base = workloads.C2 if dtype == "f32" else workloads.C3
    values = ("l2" if dtype == "f32" else "normal") if values is None else values
    return base.with_shape(name=name, B=B, H=H, n=n, d=d, dtype=dtype, values=values, index=index,
                           scale=1 / math.sqrt(d), tol=1e-4 if dtype == "f32" else 2e-2)


@pytest.mark.parametrize("n,d,dtype", [
    (1, 16, "bf16"), (77, 16, "bf16"), (131, 32, "bf16"), (333, 16, "bf16"), (700, 32, "bf16"),
    (2, 32, "f32"), (77, 16, "f32"), (130, 32, "f32"), (333, 32, "f32"), (600, 16, "f32"),
])
def test_padded_forward_all_outputs(n, d, dtype):
    """Ragged sizes on both sides of the 128 rows that the d = 64 kernels serve in their fp32-accurate variant."""
    w = _case("pad", 2, 3, n, d, dtype, index=400 + d + n)
    Q, K, V = workloads.make_inputs(w)
    ref = oracle.forward(Q, K, V, w.lam, w.scale)
    O = llla.llla_forward(Q.to(DEV), K.to(DEV), V.to(DEV), w.lam, w.scale, path="mfma")
    torch.cuda.synchronize()
    print(check(O.cpu().numpy(), ref, np.arange(n), d, w.tol, "padded n=%d d=%d %s" % (n, d, dtype)))


@pytest.mark.parametrize("n,d,dtype,padded", [(1100, 16, "bf16", True), (300, 16, "bf16", True), (20, 16, "bf16", False),
                                              (40, 32, "bf16", True), (1100, 16, "f32", False), (1100, 32, "f32", True),
                                              (600, 32, "f32", False)])
def test_what_auto_takes(n, d, dtype, padded):
    """LLLA_PATH_AUTO: bf16 with d = 16 / 32 from 32 rows on, and fp32 with d = 32 from 1024 rows on, gives the bits of the
    forced matrix-core call; the other calls those of the vector kernels.  Inside the gate either way."""
    w = _case("padauto", 1, 2, n, d, dtype, index=430 + d)
    Q, K, V = [t.to(DEV) for t in workloads.make_inputs(w)]
    a = llla.llla_forward(Q, K, V, w.lam, w.scale)
    m = llla.llla_forward(Q, K, V, w.lam, w.scale, path="mfma" if padded else "valu")
    torch.cuda.synchronize()
    assert torch.equal(a, m)
    ref = oracle.forward(Q.cpu(), K.cpu(), V.cpu(), w.lam, w.scale)
    print(check(a.cpu().numpy(), ref, np.arange(w.n), d, w.tol, "auto n=%d d=%d %s" % (n, d, dtype)))


@pytest.mark.parametrize("d", [16, 32])
def test_padded_forward_unnormalised_f32(d):
    """fp32 inputs ~ N(0,1), not normalised (rows with fewer keys than features cancel by ||z||^2 / lambda)."""
    n = 260
    w = _case("padunnorm", 2, 2, n, d, "f32", values="normal", index=440 + d)
    Q, K, V = workloads.make_inputs(w)
    ref = oracle.forward(Q, K, V, w.lam, w.scale)
    O = llla.llla_forward(Q.to(DEV), K.to(DEV), V.to(DEV), w.lam, w.scale, path="mfma")
    torch.cuda.synchronize()
    print(check(O.cpu().numpy(), ref, np.arange(n), d, w.tol, "padded unnormalised d=%d" % d))


@pytest.mark.parametrize("d,dtype", [(16, "bf16"), (32, "f32")])
def test_padded_forward_statistics_ridge_per_row_strides_and_bf16_output(d, dtype):
    """rho and delta come back un-padded, a ridge per row passes through, inputs in [B, n, H, d] memory, bf16 output."""
    n = 300
    w = _case("padex", 2, 2, n, d, dtype, index=450 + d)
    Q, K, V = workloads.make_inputs(w)
    g = torch.Generator().manual_seed(451 + d)
    lam = (10.0 ** (torch.rand(2, 2, n, generator=g) * 1.5 - 2.0)).float()
    refO, refR, refD = oracle.forward_ex(Q, K, V, lam.numpy(), w.scale)
    dev = [t.to(DEV).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (Q, K, V)]
    assert not dev[0].is_contiguous()
    O, R, Dl = llla.llla_forward(dev[0], dev[1], dev[2], lam.to(DEV), w.scale, path="mfma", return_stats=True)
    torch.cuda.synchronize()
    rows = np.arange(n)
    print(check(O.cpu().numpy(), refO, rows, d, w.tol, "padded ex"))
    print(check(R.cpu().numpy(), refR, rows, d, w.tol, "padded ex rho"))
    print(check(Dl.cpu().numpy()[..., None], refD[..., None], rows, d, w.tol, "padded ex delta"))
    out = torch.full((2, n, 2, d), 7.0, dtype=torch.bfloat16, device=DEV).permute(0, 2, 1, 3)
    llla.llla_forward(dev[0], dev[1], dev[2], lam.to(DEV), w.scale, path="mfma", out=out)
    torch.cuda.synchronize()
    print(check(out.float().cpu().numpy(), refO, rows, d, max(w.tol, 2e-2), "padded ex bf16 out, strided"))


@pytest.mark.parametrize("n,d,dtype", [(150, 16, "bf16"), (600, 32, "bf16"), (150, 32, "f32"), (600, 16, "f32")])
def test_padded_forward_non_causal(n, d, dtype):
    w = _case("padnc", 1, 2, n, d, dtype, index=460 + d + n)
    Q, K, V = workloads.make_inputs(w)
    ref = oracle.forward(Q, K, V, w.lam, w.scale, causal=False)
    O = llla.llla_forward(Q.to(DEV), K.to(DEV), V.to(DEV), w.lam, w.scale, causal=False, path="mfma")
    torch.cuda.synchronize()
    print(check(O.cpu().numpy(), ref, np.full(n, n - 1), d, w.tol, "padded noncausal n=%d d=%d %s" % (n, d, dtype)))


# ---- backward (bf16): the d = 64 matrix-core backward on the same padded copies ------------------------------------

def _upstream(w, seed):
    g = torch.Generator(device="cpu").manual_seed(workloads.SEED0 + 9000 + seed)
    return torch.randn((w.B, w.H, w.n, w.d), generator=g, dtype=torch.float32).to(workloads.torch_dtype(w))


@pytest.mark.parametrize("n,d,ridge_per_row", [(1, 16, False), (77, 16, False), (131, 32, False), (400, 32, True), (300, 16, True)])
def test_padded_backward_all_gradients(n, d, ridge_per_row):
    """dQ, dK, dV and dlambda against the backward oracle (the gate and its tolerance are those of
    tests/test_gpu_backward.py), inputs in [B, n, H, d] memory."""
    from oracle import backward as ob
    from parity import check_grad
    w = _case("padbwd", 2, 2, n, d, "bf16", index=470 + n + d)
    Q, K, V = workloads.make_inputs(w)
    G = _upstream(w, n + d)
    if ridge_per_row:
        g = torch.Generator(device="cpu").manual_seed(workloads.SEED0 + 9600 + n)
        lam = (0.03 * torch.exp(0.7 * torch.randn((w.B, w.H, n), generator=g))).float()
        lam_ref, lam_dev, lam_typ = lam.double().numpy(), lam.to(DEV), float(lam.double().mean())
    else:
        lam_ref = lam_dev = lam_typ = w.lam
    ref = ob.backward(Q, K, V, G, lam_ref, w.scale)
    dev = [t.to(DEV).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (Q, K, V, G)]
    got = llla.llla_backward(dev[0], dev[1], dev[2], dev[3], lam_dev, w.scale, path="mfma", return_dlambda=True)
    torch.cuda.synchronize()
    f = float(G.double().norm()) / math.sqrt(w.B * w.H) * float(V.double().pow(2).mean().sqrt())
    floor = {"dQ": f, "dK": f, "dV": f, "dlambda": f / lam_typ}
    for name, a, r in zip(("dQ", "dK", "dV", "dlambda"), got, ref):
        print(name, check_grad(a.cpu().numpy(), r, d, w.tol, "padded backward n=%d d=%d %s" % (n, d, name), floor=floor[name]))


def test_what_auto_takes_in_the_backward():
    """bf16 d = 32 goes to the matrix cores from 64 rows on, d = 16 from 512 rows on; below, the vector kernels."""
    for n, d, padded in ((200, 32, True), (40, 32, False), (200, 16, False), (1100, 16, True)):
        w = _case("padbwdauto", 1, 2, n, d, "bf16", index=480 + d)
        Q, K, V = [t.to(DEV) for t in workloads.make_inputs(w)]
        G = _upstream(w, d).to(DEV)
        a = llla.llla_backward(Q, K, V, G, w.lam, w.scale)
        m = llla.llla_backward(Q, K, V, G, w.lam, w.scale, path="mfma" if padded else "valu")
        torch.cuda.synchronize()
        for x, y in zip(a, m):
            assert torch.equal(x, y), (n, d)
