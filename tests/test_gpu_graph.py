"""The library's calls inside a HIP graph.  No entry point allocates, clears memory with a memset node, or
synchronises, so a serving loop can record a decode step (or a prefill) once and replay it.  Each case records one
call, then replays it several times on new input values written into the recorded tensors, with eager calls of the
library and synchronisations between the replays, and compares every replay bit by bit with the eager call on the
same values (the kernels are deterministic); one replay per case is also held against the fp64 oracle."""
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


def _record(fn):
    """fn() enqueues library calls on torch's current stream; returns the instantiated graph."""
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    torch.cuda.synchronize()
    return g


def _fresh(shape, dtype, seed):
    gen = torch.Generator(device="cpu").manual_seed(workloads.SEED0 + 31000 + seed)
    return torch.randn(shape, generator=gen, dtype=torch.float32).to(dtype).to(DEV)


@pytest.mark.parametrize("d,static", [(64, False), (128, False), (64, True)])
def test_decode_step_replayed(d, static):
    B, H, L = 2, 4, 2048
    lam, scale = 1e-2, 1 / math.sqrt(d)
    q, Kc, Vc = _fresh((B, H, d), torch.bfloat16, 1), _fresh((B, H, L, d), torch.bfloat16, 2), _fresh((B, H, L, d), torch.bfloat16, 3)
    out = torch.zeros((B, H, d), dtype=torch.float32, device=DEV)
    ws = torch.empty(llla.decode_workspace_bytes(B, H, L, d, torch.bfloat16) + 256, dtype=torch.uint8, device=DEV)

    def step(o):
        if static:
            llla.llla_decode_static(q, Kc, Vc, lam, scale, o)
        else:
            llla.llla_decode(q, Kc, Vc, lam, scale, workspace=ws, out=o, path="mfma")

    eager = torch.zeros_like(out)
    step(eager)                                   # first call outside the graph (one-time set-up of the library)
    g = _record(lambda: step(out))
    for r in range(4):
        q.copy_(_fresh(q.shape, q.dtype, 10 + r))
        Kc[:, :, r::7].mul_(-1.0)                 # new cache contents, in place
        Vc.copy_(_fresh(Vc.shape, Vc.dtype, 20 + r))
        step(eager)
        torch.cuda.synchronize()
        out.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), "replay %d differs from the eager call" % r
    ref = oracle.decode(q.cpu(), Kc.cpu(), Vc.cpu(), lam, scale)
    print(check(out.cpu().numpy()[:, :, None, :], ref[:, :, None, :], np.array([L - 1]), d, 2e-2, "graph decode d=%d" % d))


@pytest.mark.parametrize("n,d,dtype", [(300, 64, torch.bfloat16), (200, 128, torch.bfloat16), (260, 64, torch.float32),
                                       (300, 32, torch.bfloat16)])
def test_forward_replayed(n, d, dtype):
    B, H = 1, 3
    lam, scale = 1e-2, 1 / math.sqrt(d)
    mk = lambda s: _fresh((B, H, n, d), dtype, s) if dtype == torch.bfloat16 else \
        torch.nn.functional.normalize(_fresh((B, H, n, d), dtype, s), dim=-1)
    Q, K, V = mk(1), mk(2), _fresh((B, H, n, d), dtype, 3)
    out = torch.zeros((B, H, n, d), dtype=torch.float32, device=DEV)
    ws = torch.empty(llla.forward_workspace_bytes(B, H, n, d, dtype) + 256, dtype=torch.uint8, device=DEV)
    eager = torch.zeros_like(out)
    llla.llla_forward(Q, K, V, lam, scale, workspace=ws, out=eager, path="mfma")
    g = _record(lambda: llla.llla_forward(Q, K, V, lam, scale, workspace=ws, out=out, path="mfma"))
    for r in range(3):
        Q.copy_(mk(10 + r)); K.copy_(mk(20 + r)); V.copy_(_fresh(V.shape, dtype, 30 + r))
        llla.llla_forward(Q, K, V, lam, scale, workspace=ws, out=eager, path="mfma")
        torch.cuda.synchronize()
        out.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), "replay %d differs from the eager call" % r
    ref = oracle.forward(Q.cpu(), K.cpu(), V.cpu(), lam, scale)
    tol = 2e-2 if dtype == torch.bfloat16 else 1e-4
    print(check(out.cpu().numpy(), ref, np.arange(n), d, tol, "graph forward n=%d d=%d" % (n, d)))
