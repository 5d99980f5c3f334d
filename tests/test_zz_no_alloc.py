"""llla_decode_static: the decode call that allocates nothing (its partial records live in a device array inside the
library).  Through the C ABI, against llla_decode on the same inputs (same kernels: bit-identical) and against the
oracle, on two calls in a row, the second with a smaller input that leaves most of the first call's records in
the array."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2510_01450_amd as llla
import workloads
from paper_2510_01450_amd.binding import _Strides
from parity import check

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(B, H, L, d, index):
    w = workloads.C5.with_shape(name="static", B=B, H=H, n=L, d=d, index=index)
    return w, workloads.make_inputs(w)


def _static_through_the_c_abi(q, Kc, Vc, lam, scale, seqlens=None):
    """The raw entry point: plain device pointers, element strides, sizes, a stream."""
    B, H, L, d = Kc.shape
    o = torch.empty((B, H, d), dtype=torch.float32, device=DEV)
    sk = _Strides(Kc.stride(0), Kc.stride(1), Kc.stride(2))
    sv = _Strides(Vc.stride(0), Vc.stride(1), Vc.stride(2))
    st = llla.lib().llla_decode_static(q.data_ptr(), Kc.data_ptr(), Vc.data_ptr(), o.data_ptr(), sk, sv,
                                       0 if seqlens is None else seqlens.data_ptr(), B, H, L, d, 1, 0,
                                       ctypes.c_float(lam), ctypes.c_float(scale),
                                       torch.cuda.current_stream().cuda_stream)
    assert st == 0, llla.status_string(st)
    return o


@pytest.mark.parametrize("d", [64, 128])
def test_two_calls_in_a_row_the_second_smaller(d):
    for (B, H, L, index) in ((4, 8, 5000, 1200 + d), (1, 2, 1500, 1300 + d)):
        w, (q, Kc, Vc) = _case(B, H, L, d, index)
        qd, Kd, Vd = q.to(DEV), Kc.to(DEV), Vc.to(DEV)
        assert llla.decode_workspace_bytes(B, H, L, d, torch.bfloat16) > 0      # these shapes do use the scratch
        got = _static_through_the_c_abi(qd, Kd, Vd, w.lam, w.scale)
        want = llla.llla_decode(qd, Kd, Vd, w.lam, w.scale)
        torch.cuda.synchronize()
        assert torch.equal(got, want), "d=%d B=%d H=%d L=%d" % (d, B, H, L)
        ref = oracle.decode(q, Kc, Vc, w.lam, w.scale)
        print(check(got.cpu().numpy()[:, :, None, :], ref[:, :, None, :], np.array([L - 1]), d, w.tol,
                    "static decode d=%d L=%d" % (d, L)))


def test_sequence_lengths_and_the_binding():
    w, (q, Kc, Vc) = _case(3, 2, 3000, 64, 1400)
    lens = [3000, 40, 1025]
    qd, Kd, Vd = q.to(DEV), Kc.to(DEV), Vc.to(DEV)
    sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    out = torch.empty((3, 2, 64), dtype=torch.float32, device=DEV)
    got = llla.llla_decode_static(qd, Kd, Vd, w.lam, w.scale, out, seqlens=sl)
    want = llla.llla_decode(qd, Kd, Vd, w.lam, w.scale, seqlens=sl)
    torch.cuda.synchronize()
    assert got is out and torch.equal(got, want)
    ref = oracle.decode(q, Kc, Vc, w.lam, w.scale, seqlens=lens)
    for b, L in enumerate(lens):
        print(check(got.cpu().numpy()[b:b + 1, :, None, :], ref[b:b + 1, :, None, :], np.array([L - 1]), 64, w.tol,
                    "static decode seqlen %d" % L))


def test_a_call_beyond_the_array_is_refused():
    B, H, L, d = 64, 16, 32768, 64          # twice the decode configuration: 112 MB of records
    assert llla.decode_workspace_bytes(B, H, L, d, torch.bfloat16) > (64 << 20)
    fake = 0x10000                          # never dereferenced: the size check comes before any launch
    s = _Strides(H * L * d, L * d, d)
    st = llla.lib().llla_decode_static(fake, fake, fake, fake, s, s, 0, B, H, L, d, 1, 0, ctypes.c_float(1e-2),
                                       ctypes.c_float(0.125), 0)
    assert st == 6
