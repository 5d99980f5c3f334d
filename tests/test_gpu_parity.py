"""Parity of the HIP library (through the C ABI) with the fp64 oracle, element by element, on the
same seeded inputs.  Gate: tests/parity.py.  All tests need a GPU."""
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


def _run_forward(w, Q, K, V, path="auto", causal=True, out_dtype=torch.float32):
    O = llla.llla_forward(Q.to(DEV), K.to(DEV), V.to(DEV), w.lam, w.scale, causal=causal, path=path,
                          out_dtype=out_dtype)
    torch.cuda.synchronize()
    return O.float().cpu().numpy()


def _small(name, B, H, n, d, dtype, values=None, index=50, scale=None):
    """fp32 cases default to L2-normalised Q and K rows like C2 (the paper's QK-normalised regime), bf16 cases to
    plain N(0,1) like C3; the un-normalised fp32 regime has tests of its own (test_unnormalised_f32_*)."""
    base = workloads.C2 if dtype == "f32" else workloads.C3
    values = ("l2" if dtype == "f32" else "normal") if values is None else values
    return base.with_shape(name=name, B=B, H=H, n=n, d=d, dtype=dtype, values=values, index=index,
                           scale=(1 / math.sqrt(d)) if scale is None else scale,
                           tol=1e-4 if dtype == "f32" else 2e-2)


def test_c1_tiny_all_outputs():
    w = workloads.C1
    Q, K, V = workloads.make_inputs(w)
    ref = oracle.forward(Q, K, V, w.lam, w.scale)
    got = _run_forward(w, Q, K, V)
    print(check(got, ref, np.arange(w.n), w.d, w.tol, w.name))


def test_c2_all_outputs_f32():
    w = workloads.C2
    Q, K, V = workloads.make_inputs(w)
    ref = oracle.forward(Q, K, V, w.lam, w.scale)
    got = _run_forward(w, Q, K, V)
    print(check(got, ref, np.arange(w.n), w.d, w.tol, w.name))


@pytest.mark.parametrize("n,d,dtype", [
    (1, 16, "f32"), (2, 64, "f32"), (77, 16, "f32"), (130, 32, "f32"), (203, 64, "f32"), (150, 128, "f32"),
    (77, 16, "bf16"), (131, 32, "bf16"), (333, 64, "bf16"), (257, 128, "bf16"),
])
@pytest.mark.parametrize("path", ["valu", "auto"])
def test_ragged_shapes_all_outputs(n, d, dtype, path):
    """Sizes that span several tiles with a ragged tail, both dtypes, every supported d."""
    w = _small("ragged", 2, 3, n, d, dtype, index=60 + d + n)
    Q, K, V = workloads.make_inputs(w)
    ref = oracle.forward(Q, K, V, w.lam, w.scale)
    got = _run_forward(w, Q, K, V, path=path)
    print(check(got, ref, np.arange(n), d, w.tol, "%s n=%d d=%d %s" % (path, n, d, dtype)))


@pytest.mark.parametrize("n,d", [(200, 16), (250, 32), (300, 64), (300, 128)])
@pytest.mark.parametrize("path", ["valu", "auto"])
def test_unnormalised_f32_forward(n, d, path):
    """fp32 inputs that are NOT normalised: Q, K, V ~ N(0,1).  A row that sees fewer keys than features has
    rho ~ ||z||/lambda and delta ~ lambda/||z||^2 in Eq. (lla), and its output weights w (1 - z.rho)/delta cancel by a
    factor ||z||^2/lambda ~ 10^4: the library serves those rows in fp64 in key space, where nothing cancels."""
    w = _small("unnorm", 2, 2, n, d, "f32", values="normal", index=970 + d)
    Q, K, V = workloads.make_inputs(w)
    ref = oracle.forward(Q, K, V, w.lam, w.scale)
    got = _run_forward(w, Q, K, V, path=path)
    print(check(got, ref, np.arange(n), d, w.tol, "unnormalised f32 %s n=%d d=%d" % (path, n, d)))


@pytest.mark.parametrize("d", [16, 32, 64, 128])
@pytest.mark.parametrize("path", ["valu", "auto"])
def test_unnormalised_f32_decode(d, path):
    """The same regime for the decode call: caches of 1 key up to a few times d keys, with and without per-sequence
    lengths (both sides of the limit below which a sequence is served in key space)."""
    for L in (1, 5, d // 2, d, d + 1, 2 * d + 3, 4 * d + 3):
        w = _small("unnormdec", 3, 2, L, d, "f32", values="normal", index=980 + d + L).with_shape(kind="decode")
        q, Kc, Vc = workloads.make_inputs(w)
        ref = oracle.decode(q, Kc, Vc, w.lam, w.scale)
        got = llla.llla_decode(q.to(DEV), Kc.to(DEV), Vc.to(DEV), w.lam, w.scale, path=path).cpu().numpy()
        print(L, check(got[:, :, None, :], ref[:, :, None, :], np.array([L - 1]), d, w.tol, "decode L=%d d=%d" % (L, d)))
    L = 4 * d + 3
    lens = [1, min(d, 64), min(d, 64) + 1]
    ref = oracle.decode(q, Kc, Vc, w.lam, w.scale, seqlens=lens)
    sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    got = llla.llla_decode(q.to(DEV), Kc.to(DEV), Vc.to(DEV), w.lam, w.scale, seqlens=sl, path=path).cpu().numpy()
    for b, Lb in enumerate(lens):
        print(Lb, check(got[b:b + 1, :, None, :], ref[b:b + 1, :, None, :], np.array([Lb - 1]), d, w.tol,
                        "decode seqlen %d of %d, d=%d" % (Lb, L, d)))


def test_unnormalised_f32_statistics_and_ridge_per_row():
    """rho, delta and a ridge per row on un-normalised fp32 inputs (rows on both sides of the key-space limit)."""
    n, d = 150, 32
    w = _small("unnormex", 1, 2, n, d, "f32", values="normal", index=990)
    Q, K, V = workloads.make_inputs(w)
    g = torch.Generator().manual_seed(991)
    lam = (10.0 ** (torch.rand(1, 2, n, generator=g) * 2.0 - 3.0)).float()
    refO, refR, refD = oracle.forward_ex(Q, K, V, lam.numpy(), w.scale)
    O, R, Dl = llla.llla_forward(Q.to(DEV), K.to(DEV), V.to(DEV), lam.to(DEV), w.scale, return_stats=True)
    torch.cuda.synchronize()
    rows = np.arange(n)
    print(check(O.cpu().numpy(), refO, rows, d, w.tol, "unnormalised ex"))
    print(check(R.cpu().numpy(), refR, rows, d, w.tol, "unnormalised ex rho"))
    print(check(Dl.cpu().numpy()[..., None], refD[..., None], rows, d, w.tol, "unnormalised ex delta"))


@pytest.mark.parametrize("n,d,dtype,path", [
    (150, 16, "f32", "auto"), (150, 64, "f32", "valu"), (150, 64, "bf16", "valu"), (150, 128, "bf16", "valu"),
    (40, 64, "f32", "mfma"), (150, 64, "f32", "mfma"), (700, 64, "f32", "mfma"),
    (100, 64, "bf16", "mfma"), (150, 64, "bf16", "mfma"), (700, 64, "bf16", "mfma"),
    (150, 128, "bf16", "mfma"), (257, 128, "bf16", "mfma"), (600, 128, "bf16", "mfma"),
])
def test_non_causal(n, d, dtype, path):
    """causal = 0: every row sees all n keys (the matrix form of Section 3.2 without its tril mask), on the vector
    kernels and on the matrix-core kernels, below and above the row count at which the latter change variant."""
    w = _small("noncausal", 1, 2, n, d, dtype, index=70 + d + n)
    Q, K, V = workloads.make_inputs(w)
    ref = oracle.forward(Q, K, V, w.lam, w.scale, causal=False)
    got = _run_forward(w, Q, K, V, causal=False, path=path)
    # every row sees all n keys; rows are "late" rows in the sense of the gate only if n > 4d
    print(check(got, ref, np.full(w.n, w.n - 1), d, w.tol, "noncausal %s n=%d d=%d %s" % (path, n, d, dtype)))
    if path == "mfma":
        got16 = _run_forward(w, Q, K, V, causal=False, path=path, out_dtype=torch.bfloat16)
        print(check(got16, ref, np.full(w.n, w.n - 1), d, max(w.tol, 2e-2), "noncausal bf16 out"))


def test_strided_inputs_and_bf16_output():
    """[B, n, H, d] memory viewed as [B, H, n, d] (the usual projection layout), bf16 output."""
    w = _small("strided", 2, 4, 160, 64, "bf16", index=81)
    Q, K, V = workloads.make_inputs(w)
    ref = oracle.forward(Q, K, V, w.lam, w.scale)
    dev = [t.to(DEV).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (Q, K, V)]
    assert not dev[0].is_contiguous()
    O = llla.llla_forward(dev[0], dev[1], dev[2], w.lam, w.scale, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    got = O.float().cpu().numpy()
    # bf16 rounding of the output adds 2^-9 relative per element
    print(check(got, ref, np.arange(w.n), w.d, w.tol, "strided"))


@pytest.mark.parametrize("n,d", [(700, 64), (1100, 64), (600, 128), (1030, 128)])
def test_mfma_path_all_outputs_and_bf16_output(n, d):
    """The matrix-core path end to end (precise rows, fast rows, both output sweeps), forced with
    path='mfma', all outputs against the oracle; bf16 output rounding is inside the bf16 tolerance."""
    w = _small("mfma", 1, 3, n, d, "bf16", index=300 + n + d)
    Q, K, V = workloads.make_inputs(w)
    ref = oracle.forward(Q, K, V, w.lam, w.scale)
    got = _run_forward(w, Q, K, V, path="mfma")
    print(check(got, ref, np.arange(n), d, w.tol, "mfma n=%d d=%d" % (n, d)))
    got16 = _run_forward(w, Q, K, V, path="mfma", out_dtype=torch.bfloat16)
    print(check(got16, ref, np.arange(n), d, w.tol, "mfma bf16 out n=%d d=%d" % (n, d)))
    valu = _run_forward(w, Q, K, V, path="valu")
    late = np.arange(n) >= 4 * d
    err = np.linalg.norm(got[..., late, :] - valu[..., late, :]) / np.linalg.norm(valu[..., late, :])
    assert err < 2e-3, err          # the two kernel families agree far inside the tolerance


@pytest.mark.parametrize("n,values,scale", [(1024, "l2", None), (700, "normal", None), (333, "l2", 60.0), (333, "l2", -45.0),
                                            (130, "normal", 0.0)])
def test_f32_matrix_core_path_all_outputs(n, values, scale):
    """fp32 inputs at d = 64 on the matrix cores (fp32 MFMA), forced with path='mfma': all outputs, rho and delta against
    the oracle.  The logits of the scale-60 cases span more than 2^64, so the reference exponent of the weights moves
    during the sweep and the accumulated moments are rescaled (the lazy form of Algorithm 1's running maximum)."""
    w = _small("f32mfma", 2, 2, n, 64, "f32", values=values, index=1500 + n, scale=scale)
    Q, K, V = workloads.make_inputs(w)
    refO, refR, refD = oracle.forward_ex(Q, K, V, w.lam, w.scale)
    O, R, Dl = llla.llla_forward(Q.to(DEV), K.to(DEV), V.to(DEV), w.lam, w.scale, path="mfma", return_stats=True)
    torch.cuda.synchronize()
    rows = np.arange(n)
    what = "f32 mfma n=%d %s scale=%s" % (n, values, scale)
    print(check(O.cpu().numpy(), refO, rows, 64, w.tol, what))
    print(check(R.cpu().numpy(), refR, rows, 64, w.tol, what + " rho"))
    print(check(Dl.cpu().numpy()[..., None], refD[..., None], rows, 64, w.tol, what + " delta"))
    valu = llla.llla_forward(Q.to(DEV), K.to(DEV), V.to(DEV), w.lam, w.scale, path="valu").cpu().numpy()
    late = rows >= 256
    if late.any():
        assert np.linalg.norm(O.cpu().numpy()[..., late, :] - valu[..., late, :]) / np.linalg.norm(valu[..., late, :]) < 1e-4


def test_mfma_path_refuses_what_it_does_not_serve():
    x = torch.zeros(1, 1, 64, 32, dtype=torch.float32, device=DEV)
    with pytest.raises(llla.LlaError) as e:
        llla.llla_forward_cg(x, x, x, 1e-2, 0.2, 4)                 # the approximate mode serves bf16 inputs only
    assert e.value.code == 7
    y = torch.zeros(1, 1, 64, 128, dtype=torch.float32, device=DEV)
    with pytest.raises(llla.LlaError) as e:
        llla.llla_forward(y, y, y, 1e-2, 0.2, path="mfma")          # fp32 inputs at d = 128 neither
    assert e.value.code == 7
    z = torch.zeros(1, 1, 512, 64, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(llla.LlaError) as e:
        llla.llla_forward(z, z, z, 1e-2, 0.2, path="mfma", workspace=torch.zeros(256, dtype=torch.uint8, device=DEV))
    assert e.value.code == 6                                        # workspace too small


def test_lambda_and_scale_are_honoured():
    w = _small("lam", 1, 2, 200, 32, "f32", index=90)
    Q, K, V = workloads.make_inputs(w)
    for lam, scale in ((1.0, 0.1), (1e-3, 0.3), (50.0, 1.0)):
        ref = oracle.forward(Q, K, V, lam, scale)
        got = llla.llla_forward(Q.to(DEV), K.to(DEV), V.to(DEV), lam, scale).cpu().numpy()
        print(check(got, ref, np.arange(w.n), w.d, 1e-4, "lam=%g scale=%g" % (lam, scale)))


@pytest.mark.parametrize("d,dtype", [(64, "bf16"), (128, "bf16"), (64, "f32")])
@pytest.mark.parametrize("lam", [1e-3, 3e-4])
def test_small_ridge_on_the_matrix_core_paths(d, dtype, lam):
    """Ridges below the default 1e-2: the factorisation on the matrix-core paths raises a computed pivot that falls
    below half the ridge to that value (in exact arithmetic every pivot is at least the ridge), so small ridges must
    still give finite outputs, and outputs that pass the usual gate against the oracle."""
    w = _small("smallridge", 1, 2, 600, d, dtype, index=150 + d).with_shape(lam=lam)
    Q, K, V = workloads.make_inputs(w)
    ref = oracle.forward(Q, K, V, lam, w.scale)
    got = _run_forward(w, Q, K, V, path="mfma")
    assert np.isfinite(got).all()
    print(lam, check(got, ref, np.arange(w.n), d, w.tol, "small ridge %g d=%d %s" % (lam, d, dtype)))
    if dtype == "bf16":
        wd = _small("smallridgedec", 2, 2, 700, d, dtype, index=160 + d).with_shape(kind="decode", lam=lam)
        q, Kc, Vc = workloads.make_inputs(wd)
        refd = oracle.decode(q, Kc, Vc, lam, wd.scale)
        gotd = llla.llla_decode(q.to(DEV), Kc.to(DEV), Vc.to(DEV), lam, wd.scale, path="mfma").cpu().numpy()
        assert np.isfinite(gotd).all()
        print(lam, check(gotd[:, :, None, :], refd[:, :, None, :], np.array([699]), d, wd.tol, "small ridge decode %g d=%d" % (lam, d)))


def test_large_logits_do_not_overflow():
    """Row-max normalisation: logits up to +-60 (unit-norm rows, scale 60) must still give finite,
    correct outputs."""
    w = _small("big", 1, 1, 96, 16, "f32", index=91, scale=60.0)
    Q, K, V = workloads.make_inputs(w)
    ref = oracle.forward(Q, K, V, w.lam, w.scale)
    got = _run_forward(w, Q, K, V)
    print(check(got, ref, np.arange(w.n), w.d, 1e-4, "large logits"))


@pytest.mark.parametrize("path,d", [("mfma", 64), ("mfma", 128), ("valu", 64)])
def test_negative_and_zero_scale(path, d):
    """scale only has to be finite: a negative one turns the nearest keys into the farthest (the row maximum is then
    the scaled MINIMUM of the products), zero makes all weights equal."""
    for scale in (-0.11, 0.0):
        w = _small("negscale", 1, 2, 333, d, "bf16", index=140 + d).with_shape(scale=scale)
        Q, K, V = workloads.make_inputs(w)
        ref = oracle.forward(Q, K, V, w.lam, scale)
        got = llla.llla_forward(Q.to(DEV), K.to(DEV), V.to(DEV), w.lam, scale, path=path).cpu().numpy()
        print(scale, check(got, ref, np.arange(w.n), d, w.tol, "scale %g %s d=%d" % (scale, path, d)))


def test_deterministic():
    w = _small("det", 2, 2, 300, 64, "bf16", index=92)
    Q, K, V = [t.to(DEV) for t in workloads.make_inputs(w)]
    a = llla.llla_forward(Q, K, V, w.lam, w.scale)
    b = llla.llla_forward(Q, K, V, w.lam, w.scale)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


# ---- decode --------------------------------------------------------------------------------------
@pytest.mark.parametrize("L,d,dtype", [
    (1, 64, "f32"), (5, 16, "f32"), (100, 32, "f32"), (1000, 64, "f32"), (777, 128, "f32"),
    (300, 16, "bf16"), (1531, 64, "bf16"), (2049, 128, "bf16"),
])
@pytest.mark.parametrize("path", ["valu", "auto"])
def test_decode_matches_oracle(L, d, dtype, path):
    w = _small("dec", 3, 2, L, d, dtype, index=100 + d + L).with_shape(kind="decode")
    q, Kc, Vc = workloads.make_inputs(w)
    ref = oracle.decode(q, Kc, Vc, w.lam, w.scale)
    got = llla.llla_decode(q.to(DEV), Kc.to(DEV), Vc.to(DEV), w.lam, w.scale, path=path).cpu().numpy()
    rows = np.array([L - 1])
    print(check(got[:, :, None, :], ref[:, :, None, :], rows, d, w.tol, "decode L=%d d=%d %s" % (L, d, dtype)))


@pytest.mark.parametrize("B,H,L", [(1, 2, 4096), (2, 3, 5000), (4, 8, 1024), (1, 2, 20000), (1, 1, 40000), (3, 1, 16384)])
def test_decode_mfma_splits_and_bf16_output(B, H, L):
    """The single-pass matrix-core decode with several cache splits per head and a ragged last step; the long caches
    with few heads are cut into more than 16 partials per head and take the combine stage before the merge."""
    w = _small("decm", B, H, L, 64, "bf16", index=400 + L).with_shape(kind="decode")
    q, Kc, Vc = workloads.make_inputs(w)
    ref = oracle.decode(q, Kc, Vc, w.lam, w.scale)
    for od in (torch.float32, torch.bfloat16):
        got = llla.llla_decode(q.to(DEV), Kc.to(DEV), Vc.to(DEV), w.lam, w.scale, path="mfma", out_dtype=od)
        got = got.float().cpu().numpy()
        print(check(got[:, :, None, :], ref[:, :, None, :], np.array([L - 1]), 64, w.tol, "decode mfma L=%d" % L))
    valu = llla.llla_decode(q.to(DEV), Kc.to(DEV), Vc.to(DEV), w.lam, w.scale, path="valu").cpu().numpy()
    assert np.linalg.norm(got - valu) / np.linalg.norm(valu) < 1e-2


@pytest.mark.parametrize("B,H,L", [(1, 2, 4096), (2, 3, 5000), (4, 8, 1024), (1, 1, 40000), (3, 1, 16384), (70, 8, 1500)])
def test_decode_mfma_d128_splits_and_bf16_output(B, H, L):
    """d = 128: the four waves of a workgroup share one key stream and each owns a quarter of the moment tiles; 1 to
    32 workgroups per head, ragged last steps, both output types."""
    w = _small("decm128", B, H, L, 128, "bf16", index=500 + L).with_shape(kind="decode")
    q, Kc, Vc = workloads.make_inputs(w)
    ref = oracle.decode(q, Kc, Vc, w.lam, w.scale)
    for od in (torch.float32, torch.bfloat16):
        got = llla.llla_decode(q.to(DEV), Kc.to(DEV), Vc.to(DEV), w.lam, w.scale, path="mfma", out_dtype=od)
        got = got.float().cpu().numpy()
        print(check(got[:, :, None, :], ref[:, :, None, :], np.array([L - 1]), 128, w.tol, "decode mfma d=128 L=%d" % L))
    valu = llla.llla_decode(q.to(DEV), Kc.to(DEV), Vc.to(DEV), w.lam, w.scale, path="valu").cpu().numpy()
    assert np.linalg.norm(got - valu) / np.linalg.norm(valu) < 1e-2


@pytest.mark.parametrize("d", [64, 128])
def test_decode_mfma_short_caches(d):
    """Cache capacities from 256 rows up on the matrix-core decode (a wave then has as little as two 32-key steps),
    with the full length and with shorter per-sequence lengths; below 256 rows the matrix-core path does not serve."""
    for L in (256, 300, 511, 777, 1023):
        w = _small("decshortcache", 3, 2, L, d, "bf16", index=1600 + d + L).with_shape(kind="decode")
        q, Kc, Vc = workloads.make_inputs(w)
        ref = oracle.decode(q, Kc, Vc, w.lam, w.scale)
        got = llla.llla_decode(q.to(DEV), Kc.to(DEV), Vc.to(DEV), w.lam, w.scale, path="mfma").cpu().numpy()
        print(L, check(got[:, :, None, :], ref[:, :, None, :], np.array([L - 1]), d, w.tol, "decode mfma d=%d L=%d" % (d, L)))
        lens = [L, 1, L // 2 + 1]
        ref = oracle.decode(q, Kc, Vc, w.lam, w.scale, seqlens=lens)
        sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
        got = llla.llla_decode(q.to(DEV), Kc.to(DEV), Vc.to(DEV), w.lam, w.scale, seqlens=sl, path="mfma").cpu().numpy()
        for b, Lb in enumerate(lens):
            print(check(got[b:b + 1, :, None, :], ref[b:b + 1, :, None, :], np.array([Lb - 1]), d, w.tol,
                        "decode mfma d=%d seqlen %d of %d" % (d, Lb, L)))
    x = torch.zeros(1, 1, 255, d, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(llla.LlaError) as e:
        llla.llla_decode(x[:, :, 0], x, x, 1e-2, 0.1, path="mfma")
    assert e.value.code == 7


def test_decode_mfma_d128_seqlens_ignore_the_tail_and_strided_cache():
    """d = 128 with per-sequence lengths (a sequence of one key, idle workgroups beyond a short sequence, a ragged
    last step) on a cache whose tail is poisoned with NaN; the cache is a view with a row pitch of 2 d."""
    w = _small("decsl128", 5, 2, 9000, 128, "bf16", index=123).with_shape(kind="decode")
    q, Kc, Vc = workloads.make_inputs(w)
    lens = [9000, 1, 33, 1024, 8999]
    ref = oracle.decode(q, Kc, Vc, w.lam, w.scale, seqlens=lens)
    Kw = torch.full((5, 2, 9000, 256), float("nan"), dtype=torch.bfloat16)
    Vw = torch.full((5, 2, 9000, 256), float("nan"), dtype=torch.bfloat16)
    Kw[..., :128] = Kc
    Vw[..., 128:] = Vc
    for b, L in enumerate(lens):
        Kw[b, :, L:] = float("nan")
        Vw[b, :, L:] = float("nan")
    Kd, Vd = Kw.to(DEV)[..., :128], Vw.to(DEV)[..., 128:]
    sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    got = llla.llla_decode(q.to(DEV), Kd, Vd, w.lam, w.scale, seqlens=sl, path="mfma").cpu().numpy()
    for b, L in enumerate(lens):
        print(check(got[b:b + 1, :, None, :], ref[b:b + 1, :, None, :], np.array([L - 1]), w.d, w.tol,
                    "decode d=128 seqlen %d of 9000" % L))


@pytest.mark.parametrize("d", [64, 128])
def test_decode_mfma_short_sequences_in_a_long_cache(d):
    """Sequences with fewer keys than features, about as many, and a few times as many (the ill-conditioned range,
    where only the ridge holds some directions) in a cache long enough for the matrix-core path."""
    lens = [17, 100, 127, 128, 129, 200, 256, 400, 512, 513, 700, 1024]
    w = _small("decshort", len(lens), 2, 1024, d, "bf16", index=124 + d).with_shape(kind="decode")
    q, Kc, Vc = workloads.make_inputs(w)
    ref = oracle.decode(q, Kc, Vc, w.lam, w.scale, seqlens=lens)
    sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    got = llla.llla_decode(q.to(DEV), Kc.to(DEV), Vc.to(DEV), w.lam, w.scale, seqlens=sl, path="mfma").cpu().numpy()
    for b, L in enumerate(lens):
        print(L, check(got[b:b + 1, :, None, :], ref[b:b + 1, :, None, :], np.array([L - 1]), w.d, w.tol,
                       "decode d=%d seqlen %d of 1024" % (d, L)))


@pytest.mark.parametrize("d", [64, 128])
def test_decode_mfma_is_deterministic_and_independent_of_order_and_split(d):
    """The decode moments are sums over a set of keys: the output may not depend on the order of the cache rows, on
    the number of workgroups a head is cut into (set by the cache capacity and the batch), or on the run."""
    L = 6000
    w = _small("decinv", 2, 2, L, d, "bf16", index=130 + d).with_shape(kind="decode")
    q, Kc, Vc = workloads.make_inputs(w)
    ref = oracle.decode(q, Kc, Vc, w.lam, w.scale)
    qd, Kd, Vd = q.to(DEV), Kc.to(DEV), Vc.to(DEV)
    a = llla.llla_decode(qd, Kd, Vd, w.lam, w.scale, path="mfma")
    b = llla.llla_decode(qd, Kd, Vd, w.lam, w.scale, path="mfma")
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    a = a.cpu().numpy()
    print(check(a[:, :, None, :], ref[:, :, None, :], np.array([L - 1]), d, w.tol, "decode d=%d" % d))
    # the same keys in another order
    perm = torch.randperm(L, generator=torch.Generator().manual_seed(7))
    p = llla.llla_decode(qd, Kc[:, :, perm].contiguous().to(DEV), Vc[:, :, perm].contiguous().to(DEV), w.lam, w.scale,
                         path="mfma").cpu().numpy()
    print(check(p[:, :, None, :], ref[:, :, None, :], np.array([L - 1]), d, w.tol, "decode d=%d, permuted cache" % d))
    assert np.linalg.norm(p - a) / np.linalg.norm(a) < 1e-3
    # the same sequences in a cache of four times the capacity (more workgroups per head), and in a batch large
    # enough that every head gets a single workgroup
    big = torch.zeros(2, 2, 4 * L, d, dtype=torch.bfloat16)
    Kb, Vb = big.clone(), big.clone()
    Kb[:, :, :L], Vb[:, :, :L] = Kc, Vc
    sl = torch.full((2,), L, dtype=torch.int32, device=DEV)
    c = llla.llla_decode(qd, Kb.to(DEV), Vb.to(DEV), w.lam, w.scale, seqlens=sl, path="mfma").cpu().numpy()
    assert np.linalg.norm(c - a) / np.linalg.norm(a) < 1e-3
    rep = 160
    e = llla.llla_decode(qd.repeat(rep, 1, 1), Kd.repeat(rep, 1, 1, 1), Vd.repeat(rep, 1, 1, 1), w.lam, w.scale,
                         path="mfma").cpu().numpy()
    # (copies of a head in different batch entries sweep their keys from different starting points: equal up to
    # rounding, not bit by bit)
    assert np.linalg.norm(e[:2] - a) / np.linalg.norm(a) < 1e-3 and np.linalg.norm(e[-2:] - a) / np.linalg.norm(a) < 1e-3


def test_decode_seqlens_and_forward_last_row():
    w = _small("decsl", 4, 2, 600, 64, "bf16", index=120).with_shape(kind="decode")
    q, Kc, Vc = workloads.make_inputs(w)
    lens = [600, 1, 257, 64]
    ref = oracle.decode(q, Kc, Vc, w.lam, w.scale, seqlens=lens)
    sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    got = llla.llla_decode(q.to(DEV), Kc.to(DEV), Vc.to(DEV), w.lam, w.scale, seqlens=sl).cpu().numpy()
    for b, L in enumerate(lens):
        print(check(got[b:b + 1, :, None, :], ref[b:b + 1, :, None, :], np.array([L - 1]), w.d, w.tol,
                    "decode seqlen %d" % L))
    # decode == last row of the forward over the same keys (query independence, Section 3.2)
    Qf = torch.randn(1, 2, 600, 64).to(torch.bfloat16)
    Qf[:, :, -1] = q[0:1]
    fwd = llla.llla_forward(Qf.to(DEV), Kc[0:1].to(DEV), Vc[0:1].to(DEV), w.lam, w.scale).cpu().numpy()
    err = np.linalg.norm(fwd[0, :, -1] - got[0]) / np.linalg.norm(got[0])
    assert err < 1e-3, err


def test_decode_seqlens_with_many_partials():
    """Few heads, long cache, short and long sequences: partials beyond a sequence's length are empty and the combine
    stage has to carry them (all-empty groups included)."""
    w = _small("decsl3", 3, 1, 20000, 64, "bf16", index=122).with_shape(kind="decode")
    q, Kc, Vc = workloads.make_inputs(w)
    lens = [20000, 700, 9000]
    ref = oracle.decode(q, Kc, Vc, w.lam, w.scale, seqlens=lens)
    Kp, Vp = Kc.clone(), Vc.clone()
    for b, L in enumerate(lens):
        Kp[b, :, L:] = float("nan")
        Vp[b, :, L:] = float("nan")
    sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    got = llla.llla_decode(q.to(DEV), Kp.to(DEV), Vp.to(DEV), w.lam, w.scale, seqlens=sl, path="mfma").cpu().numpy()
    for b, L in enumerate(lens):
        print(check(got[b:b + 1, :, None, :], ref[b:b + 1, :, None, :], np.array([L - 1]), w.d, w.tol,
                    "decode seqlen %d of 20000" % L))


@pytest.mark.parametrize("path", ["mfma", "valu"])
def test_decode_seqlens_long_cache_ignores_the_tail(path):
    """Per-sequence lengths on a cache long enough for the matrix-core path; everything at and beyond a
    sequence's length is poisoned with NaN and must not reach the output."""
    w = _small("decsl2", 5, 2, 3000, 64, "bf16", index=121).with_shape(kind="decode")
    q, Kc, Vc = workloads.make_inputs(w)
    lens = [3000, 1, 33, 1024, 2999]
    ref = oracle.decode(q, Kc, Vc, w.lam, w.scale, seqlens=lens)
    Kp, Vp = Kc.clone(), Vc.clone()
    for b, L in enumerate(lens):
        Kp[b, :, L:] = float("nan")
        Vp[b, :, L:] = float("nan")
    sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    got = llla.llla_decode(q.to(DEV), Kp.to(DEV), Vp.to(DEV), w.lam, w.scale, seqlens=sl, path=path).cpu().numpy()
    for b, L in enumerate(lens):
        print(check(got[b:b + 1, :, None, :], ref[b:b + 1, :, None, :], np.array([L - 1]), w.d, w.tol,
                    "decode %s seqlen %d of 3000" % (path, L)))


# ---- the large configurations: sampled rows --------------------------------------------------------
def _sampled(w, heads):
    Q, K, V = workloads.make_inputs(w)
    rows = workloads.sample_rows(w)
    O = llla.llla_forward(Q.to(DEV), K.to(DEV), V.to(DEV), w.lam, w.scale)
    torch.cuda.synchronize()
    O = O.cpu().numpy()
    assert np.all(np.isfinite(O))
    for (b, h) in heads:
        ref = oracle.forward_head(Q[b, h], K[b, h], V[b, h], w.lam, w.scale, rows=rows)
        print((b, h), check(O[b, h][rows][None, None], ref[None, None], rows, w.d, w.tol, "%s head %s" % (w.name, (b, h))))


def test_c3_prefill_sampled_rows():
    w = workloads.C3
    _sampled(w, [(0, h) for h in range(w.H)] + [(3, 7), (2, 15)])


def test_c3b_prefill_n8192_sampled_rows():
    """The shape the matrix-core utilisation target is quoted for (d = 64, n = 8192)."""
    w = workloads.C3B
    _sampled(w, [(0, h) for h in range(w.H)] + [(1, 15), (1, 6)])


def test_c4_long_context_sampled_rows():
    w = workloads.C4
    _sampled(w, [(0, h) for h in range(w.H)])


@pytest.mark.parametrize("n,d,H", [(65536, 64, 2), (49152 + 77, 128, 1)])
def test_very_long_sequences_sampled_rows(n, d, H):
    """Sequences eight times the longest benchmark shape (1024 key blocks per row, a ragged last block at d = 128):
    offsets into the re-tiled keys, the row maxima and the y rows far beyond 2^16 rows, rows at both ends and at block
    boundaries in between."""
    w = _small("verylong", 1, H, n, d, "bf16", index=1700 + d)
    Q, K, V = workloads.make_inputs(w)
    rows = np.array(sorted({0, 1, 63, 64, 2 * d - 1, 2 * d, 4095, 4096, 32767, 32768, 32769, n // 2 + 31, n - 65, n - 64, n - 2,
                            n - 1}))
    O = llla.llla_forward(Q.to(DEV), K.to(DEV), V.to(DEV), w.lam, w.scale)
    torch.cuda.synchronize()
    O = O.cpu().numpy()
    assert np.all(np.isfinite(O))
    for h in range(H):
        ref = oracle.forward_head(Q[0, h], K[0, h], V[0, h], w.lam, w.scale, rows=rows)
        print(h, check(O[0, h][rows][None, None], ref[None, None], rows, d, w.tol, "n=%d d=%d head %d" % (n, d, h)))


def test_c5_decode_all_heads():
    """Every one of the 512 outputs of the decode configuration against the oracle, one sequence (16 heads) at a time."""
    w = workloads.C5
    q, Kc, Vc = workloads.make_inputs(w)
    got = llla.llla_decode(q.to(DEV), Kc.to(DEV), Vc.to(DEV), w.lam, w.scale)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    assert np.all(np.isfinite(got))
    worst = 0.0
    for b in range(w.B):
        ref = oracle.decode(q[b:b + 1], Kc[b:b + 1], Vc[b:b + 1], w.lam, w.scale)
        s = check(got[b:b + 1, :, None, :], ref[:, :, None, :], np.array([w.n - 1]), w.d, w.tol, "C5 sequence %d" % b)
        worst = max(worst, s["worst_ratio_to_bound"])
    print("C5, all %d heads: worst error / bound = %.3f" % (w.B * w.H, worst))


def test_c5d128_decode_sampled_heads():
    """The d = 128 decode shape that bench.py times (256 heads x 32768 cached keys), sampled heads."""
    w = workloads.C5D128
    q, Kc, Vc = workloads.make_inputs(w)
    got = llla.llla_decode(q.to(DEV), Kc.to(DEV), Vc.to(DEV), w.lam, w.scale)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    assert np.all(np.isfinite(got))
    for (b, h) in [(0, 0), (0, 15), (7, 3), (15, 15), (15, 0), (12, 12), (3, 9), (9, 1)]:
        ref = oracle.decode(q[b:b + 1, h:h + 1], Kc[b:b + 1, h:h + 1], Vc[b:b + 1, h:h + 1], w.lam, w.scale)
        print((b, h), check(got[b:b + 1, h:h + 1, None, :], ref[:, :, None, :], np.array([w.n - 1]), w.d, w.tol,
                            "C5d128 head %s" % ((b, h),)))


# ---- extended forward: a ridge per row (Appendix C) and the statistics rho, delta of Eq. (lla) -----------
def _stat_check(got_r, ref_r, got_d, ref_d, rows, d, tol, what):
    """rho and delta against the oracle with the same gate as the outputs (delta as a 1-vector per row)."""
    print(check(got_r, ref_r, rows, d, tol, what + " rho"))
    print(check(got_d[..., None], ref_d[..., None], rows, d, tol, what + " delta"))


@pytest.mark.parametrize("n,d,dtype,path", [
    (130, 32, "f32", "valu"), (203, 64, "f32", "auto"), (150, 128, "f32", "auto"),
    (131, 32, "bf16", "auto"), (333, 64, "bf16", "valu"), (333, 64, "bf16", "mfma"), (600, 64, "bf16", "mfma"),
    (290, 128, "bf16", "mfma"),
])
def test_forward_ex_per_row_ridge_and_statistics(n, d, dtype, path):
    w = _small("ex", 2, 2, n, d, dtype, index=700 + d + n)
    Q, K, V = workloads.make_inputs(w)
    g = torch.Generator().manual_seed(900 + n)
    lam = (10.0 ** (torch.rand(2, 2, n, generator=g) * 2.0 - 3.0)).float()        # 1e-3 .. 1e-1, per row
    refO, refR, refD = oracle.forward_ex(Q, K, V, lam.numpy(), w.scale)
    O, R, Dl = llla.llla_forward(Q.to(DEV), K.to(DEV), V.to(DEV), lam.to(DEV), w.scale, path=path, return_stats=True)
    torch.cuda.synchronize()
    rows = np.arange(n)
    print(check(O.cpu().numpy(), refO, rows, d, w.tol, "ex %s n=%d d=%d %s" % (path, n, d, dtype)))
    _stat_check(R.cpu().numpy(), refR, Dl.cpu().numpy(), refD, rows, d, w.tol, "ex %s n=%d d=%d %s" % (path, n, d, dtype))
    # a constant per-row ridge and the scalar give the same output; statistics do not disturb it
    lam_c = torch.full((2, 2, n), w.lam, dtype=torch.float32, device=DEV)
    a = llla.llla_forward(Q.to(DEV), K.to(DEV), V.to(DEV), lam_c, w.scale, path=path)
    b, _, _ = llla.llla_forward(Q.to(DEV), K.to(DEV), V.to(DEV), w.lam, w.scale, path=path, return_stats=True)
    c = llla.llla_forward(Q.to(DEV), K.to(DEV), V.to(DEV), w.lam, w.scale, path=path)
    assert torch.equal(a, c) and torch.equal(b, c)


def test_forward_ex_rejects_a_host_ridge_tensor():
    w = _small("exbad", 1, 1, 64, 16, "f32")
    Q, K, V = [t.to(DEV) for t in workloads.make_inputs(w)]
    with pytest.raises(ValueError):
        llla.llla_forward(Q, K, V, torch.full((1, 1, 64), 0.01), w.scale)


# ---- approximate mode: rho from T conjugate-gradient steps (Section 3.1 / Appendix C) ------------------------
@pytest.mark.parametrize("n,d,T", [(333, 64, 0), (333, 64, 1), (333, 64, 2), (600, 64, 2), (290, 128, 1), (290, 128, 2)])
def test_forward_cg_first_steps_match_the_cg_oracle(n, d, T):
    """Element-wise against the fp64 CG oracle with the same number of steps.  Only the first steps can be compared
    this way: CG iterates of an ill-conditioned system are not stable under rounding (two fp64 runs already drift
    apart, see the SciPy pin), so later iterates are checked through their residuals instead (next test)."""
    w = _small("cg", 1, 2, n, d, "bf16", index=800 + d + n + T)
    Q, K, V = workloads.make_inputs(w)
    O, R, Dl, steps = llla.llla_forward_cg(Q.to(DEV), K.to(DEV), V.to(DEV), w.lam, w.scale, T, 0.0, return_stats=True)
    torch.cuda.synchronize()
    O, R, Dl, steps = O.cpu().numpy(), R.cpu().numpy(), Dl.cpu().numpy(), steps.cpu().numpy()
    rows = np.arange(n)
    for h in range(2):
        refO, refR, refD, used = oracle.forward_head_cg(Q[0, h], K[0, h], V[0, h], w.lam, w.scale, T, 0.0)
        what = "cg T=%d n=%d d=%d head %d" % (T, n, d, h)
        print(check(O[0:1, h:h + 1], refO[None, None], rows, d, w.tol, what))
        assert np.array_equal(steps[0, h], used)
        if T > 0:
            print(check(R[0:1, h:h + 1], refR[None, None], rows, d, w.tol, what + " rho"))
            # delta = omega - mu . rho is formed by cancellation in this mode (a row that has converged has
            # delta << omega): fp32 holds it to a fraction of omega, not of delta
            Qd, Kd = Q[0, h].double().numpy(), K[0, h].double().numpy()
            omega = np.array([np.exp(w.scale * (Kd[: i + 1] @ Qd[i]) - (w.scale * (Kd[: i + 1] @ Qd[i])).max()).sum()
                              for i in rows])
            assert np.all(np.abs(Dl[0, h] - refD) <= w.tol * np.abs(refD) + 2e-4 * omega), what + " delta"


@pytest.mark.parametrize("n,d,T,eps", [(333, 64, 4, 0.0), (333, 64, 12, 0.0), (600, 64, 40, 0.0), (290, 128, 8, 0.0),
                                       (333, 64, 60, 1e-3)])
def test_forward_cg_later_steps_reduce_the_residual_like_the_oracle(n, d, T, eps):
    """What is well defined about a later CG iterate is how far it has brought the residual down.  For sampled rows
    the residual of the GPU's rho, evaluated here in fp64 from the definitions of mu_i and Sigma_i, must be within a
    small factor of the residual of the fp64 CG oracle after the same number of steps, or after two thirds of them
    (down to the floor set by the 16-bit operand splits of the matrix-free product); delta must be
    omega - mu . rho for that same rho."""
    w = _small("cg", 1, 2, n, d, "bf16", index=800 + d + n + T)
    Q, K, V = workloads.make_inputs(w)
    O, R, Dl, steps = llla.llla_forward_cg(Q.to(DEV), K.to(DEV), V.to(DEV), w.lam, w.scale, T, eps, return_stats=True)
    torch.cuda.synchronize()
    R, Dl, steps = R.cpu().numpy().astype(np.float64), Dl.cpu().numpy().astype(np.float64), steps.cpu().numpy()
    assert np.all(np.isfinite(O.cpu().numpy()))
    rows = np.unique(np.concatenate([np.arange(0, n, 17), [1, 63, 64, 65, n - 1]]))
    for h in range(2):
        Qd, Kd = Q[0, h].double().numpy(), K[0, h].double().numpy()
        _, refR, _, used = oracle.forward_head_cg(Q[0, h], K[0, h], V[0, h], w.lam, w.scale, T, eps, rows=rows)
        # rounding delays CG (loss of orthogonality): allow the GPU run to lag the fp64 run by a third of the steps
        _, lagR, _, _ = oracle.forward_head_cg(Q[0, h], K[0, h], V[0, h], w.lam, w.scale, max(1, (2 * T) // 3), eps, rows=rows)
        for t, i in enumerate(rows):
            sc = w.scale * (Kd[: i + 1] @ Qd[i])
            wg = np.exp(sc - sc.max())
            Z = Kd[: i + 1] - Qd[i]
            omega, mu = wg.sum(), (wg[:, None] * Z).sum(0)
            Sigma = (Z.T * wg) @ Z + w.lam * np.eye(d)
            nmu = max(np.linalg.norm(mu), 1e-30)
            res_gpu = np.linalg.norm(mu - Sigma @ R[0, h, i]) / nmu
            res_ref = max(np.linalg.norm(mu - Sigma @ refR[t]), np.linalg.norm(mu - Sigma @ lagR[t])) / nmu
            if eps == 0.0:
                assert res_gpu <= 4.0 * res_ref + 1e-5, (h, i, res_gpu, res_ref)
                # both run all T steps unless the residual became exactly zero (which fp32 reaches sooner)
                assert steps[0, h, i] == used[t] or (used[t] < T and steps[0, h, i] <= T) or res_gpu <= 1e-5
            else:       # frozen once the residual is at or below eps (the GPU judges it in fp32, one step of slack)
                assert res_gpu * nmu <= 4.0 * eps or steps[0, h, i] == T, (h, i, res_gpu * nmu, steps[0, h, i])
                assert int(used[t]) <= int(steps[0, h, i]) + 2 and int(steps[0, h, i]) <= (3 * int(used[t])) // 2 + 2, (h, i, steps[0, h, i], used[t])
            # delta against the definition with the GPU's own rho: fp32 cancellation scales with omega
            assert abs(Dl[0, h, i] - (omega - mu @ R[0, h, i])) <= 2e-4 * omega + 1e-6, (h, i)


@pytest.mark.parametrize("n,d,T", [(600, 64, 8), (600, 64, 16), (400, 128, 8), (400, 128, 16), (300, 32, 8), (300, 16, 8)])
def test_forward_cg_well_conditioned_iterates_match_the_cg_oracle(n, d, T):
    """The iterates at the step counts the paper has in mind (a constant number of steps), element by element against the
    fp64 CG oracle, on systems where a CG iterate is a well-defined quantity: L2-normalised queries and keys and a ridge
    of 1 keep the condition number of Sigma_i in the hundreds, so that rounding does not move the iterates.  Outputs,
    rho, delta and the step counts are compared.  A row that sees i + 1 keys has at most i + 2 distinct eigenvalues, so
    CG has converged on it (to rounding) after i + 2 steps and what later steps do is rounding noise around the
    solution: its outputs are compared like all others, its step count only has to lie between i + 1 and T."""
    lam = 1.0
    w = _small("cgw", 1, 2, n, d, "bf16", values="l2", index=860 + d + T)
    Q, K, V = workloads.make_inputs(w)
    O, R, Dl, steps = llla.llla_forward_cg(Q.to(DEV), K.to(DEV), V.to(DEV), lam, w.scale, T, 0.0, return_stats=True)
    torch.cuda.synchronize()
    O, R, Dl, steps = O.cpu().numpy(), R.cpu().numpy(), Dl.cpu().numpy(), steps.cpu().numpy()
    rows = np.arange(n)
    for h in range(2):
        refO, refR, refD, used = oracle.forward_head_cg(Q[0, h], K[0, h], V[0, h], lam, w.scale, T, 0.0)
        what = "cg well-conditioned T=%d n=%d d=%d head %d" % (T, n, d, h)
        print(check(O[0:1, h:h + 1], refO[None, None], rows, d, w.tol, what))
        # row 0 sees one key whose z = k - q carries the bf16 rounding of both; rho_0 is compared with the others
        print(check(R[0:1, h:h + 1], refR[None, None], rows, d, w.tol, what + " rho"))
        print(check(Dl[0:1, h:h + 1, :, None], refD[None, None, :, None], rows, d, w.tol, what + " delta"))
        late = rows > T
        assert np.array_equal(steps[0, h][late], used[late]) and np.all(used[late] == T), what + " steps"
        assert np.all(steps[0, h][~late] <= T) and np.all(steps[0, h][~late] >= np.minimum(rows[~late] + 1, T)), what


def test_forward_cg_zero_steps_is_softmax_attention():
    w = _small("cg0", 1, 2, 300, 64, "bf16", index=850)
    Q, K, V = workloads.make_inputs(w)
    O = llla.llla_forward_cg(Q.to(DEV), K.to(DEV), V.to(DEV), w.lam, w.scale, 0).cpu()
    ref = torch.nn.functional.scaled_dot_product_attention(Q.double(), K.double(), V.double(), is_causal=True, scale=w.scale)
    err = (O.double() - ref).norm(dim=-1) / ref.norm(dim=-1)
    assert float(err.max()) < 5e-3, float(err.max())


def test_forward_cg_many_steps_approaches_the_exact_forward():
    """With enough steps the approximate mode reaches the exact minimiser: distance to the fp64 ORACLE's exact forward
    (not to the library's own) on rows past 4d, for growing step counts."""
    w = _small("cgx", 1, 2, 400, 64, "bf16", index=851)
    Q, K, V = workloads.make_inputs(w)
    exact = oracle.forward(Q, K, V, w.lam, w.scale)[:, :, 256:]
    Qd, Kd, Vd = Q.to(DEV), K.to(DEV), V.to(DEV)
    errs = []
    for T in (2, 8, 32, 128):
        O = llla.llla_forward_cg(Qd, Kd, Vd, w.lam, w.scale, T, 1e-6).cpu().numpy()[:, :, 256:]
        errs.append(float((np.linalg.norm(O - exact, axis=-1) / np.linalg.norm(exact, axis=-1)).max()))
    print("max rel. distance to the oracle's exact forward on rows >= 256 for T = 2, 8, 32, 128:", errs)
    assert errs[-1] < 2e-2 and errs[-1] <= errs[0]


def test_f16_value_range_of_the_matrix_core_forward():
    """What include/llla.h states about values beyond the f16 range: the matrix-core kernels hand the keys to the MFMA
    units as f16, so a bf16 key entry of 1e5 becomes infinite and every row that sees that key is NaN, with no status
    (as are the rows just before it whose last 64-key block holds the key under a zero weight: 0 times infinity); rows
    whose blocks end before it are untouched and inside the gate."""
    n, d, j0 = 300, 64, 180
    w = _small("range", 1, 1, n, d, "bf16", index=1800)
    Q, K, V = workloads.make_inputs(w)
    K[0, 0, j0, 5] = 1e5
    ref = oracle.forward(Q, K, V, w.lam, w.scale)
    got = _run_forward(w, Q, K, V, path="mfma")
    clean = 64 * (j0 // 64)
    assert np.isfinite(got[0, 0, :clean]).all() and not np.isfinite(got[0, 0, j0:]).any()
    rows = np.arange(clean)
    print(check(got[:, :, :clean], ref[:, :, :clean], rows, d, w.tol, "rows before the out-of-range key's block"))
