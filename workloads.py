"""Seeded synthetic inputs for the LLA forward / decode workloads.

This module holds no arithmetic of the method: it only draws the random tensors (on the CPU, so the
same values reach both the fp64 oracle and the GPU library) and names the shapes.  The paper
benchmarks its kernel on unspecified random tensors "across a range of dimensions and batch sizes"
(Section 3.2, last paragraph) and builds its regression experiments from Gaussian keys with
linear-plus-noise values (Section 4, test-time regression); the configs below stand in for both.

Recipe: ``torch.Generator('cpu').manual_seed(20251001 + config_index)``; draw fp32 in the order
Q, K, V (then A, noise where used); apply the config's transform in fp32; cast to the config dtype.
The oracle consumes the cast values.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import torch

SEED0 = 20251001


@dataclass(frozen=True)
class Workload:
    name: str
    index: int            # seed offset
    kind: str             # "forward" or "decode"
    B: int
    H: int
    n: int                # sequence length (forward) or cache length L (decode)
    d: int
    dtype: str            # "f32" or "bf16"
    values: str           # "normal", "scaled" (Q,K * 1/sqrt(d)), "l2" (rows of Q,K normalised),
                          # "regression" (V = K A^T + 0.1 noise), "piecewise" (the piecewise-linear task:
                          # keys from one cone per segment, one linear map per segment, Q = K)
    lam: float
    scale: float
    tol: float            # relative-error bound of the parity gate
    segment: int = 0      # "piecewise" only: segment size S (n / S segments, a power of two of them)
    noise: float = 0.1    # "piecewise" only: standard deviation of the value noise

    def with_shape(self, **kw) -> "Workload":
        return replace(self, **kw)


def _w(name, index, kind, B, H, n, d, dtype, values, scale=None):
    tol = 1e-4 if dtype == "f32" else 2e-2
    scale = (1.0 / math.sqrt(d)) if scale is None else scale
    return Workload(name, index, kind, B, H, n, d, dtype, values, 1e-2, scale, tol)


# C1..C5 are the five configurations of the baseline file; C3b is the d=64, n=8192 prefill shape.
C1 = _w("C1_tiny_f32", 0, "forward", 1, 1, 128, 16, "f32", "scaled", scale=1.0)
C2 = _w("C2_f32_n1024_d64", 1, "forward", 2, 8, 1024, 64, "f32", "l2")
C3 = _w("C3_prefill_bf16_n4096_d64", 2, "forward", 4, 16, 4096, 64, "bf16", "normal")
C3B = _w("C3b_prefill_bf16_n8192_d64", 5, "forward", 2, 16, 8192, 64, "bf16", "normal")
C4 = _w("C4_longctx_bf16_n8192_d128", 3, "forward", 1, 16, 8192, 128, "bf16", "regression")
C5 = _w("C5_decode_bf16_L32768_d64", 4, "decode", 32, 16, 32768, 64, "bf16", "normal")
# the decode shape at head dimension 128 with the same cache bytes as C5 (half the sequences)
C5D128 = _w("C5d128_decode_bf16_L32768_d128", 8, "decode", 16, 16, 32768, 128, "bf16", "normal")
# the prefill shape at head dimension 32 (served by the d = 64 matrix-core kernels on zero-padded copies)
C3D32 = _w("C3d32_prefill_bf16_n4096_d32", 9, "forward", 4, 16, 4096, 32, "bf16", "normal")
# a small-batch decode step: one sequence, 16 heads, 4096 cached keys (bound by the kernels' latency, not by the stream)
C5S = _w("C5s_decode_bf16_L4096_d64", 10, "decode", 1, 16, 4096, 64, "bf16", "normal")
# E2: the paper's test-time regression task (Section 4 and Appendix "Experiments": L = 1024, d = 64, S = 256), one
# sequence per batch entry; E2S is the same task at a size the oracle finishes in seconds.
E2 = replace(_w("E2_piecewise_bf16_L1024_d64", 6, "forward", 1024, 1, 1024, 64, "bf16", "piecewise"), segment=256)
E2S = replace(_w("E2s_piecewise_f32_L256_d16", 7, "forward", 8, 1, 256, 16, "f32", "piecewise"), segment=32)
ALL = {w.name.split("_")[0].upper(): w for w in (C1, C2, C3, C3B, C3D32, C4, C5, C5S, C5D128, E2, E2S)}


def torch_dtype(w: Workload):
    return torch.float32 if w.dtype == "f32" else torch.bfloat16


def cone_signs(n_segments: int) -> torch.Tensor:
    """[n_segments, m] matrix of +-1, m = log2(n_segments): row c holds the m least-significant bits of c
    (bit j set -> +1), the sign pattern of segment c's cone (Appendix "Piecewise Linear Data Generation")."""
    m = n_segments.bit_length() - 1
    if n_segments < 1 or (1 << m) != n_segments:
        raise ValueError("the number of segments must be a power of two")
    c = torch.arange(n_segments).unsqueeze(1)
    return (((c >> torch.arange(m).unsqueeze(0)) & 1) * 2 - 1).to(torch.float32).reshape(n_segments, m)


def piecewise_linear(w: Workload):
    """The piecewise-linear regression task: every (batch, head) entry is one length-n sequence cut into n / S
    segments; segment c draws Gaussian keys whose first m coordinates carry the cone's signs, and its values are
    A_c k + noise with a Gaussian matrix A_c of its own.  The query at a position is that position's key.
    Draw order: Z, A, noise.  Keys are cast to the workload dtype BEFORE the maps are applied, so the linear
    relation holds for the stored keys.  Returns (Q, K, V, A, segment index of every position)."""
    S = w.segment
    if S <= 0 or w.n % S:
        raise ValueError("segment size must divide the sequence length")
    nseg = w.n // S
    signs = cone_signs(nseg)
    m = signs.shape[1]
    if m > w.d:
        raise ValueError("more sign coordinates than dimensions")
    g = torch.Generator(device="cpu").manual_seed(SEED0 + w.index)
    Z = torch.randn((w.B, w.H, w.n, w.d), generator=g, dtype=torch.float32)
    A = torch.randn((w.B, w.H, nseg, w.d, w.d), generator=g, dtype=torch.float32)
    E = torch.randn((w.B, w.H, w.n, w.d), generator=g, dtype=torch.float32)
    seg = torch.arange(w.n) // S
    K = Z.clone()
    K[..., :m] = Z[..., :m].abs() * signs[seg]
    dt = torch_dtype(w)
    K = K.to(dt)
    Kseg = K.float().reshape(w.B, w.H, nseg, S, w.d)
    V = torch.matmul(Kseg, A.transpose(-1, -2)).reshape(w.B, w.H, w.n, w.d) + w.noise * E
    return K.clone(), K, V.to(dt), A, seg


def make_inputs(w: Workload):
    """Returns CPU tensors in the workload dtype.
    forward: (Q, K, V) each [B, H, n, d].   decode: (q [B, H, d], Kc, Vc [B, H, n, d])."""
    if w.values == "piecewise":
        return piecewise_linear(w)[:3]
    g = torch.Generator(device="cpu").manual_seed(SEED0 + w.index)
    shape = (w.B, w.H, w.n, w.d)
    qshape = shape if w.kind == "forward" else (w.B, w.H, w.d)
    Q = torch.randn(qshape, generator=g, dtype=torch.float32)
    K = torch.randn(shape, generator=g, dtype=torch.float32)
    V = torch.randn(shape, generator=g, dtype=torch.float32)
    if w.values == "scaled":
        Q = Q / math.sqrt(w.d)
        K = K / math.sqrt(w.d)
    elif w.values == "l2":
        Q = Q / Q.norm(dim=-1, keepdim=True)
        K = K / K.norm(dim=-1, keepdim=True)
    elif w.values == "regression":
        # per-head random map A with entries N(0, 1/d): Var(A k) = 1, so 0.1 noise is a 10 % term
        A = torch.randn((w.B, w.H, w.d, w.d), generator=g, dtype=torch.float32) / math.sqrt(w.d)
        V = torch.matmul(K, A.transpose(-1, -2)) + 0.1 * V
    elif w.values != "normal":
        raise ValueError(w.values)
    dt = torch_dtype(w)
    return Q.to(dt), K.to(dt), V.to(dt)


def sample_rows(w: Workload, n_random: int = 96):
    """Rows checked one by one against the oracle when the full output is too expensive:
    0..4d, every multiple of 64 (hence of 128 and 256: the tile boundaries of every kernel) with both
    neighbours, n_random uniform rows, the last."""
    n, d = w.n, w.d
    rows = set(range(min(n, 4 * d + 1)))
    for r in range(64, n, 64):
        rows.update(x for x in (r - 1, r, r + 1) if 0 <= x < n)
    g = torch.Generator(device="cpu").manual_seed(SEED0 + 1000 + w.index)
    rows.update(int(x) for x in torch.randint(0, n, (n_random,), generator=g))
    rows.add(n - 1)
    return sorted(rows)
