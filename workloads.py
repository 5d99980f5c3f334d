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
                          # "regression" (V = K A^T + 0.1 noise)
    lam: float
    scale: float
    tol: float            # relative-error bound of the parity gate

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
ALL = {w.name.split("_")[0]: w for w in (C1, C2, C3, C3B, C4, C5)}


def torch_dtype(w: Workload):
    return torch.float32 if w.dtype == "f32" else torch.bfloat16


def make_inputs(w: Workload):
    """Returns CPU tensors in the workload dtype.
    forward: (Q, K, V) each [B, H, n, d].   decode: (q [B, H, d], Kc, Vc [B, H, n, d])."""
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


def sample_rows(w: Workload, n_random: int = 256):
    """Rows checked one by one against the oracle when the full output is too expensive:
    0..4d, every multiple of 64/128/256 with both neighbours, n_random uniform rows, the last."""
    n, d = w.n, w.d
    rows = set(range(min(n, 4 * d + 1)))
    for step in (64, 128, 256):
        for r in range(step, n, step * 8):
            rows.update(x for x in (r - 1, r, r + 1) if 0 <= x < n)
    g = torch.Generator(device="cpu").manual_seed(SEED0 + 1000 + w.index)
    rows.update(int(x) for x in torch.randint(0, n, (n_random,), generator=g))
    rows.add(n - 1)
    return sorted(rows)
