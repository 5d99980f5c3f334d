"""Error metrics of the parity gate (shared by the GPU tests and the benchmark's self-check).

Gate, with tol = 1e-4 for fp32 inputs and 2e-2 for bf16 inputs:
  * per row, ||o_i - o*_i||_2 / ||o*_i||_2 <= tol for rows i >= 4d and <= 10*tol for rows i < 4d
    (the normal matrix of the earliest rows has rank <= i before the ridge, so their conditioning
    is worse by orders of magnitude);
  * per (batch, head), the Frobenius-relative error over the checked rows i >= 4d is <= tol, over
    the checked rows i < 4d it is <= 10*tol, and over all checked rows it is <= tol whenever at
    least half of them are late rows (every named configuration is; tiny ragged cases are not).
"""
import numpy as np


def row_errors(got, ref):
    """got, ref: [..., rows, dv].  Per-row relative L2 error."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    num = np.linalg.norm(got - ref, axis=-1)
    den = np.maximum(np.linalg.norm(ref, axis=-1), 1e-30)
    return num / den


def frobenius_error(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return np.linalg.norm((got - ref).reshape(-1)) / max(np.linalg.norm(ref.reshape(-1)), 1e-30)


def check(got, ref, rows, d, tol, what=""):
    """got, ref: [B, H, len(rows), dv]; rows: the query index of each row.  Asserts the gate and
    returns a summary dict."""
    rows = np.asarray(rows)
    assert np.all(np.isfinite(np.asarray(got, dtype=np.float64))), what + ": non-finite output"
    err = row_errors(got, ref)                                   # [B, H, R]
    early = rows < 4 * d
    bound = np.where(early, 10.0 * tol, tol)
    worst = np.unravel_index(np.argmax(err / bound), err.shape)
    summary = {
        "median": float(np.median(err)), "p99": float(np.quantile(err, 0.99)),
        "max": float(err.max()), "worst_row": int(rows[worst[-1]]),
        "worst_ratio_to_bound": float((err / bound).max()),
    }
    B, H = err.shape[:2]
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    late = ~early
    fro_all = max(frobenius_error(got[b, h], ref[b, h]) for b in range(B) for h in range(H))
    summary["frobenius_max"] = float(fro_all)
    if late.any():
        fro = max(frobenius_error(got[b, h][late], ref[b, h][late]) for b in range(B) for h in range(H))
        summary["frobenius_late"] = float(fro)
        assert fro <= tol, "%s: Frobenius error (rows >= 4d) %.3e > %.1e (%s)" % (what, fro, tol, summary)
    if early.any():
        fro = max(frobenius_error(got[b, h][early], ref[b, h][early]) for b in range(B) for h in range(H))
        summary["frobenius_early"] = float(fro)
        assert fro <= 10 * tol, "%s: Frobenius error (rows < 4d) %.3e > %.1e (%s)" % (what, fro, 10 * tol, summary)
    if late.sum() >= early.sum():
        assert fro_all <= tol, "%s: Frobenius error %.3e > %.1e (%s)" % (what, fro_all, tol, summary)
    assert np.all(err <= bound), "%s: row %d error %.3e exceeds %.1e (%s)" % (
        what, summary["worst_row"], err[worst], bound[worst[-1]], summary)
    return summary


def check_grad(got, ref, d, tol, what="", floor=0.0):
    """Gate for a gradient tensor.  got, ref: [B, H, n, c] (or [B, H, n] for per-row scalars).
    Per (batch, head): Frobenius-relative error <= tol.  Per row i: ||got_i - ref_i|| <= f * tol * (||ref_i|| + rms),
    rms = root-mean-square row norm of that head's reference (rows whose exact gradient is zero or tiny -- the first
    row's dQ, keys no sampled row sees -- have no meaningful relative error of their own), f = 10 for rows i < 4d and 1
    afterwards, as in the forward gate.  `floor`: the size of the terms a gradient is the sum of (the caller passes
    ||dO|| * rms(V) of a head); a head whose exact gradient is smaller than that -- n = 1, where dQ and dK vanish
    identically -- is measured against the floor instead of its own norm.  Returns a summary dict."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what + ": non-finite gradient"
    if got.ndim == 3:
        got, ref = got[..., None], ref[..., None]
    B, H, n = got.shape[:3]
    rown = np.linalg.norm(ref, axis=-1)                                   # [B, H, n]
    rms = np.maximum(np.sqrt(np.mean(rown ** 2, axis=-1, keepdims=True)), floor / np.sqrt(n))
    err = np.linalg.norm(got - ref, axis=-1)
    factor = np.where(np.arange(n) < 4 * d, 10.0, 1.0)
    ratio = err / (factor * tol * (rown + rms) + 1e-300)
    fro = np.array([[np.linalg.norm(got[b, h] - ref[b, h]) / max(np.linalg.norm(ref[b, h]), floor, 1e-300)
                     for h in range(H)] for b in range(B)])
    worst = np.unravel_index(np.argmax(ratio), ratio.shape)
    summary = {"frobenius_max": float(fro.max()), "worst_row": int(worst[-1]),
               "worst_row_ratio_to_bound": float(ratio.max())}
    assert fro.max() <= tol, "%s: Frobenius error %.3e > %.1e (%s)" % (what, fro.max(), tol, summary)
    assert ratio.max() <= 1.0, "%s: row %d off by %.2f x its bound (%s)" % (what, worst[-1], ratio.max(), summary)
    return summary
