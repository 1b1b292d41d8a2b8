"""Helpers of the GPU parity tests: error measures and oracle calls."""
import numpy as np
import torch

from oracle import gc_oracle as O
from paper_2101_06983_amd import synth

TOL_F32 = 1e-5    # fp32 inputs (spec tolerance)
TOL_BF16 = 2e-3   # bf16 inputs, fp32 accumulation


def relerr(got, want):
    """max |got - want| / max |want| per tensor (elementwise relative error is
    meaningless at zero crossings)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    den = np.abs(want).max()
    if den == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got - want).max() / den)


def check(label, err, tol):
    """Asserts err <= tol and prints both, so that the margin under every bound is on record
    (`pytest -rP` shows the lines of passing tests)."""
    print("parity %-44s err %.3e  tol %.3e  (%.0f %% of the bound)" % (label, err, tol, 100.0 * err / tol if tol > 0 else 0.0))
    assert err <= tol, "%s: %.4e > %.4e" % (label, err, tol)


def check_loss(label, got, want, tol, abs_floor=0.0):
    check(label, abs(float(got) - float(want)), tol * abs(float(want)) + abs_floor)


def normerr(got, want):
    """Frobenius norm of the difference over the Frobenius norm of the expected tensor."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300))


def to_np(t):
    return t.detach().cpu().to(torch.float64).numpy() if t.is_floating_point() else t.detach().cpu().numpy()


def oracle_loss(q, p, r, scale=1.0, temp=1.0, mask_self=False):
    return O.loss_and_rep_grad(synth.widen(q), synth.widen(p), synth.widen(r), scale, temp, mask_self)


def check_argmax(got, want_out, q64, p64, alpha, gap_tol):
    """Bit-exact argmax, except rows whose fp64 top-2 gap is below gap_tol (fp32
    summation order may legitimately flip those): either of the two is accepted."""
    got = np.asarray(got)
    want = want_out["argmax"]
    bad = np.nonzero(got != want)[0]
    ambiguous = 0
    for i in bad:
        s = alpha * (q64[i] @ p64.T)
        top = np.sort(s)[-2:]
        assert top[1] - top[0] < gap_tol, "row %d: argmax %d != %d with gap %g" % (i, got[i], want[i], top[1] - top[0])
        assert s[got[i]] >= top[0] - 1e-12
        ambiguous += 1
    return ambiguous
