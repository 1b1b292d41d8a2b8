"""GPU parity of the symmetric (anchors->targets and targets->anchors) loss entry point
against the fp64 oracle; calls go through the C ABI."""
import math

import numpy as np
import pytest
import torch

from oracle import gc_oracle as O
from paper_2101_06983_amd import binding as gc
from paper_2101_06983_amd import synth
from parity import TOL_BF16, check, check_loss, relerr, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def problem(n, d, seed, mix=0.5):
    rng = np.random.default_rng(seed)
    r = torch.from_numpy(rng.permutation(n).astype(np.int32))
    q, p, _ = synth.dpr_batch(n, n, d, seed=seed, positive_mix=mix, pos_idx=r)
    return q, p, r


def run(q, p, r, scale, temp):
    out = gc.gc_bidirectional_loss_and_rep_grad_bf16(q.to(DEV), p.to(DEV), r.to(DEV), scale, temp)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("n,d,scale,temp,tol", [(96, 128, 1.0, 0.5, TOL_BF16), (300, 256, 2.0, 1.0, TOL_BF16),
                                                (257, 64, 1.0, 0.1, TOL_BF16), (1024, 768, 1.0, 1.0, TOL_BF16),
                                                (1500, 128, 1.0, 0.07, TOL_BF16),
                                                (1500, 256, 1.0, 0.07, TOL_BF16),
                                                (200, 384, 1.0, 1.0, TOL_BF16), (333, 512, 1.5, 0.5, TOL_BF16),
                                                (130, 640, 1.0, 0.2, TOL_BF16), (64, 96, 1.0, 1.0, TOL_BF16)])
def test_bidirectional_matches_the_oracle(n, d, scale, temp, tol):
    q, p, r = problem(n, d, 6000 + n)
    q64, p64 = synth.widen(q), synth.widen(p)
    want = O.bidirectional(q64, p64, r.numpy(), scale, temp)
    out = run(q, p, r, scale, temp)
    tag = "bidir n=%d d=%d" % (n, d)
    check_loss(tag + " loss", out["loss"].item(), want["loss"], 1e-5)     # the loss has no bf16 step
    for k in ("dq", "dp"):
        if d % 128 == 0:     # MFMA kernels: bf16 coefficients
            check(tag + " " + k, relerr(to_np(out[k]), want[k]), tol)
        else:                # fp32-FMA kernels: nothing is rounded to bf16
            check(tag + " " + k, relerr(to_np(out[k]), want[k]), 1e-5)


def test_bidirectional_at_the_benchmark_size():
    """n = 8192, d = 768 (the shape `bench.py --workload bidir` times): every output against the oracle."""
    n, d = 8192, 768
    q, p, r = problem(n, d, 6400)
    want = O.bidirectional(synth.widen(q), synth.widen(p), r.numpy(), 1.0, 1.0)
    out = run(q, p, r, 1.0, 1.0)
    check_loss("bidir n=8192 loss", out["loss"].item(), want["loss"], 1e-5)
    for k in ("dq", "dp"):
        check("bidir n=8192 " + k, relerr(to_np(out[k]), want[k]), TOL_BF16)
    # Euler identity: sum_i <q_i, dq_i> = sum_j <p_j, dp_j> (both are (alpha/n) sum_ij g_ij <q_i, p_j>)
    a = float((synth.widen(q) * to_np(out["dq"])).sum()), float((synth.widen(p) * to_np(out["dp"])).sum())
    assert abs(a[0] - a[1]) <= 1e-3 * max(abs(a[0]), abs(a[1]), 1e-6)


def test_bidirectional_with_equal_sides_is_twice_symmetric():
    """With q == p and the identity pairing the two directions are the same problem:
    the loss equals the one-direction loss and dq == dp (each the sum of Eq. 5 and Eq. 6, halved)."""
    n, d = 384, 128
    q, _, _ = problem(n, d, 6100)
    r = torch.arange(n, dtype=torch.int32)
    out = run(q, q, r, 1.0, 1.0)
    one = O.loss_and_rep_grad(synth.widen(q), synth.widen(q), r.numpy())
    assert abs(out["loss"].item() - one["loss"]) <= TOL_BF16 * abs(one["loss"])
    assert relerr(to_np(out["dq"]), 0.5 * (one["dq"] + one["dp"])) <= TOL_BF16
    assert torch.equal(out["dq"], out["dp"])


def test_repeat_is_bitwise_and_reuses_buffers():
    q, p, r = problem(640, 256, 6200)
    qd, pd, rd = q.to(DEV), p.to(DEV), r.to(DEV)
    ws = gc.alloc_workspace(gc.load().gc_bidirectional_workspace_bytes(640, 256), DEV)
    a = gc.gc_bidirectional_loss_and_rep_grad_bf16(qd, pd, rd, 1.0, 0.2, ws)
    keep = {k: v.clone() for k, v in a.items()}
    b = gc.gc_bidirectional_loss_and_rep_grad_bf16(qd, pd, rd, 1.0, 0.2, ws, out=a)
    torch.cuda.synchronize()
    assert gc.gc_check_async_error(ws) == gc.GC_OK
    for k in ("loss", "dq", "dp"):
        assert torch.equal(keep[k], b[k])


def test_a_pairing_that_is_no_bijection_is_reported():
    q, p, r = problem(200, 128, 6300)
    r = r.clone()
    r[7] = r[8]                      # in range, but one target is named twice and one never
    qd, pd, rd = q.to(DEV), p.to(DEV), r.to(DEV)
    ws = gc.alloc_workspace(gc.load().gc_bidirectional_workspace_bytes(200, 128), DEV)
    out = gc.gc_bidirectional_loss_and_rep_grad_bf16(qd, pd, rd, 1.0, 1.0, ws)
    torch.cuda.synchronize()
    assert math.isnan(out["loss"].item())
    assert gc.gc_check_async_error(ws) == gc.GC_ERR_POS_IDX
    r[8] = 200                       # out of range
    out = gc.gc_bidirectional_loss_and_rep_grad_bf16(qd, pd, r.to(DEV), 1.0, 1.0, ws)
    torch.cuda.synchronize()
    assert math.isnan(out["loss"].item())
    assert gc.gc_check_async_error(ws) == gc.GC_ERR_POS_IDX
