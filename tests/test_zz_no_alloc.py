"""GPU test of the entry point that allocates nothing (gc_loss_and_rep_grad_bf16_static): its output against the
allocating entry point's (gc_loss_and_rep_grad_bf16; same kernels, so bit for bit) and against the oracle, on two
calls in a row, the second with a smaller input (the static array then still holds the first call's contents)."""
import math

import pytest
import torch

from paper_2101_06983_amd import binding as gc
from paper_2101_06983_amd import synth
from parity import TOL_BF16, check, check_loss, oracle_loss, relerr, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def one_call(B, P, d, seed, temp):
    q, p, r = synth.dpr_batch(B, P, d, seed=seed, positive_mix=0.3)
    qd, pd, rd = q.to(DEV), p.to(DEV), r.to(DEV)
    out = (torch.empty(1, dtype=torch.float32, device=DEV), torch.empty(B, d, dtype=torch.float32, device=DEV),
           torch.empty(P, d, dtype=torch.float32, device=DEV))
    loss, dq, dp = gc.gc_loss_and_rep_grad_bf16_static(qd, pd, rd, 1.0, temp, out=out)
    torch.cuda.synchronize()
    assert gc.gc_check_async_error() == gc.GC_OK
    ref_loss, ref_dq, ref_dp = gc.gc_loss_and_rep_grad_bf16(qd, pd, rd, 1.0, temp)
    torch.cuda.synchronize()
    assert loss.item() == ref_loss.item()
    assert torch.equal(dq, ref_dq) and torch.equal(dp, ref_dp)
    want = oracle_loss(q, p, r, 1.0, temp)
    tag = "static %dx%dx%d" % (B, P, d)
    check_loss(tag + " loss", loss.item(), want["loss"], TOL_BF16)
    check(tag + " dq", relerr(to_np(dq), want["dq"]), TOL_BF16)
    check(tag + " dp", relerr(to_np(dp), want["dp"]), TOL_BF16)


def test_static_scratch_entry_point_two_calls_in_a_row():
    one_call(512, 1024, 768, 9100, 1.0)      # config 5's loss shape: split partials of both outputs in the scratch
    one_call(130, 257, 256, 9101, 0.5)       # smaller, ragged: the array still holds the first call's contents
    one_call(512, 1024, 768, 9100, 1.0)      # and the large one again


def test_static_scratch_rejects_what_does_not_fit_and_reports_bad_positives():
    lib = gc.load()
    assert lib.gc_workspace_bytes(4096, 8192, 768, gc.GC_BF16) > gc.GC_STATIC_SCRATCH_BYTES
    q, p, r = synth.dpr_batch(64, 128, 128, seed=9102)
    qd, pd, rd = q.to(DEV), p.to(DEV), r.to(DEV)
    big = torch.empty(1, dtype=torch.bfloat16, device=DEV)
    # sizes beyond the array: rejected on the host, nothing enqueued (the pointers are never touched)
    rc = lib.gc_loss_and_rep_grad_bf16_static(big.data_ptr(), big.data_ptr(), rd.data_ptr(), 4096, 8192, 768, 1.0, 1.0,
                                              big.data_ptr(), big.data_ptr(), big.data_ptr(), None)
    assert rc == gc.GC_ERR_TOO_LARGE and "static" in gc.strerror(rc)
    r2 = r.clone()
    r2[3] = 128
    loss, _, _ = gc.gc_loss_and_rep_grad_bf16_static(qd, pd, r2.to(DEV))
    torch.cuda.synchronize()
    assert math.isnan(loss.item())
    assert gc.gc_check_async_error() == gc.GC_ERR_POS_IDX
    loss, _, _ = gc.gc_loss_and_rep_grad_bf16_static(qd, pd, rd)
    torch.cuda.synchronize()
    assert math.isfinite(loss.item()) and gc.gc_check_async_error() == gc.GC_OK
