"""GPU parity of the loss / representation-gradient path against the fp64 oracle.
Every call goes through the C ABI (ctypes binding)."""
import math

import numpy as np
import pytest
import torch

from paper_2101_06983_amd import binding as gc
from paper_2101_06983_amd import synth
from oracle import gc_oracle as O
from parity import TOL_BF16, TOL_F32, check, check_argmax, check_loss, oracle_loss, relerr, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


# the two kernel sequences of the bf16 MFMA shapes from d = 256 (the flag is ignored where only one exists)
PATHS = [gc.GC_PATH_ONLINE, gc.GC_PATH_STATS_PASS]


def run_ex(q, p, r, scale=1.0, temp=1.0, flags=0):
    out = gc.gc_loss_and_rep_grad_ex(q.to(DEV), p.to(DEV), r.to(DEV), scale, temp, flags)
    torch.cuda.synchronize()
    assert gc.gc_check_async_error(out["workspace"]) == gc.GC_OK
    return out


def compare(out, want, tol, q=None, p=None, alpha=1.0, gap_tol=1e-5, label=""):
    check_loss(label + " loss", out["loss"].item(), want["loss"], tol, 1e-30)
    check(label + " dq", relerr(to_np(out["dq"]), want["dq"]), tol)
    check(label + " dp", relerr(to_np(out["dp"]), want["dp"]), tol)
    check(label + " lse", relerr(to_np(out["lse"]), want["lse"]), tol)
    amb = check_argmax(to_np(out["argmax"]), want, synth.widen(q), synth.widen(p), alpha, gap_tol)
    assert amb <= max(1, len(want["argmax"]) // 1000)


def test_config1_tiny_fp32():
    q, p, r = synth.config1()
    want = oracle_loss(q, p, r)
    import json
    import os
    gold = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "config1_oracle.json")))
    assert abs(want["loss"] - gold["loss"]) < 1e-12   # the stored oracle values are the ones compared against
    loss, dq, dp = gc.gc_loss_and_rep_grad_f32(q.to(DEV), p.to(DEV), r.to(DEV))
    torch.cuda.synchronize()
    assert gc.gc_check_async_error() == gc.GC_OK
    check_loss("config1 loss", loss.item(), want["loss"], TOL_F32)
    check("config1 dq", relerr(to_np(dq), want["dq"]), TOL_F32)
    check("config1 dp", relerr(to_np(dp), want["dp"]), TOL_F32)
    compare(run_ex(q, p, r), want, TOL_F32, q, p, label="config1 ex")


@pytest.mark.parametrize("B,P,d,scale,temp", [(37, 53, 20, 1.0, 1.0), (1, 1, 7, 1.0, 1.0), (1, 40, 64, 2.0, 0.5),
                                              (130, 70, 33, 1.0, 0.1), (16, 16, 128, 1.0, 1.0)])
def test_fp32_general_shapes(B, P, d, scale, temp):
    q, p, r = synth.dpr_batch(B, P, d, torch.float32, seed=1000 + B)
    g = np.random.default_rng(B)
    r = torch.from_numpy(g.integers(0, P, size=B).astype(np.int32))   # shared positives, unused targets
    want = oracle_loss(q, p, r, scale, temp)
    compare(run_ex(q, p, r, scale, temp), want, TOL_F32, q, p, scale / temp, label="fp32 %dx%dx%d" % (B, P, d))


def test_config2_dpr_shaped_bf16():
    q, p, r = synth.config2()
    want = oracle_loss(q, p, r)
    assert 4.9 < want["loss"] < 5.2
    loss, dq, dp = gc.gc_loss_and_rep_grad_bf16(q.to(DEV), p.to(DEV), r.to(DEV))
    torch.cuda.synchronize()
    check_loss("config2 loss", loss.item(), want["loss"], TOL_BF16)
    check("config2 dq", relerr(to_np(dq), want["dq"]), TOL_BF16)
    check("config2 dp", relerr(to_np(dp), want["dp"]), TOL_BF16)
    compare(run_ex(q, p, r), want, TOL_BF16, q, p, label="config2 ex")


@pytest.mark.parametrize("B,P,d,scale,temp", [
    (100, 300, 128, 1.0, 1.0),     # ragged in both directions, several stream tiles
    (65, 257, 256, 1.0, 0.5),      # one row past a tile edge
    (1, 1, 128, 1.0, 1.0),         # closed form: loss 0, gradients 0
    (1, 1000, 384, 3.0, 1.0),
    (300, 31, 512, 1.0, 1.0),      # fewer targets than one stream tile
    (257, 513, 768, 1.0, 0.25),
    (600, 1100, 128, 1.0, 0.2),    # d = 128 kernel: several 256-row owner blocks, ragged owner and stream ends
    (257, 64, 128, 2.0, 1.0),      # d = 128: one row past an owner block, two stream tiles
    (2048, 4096, 128, 1.0, 1.0),   # d = 128: long streams, split partials
    (1030, 16390, 384, 1.0, 0.5),  # several splits of a long ragged stream, a ragged last owner block, on both sequences
    (64, 96, 96, 1.0, 1.0),        # d not a multiple of 128: general kernel on bf16 storage
    (20, 50, 8, 1.0, 1.0),
])
def test_bf16_shapes_and_edges(B, P, d, scale, temp):
    q, p, _ = synth.dpr_batch(B, P, d, torch.bfloat16, seed=2000 + B + P)
    g = np.random.default_rng(B + P)
    r = torch.from_numpy(g.integers(0, P, size=B).astype(np.int32))
    want = oracle_loss(q, p, r, scale, temp)
    for path in PATHS:
        out = run_ex(q, p, r, scale, temp, flags=path)
        if P == 1:
            assert out["loss"].item() == 0.0
            assert float(out["dq"].abs().max()) == 0.0 and float(out["dp"].abs().max()) == 0.0
        tag = "bf16 %dx%dx%d path %d" % (B, P, d, path)
        compare(out, want, TOL_BF16, q, p, scale / temp, label=tag)


@pytest.mark.parametrize("B,P,d,temp", [(700, 1400, 128, 0.07), (500, 1000, 256, 0.05), (384, 2000, 768, 0.05)])
def test_peaked_softmax_at_low_temperature(B, P, d, temp):
    """Strong positives and a low temperature: a few coefficients carry each gradient row.  The largest of them, the
    positive's own, is kept in fp32 (it is not part of the bf16 contractions), so these cases meet the stated
    tolerance like any other."""
    q, p, r = synth.dpr_batch(B, P, d, torch.bfloat16, seed=2500 + B, positive_mix=0.5)
    q64, p64 = synth.widen(q), synth.widen(p)
    want = O.loss_and_rep_grad(q64, p64, r.numpy(), 1.0, temp)
    for path in PATHS:
        out = run_ex(q, p, r, 1.0, temp, flags=path)
        tag = "peaked %dx%dx%d path %d" % (B, P, d, path)
        check_loss(tag + " loss", out["loss"].item(), want["loss"], 1e-5)
        check(tag + " lse", relerr(to_np(out["lse"]), want["lse"]), 1e-5)
        for k in ("dq", "dp"):
            check(tag + " " + k, relerr(to_np(out[k]), want[k]), TOL_BF16)


@pytest.mark.parametrize("B,P,d,dtype", [(200, 700, 256, torch.bfloat16), (90, 300, 768, torch.bfloat16),
                                         (64, 200, 128, torch.bfloat16), (40, 90, 48, torch.float32)])
@pytest.mark.parametrize("path", PATHS)
def test_very_large_logits_neither_overflow_nor_vanish(B, P, d, dtype, path):
    """Logits of 200 to 400 (scale 400 on unit-norm rows): every exponent the kernels form is <= 0, so nothing
    overflows, and each row's largest term is 1, so no row sum vanishes; the softmax is one-hot up to fp32."""
    q, p, r = synth.dpr_batch(B, P, d, dtype, seed=2700 + B, positive_mix=0.6)
    scale = 400.0
    q64, p64 = synth.widen(q), synth.widen(p)
    want = O.loss_and_rep_grad(q64, p64, r.numpy(), scale, 1.0)
    assert np.abs(scale * q64 @ p64.T).max() > 200.0
    out = run_ex(q, p, r, scale, 1.0, flags=path)
    for k in ("loss", "dq", "dp", "lse"):
        assert torch.isfinite(out[k]).all(), k
    assert abs(out["loss"].item() - want["loss"]) <= 1e-4 * abs(want["loss"])
    assert relerr(to_np(out["lse"]), want["lse"]) <= 1e-5
    # The softmax is saturated here (g_ij is 0 or -1 + 1 up to 1e-40), so the true gradients are next to nothing and
    # a relative error says nothing.  What the arithmetic fixes is the absolute error of a coefficient: t and lse2
    # are fp32 numbers of size |logit| log2(e), so 2^(t - lse2) near 1 is off by about ln2 (ulp(t) + ulp(lse2)) <=
    # 4 * 2^-24 |t|, on top of the bf16 rounding of g; a gradient row is (alpha/B) sum_j g_ij p_j.
    t_max = np.abs(scale * q64 @ p64.T).max() * math.log2(math.e)
    g_err = (2.0 ** -8 if dtype == torch.bfloat16 else 0.0) * 1e-3 + 4 * 2.0 ** -24 * t_max
    assert np.abs(to_np(out["dq"]) - want["dq"]).max() <= scale / B * np.abs(p64).max() * g_err * 4
    assert np.abs(to_np(out["dp"]) - want["dp"]).max() <= scale / B * np.abs(q64).max() * g_err * 4
    assert np.array_equal(to_np(out["argmax"]), want["argmax"])


@pytest.mark.parametrize("order", ["rising", "falling"])
@pytest.mark.parametrize("B,P,d", [(200, 2000, 256), (70, 3000, 768)])
@pytest.mark.parametrize("path", PATHS)
def test_scores_that_rise_or_fall_along_the_stream(B, P, d, order, path):
    """Logits that grow steadily along the targets (about 7 in base 2 per 16-row tile, 600 in all): the walk that
    forms the statistics as it goes has to raise its per-row reference, and rescale what it has accumulated, every
    few tiles; falling, it keeps the first reference and most later terms underflow to nothing."""
    g = np.random.default_rng(2800 + B)
    u = g.standard_normal(d) / np.sqrt(d)
    ramp = np.linspace(0.0, 1.0, P) if order == "rising" else np.linspace(1.0, 0.0, P)
    q = torch.tensor(u[None, :] + 0.05 * g.standard_normal((B, d)) / np.sqrt(d), dtype=torch.float32).to(torch.bfloat16)
    p = torch.tensor(ramp[:, None] * u[None, :] + 0.05 * g.standard_normal((P, d)) / np.sqrt(d), dtype=torch.float32).to(torch.bfloat16)
    r = torch.from_numpy(g.integers(0, P, size=B).astype(np.int32))
    scale = 600.0
    q64, p64 = synth.widen(q), synth.widen(p)
    want = O.loss_and_rep_grad(q64, p64, r.numpy(), scale, 1.0)
    out = run_ex(q, p, r, scale, 1.0, flags=path)
    for k in ("loss", "dq", "dp", "lse"):
        assert torch.isfinite(out[k]).all(), k
    assert abs(out["loss"].item() - want["loss"]) <= 1e-4 * abs(want["loss"])
    assert relerr(to_np(out["lse"]), want["lse"]) <= 1e-5
    t_max = np.abs(scale * q64 @ p64.T).max() * math.log2(math.e)
    g_err = 2.0 ** -8 + 4 * 2.0 ** -24 * t_max            # bf16 coefficient + fp32 exponent, see the large-logit test
    assert np.abs(to_np(out["dq"]) - want["dq"]).max() <= scale / B * np.abs(p64).max() * g_err * 4
    # every anchor's softmax sits on the same few targets here, so a row of dP sums B coefficients of size 1: their
    # errors add like a random walk
    assert np.abs(to_np(out["dp"]) - want["dp"]).max() <= scale / B * np.abs(q64).max() * g_err * 4 * math.sqrt(B)
    amb = check_argmax(to_np(out["argmax"]), want, q64, p64, scale, 1e-3)
    assert amb <= 2


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("B,P,d", [(128, 256, 768), (300, 1000, 128), (65, 257, 256), (1024, 16384, 384)])
def test_cache_in_bf16(B, P, d, path):
    """GC_CACHE_BF16: dq, dp are the fp32 results rounded to nearest even, bit for bit, on either kernel sequence
    (the last shape is one where the library itself picks the online walk and where both outputs have split partials)."""
    q, p, _ = synth.dpr_batch(B, P, d, seed=2900 + B, positive_mix=0.3)
    r = torch.from_numpy(np.random.default_rng(B).integers(0, P, size=B).astype(np.int32))
    f32 = run_ex(q, p, r, 1.0, 0.5, flags=path)
    b16 = run_ex(q, p, r, 1.0, 0.5, flags=path | gc.GC_CACHE_BF16)
    assert b16["dq"].dtype == torch.bfloat16 and b16["dp"].dtype == torch.bfloat16
    assert b16["loss"].item() == f32["loss"].item()
    assert torch.equal(b16["dq"], f32["dq"].to(torch.bfloat16))
    assert torch.equal(b16["dp"], f32["dp"].to(torch.bfloat16))
    want = oracle_loss(q, p, r, 1.0, 0.5)
    check("bf16 cache dq", relerr(to_np(b16["dq"].float()), want["dq"]), TOL_BF16 + 2.0 ** -8)
    check("bf16 cache dp", relerr(to_np(b16["dp"].float()), want["dp"]), TOL_BF16 + 2.0 ** -8)


def test_cache_in_bf16_needs_the_mfma_shapes():
    q, p, r = synth.dpr_batch(20, 40, 96, seed=2950)
    with pytest.raises(gc.GradCacheError):
        gc.gc_loss_and_rep_grad_ex(q.to(DEV), p.to(DEV), r.to(DEV), flags=gc.GC_CACHE_BF16)
    q, p, r = synth.dpr_batch(20, 40, 128, torch.float32, seed=2951)
    with pytest.raises(gc.GradCacheError):
        gc.gc_loss_and_rep_grad_ex(q.to(DEV), p.to(DEV), r.to(DEV), flags=gc.GC_CACHE_BF16)


@pytest.mark.parametrize("n,d,dtype", [(96, 128, torch.bfloat16), (70, 24, torch.float32), (322, 256, torch.bfloat16)])
def test_mask_self(n, d, dtype):
    q, p, _ = synth.dpr_batch(n, n, d, dtype, seed=3000 + n)
    r = torch.arange(n, dtype=torch.int32) ^ 1
    want = oracle_loss(q, p, r, 1.0, 0.5, mask_self=True)
    for path in PATHS:
        out = run_ex(q, p, r, 1.0, 0.5, flags=gc.GC_MASK_SELF | path)
        compare(out, want, TOL_BF16 if dtype == torch.bfloat16 else TOL_F32, q, p, 2.0, label="mask_self n=%d d=%d path %d" % (n, d, path))


@pytest.mark.parametrize("n,d,dtype", [(96, 128, torch.bfloat16), (70, 24, torch.float32), (322, 256, torch.bfloat16),
                                       (200, 768, torch.bfloat16)])
def test_mask_self_with_a_positive_on_the_diagonal_gives_an_infinite_loss(n, d, dtype):
    """Eq. 1 with s_ii = -inf and r_i = i for one anchor: that anchor's positive logit is -inf, so the loss is
    +inf (as in the oracle), never a stale or unmasked value; the other rows' statistics are unaffected."""
    q, p, _ = synth.dpr_batch(n, n, d, dtype, seed=3100 + n)
    r = torch.arange(n, dtype=torch.int32) ^ 1
    r[5] = 5
    want = oracle_loss(q, p, r, 1.0, 0.5, mask_self=True)
    assert want["loss"] == math.inf
    for path in PATHS:
        out = run_ex(q, p, r, 1.0, 0.5, flags=gc.GC_MASK_SELF | path)
        assert out["loss"].item() == math.inf, path
        check("diagonal positive n=%d path %d lse" % (n, path), relerr(to_np(out["lse"]), want["lse"]),
              TOL_BF16 if dtype == torch.bfloat16 else TOL_F32)


def test_optional_outputs_and_reuse_of_workspace():
    """Asking for fewer outputs changes which kernels run (with dQ the statistics come from the dQ walk itself,
    without it from the statistics pass), so across such calls the results agree to fp32 rounding, not bit for bit;
    the same call twice does."""
    q, p, r = synth.config2()
    qd, pd, rd = q.to(DEV), p.to(DEV), r.to(DEV)
    full = gc.gc_loss_and_rep_grad_ex(qd, pd, rd, flags=gc.GC_PATH_ONLINE)
    only = gc.gc_loss_and_rep_grad_ex(qd, pd, rd, want=("loss",), workspace=full["workspace"])
    torch.cuda.synchronize()
    assert abs(only["loss"].item() - full["loss"].item()) <= 1e-6 * abs(full["loss"].item())
    only_dp = gc.gc_loss_and_rep_grad_ex(qd, pd, rd, want=("dp",), workspace=full["workspace"])
    again_dp = gc.gc_loss_and_rep_grad_ex(qd, pd, rd, want=("dp",), workspace=full["workspace"])
    only_dq = gc.gc_loss_and_rep_grad_ex(qd, pd, rd, flags=gc.GC_PATH_ONLINE, want=("loss", "dq"), workspace=full["workspace"])
    torch.cuda.synchronize()
    assert relerr(to_np(only_dp["dp"]), to_np(full["dp"])) <= 1e-5
    assert torch.equal(only_dp["dp"], again_dp["dp"])
    assert torch.equal(only_dq["dq"], full["dq"]) and only_dq["loss"].item() == full["loss"].item()


def test_calls_on_two_streams_that_share_the_library_buffer_are_ordered():
    # the entry points without a workspace argument share one buffer per device; calls on different streams are put in
    # order by the library (an event behind each call), so each still gets its own result
    cases = []
    for k in range(6):
        q, p, r = synth.dpr_batch(512 + 64 * k, 1024, 256, seed=9100 + k)
        cases.append((q.to(DEV), p.to(DEV), r.to(DEV)))
    want = [gc.gc_loss_and_rep_grad_ex(q, p, r, want=("loss", "dq", "dp")) for q, p, r in cases]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    got = [gc.gc_loss_and_rep_grad_bf16(q, p, r, stream=streams[k % 2]) for k, (q, p, r) in enumerate(cases)]
    torch.cuda.synchronize()
    assert gc.gc_check_async_error(None) == gc.GC_OK
    for k, ((loss, dq, dp), w) in enumerate(zip(got, want)):
        assert loss.item() == w["loss"].item(), k
        assert torch.equal(dq, w["dq"]) and torch.equal(dp, w["dp"]), k


@pytest.mark.parametrize("path", PATHS)
def test_pos_idx_out_of_range_is_reported_not_faulted(path):
    q, p, r = synth.config2()
    r = r.clone()
    r[5] = 256          # == P
    out = gc.gc_loss_and_rep_grad_ex(q.to(DEV), p.to(DEV), r.to(DEV), flags=path, want=("loss", "dq", "dp"))
    torch.cuda.synchronize()
    assert gc.gc_check_async_error(out["workspace"]) == gc.GC_ERR_POS_IDX
    assert math.isnan(out["loss"].item())
    r[5] = -3
    out = gc.gc_loss_and_rep_grad_ex(q.to(DEV), p.to(DEV), r.to(DEV), flags=path, want=("loss", "dq"), workspace=out["workspace"])
    torch.cuda.synchronize()
    assert gc.gc_check_async_error(out["workspace"]) == gc.GC_ERR_POS_IDX
    r[5] = 7            # and the error word clears again
    out = gc.gc_loss_and_rep_grad_ex(q.to(DEV), p.to(DEV), r.to(DEV), flags=path, want=("loss", "dq"), workspace=out["workspace"])
    torch.cuda.synchronize()
    assert gc.gc_check_async_error(out["workspace"]) == gc.GC_OK and math.isfinite(out["loss"].item())


def test_config3_full_size_parity_invariants_and_reproducibility():
    q, p, r = synth.config3()
    want = oracle_loss(q, p, r)
    assert abs(want["loss"] - (math.log(8192) + 1 / 1536)) < 0.01
    out = run_ex(q, p, r)
    compare(out, want, TOL_BF16, q, p, 1.0, gap_tol=2e-6, label="config3 (library's choice: online walk)")
    # the other kernel sequence (statistics pass, then both walks in one launch: what every call without dq takes)
    compare(run_ex(q, p, r, flags=gc.GC_PATH_STATS_PASS), want, TOL_BF16, q, p, 1.0, gap_tol=2e-6, label="config3 statistics pass")
    dq, dp = to_np(out["dq"]), to_np(out["dp"])
    q64, p64 = synth.widen(q), synth.widen(p)
    # I1: rows of softmax - Y sum to zero  =>  sum_j dp_j = 0
    assert np.abs(dp.sum(axis=0)).max() <= TOL_BF16 * np.abs(dp).max() * 8
    # I2: sum_i <q_i, dq_i> = sum_j <p_j, dp_j>
    eq, ep = np.sum(q64 * dq), np.sum(p64 * dp)
    assert abs(eq - ep) <= 2e-3 * max(abs(eq), abs(ep), np.abs(dq).max())
    # I5: bit-identical from run to run, and through the plain entry point
    again = run_ex(q, p, r)
    for k in ("loss", "dq", "dp", "lse", "argmax"):
        assert torch.equal(out[k], again[k]), k
    loss, dq2, dp2 = gc.gc_loss_and_rep_grad_bf16(q.to(DEV), p.to(DEV), r.to(DEV))
    torch.cuda.synchronize()
    assert torch.equal(dq2, out["dq"]) and torch.equal(dp2, out["dp"]) and loss.item() == out["loss"].item()


def test_i4_permuting_targets_permutes_dp():
    q, p, r = synth.dpr_batch(200, 500, 256, torch.bfloat16, seed=77)
    a = run_ex(q, p, r)
    perm = torch.from_numpy(np.random.default_rng(5).permutation(500))
    inv = torch.argsort(perm)
    b = run_ex(q, p[perm].contiguous(), inv[r.long()].to(torch.int32))
    assert abs(a["loss"].item() - b["loss"].item()) <= 1e-5 * abs(a["loss"].item())
    assert relerr(to_np(b["dq"]), to_np(a["dq"])) <= 1e-3
    assert relerr(to_np(b["dp"]), to_np(a["dp"])[perm.numpy()]) <= 1e-3
