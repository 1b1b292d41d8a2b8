"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and rejects bad arguments on the host before any HIP call."""
import ctypes
import os
import re

import pytest

from paper_2101_06983_amd import binding as gc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "gradcache.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gc_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = gc.load()
    names = header_functions()
    assert len(names) >= 13
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(names) == sorted(gc.EXPORTS)


def test_strerror_texts():
    assert gc.strerror(0) == "ok"
    for code in range(-7, 0):
        assert gc.strerror(code) and "unknown" not in gc.strerror(code)
    assert "unknown" in gc.strerror(-99)


def test_workspace_bytes_is_linear_in_rows_not_quadratic():
    # persistent state is O((B + P) d): the cache of Sec. "Gradient Cache Technique", never O(B P)
    lib = gc.load()
    w1 = lib.gc_workspace_bytes(4096, 8192, 768, gc.GC_BF16)
    assert 0 < w1 < 8 * (4096 + 8192) * 768 * 4
    # (at this size a split of the stream costs a partial copy of an output, 8 B per row and column, so the
    # workspace is of the order of a bf16 score matrix; it does not grow with B * P:)
    w2 = lib.gc_workspace_bytes(8192, 16384, 768, gc.GC_BF16)
    assert w2 < 3 * w1
    assert w2 < 8192 * 16384 * 2 / 2      # well below a bf16 score matrix
    w3 = lib.gc_workspace_bytes(32768, 65536, 768, gc.GC_BF16)
    assert w3 < 16 * (32768 + 65536) * 4 + 4096 or w3 < 2 * (32768 + 65536) * 768 * 4
    assert lib.gc_workspace_bytes(0, 5, 8, gc.GC_F32) == 0
    assert lib.gc_workspace_bytes(5, 5, 8, 7) == 0
    assert lib.gc_ntxent_workspace_bytes(7, 128) == 0
    assert lib.gc_ntxent_workspace_bytes(16384, 128) > 0


def test_argument_errors_are_raised_on_the_host():
    lib = gc.load()
    vp = ctypes.c_void_p
    fake = vp(256)  # never dereferenced: all checks below fail before any HIP call
    f = lib.gc_loss_and_rep_grad_bf16
    assert f(None, fake, fake, 8, 16, 128, 1.0, 1.0, fake, fake, fake, None) == gc.GC_ERR_NULL
    assert f(fake, fake, None, 8, 16, 128, 1.0, 1.0, fake, fake, fake, None) == gc.GC_ERR_NULL
    assert f(fake, fake, fake, 8, 16, 128, 1.0, 1.0, None, fake, fake, None) == gc.GC_ERR_NULL
    assert f(fake, fake, fake, 0, 16, 128, 1.0, 1.0, fake, fake, fake, None) == gc.GC_ERR_SHAPE
    assert f(fake, fake, fake, 8, -1, 128, 1.0, 1.0, fake, fake, fake, None) == gc.GC_ERR_SHAPE
    assert f(fake, fake, fake, 8, 16, 0, 1.0, 1.0, fake, fake, fake, None) == gc.GC_ERR_SHAPE
    assert f(fake, fake, fake, 8, 16, 128, 1.0, 0.0, fake, fake, fake, None) == gc.GC_ERR_SHAPE
    assert f(fake, fake, fake, 8, 16, 128, float("nan"), 1.0, fake, fake, fake, None) == gc.GC_ERR_SHAPE
    assert f(fake, fake, fake, 8, 16, 128, float("inf"), 1.0, fake, fake, fake, None) == gc.GC_ERR_SHAPE
    st = lib.gc_loss_and_rep_grad_bf16_static
    assert st(None, fake, fake, 8, 16, 128, 1.0, 1.0, fake, fake, fake, None) == gc.GC_ERR_NULL
    assert st(fake, fake, fake, 8, 16, 128, 1.0, 1.0, fake, None, fake, None) == gc.GC_ERR_NULL
    assert st(fake, fake, fake, 8, 0, 128, 1.0, 1.0, fake, fake, fake, None) == gc.GC_ERR_SHAPE
    assert st(fake, fake, fake, 4096, 8192, 768, 1.0, 1.0, fake, fake, fake, None) == gc.GC_ERR_TOO_LARGE
    ex = lib.gc_loss_and_rep_grad_ex
    args = lambda **k: [k.get("dt", gc.GC_BF16), fake, fake, fake, k.get("B", 8), k.get("P", 16), 128, 1.0, 1.0,
                        k.get("flags", 0), fake, fake, fake, None, None, k.get("ws", fake), k.get("wsb", 1 << 30), None]
    assert ex(*args(dt=5)) == gc.GC_ERR_UNSUPPORTED
    assert ex(*args(flags=16)) == gc.GC_ERR_UNSUPPORTED
    assert ex(*args(flags=gc.GC_CACHE_BF16, dt=gc.GC_F32)) == gc.GC_ERR_UNSUPPORTED   # bf16 cache: MFMA shapes only
    assert ex(*args(flags=gc.GC_PATH_ONLINE | gc.GC_PATH_STATS_PASS)) == gc.GC_ERR_UNSUPPORTED
    assert ex(*args(flags=gc.GC_MASK_SELF)) == gc.GC_ERR_SHAPE          # B != P
    assert ex(*args(ws=None)) == gc.GC_ERR_WORKSPACE
    assert ex(*args(ws=vp(264))) == gc.GC_ERR_WORKSPACE                  # misaligned
    assert ex(*args(wsb=16)) == gc.GC_ERR_WORKSPACE
    nt = lib.gc_ntxent_loss_and_grad_bf16
    assert nt(None, 16, 128, 0.1, fake, fake, fake, 1 << 30, None) == gc.GC_ERR_NULL
    assert nt(fake, 15, 128, 0.1, fake, fake, fake, 1 << 30, None) == gc.GC_ERR_SHAPE
    assert nt(fake, 16, 128, -1.0, fake, fake, fake, 1 << 30, None) == gc.GC_ERR_SHAPE
    assert nt(fake, 16, 128, 0.1, fake, fake, fake, 8, None) == gc.GC_ERR_WORKSPACE
    bd = lib.gc_bidirectional_loss_and_rep_grad_bf16
    assert bd(fake, None, fake, 16, 128, 1.0, 1.0, fake, fake, fake, fake, 1 << 30, None) == gc.GC_ERR_NULL
    assert bd(fake, fake, fake, 16, 128, 1.0, 1.0, fake, None, fake, fake, 1 << 30, None) == gc.GC_ERR_NULL
    assert bd(fake, fake, fake, 0, 128, 1.0, 1.0, fake, fake, fake, fake, 1 << 30, None) == gc.GC_ERR_SHAPE
    assert bd(fake, fake, fake, 16, 128, 1.0, 0.0, fake, fake, fake, fake, 1 << 30, None) == gc.GC_ERR_SHAPE
    assert bd(fake, fake, fake, 16, 128, 1.0, 1.0, fake, fake, fake, None, 1 << 30, None) == gc.GC_ERR_WORKSPACE
    assert bd(fake, fake, fake, 16, 128, 1.0, 1.0, fake, fake, fake, fake, 64, None) == gc.GC_ERR_WORKSPACE
    bl = lib.gc_bilinear_loss_and_grads_bf16
    bargs = lambda **k: [k.get("q", fake), fake, fake, k.get("B", 8), 16, k.get("d", 128), k.get("om", fake), 1.0,
                         k.get("temp", 1.0), fake, fake, fake, k.get("dom", fake), k.get("ws", fake), k.get("wsb", 1 << 30), None]
    assert bl(*bargs(q=None)) == gc.GC_ERR_NULL
    assert bl(*bargs(om=None)) == gc.GC_ERR_NULL
    assert bl(*bargs(dom=None)) == gc.GC_ERR_NULL
    assert bl(*bargs(B=0)) == gc.GC_ERR_SHAPE
    assert bl(*bargs(temp=0.0)) == gc.GC_ERR_SHAPE
    assert bl(*bargs(d=96)) == gc.GC_ERR_UNSUPPORTED
    assert bl(*bargs(d=1024)) == gc.GC_ERR_UNSUPPORTED
    assert bl(*bargs(ws=None)) == gc.GC_ERR_WORKSPACE
    assert bl(*bargs(wsb=1024)) == gc.GC_ERR_WORKSPACE
    assert lib.gc_bilinear_workspace_bytes(8, 16, 96) == 0 and lib.gc_bilinear_workspace_bytes(8, 16, 128) > 0
    dd = lib.gc_deepdist_loss_and_grads_bf16
    dargs = lambda **k: [k.get("q", fake), fake, fake, k.get("B", 8), 16, k.get("d", 128), fake, fake, k.get("w", fake),
                         k.get("h", 128), 1.0, k.get("temp", 1.0), fake, fake, fake, fake, fake, k.get("dw", fake),
                         k.get("ws", fake), k.get("wsb", 1 << 30), None]
    assert dd(*dargs(q=None)) == gc.GC_ERR_NULL
    assert dd(*dargs(w=None)) == gc.GC_ERR_NULL
    assert dd(*dargs(dw=None)) == gc.GC_ERR_NULL
    assert dd(*dargs(B=0)) == gc.GC_ERR_SHAPE
    assert dd(*dargs(temp=-1.0)) == gc.GC_ERR_SHAPE
    assert dd(*dargs(d=96)) == gc.GC_ERR_UNSUPPORTED
    assert dd(*dargs(h=64)) == gc.GC_ERR_UNSUPPORTED
    assert dd(*dargs(ws=None)) == gc.GC_ERR_WORKSPACE
    assert dd(*dargs(wsb=1024)) == gc.GC_ERR_WORKSPACE
    assert lib.gc_deepdist_workspace_bytes(8, 16, 96, 128) == 0 and lib.gc_deepdist_workspace_bytes(8, 16, 128, 64) == 0
    # linear in the rows (split partials of the h-wide pair gradients), never the B x P distance gradient cache
    w1 = lib.gc_deepdist_workspace_bytes(4096, 8192, 768, 128)
    assert 0 < w1 < 4096 * 8192 * 4
    w2 = lib.gc_deepdist_workspace_bytes(8192, 16384, 768, 128)
    assert w2 < 2 * w1 and w2 < 8192 * 16384 * 4 / 4
    # loss workspaces (split partials included; four gradient buffers for widths the MFMA kernels do not take):
    # never the n x n scores
    for n in (4096, 8192, 65536):
        assert 0 < lib.gc_bidirectional_workspace_bytes(n, 768) < 16 * n * 768 * 4
        assert 4 * n * 96 * 4 < lib.gc_bidirectional_workspace_bytes(n, 96) < 16 * n * 96 * 4
    assert lib.gc_bidirectional_workspace_bytes(0, 768) == 0


def test_mlp_argument_errors_are_raised_on_the_host():
    lib = gc.load()
    vp = ctypes.c_void_p
    fake = 256  # never dereferenced
    ok = gc.gc_mlp_params(fake, fake, fake, fake, 1024, 3072, 768)
    grads = gc.gc_mlp_grads(fake, fake, fake, fake)
    ref = ctypes.byref
    # workspace sizes: 0 for bad shapes, linear in the rows of a sub-batch otherwise
    assert lib.gc_mlp_workspace_bytes(32, ref(gc.gc_mlp_params(fake, fake, fake, fake, 1000, 3072, 768))) == 0
    w32, w64 = lib.gc_mlp_workspace_bytes(32, ref(ok)), lib.gc_mlp_workspace_bytes(64, ref(ok))
    assert 0 < w32 < w64 and w64 - w32 == 32 * 3072 * 4 * 3
    assert lib.gc_step_mlp_workspace_bytes(512, 1024, 32, 32, ref(ok)) > w32
    assert lib.gc_step_mlp_workspace_bytes(512, 1024, 0, 32, ref(ok)) == 0
    fwd = lib.gc_mlp_forward_nograd_bf16
    assert fwd(None, 32, ref(ok), vp(fake), vp(fake), 1 << 30, None) == gc.GC_ERR_NULL
    assert fwd(vp(fake), 32, None, vp(fake), vp(fake), 1 << 30, None) == gc.GC_ERR_NULL
    assert fwd(vp(fake), 0, ref(ok), vp(fake), vp(fake), 1 << 30, None) == gc.GC_ERR_SHAPE
    assert fwd(vp(fake), 32, ref(ok), vp(fake), vp(fake), 64, None) == gc.GC_ERR_WORKSPACE
    assert fwd(vp(fake), 32, ref(ok), vp(fake), vp(264), 1 << 30, None) == gc.GC_ERR_WORKSPACE
    bad_dh = gc.gc_mlp_params(fake, fake, fake, fake, 1024, 3000, 768)
    assert fwd(vp(fake), 32, ref(bad_dh), vp(fake), vp(fake), 1 << 30, None) == gc.GC_ERR_UNSUPPORTED
    no_w2 = gc.gc_mlp_params(fake, fake, None, fake, 1024, 3072, 768)
    assert fwd(vp(fake), 32, ref(no_w2), vp(fake), vp(fake), 1 << 30, None) == gc.GC_ERR_NULL
    bwd = lib.gc_chunk_surrogate_backward_bf16
    assert bwd(vp(fake), 32, ref(ok), None, ref(grads), vp(fake), 1 << 30, None) == gc.GC_ERR_NULL
    assert bwd(vp(fake), 32, ref(ok), vp(fake), ref(gc.gc_mlp_grads(fake, None, fake, fake)), vp(fake), 1 << 30, None) == gc.GC_ERR_NULL
    assert bwd(vp(fake), 32, ref(ok), vp(fake), ref(grads), vp(fake), 8, None) == gc.GC_ERR_WORKSPACE
    step = lib.gc_step_mlp_bf16
    sargs = lambda **k: [vp(fake), k.get("B", 512), vp(fake), 1024, vp(fake), k.get("cq", 32), 32, ref(ok), 1.0, k.get("temp", 1.0),
                         k.get("loss", vp(fake)), ref(grads), None, None, None, None, k.get("ws", vp(fake)), k.get("wsb", 1 << 40), None]
    assert step(*sargs(B=0)) == gc.GC_ERR_SHAPE
    assert step(*sargs(cq=0)) == gc.GC_ERR_SHAPE
    assert step(*sargs(temp=0.0)) == gc.GC_ERR_SHAPE
    assert step(*sargs(loss=None)) == gc.GC_ERR_NULL
    assert step(*sargs(ws=None)) == gc.GC_ERR_WORKSPACE
    assert step(*sargs(wsb=1024)) == gc.GC_ERR_WORKSPACE


def test_host_checks_run_clean_under_ubsan(tmp_path):
    """The same argument-check tests against a build whose host code carries UndefinedBehaviorSanitizer checks that
    abort at the first finding (an enum loaded from an invalid integer, arithmetic on a null workspace base, an
    overflowing size): every rejected call must be rejected by defined behaviour."""
    import subprocess
    import sys

    from paper_2101_06983_amd import build

    if os.environ.get("GRADCACHE_LIB"):
        pytest.skip("already running against a substituted library")
    try:
        lib = build.build_host_checked(str(tmp_path / "libgradcache_ubsan.so"), str(tmp_path))
    except FileNotFoundError as e:
        pytest.skip("no ordinary build to take the loss_mfma object from, or no shared UBSan runtime: %s" % e)
    env = dict(os.environ, GRADCACHE_LIB=lib, UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.abspath(__file__), "-q", "-x", "-s", "-p", "no:cacheprovider"],
                       env=env, capture_output=True, text=True, timeout=600, cwd=os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    out = r.stdout + r.stderr
    assert "runtime error" not in out, out[-4000:]
    assert r.returncode == 0, out[-4000:]
    assert " passed" in out and "1 skipped" in out
