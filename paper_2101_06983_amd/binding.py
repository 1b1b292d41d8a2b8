"""ctypes binding of libgradcache.so: same names as include/gradcache.h.

Argument marshalling only: torch supplies device buffers and the current HIP
stream, every step of the path runs inside the library's kernels.  There is no
fallback: if the library has not been built, or a call fails, an error is raised.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("GRADCACHE_LIB") or os.path.join(_HERE, "libgradcache.so")

GC_OK = 0
GC_ERR_NULL, GC_ERR_SHAPE, GC_ERR_UNSUPPORTED, GC_ERR_WORKSPACE, GC_ERR_POS_IDX, GC_ERR_HIP = -1, -2, -3, -4, -5, -6
GC_ERR_TOO_LARGE = -7
GC_STATIC_SCRATCH_BYTES = 16 << 20
GC_F32, GC_BF16 = 0, 1
GC_MASK_SELF = 1
GC_PATH_ONLINE, GC_PATH_STATS_PASS = 2, 4
GC_CACHE_BF16 = 8

EXPORTS = [
    "gc_strerror", "gc_workspace_bytes", "gc_loss_and_rep_grad_bf16", "gc_loss_and_rep_grad_f32",
    "gc_loss_and_rep_grad_bf16_static",
    "gc_loss_and_rep_grad_ex", "gc_check_async_error", "gc_ntxent_workspace_bytes",
    "gc_ntxent_loss_and_grad_bf16", "gc_bidirectional_workspace_bytes",
    "gc_bidirectional_loss_and_rep_grad_bf16", "gc_bilinear_workspace_bytes", "gc_bilinear_workspace_layout",
    "gc_bilinear_loss_and_grads_bf16", "gc_deepdist_workspace_bytes", "gc_deepdist_loss_and_grads_bf16",
    "gc_mlp_workspace_bytes", "gc_mlp_forward_nograd_bf16",
    "gc_chunk_surrogate_backward_bf16", "gc_step_mlp_workspace_bytes", "gc_step_mlp_bf16",
    "gc_step_mlp_grouped_workspace_bytes", "gc_step_mlp_grouped_bf16",
    "gc_step_mlp_release", "gc_profile_begin", "gc_profile_end",
]


class GradCacheError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, strerror(status), status))


class gc_mlp_params(ctypes.Structure):
    _fields_ = [("W1", ctypes.c_void_p), ("b1", ctypes.c_void_p), ("W2", ctypes.c_void_p), ("b2", ctypes.c_void_p),
                ("din", ctypes.c_int), ("dh", ctypes.c_int), ("dout", ctypes.c_int)]


class gc_mlp_grads(ctypes.Structure):
    _fields_ = [("dW1", ctypes.c_void_p), ("db1", ctypes.c_void_p), ("dW2", ctypes.c_void_p), ("db2", ctypes.c_void_p)]


_lib = None


def load():
    """Loads the built library (raises if it is missing: build it with
    `python -m paper_2101_06983_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libgradcache.so is not built (%s); run python -m paper_2101_06983_amd.build" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, cf, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.gc_strerror.restype = ctypes.c_char_p
    lib.gc_strerror.argtypes = [ci]
    lib.gc_workspace_bytes.restype = sz
    lib.gc_workspace_bytes.argtypes = [ci, ci, ci, ci]
    for name in ("gc_loss_and_rep_grad_bf16", "gc_loss_and_rep_grad_f32", "gc_loss_and_rep_grad_bf16_static"):
        f = getattr(lib, name)
        f.restype = ci
        f.argtypes = [vp, vp, vp, ci, ci, ci, cf, cf, vp, vp, vp, vp]
    lib.gc_loss_and_rep_grad_ex.restype = ci
    lib.gc_loss_and_rep_grad_ex.argtypes = [ci, vp, vp, vp, ci, ci, ci, cf, cf, ctypes.c_uint, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.gc_check_async_error.restype = ci
    lib.gc_check_async_error.argtypes = [vp]
    lib.gc_ntxent_workspace_bytes.restype = sz
    lib.gc_ntxent_workspace_bytes.argtypes = [ci, ci]
    lib.gc_ntxent_loss_and_grad_bf16.restype = ci
    lib.gc_ntxent_loss_and_grad_bf16.argtypes = [vp, ci, ci, cf, vp, vp, vp, sz, vp]
    lib.gc_bidirectional_workspace_bytes.restype = sz
    lib.gc_bidirectional_workspace_bytes.argtypes = [ci, ci]
    lib.gc_bidirectional_loss_and_rep_grad_bf16.restype = ci
    lib.gc_bidirectional_loss_and_rep_grad_bf16.argtypes = [vp, vp, vp, ci, ci, cf, cf, vp, vp, vp, vp, sz, vp]
    lib.gc_bilinear_workspace_bytes.restype = sz
    lib.gc_bilinear_workspace_bytes.argtypes = [ci, ci, ci]
    lib.gc_bilinear_workspace_layout.restype = ci
    lib.gc_bilinear_workspace_layout.argtypes = [ci, ci, ci, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    lib.gc_bilinear_loss_and_grads_bf16.restype = ci
    lib.gc_bilinear_loss_and_grads_bf16.argtypes = [vp, vp, vp, ci, ci, ci, vp, cf, cf, vp, vp, vp, vp, vp, sz, vp]
    lib.gc_deepdist_workspace_bytes.restype = sz
    lib.gc_deepdist_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.gc_deepdist_loss_and_grads_bf16.restype = ci
    lib.gc_deepdist_loss_and_grads_bf16.argtypes = [vp, vp, vp, ci, ci, ci, vp, vp, vp, ci, cf, cf, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    pp, pg = ctypes.POINTER(gc_mlp_params), ctypes.POINTER(gc_mlp_grads)
    lib.gc_mlp_workspace_bytes.restype = sz
    lib.gc_mlp_workspace_bytes.argtypes = [ci, pp]
    lib.gc_mlp_forward_nograd_bf16.restype = ci
    lib.gc_mlp_forward_nograd_bf16.argtypes = [vp, ci, pp, vp, vp, sz, vp]
    lib.gc_chunk_surrogate_backward_bf16.restype = ci
    lib.gc_chunk_surrogate_backward_bf16.argtypes = [vp, ci, pp, vp, pg, vp, sz, vp]
    lib.gc_step_mlp_workspace_bytes.restype = sz
    lib.gc_step_mlp_workspace_bytes.argtypes = [ci, ci, ci, ci, pp]
    lib.gc_step_mlp_bf16.restype = ci
    lib.gc_step_mlp_bf16.argtypes = [vp, ci, vp, ci, vp, ci, ci, pp, cf, cf, vp, pg, vp, vp, vp, vp, vp, sz, vp]
    lib.gc_step_mlp_grouped_workspace_bytes.restype = sz
    lib.gc_step_mlp_grouped_workspace_bytes.argtypes = [ci, ci, ci, ci, pp, ci]
    lib.gc_step_mlp_grouped_bf16.restype = ci
    lib.gc_step_mlp_grouped_bf16.argtypes = [vp, ci, vp, ci, vp, ci, ci, ci, pp, cf, cf, vp, pg, vp, vp, vp, vp, vp, sz, vp]
    lib.gc_step_mlp_release.restype = ci
    lib.gc_step_mlp_release.argtypes = []
    lib.gc_profile_begin.restype = ci
    lib.gc_profile_begin.argtypes = [ci]
    fp = ctypes.POINTER(ctypes.c_float)
    lib.gc_profile_end.restype = ci
    lib.gc_profile_end.argtypes = [fp, fp, fp, fp, ctypes.POINTER(ci)]
    _lib = lib
    return lib


def strerror(status):
    return load().gc_strerror(int(status)).decode()


def _check(rc, where):
    if rc != GC_OK:
        raise GradCacheError(rc, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev_contig(t, dtype, what):
    if t.dtype != dtype or not t.is_cuda or not t.is_contiguous():
        raise ValueError("%s must be a contiguous %s device tensor" % (what, dtype))
    return t


def alloc_workspace(nbytes, device):
    return torch.empty(max(int(nbytes), 256) + 256, dtype=torch.uint8, device=device)


def _ws_ptr(ws):
    base = ws.data_ptr()
    aligned = (base + 255) // 256 * 256
    return ctypes.c_void_p(aligned), ws.numel() - (aligned - base)


def gc_workspace_bytes(B, P, d, dt):
    return load().gc_workspace_bytes(B, P, d, dt)


def _simple(fn_name, dtype, q, p, pos_idx, scale, temp, stream, out=None):
    lib = load()
    _dev_contig(q, dtype, "q"); _dev_contig(p, dtype, "p"); _dev_contig(pos_idx, torch.int32, "pos_idx")
    B, d = q.shape
    P = p.shape[0]
    if out is not None:
        loss, dq, dp = out
        _dev_contig(loss, torch.float32, "loss"); _dev_contig(dq, torch.float32, "dq"); _dev_contig(dp, torch.float32, "dp")
        if loss.numel() != 1 or tuple(dq.shape) != (B, d) or tuple(dp.shape) != (P, d):
            raise ValueError("preallocated outputs must be loss[1], dq[B,d], dp[P,d]")
    else:
        loss = torch.empty(1, dtype=torch.float32, device=q.device)
        dq = torch.empty(B, d, dtype=torch.float32, device=q.device)
        dp = torch.empty(P, d, dtype=torch.float32, device=q.device)
    rc = getattr(lib, fn_name)(_ptr(q), _ptr(p), _ptr(pos_idx), B, P, d, scale, temp, _ptr(loss), _ptr(dq), _ptr(dp),
                               _stream(stream))
    _check(rc, fn_name)
    return loss, dq, dp


def gc_loss_and_rep_grad_bf16(q, p, pos_idx, scale=1.0, temp=1.0, stream=None):
    return _simple("gc_loss_and_rep_grad_bf16", torch.bfloat16, q, p, pos_idx, scale, temp, stream)


def gc_loss_and_rep_grad_bf16_static(q, p, pos_idx, scale=1.0, temp=1.0, stream=None, out=None):
    """The call that allocates nothing inside the library (its workspace is a fixed array in the device image).
    `out` = (loss, dq, dp) preallocated makes the whole call allocation-free."""
    return _simple("gc_loss_and_rep_grad_bf16_static", torch.bfloat16, q, p, pos_idx, scale, temp, stream, out)


def gc_loss_and_rep_grad_f32(q, p, pos_idx, scale=1.0, temp=1.0, stream=None):
    return _simple("gc_loss_and_rep_grad_f32", torch.float32, q, p, pos_idx, scale, temp, stream)


def gc_loss_and_rep_grad_ex(q, p, pos_idx, scale=1.0, temp=1.0, flags=0, want=("loss", "dq", "dp", "lse", "argmax"),
                            workspace=None, out=None, stream=None):
    """Returns a dict of the requested outputs (+ 'workspace').  `out` may hold
    preallocated output tensors to write into."""
    lib = load()
    if q.dtype == torch.bfloat16:
        dt = GC_BF16
    elif q.dtype == torch.float32:
        dt = GC_F32
    else:
        raise ValueError("q must be bf16 or fp32")
    _dev_contig(q, q.dtype, "q"); _dev_contig(p, q.dtype, "p"); _dev_contig(pos_idx, torch.int32, "pos_idx")
    B, d = q.shape
    P = p.shape[0]
    dev = q.device
    out = dict(out or {})
    cache = torch.bfloat16 if (flags & GC_CACHE_BF16) else torch.float32
    shapes = dict(loss=((1,), torch.float32), dq=((B, d), cache), dp=((P, d), cache),
                  lse=((B,), torch.float32), argmax=((B,), torch.int32))
    for k in want:
        if k not in out:
            out[k] = torch.empty(shapes[k][0], dtype=shapes[k][1], device=dev)
        elif out[k].dtype != shapes[k][1] or tuple(out[k].shape) != shapes[k][0] or not out[k].is_contiguous():
            raise ValueError("preallocated %s must be a contiguous %s tensor of shape %s" % (k, shapes[k][1], shapes[k][0]))
    need = lib.gc_workspace_bytes(B, P, d, dt)
    if workspace is None:
        workspace = alloc_workspace(need, dev)
    wp, wn = _ws_ptr(workspace)
    rc = lib.gc_loss_and_rep_grad_ex(dt, _ptr(q), _ptr(p), _ptr(pos_idx), B, P, d, scale, temp, flags,
                                     _ptr(out.get("loss")), _ptr(out.get("dq")), _ptr(out.get("dp")),
                                     _ptr(out.get("lse")), _ptr(out.get("argmax")), wp, wn, _stream(stream))
    _check(rc, "gc_loss_and_rep_grad_ex")
    out["workspace"] = workspace
    return out


def gc_check_async_error(workspace=None):
    lib = load()
    if workspace is None:
        return lib.gc_check_async_error(None)
    return lib.gc_check_async_error(_ws_ptr(workspace)[0])


def gc_profile_begin(max_calls):
    _check(load().gc_profile_begin(int(max_calls)), "gc_profile_begin")


def gc_profile_end():
    """Returns dict(ms_stats, ms_merge, ms_grad, ms_reduce, calls): mean device milliseconds per call."""
    a, b, c, d, n = ctypes.c_float(), ctypes.c_float(), ctypes.c_float(), ctypes.c_float(), ctypes.c_int()
    _check(load().gc_profile_end(ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(d), ctypes.byref(n)),
           "gc_profile_end")
    return dict(ms_stats=a.value, ms_merge=b.value, ms_grad=c.value, ms_reduce=d.value, calls=n.value)


def gc_ntxent_loss_and_grad_bf16(z, temp, workspace=None, stream=None):
    lib = load()
    _dev_contig(z, torch.bfloat16, "z")
    n, d = z.shape
    loss = torch.empty(1, dtype=torch.float32, device=z.device)
    dz = torch.empty(n, d, dtype=torch.float32, device=z.device)
    if workspace is None:
        workspace = alloc_workspace(lib.gc_ntxent_workspace_bytes(n, d), z.device)
    wp, wn = _ws_ptr(workspace)
    rc = lib.gc_ntxent_loss_and_grad_bf16(_ptr(z), n, d, temp, _ptr(loss), _ptr(dz), wp, wn, _stream(stream))
    _check(rc, "gc_ntxent_loss_and_grad_bf16")
    return loss, dz


def gc_bidirectional_loss_and_rep_grad_bf16(q, p, pos_idx, scale=1.0, temp=1.0, workspace=None, out=None, stream=None):
    """Symmetric loss; returns dict(loss, dq, dp).  `out` may carry the three buffers to reuse."""
    lib = load()
    _dev_contig(q, torch.bfloat16, "q")
    _dev_contig(p, torch.bfloat16, "p")
    _dev_contig(pos_idx, torch.int32, "pos_idx")
    n, d = q.shape
    if tuple(p.shape) != (n, d) or tuple(pos_idx.shape) != (n,):
        raise GradCacheError(GC_ERR_SHAPE, "gc_bidirectional_loss_and_rep_grad_bf16")
    if out is None:
        out = dict(loss=torch.empty(1, dtype=torch.float32, device=q.device),
                   dq=torch.empty(n, d, dtype=torch.float32, device=q.device),
                   dp=torch.empty(n, d, dtype=torch.float32, device=q.device))
    if workspace is None:
        workspace = alloc_workspace(lib.gc_bidirectional_workspace_bytes(n, d), q.device)
    wp, wn = _ws_ptr(workspace)
    rc = lib.gc_bidirectional_loss_and_rep_grad_bf16(_ptr(q), _ptr(p), _ptr(pos_idx), n, d, scale, temp, _ptr(out["loss"]),
                                                     _ptr(out["dq"]), _ptr(out["dp"]), wp, wn, _stream(stream))
    _check(rc, "gc_bidirectional_loss_and_rep_grad_bf16")
    return out


def gc_bilinear_loss_and_grads_bf16(q, p, pos_idx, omega, scale=1.0, temp=1.0, workspace=None, out=None, stream=None):
    """Bilinear distance f^T Omega g; returns dict(loss, u, v, domega, workspace)."""
    lib = load()
    for t, name in ((q, "q"), (p, "p"), (omega, "omega")):
        _dev_contig(t, torch.bfloat16, name)
    _dev_contig(pos_idx, torch.int32, "pos_idx")
    B, d = q.shape
    P = p.shape[0]
    if p.shape[1] != d or tuple(omega.shape) != (d, d) or tuple(pos_idx.shape) != (B,):
        raise GradCacheError(GC_ERR_SHAPE, "gc_bilinear_loss_and_grads_bf16")
    if out is None:
        f32 = dict(dtype=torch.float32, device=q.device)
        out = dict(loss=torch.empty(1, **f32), u=torch.empty(B, d, **f32), v=torch.empty(P, d, **f32),
                   domega=torch.empty(d, d, **f32))
    if workspace is None:
        need = lib.gc_bilinear_workspace_bytes(B, P, d)
        if need == 0:
            raise GradCacheError(GC_ERR_UNSUPPORTED, "gc_bilinear_workspace_bytes")
        workspace = alloc_workspace(need, q.device)
    wp, wn = _ws_ptr(workspace)
    rc = lib.gc_bilinear_loss_and_grads_bf16(_ptr(q), _ptr(p), _ptr(pos_idx), B, P, d, _ptr(omega), scale, temp,
                                             _ptr(out["loss"]), _ptr(out["u"]), _ptr(out["v"]), _ptr(out["domega"]),
                                             wp, wn, _stream(stream))
    _check(rc, "gc_bilinear_loss_and_grads_bf16")
    out["workspace"] = workspace
    return out


def gc_deepdist_loss_and_grads_bf16(q, p, pos_idx, omega, scale=1.0, temp=1.0, workspace=None, out=None, stream=None):
    """Deep distance Phi = sum_k w_k tanh((A f)_k + (C g)_k); omega = dict(A [h,d], C [h,d], w [h]) of bf16 device
    tensors.  Returns dict(loss, u, v, dA, dC, dw, workspace)."""
    lib = load()
    A, C, w = omega["A"], omega["C"], omega["w"]
    for t, name in ((q, "q"), (p, "p"), (A, "A"), (C, "C"), (w, "w")):
        _dev_contig(t, torch.bfloat16, name)
    _dev_contig(pos_idx, torch.int32, "pos_idx")
    B, d = q.shape
    P = p.shape[0]
    h = A.shape[0]
    if p.shape[1] != d or tuple(A.shape) != (h, d) or tuple(C.shape) != (h, d) or tuple(w.shape) != (h,) or tuple(pos_idx.shape) != (B,):
        raise GradCacheError(GC_ERR_SHAPE, "gc_deepdist_loss_and_grads_bf16")
    if out is None:
        f32 = dict(dtype=torch.float32, device=q.device)
        out = dict(loss=torch.empty(1, **f32), u=torch.empty(B, d, **f32), v=torch.empty(P, d, **f32),
                   dA=torch.empty(h, d, **f32), dC=torch.empty(h, d, **f32), dw=torch.empty(h, **f32))
    if workspace is None:
        need = lib.gc_deepdist_workspace_bytes(B, P, d, h)
        if need == 0:
            raise GradCacheError(GC_ERR_UNSUPPORTED, "gc_deepdist_workspace_bytes")
        workspace = alloc_workspace(need, q.device)
    wp, wn = _ws_ptr(workspace)
    rc = lib.gc_deepdist_loss_and_grads_bf16(_ptr(q), _ptr(p), _ptr(pos_idx), B, P, d, _ptr(A), _ptr(C), _ptr(w), h, scale,
                                             temp, _ptr(out["loss"]), _ptr(out["u"]), _ptr(out["v"]), _ptr(out["dA"]),
                                             _ptr(out["dC"]), _ptr(out["dw"]), wp, wn, _stream(stream))
    _check(rc, "gc_deepdist_loss_and_grads_bf16")
    out["workspace"] = workspace
    return out


def gc_step_mlp_release():
    """Waits for the device and drops the graphs gc_step_mlp_bf16 has recorded on it."""
    _check(load().gc_step_mlp_release(), "gc_step_mlp_release")


def gc_bilinear_workspace_layout(B, P, d):
    """(off_h, off_a): byte offsets, from the 256-byte aligned workspace start, of H [B,d] bf16 and A [B,d] float."""
    a, b = ctypes.c_size_t(), ctypes.c_size_t()
    _check(load().gc_bilinear_workspace_layout(B, P, d, ctypes.byref(a), ctypes.byref(b)), "gc_bilinear_workspace_layout")
    return a.value, b.value


def bilinear_intermediates(workspace, B, P, d):
    """Views (no copy) of the H and A a gc_bilinear_loss_and_grads_bf16 call left in `workspace`."""
    off_h, off_a = gc_bilinear_workspace_layout(B, P, d)
    base = workspace.data_ptr()
    skip = (base + 255) // 256 * 256 - base
    h = workspace[skip + off_h: skip + off_h + B * d * 2].view(torch.bfloat16).view(B, d)
    a = workspace[skip + off_a: skip + off_a + B * d * 4].view(torch.float32).view(B, d)
    return h, a


# ----------------------------------------------------------------------------- stand-in encoder
def make_mlp_params(params):
    """params: dict W1 [din,dh], b1, W2 [dh,dout], b2 of contiguous bf16 device tensors."""
    for k in ("W1", "b1", "W2", "b2"):
        _dev_contig(params[k], torch.bfloat16, k)
    din, dh = params["W1"].shape
    dout = params["W2"].shape[1]
    return gc_mlp_params(params["W1"].data_ptr(), params["b1"].data_ptr(), params["W2"].data_ptr(),
                         params["b2"].data_ptr(), din, dh, dout)


def make_mlp_grads(grads):
    for k in ("W1", "b1", "W2", "b2"):
        _dev_contig(grads[k], torch.float32, "grad " + k)
    return gc_mlp_grads(grads["W1"].data_ptr(), grads["b1"].data_ptr(), grads["W2"].data_ptr(), grads["b2"].data_ptr())


def zero_mlp_grads(params):
    return {k: torch.zeros(params[k].shape, dtype=torch.float32, device=params[k].device) for k in ("W1", "b1", "W2", "b2")}


def gc_mlp_forward_nograd_bf16(x, params, workspace=None, stream=None):
    lib = load()
    _dev_contig(x, torch.bfloat16, "x")
    w = make_mlp_params(params)
    rows = x.shape[0]
    y = torch.empty(rows, w.dout, dtype=torch.bfloat16, device=x.device)
    if workspace is None:
        workspace = alloc_workspace(lib.gc_mlp_workspace_bytes(rows, ctypes.byref(w)), x.device)
    wp, wn = _ws_ptr(workspace)
    rc = lib.gc_mlp_forward_nograd_bf16(_ptr(x), rows, ctypes.byref(w), _ptr(y), wp, wn, _stream(stream))
    _check(rc, "gc_mlp_forward_nograd_bf16")
    return y


def gc_chunk_surrogate_backward_bf16(x_chunk, params, cached_grad_rows, grads, workspace=None, stream=None):
    lib = load()
    _dev_contig(x_chunk, torch.bfloat16, "x_chunk")
    _dev_contig(cached_grad_rows, torch.float32, "cached_grad_rows")
    w = make_mlp_params(params)
    g = make_mlp_grads(grads)
    rows = x_chunk.shape[0]
    if cached_grad_rows.shape != (rows, w.dout):
        raise ValueError("cached_grad_rows must be [rows, dout]")
    if workspace is None:
        workspace = alloc_workspace(lib.gc_mlp_workspace_bytes(rows, ctypes.byref(w)), x_chunk.device)
    wp, wn = _ws_ptr(workspace)
    rc = lib.gc_chunk_surrogate_backward_bf16(_ptr(x_chunk), rows, ctypes.byref(w), _ptr(cached_grad_rows),
                                              ctypes.byref(g), wp, wn, _stream(stream))
    _check(rc, "gc_chunk_surrogate_backward_bf16")
    return grads


def gc_step_mlp_bf16(x_q, x_p, pos_idx, chunk_q, chunk_p, params, scale=1.0, temp=1.0, grads=None, keep=False,
                     workspace=None, stream=None, out=None, accumulate_group=1):
    """One Gradient Cache step.  Returns dict(loss, grads[, q, p, dq, dp]).  Passing the dict a
    previous call returned as `out` reuses its buffers (loss, grads, kept outputs, workspace):
    the library replays a recorded graph when a call repeats with the same buffers.
    accumulate_group > 1 calls gc_step_mlp_grouped_bf16."""
    if out is not None:
        grads = out["grads"] if grads is None else grads
        workspace = out["workspace"] if workspace is None else workspace
        keep = keep or "q" in out
    lib = load()
    _dev_contig(x_q, torch.bfloat16, "x_q"); _dev_contig(x_p, torch.bfloat16, "x_p")
    _dev_contig(pos_idx, torch.int32, "pos_idx")
    w = make_mlp_params(params)
    if grads is None:
        grads = zero_mlp_grads(params)
    g = make_mlp_grads(grads)
    B, P = x_q.shape[0], x_p.shape[0]
    dev = x_q.device
    prev = out or {}
    loss = prev.get("loss")
    if loss is None:
        loss = torch.empty(1, dtype=torch.float32, device=dev)
    out = dict(loss=loss, grads=grads)
    if keep:
        for name, n, dt in (("q", B, torch.bfloat16), ("p", P, torch.bfloat16), ("dq", B, torch.float32), ("dp", P, torch.float32)):
            t = prev.get(name)
            out[name] = t if t is not None else torch.empty(n, w.dout, dtype=dt, device=dev)
    if workspace is None:
        workspace = alloc_workspace(lib.gc_step_mlp_grouped_workspace_bytes(B, P, chunk_q, chunk_p, ctypes.byref(w),
                                                                            accumulate_group), dev)
    wp, wn = _ws_ptr(workspace)
    if accumulate_group == 1:
        rc = lib.gc_step_mlp_bf16(_ptr(x_q), B, _ptr(x_p), P, _ptr(pos_idx), chunk_q, chunk_p, ctypes.byref(w), scale, temp,
                                  _ptr(loss), ctypes.byref(g), _ptr(out.get("q")), _ptr(out.get("p")), _ptr(out.get("dq")),
                                  _ptr(out.get("dp")), wp, wn, _stream(stream))
    else:
        rc = lib.gc_step_mlp_grouped_bf16(_ptr(x_q), B, _ptr(x_p), P, _ptr(pos_idx), chunk_q, chunk_p, accumulate_group,
                                          ctypes.byref(w), scale, temp, _ptr(loss), ctypes.byref(g), _ptr(out.get("q")),
                                          _ptr(out.get("p")), _ptr(out.get("dq")), _ptr(out.get("dp")), wp, wn,
                                          _stream(stream))
    _check(rc, "gc_step_mlp_bf16")
    out["workspace"] = workspace
    return out
