"""fp64 CPU oracle for the Gradient Cache hot path (arXiv 2101.06983).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
HIP kernels are checked against.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import it; the product path never does.  It
shares no code with the package under paper_2101_06983_amd/ and imports
nothing from it.

Everything is numpy float64.  Inputs that the GPU stores in bf16 or fp32 are
widened exactly to float64 by the caller, so input quantisation is not part of
the comparison.  The B x P score matrix is materialised on purpose: the method
is exact (Sec. "Gradient Cache Technique", Step 3 and the Conclusion), so the
oracle is the plain full-batch definition.

Notation follows the paper: F = {f(s_i)} are the anchor (query) rows Q[B, d],
G = {g(t_j)} the target (passage) rows P[P, d], r_i = pos_idx[i] the index of
the related target of anchor i, tau the temperature.

Every function is pinned by tests/test_oracle_pins.py against closed forms,
invariants, central finite differences, brute-force enumeration and the
torch.nn.functional.cross_entropy / autograd library routine; none is
"parity unpinned".
"""
import numpy as np
from scipy.special import erf

__all__ = [
    "loss_and_rep_grad", "ntxent", "bidirectional", "bilinear_distance", "deep_distance", "mlp_forward", "mlp_backward",
    "mlp_fullbatch_grad", "mlp_chunked_grad", "mlp_accumulation_grad", "round_to_bf16",
]


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def loss_and_rep_grad(q, p, pos_idx, scale=1.0, temp=1.0, mask_self=False):
    """Contrastive loss (Eq. 1) and its representation gradients (Eq. 4-7).

    q: [B, d] anchors f(s_i); p: [P, d] targets g(t_j); pos_idx: [B] ints r_i.
    Logits are s_ij = (scale / temp) * <q_i, p_j>  (Eq. 1 with the 1/tau kept;
    `scale` is an extra multiplier on the dot product, 1 in the paper).
    mask_self: s_ii = -inf (needs B == P), used by the NT-Xent variation.

    Returns dict with
      loss      Eq. 1, mean over the B anchors
      lse       [B]  log sum_j exp(s_ij)
      pos_logit [B]  s_{i, r_i}
      argmax    [B]  smallest j attaining max_j s_ij
      dq        [B, d]  dL/df(s_i), Eq. 5 (with the factor scale/temp)
      dp        [P, d]  dL/dg(t_j), Eq. 6 with eps_j = sum of f(s_k) over every
                        k that has r_k = j (Eq. 7; several anchors may share one
                        positive, none gives eps_j = 0)
    """
    q = _f64(q)
    p = _f64(p)
    r = np.asarray(pos_idx, dtype=np.int64)
    B, d = q.shape
    P, d2 = p.shape
    assert d == d2 and r.shape == (B,)
    assert np.all((r >= 0) & (r < P))
    alpha = float(scale) / float(temp)

    # scores: s_ij = alpha * f(s_i)^T g(t_j)
    s = alpha * (q @ p.T)
    if mask_self:
        assert B == P and P >= 2
        s[np.arange(B), np.arange(B)] = -np.inf

    # Eq. 4: p_ij = exp(s_ij) / sum_t exp(s_it), computed through the row max
    m = s.max(axis=1)
    e = np.exp(s - m[:, None])
    lse = m + np.log(e.sum(axis=1))
    argmax = np.argmax(s, axis=1)          # first occurrence = smallest index
    pos_logit = s[np.arange(B), r]

    # Eq. 1
    loss = np.sum(lse - pos_logit) / B

    # g_ij = p_ij - [j == r_i]
    g = np.exp(s - lse[:, None])
    g[np.arange(B), r] -= 1.0

    # Eq. 5:  dL/df(s_i) = -(1/|S|) (g(t_{r_i}) - sum_j p_ij g(t_j))      (* alpha)
    dq = (alpha / B) * (g @ p)
    # Eq. 6:  dL/dg(t_j) = -(1/|S|) (eps_j - sum_i p_ij f(s_i))           (* alpha)
    dp = (alpha / B) * (g.T @ q)
    return dict(loss=float(loss), lse=lse, pos_logit=pos_logit,
                argmax=argmax.astype(np.int64), dq=dq, dp=dp)


def ntxent(z, temp):
    """NT-Xent over 2N views (the loss variation named in Sec. Related Work /
    Step 2's remark that other contrastive losses are supported).

    z: [2N, d], rows already L2-normalised by the caller (normalisation is not
    part of the path).  Views 2k and 2k+1 are a positive pair.  Each view is an
    anchor against all other views (self-similarity removed); the loss is the
    mean over all 2N anchors, which averages both directions of every pair.
    Returns dict(loss, dz, lse) with dz = dL/dz: every row is both an anchor
    and a target, so its gradient is the sum of Eq. 5 and Eq. 6.
    """
    z = _f64(z)
    n = z.shape[0]
    assert n % 2 == 0 and n >= 2
    r = np.arange(n) ^ 1
    out = loss_and_rep_grad(z, z, r, scale=1.0, temp=temp, mask_self=True)
    return dict(loss=out["loss"], dz=out["dq"] + out["dp"], lse=out["lse"])


def bidirectional(q, p, pos_idx, scale=1.0, temp=1.0):
    """Symmetric in-batch-negative loss: anchors against targets and targets
    against anchors (one of the loss variations Step 2 admits; the method only
    needs dL/df(s_i) and dL/dg(t_j)).  B = P = n and r must be a bijection:
      L = 1/2 [ L(F, G, r) + L(G, F, r^-1) ],
    each term Eq. 1, the second with the roles of the two sides exchanged.
    Both terms are functions of the same scores s_ij: the first normalises
    every row (Eq. 4), the second every column, and both have their positive at
    (i, r_i).  So dL/ds_ij = g_ij / n with
      g_ij = 1/2 (p^row_ij + p^col_ij) - [j == r_i],
    and dL/df(s_i) = (alpha/n) sum_j g_ij g(t_j), dL/dg(t_j) = (alpha/n) sum_i g_ij f(s_i)
    (Eq. 5 of one term plus Eq. 6 of the other, halved).
    Returns dict(loss, dq, dp)."""
    q = _f64(q)
    p = _f64(p)
    r = np.asarray(pos_idx, dtype=np.int64)
    n = q.shape[0]
    assert p.shape == q.shape and sorted(r.tolist()) == list(range(n))
    alpha = float(scale) / float(temp)
    s = alpha * (q @ p.T)
    pos = s[np.arange(n), r]
    lse_row = loss_and_rep_grad(q, p, r, scale, temp)["lse"]          # over the targets, per anchor
    m = s.max(axis=0)
    lse_col = m + np.log(np.exp(s - m[None, :]).sum(axis=0))          # over the anchors, per target
    loss = 0.5 * (np.sum(lse_row - pos) + np.sum(lse_col[r] - pos)) / n
    g = 0.5 * (np.exp(s - lse_row[:, None]) + np.exp(s - lse_col[None, :]))
    g[np.arange(n), r] -= 1.0
    return dict(loss=float(loss), dq=(alpha / n) * (g @ p), dp=(alpha / n) * (g.T @ q))


def bilinear_distance(q, p, pos_idx, omega, scale=1.0, temp=1.0, rep_dtype=None):
    """Loss with a parameterised distance function (Sec. "Extend to Deep Distance
    Function"), for the bilinear form Phi_Omega(f, g) = f^T Omega g, Omega [d, d]:
      d_ij = f(s_i)^T Omega g(t_j)                     (the section's first equation)
      logits alpha * d_ij, loss as Eq. 1
      w_ij = dL/dd_ij = (alpha/B) (p_ij - [j == r_i])  (the Distance Gradient Cache)
      dOmega = sum_ij w_ij f(s_i) g(t_j)^T             (its gradient of Omega: d Phi / d Omega = f g^T)
      u_i = sum_j w_ij Omega g(t_j)                    (d d_ij / d f(s_i) = Omega g(t_j))
      v_j = sum_i w_ij Omega^T f(s_i)                  (d d_ij / d g(t_j) = Omega^T f(s_i))
    The B x P matrix w is materialised here, as the paper's description stores it.
    rep_dtype="bf16": the products h_i = Omega^T f(s_i) are stored in bf16 before
    they meet the targets (scores d_ij = <h_i, g(t_j)> and v_j = sum_i w_ij h_i use
    the stored values); u and dOmega flow through the unrounded bilinear form.
    Returns dict(loss, w, u, v, domega)."""
    q = _f64(q)
    p = _f64(p)
    om = _f64(omega)
    r = np.asarray(pos_idx, dtype=np.int64)
    B, d = q.shape
    P = p.shape[0]
    assert om.shape == (d, d) and p.shape[1] == d and r.shape == (B,)
    assert np.all((r >= 0) & (r < P))
    alpha = float(scale) / float(temp)
    h = _store(q @ om, rep_dtype)                # h_i^T = f(s_i)^T Omega
    s = alpha * (h @ p.T)
    m = s.max(axis=1)
    lse = m + np.log(np.exp(s - m[:, None]).sum(axis=1))
    loss = np.sum(lse - s[np.arange(B), r]) / B
    g = np.exp(s - lse[:, None])
    g[np.arange(B), r] -= 1.0
    w = (alpha / B) * g
    a = w @ p                                    # sum_j w_ij g(t_j)
    return dict(loss=float(loss), w=w, u=a @ om.T, v=w.T @ h, domega=q.T @ a)


def deep_distance(q, p, pos_idx, omega, scale=1.0, temp=1.0, block=8):
    """Loss with a deep (non-bilinear) distance function (Sec. "Extend to Deep Distance
    Function", all four equations), for the additive interaction
      Phi_Omega(f, g) = sum_k w_k tanh((A f)_k + (C g)_k),   Omega = (A [h, d], C [h, d], w [h]),
    a one-hidden-layer network on the pair (f, g); it does not factor into a product of
    a function of f and a function of g, so every one of the B * P distances is an
    evaluation of Phi of its own (the early-interaction case the section ends with).
      d_ij = Phi(f(s_i), g(t_j))                                    first equation
      logits alpha * d_ij, loss as Eq. 1
      w_ij = dL/dd_ij = (alpha / B) (p_ij - [j == r_i])             the Distance Gradient Cache, B x P, materialised
      dOmega = sum_ij w_ij dPhi(f_i, g_j)/dOmega                    second equation (the sub-batch double sum, all pairs)
      u_i = sum_j w_ij dd_ij/df(s_i)                                third equation
      v_j = sum_i w_ij dd_ij/dg(t_j)                                fourth equation
    With z_ijk = (A f_i)_k + (C g_j)_k, t = tanh z, t' = 1 - t^2:
      dd_ij/df_i = A^T (w * t'_ij),  dd_ij/dg_j = C^T (w * t'_ij),
      dPhi/dw_k = t_ijk,  dPhi/dA = (w * t'_ij) f_i^T,  dPhi/dC = (w * t'_ij) g_j^T.
    The pairs are visited `block` anchors at a time (a [block, P, h] array), nothing else is blocked.
    omega: dict(A, C, w).  Returns dict(loss, lse, w (the cache, called `cache` to keep it apart
    from the parameter w), u, v, dA, dC, dw)."""
    q = _f64(q)
    p = _f64(p)
    A, C, wv = _f64(omega["A"]), _f64(omega["C"]), _f64(omega["w"])
    r = np.asarray(pos_idx, dtype=np.int64)
    B, d = q.shape
    P = p.shape[0]
    h = A.shape[0]
    assert A.shape == (h, d) and C.shape == (h, d) and wv.shape == (h,) and p.shape[1] == d and r.shape == (B,)
    assert np.all((r >= 0) & (r < P))
    alpha = float(scale) / float(temp)
    a = q @ A.T                                   # (A f_i)_k
    c = p @ C.T                                   # (C g_j)_k
    # first forward: all distances
    dist = np.empty((B, P))
    for i0 in range(0, B, block):
        z = a[i0:i0 + block, None, :] + c[None, :, :]
        dist[i0:i0 + block] = np.tanh(z) @ wv
    s = alpha * dist
    m = s.max(axis=1)
    lse = m + np.log(np.exp(s - m[:, None]).sum(axis=1))
    loss = np.sum(lse - s[np.arange(B), r]) / B
    cache = np.exp(s - lse[:, None])
    cache[np.arange(B), r] -= 1.0
    cache *= alpha / B                            # w_ij
    # the three sums over the cached w_ij
    u = np.zeros((B, d))
    v = np.zeros((P, d))
    dA = np.zeros((h, d))
    dC = np.zeros((h, d))
    dw = np.zeros(h)
    for i0 in range(0, B, block):
        sl = slice(i0, min(i0 + block, B))
        t = np.tanh(a[sl, None, :] + c[None, :, :])              # [b, P, h]
        wij = cache[sl][:, :, None]                              # [b, P, 1]
        e = wij * (wv * (1.0 - t * t))                           # w_ij (w * t'_ij): [b, P, h]
        dw += (wij * t).sum(axis=(0, 1))
        ei = e.sum(axis=1)                                       # sum_j ...: [b, h]
        ej = e.sum(axis=0)                                       # sum_i (this block) ...: [P, h]
        u[sl] = ei @ A
        v += ej @ C
        dA += ei.T @ q[sl]
        dC += ej.T @ p
    return dict(loss=float(loss), lse=lse, cache=cache, u=u, v=v, dA=dA, dC=dC, dw=dw)


# ---------------------------------------------------------------------------
# Stand-in encoder: y = GELU(x W1 + b1) W2 + b2 (exact erf GELU), one parameter
# set shared by f and g (Theta = Lambda), so Eq. 2 and Eq. 3 add up.
# params = dict(W1 [din, dh], b1 [dh], W2 [dh, dout], b2 [dout])
# ---------------------------------------------------------------------------
def _gelu(h):
    return 0.5 * h * (1.0 + erf(h / np.sqrt(2.0)))


def _gelu_prime(h):
    # d/dh [h Phi(h)] = Phi(h) + h phi(h)
    return 0.5 * (1.0 + erf(h / np.sqrt(2.0))) + h * np.exp(-0.5 * h * h) / np.sqrt(2.0 * np.pi)


def _params64(params):
    return {k: _f64(params[k]) for k in ("W1", "b1", "W2", "b2")}


def mlp_forward(x, params, keep=False):
    """Encoder forward.  keep=False is the graph-less forward of Step 1."""
    w = _params64(params)
    x = _f64(x)
    h = x @ w["W1"] + w["b1"]
    a = _gelu(h)
    y = a @ w["W2"] + w["b2"]
    if keep:
        return y, h, a
    return y


def mlp_backward(x, params, upstream):
    """Parameter gradient of <f(x), upstream> for one (sub-)batch: the inner sum
    of Eq. 8 / Eq. 9 with u_i (v_i) = rows of `upstream`."""
    w = _params64(params)
    x = _f64(x)
    u = _f64(upstream)
    _, h, a = mlp_forward(x, w, keep=True)
    dW2 = a.T @ u
    db2 = u.sum(axis=0)
    da = u @ w["W2"].T
    dh = da * _gelu_prime(h)
    dW1 = x.T @ dh
    db1 = dh.sum(axis=0)
    return dict(W1=dW1, b1=db1, W2=dW2, b2=db2)


def _add(acc, g):
    for k in acc:
        acc[k] = acc[k] + g[k]
    return acc


def _zeros_like_params(params):
    return {k: np.zeros_like(_f64(params[k])) for k in ("W1", "b1", "W2", "b2")}


def round_to_bf16(a):
    """Round-to-nearest-even of every entry to the bf16 grid (8 significant bits),
    returned as float64.  Used for one stated storage precision: representations
    that a workload keeps in bf16 (Step 1 stores all representations).
    Pinned against torch's bfloat16 cast in the tests."""
    x = np.ascontiguousarray(np.asarray(a, dtype=np.float64).astype(np.float32))
    u = x.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape).astype(np.float64)


def _store(rep, rep_dtype):
    if rep_dtype is None:
        return rep
    assert rep_dtype == "bf16"
    return round_to_bf16(rep)


def mlp_fullbatch_grad(xq, xp, pos_idx, params, scale=1.0, temp=1.0, rep_dtype=None):
    """Direct large-batch update (Eq. 2-3): encode everything, loss, backprop
    all B + P rows at once.  rep_dtype="bf16": the loss sees representations
    rounded to their storage type (the gradient still flows through the
    un-rounded encoder, as it does when the cached rows are back-propagated)."""
    fq = _store(mlp_forward(xq, params), rep_dtype)
    gp = _store(mlp_forward(xp, params), rep_dtype)
    out = loss_and_rep_grad(fq, gp, pos_idx, scale, temp)
    grads = _zeros_like_params(params)
    _add(grads, mlp_backward(xq, params, out["dq"]))
    _add(grads, mlp_backward(xp, params, out["dp"]))
    return dict(loss=out["loss"], grads=grads, dq=out["dq"], dp=out["dp"], q=fq, p=gp)


def _chunks(n, size):
    return [(a, min(a + size, n)) for a in range(0, n, size)]


def mlp_chunked_grad(xq, xp, pos_idx, params, chunk_q, chunk_p, scale=1.0, temp=1.0, rep_dtype=None):
    """Gradient Cache, Steps 1-3: graph-less forward per sub-batch, loss and
    representation-gradient cache on the stored representations, then per
    sub-batch re-encode and backprop of the cached rows (Eq. 8-9).  Sub-batches
    are taken in index order; the last one may be short."""
    xq = _f64(xq)
    xp = _f64(xp)
    # Step 1
    fq = _store(np.concatenate([mlp_forward(xq[a:b], params) for a, b in _chunks(len(xq), chunk_q)]), rep_dtype)
    gp = _store(np.concatenate([mlp_forward(xp[a:b], params) for a, b in _chunks(len(xp), chunk_p)]), rep_dtype)
    # Step 2
    out = loss_and_rep_grad(fq, gp, pos_idx, scale, temp)
    u, v = out["dq"], out["dp"]          # the Representation Gradient Cache
    # Step 3
    grads = _zeros_like_params(params)
    for a, b in _chunks(len(xq), chunk_q):
        _add(grads, mlp_backward(xq[a:b], params, u[a:b]))
    for a, b in _chunks(len(xp), chunk_p):
        _add(grads, mlp_backward(xp[a:b], params, v[a:b]))
    return dict(loss=out["loss"], grads=grads, dq=u, dp=v, q=fq, p=gp)


def mlp_accumulation_grad(xq, xp, pos_idx, params, n_chunks, scale=1.0, temp=1.0):
    """Plain gradient accumulation (the paper's "Accumulation" system): each of
    n_chunks sub-batches sees only its own targets as negatives.  Used as a
    negative control: it must NOT equal the full-batch gradient (Introduction;
    the remark under Eq. 7).  Requires the layout r_i = (P/B) * i so that a
    contiguous split keeps every positive inside its chunk."""
    xq = _f64(xq)
    xp = _f64(xp)
    B, P = len(xq), len(xp)
    assert B % n_chunks == 0 and P % B == 0
    k = P // B
    r = np.asarray(pos_idx)
    assert np.array_equal(r, k * np.arange(B))
    cb = B // n_chunks
    grads = _zeros_like_params(params)
    loss = 0.0
    for c in range(n_chunks):
        qs = slice(c * cb, (c + 1) * cb)
        ps = slice(c * cb * k, (c + 1) * cb * k)
        sub = mlp_fullbatch_grad(xq[qs], xp[ps], k * np.arange(cb), params, scale, temp)
        loss += sub["loss"] / n_chunks
        for key in grads:
            grads[key] = grads[key] + sub["grads"][key] / n_chunks
    return dict(loss=loss, grads=grads)
