"""Seeded synthetic inputs for the five workloads.

This module only draws random numbers and rounds them to the storage type.  It
holds none of the method's arithmetic, so both the HIP path and the CPU oracle
may take their inputs from it.  The paper measured on Natural Questions with
BERT encoders (Sec. Experiments); the path consumes only representation
matrices, so tensors with the paper's shapes (batch 128 with one positive and
one hard negative per question, batch 4096 from the Introduction, width 768)
stand in for them.

All generators return CPU torch tensors in the storage dtype (fp32 or bf16,
round-to-nearest-even).  `widen()` gives the exact float64 numpy view of a
stored tensor for the oracle.
"""
import numpy as np
import torch

SEED0 = 210106983


def _normal(rng, shape, std):
    return torch.from_numpy((rng.standard_normal(shape) * std).astype(np.float32))


def widen(t):
    """Exact float64 numpy copy of a stored (fp32 / bf16 / int) tensor."""
    if t.dtype in (torch.int32, torch.int64):
        return t.cpu().numpy().astype(np.int64)
    return t.detach().cpu().to(torch.float64).numpy()


def dpr_batch(B, P, d, dtype=torch.bfloat16, seed=SEED0 + 3, positive_mix=0.0, pos_idx=None):
    """Queries Q[B, d], passages P[P, d], entries iid N(0, variance 1/d).

    pos_idx defaults to r_i = (P // B) * i (P = 2B: passage 2i is the positive,
    2i + 1 the hard negative of query i).  positive_mix = m shifts each positive
    toward its query: p_{r_i} = m q_i + (1 - m) eps.
    """
    rng = np.random.default_rng(seed)
    std = d ** -0.5
    q = _normal(rng, (B, d), std)
    p = _normal(rng, (P, d), std)
    if pos_idx is None:
        k = max(P // B, 1)
        pos_idx = torch.arange(B, dtype=torch.int32) * k
        pos_idx = torch.clamp(pos_idx, max=P - 1)
    else:
        pos_idx = torch.as_tensor(pos_idx, dtype=torch.int32)
    if positive_mix != 0.0:
        idx = pos_idx.long()
        p[idx] = positive_mix * q + (1.0 - positive_mix) * p[idx]
    return q.to(dtype), p.to(dtype), pos_idx


def config1():
    """Tiny DPR-style: B=8, P=16, d=64, fp32."""
    return dpr_batch(8, 16, 64, torch.float32, SEED0 + 1)


def config2():
    """DPR-shaped: B=128, P=256, d=768, bf16, positives p = 0.5 q + 0.5 eps."""
    return dpr_batch(128, 256, 768, torch.bfloat16, SEED0 + 2, positive_mix=0.5)


def config3():
    """Large-batch ICT-shaped: B=4096, P=8192, d=768, bf16."""
    return dpr_batch(4096, 8192, 768, torch.bfloat16, SEED0 + 3)


def ntxent_views(n_views=16384, d=128, dtype=torch.bfloat16, seed=SEED0 + 4):
    """Config 4: rows iid N(0,1), L2-normalised in fp32, then rounded."""
    rng = np.random.default_rng(seed)
    z = _normal(rng, (n_views, d), 1.0)
    z = z / z.norm(dim=1, keepdim=True)
    return z.to(dtype)


def mlp_problem(B=512, P=1024, din=1024, dh=3072, dout=768, dtype=torch.bfloat16, seed=SEED0 + 5):
    """Config 5: inputs iid N(0,1); weights and biases ~ N(0, std 0.02)."""
    rng = np.random.default_rng(seed)
    xq = _normal(rng, (B, din), 1.0).to(dtype)
    xp = _normal(rng, (P, din), 1.0).to(dtype)
    params = dict(
        W1=_normal(rng, (din, dh), 0.02).to(dtype),
        b1=_normal(rng, (dh,), 0.02).to(dtype),
        W2=_normal(rng, (dh, dout), 0.02).to(dtype),
        b2=_normal(rng, (dout,), 0.02).to(dtype),
    )
    k = max(P // B, 1)
    pos_idx = torch.clamp(torch.arange(B, dtype=torch.int32) * k, max=P - 1)
    return xq, xp, pos_idx, params


def bilinear_omega(d, dtype=torch.bfloat16, seed=SEED0 + 6, noise=0.5):
    """Parameter matrix of the bilinear distance: the identity (the dot product of the main text) plus
    `noise` times an iid N(0, 1/d) matrix, rounded to the storage type."""
    rng = np.random.default_rng(seed)
    return (torch.eye(d) + noise * _normal(rng, (d, d), d ** -0.5)).to(dtype)


def deep_omega(d, h=128, dtype=torch.bfloat16, seed=SEED0 + 7):
    """Parameters of the deep distance Phi = sum_k w_k tanh((A f)_k + (C g)_k): A, C [h, d] iid N(0, 1) (with
    representation entries of variance 1/d the pre-activations then have variance about 2), w [h] iid N(0, 1/h),
    rounded to the storage type."""
    rng = np.random.default_rng(seed)
    return dict(A=_normal(rng, (h, d), 1.0).to(dtype), C=_normal(rng, (h, d), 1.0).to(dtype),
                w=_normal(rng, (h,), h ** -0.5).to(dtype))
