"""GPU parity of the NT-Xent entry point against the fp64 oracle."""
import math

import pytest
import torch

from oracle import gc_oracle as O
from paper_2101_06983_amd import binding as gc
from paper_2101_06983_amd import synth
from parity import TOL_BF16, check, check_loss, relerr, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("n,d,tau", [(512, 128, 0.07), (130, 128, 0.5), (66, 64, 0.2), (1000, 256, 0.1),
                                     (300, 384, 0.2), (258, 512, 0.1), (192, 640, 0.5), (700, 768, 0.07),
                                     (2, 128, 0.5), (4100, 128, 0.1)])
def test_ntxent_small(n, d, tau):
    z = synth.ntxent_views(n, d, seed=4000 + n)
    want = O.ntxent(synth.widen(z), tau)
    loss, dz = gc.gc_ntxent_loss_and_grad_bf16(z.to(DEV), tau)
    torch.cuda.synchronize()
    check_loss("ntxent n=%d d=%d loss" % (n, d), loss.item(), want["loss"], TOL_BF16)
    check("ntxent n=%d d=%d dz" % (n, d), relerr(to_np(dz), want["dz"]), TOL_BF16)


def test_config4_full_size():
    z = synth.ntxent_views()
    tau = 0.07
    want = O.ntxent(synth.widen(z), tau)
    assert abs(want["loss"] - (math.log(16383) + 1 / (2 * 128 * tau * tau))) < 0.1
    loss, dz = gc.gc_ntxent_loss_and_grad_bf16(z.to(DEV), tau)
    torch.cuda.synchronize()
    check_loss("config4 loss", loss.item(), want["loss"], TOL_BF16)
    check("config4 dz", relerr(to_np(dz), want["dz"]), TOL_BF16)
    loss2, dz2 = gc.gc_ntxent_loss_and_grad_bf16(z.to(DEV), tau)
    torch.cuda.synchronize()
    assert torch.equal(dz, dz2) and loss.item() == loss2.item()
