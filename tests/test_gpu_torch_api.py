"""End to end with real autograd gradients: K small torch models trained with the
LASGD wrapper on the GPU; the oracle is fed the very gradients autograd
produced (copied to the host each step) and must land on the same parameters."""
import copy

import numpy as np
import pytest
import torch

from oracle import lasgd_oracle as O32
from paper_2203_13085_amd import binding as B
from tests.parity_util import assert_close

pytestmark = pytest.mark.gpu


def _flat(tensors):
    return np.concatenate([t.detach().float().cpu().numpy().ravel() for t in tensors])


@pytest.mark.parametrize("m", [1, 3])
def test_k_models_with_autograd_gradients(m):
    from paper_2203_13085_amd.torch_api import LASGD
    torch.manual_seed(0)
    dev = torch.device("cuda:0")
    K, steps, lr, mu, wd = 3, 9, 0.05, 0.9, 1e-3
    base = torch.nn.Sequential(torch.nn.Linear(20, 33), torch.nn.ReLU(), torch.nn.Linear(33, 5)).to(dev)
    replicas = [copy.deepcopy(base) for _ in range(K)]
    opt = LASGD(replicas, lr=lr, momentum=mu, nesterov=True, weight_decay=wd, m=m, no_decay_1d=True)
    params0 = [p for p in base.parameters()]
    numels = [p.numel() for p in params0]
    wds = [0.0 if p.dim() <= 1 else wd for p in params0]
    orc = O32.Oracle(K, numels, mu, True, wds)
    orc.set_model(_flat(params0))
    try:
        started, tau = False, 0
        for step in range(steps):
            opt.zero_grad()
            for k, model in enumerate(replicas):
                g = torch.Generator(device=dev); g.manual_seed(1000 * step + k)
                x = torch.randn(16, 20, generator=g, device=dev)
                y = torch.randn(16, 5, generator=g, device=dev)
                torch.nn.functional.mse_loss(model(x), y).backward()
            torch.cuda.synchronize()
            grads = [_flat([p.grad for p in model.parameters()]) for model in replicas]
            fired = opt.step()
            orc.local_step(grads, lr)
            if not started:
                orc.snapshot(); orc.average(); started = True
                assert not fired
            else:
                tau += 1
                if tau == m:
                    orc.merge(True); orc.average(); tau = 0
                    assert fired
                else:
                    assert not fired
            torch.cuda.synchronize()
            for k, model in enumerate(replicas):
                assert_close(_flat(list(model.parameters())), orc.x[k], f"step {step} replica {k}")
        assert_close(opt.center().numpy(), orc.z, "centre")
        # replicas have moved apart and back: they differ, but not by much
        a, b = _flat(list(replicas[0].parameters())), _flat(list(replicas[1].parameters()))
        assert 0 < np.abs(a - b).max() < 0.5
    finally:
        opt.close()
