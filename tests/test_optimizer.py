"""AdamW step and learning-rate schedule of the library against the oracle (App. C)."""
import ctypes
import math

import numpy as np
import pytest

from paper_2402_04902_amd import binding, inputs
from paper_2402_04902_amd.inputs import DTYPE_BF16, DTYPE_F32, LayerSpec


def test_cosine_lr_host_function_matches_oracle():
    from oracle import optim_oracle as OO
    for total in (10, 1000, 25000):
        for step in list(range(0, min(total, 130))) + [total // 2, total - 1, total, total + 5]:
            got = binding.l4q_cosine_lr(step, total, 5e-5, 0.1)
            assert math.isclose(got, OO.cosine_lr(step, total, 5e-5, 0.1), rel_tol=2e-6, abs_tol=1e-12), (total, step)


def test_adamw_argument_checks():
    lib = binding.load_library()
    d = binding.make_desc(LayerSpec("x", 8, 256, 64, 4, 8.0, 4, 64, DTYPE_F32))
    hp = binding.L4QAdamW(1e-3, 0.9, 0.999, 1e-8, 0.01, 0)
    args = [16] * 10 + [None, None, None]
    assert lib.l4q_adamw_step(ctypes.byref(d), ctypes.byref(hp), *args) == -2      # step < 1
    hp.step = 1
    assert lib.l4q_adamw_step(ctypes.byref(d), ctypes.byref(hp), *([None] + [16] * 9 + [None, None, None])) == -1
    assert lib.l4q_adamw_step(ctypes.byref(d), ctypes.byref(hp), *([16] * 10 + [16, None, None])) == -4  # bf16 copy, fp32 desc


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [DTYPE_F32, DTYPE_BF16])
def test_adamw_steps_match_oracle(dtype):
    import torch
    from oracle import optim_oracle as OO
    spec = LayerSpec("adamw", 8, 512, 136, 8, 16.0, 4, 64, dtype)
    rng = np.random.default_rng(5)
    shapes = [(spec.rank, spec.in_features), (spec.out_features, spec.rank),
              (spec.out_features, spec.groups), (spec.out_features, spec.groups)]
    params = [rng.standard_normal(s).astype(np.float32) * 0.05 for s in shapes]
    n = sum(p.size for p in params)
    dev = torch.device("cuda:0")
    tp = [torch.from_numpy(p.copy()).to(dev) for p in params]
    m = torch.zeros(n, dtype=torch.float32, device=dev)
    v = torch.zeros(n, dtype=torch.float32, device=dev)
    copies = [torch.zeros(s, dtype=torch.bfloat16, device=dev) for s in shapes[:2]] if dtype == DTYPE_BF16 else [None, None]
    ref = [p.astype(np.float64) for p in params]
    rm = [np.zeros_like(p) for p in ref]
    rv = [np.zeros_like(p) for p in ref]
    desc = binding.make_desc(spec)
    for step in range(1, 6):
        grads = [(rng.standard_normal(s) * (10.0 ** int(rng.integers(-4, 0)))).astype(np.float32) for s in shapes]
        tg = [torch.from_numpy(g).to(dev) for g in grads]
        lr = binding.l4q_cosine_lr(step - 1, 20, 2e-3, 0.1)
        hp = binding.L4QAdamW(lr, 0.9, 0.999, 1e-8, 0.01, step)
        binding.l4q_adamw_step(desc, hp, *tp, *tg, m, v, *copies)
        torch.cuda.synchronize()
        for k in range(4):
            ref[k], rm[k], rv[k] = OO.adamw_step(ref[k], grads[k], rm[k], rv[k], lr, 0.9, 0.999, 1e-8, 0.01, step)
            got = tp[k].cpu().numpy().astype(np.float64)
            assert np.allclose(got, ref[k], rtol=2e-5, atol=1e-7), (step, k, np.abs(got - ref[k]).max())
    mm = m.cpu().numpy()
    assert np.allclose(mm, np.concatenate([x.ravel() for x in rm]), rtol=1e-5, atol=1e-9)
    if dtype == DTYPE_BF16:
        for k in range(2):
            assert torch.equal(copies[k], tp[k].to(torch.bfloat16))
