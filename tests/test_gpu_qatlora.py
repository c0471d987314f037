"""GPU parity of the QAT-LoRA layer (Sec. 3.1) against its oracle, through the C ABI."""
import numpy as np
import pytest

from paper_2402_04902_amd import inputs
from paper_2402_04902_amd.inputs import DTYPE_BF16, DTYPE_F32, LayerSpec

from parity_util import BOUNDS, compare_tensor

pytestmark = pytest.mark.gpu


def _run(spec, seed, shrink=0.8, accumulate=False):
    import torch
    from oracle import l4q_oracle as O
    from oracle import qatlora_oracle as Q
    from paper_2402_04902_amd import binding
    print(f"case {spec.name} T={spec.tokens} i={spec.in_features} o={spec.out_features} r={spec.rank} n={spec.bits} "
          f"g={spec.group_size} dtype={spec.dtype} seed={seed} accumulate={accumulate}", flush=True)
    arrs = inputs.make_layer_inputs(spec, seed)
    s, b = O.init_qparams(np.asarray(arrs["W0"], np.float64), spec.bits, spec.group_size, "asymm")
    s, b = (s * shrink).astype(np.float32), b.astype(np.float32)
    # decisions of the strict binary32 chain with the LoRA term switched off: the quantizer sees W0 alone
    dec, _, _ = O.decide_f32(arrs["W0"], arrs["A"], np.zeros_like(arrs["B"]), s, b, spec.bits, spec.group_size, spec.alpha)
    Y = Q.forward(arrs["X"], arrs["W0"], arrs["A"], arrs["B"], s, b, spec.bits, spec.group_size, spec.alpha, dec)
    gr = Q.backward(arrs["X"], arrs["dY"], arrs["W0"], arrs["A"], arrs["B"], s, b, spec.bits, spec.group_size,
                    spec.alpha, dec)
    layer = binding.upload(spec, arrs, s, b)
    fb, bb = binding.l4q_qatlora_workspace_bytes(layer.desc)
    ws = torch.empty(max(fb, bb), dtype=torch.uint8, device=layer.X.device)
    binding.l4q_qatlora_forward(layer.desc, layer.X, layer.W0, layer.A, layer.B, layer.scale, layer.zero, layer.Y, ws)
    args = (layer.X, layer.dY, layer.W0, layer.A, layer.B, layer.scale, layer.zero, layer.dX, layer.dA, layer.dB,
            layer.dscale, layer.dzero, ws)
    binding.l4q_qatlora_backward(layer.desc, *args)
    times = 1
    if accumulate:
        layer.desc.flags = binding.FLAG_ACCUMULATE_GRADS
        binding.l4q_qatlora_backward(layer.desc, *args)
        times = 2
    torch.cuda.synchronize()
    assert (~dec.mask).sum() > 0
    for name, got, ref in [("Y", layer.Y, Y), ("dX", layer.dX, gr.dX), ("dA", layer.dA, times * gr.dA),
                           ("dB", layer.dB, times * gr.dB), ("dscale", layer.dscale, times * gr.dscale),
                           ("dzero", layer.dzero, times * gr.dzero)]:
        # Y and dX are rounded twice in bfloat16 mode (main product, then the LoRA term): the L4Q bounds hold
        fro_tol, elem_tol = BOUNDS[spec.dtype][name]
        compare_tensor(spec.name + " " + name, got.double().cpu().numpy(), ref, fro_tol, elem_tol)
    return fb, bb


@pytest.mark.parametrize("dtype", [DTYPE_F32, DTYPE_BF16])
def test_qatlora_ragged(dtype):
    _run(LayerSpec("ql_ragged", 70, 200 if dtype == DTYPE_F32 else 320, 136, 3, 6.0, 4, 8 if dtype == DTYPE_BF16 else 4,
                   dtype, outliers=False), seed=21)


def test_qatlora_rank_above_one_chunk_and_accumulate():
    _run(LayerSpec("ql_r40", 130, 256, 72, 40, 80.0, 3, 64, DTYPE_BF16), seed=22, accumulate=True)
    _run(LayerSpec("ql_r40_f32", 33, 64, 24, 20, 40.0, 4, 16, DTYPE_F32), seed=23, accumulate=True)


def test_qatlora_mid_size_bf16_and_workspace_holds_the_weight_gradient():
    spec = LayerSpec("ql_mid", 512, 1024, 1536, 16, 32.0, 4, 128, DTYPE_BF16)
    fb, bb = _run(spec, seed=24)
    from paper_2402_04902_amd import binding
    _, l4q_bb = binding.l4q_workspace_bytes(binding.make_desc(spec))
    # the stored binary32 weight gradient alone is o * i * 4 bytes; the L4Q backward keeps no such array
    assert bb >= spec.out_features * spec.in_features * 4
    assert bb > l4q_bb
