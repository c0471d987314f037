"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element,
on the same seeded inputs.  Integer codes, masks and the merged weight must match bit for bit;
floating-point outputs within 1e-4 (binary32 mode) / 2e-2 (bfloat16 I/O) Frobenius-relative."""
import json
import os

import numpy as np
import pytest

from paper_2402_04902_amd import inputs
from paper_2402_04902_amd.inputs import DTYPE_BF16, DTYPE_F32, LayerSpec

from parity_util import (BOUNDS, check_discrete, check_float_outputs, check_workspace_state, compare_tensor,
                         host_qparams, oracle_all)

pytestmark = pytest.mark.gpu

FUSED_MAX_RANK = 32   # ranks the fused weight-gradient epilogue covers

# optional: a file that collects one JSON line of measured errors per case
REPORT = os.environ.get("L4Q_PARITY_REPORT", "")


def run_case(spec, seed=0, method="asymm", shrink=1.0, flags=0, mutate=None, discrete=True):
    import torch
    from paper_2402_04902_amd import binding
    print(f"case {spec.name} T={spec.tokens} i={spec.in_features} o={spec.out_features} r={spec.rank} "
          f"n={spec.bits} g={spec.group_size} dtype={spec.dtype} seed={seed} init={method} shrink={shrink} "
          f"flags={flags}", flush=True)
    arrs = inputs.make_layer_inputs(spec, seed)
    if mutate is not None:
        mutate(arrs)
    s, b = host_qparams(spec, arrs, method, shrink)
    dec, Wc32, w32, Y, gr = oracle_all(spec, arrs, s, b)
    layer = binding.upload(spec, arrs, s, b, flags=flags)
    rep = {"case": spec.name, "init": method, "shrink": shrink, "flags": flags,
           "clipped": int((~dec.mask).sum()), "elements": int(dec.mask.size)}
    if discrete:
        rep.update(check_discrete(spec, layer, arrs, s, b, dec, Wc32))
    layer.forward()
    layer.backward()
    torch.cuda.synchronize()
    check_float_outputs(spec, layer, Y, gr, rep)
    if spec.dtype == DTYPE_BF16:
        # the factor array survives the call only where the epilogue forms dA / dB itself (rank <= 32)
        fused = (flags & binding.FLAG_UNFUSED_BACKWARD) == 0 and spec.rank <= FUSED_MAX_RANK and \
            spec.group_size in (32, 64, 128, 256)
        check_workspace_state(spec, layer, dec, w32, s, b, fused)
    if REPORT:
        try:
            with open(REPORT, "a") as f:
                f.write(json.dumps(rep) + "\n")
        except OSError:
            pass
    print("   ", rep, flush=True)
    return rep, layer, gr


# ------------------------------------------------------------------ configuration 1 (binary32)

@pytest.mark.parametrize("method,shrink", [("asymm", 1.0), ("asymm", 0.8), ("l4q", 1.0)])
def test_config1_fp32(method, shrink):
    rep, _, _ = run_case(inputs.config1()[0], seed=0, method=method, shrink=shrink)
    if shrink < 1.0:
        assert rep["clipped"] > 0


def test_fp32_ragged_shapes():
    run_case(LayerSpec("f32_ragged", 37, 96, 50, 3, 6.0, 4, 32, DTYPE_F32, outliers=False), seed=3, shrink=0.7)
    run_case(LayerSpec("f32_rank20", 130, 192, 70, 20, 10.0, 3, 64, DTYPE_F32), seed=4, shrink=0.8)
    run_case(LayerSpec("f32_one_token", 1, 64, 9, 1, 2.0, 8, 4, DTYPE_F32), seed=5, shrink=0.9)


# ------------------------------------------------------------------ bfloat16, several tiles + ragged tails

@pytest.mark.parametrize("T,i,o,r,bits,g", [
    (300, 640, 264, 16, 4, 128),     # nothing a multiple of the 256 tile; T not a multiple of 8
    (1000, 1024, 520, 4, 3, 64),
    (513, 768, 1032, 20, 4, 256),    # rank above one register chunk
    (64, 512, 8, 1, 2, 32),          # one row block, rank 1, 2 bits
    (777, 2048, 776, 8, 8, 2048),    # one group per row
    (70, 40, 24, 2, 4, 8),           # in-features not a multiple of the 32-wide k-step, tiny group
    (45, 200, 136, 4, 4, 8),
])
@pytest.mark.parametrize("shrink", [1.0, 0.8])
def test_bf16_small_shapes(T, i, o, r, bits, g, shrink):
    spec = LayerSpec(f"bf16_{T}x{i}x{o}", T, i, o, r, 2.0 * r, bits, g, DTYPE_BF16)
    rep, _, _ = run_case(spec, seed=T, shrink=shrink)
    if shrink < 1.0:
        assert rep["clipped"] > 0


@pytest.mark.parametrize("T,i,o,r,bits,g", [
    (33, 96, 40, 8, 4, 32),        # one and a half 64-column strips, two groups per strip, a partial row block
    (70, 160, 72, 24, 3, 32),      # rank = one and a half chunks of 16; in-features not a multiple of 64
    (129, 320, 200, 72, 4, 64),    # five rank chunks (the last half full), 6.25 row blocks
    (40, 1088, 24, 16, 8, 64),     # 4.25 column tiles of 256, fewer rows than one row block
    (64, 2048, 1000, 16, 2, 2048), # one group per row, 31.25 row blocks: uneven runs per wavefront
    (17, 64, 8, 8, 4, 64),         # the smallest: one strip, one partial row block
])
@pytest.mark.parametrize("shrink", [1.0, 0.7])
def test_bf16_streaming_merge_edges(T, i, o, r, bits, g, shrink):
    """Shapes at the edges of the streaming merge + quantize kernel (64-column strips, 32-row blocks, rank chunks of
    16, one or two groups per strip): codes / mask / merged weight through the export form, Wq / Wq^T / factor through
    the workspace, all bit for bit, plus the float outputs."""
    spec = LayerSpec(f"bf16_stream_{T}x{i}x{o}_r{r}", T, i, o, r, 2.0 * r, bits, g, DTYPE_BF16)
    rep, _, _ = run_case(spec, seed=i + r, shrink=shrink)
    if shrink < 1.0:
        assert rep["clipped"] > 0


def test_bf16_scale_outside_the_reciprocal_range_takes_the_ieee_divide():
    """Scales below 2^-60 (and zeros of the same order) leave the range in which the streaming kernel divides by
    multiplication; the wave-uniform fallback must give the same bits as the oracle's division."""
    def tiny(arrs):
        for k in ("W0", "B"):
            arrs[k] *= np.float32(2.0 ** -70)
            arrs[k][...] = inputs.round_to_bf16(arrs[k])
    spec = LayerSpec("bf16_tiny_scales", 64, 256, 72, 8, 16.0, 4, 64, DTYPE_BF16)
    arrs = inputs.make_layer_inputs(spec, 3)
    tiny(arrs)
    from oracle import l4q_oracle as O
    s, _ = host_qparams(spec, arrs, "asymm", 0.8)
    assert s.max() < 2.0 ** -60 and s.min() > 0
    rep, _, _ = run_case(spec, seed=3, shrink=0.8, mutate=tiny)
    assert rep["clipped"] > 0


def _random_cases(count=16, seed=2402):
    """Seeded draw of layer shapes: group a power of two, in-features a multiple of it, ranks on both sides of the
    fused epilogue's limit, every code width, both storage types, scale shrunk so that some weights clip."""
    rng = np.random.default_rng(seed)
    cases = []
    for k in range(count):
        bf16 = k % 3 != 0
        g = int(rng.choice([8, 16, 32, 64, 128, 256] if bf16 else [4, 8, 32, 64]))
        i = g * int(rng.integers(1, 13 if g <= 64 else 7))
        o = 8 * int(rng.integers(1, 90)) if bf16 else int(rng.integers(1, 300))
        T = int(rng.integers(1, 600))
        r = int(rng.choice([1, 4, 8, 16, 64]))
        bits = int(rng.choice([2, 3, 4, 8]))
        shrink = float(rng.choice([1.0, 0.8, 0.6]))
        cases.append((k, T, i, o, r, bits, g, DTYPE_BF16 if bf16 else DTYPE_F32, shrink))
    return cases


@pytest.mark.parametrize("k,T,i,o,r,bits,g,dtype,shrink", _random_cases())
def test_random_shapes(k, T, i, o, r, bits, g, dtype, shrink):
    spec = LayerSpec(f"rand{k}_{T}x{i}x{o}", T, i, o, r, 2.0 * r, bits, g, dtype)
    rep, _, _ = run_case(spec, seed=1000 + k, shrink=shrink)
    if shrink < 1.0:
        assert rep["clipped"] > 0


def _random_mid_cases(count=14, seed=4902):
    """Seeded draw of bfloat16 layers of a few hundred to a few thousand features: long k ranges at few tokens (the
    k-split forward / dX products, with and without a row tail), ranks on both sides of 16 and of 32 (streaming merge
    kernel with and without further rank chunks, both forms of the weight-gradient epilogue, k-split dA / dB
    products), out-features that are not whole row blocks."""
    rng = np.random.default_rng(seed)
    cases = []
    for k in range(count):
        g = int(rng.choice([32, 64, 128, 256]))
        i = g * int(rng.integers(max(1, 512 // g), 4096 // g + 1))
        o = 8 * int(rng.integers(32, 513))
        T = int(rng.choice([1, 17, 64, 100, 256, 300, 700, 1100]))
        r = int(rng.choice([8, 16, 24, 40, 64, 96]))
        if r > 32 and i % 32 != 0:
            r = 16
        bits = int(rng.choice([3, 4]))
        shrink = float(rng.choice([1.0, 0.8]))
        cases.append((k, T, i, o, r, bits, g, shrink))
    return cases


@pytest.mark.parametrize("k,T,i,o,r,bits,g,shrink", _random_mid_cases())
def test_random_mid_size_bf16_shapes(k, T, i, o, r, bits, g, shrink):
    spec = LayerSpec(f"mid{k}_{T}x{i}x{o}_r{r}", T, i, o, r, 2.0 * r, bits, g, DTYPE_BF16)
    run_case(spec, seed=2000 + k, shrink=shrink)


@pytest.mark.parametrize("T,i,o,r,bits,g", [(300, 640, 264, 16, 4, 128), (513, 768, 1032, 8, 4, 64)])
def test_bf16_unfused_backward_flag(T, i, o, r, bits, g):
    """The unfused backward (dWq through the workspace) must agree with the oracle as well."""
    from paper_2402_04902_amd import binding
    spec = LayerSpec(f"bf16_unfused_{T}x{i}x{o}", T, i, o, r, 2.0 * r, bits, g, DTYPE_BF16)
    run_case(spec, seed=T + 1, shrink=0.8, flags=binding.FLAG_UNFUSED_BACKWARD, discrete=False)


@pytest.mark.parametrize("r,T,i,o,g", [(40, 200, 512, 264, 128), (64, 300, 1024, 520, 64), (128, 513, 768, 1032, 256),
                                       (256, 70, 256, 136, 32), (48, 45, 200, 136, 8), (36, 64, 512, 264, 128)])
def test_bf16_ranks_above_32(r, T, i, o, g):
    """Ranks of the paper's rank sweep beyond 32 (App. D): the weight-gradient kernel keeps d(scale) / d(zero) in its
    epilogue and hands the masked gradient on as bfloat16 for the two thin dA / dB products; no binary32 weight
    gradient is stored (the backward workspace stays below what the unfused path asks for by more than o i 2 bytes).
    In-features 200 (not a multiple of 32), group 8 and rank 36 (not a multiple of 8) take the unfused kernels."""
    from paper_2402_04902_amd import binding
    spec = LayerSpec(f"bf16_rank{r}", T, i, o, r, 2.0 * r, 4, g, DTYPE_BF16)
    run_case(spec, seed=r, shrink=0.8)
    _, bwd = binding.l4q_workspace_bytes(binding.make_desc(spec))
    _, bwd_unfused = binding.l4q_workspace_bytes(binding.make_desc(spec, binding.FLAG_UNFUSED_BACKWARD))
    if i % 32 == 0 and g >= 32 and r % 8 == 0:
        assert bwd < bwd_unfused - o * i * 2 + 4 * r * (i + o) + 4096
    else:
        assert bwd == bwd_unfused


def test_bf16_zero_B_is_plain_qat_and_kills_dA():
    """The paper initialises B = 0: the layer is then plain group-wise QAT of W0 and dA vanishes."""
    def zero_b(arrs):
        arrs["B"][...] = 0.0
    spec = LayerSpec("bf16_zeroB", 256, 512, 256, 8, 16.0, 4, 128, DTYPE_BF16)
    _, layer, _ = run_case(spec, seed=11, shrink=0.8, mutate=zero_b)
    assert float(layer.dA.abs().max()) == 0.0


def test_bf16_fully_clipped_groups():
    """A tiny scale clips every element of some groups: only the Q_N / Q_P branches contribute."""
    spec = LayerSpec("bf16_allclip", 128, 256, 64, 4, 8.0, 4, 64, DTYPE_BF16)
    rep, layer, gr = run_case(spec, seed=12, shrink=1e-3)
    assert rep["clipped"] > 0.9 * rep["elements"]


# ------------------------------------------------------------------ the published configurations at their stated
# sizes (whole tensors), each in the initial state (min/max scales: nothing clips, two weights per group sit on the
# grid ends) and in a clipped state (scales shrunk to 0.8: what training moves towards)

STATES = [1.0, 0.8]


def _full_case(spec, seed, shrink):
    rep, _, _ = run_case(spec, seed=seed, shrink=shrink)
    if shrink < 1.0:
        assert rep["clipped"] > 0
    else:
        assert rep["near_boundaries"] >= 2 * spec.out_features * spec.groups * 0.9


@pytest.mark.parametrize("shrink", STATES)
def test_config2_full_size(shrink):
    _full_case(inputs.config2()[0], 0, shrink)


@pytest.mark.parametrize("shrink", STATES)
@pytest.mark.parametrize("idx", [0, 1])
def test_config3_full_size(idx, shrink):
    _full_case(inputs.config3()[idx], idx, shrink)


@pytest.mark.parametrize("shrink", STATES)
@pytest.mark.parametrize("idx", [0, 1, 2, 3])
def test_config4_three_bit_full_size(idx, shrink):
    """3 bits, T = 4096: up and down projection at g = 128, the up projection at g = 64 and g = 256."""
    _full_case(inputs.config4()[idx], 40 + idx, shrink)


@pytest.mark.parametrize("shrink", STATES)
@pytest.mark.parametrize("idx", range(7))
def test_config5_mistral_block_full_size(idx, shrink):
    """All seven linear layers of the Mistral-7B-shaped block at T = 8192: q, k, v, o, gate, up, down."""
    _full_case(inputs.config5()[idx], 50 + idx, shrink)


def test_larger_model_shapes():
    """Projections of larger models than the benchmark's (13B-class up projection, 70B-class down projection): operands of
    0.14 and 0.47 GB, the largest the 32-bit byte offsets of the matrix-core kernels are asked to address here."""
    run_case(LayerSpec("up_5120x13824_T256", 256, 5120, 13824, 16, 32.0, 4, 128, DTYPE_BF16), seed=13, shrink=0.8)
    run_case(LayerSpec("down_28672x8192_T64", 64, 28672, 8192, 16, 32.0, 4, 128, DTYPE_BF16), seed=70, shrink=0.8)


def test_bf16_few_tokens_split_k_with_a_k_tail():
    """The k-split forward / dX products where the caller's rows end inside the last slice (1032 and 1096 features:
    multiples of 8, not of 32)."""
    run_case(LayerSpec("split_k_tail_1096x1032_T70", 70, 1032, 1096, 8, 16.0, 4, 8, DTYPE_BF16), seed=95, shrink=0.8)


@pytest.mark.parametrize("tokens", [256, 200, 1000])
def test_bf16_few_tokens_split_k(tokens):
    """Benchmark layers at token counts whose forward / dX products have too few tiles for the chip (one to four tile
    rows): the k range is split over workgroups and the slices are added in a fixed order.  200 and 1000: ragged last
    tile row.  Run twice: the same bits."""
    import torch
    for idx, (o, i) in enumerate(((11008, 4096), (4096, 11008))):
        spec = LayerSpec(f"split_k_{o}x{i}_T{tokens}", tokens, i, o, 16, 32.0, 4, 128, DTYPE_BF16)
        _, layer, _ = run_case(spec, seed=90 + idx, shrink=0.8, discrete=False)
        y1, dx1 = layer.Y.clone(), layer.dX.clone()
        layer.forward()
        layer.backward()
        torch.cuda.synchronize()
        assert torch.equal(y1.view(torch.int16), layer.Y.view(torch.int16))
        assert torch.equal(dx1.view(torch.int16), layer.dX.view(torch.int16))


# ------------------------------------------------------------------ initialisation kernel

@pytest.mark.parametrize("dtype", [DTYPE_F32, DTYPE_BF16])
@pytest.mark.parametrize("method,mid", [("asymm", 0), ("symm", 1), ("l4q", 2)])
def test_init_qparams_bit_exact(dtype, method, mid):
    import torch
    from oracle import l4q_oracle as O
    from paper_2402_04902_amd import binding
    for g in (32, 128, 512):
        spec = LayerSpec(f"init_{method}_g{g}", 8, 1024, 72, 8, 16.0, 4, g, dtype)
        print("case", spec.name, "dtype", dtype, flush=True)
        arrs = inputs.make_layer_inputs(spec, seed=g)
        layer = binding.upload(spec, arrs)
        binding.l4q_init_qparams(layer.desc, layer.W0, layer.A, layer.B, mid, layer.scale, layer.zero)
        torch.cuda.synchronize()
        Wc32 = O.merge_f32(arrs["W0"], arrs["A"], arrs["B"], spec.alpha)
        s, b = O.init_qparams(Wc32, spec.bits, g, method, dtype=np.float32)
        assert np.array_equal(layer.scale.cpu().numpy().view(np.uint32), s.view(np.uint32))
        assert np.array_equal(layer.zero.cpu().numpy().view(np.uint32), b.view(np.uint32))
        # and the float64 formulas within rounding
        s64, b64 = O.init_qparams(O.merge(arrs["W0"], arrs["A"], arrs["B"], spec.alpha), spec.bits, g, method)
        assert np.allclose(s, s64, rtol=1e-5, atol=0) and np.allclose(b, b64, rtol=1e-4, atol=1e-7)


@pytest.mark.parametrize("dtype", [DTYPE_F32, DTYPE_BF16])
def test_init_lsqplus_and_error_sums(dtype):
    """LSQ+ initialisation (App. B) within binary32 rounding of the oracle; E_quant / E_clip sums of the
    resulting (clipping) state against the oracle's float64 sums."""
    import torch
    from oracle import l4q_oracle as O
    from paper_2402_04902_amd import binding
    for g in (32, 128, 256):
        spec = LayerSpec(f"lsqplus_g{g}", 8, 1280, 200, 8, 16.0, 4, g, dtype)
        print("case", spec.name, "dtype", dtype, flush=True)
        arrs = inputs.make_layer_inputs(spec, seed=g + 1)
        layer = binding.upload(spec, arrs)
        binding.l4q_init_qparams(layer.desc, layer.W0, layer.A, layer.B, binding.INIT_LSQPLUS, layer.scale, layer.zero)
        torch.cuda.synchronize()
        Wc = O.merge(arrs["W0"], arrs["A"], arrs["B"], spec.alpha)
        s64, b64 = O.init_qparams(Wc, spec.bits, g, "lsq+")
        s_gpu = layer.scale.cpu().numpy()
        assert np.allclose(s_gpu, s64, rtol=2e-5, atol=0)
        assert not layer.zero.cpu().numpy().any() and not b64.any()
        # error sums with the GPU's own (float32) scales: LSQ+ clips the outliers
        errors = torch.zeros(4, dtype=torch.float32, device=layer.W0.device)
        ws = torch.empty(spec.out_features * ((spec.in_features + 255) // 256) * 8, dtype=torch.uint8,
                         device=layer.W0.device)
        binding.l4q_quant_errors(layer.desc, layer.W0, layer.A, layer.B, layer.scale, layer.zero, errors, ws)
        torch.cuda.synchronize()
        e = errors.cpu().numpy()
        eq = O.quantization_error(Wc, s_gpu, b64, spec.bits, g)
        ec = O.clipping_error(Wc, s_gpu, b64, spec.bits, g)
        assert ec > 0
        assert abs(e[0] - eq) <= 1e-4 * eq and abs(e[1] - ec) <= 1e-4 * ec, (e, eq, ec)


# ------------------------------------------------------------------ run-to-run reproducibility

def test_backward_is_bit_reproducible():
    import torch
    from paper_2402_04902_amd import binding
    spec = LayerSpec("repro", 512, 1024, 512, 16, 32.0, 4, 128, DTYPE_BF16)
    arrs = inputs.make_layer_inputs(spec, 21)
    s, b = host_qparams(spec, arrs, "asymm", 0.8)
    layer = binding.upload(spec, arrs, s, b)
    outs = []
    for _ in range(2):
        layer.forward()
        layer.backward()
        torch.cuda.synchronize()
        outs.append([t.clone() for t in (layer.Y, layer.dX, layer.dA, layer.dB, layer.dscale, layer.dzero)])
    for a, c in zip(*outs):
        assert torch.equal(a, c)


# ------------------------------------------------------------------ gradient accumulation over micro-batches

@pytest.mark.parametrize("dtype,flags", [(DTYPE_F32, 0), (DTYPE_BF16, 0), (DTYPE_BF16, 1)])
def test_backward_accumulates_parameter_gradients(dtype, flags):
    """Two micro-batches: the second backward call carries the accumulate flag.  dA, dB, dscale, dzero must hold the
    oracle's sum of both contributions, dX the second micro-batch's alone."""
    import torch
    from paper_2402_04902_amd import binding
    spec = LayerSpec("accum", 70, 256, 264, 4, 8.0, 4, 64, dtype)
    print("case", spec.name, "dtype", dtype, "flags", flags, flush=True)
    a1 = inputs.make_layer_inputs(spec, seed=11)
    a2 = dict(a1)
    other = inputs.make_layer_inputs(spec, seed=12)
    a2["X"], a2["dY"] = other["X"], other["dY"]          # same parameters, another micro-batch
    s, b = host_qparams(spec, a1, "asymm", 0.8)
    _, _, _, _, g1 = oracle_all(spec, a1, s, b)
    _, _, _, _, g2 = oracle_all(spec, a2, s, b)
    layer = binding.upload(spec, a1, s, b, flags=flags)
    layer.backward()
    layer.X.copy_(torch.from_numpy(a2["X"]).to(layer.X.device).to(layer.X.dtype))
    layer.dY.copy_(torch.from_numpy(a2["dY"]).to(layer.dY.device).to(layer.dY.dtype))
    layer.desc.flags = flags | binding.FLAG_ACCUMULATE_GRADS
    layer.backward()
    torch.cuda.synchronize()
    for name, got, ref in [("dA", layer.dA, g1.dA + g2.dA), ("dB", layer.dB, g1.dB + g2.dB),
                           ("dscale", layer.dscale, g1.dscale + g2.dscale), ("dzero", layer.dzero, g1.dzero + g2.dzero),
                           ("dX", layer.dX, g2.dX)]:
        compare_tensor(name, got.double().cpu().numpy(), ref, *BOUNDS[dtype][name])


# ------------------------------------------------------------------ maximum operand sizes of the bf16 path

@pytest.mark.parametrize("name,T,i,o", [
    ("max_tokens_x_out", 32768, 64, 16344),    # Y and dY just below the 2^29 - 2^20 element limit (1 GiB of bf16)
    ("max_out_x_in", 8, 32768, 16320),         # W0, Wq, Wq^T (rows padded to a multiple of 32), the fp16 factor just below it
])
def test_bf16_largest_operands(name, T, i, o):
    """Byte offsets of the matrix-core kernels are 32-bit: operands of the largest accepted size must still be
    addressed correctly at their far end.  Whole-tensor comparison against the oracle."""
    assert T * o < (1 << 29) - (1 << 20) and (o + 31) // 32 * 32 * i < (1 << 29) - (1 << 20)
    spec = LayerSpec(name, T, i, o, 2, 4.0, 4, 32, DTYPE_BF16, outliers=False)
    run_case(spec, seed=5, shrink=0.8, discrete=False)
    from paper_2402_04902_amd import binding
    big = inputs.LayerSpec(name, T, i, o + 8, 2, 4.0, 4, 32, DTYPE_BF16) if name == "max_tokens_x_out" else \
        inputs.LayerSpec(name, T, i, o + 32, 2, 4.0, 4, 32, DTYPE_BF16)
    with pytest.raises(RuntimeError):
        binding.l4q_workspace_bytes(binding.make_desc(big))   # one step further is rejected, not mis-addressed


# ------------------------------------------------------------------ a non-finite row stays in its own row

@pytest.mark.parametrize("i,o", [(264, 136), (1032, 1096)])
def test_bf16_non_finite_row_does_not_reach_its_neighbours(i, o):
    """In- and out-features that are multiples of 8 but not of the 32-wide k-step of the matrix-core kernels (the
    second pair long enough for the few-token form that splits the k range over workgroups: the rows' ends then lie
    inside the last slice).  An Inf planted in one row of X (or dY) must poison that row of Y (dX) only: all other
    rows stay bit for bit what they were."""
    import torch
    from paper_2402_04902_amd import binding
    spec = LayerSpec(f"bf16_k_tail_{i}x{o}", 70, i, o, 4, 8.0, 4, 8, DTYPE_BF16)
    print("case", spec.name, flush=True)
    arrs = inputs.make_layer_inputs(spec, seed=9)
    s, b = host_qparams(spec, arrs, "asymm", 0.8)
    layer = binding.upload(spec, arrs, s, b)
    layer.forward()
    layer.backward()
    torch.cuda.synchronize()
    Y0, dX0 = layer.Y.clone(), layer.dX.clone()
    layer.X[5, :] = float("inf")
    layer.dY[9, :] = float("inf")
    layer.forward()
    layer.backward()
    torch.cuda.synchronize()
    keep_y = [t for t in range(spec.tokens) if t != 5]
    keep_dx = [t for t in range(spec.tokens) if t != 9]
    assert torch.equal(layer.Y[keep_y].view(torch.int16), Y0[keep_y].view(torch.int16))
    assert torch.equal(layer.dX[keep_dx].view(torch.int16), dX0[keep_dx].view(torch.int16))
    assert not torch.isfinite(layer.Y[5].float()).all() and not torch.isfinite(layer.dX[9].float()).all()
