"""GPU parity of the fully quantized layer: packed export (bit-exact) and the forward pass that uses
only the packed codes, scale and zero (Sec. 3.2), against the oracle and against the training forward."""
import numpy as np
import pytest

from paper_2402_04902_amd import inputs
from paper_2402_04902_amd.inputs import DTYPE_BF16, DTYPE_F32, LayerSpec

from parity_util import compare_tensor, host_qparams, rel_fro

pytestmark = pytest.mark.gpu


def packed_on_gpu(spec, layer):
    import torch
    from paper_2402_04902_amd import binding
    o, i = spec.out_features, spec.in_features
    packed = torch.empty((o, spec.bits * i // 32), dtype=torch.int32, device=layer.W0.device)
    ws = torch.empty(o * i, dtype=torch.uint8, device=layer.W0.device)
    binding.l4q_export_packed(layer.desc, layer.W0, layer.A, layer.B, layer.scale, layer.zero, packed, ws)
    torch.cuda.synchronize()
    return packed


@pytest.mark.parametrize("dtype", [DTYPE_F32, DTYPE_BF16])
@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_packed_export_bit_exact(dtype, bits):
    from oracle import l4q_oracle as O
    from paper_2402_04902_amd import binding
    spec = LayerSpec(f"pack_{bits}", 8, 320, 136, 4, 8.0, bits, 32, dtype)
    print("case", spec.name, "dtype", dtype, flush=True)
    arrs = inputs.make_layer_inputs(spec, seed=bits)
    s, b = host_qparams(spec, arrs, "asymm", 0.8)
    layer = binding.upload(spec, arrs, s, b)
    got = packed_on_gpu(spec, layer).cpu().numpy().view(np.uint32)
    dec, _, _ = O.decide_f32(arrs["W0"], arrs["A"], arrs["B"], s, b, bits, spec.group_size, spec.alpha)
    want = O.pack_codes(dec.codes, bits)
    assert got.shape == want.shape and np.array_equal(got, want)


def _random_forward_cases(count=20, seed=4902):
    """Seeded draw of decode-size problems: every code width, group sizes 8 .. 256, 1 .. 100 tokens, ragged row
    counts, row lengths that do and do not make whole cache lines of packed codes."""
    rng = np.random.default_rng(seed)
    cases = []
    for k in range(count):
        bits = int(rng.choice([2, 3, 4, 8]))
        g = int(rng.choice([8, 16, 32, 64, 128, 256]))
        i = 64 * int(rng.integers(1, 40))
        while i % g != 0:
            i += 64
        o = 8 * int(rng.integers(1, 160))
        T = int(rng.choice([1, 1, 2, 3, 5, 8, 12, 13, 16, 17, 31, 32, 33, 48, 64, 65, 100]))
        cases.append((k, T, i, o, bits, g))
    return cases


@pytest.mark.parametrize("k,T,i,o,bits,g", _random_forward_cases())
def test_quantized_forward_random_shapes(k, T, i, o, bits, g):
    test_quantized_forward_matches_oracle_and_training_forward(T, i, o, bits, g)


def _random_tile_cases(count=18, seed=2402):
    """Seeded draw of problems for the 64-row tile kernel: wide layers (every compute unit gets a tile) and narrow
    ones with long rows (k-slices through the workspace), 3, 4 and 8 bits, groups of one to four sub-steps, 1 .. 100
    tokens (every count of token blocks, several passes), ragged last row tiles."""
    rng = np.random.default_rng(seed)
    cases = []
    for k in range(count):
        bits = int(rng.choice([3, 4, 8]))
        unit = 128 if bits == 8 else 256            # codes of an activation stage
        g = int(rng.choice([unit // 2, unit, 2 * unit]))
        if k % 2 == 0:                              # wide
            o = 10240 + 8 * int(rng.integers(0, 200))
            i = unit * int(rng.integers(1, 9))
        else:                                       # narrow, long rows
            o = 2048 + 8 * int(rng.integers(0, 500))
            i = unit * int(rng.integers(8, 24))
        while i % g != 0:
            i += unit
        T = int(rng.choice([1, 7, 16, 17, 30, 32, 33, 47, 48, 49, 64, 65, 81, 100]))
        cases.append((k, T, i, o, bits, g))
    return cases


@pytest.mark.parametrize("k,T,i,o,bits,g", _random_tile_cases())
def test_quantized_forward_random_tile_shapes(k, T, i, o, bits, g):
    test_quantized_forward_matches_oracle_and_training_forward(T, i, o, bits, g)


def _random_in_register_cases(count=24, seed=355):
    """Seeded draw over the domain of the in-register form: every code width, power-of-two groups from 128 up to the
    row length, rows of 1 .. 64 chunks of 256 (with half chunks), 128 .. 16800 output rows in steps of 8 (one to four
    tiles per workgroup, ragged last tiles, layers too small to fill the chip), 1 .. 64 tokens around the block and
    pass boundaries; at most 48 M weights
    so that the oracle stays fast.  The library picks the form (and its shape) per case; with the workspace the k-sliced
    forms run as well."""
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        bits = int(rng.choice([2, 3, 4, 4, 8]))
        i = 128 * int(rng.integers(1, 129))
        o = 8 * int(rng.integers(16, 2101))
        if o * i > 48_000_000:
            continue
        gs = [g for g in (128, 256, 512, 1024, 2048, 4096, 8192) if i % g == 0]
        g = int(rng.choice(gs))
        T = int(rng.choice([1, 2, 3, 5, 8, 9, 12, 15, 16, 17, 20, 24, 31, 32, 33, 40, 49, 56, 64]))
        cases.append((len(cases), T, i, o, bits, g))
    return cases


@pytest.mark.parametrize("k,T,i,o,bits,g", _random_in_register_cases())
def test_quantized_forward_random_in_register_shapes(k, T, i, o, bits, g):
    test_quantized_forward_matches_oracle_and_training_forward(T, i, o, bits, g)


@pytest.mark.parametrize("T,i,o,bits,g", [
    # Shapes and batches the weights-in-registers form takes (groups of 128 and more, a few token blocks), one per
    # combination of row tiles per workgroup (1 .. 4: up to 4096 / 8192 / 12288 / more rows on 256 compute units) and
    # 256-wide chunks per wave (1 .. 4: up to 4096 / 8192 / 12288 / 16384 columns), for every code width that has it.
    # 4 bits: three tiles at 33 tokens with a ragged last tile; two tiles with half a chunk at the end of k; four
    # tiles with groups of 256; (1, 2); (2, 2) with groups of 512; three chunks (4 bits: a streaming form); (1, 4); (1, 4) with groups of 1024 and a
    # ragged tile; two token blocks on a 256-tile layer; four tiles over three token blocks; one token
    (33, 4096, 11000, 4, 128), (5, 2048 + 128, 6000, 4, 128), (40, 1024, 13000, 4, 256), (9, 8192, 3000, 4, 128),
    (20, 5120, 8000, 4, 512), (5, 11008, 4096, 3, 128), (7, 14336, 2400, 4, 128), (3, 16384, 2056, 4, 1024),
    (20, 4096, 4096, 4, 128), (48, 4096, 12296, 4, 128), (1, 4096, 11008, 4, 128),
    # 3 bits (12-byte pieces): (3, 1) over three token blocks, (1, 3), (2, 2), (1, 4) with groups of 256, one token
    (48, 4096, 11000, 3, 128), (16, 11008, 4096, 3, 128), (30, 8192, 8192, 3, 128), (2, 16384, 2056, 3, 256),
    (1, 4096, 4000, 3, 128),
    # 2 bits (8-byte pieces): (3, 1), (2, 1) over four token blocks, (1, 3), (2, 2) with groups of 256, three tokens
    (5, 4096, 11008, 2, 128), (64, 4096, 6000, 2, 128), (16, 11008, 4096, 2, 128), (33, 8192, 8192, 2, 256),
    (3, 4096, 4000, 2, 128),
    # 8 bits (one tile, one chunk only): one token, half a chunk at the end of k, groups of 256 with a ragged tile
    (1, 4096, 4096, 8, 128), (20, 2048 + 128, 4000, 8, 128), (32, 4096, 2072, 8, 256),
    # 17 .. 32 tokens on layers of up to 4096 columns: the 8-wave shape of the same kernel (two chunks per wave, two
    # token blocks per pass), every tiles x chunks combination it has, at 4, 3 and 2 bits; a ragged last tile, half a
    # chunk at the end of k, groups of 256, a partial second block
    (24, 4096, 11000, 4, 128), (24, 4096, 11000, 3, 128), (24, 4096, 11000, 2, 128),
    (17, 4096, 6000, 4, 128), (17, 4096, 6000, 3, 128), (17, 4096, 6000, 2, 128),
    (32, 2176, 4000, 4, 128), (32, 2176, 4000, 3, 128), (32, 2176, 4000, 2, 128),
    (20, 2048, 11008, 4, 128), (20, 2048, 11008, 3, 128), (20, 2048, 11008, 2, 128),
    (25, 1024, 6008, 4, 256), (25, 1024, 6008, 3, 256), (25, 1024, 6008, 2, 256),
    (31, 1152, 1000, 4, 128), (31, 1152, 1000, 3, 128), (31, 1152, 1000, 2, 128),
    # long rows on layers of 128 .. 256 row tiles, with the workspace: k-slices of 16 chunks (3, 2, 4 and 3 slices; the
    # last slice short; 16- and 8-wave shapes; groups of 256, of 512, and of 8192, which span two slices; a ragged
    # last tile)
    (12, 11008, 4096, 4, 128), (12, 11008, 4096, 3, 128), (12, 11008, 4096, 2, 128), (24, 8192, 4096, 4, 128),
    (9, 14336, 2400, 4, 128), (20, 14336, 2400, 3, 256), (16, 12288, 3000, 2, 128), (10, 11264, 4096, 4, 512),
    (8, 16384, 2056, 4, 8192),
    # ... and two passes of it (49 .. 64 tokens), the last block partial
    (64, 4096, 11000, 4, 128), (64, 4096, 11000, 3, 128), (64, 4096, 11000, 2, 128), (50, 4096, 6000, 2, 128),
])
def test_quantized_forward_weights_in_registers(T, i, o, bits, g):
    test_quantized_forward_matches_oracle_and_training_forward(T, i, o, bits, g)


@pytest.mark.parametrize("T,i,o,bits,g", [
    (1, 256, 72, 4, 64), (7, 512, 264, 4, 128), (64, 1024, 520, 3, 64), (33, 256, 40, 2, 8), (100, 320 * 2, 96, 8, 32),
    (16, 4096, 11008, 4, 128),      # LLaMA-7B up projection at a decode batch
    (64, 4096, 1024, 3, 128),       # 3-bit, 64 tokens
    (1, 4096, 11008, 4, 128), (1, 11008, 4096, 4, 128),   # single-token decode, both projections
    (17, 11008, 1000, 4, 64),       # odd stage count (43), 17 tokens -> 32-row tiles, ragged rows
    (5, 640, 88, 8, 64), (40, 1280, 200, 8, 128),         # 8-bit streaming form, 16- and 32-row tiles
    (16, 384, 48, 4, 128),          # packed rows not a whole number of cache lines -> general kernel
    (3, 256, 8, 4, 128),            # one stage, a single partial row tile
    # activations held in LDS (small batches): both projections at 2..12 tokens, ragged row tile, even and odd
    # group counts per row, 8-bit, a row length whose activations no longer fit (falls back to register fragments)
    (2, 4096, 11008, 4, 128), (12, 4096, 11008, 4, 128), (4, 11008, 4096, 4, 128), (5, 11008, 4096, 4, 128),
    (3, 1024, 1000, 4, 128), (2, 768, 40, 4, 256), (9, 2048, 520, 8, 64), (13, 4096, 264, 4, 64),
    (1, 28672, 64, 4, 128), (16, 4096, 72, 4, 128),
    # wide layers (enough 64-row tiles for most compute units): tiles sharing the activation stage, 4, 3, 2 and 1
    # token blocks per pass, a ragged last row tile, odd stage count, 8-bit, groups of two sub-steps (4-bit g = 256,
    # 8-bit g = 128), long rows that leave LDS for two token blocks only, a small batch too long for the LDS-resident
    # form
    (64, 4096, 11008, 4, 128), (70, 1024, 10248, 4, 128), (40, 896, 10312, 8, 128), (48, 11008, 10240, 4, 128),
    (24, 2048, 10304, 4, 256), (13, 4096, 10240, 4, 64), (30, 1024, 10240, 8, 64),
    # few row tiles and long rows with a workspace: k-slices over the compute units (4, 2 and 3 slices; a slice
    # boundary inside a group (g = 1024); 8-bit; two passes; stage counts that do not divide by the slices)
    (64, 11008, 4096, 4, 128), (33, 8192, 8192, 4, 128), (48, 5120, 5000, 4, 1024), (80, 2304, 4104, 8, 128),
    (17, 4096, 4096, 4, 128),
    # 3 bits at the smallest batches: both projections (rows of 11008 codes are neither whole cache lines nor whole
    # three-stage units), ragged row tiles, row lengths of 1.125, 2 and 1/8 units, groups of 256, 16 tokens
    (1, 4096, 11008, 3, 128), (1, 11008, 4096, 3, 128), (12, 4096, 1000, 3, 128), (5, 1152, 264, 3, 128),
    (16, 2048, 72, 3, 256), (3, 128, 40, 3, 128), (4, 11008, 4096, 3, 128),
    # 3 bits at larger batches (64-row tiles with weights in units of three stages where the in-register form does
    # not take the case): both projections (the narrow one in k-slices of whole units, the last one short), one to
    # three token blocks per pass, two passes, a row of less than one unit, ragged last row tile, groups of 256
    (64, 4096, 11008, 3, 128), (40, 11008, 4096, 3, 128), (16, 4096, 10240, 3, 128), (33, 1024, 10312, 3, 256),
    (24, 2048, 10304, 3, 128), (70, 768, 10248, 3, 128),
    # ... and few tokens on narrow layers
    (16, 4096, 4096, 3, 128), (7, 11008, 4096, 3, 128),
    # 70B-class projections: the widest layer at a small batch, the longest rows (too many groups for the tile kernel's
    # tables: the streaming forms take it)
    (4, 8192, 28672, 4, 128), (40, 28672, 8192, 4, 128),
    # 2 bits at small batches (the LDS-resident form with half-chunk sub-steps on narrow layers, else the in-register
    # form): both projections at one token and a few (rows of 11008 codes are 21.5 stages: the last stage runs into
    # the next row), groups of 256, a ragged row tile, a row of less than one stage, 12 tokens of a short row
    (1, 4096, 11008, 2, 128), (1, 11008, 4096, 2, 128), (4, 4096, 11008, 2, 128), (8, 11008, 4096, 2, 128),
    (3, 2048, 1000, 2, 256), (5, 256, 40, 2, 128), (12, 1024, 264, 2, 128), (16, 4096, 520, 2, 128),
    # 4 and 8 bits with packed rows that are not whole stages (16-byte aligned only): the last stage is shared with
    # the next row; the last row's runs past the matrix
    (2, 4096 + 128, 1000, 4, 128), (7, 1152, 264, 4, 128), (3, 2048 + 64, 72, 8, 64), (1, 11008 + 128, 4096, 4, 128),
])
def test_quantized_forward_matches_oracle_and_training_forward(T, i, o, bits, g):
    import torch
    from oracle import l4q_oracle as O
    from paper_2402_04902_amd import binding
    spec = LayerSpec(f"qfwd_{T}x{i}x{o}_{bits}b", T, i, o, 8, 16.0, bits, g, DTYPE_BF16)
    print("case", spec.name, flush=True)
    arrs = inputs.make_layer_inputs(spec, seed=T + bits)
    s, b = host_qparams(spec, arrs, "asymm", 0.9)
    layer = binding.upload(spec, arrs, s, b)
    packed = packed_on_gpu(spec, layer)
    Yq = torch.empty_like(layer.Y)
    binding.l4q_quantized_forward(layer.desc, layer.X, packed, layer.scale, layer.zero, Yq)
    # the optional workspace (k-slices over the compute units for layers with few row tiles); a second result
    Yw = None
    ws_bytes = binding.l4q_quantized_forward_workspace_bytes(layer.desc)
    if ws_bytes > 0:
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda:0")
        Yw = torch.full_like(layer.Y, float("nan"))
        binding.l4q_quantized_forward(layer.desc, layer.X, packed, layer.scale, layer.zero, Yw, ws)
    layer.forward()
    torch.cuda.synchronize()
    dec, _, _ = O.decide_f32(arrs["W0"], arrs["A"], arrs["B"], s, b, bits, g, spec.alpha)
    ref = O.quantized_forward(arrs["X"], O.pack_codes(dec.codes, bits), s, b, bits, g)
    for Yg in (Yq, Yw):
        if Yg is None:
            continue
        got = Yg.double().cpu().numpy()
        compare_tensor(spec.name, got, ref, 2e-2, 2e-2)   # whole tensor, rows, columns, elements
        # single forward path: the quantized-only output equals the training-time forward up to summation order
        assert rel_fro(got, layer.Y.double().cpu().numpy()) <= 5e-3


@pytest.mark.parametrize("T,i,o,bits,g", [
    (1, 4096, 11008, 4, 128),     # activations resident in LDS
    (16, 4096, 10240, 4, 128),    # 64-row tiles
    (48, 5120, 5000, 4, 1024),    # k-slices into the workspace + the sum over the slices
    (20, 512, 264, 3, 64),        # general kernel
])
def test_quantized_forward_replayed_from_a_graph(T, i, o, bits, g):
    """A serving loop replays the layer from a captured graph: the call allocates nothing, launches only kernels on the
    caller's stream and keeps no state between calls, so every replay - with eager work and synchronisation in
    between - must give exactly what the eager call gives on the same inputs."""
    import torch
    from paper_2402_04902_amd import binding
    spec = LayerSpec(f"qgraph_{T}x{i}x{o}_{bits}b", T, i, o, 8, 16.0, bits, g, DTYPE_BF16)
    print("case", spec.name, flush=True)
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(T * 131 + bits)
    packed = torch.randint(-2**31, 2**31 - 1, (o, bits * i // 32), dtype=torch.int32, device=dev, generator=gen)
    s = torch.rand(o, i // g, device=dev, generator=gen) * 0.01 + 0.001
    b = torch.randn(o, i // g, device=dev, generator=gen) * 0.01
    X = torch.zeros(T, i, dtype=torch.bfloat16, device=dev)
    Yg = torch.zeros(T, o, dtype=torch.bfloat16, device=dev)
    Ye = torch.zeros(T, o, dtype=torch.bfloat16, device=dev)
    d = binding.make_desc(spec)
    ws = torch.empty(max(256, binding.l4q_quantized_forward_workspace_bytes(d)), dtype=torch.uint8, device=dev)
    ws2 = torch.empty_like(ws)
    binding.l4q_quantized_forward(d, X, packed, s, b, Yg, ws)   # first call outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        binding.l4q_quantized_forward(d, X, packed, s, b, Yg, ws)
    for rep in range(4):
        X.copy_(torch.randn(T, i, device=dev, generator=gen).to(torch.bfloat16))
        Yg.fill_(float("nan"))
        binding.l4q_quantized_forward(d, X, packed, s, b, Ye, ws2)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.isfinite(Yg.float()).all()
        assert torch.equal(Yg.view(torch.int16), Ye.view(torch.int16)), f"replay {rep}"


def test_quantized_forward_ignores_a_short_workspace():
    """A workspace smaller than the layer can use is ignored: the result is the one computed without any, bit for bit,
    and nothing is written past the bytes that were passed."""
    import torch
    from paper_2402_04902_amd import binding
    T, i, o, bits, g = 64, 4096, 4096, 4, 128   # (a batch the k-sliced tile form takes)
    spec = LayerSpec("qshort_ws", T, i, o, 8, 16.0, bits, g, DTYPE_BF16)
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(77)
    packed = torch.randint(-2**31, 2**31 - 1, (o, bits * i // 32), dtype=torch.int32, device=dev, generator=gen)
    s = torch.rand(o, i // g, device=dev, generator=gen) * 0.01 + 0.001
    b = torch.randn(o, i // g, device=dev, generator=gen) * 0.01
    X = torch.randn(T, i, device=dev, generator=gen).to(torch.bfloat16)
    d = binding.make_desc(spec)
    need = binding.l4q_quantized_forward_workspace_bytes(d)
    assert need > 0
    guard = torch.full((need,), 0x5A, dtype=torch.uint8, device=dev)
    Y0 = torch.empty(T, o, dtype=torch.bfloat16, device=dev)
    Y1 = torch.empty_like(Y0)
    Y2 = torch.empty_like(Y0)
    binding.l4q_quantized_forward(d, X, packed, s, b, Y0)
    binding.l4q_quantized_forward(d, X, packed, s, b, Y1, guard[: need // 2])
    torch.cuda.synchronize()
    assert torch.equal(Y0.view(torch.int16), Y1.view(torch.int16))
    assert bool((guard == 0x5A).all())
    binding.l4q_quantized_forward(d, X, packed, s, b, Y2, guard)   # the full workspace is used
    torch.cuda.synchronize()
    assert not bool((guard == 0x5A).all())
    assert float((Y2.float() - Y0.float()).abs().max()) <= 0.02 * float(Y0.float().abs().max())
