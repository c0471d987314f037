"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, sizes its workspace sensibly and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

from paper_2402_04902_amd import binding, inputs
from paper_2402_04902_amd.inputs import DTYPE_BF16, DTYPE_F32, LayerSpec

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2402_04902_amd import build
        build.build_library()
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "l4q.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(l4q_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(binding.EXPORTED) <= set(names)
    assert len(names) >= 7
    for n in names:
        assert hasattr(lib, n), n
    assert lib.l4q_version() == 100


def test_status_strings(lib):
    seen = set()
    for st in range(0, -9, -1):
        s = binding.status_string(st)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 9
    assert binding.status_string(-99) == "unknown status"


def test_workspace_bytes(lib):
    spec = inputs.config3()[0]
    f, b = binding.l4q_workspace_bytes(binding.make_desc(spec))
    o, i, T = spec.out_features, spec.in_features, spec.tokens
    assert f >= 2 * o * i and f < 2 * o * i + 4096          # one transient bf16 Wq
    assert b >= f
    assert b < 8 * (o * i + T * i + T * o)                  # no token-sized fp32 buffers, no 2nd fp32 weight copy
    f32 = binding.make_desc(inputs.config1()[0])
    f1, b1 = binding.l4q_workspace_bytes(f32)
    assert f1 >= 4 * 256 * 256 and b1 >= 2 * 4 * 256 * 256


@pytest.mark.parametrize("field,value,status", [
    ("tokens", 0, -2), ("in_features", 0, -2), ("out_features", -1, -2), ("rank", 0, -2), ("rank", 257, -2),
    ("group_size", 96, -2), ("group_size", 2, -2), ("group_size", 4096 * 2, -2),
    ("bits", 1, -3), ("bits", 9, -3), ("dtype", 2, -4), ("flags", 8, -4), ("out_features", 4100, -2),
])
def test_bad_descriptors_are_rejected(lib, field, value, status):
    spec = LayerSpec("x", 64, 4096, 4096, 16, 32.0, 4, 128, DTYPE_BF16)
    d = binding.make_desc(spec)
    setattr(d, field, value)
    f = ctypes.c_size_t(0)
    assert lib.l4q_workspace_bytes(ctypes.byref(d), ctypes.byref(f), None) == status
    # the compute entry points validate before touching the GPU
    assert lib.l4q_forward(ctypes.byref(d), 16, 16, 16, 16, 16, 16, 16, 256, 1 << 40, None) == status
    assert lib.l4q_backward(ctypes.byref(d), 16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 256, 1 << 40,
                            None) == status


def test_null_alignment_and_workspace_errors(lib):
    spec = LayerSpec("x", 64, 256, 256, 8, 16.0, 4, 64, DTYPE_F32)
    d = binding.make_desc(spec)
    r = ctypes.byref(d)
    assert lib.l4q_forward(None, 16, 16, 16, 16, 16, 16, 16, 256, 1 << 40, None) == -1
    assert lib.l4q_forward(r, None, 16, 16, 16, 16, 16, 16, 256, 1 << 40, None) == -1
    assert lib.l4q_forward(r, 16, 16, 16, 16, 16, 16, None, 256, 1 << 40, None) == -1
    assert lib.l4q_forward(r, 16, 24, 16, 16, 16, 16, 16, 256, 1 << 40, None) == -5
    assert lib.l4q_forward(r, 16, 16, 16, 16, 16, 16, 16, None, 1 << 40, None) == -6
    assert lib.l4q_forward(r, 16, 16, 16, 16, 16, 16, 16, 256, 1024, None) == -6
    assert lib.l4q_forward(r, 16, 16, 16, 16, 16, 16, 16, 128, 1 << 40, None) == -5
    assert lib.l4q_backward(r, 16, 16, 16, 16, 16, 16, 16, 16, None, 16, 16, 16, 256, 1 << 40, None) == -1
    assert lib.l4q_backward(r, 16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 256, 8, None) == -6
    assert lib.l4q_export_codes(r, None, 16, 16, 16, 16, None, None, None, None) == -1
    assert lib.l4q_export_codes(r, 16, 16, 16, 16, 16, 8, None, None, None) == -5
    assert lib.l4q_init_qparams(r, 16, 16, 16, 7, 16, 16, None) == -8
    assert lib.l4q_init_qparams(r, 16, 16, 16, 0, None, 16, None) == -1
    assert lib.l4q_quant_errors(r, 16, 16, 16, 16, 16, 16, 256, 8, None) == -6
    assert lib.l4q_quant_errors(r, 16, 16, 16, 16, 16, None, 256, 1 << 30, None) == -1
    assert lib.l4q_mfma_probe(None, 1, 1, 16, None, None) == -1
    assert lib.l4q_mfma_probe(16, 0, 1, 16, None, None) == -2


def test_descriptor_layout_matches_header():
    assert ctypes.sizeof(binding.L4QDesc) == 48
    assert binding.L4QDesc.alpha.offset == 36 and binding.L4QDesc.flags.offset == 44


def test_quantized_forward_workspace_query_and_argument_checks(lib):
    """The optional workspace of the quantized forward: its size is a host computation (k-slices x tokens of a pass x
    rows of fp32 for layers with few 64-row tiles and long rows, nothing otherwise); arguments are checked before
    anything is launched."""
    n = ctypes.c_size_t(7)
    narrow = binding.make_desc(LayerSpec("down", 64, 11008, 4096, 16, 32.0, 4, 128, DTYPE_BF16))
    assert lib.l4q_quantized_forward_workspace_bytes(ctypes.byref(narrow), ctypes.byref(n)) == 0
    assert n.value > 0 and n.value % (4096 * 4) == 0 and n.value <= 8 * 64 * 4096 * 4
    wide = binding.make_desc(LayerSpec("up", 64, 4096, 11008 * 2, 16, 32.0, 4, 128, DTYPE_BF16))
    assert lib.l4q_quantized_forward_workspace_bytes(ctypes.byref(wide), ctypes.byref(n)) == 0 and n.value == 0
    narrow3 = binding.make_desc(LayerSpec("down3", 64, 11008, 4096, 16, 32.0, 3, 128, DTYPE_BF16))
    assert lib.l4q_quantized_forward_workspace_bytes(ctypes.byref(narrow3), ctypes.byref(n)) == 0
    assert n.value > 0 and n.value % (4096 * 4) == 0          # 3 bits: k-slices of whole three-stage units
    narrow2 = binding.make_desc(LayerSpec("down2", 64, 11008, 4096, 16, 32.0, 2, 128, DTYPE_BF16))
    assert lib.l4q_quantized_forward_workspace_bytes(ctypes.byref(narrow2), ctypes.byref(n)) == 0
    assert n.value == 3 * 32 * 4096 * 4                       # 2 bits: the in-register form's three k-slices, 32 tokens
    f32 = binding.make_desc(LayerSpec("f", 64, 11008, 4096, 16, 32.0, 4, 128, DTYPE_F32))
    assert lib.l4q_quantized_forward_workspace_bytes(ctypes.byref(f32), ctypes.byref(n)) == 0 and n.value == 0
    assert lib.l4q_quantized_forward_workspace_bytes(ctypes.byref(narrow), None) == -1
    assert lib.l4q_quantized_forward_workspace_bytes(None, ctypes.byref(n)) == -1
    r = ctypes.byref(narrow)
    assert lib.l4q_quantized_forward(r, 16, 16, 16, 16, None, None, 0, None) == -1
    assert lib.l4q_quantized_forward(r, 16, 16, 16, 16, 24, None, 0, None) == -5
    assert lib.l4q_quantized_forward(r, 16, 16, 16, 16, 16, 128, 1 << 30, None) == -5   # workspace not 256-aligned
    assert lib.l4q_quantized_forward(ctypes.byref(f32), 16, 16, 16, 16, 16, None, 0, None) == -4


def test_header_is_plain_c_and_agrees_with_the_binding(tmp_path):
    """include/l4q.h compiles as C99 on its own, and a C program reports the struct layout and enum values the
    ctypes binding assumes."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "layout.c"
    src.write_text(
        '#include <stdio.h>\n#include <stddef.h>\n#include "l4q.h"\n'
        'int main(void) {\n'
        '  printf("%zu %zu %zu %zu %d %d %d %d\\n", sizeof(l4q_desc), offsetof(l4q_desc, rank),\n'
        '         offsetof(l4q_desc, alpha), offsetof(l4q_desc, flags), (int)L4Q_DTYPE_BF16,\n'
        '         (int)L4Q_FLAG_UNFUSED_BACKWARD, (int)L4Q_FLAG_ACCUMULATE_GRADS, (int)L4Q_ERR_SHAPE);\n'
        '  return 0;\n}\n')
    exe = tmp_path / "layout"
    subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), str(src),
                    "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert [int(v) for v in out] == [ctypes.sizeof(binding.L4QDesc), binding.L4QDesc.rank.offset,
                                     binding.L4QDesc.alpha.offset, binding.L4QDesc.flags.offset, DTYPE_BF16,
                                     binding.FLAG_UNFUSED_BACKWARD, binding.FLAG_ACCUMULATE_GRADS, -2]


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2402_04902_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in text.lower(), (fn, "mentions the oracle")
    bench = open(os.path.join(ROOT, "bench.py")).read() if os.path.exists(os.path.join(ROOT, "bench.py")) else ""
    # the benchmark may touch the oracle only inside its cpu_baseline leg
    for line_no, line in enumerate(bench.splitlines(), 1):
        if "import" in line and "oracle" in line:
            assert line.startswith("    "), f"bench.py:{line_no} imports the oracle at module level"
