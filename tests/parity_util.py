"""Shared helpers for the GPU-vs-oracle parity tests."""
from __future__ import annotations

import numpy as np

from oracle import l4q_oracle as O
from paper_2402_04902_amd import inputs

TOL = {inputs.DTYPE_F32: 1e-4, inputs.DTYPE_BF16: 2e-2}


def host_qparams(spec, arrs, method="asymm", shrink=1.0):
    """scale/zero from the oracle's float64 initialisation, rounded to float32."""
    Wc = O.merge(arrs["W0"], arrs["A"], arrs["B"], spec.alpha)
    s, b = O.init_qparams(Wc, spec.bits, spec.group_size, method)
    return (s * shrink).astype(np.float32), b.astype(np.float32)


def oracle_all(spec, arrs, s, b):
    """Oracle outputs with the discrete decisions of its strict binary32 chain."""
    dec, Wc32, w32 = O.decide_f32(arrs["W0"], arrs["A"], arrs["B"], s, b, spec.bits, spec.group_size, spec.alpha)
    Y = O.forward(arrs["X"], arrs["W0"], arrs["A"], arrs["B"], s, b, spec.bits, spec.group_size, spec.alpha, dec)
    gr = O.backward(arrs["X"], arrs["dY"], arrs["W0"], arrs["A"], arrs["B"], s, b, spec.bits, spec.group_size,
                    spec.alpha, dec)
    return dec, Wc32, w32, Y, gr


def rel_fro(got, ref):
    ref = np.asarray(ref, np.float64)
    got = np.asarray(got, np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


# Per output tensor: (Frobenius-relative bound, element-wise bound).
# binary32 mode: 1e-4 throughout (the stated tolerance).
# bfloat16 mode: Y and dX are rounded to bfloat16 on the way out (2^-9 of the element) and carry the
# bfloat16 rounding of the Wq operand (about 2.2e-3 of rms(ref) per element, 5.5 sigma over 4.5e7 elements =
# 1.2e-2): 2e-2 for both bounds.  dA, dB, dscale, dzero are binary32 end to end apart from one operand
# rounding each (the masked gradient to bfloat16 for dA / dB: 2^-9 / sqrt(3) = 1.1e-3 of a term, observed
# 1.7e-3 of the tensor; the d(Wq)/d(scale) factor to binary16: 2^-12 absolute on |f| <= 1/2, observed 2.3e-5),
# so their Frobenius bound is 5e-3.  Element-wise, dA / dB sum o (or i) terms with independent roundings, the
# largest of 1e5 elements lies 4.5 sigma out (7.6e-3 of rms): 2e-2; dscale / dzero: 5e-3.
BOUNDS = {
    inputs.DTYPE_F32: {n: (1e-4, 1e-4) for n in ("Y", "dX", "dA", "dB", "dscale", "dzero")},
    inputs.DTYPE_BF16: {"Y": (2e-2, 2e-2), "dX": (2e-2, 2e-2), "dA": (5e-3, 2e-2), "dB": (5e-3, 2e-2),
                        "dscale": (5e-3, 5e-3), "dzero": (5e-3, 5e-3)},
}


def compare_tensor(name, got, ref, fro_tol, elem_tol):
    """Whole-tensor, per-row, per-column and per-element comparison of one 2-D output (numpy, CPU).

    fro:   ||got - ref||_F <= fro_tol ||ref||_F
    elem:  |got - ref| <= elem_tol (|ref| + rms(ref))                        for every element
    rows:  ||got[r] - ref[r]|| <= elem_tol (||ref[r]|| + rms(ref) sqrt(ncols)) for every row (and likewise columns):
           a row that is wrong as a whole (dropped, shifted, stale) has an error of the size of its own norm and
           fails this whatever the size of the tensor, where the whole-tensor norm would dilute it.  (The element
           tolerance, because a row or column may be as short as one element: rank 1, one group per row.)
    Returns the four measured figures (each relative to its bound's right-hand side without the tolerance)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.isfinite(got).all(), name
    diff = got - ref
    rms = float(np.sqrt(np.mean(ref * ref)))
    fro = float(np.linalg.norm(diff) / max(np.linalg.norm(ref), 1e-300))
    elem = float((np.abs(diff) / (np.abs(ref) + rms + 1e-300)).max())
    row = float((np.linalg.norm(diff, axis=1) /
                 (np.linalg.norm(ref, axis=1) + rms * np.sqrt(ref.shape[1]) + 1e-300)).max())
    col = float((np.linalg.norm(diff, axis=0) /
                 (np.linalg.norm(ref, axis=0) + rms * np.sqrt(ref.shape[0]) + 1e-300)).max())
    assert fro <= fro_tol, (name, "frobenius", fro, fro_tol)
    assert elem <= elem_tol, (name, "element", elem, elem_tol)
    assert row <= elem_tol, (name, "row", row, elem_tol)
    assert col <= elem_tol, (name, "column", col, elem_tol)
    return {"fro": fro, "elem": elem, "row": row, "col": col}


def compare_outputs(dtype, group_size, outputs, Y, gr):
    """outputs: dict name -> numpy array of the implementation; Y, gr: the oracle's.  dzero is identically zero
    when nothing clips; it is then compared absolutely against tol * rms(dWq) * sqrt(g) (a relative error has no
    meaning there)."""
    refs = {"Y": Y, "dX": gr.dX, "dA": gr.dA, "dB": gr.dB, "dscale": gr.dscale, "dzero": gr.dzero}
    out = {}
    for name, ref in refs.items():
        fro_tol, elem_tol = BOUNDS[dtype][name]
        g = np.asarray(outputs[name], np.float64)
        if name == "dzero" and np.linalg.norm(ref) == 0.0:
            assert g.shape == ref.shape and np.isfinite(g).all(), name
            bound = fro_tol * np.sqrt(np.mean(gr.dWq ** 2)) * np.sqrt(group_size)
            assert np.abs(g).max() <= bound, (name, np.abs(g).max(), bound)
            out[name] = 0.0
            continue
        m = compare_tensor(name, g, ref, fro_tol, elem_tol)
        out[name] = m["fro"]
        out[name + "_elem"] = m["elem"]
        out[name + "_rowcol"] = max(m["row"], m["col"])
    return out


def check_float_outputs(spec, layer, Y, gr, report=None):
    """Every floating-point output of the layer against the oracle: compare_outputs on the device tensors."""
    outputs = {n: getattr(layer, n).double().cpu().numpy() for n in ("Y", "dX", "dA", "dB", "dscale", "dzero")}
    out = compare_outputs(spec.dtype, spec.group_size, outputs, Y, gr)
    if report is not None:
        report.update(out)
    return out


def check_discrete(spec, layer, arrs, s, b, dec, Wc32):
    """Codes, mask and merged weight from l4q_export_codes: bit-exact against the binary32 chain.
    Differences between the binary32 and binary64 chains are counted; all of them must sit on
    rounding ties or on the grid ends."""
    import torch
    from paper_2402_04902_amd import binding
    o, i = spec.out_features, spec.in_features
    dev = layer.W0.device
    codes = torch.empty((o, i), dtype=torch.int8, device=dev)
    wcomb = torch.empty((o, i), dtype=torch.float32, device=dev)
    mask = torch.empty((o, i), dtype=torch.uint8, device=dev)
    binding.l4q_export_codes(layer.desc, layer.W0, layer.A, layer.B, layer.scale, layer.zero, codes, wcomb, mask)
    torch.cuda.synchronize()
    c = codes.cpu().numpy()
    wc = wcomb.cpu().numpy()
    m = mask.cpu().numpy().astype(bool)
    assert np.array_equal(wc.view(np.uint32), Wc32.view(np.uint32)), "merged weight differs in bits"
    assert np.array_equal(c, dec.codes), f"{(c != dec.codes).sum()} codes differ"
    assert np.array_equal(m, dec.mask), f"{(m != dec.mask).sum()} mask bits differ"
    qn, qp = O.q_bounds(spec.bits)
    assert c.min() >= qn and c.max() <= qp
    # binary64 chain: report ties / boundaries
    Wc64 = O.merge(arrs["W0"], arrs["A"], arrs["B"], spec.alpha)
    w64 = O.prequant(Wc64, s, b, spec.group_size)
    dec64 = O.Decisions(O.codes_from_w(w64, spec.bits), O.ste_mask(w64, spec.bits))
    tie, bnd = O.tie_and_boundary_sets(w64, spec.bits)
    cd = c.astype(np.int64) != dec64.codes.astype(np.int64)
    md = m != dec64.mask
    assert not (cd & ~tie).any(), "code differs from the float64 chain away from a rounding tie"
    assert not (md & ~bnd).any(), "mask differs from the float64 chain away from the grid ends"
    return {"near_ties": int(tie.sum()), "near_boundaries": int(bnd.sum()), "codes_vs_f64": int(cd.sum()),
            "mask_vs_f64": int(md.sum())}


def check_workspace_state(spec, layer, dec, w32, s, b, fused):
    """bfloat16 layers: what the merge + quantize pass of the forward and of the backward call left in the workspace,
    bit for bit against the oracle's binary32 chain.  The training path takes its discrete decisions in kernels of its
    own (not the export kernel check_discrete looks at), and they reach the outputs only through floating-point sums;
    here they are looked at directly.  Workspace layout (documented with the library's design): forward Wq [o, ipad]
    bfloat16 first, stored in blocks of 32 columns as [ipad / 32][o][32]; backward Wq^T [i, opad] bfloat16 first, in
    blocks of 32 rows of Wq as [opad / 32][i][32], then (fused weight-gradient kernel only) the binary16 factor
    d(Wq)/d(scale) [o, i] row-major, each 256-byte aligned; ipad / opad = i / o rounded up to 32.
    Call after layer.forward() and layer.backward() in this order, synchronised."""
    import torch
    o, i = spec.out_features, spec.in_features
    ipad, opad = (i + 31) // 32 * 32, (o + 31) // 32 * 32
    g = spec.group_size
    s32 = np.repeat(np.asarray(s, np.float32), g, axis=1)
    b32 = np.repeat(np.asarray(b, np.float32), g, axis=1)
    codes = dec.codes.astype(np.float32)
    # Wq = fma(code, s, b) rounded once to binary32 (exact product, one binary64 addition: 53 bits hold it in all but
    # astronomically rare cases), then to bfloat16
    wq32 = (codes.astype(np.float64) * s32.astype(np.float64) + b32.astype(np.float64)).astype(np.float32)
    wq_bits = inputs.bf16_bits(inputs.round_to_bf16(wq32))
    # backward workspace (the last call): Wq^T and the factor
    ws = layer.ws
    wqT = ws[: i * opad * 2].view(torch.int16).reshape(opad // 32, i, 32).cpu().numpy().view(np.uint16)
    wqT = np.ascontiguousarray(wqT.transpose(1, 0, 2)).reshape(i, opad)
    assert np.array_equal(wqT[:, :o], wq_bits.T), f"{(wqT[:, :o] != wq_bits.T).sum()} elements of Wq^T differ"
    assert not wqT[:, o:].any(), "padding of Wq^T is not zero"
    if fused:
        off = (i * opad * 2 + 255) // 256 * 256
        f = ws[off: off + o * i * 2].view(torch.int16).reshape(o, i).cpu().numpy().view(np.uint16)
        want = np.where(dec.mask, codes - w32.astype(np.float32), codes).astype(np.float16).view(np.uint16)
        assert np.array_equal(f, want), f"{(f != want).sum()} gradient factors differ"
    # forward workspace: run the forward pass once more (it overwrites the workspace)
    layer.forward()
    torch.cuda.synchronize()
    wq = ws[: o * ipad * 2].view(torch.int16).reshape(ipad // 32, o, 32).cpu().numpy().view(np.uint16)
    wq = np.ascontiguousarray(wq.transpose(1, 0, 2)).reshape(o, ipad)
    assert np.array_equal(wq[:, :i], wq_bits), f"{(wq[:, :i] != wq_bits).sum()} elements of Wq differ"
    assert not wq[:, i:].any(), "padding of Wq is not zero"
