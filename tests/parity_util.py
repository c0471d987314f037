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


def check_float_outputs(spec, layer, Y, gr, report=None):
    """Frobenius relative error per output tensor against the stated tolerance.

    dzero is identically zero when nothing clips; it is then compared absolutely against
    tol * rms(dWq) * sqrt(g) (an element-wise relative error has no meaning there)."""
    tol = TOL[spec.dtype]
    pairs = [("Y", layer.Y, Y), ("dX", layer.dX, gr.dX), ("dA", layer.dA, gr.dA), ("dB", layer.dB, gr.dB),
             ("dscale", layer.dscale, gr.dscale), ("dzero", layer.dzero, gr.dzero)]
    out = {}
    for name, got, ref in pairs:
        g = got.double().cpu().numpy()
        assert g.shape == ref.shape, (name, g.shape, ref.shape)
        assert np.isfinite(g).all(), name
        if name == "dzero" and np.linalg.norm(ref) == 0.0:
            bound = tol * np.sqrt(np.mean(gr.dWq ** 2)) * np.sqrt(spec.group_size)
            assert np.abs(g).max() <= bound, (name, np.abs(g).max(), bound)
            out[name] = 0.0
            continue
        err = rel_fro(g, ref)
        out[name] = err
        assert err <= tol, (spec.name, name, err, tol)
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
