"""Pins of the QAT-LoRA oracle (Sec. 3.1): reductions to pinned functions, the textbook LoRA form, and
finite differences where the function is smooth."""
import numpy as np

from oracle import l4q_oracle as O
from oracle import qatlora_oracle as Q


def _case(seed=0, T=9, i=32, o=12, r=3, bits=4, g=8, alpha=6.0):
    rng = np.random.default_rng(seed)
    X = rng.normal(size=(T, i))
    W0 = rng.normal(scale=0.05, size=(o, i))
    A = rng.uniform(-1, 1, size=(r, i)) / np.sqrt(i)
    B = rng.normal(scale=0.05, size=(o, r))
    dY = rng.normal(size=(T, o))
    s, b = O.init_qparams(W0, bits, g, "asymm")
    return X, W0, A, B, dY, s * 0.8, b, bits, g, alpha


def test_zero_lora_factor_reduces_to_the_l4q_layer():
    X, W0, A, B, dY, s, b, bits, g, alpha = _case()
    Z = np.zeros_like(B)
    assert np.allclose(Q.forward(X, W0, A, Z, s, b, bits, g, alpha), O.forward(X, W0, A, Z, s, b, bits, g, alpha),
                       rtol=0, atol=1e-13)
    gq = Q.backward(X, dY, W0, A, Z, s, b, bits, g, alpha)
    gl = O.backward(X, dY, W0, A, Z, s, b, bits, g, alpha)
    for name in ("dX", "dscale", "dzero", "dWq"):
        assert np.allclose(getattr(gq, name), getattr(gl, name), rtol=0, atol=1e-12), name
    assert np.abs(gq.dscale).max() > 0 and np.abs(gq.dzero).max() > 0  # the clipped branch is exercised
    assert np.abs(gq.dA).max() == 0.0                                   # dA = gamma (dY B)^T X vanishes with B


def test_quantizer_does_not_see_the_lora_factors():
    X, W0, A, B, dY, s, b, bits, g, alpha = _case(1)
    g1 = Q.backward(X, dY, W0, A, B, s, b, bits, g, alpha)
    g2 = Q.backward(X, dY, W0, 3.0 * A, -2.0 * B, s, b, bits, g, alpha)
    assert np.array_equal(g1.dscale, g2.dscale) and np.array_equal(g1.dzero, g2.dzero)


def test_lora_part_is_the_textbook_form_in_the_other_association_order():
    X, W0, A, B, dY, s, b, bits, g, alpha = _case(2)
    gamma = alpha / A.shape[0]
    Wq = O.dequant(Q.decisions_f64(W0, s, b, bits, g).codes, s, b, g)
    Y = Q.forward(X, W0, A, B, s, b, bits, g, alpha)
    assert np.allclose(Y - X @ Wq.T, gamma * (X @ (B @ A).T), rtol=0, atol=1e-12)   # delta W = gamma B A applied as a matrix
    gr = Q.backward(X, dY, W0, A, B, s, b, bits, g, alpha)
    dW = dY.T @ X                                                                     # gradient w.r.t. the dense update
    assert np.allclose(gr.dA, gamma * (B.T @ dW), rtol=0, atol=1e-11)
    assert np.allclose(gr.dB, gamma * (dW @ A.T), rtol=0, atol=1e-11)
    assert np.allclose(gr.dX, dY @ (Wq + gamma * B @ A), rtol=0, atol=1e-11)


def test_gradients_against_central_differences():
    X, W0, A, B, dY, s, b, bits, g, alpha = _case(3)
    gr = Q.backward(X, dY, W0, A, B, s, b, bits, g, alpha)
    loss = lambda X_, A_, B_: float((dY * Q.forward(X_, W0, A_, B_, s, b, bits, g, alpha)).sum())
    rng = np.random.default_rng(9)
    h = 1e-4
    for name, ref, idxs in (("dA", gr.dA, A.shape), ("dB", gr.dB, B.shape), ("dX", gr.dX, X.shape)):
        for _ in range(6):
            idx = tuple(int(rng.integers(n)) for n in idxs)
            args = {"dA": [X, A.copy(), B], "dB": [X, A, B.copy()], "dX": [X.copy(), A, B]}[name]
            k = {"dA": 1, "dB": 2, "dX": 0}[name]
            args[k][idx] += h
            up = loss(*args)
            args[k][idx] -= 2 * h
            dn = loss(*args)
            assert abs((up - dn) / (2 * h) - ref[idx]) <= 1e-6 * max(1.0, abs(ref[idx])), (name, idx)


def test_scale_and_zero_gradients_by_brute_force_on_a_tiny_layer():
    X, W0, A, B, dY, s, b, bits, g, alpha = _case(4, T=3, i=8, o=2, r=1, g=4)
    gr = Q.backward(X, dY, W0, A, B, s, b, bits, g, alpha)
    qn, qp = O.q_bounds(bits)
    for p in range(2):
        for q in range(2):
            ds = db = 0.0
            for j in range(4 * q, 4 * q + 4):
                dwq = sum(dY[t, p] * X[t, j] for t in range(3))
                w = (W0[p, j] - b[p, q]) / s[p, q]
                inside = qn <= w <= qp
                code = np.rint(min(max(w, qn), qp))
                ds += dwq * ((code - w) if inside else code)
                db += dwq * (0.0 if inside else 1.0)
            assert abs(ds - gr.dscale[p, q]) <= 1e-12 and abs(db - gr.dzero[p, q]) <= 1e-12
