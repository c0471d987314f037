"""Pins for the CPU oracle: each test ties a part of oracle/l4q_oracle.py to something
the paper or plain mathematics fixes, independently of the oracle's own code."""
import math
import os

import numpy as np
import pytest

from oracle import l4q_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))


def small_problem(seed=0, T=5, o=6, i=16, r=3, g=4, bits=4, alpha=6.0, shrink=1.0, method="asymm"):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((T, i))
    dY = rng.standard_normal((T, o)) * 0.1
    W0 = rng.standard_normal((o, i)) * 0.05
    A = rng.uniform(-1, 1, (r, i)) / math.sqrt(i)
    B = rng.standard_normal((o, r)) * 0.05
    Wc = O.merge(W0, A, B, alpha)
    s, b = O.init_qparams(Wc, bits, g, method)
    s = s * shrink
    return dict(X=X, dY=dY, W0=W0, A=A, B=B, s=s, b=b, bits=bits, g=g, alpha=alpha)


def call_bwd(p, **over):
    q = dict(p)
    q.update(over)
    return O.backward(q["X"], q["dY"], q["W0"], q["A"], q["B"], q["s"], q["b"], q["bits"], q["g"], q["alpha"])


def call_fwd(p, **over):
    q = dict(p)
    q.update(over)
    return O.forward(q["X"], q["W0"], q["A"], q["B"], q["s"], q["b"], q["bits"], q["g"], q["alpha"])


# ---------------------------------------------------------------- grid (Sec. 2.2)

@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_grid_has_exactly_2_pow_n_levels(bits):
    qn, qp = O.q_bounds(bits)
    assert qn == -(2 ** (bits - 1)) and qp == 2 ** (bits - 1) - 1
    assert qp - qn + 1 == 2 ** bits
    p = small_problem(seed=bits, o=8, i=64, g=32, bits=bits, shrink=0.7)
    w = O.prequant(O.merge(p["W0"], p["A"], p["B"], p["alpha"]), p["s"], p["b"], p["g"])
    c = O.codes_from_w(w, bits)
    assert np.all(c == np.round(c)) and c.min() >= qn and c.max() <= qp
    Wq = O.dequant(c, p["s"], p["b"], p["g"])
    for row in Wq.reshape(8, 2, 32):
        for grp in row:
            assert len(np.unique(grp)) <= 2 ** bits
    # shrunk scale: the extreme codes are certainly used
    assert c.min() == qn and c.max() == qp


def test_asymm_init_reaches_both_ends_in_every_group():
    p = small_problem(seed=3, o=10, i=128, g=32)
    qn, qp = O.q_bounds(4)
    c = O.decide_f64(p["W0"], p["A"], p["B"], p["s"], p["b"], 4, 32, p["alpha"]).codes.reshape(10, 4, 32)
    assert np.all(c.min(axis=2) == qn) and np.all(c.max(axis=2) == qp)


# ---------------------------------------------------------------- rounding (Eq. quant)

def test_round_half_even_and_clamp_round_commute():
    w = np.array([0.5, -0.5, 1.5, -1.5, 2.5, 3.5, -2.5, 6.5, 7.5, 7.49, -8.5, -7.5, 100.0, -100.0])
    expect = np.array([0, -0, 2, -2, 2, 4, -2, 6, 7, 7, -8, -8, 7, -8], dtype=float)
    assert np.array_equal(O.codes_from_w(w, 4), expect)
    rng = np.random.default_rng(1)
    w = rng.standard_normal(100000) * 6
    qn, qp = O.q_bounds(4)
    assert np.array_equal(O.codes_from_w(w, 4), np.clip(np.rint(w), qn, qp))


def test_mask_is_inclusive_on_the_pre_round_value():
    w = np.array([-8.0, 7.0, 7.3, -8.2, 7.0000001, 0.0])
    assert O.ste_mask(w, 4).tolist() == [True, True, False, False, False, True]
    # 7.3 rounds to Q_P but counts as clipped
    assert O.codes_from_w(np.array([7.3]), 4)[0] == 7


# ---------------------------------------------------------------- B = 0: plain group-wise QAT

def plain_groupwise_fake_quant(W, s, b, bits, g):
    """Independent textbook routine: scalar loops over rows, groups, elements."""
    lo, hi = -(2 ** (bits - 1)), 2 ** (bits - 1) - 1
    out = np.empty_like(W)
    for p in range(W.shape[0]):
        for j in range(W.shape[1]):
            q = j // g
            v = (W[p, j] - b[p, q]) / s[p, q]
            v = min(max(v, lo), hi)
            out[p, j] = round(v) * s[p, q] + b[p, q]  # Python's round is half-even
    return out


def test_zero_B_reduces_to_plain_groupwise_qat():
    p = small_problem(seed=5, T=7, o=9, i=24, r=2, g=8, shrink=0.8)
    Bz = np.zeros_like(p["B"])
    Wq_ref = plain_groupwise_fake_quant(p["W0"], p["s"], p["b"], p["bits"], p["g"])
    Y = call_fwd(p, B=Bz)
    Y_ref = np.array([[sum(p["X"][t, j] * Wq_ref[o_, j] for j in range(24)) for o_ in range(9)] for t in range(7)])
    assert np.allclose(Y, Y_ref, rtol=1e-13, atol=1e-13)
    gr = call_bwd(p, B=Bz)
    assert np.all(gr.dA == 0.0)
    assert np.abs(gr.dB).max() > 0


# ---------------------------------------------------------------- zero clipping at init (Table 5)

def read_golden():
    rows = {}
    with open(os.path.join(HERE, "golden", "table5_init_clip.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                rows[k] = float(v)
    return rows


@pytest.mark.parametrize("method", ["asymm", "l4q"])
def test_minmax_inits_clip_nothing(method):
    printed = read_golden()[method]
    rng = np.random.default_rng(11)
    W0 = rng.standard_normal((64, 512)) * 0.02
    W0[rng.random(W0.shape) < 1e-3] *= 20
    A = rng.uniform(-1, 1, (4, 512)) / math.sqrt(512)
    B = rng.standard_normal((64, 4)) * 1e-3
    Wc = O.merge(W0, A, B, 8.0)
    s, b = O.init_qparams(Wc, 4, 128, method)
    e_clip = O.clipping_error(Wc, s, b, 4, 128)
    assert round(e_clip / 1e3, 1) == printed
    assert e_clip <= 1e-12 * np.abs(Wc).sum()
    w = O.prequant(Wc, s, b, 128)
    qn, qp = O.q_bounds(4)
    assert w.min() >= qn - 1e-9 and w.max() <= qp + 1e-9
    if method == "l4q":
        assert np.all(b == 0)
    # a scale shrunk below min/max does clip
    assert O.clipping_error(Wc, s * 0.8, b, 4, 128) > 0


def test_init_formulas_appendix_b():
    W = np.array([[-0.8, 0.1, 0.35, 0.7]])
    s, b = O.init_qparams(W, 4, 4, "asymm")
    assert np.isclose(s[0, 0], 1.5 / 15) and np.isclose(b[0, 0], 0.7 - 0.1 * 7) and np.isclose(b[0, 0], -0.8 + 0.1 * 8)
    s, b = O.init_qparams(W, 4, 4, "symm")
    assert np.isclose(s[0, 0], 0.8 / 8) and b[0, 0] == 0
    s, b = O.init_qparams(W, 4, 4, "l4q")
    assert np.isclose(s[0, 0], max(0.8 / 8, 0.7 / 7)) and b[0, 0] == 0
    s, b = O.init_qparams(W, 4, 4, "lsq+")
    mu, sd = W.mean(), W.std()
    assert np.isclose(s[0, 0], max(abs(mu - 3 * sd), abs(mu + 3 * sd)) / 8)


# ---------------------------------------------------------------- mask == 1: plain LoRA gradients

def test_unclipped_state_gives_plain_lora_gradients():
    p = small_problem(seed=7, T=11, o=10, i=32, r=3, g=8, shrink=1.0001)  # slightly wide: nothing clips
    gr = call_bwd(p)
    w = O.prequant(O.merge(p["W0"], p["A"], p["B"], p["alpha"]), p["s"], p["b"], p["g"])
    assert O.ste_mask(w, 4).all()
    gamma = p["alpha"] / 3
    Xt = p["X"] @ p["A"].T                      # [T, r]  (the LoRA intermediate AX)
    dXt = p["dY"] @ p["B"]                      # [T, r]
    dA_lora = gamma * dXt.T @ p["X"]            # Eq. lora_backward, first half
    dB_lora = gamma * p["dY"].T @ Xt            # Eq. lora_backward, second half
    assert np.allclose(gr.dA, dA_lora, rtol=1e-11, atol=1e-13)
    assert np.allclose(gr.dB, dB_lora, rtol=1e-11, atol=1e-13)
    assert np.all(gr.dzero == 0.0)


# ---------------------------------------------------------------- brute force on tiny shapes

def test_matmuls_against_triple_loops():
    p = small_problem(seed=9, T=4, o=5, i=8, r=2, g=4, shrink=0.75)
    T, o, i = 4, 5, 8
    dec = O.decide_f64(p["W0"], p["A"], p["B"], p["s"], p["b"], 4, 4, p["alpha"])
    Wq = O.dequant(dec.codes, p["s"], p["b"], 4)
    Y = call_fwd(p)
    gr = call_bwd(p)
    for t in range(T):
        for q in range(o):
            assert math.isclose(Y[t, q], sum(p["X"][t, j] * Wq[q, j] for j in range(i)), rel_tol=1e-12, abs_tol=1e-14)
    for t in range(T):
        for j in range(i):
            assert math.isclose(gr.dX[t, j], sum(p["dY"][t, q] * Wq[q, j] for q in range(o)), rel_tol=1e-12, abs_tol=1e-14)
    for q in range(o):
        for j in range(i):
            assert math.isclose(gr.dWq[q, j], sum(p["dY"][t, q] * p["X"][t, j] for t in range(T)), rel_tol=1e-12, abs_tol=1e-14)
    # merge, written with scalar loops
    gamma = p["alpha"] / 2
    Wc = O.merge(p["W0"], p["A"], p["B"], p["alpha"])
    for q in range(o):
        for j in range(i):
            ref = p["W0"][q, j] + gamma * sum(p["B"][q, k] * p["A"][k, j] for k in range(2))
            assert math.isclose(Wc[q, j], ref, rel_tol=1e-13, abs_tol=1e-15)


def test_layer_is_linear_in_X_and_dX_is_its_exact_derivative():
    p = small_problem(seed=13, T=3, o=4, i=8, r=2, g=4, shrink=0.9)
    Y = call_fwd(p)
    assert np.allclose(call_fwd(p, X=2 * p["X"]), 2 * Y, rtol=1e-14)
    gr = call_bwd(p)
    # L = sum(dY * Y); dL/dX[t,j] by a finite difference (exact up to rounding: L is linear in X)
    for t in range(3):
        for j in range(8):
            Xp = p["X"].copy()
            Xp[t, j] += 1.0
            fd = (p["dY"] * (call_fwd(p, X=Xp) - Y)).sum()
            assert math.isclose(gr.dX[t, j], fd, rel_tol=1e-9, abs_tol=1e-12)


# ---------------------------------------------------------------- closed forms vs dual numbers (App. A.1 / A.2)

class Dual:
    __slots__ = ("v", "d")

    def __init__(self, v, d=0.0):
        self.v, self.d = float(v), float(d)

    @staticmethod
    def lift(x):
        return x if isinstance(x, Dual) else Dual(x)

    def __add__(self, o):
        o = Dual.lift(o)
        return Dual(self.v + o.v, self.d + o.d)

    __radd__ = __add__

    def __sub__(self, o):
        o = Dual.lift(o)
        return Dual(self.v - o.v, self.d - o.d)

    def __mul__(self, o):
        o = Dual.lift(o)
        return Dual(self.v * o.v, self.d * o.v + self.v * o.d)

    __rmul__ = __mul__

    def __truediv__(self, o):
        o = Dual.lift(o)
        return Dual(self.v / o.v, (self.d * o.v - self.v * o.d) / (o.v * o.v))


def clamp_dual(x, lo, hi):
    if x.v < lo:
        return Dual(lo, 0.0)
    if x.v > hi:
        return Dual(hi, 0.0)
    return Dual(x.v, x.d)


def round_ste(x):
    """Rounding with the straight-through estimator: value rounds, tangent passes unchanged."""
    return Dual(round(x.v), x.d)


def loss_tangent(p, seed_of):
    """dL/dtheta for L = sum(dY * Y), theta selected by seed_of(name, idx) -> tangent seed."""
    T, i = p["X"].shape
    o = p["W0"].shape[0]
    r = p["A"].shape[0]
    g, bits = p["g"], p["bits"]
    lo, hi = -(2 ** (bits - 1)), 2 ** (bits - 1) - 1
    gamma = p["alpha"] / r
    total = 0.0
    for q in range(o):
        for j in range(i):
            acc = Dual(0.0)
            for k in range(r):
                acc = acc + Dual(p["B"][q, k], seed_of("B", (q, k))) * Dual(p["A"][k, j], seed_of("A", (k, j)))
            wc = Dual(p["W0"][q, j]) + gamma * acc
            s = Dual(p["s"][q, j // g], seed_of("s", (q, j // g)))
            b = Dual(p["b"][q, j // g], seed_of("b", (q, j // g)))
            w = (wc - b) / s
            wq = round_ste(clamp_dual(w, lo, hi)) * s + b
            # dL/dWq[q,j] = sum_t dY[t,q] X[t,j]
            total += wq.d * sum(p["dY"][t, q] * p["X"][t, j] for t in range(T))
    return total


@pytest.mark.parametrize("shrink", [1.0001, 0.6])
def test_closed_form_gradients_match_dual_numbers(shrink):
    p = small_problem(seed=17, T=3, o=4, i=8, r=2, g=4, shrink=shrink)
    gr = call_bwd(p)
    w = O.prequant(O.merge(p["W0"], p["A"], p["B"], p["alpha"]), p["s"], p["b"], p["g"])
    if shrink < 1:
        m = O.ste_mask(w, 4)
        assert (~m).sum() >= 3 and (w < -8).any() and (w > 7).any()  # both clipped branches occur

    def one_hot(name, idx):
        return lambda n, ix: 1.0 if (n == name and ix == idx) else 0.0

    for q in range(4):
        for G in range(2):
            assert math.isclose(gr.dscale[q, G], loss_tangent(p, one_hot("s", (q, G))), rel_tol=1e-10, abs_tol=1e-12)
            assert math.isclose(gr.dzero[q, G], loss_tangent(p, one_hot("b", (q, G))), rel_tol=1e-10, abs_tol=1e-12)
        for k in range(2):
            assert math.isclose(gr.dB[q, k], loss_tangent(p, one_hot("B", (q, k))), rel_tol=1e-10, abs_tol=1e-12)
    for k in range(2):
        for j in range(8):
            assert math.isclose(gr.dA[k, j], loss_tangent(p, one_hot("A", (k, j))), rel_tol=1e-10, abs_tol=1e-12)


def test_clipped_group_gradients_by_finite_differences():
    """Where every element of a group is clipped, Wq = Q_{N/P} s + b is smooth in s and b."""
    p = small_problem(seed=19, T=4, o=3, i=8, r=2, g=4)
    s = p["s"].copy()
    s[1, 0] *= 1e-3          # group (row 1, group 0): everything overflows the grid
    w = O.prequant(O.merge(p["W0"], p["A"], p["B"], p["alpha"]), s, p["b"], 4)
    assert not O.ste_mask(w, 4)[1, 0:4].any()
    gr = call_bwd(p, s=s)
    L0 = (p["dY"] * call_fwd(p, s=s)).sum()
    h = 1e-9
    sp = s.copy()
    sp[1, 0] += h
    fd_s = ((p["dY"] * call_fwd(p, s=sp)).sum() - L0) / h
    bp = p["b"].copy()
    bp[1, 0] += 1e-6
    fd_b = ((p["dY"] * call_fwd(p, s=s, b=bp)).sum() - L0) / 1e-6
    assert math.isclose(gr.dscale[1, 0], fd_s, rel_tol=1e-4)
    assert math.isclose(gr.dzero[1, 0], fd_b, rel_tol=1e-6)
    # clipped elements pass nothing to the LoRA factors: dB row 1 only sees group 1
    dWp = gr.dWq.copy()
    dWp[1, 0:4] = 0
    m = O.ste_mask(w, 4)
    gamma = p["alpha"] / 2
    assert np.allclose(gr.dB, gamma * np.where(m, gr.dWq, 0) @ p["A"].T)
    assert np.allclose(gr.dB[1], gamma * dWp[1] @ p["A"].T) or (~m[1, 4:]).any()


# ---------------------------------------------------------------- invariants at a moderate shape

def test_invariants_moderate_shape():
    p = small_problem(seed=23, T=96, o=80, i=192, r=4, g=32, shrink=0.8)
    gr = call_bwd(p)
    w = O.prequant(O.merge(p["W0"], p["A"], p["B"], p["alpha"]), p["s"], p["b"], 32)
    m = O.ste_mask(w, 4)
    assert 0 < (~m).sum() < m.size // 4
    assert np.allclose(gr.dzero.sum(axis=1), np.where(m, 0, gr.dWq).sum(axis=1))
    bound = (np.abs(gr.dWq).reshape(80, 6, 32).sum(axis=2)) * 8.0
    assert np.all(np.abs(gr.dscale) <= bound + 1e-12)
    # shapes: nothing transposed
    assert gr.dX.shape == (96, 192) and gr.dA.shape == (4, 192) and gr.dB.shape == (80, 4)
    assert gr.dscale.shape == (80, 6) and gr.dzero.shape == (80, 6)


# ---------------------------------------------------------------- binary32 decisions vs binary64

def test_f32_decisions_differ_from_f64_only_on_ties_and_boundaries():
    rng = np.random.default_rng(29)
    o, i, r, g, bits, alpha = 96, 512, 8, 64, 4, 16.0
    W0 = (rng.standard_normal((o, i)) * 0.02).astype(np.float32)
    A = (rng.uniform(-1, 1, (r, i)) / math.sqrt(i)).astype(np.float32)
    B = (rng.standard_normal((o, r)) * 1e-3).astype(np.float32)
    Wc = O.merge(W0, A, B, alpha)
    s, b = O.init_qparams(Wc, bits, g, "asymm")
    s, b = s.astype(np.float32), b.astype(np.float32)
    dec32, Wc32, w32 = O.decide_f32(W0, A, B, s, b, bits, g, alpha)
    assert Wc32.dtype == np.float32 and w32.dtype == np.float32
    assert np.linalg.norm(Wc32 - Wc) <= 1e-6 * np.linalg.norm(Wc)
    dec64 = O.decide_f64(W0, A, B, s, b, bits, g, alpha)
    w64 = O.prequant(Wc, s, b, g)
    tie, bnd = O.tie_and_boundary_sets(w64, bits)
    code_diff = dec32.codes.astype(np.int64) != dec64.codes.astype(np.int64)
    mask_diff = dec32.mask != dec64.mask
    assert not (code_diff & ~tie).any()
    assert not (mask_diff & ~bnd).any()
    # min/max init parks two elements per group on the grid ends
    assert bnd.sum() >= 2 * o * (i // g) * 0.9


def test_f32_merge_order_is_sequential_unfused():
    """Reproduce merge_f32 with scalar binary32 arithmetic on a few elements."""
    rng = np.random.default_rng(31)
    W0 = rng.standard_normal((3, 4)).astype(np.float32)
    A = rng.standard_normal((5, 4)).astype(np.float32)
    B = rng.standard_normal((3, 5)).astype(np.float32)
    got = O.merge_f32(W0, A, B, 7.0)
    f = np.float32
    gamma = f(f(7.0) / f(5))
    for p in range(3):
        for j in range(4):
            acc = f(0)
            for k in range(5):
                acc = f(acc + f(B[p, k] * A[k, j]))
            assert got[p, j] == f(W0[p, j] + f(gamma * acc))


# ---------------------------------------------------------------- packed codes, single forward path (Sec. 3.2)

@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_pack_unpack_roundtrip_and_bit_positions(bits):
    rng = np.random.default_rng(37 + bits)
    qn, qp = O.q_bounds(bits)
    codes = rng.integers(qn, qp + 1, size=(5, 64))
    packed = O.pack_codes(codes, bits)
    assert packed.dtype == np.uint32 and packed.shape == (5, bits * 64 // 32)
    assert np.array_equal(O.unpack_codes(packed, bits, 64), codes)
    # field j sits at bit n*j of the row's little-endian bit string: rebuild row 0 as one big integer
    big = 0
    for w, word in enumerate(packed[0]):
        big |= int(word) << (32 * w)
    for j in range(64):
        assert ((big >> (bits * j)) & ((1 << bits) - 1)) + qn == codes[0, j]
    # extreme codes map to all-zero / all-one fields
    assert O.pack_codes(np.full((1, 32), qn), bits).max() == 0
    assert O.pack_codes(np.full((1, 32), qp), bits).min() == 0xFFFFFFFF


def test_packed_forward_is_the_layer_forward():
    """The fully quantized path (codes, scale, zero only) gives exactly the layer's training-time output."""
    p = small_problem(seed=41, T=6, o=7, i=64, r=3, g=32, bits=4, shrink=0.8)
    dec = O.decide_f64(p["W0"], p["A"], p["B"], p["s"], p["b"], 4, 32, p["alpha"])
    packed = O.pack_codes(dec.codes, 4)
    Yq = O.quantized_forward(p["X"], packed, p["s"], p["b"], 4, 32)
    assert np.array_equal(Yq, call_fwd(p))
    # and independently: dequantize by hand from the unpacked fields
    c = O.unpack_codes(packed, 4, 64)
    Wq = np.array([[c[q, j] * p["s"][q, j // 32] + p["b"][q, j // 32] for j in range(64)] for q in range(7)])
    assert np.allclose(Yq, p["X"] @ Wq.T, rtol=1e-13)


# ---------------------------------------------------------------- error sums (App. B, initialisation table)

def test_error_sums_on_a_hand_worked_row():
    """Two groups of four weights with scales and biases that are exact in binary, so every figure below is exact:
    group 0 (s = 1/4, b = 1/2, 3 bits: Q_N = -4, Q_P = 3): w = 1.25, 3.75 (clipped above), 0.5 (a rounding tie), -5
    (clipped below); group 1 (s = 1/2, b = -1): w = 2.5 (tie), -4 (on the lower grid end, in range), 3.5 (clipped), 0."""
    s = np.array([[0.25, 0.5]])
    b = np.array([[0.5, -1.0]])
    w = np.array([[1.25, 3.75, 0.5, -5.0, 2.5, -4.0, 3.5, 0.0]])
    Wc = np.array([[0.8125, 1.4375, 0.625, -0.75, 0.25, -3.0, 0.75, -1.0]])      # b + s w, written out
    assert np.array_equal(O.prequant(Wc, s, b, 4), w)
    # |Wc - Wq| = s |w - round(clamp(w))|:  .25 (.25 + .75 + .5 + 1) + .5 (.5 + 0 + .5 + 0)
    assert O.quantization_error(Wc, s, b, 3, 4) == 0.625 + 0.5
    # |Wc - (clamp(w) s + b)| = s |w - clamp(w)|:  .25 (0 + .75 + 0 + 1) + .5 (0 + 0 + .5 + 0)
    assert O.clipping_error(Wc, s, b, 3, 4) == 0.4375 + 0.25
    # one more bit: nothing clips any more, the rounding error remains: .25 (.25 + .25 + .5 + 0) + .5 (.5 + 0 + .5 + 0)
    assert O.clipping_error(Wc, s, b, 4, 4) == 0.0
    assert O.quantization_error(Wc, s, b, 4, 4) == 0.25 + 0.5


def test_quantization_error_splits_into_clipping_and_rounding_parts():
    """|Wc - Wq| = s |w - c|: outside the grid c = clamp(w) and the whole difference is clipping; inside it
    clamp(w) = w and the whole difference is rounding.  So E_quant = E_clip + sum s |clamp(w) - round(clamp(w))|,
    evaluated here without any oracle function on the right-hand side."""
    rng = np.random.default_rng(41)
    o, i, g, bits = 24, 256, 32, 3
    Wc = rng.standard_normal((o, i)) * 0.02
    Wc[rng.random(Wc.shape) < 5e-3] *= 20
    s = (Wc.reshape(o, i // g, g).max(axis=2) - Wc.reshape(o, i // g, g).min(axis=2)) / 7 * 0.7   # clips
    b = rng.standard_normal(s.shape) * 0.01
    se, be = np.repeat(s, g, axis=1), np.repeat(b, g, axis=1)
    w = (Wc - be) / se
    cl = np.clip(w, -4, 3)
    rounding = float((se * np.abs(cl - np.round(cl))).sum())
    clipping = float((se * np.abs(w - cl)).sum())
    assert clipping > 0
    assert math.isclose(O.clipping_error(Wc, s, b, bits, g), clipping, rel_tol=1e-11)
    assert math.isclose(O.quantization_error(Wc, s, b, bits, g), clipping + rounding, rel_tol=1e-11)
    # the two sums respond differently to a mistake: dropping the clamp from E_quant, or the rounding from it
    assert not math.isclose(clipping + rounding, rounding, rel_tol=1e-3)


# ---------------------------------------------------------------- LSQ+ initialisation (App. B, Eq. quant_inits)

def test_lsqplus_init_uses_mean_and_population_deviation():
    """Group {1, 2, 3, 6}: mean 3, squared deviations 4 + 1 + 0 + 9 = 14, population variance 14 / 4 = 3.5.
    s = max(|3 - 3 sqrt(3.5)|, |3 + 3 sqrt(3.5)|) / 2^(n-1).  (The sample deviation sqrt(14 / 3) would give 1.185 at
    4 bits instead of 1.0766, a factor 2 sigma 0.843, a denominator Q_P 1.2304.)"""
    W = np.array([[1.0, 2.0, 3.0, 6.0, -1.0, -2.0, -3.0, -6.0]])
    s, b = O.init_qparams(W, 4, 4, "lsq+")
    assert s.shape == (1, 2) and not b.any()
    assert abs(s[0, 0] - 1.076560760020114) < 1e-15            # (3 + 3 * 1.8708286933869707) / 8
    assert abs(s[0, 1] - 1.076560760020114) < 1e-15            # mirrored group: |mu - 3 sigma| is the larger one
    s3, _ = O.init_qparams(W, 3, 4, "lsq+")
    assert abs(s3[0, 0] - 2.153121520040228) < 1e-15           # / 4 at 3 bits


# ---------------------------------------------------------------- binary32 initialisation: operation order

@pytest.mark.parametrize("bits", [3, 4])
def test_f32_init_operation_order(bits):
    """init_qparams(dtype=float32) is the bit-exact referee of the GPU initialisation kernel: re-evaluate every scheme
    with scalar binary32 operations, one rounding per written operation, on a few groups."""
    f = np.float32
    rng = np.random.default_rng(43)
    g = 8
    W = (rng.standard_normal((3, 4 * g)) * 0.03).astype(f)
    qn, qp = f(-(1 << (bits - 1))), f((1 << (bits - 1)) - 1)
    got = {m: O.init_qparams(W, bits, g, m, dtype=f) for m in ("asymm", "symm", "l4q", "lsq+")}
    for m in got:
        assert got[m][0].dtype == f and got[m][1].dtype == f
    for p in range(3):
        for q in range(4):
            grp = W[p, q * g:(q + 1) * g]
            lo, hi = f(min(grp)), f(max(grp))
            s = f(f(hi - lo) / f(qp - qn))
            assert got["asymm"][0][p, q] == s
            assert got["asymm"][1][p, q] == f(lo - f(s * qn))
            assert got["symm"][0][p, q] == f(f(max(abs(lo), abs(hi))) / f(1 << (bits - 1)))
            assert got["symm"][1][p, q] == 0
            assert got["l4q"][0][p, q] == f(max(abs(f(lo / qn)), abs(f(hi / qp))))
            assert got["l4q"][1][p, q] == 0
            # LSQ+ sums in an unspecified binary32 order: within a few units of the last place of the float64 value
            g64 = grp.astype(np.float64)
            mu = g64.sum() / g
            sd = math.sqrt(((g64 - mu) ** 2).sum() / g)
            want = max(abs(mu - 3 * sd), abs(mu + 3 * sd)) / (1 << (bits - 1))
            assert abs(float(got["lsq+"][0][p, q]) - want) <= 4e-7 * want
    # the fused form lo - s qn in one rounding would differ somewhere on data like this; so would s = (hi - lo) * (1 / 15)
    lo = W.reshape(3, 4, g).min(axis=2)
    hi = W.reshape(3, 4, g).max(axis=2)
    assert got["asymm"][0].tobytes() == ((hi - lo) / f(qp - qn)).astype(f).tobytes()
