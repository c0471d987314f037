"""CPU oracle for the L4Q quantization-aware LoRA linear layer (arXiv 2402.04902).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP
kernels are checked against.  It shares no code with the HIP path and must not
be imported by the product; only tests, the smoke check and the CPU-baseline
leg of the benchmark use it.

Everything is written in the row-major "tokens first" orientation
    Y[T,o] = X[T,i] . Wq[o,i]^T
which is the transposed statement of the paper's Y = Wq X (Sec. 3.2,
Eq. l4q_forward).  Quantization groups are g consecutive elements along the
in-feature axis of one weight row; scale s and bias ("zero") b have shape
[o, i/g] and are real-valued (Sec. 2.2, Eq. quant).  The LoRA scaling constant
the paper calls alpha is gamma = alpha / r here.

Two families of functions:

* float64 functions follow the paper's equations one by one with no blocking,
  fusion or reordering; numpy's matmul is the only library primitive.
* ``*_f32`` functions evaluate the discrete part (merge, pre-round value,
  code, straight-through mask) in strict IEEE binary32 with a fixed operation
  order.  Integer codes and masks of the HIP path are compared bit for bit
  with these; the float64 gradient functions accept such decisions so that a
  code sitting on a rounding tie does not pollute a floating-point comparison.

Pins (see tests/test_oracle_*.py): grid size 2^n; clamp/round commutation and
half-even ties; B = 0 reduces to plain group-wise fake quantization; min/max
initialisation gives zero clipping error (Table 5, E_clip = 0.0 at init);
mask == 1 reduces dA, dB to the plain LoRA gradients (Eq. lora_backward);
closed forms of d(scale), d(zero), dA, dB against hand-rolled forward-mode
dual numbers (App. A.1, A.2); finite differences on clipped groups and on X;
brute-force triple loops on tiny shapes; the error sums E_quant / E_clip on a
hand-worked row and through their split into a clipping and a rounding part;
LSQ+ initialisation on a group whose mean and population deviation are written
out; the binary32 initialisation re-evaluated with scalar binary32 operations.
"""
from __future__ import annotations

from typing import NamedTuple, Optional, Tuple

import numpy as np

F64 = np.float64
F32 = np.float32


def q_bounds(bits: int) -> Tuple[int, int]:
    """Q_N = -2^(n-1), Q_P = 2^(n-1) - 1  (Sec. 2.2, text after Eq. quant)."""
    return -(1 << (bits - 1)), (1 << (bits - 1)) - 1


def _per_element(v: np.ndarray, g: int) -> np.ndarray:
    """Broadcast a per-group array [o, i/g] to per-element [o, i]."""
    return np.repeat(v, g, axis=1)


# --------------------------------------------------------------------------
# float64 definition
# --------------------------------------------------------------------------

def merge(W0, A, B, alpha: float) -> np.ndarray:
    """W_comb = W0 + gamma * B A   (Sec. 3.2, Eq. l4q_Wcombine), gamma = alpha / r."""
    W0, A, B = (np.asarray(v, F64) for v in (W0, A, B))
    gamma = float(alpha) / A.shape[0]
    return W0 + gamma * (B @ A)


def prequant(Wc, s, b, g: int) -> np.ndarray:
    """w = (W_comb - b) / s   (App. A.2, Eq. appen_l4q_w)."""
    return (np.asarray(Wc, F64) - _per_element(np.asarray(b, F64), g)) / _per_element(np.asarray(s, F64), g)


def codes_from_w(w: np.ndarray, bits: int) -> np.ndarray:
    """w~ = round(clamp(w, Q_N, Q_P))   (Eq. l4q_Wquant); ties go to the even integer."""
    qn, qp = q_bounds(bits)
    return np.rint(np.minimum(np.maximum(w, qn), qp))


def ste_mask(w: np.ndarray, bits: int) -> np.ndarray:
    """1 where Q_N <= w <= Q_P on the pre-round value, else 0   (App. A.1, Eq. appen_ste)."""
    qn, qp = q_bounds(bits)
    return (w >= qn) & (w <= qp)


def dequant(c, s, b, g: int) -> np.ndarray:
    """W_q = w~ * s + b   (Eq. l4q_Wdequant)."""
    return np.asarray(c, F64) * _per_element(np.asarray(s, F64), g) + _per_element(np.asarray(b, F64), g)


class Decisions(NamedTuple):
    """Discrete outcomes of the quantizer: integer codes and straight-through mask."""
    codes: np.ndarray  # [o, i] integer valued
    mask: np.ndarray   # [o, i] bool


def decide_f64(W0, A, B, s, b, bits: int, g: int, alpha: float) -> Decisions:
    w = prequant(merge(W0, A, B, alpha), s, b, g)
    return Decisions(codes_from_w(w, bits), ste_mask(w, bits))


def quantized_weight(W0, A, B, s, b, bits, g, alpha, decisions: Optional[Decisions] = None) -> np.ndarray:
    if decisions is None:
        decisions = decide_f64(W0, A, B, s, b, bits, g, alpha)
    return dequant(decisions.codes, s, b, g)


def forward(X, W0, A, B, s, b, bits: int, g: int, alpha: float,
            decisions: Optional[Decisions] = None) -> np.ndarray:
    """Y = X Wq^T   (Eq. l4q_forward)."""
    Wq = quantized_weight(W0, A, B, s, b, bits, g, alpha, decisions)
    return np.asarray(X, F64) @ Wq.T


class Grads(NamedTuple):
    dX: np.ndarray      # [T, i]
    dA: np.ndarray      # [r, i]
    dB: np.ndarray      # [o, r]
    dscale: np.ndarray  # [o, i/g]
    dzero: np.ndarray   # [o, i/g]
    dWq: np.ndarray     # [o, i]  (local weight gradient, for inspection)


def backward(X, dY, W0, A, B, s, b, bits: int, g: int, alpha: float,
             decisions: Optional[Decisions] = None) -> Grads:
    """Gradients of L with upstream dL/dY = dY.

    dX    = dY Wq                                  (transpose of Eq. l4q_forward)
    dWq   = dY^T X                                 (Sec. 3.2 "Memory Efficient QAT"; Eq. appen_wq)
    ds    = sum_group dWq * dWq/ds,  dWq/ds = w~ - w in range, Q_N / Q_P when clipped
                                                   (Eq. quant_lsq_s and the case list of App. A.1)
    db    = sum_group dWq * dWq/db,  dWq/db = 0 in range, 1 when clipped   (Eq. appen_lsq_b)
    dA    = gamma B^T (mask * dWq),  dB = gamma (mask * dWq) A^T           (Eq. appen_l4q_a / appen_l4q_b,
                                                   mask applied per element as the chain rule of
                                                   Eq. appen_a / appen_b requires)
    No extra LSQ gradient scaling is applied: the paper states a plain product.
    """
    X, dY, A, B = (np.asarray(v, F64) for v in (X, dY, A, B))
    o, i = np.asarray(W0).shape
    r = A.shape[0]
    gamma = float(alpha) / r
    w = prequant(merge(W0, A, B, alpha), s, b, g)
    if decisions is None:
        decisions = Decisions(codes_from_w(w, bits), ste_mask(w, bits))
    c = np.asarray(decisions.codes, F64)
    m = np.asarray(decisions.mask, bool)
    Wq = dequant(c, s, b, g)

    dX = dY @ Wq
    dWq = dY.T @ X
    # when clipped, the code c already equals Q_N or Q_P
    dWq_ds = np.where(m, c - w, c)
    dWq_db = np.where(m, 0.0, 1.0)
    G = i // g
    dscale = (dWq * dWq_ds).reshape(o, G, g).sum(axis=2)
    dzero = (dWq * dWq_db).reshape(o, G, g).sum(axis=2)
    dWp = np.where(m, dWq, 0.0)
    dA = gamma * (B.T @ dWp)
    dB = gamma * (dWp @ A.T)
    return Grads(dX, dA, dB, dscale, dzero, dWq)


# --------------------------------------------------------------------------
# strict binary32 evaluation of the discrete part
# --------------------------------------------------------------------------

def merge_f32(W0, A, B, alpha: float) -> np.ndarray:
    """Binary32 merged weight with a fixed operation order.

    acc = 0; for k = 0..r-1: acc = fl(acc + fl(B[p,k] * A[k,j]));
    W_comb = fl(W0 + fl(gamma * acc)),  gamma = fl(fl(alpha) / fl(r)).
    Every operation is one correctly rounded binary32 operation (no fused
    multiply-add).  With bfloat16 inputs the products are exact, so a fused
    multiply-add gives the same bits.
    """
    W0, A, B = (np.ascontiguousarray(v, F32) for v in (W0, A, B))
    r = A.shape[0]
    acc = np.zeros(W0.shape, F32)
    for k in range(r):
        acc = acc + B[:, k:k + 1] * A[k:k + 1, :]
    gamma = F32(alpha) / F32(r)
    return W0 + gamma * acc


def prequant_f32(Wc32, s, b, g: int) -> np.ndarray:
    """w = fl(fl(W_comb - b) / s) in binary32: one subtract, one correctly rounded divide."""
    Wc32 = np.ascontiguousarray(Wc32, F32)
    s32 = _per_element(np.asarray(s, F32), g)
    b32 = _per_element(np.asarray(b, F32), g)
    return (Wc32 - b32) / s32


def decide_f32(W0, A, B, s, b, bits: int, g: int, alpha: float) -> Tuple[Decisions, np.ndarray, np.ndarray]:
    """Codes and mask from the binary32 chain; also returns W_comb (f32) and w (f32)."""
    qn, qp = q_bounds(bits)
    Wc32 = merge_f32(W0, A, B, alpha)
    w32 = prequant_f32(Wc32, np.asarray(s, F32), np.asarray(b, F32), g)
    codes = np.rint(np.minimum(np.maximum(w32, F32(qn)), F32(qp))).astype(np.int8)
    mask = (w32 >= F32(qn)) & (w32 <= F32(qp))
    return Decisions(codes, mask), Wc32, w32


def tie_and_boundary_sets(w64: np.ndarray, bits: int, rel: float = 2.0 ** -20) -> Tuple[np.ndarray, np.ndarray]:
    """Elements whose code or mask may legitimately differ between binary32 and binary64.

    near-tie: |frac(w) - 1/2| < rel * max(1, |w|); near-boundary: |w - Q_N| or |w - Q_P|
    below the same threshold.
    """
    qn, qp = q_bounds(bits)
    thr = rel * np.maximum(1.0, np.abs(w64))
    frac = w64 - np.floor(w64)
    near_tie = np.abs(frac - 0.5) < thr
    near_bnd = (np.abs(w64 - qn) < thr) | (np.abs(w64 - qp) < thr)
    return near_tie, near_bnd


# --------------------------------------------------------------------------
# quantization-parameter initialisation (Sec. 3.3, App. B Eq. quant_inits)
# --------------------------------------------------------------------------

def init_qparams(Wc, bits: int, g: int, method: str = "asymm", dtype=F64) -> Tuple[np.ndarray, np.ndarray]:
    """Per-group scale s and bias b from the merged weight.

    asymm : s = (max - min) / (Q_P - Q_N),  b = min - s Q_N
    symm  : s = max|W| / 2^(n-1),           b = 0
    l4q   : s = max(|min / Q_N|, |max / Q_P|), b = 0      (Eq. l4q_quant_init)
    lsq+  : s = max(|mu - 3 sigma|, |mu + 3 sigma|) / 2^(n-1), b = 0
    With dtype=float32 each step is one binary32 operation in the order written.
    """
    qn, qp = q_bounds(bits)
    Wc = np.asarray(Wc, dtype)
    o, i = Wc.shape
    grp = Wc.reshape(o, i // g, g)
    lo, hi = grp.min(axis=2), grp.max(axis=2)
    T = dtype
    if method == "asymm":
        s = (hi - lo) / T(qp - qn)
        b = lo - s * T(qn)
    elif method == "symm":
        s = np.maximum(np.abs(lo), np.abs(hi)) / T(1 << (bits - 1))
        b = np.zeros_like(s)
    elif method == "l4q":
        s = np.maximum(np.abs(lo / T(qn)), np.abs(hi / T(qp)))
        b = np.zeros_like(s)
    elif method == "lsq+":
        mu = grp.mean(axis=2)
        sd = grp.std(axis=2)
        s = np.maximum(np.abs(mu - 3 * sd), np.abs(mu + 3 * sd)) / T(1 << (bits - 1))
        b = np.zeros_like(s)
    else:
        raise ValueError(method)
    return s.astype(dtype), b.astype(dtype)


def clipping_error(Wc, s, b, bits: int, g: int) -> float:
    """E_clip = sum |W_comb - (clamp(w) s + b)|: what overflowed outliers lose (App. B, Table 5).

    The paper names the quantity without a formula; this is the reading used here.
    """
    qn, qp = q_bounds(bits)
    w = prequant(Wc, s, b, g)
    back = dequant(np.minimum(np.maximum(w, qn), qp), s, b, g)
    return float(np.abs(np.asarray(Wc, F64) - back).sum())


def quantization_error(Wc, s, b, bits: int, g: int) -> float:
    """E_quant = sum |W_comb - W_q|  (App. B, Table 5; formula is this file's reading)."""
    w = prequant(Wc, s, b, g)
    return float(np.abs(np.asarray(Wc, F64) - dequant(codes_from_w(w, bits), s, b, g)).sum())


# --------------------------------------------------------------------------
# fully quantized layer: packed integer codes and the single forward path
# (Sec. 3.2: inference uses only Wq = w~ s + b; Eq. l4q_forward)
# --------------------------------------------------------------------------

def pack_codes(codes, bits: int) -> np.ndarray:
    """Pack integer codes [o, i] into 32-bit words [o, bits*i/32].

    The unsigned field u = w~ - Q_N (0 .. 2^n - 1) of column j occupies bits [n j, n j + n) of the
    row's little-endian bit string; i must be a multiple of 32 so that rows end on a word.
    The paper fixes no storage format; this is the layout of this repository.
    """
    qn, _ = q_bounds(bits)
    c = np.asarray(codes).astype(np.int64)
    o, i = c.shape
    assert i % 32 == 0
    u = (c - qn).astype(np.uint64)
    words = np.zeros((o, bits * i // 32), dtype=np.uint64)
    for j in range(i):
        bit = bits * j
        w, sh = bit >> 5, bit & 31
        words[:, w] |= (u[:, j] << np.uint64(sh)) & np.uint64(0xFFFFFFFF)
        if sh + bits > 32:
            words[:, w + 1] |= u[:, j] >> np.uint64(32 - sh)
    return words.astype(np.uint32)


def unpack_codes(packed, bits: int, i: int) -> np.ndarray:
    """Inverse of pack_codes: integer codes [o, i] (int64)."""
    qn, _ = q_bounds(bits)
    p = np.asarray(packed).astype(np.uint64)
    o = p.shape[0]
    out = np.empty((o, i), dtype=np.int64)
    mask = np.uint64((1 << bits) - 1)
    for j in range(i):
        bit = bits * j
        w, sh = bit >> 5, bit & 31
        v = p[:, w] >> np.uint64(sh)
        if sh + bits > 32:
            v = v | (p[:, w + 1] << np.uint64(32 - sh))
        out[:, j] = (v & mask).astype(np.int64) + qn
    return out


def quantized_forward(X, packed, s, b, bits: int, g: int) -> np.ndarray:
    """Y = X Wq^T with Wq = w~ s + b rebuilt from the packed codes alone (no W0, A, B)."""
    i = np.asarray(X).shape[1]
    Wq = dequant(unpack_codes(packed, bits, i), s, b, g)
    return np.asarray(X, F64) @ Wq.T
