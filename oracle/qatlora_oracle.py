"""CPU oracle for the QAT-LoRA layer, the straightforward integration of QAT and LoRA that the paper
starts from and then replaces (Sec. 3.1 "Straight Integration of QAT and LoRA").

TEST INFRASTRUCTURE ONLY; shares no code with the HIP path.  It reuses the quantizer definitions of
l4q_oracle (same Eq. quant) and follows the section's description: the frozen weight alone goes
through the quantizer, the LoRA path stays in high precision next to it, the weight gradient
dL/dWq is materialised to update scale and zero, and the LoRA factors get the plain LoRA gradients
(Eq. lora_forward / lora_backward) -- the two sets of gradients do not see each other.

    Wq   = dequant(round(clamp((W0 - b) / s)))                                  (Eq. quant)
    Y    = X Wq^T + gamma (X A^T) B^T                                           (Sec. 3.1, Eq. lora_forward)
    dX   = dY Wq + gamma (dY B) A
    dWq  = dY^T X                                                               (kept: the memory overhead the section names)
    ds, db from dWq exactly as in Eq. quant_lsq_s / quant_lsq_b (App. A.1 case list), w taken from W0 alone
    dA   = gamma (dY B)^T X,   dB = gamma dY^T (X A^T)                          (Eq. lora_backward)

gamma = alpha / r as everywhere in this build.  float64 throughout; the discrete decisions may be
passed in (the binary32 chain of l4q_oracle.decide_f32 evaluated with B = 0).

Pins (tests/test_oracle_qatlora.py): B = 0 gives the L4Q oracle's output, d(scale) and d(zero) at
B = 0; the LoRA part equals the textbook form computed in the other association order; dA, dB and dX
against central finite differences of sum(dY * Y) (Y is bilinear in A, B and linear in X, and the
quantizer does not see them, so the differences are exact up to rounding).
"""
from __future__ import annotations

from typing import NamedTuple, Optional

import numpy as np

from oracle import l4q_oracle as O

F64 = np.float64


def decisions_f64(W0, s, b, bits: int, g: int) -> O.Decisions:
    w = O.prequant(np.asarray(W0, F64), s, b, g)
    return O.Decisions(O.codes_from_w(w, bits), O.ste_mask(w, bits))


def forward(X, W0, A, B, s, b, bits: int, g: int, alpha: float,
            decisions: Optional[O.Decisions] = None) -> np.ndarray:
    X, A, B = (np.asarray(v, F64) for v in (X, A, B))
    if decisions is None:
        decisions = decisions_f64(W0, s, b, bits, g)
    Wq = O.dequant(decisions.codes, s, b, g)
    gamma = float(alpha) / A.shape[0]
    return X @ Wq.T + gamma * ((X @ A.T) @ B.T)


class Grads(NamedTuple):
    dX: np.ndarray      # [T, i]
    dA: np.ndarray      # [r, i]
    dB: np.ndarray      # [o, r]
    dscale: np.ndarray  # [o, i/g]
    dzero: np.ndarray   # [o, i/g]
    dWq: np.ndarray     # [o, i]


def backward(X, dY, W0, A, B, s, b, bits: int, g: int, alpha: float,
             decisions: Optional[O.Decisions] = None) -> Grads:
    X, dY, A, B = (np.asarray(v, F64) for v in (X, dY, A, B))
    o, i = np.asarray(W0).shape
    gamma = float(alpha) / A.shape[0]
    w = O.prequant(np.asarray(W0, F64), s, b, g)
    if decisions is None:
        decisions = O.Decisions(O.codes_from_w(w, bits), O.ste_mask(w, bits))
    c = np.asarray(decisions.codes, F64)
    m = np.asarray(decisions.mask, bool)
    Wq = O.dequant(c, s, b, g)

    dYB = dY @ B                      # [T, r]
    XA = X @ A.T                      # [T, r]
    dX = dY @ Wq + gamma * (dYB @ A)
    dWq = dY.T @ X
    G = i // g
    dscale = (dWq * np.where(m, c - w, c)).reshape(o, G, g).sum(axis=2)
    dzero = (dWq * np.where(m, 0.0, 1.0)).reshape(o, G, g).sum(axis=2)
    dA = gamma * (dYB.T @ X)
    dB = gamma * (dY.T @ XA)
    return Grads(dX, dA, dB, dscale, dzero, dWq)
