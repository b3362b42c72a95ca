"""CPU oracle of the paper's two-input lookup, integer cross-entropy loss derivative (Algorithm "IntCELossDeriv",
Sec. "Integer Cross-Entropy Loss Derivative") and clipped weight update (last step of Algorithm "End-to-End Training").

TEST INFRASTRUCTURE ONLY: imported by tests/ and by bench.py's cpu_baseline leg; the GPU library never imports it.

As in gadgets.py there are two layers: clear-integer clones in plain numpy, and the same steps on LWE ciphertexts with
every lookup being one programmable bootstrapping + one keyswitch of the CGGI oracle.

Readings of points the paper leaves open or prints garbled:
  R10 A lookup with two encrypted inputs x in [0, 2^bx) and y in [0, 2^by), bx + by <= msg_bits, is one lookup on the packed
      value 2^by x + y (the paper names the two-input lookup and gives no packing; R2 is the case bx = by = 4).
  R11 The first two lines of the algorithm are taken as a data flow: E = ReLU(Y^), then the exponential lookup on E.  The
      exponential table is v -> round(2^kappa e^(v - (2^gamma - 1))), gamma = Gamma - 1 (the figure's formula; the largest
      logit 2^gamma - 1 maps to 2^kappa), rounding to nearest, ties to even, as the algorithm's comment says.
  R12 The argument of the two-input lookup is printed without brackets.  It is read as round((E 2^kappa + 1) / (S + 1)), ties to
      even: the "+ 1" below keeps the division defined when every exponential rounds to 0 (S = 0), and the "+ 1" above then
      gives every class the same share, which is what softmax gives for equal logits.  Input widths: E <= 2^kappa takes
      kappa + 1 bits, S <= b 2^kappa takes ceil(log2(b 2^kappa + 1)) bits; both together must fit the message space.
  R13 E - Y sum(E): the labels are encrypted like the rest of the training data, so Y_i sum(E) is a product of two encrypted
      values, taken as one two-input lookup on 2^sb Y_i + sum(E) (the row sum of the shares stays below 2^sb).
      The error E - Y sum(E) can be negative, and a negative difference of two ciphertexts would land in the padding half of
      the torus; as in R4 it is moved up by the constant t / 2 before the sign lookup, whose table is v -> sign(v - t / 2).
  R14 The clipped weight update clip(W - G) is one two-input lookup on 4 (W + 2^(alpha-1)) + (G + 1) for signed alpha-bit
      weights W and G in {-1, 0, 1}; it needs alpha + 2 <= msg_bits, and clips to [-2^(alpha-1), 2^(alpha-1) - 1] (the
      paper's [-128, 127] is alpha = 8).  W comes encoded with negatives in the upper half of Z_t (4 W is then right modulo
      2 t); the second operand comes as the code G + 1 in {0, 1, 2}, i.e. the sign gadget is asked for the results (0, 1, 2)
      instead of (-1, 0, 1): an encoded -1 = t - 1 added with weight 1 would set the padding bit.
"""
from __future__ import annotations

import numpy as np

from .gadgets import _add_const, _lookup, signed_decode, signed_encode


def _bits(v: int) -> int:
    """ceil(log2(v + 1)): bits needed for the values 0..v."""
    return int(v).bit_length()


def round_half_even_div(num, den):
    """round(num / den) for non-negative integers, ties to the even neighbour; exact integer arithmetic."""
    num = np.asarray(num, dtype=np.int64)
    den = np.asarray(den, dtype=np.int64)
    q, r = np.divmod(num, den)
    up = (2 * r > den) | ((2 * r == den) & (q % 2 == 1))
    return q + up.astype(np.int64)


# ---- two-input lookup (R10) -------------------------------------------------------------------------------------------
def bivariate_table(p, f, bx: int, by: int) -> np.ndarray:
    """Table over Z_t of the packed index u = 2^by x + y -> f(x, y) mod t; entries past 2^(bx+by) are 0."""
    t = 1 << p.msg_bits
    if bx + by > p.msg_bits:
        raise ValueError("the packed index needs %d bits, the message space has %d" % (bx + by, p.msg_bits))
    tab = np.zeros(t, dtype=np.int64)
    for x in range(1 << bx):
        for y in range(1 << by):
            tab[(x << by) + y] = int(f(x, y)) % t
    return tab.astype(np.uint64)


def bivariate_lookup_encrypted(p, x_cts, y_cts, by: int, tables, idx, bsk, ksk) -> np.ndarray:
    """One two-input lookup per ciphertext pair: the packed ciphertext 2^by x + y, then table idx[c]."""
    with np.errstate(over="ignore"):
        packed = x_cts * np.uint64(1 << by) + y_cts
    return _lookup(p, packed, tables, idx, bsk, ksk)


# ---- IntCELossDeriv ------------------------------------------------------------------------------------------------------
def exp_value(v, Gamma: int, kappa: int):
    """The approximated exponential of the figure "exp_approx": round(e^v / e^(2^gamma - 1) 2^kappa), gamma = Gamma - 1."""
    top = (1 << (Gamma - 1)) - 1
    return np.rint(np.exp(np.asarray(v, dtype=np.float64) - top) * (1 << kappa)).astype(np.int64)     # rint: ties to even


def loss_widths(b: int, kappa: int):
    """(bits of an exponential, bits of a row sum of b of them)."""
    return _bits(1 << kappa), _bits(b << kappa)


def int_ce_loss_deriv_clear(Yhat, Y, Gamma: int, kappa: int, return_error: bool = False) -> np.ndarray:
    """Algorithm "IntCELossDeriv" on clear integers.  Yhat: a x b signed Gamma-bit logits, Y: a x b one-hot labels.
    Returns the sign of the error, a x b in {-1, 0, 1} (with return_error: the error before the sign step)."""
    Yhat = np.asarray(Yhat, dtype=np.int64)
    Y = np.asarray(Y, dtype=np.int64)
    a, b = Yhat.shape
    if b > 16:
        raise ValueError("at most 16 output neurons")
    E = np.maximum(Yhat, 0)
    E = exp_value(E, Gamma, kappa)
    S = E.sum(axis=1).reshape(a, 1)
    E = round_half_even_div(E * (1 << kappa) + 1, S + 1)
    E = E - Y * E.sum(axis=1).reshape(a, 1)
    if return_error:
        return E
    return (E > 0).astype(np.int64) - (E < 0).astype(np.int64)


def loss_tables(p, b: int, Gamma: int, kappa: int) -> np.ndarray:
    """The five tables of the encrypted algorithm over Z_t: ReLU (signed input), exponential, share (E, S) ->
    round((E 2^kappa + 1) / (S + 1)), product (Y, T) -> Y T, and v -> sign(v - t / 2) (results -1, 0, 1 encoded with negatives
    in the upper half)."""
    t = 1 << p.msg_bits
    eb, sb = loss_widths(b, kappa)
    if Gamma < 2 or Gamma > p.msg_bits or eb + sb > p.msg_bits:
        raise ValueError("Gamma = %d, kappa = %d, b = %d do not fit a %d-bit message space" % (Gamma, kappa, b, p.msg_bits))
    v = np.arange(t, dtype=np.int64)
    sv = signed_decode(v, t)
    relu = np.maximum(sv, 0)
    ex = np.where(v < (1 << (Gamma - 1)), exp_value(np.minimum(v, (1 << (Gamma - 1)) - 1), Gamma, kappa), 0)
    share = bivariate_table(p, lambda e, s: round_half_even_div(e * (1 << kappa) + 1, s + 1), eb, sb).astype(np.int64)
    prod = bivariate_table(p, lambda y, s: y * s, 1, sb).astype(np.int64)
    sgn = signed_encode((v > t // 2).astype(np.int64) - (v < t // 2).astype(np.int64), t)
    return np.stack([relu, ex, share, prod, sgn]).astype(np.uint64)


def int_ce_loss_deriv_encrypted(p, yhat_cts, y_cts, Gamma: int, kappa: int, bsk, ksk) -> np.ndarray:
    """Algorithm "IntCELossDeriv" on ciphertexts.  yhat_cts: a x b x (n+1) encryptions of signed logits (negatives in the upper
    half of Z_t), y_cts: a x b x (n+1) encryptions of the one-hot labels.  Returns a x b x (n+1) encryptions of the sign."""
    a, b = yhat_cts.shape[:2]
    tabs = loss_tables(p, b, Gamma, kappa)
    _, sb = loss_widths(b, kappa)
    which = lambda i: np.full((a, b), i, dtype=np.uint32)
    E = _lookup(p, yhat_cts, tabs, which(0), bsk, ksk)
    E = _lookup(p, E, tabs, which(1), bsk, ksk)
    with np.errstate(over="ignore"):
        S = np.broadcast_to(E.sum(axis=1, dtype=np.uint64)[:, None, :], E.shape)
    E = bivariate_lookup_encrypted(p, E, S, sb, tabs, which(2), bsk, ksk)
    with np.errstate(over="ignore"):
        T = np.broadcast_to(E.sum(axis=1, dtype=np.uint64)[:, None, :], E.shape)
    P = bivariate_lookup_encrypted(p, np.asarray(y_cts, dtype=np.uint64), T, sb, tabs, which(3), bsk, ksk)
    with np.errstate(over="ignore"):
        E = _add_const(p, E - P, (1 << p.msg_bits) // 2)
    return _lookup(p, E, tabs, which(4), bsk, ksk)


# ---- clipped weight update (R14) ------------------------------------------------------------------------------------
def weight_update_clear(W, G, alpha: int) -> np.ndarray:
    """clip(W - G) to the signed alpha-bit range."""
    lo, hi = -(1 << (alpha - 1)), (1 << (alpha - 1)) - 1
    return np.clip(np.asarray(W, dtype=np.int64) - np.asarray(G, dtype=np.int64), lo, hi)


def weight_update_table(p, alpha: int) -> np.ndarray:
    """Table of the packed index 4 (w + 2^(alpha-1)) + (g + 1) -> clip(w - g), signed result encoded in Z_t."""
    t = 1 << p.msg_bits
    if alpha < 2 or alpha + 2 > p.msg_bits:
        raise ValueError("alpha + 2 must fit the message space")
    half = 1 << (alpha - 1)

    def f(wu, gu):
        g = min(gu, 2) - 1                                           # code 3 is never produced; treated as +1
        return int(weight_update_clear(wu - half, g, alpha)) % t
    return bivariate_table(p, f, alpha, 2)[None]


def weight_update_encrypted(p, w_cts, gcode_cts, alpha: int, bsk, ksk) -> np.ndarray:
    """The clipped update on ciphertexts, count x (n+1) each: w_cts signed weights (negatives in the upper half of Z_t),
    gcode_cts the codes G + 1 in {0, 1, 2}."""
    with np.errstate(over="ignore"):
        packed = _add_const(p, w_cts * np.uint64(4) + gcode_cts, 4 * (1 << (alpha - 1)))
    return _lookup(p, packed, weight_update_table(p, alpha), np.zeros(w_cts.shape[0], dtype=np.uint32), bsk, ksk)
