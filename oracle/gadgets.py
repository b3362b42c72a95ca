"""CPU oracle of the paper's Matmul^RNS (Algorithm "Matmul^RNS", Sec. "Low-bitwidth Matrix Multiplication"), and further down
of RNS2MRNS, Sign^RNS, Shift2MSBs^+/+- and MatmulHighRes^RNS (each section has its own header).

TEST INFRASTRUCTURE ONLY: imported by tests/ and by bench.py's cpu_baseline leg; the GPU library never imports it.

Two layers:

* `matmul_rns_clear`: the clear-integer clone (the paper validates its encrypted runs against such a clone,
  Sec. "Evaluation").  Plain numpy integers.
* `matmul_rns_encrypted`: the same steps on LWE ciphertexts, every table lookup (`mod`, the product of two encrypted
  residues, the reduction of a block sum) being one programmable bootstrapping followed by one keyswitch of the CGGI
  oracle in `tfhe_oracle.c`, and every sum a wrapping integer sum of ciphertext vectors.

Readings of points the paper leaves open:
  R1  Signed inputs (the set I_8) are encoded in Z_t, t = 2^msg_bits >= 256, as the paper encodes signed values in a ring:
      non-negative values in the lower half, negative ones in the upper half (v -> v + t).
  R2  The product of two encrypted residues is a lookup on the packed value 16 x' + w' (both residues are below 16 since the
      moduli are at most 4 bits wide); the paper names a two-input lookup and gives no packing.
  R3  In step 3 the loop as printed sums slices of Y; it is read as summing the slices Y*[:, :, i:j, :] of the partial
      products (the text: sub-sums of at most 15 summands, then summed modulo the base), and `Y <- Y + Y' mod m'` as
      (Y + Y') mod m': Y + Y' <= 14 + 15 * 14 = 224 still fits 8 bits, so one lookup reduces it.
"""
from __future__ import annotations

import math

import numpy as np

from . import keyswitch_batch, lut_encode, pbs_batch

# Table "RNS bases used in Silenzio": number of moduli -> base (4-bit moduli, the most significant one even)
RNS_BASES = {2: (15, 14), 3: (13, 15, 14), 4: (11, 13, 15, 14), 5: (7, 11, 13, 15, 8), 6: (5, 7, 9, 11, 13, 8)}
BLOCK = 15      # summands per sub-sum (step 3)


def rns_base_bitwidth(base) -> float:
    """log2 of the number of values the base represents (the table's "Max. Bitwidth" column)."""
    return math.log2(math.prod(base))


def get_rns_base(bits: float):
    """Smallest base of the table that represents `bits`-bit values (the paper's getRNSBase)."""
    for k in sorted(RNS_BASES):
        if rns_base_bitwidth(RNS_BASES[k]) >= bits:
            return RNS_BASES[k]
    raise ValueError("no base of the table holds %.2f bits" % bits)


def signed_encode(x, M: int) -> np.ndarray:
    """Signed value -> Z_M, negatives in the upper half."""
    return np.mod(np.asarray(x, dtype=np.int64), M)


def signed_decode(v, M: int) -> np.ndarray:
    """Z_M -> signed value: the lower half (v <= (M-1)/2) is non-negative, the upper half is v - M."""
    v = np.asarray(v, dtype=np.int64)
    return np.where(2 * v <= M - 1, v, v - M)


def crt_reconstruct(Y, m) -> np.ndarray:
    """RNS tensor (k, ...) -> signed integers in the centred range of Z_{M_k}."""
    m = [int(q) for q in m]
    M = math.prod(m)
    acc = np.zeros(np.asarray(Y).shape[1:], dtype=np.int64)
    for i, q in enumerate(m):
        Mi = M // q
        acc = (acc + np.asarray(Y[i], dtype=np.int64) * (Mi * pow(Mi, -1, q) % M)) % M
    return signed_decode(acc, M)


def matmul_rns_clear(X, W, m) -> np.ndarray:
    """Algorithm "Matmul^RNS" on clear integers.  X: a x b, W: b x c (signed), m: k moduli.  Returns Y: k x a x c residues.

    What the algorithm computes, written from its definition: per modulus q the residues of both inputs, all a b c
    products of residues reduced modulo q, the products of one output entry cut into consecutive blocks of at most 15,
    each block summed as plain integers, and the block sums folded left to right with one reduction modulo q per block.
    The quantity the block size exists for, (previous residue) + (block sum) < 256, is asserted."""
    X = np.asarray(X, dtype=np.int64)
    W = np.asarray(W, dtype=np.int64)
    a, b = X.shape
    c = W.shape[1]
    n_blocks = -(-b // BLOCK)
    out = []
    for q in (int(v) for v in m):
        products = (np.mod(X, q)[:, :, None] * np.mod(W, q)[None, :, :]) % q                    # a x b x c, each below q
        padded = np.zeros((a, n_blocks * BLOCK, c), dtype=np.int64)
        padded[:, :b, :] = products                                                              # zero products change no sum
        block_sums = padded.reshape(a, n_blocks, BLOCK, c).sum(axis=2)                           # a x blocks x c
        y = np.zeros((a, c), dtype=np.int64)
        for blk in range(n_blocks):
            assert int((y + block_sums[:, blk, :]).max()) < 256                                  # stays an 8-bit value
            y = (y + block_sums[:, blk, :]) % q
        out.append(y)
    return np.stack(out)


def lookup_tables(p, m):
    """The three families of lookup tables over Z_t (t = 2^msg_bits >= 256), one table per modulus each:
    reduce_signed[i][v] = signed(v) mod m_i;  product[i][u] = (u >> 4)(u & 15) mod m_i (u < 256);  reduce[i][v] = v mod m_i."""
    t = 1 << p.msg_bits
    if t < 256:
        raise ValueError("Matmul^RNS needs an 8-bit message space")
    v = np.arange(t, dtype=np.int64)
    red_s = np.stack([np.mod(signed_decode(v, t), q) for q in m])
    prod = np.stack([np.where(v < 256, np.mod((v >> 4) * (v & 15), q), 0) for q in m])
    red = np.stack([np.mod(v, q) for q in m])
    return red_s.astype(np.uint64), prod.astype(np.uint64), red.astype(np.uint64)


def _lookup(p, cts, tables, idx, bsk, ksk) -> np.ndarray:
    """One table lookup per ciphertext: programmable bootstrapping with table idx[c], then keyswitch back to the small key."""
    flat = np.ascontiguousarray(cts.reshape(-1, p.n + 1))
    big = pbs_batch(p, flat, lut_encode(p, tables), np.ascontiguousarray(idx.reshape(-1).astype(np.uint32)), bsk)
    return keyswitch_batch(p, big, ksk).reshape(cts.shape)


def matmul_rns_encrypted(p, x_cts, w_cts, m, bsk, ksk) -> np.ndarray:
    """Algorithm "Matmul^RNS" on ciphertexts.  x_cts: a x b x (n+1) encryptions of signed 8-bit values (R1), w_cts: b x c x (n+1).
    Returns k x a x c x (n+1) encryptions of the residues of X W."""
    m = [int(q) for q in m]
    k = len(m)
    a, b = x_cts.shape[:2]
    c = w_cts.shape[1]
    red_s, prod, red = lookup_tables(p, m)
    kk = np.arange(k, dtype=np.uint32)
    # Step 1: X' = X mod m', W' = W mod m'
    Xr = _lookup(p, np.broadcast_to(x_cts[None], (k, a, b, p.n + 1)), red_s, np.broadcast_to(kk[:, None, None], (k, a, b)), bsk, ksk)
    Wr = _lookup(p, np.broadcast_to(w_cts[None], (k, b, c, p.n + 1)), red_s, np.broadcast_to(kk[:, None, None], (k, b, c)), bsk, ksk)
    # Step 2: partial products, a lookup on 16 x' + w' (R2)
    with np.errstate(over="ignore"):
        packed = Xr[:, :, :, None, :] * np.uint64(16) + Wr[:, None, :, :, :]                     # k x a x b x c x (n+1)
    Ys = _lookup(p, packed, prod, np.broadcast_to(kk[:, None, None, None], (k, a, b, c)), bsk, ksk)
    # Step 3: block-wise summation (R3)
    idx = np.broadcast_to(kk[:, None, None], (k, a, c))
    n = min(BLOCK, b)
    with np.errstate(over="ignore"):
        Y = _lookup(p, Ys[:, :, :n, :, :].sum(axis=2, dtype=np.uint64), red, idx, bsk, ksk)
        i = n
        while i < b:
            j = min(i + n, b)
            Yp = Ys[:, :, i:j, :, :].sum(axis=2, dtype=np.uint64)
            Y = _lookup(p, Y + Yp, red, idx, bsk, ksk)
            i += n
    return Y


# ---------------------------------------------------------------------------------------------------------------------
# RNS-to-MRNS conversion (Algorithm "RNS2MRNS") and sign determination (Sec. "Sign Determination in RNS")
#
# Readings of points the paper leaves open:
#   R4  Each update (y_j - y_{i-1}) * (m_{i-1}^-1 mod m_j) of the conversion is one lookup, taken on the difference moved
#       into the non-negative range by the constant OFFSET = 16 (both operands are below 16): table v -> (v - 16) t mod m_j.
#   R5  Sign_(n,z,p): the top mixed-radix digit decides the sign (negative iff y_k >= r_k / 2, which needs r_k even); the
#       zero test is "sum of the mixed-radix digits == 0" as the paper states.  Both flags are combined in one lookup on
#       sum + 128 [negative] (the digit sum of at most six 4-bit digits stays below 128): 0 -> z, 1..127 -> p, >= 128 -> n.
OFFSET = 16


def rns_encode(x, m) -> np.ndarray:
    """Signed integers -> residues, shape (k, ...)."""
    x = np.asarray(x, dtype=np.int64)
    return np.stack([np.mod(x, int(q)) for q in m])


def rns2mrns_clear(x, m) -> np.ndarray:
    """Algorithm "RNS2MRNS" (Szabo-Tanaka): residues (k, ...) -> mixed-radix digits (k, ...) of the associated base."""
    m = [int(q) for q in m]
    k = len(m)
    y = np.array(x, dtype=np.int64)
    for i in range(1, k):
        for j in range(i, k):
            t = pow(m[i - 1], -1, m[j])
            y[j] = np.mod((y[j] - y[i - 1]) * t, m[j])
    return y


def mrns_value(y, r) -> np.ndarray:
    """x = y_1 + sum_{i >= 2} y_i prod_{j < i} r_j."""
    acc = np.zeros(np.asarray(y).shape[1:], dtype=np.int64)
    w = 1
    for i, q in enumerate(r):
        acc = acc + np.asarray(y[i], dtype=np.int64) * w
        w *= int(q)
    return acc


def sign_rns_clear(x, m, n: int, z: int, p: int) -> np.ndarray:
    """Sign_(n,z,p)^RNS on residues (k, ...): n for negative values (upper half of Z_M), z for zero, p for positive ones."""
    m = [int(q) for q in m]
    if m[-1] % 2:
        raise ValueError("the most significant modulus must be even")
    y = rns2mrns_clear(x, m)
    neg = y[-1] >= m[-1] // 2
    digit_sum = y.sum(axis=0)
    return np.where(neg, n, np.where(digit_sum == 0, z, p)).astype(np.int64)


def rns2mrns_tables(p, m):
    """Lookup tables of the conversion, one per pair i < j in the order (0,1), (0,2), .., (1,2), ..: v -> (v - 16) t_ij mod m_j."""
    t = 1 << p.msg_bits
    if t < 256:
        raise ValueError("the RNS gadgets need an 8-bit message space")
    v = np.arange(t, dtype=np.int64)
    m = [int(q) for q in m]
    tabs = []
    for i in range(len(m) - 1):
        for j in range(i + 1, len(m)):
            tabs.append(np.mod((v - OFFSET) * pow(m[i], -1, m[j]), m[j]))
    return np.stack(tabs).astype(np.uint64)


def pair_index(k: int, i: int, j: int) -> int:
    """Position of the pair i < j in rns2mrns_tables."""
    return i * k - i * (i + 1) // 2 + (j - i - 1)


def sign_tables(p, m, n: int, z: int, pos: int):
    """The two extra tables of the sign gadget: top digit -> [digit >= r_k / 2], and sum + 128 [negative] -> n / z / p (signed
    results encoded in Z_t with negatives in the upper half)."""
    t = 1 << p.msg_bits
    v = np.arange(t, dtype=np.int64)
    top = (v >= int(m[-1]) // 2).astype(np.int64)
    top[int(m[-1]):] = 0                                            # not reachable: a digit is below its radix
    sel = np.where(v == 0, z, np.where(v < 128, pos, n))
    return np.stack([top, signed_encode(sel, t)]).astype(np.uint64)


def _add_const(p, cts, c: int) -> np.ndarray:
    """Adds the clear constant c to every ciphertext (c Delta on the body)."""
    out = np.array(cts, dtype=np.uint64)
    with np.errstate(over="ignore"):
        out[..., -1] += np.uint64((c << (63 - p.msg_bits)) & 0xFFFFFFFFFFFFFFFF)
    return out


def rns2mrns_encrypted(p, x_cts, m, bsk, ksk) -> np.ndarray:
    """Algorithm "RNS2MRNS" on ciphertexts.  x_cts: k x count x (n+1) encryptions of residues.  Returns the digits, same shape."""
    m = [int(q) for q in m]
    k = len(m)
    tabs = rns2mrns_tables(p, m)
    y = np.array(x_cts, dtype=np.uint64)
    count = y.shape[1]
    for i in range(1, k):
        with np.errstate(over="ignore"):
            diff = _add_const(p, y[i:] - y[i - 1][None], OFFSET)                       # (k - i) x count x (n+1)
        idx = np.repeat(np.array([pair_index(k, i - 1, j) for j in range(i, k)], dtype=np.uint32), count).reshape(k - i, count)
        y[i:] = _lookup(p, diff, tabs, idx, bsk, ksk)
    return y


def sign_rns_encrypted(p, x_cts, m, n: int, z: int, pos: int, bsk, ksk) -> np.ndarray:
    """Sign_(n,z,p)^RNS on ciphertexts: k x count x (n+1) -> count x (n+1)."""
    y = rns2mrns_encrypted(p, x_cts, m, bsk, ksk)
    st = sign_tables(p, m, n, z, pos)
    count = y.shape[1]
    neg = _lookup(p, y[-1], st[:1], np.zeros(count, dtype=np.uint32), bsk, ksk)
    with np.errstate(over="ignore"):
        packed = y.sum(axis=0, dtype=np.uint64) + neg * np.uint64(128)
    return _lookup(p, packed, st[1:], np.zeros(count, dtype=np.uint32), bsk, ksk)


# ---------------------------------------------------------------------------------------------------------------------
# Shift2MSBs^+ and Shift2MSBs^+- (Algorithms "Shift2MSBs^+" and "Shift2MSBs^+-"): approximate block scaling of an RNS tensor
# to its gamma most significant bits, viewing the mixed-radix digits as w-bit chunks of a binary number.
#
# Readings of points the paper leaves open:
#   R6  Step 2's lookup ceil(log2(x + 1)) + i w is the 1-indexed position of the digit's highest set bit; a zero digit has no
#       set bit and contributes 0 (the step's title; the formula as printed would give i w and force a shift for every
#       input with two or more moduli).  The paper's worked example does not separate the two readings: PARITY UNPINNED
#       for this choice (a test shows an input on which they differ).
#   R7  The maximum over the tensor is a binary tree of pairwise maxima, max(a, b) = b + ReLU(a - b), one lookup per pair on
#       a - b + 32 (positions are at most 6 * 4 = 24); level by level, element 2j with element 2j + 1, an odd last element
#       passing through.  The paper uses Concrete's max as a black box.
#   R8  Steps 3 and 4: per digit position one lookup turns maxBit into a shift code (lshift for digitShift >= 0, else
#       8 + min(rshift, w): a right shift of w or more clears a w-bit digit), and one two-input lookup per digit on
#       16 code + digit applies it.
#   R9  Shift2MSBs^+-: the sign is taken as the flag [x < 0] (Sign_(1,0,0)); s X mod m is a two-input lookup on
#       16 flag + residue, and s Y^+ one on 128 flag + Y^+ (Y^+ < 2^(Gamma-1) <= 128), its result signed in Z_t.
MAX_OFFSET = 32


def bit_position(x) -> np.ndarray:
    """1-indexed position of the highest set bit, 0 for 0 (= ceil(log2(x + 1)))."""
    x = np.asarray(x, dtype=np.int64)
    out = np.zeros_like(x)
    for b in range(1, 40):
        out = np.where(x >= (1 << (b - 1)), b, out)
    return out


def shift_code(max_bit, i: int, w: int, gamma: int) -> np.ndarray:
    """Step 3 for digit position i as one number: lshift if digitShift >= 0, else 8 + min(rshift, w)."""
    max_bit = np.asarray(max_bit, dtype=np.int64)
    any_shift = (max_bit > w).astype(np.int64)
    digit_shift = (gamma - (max_bit - w * i)) * any_shift
    lshift = np.minimum(np.maximum(digit_shift, 0), gamma - 1)
    rshift = np.maximum(-digit_shift, 0)
    return np.where(digit_shift >= 0, lshift, 8 + np.minimum(rshift, w))


def apply_shift_code(code, x) -> np.ndarray:
    code = np.asarray(code, dtype=np.int64)
    x = np.asarray(x, dtype=np.int64)
    return np.where(code < 8, x << np.minimum(code, 7), x >> np.maximum(code - 8, 0))


def shift2msbs_plus_digits_clear(Xd, w: int, gamma: int):
    """What "Shift2MSBs^+" computes from the mixed-radix digits Xd (k, ...), digit i read as bits [i w, (i + 1) w) of a
    binary number.  maxBit is the highest set bit (1-indexed) over the whole tensor under that reading, 0 for an all-zero
    tensor (R6: a zero digit has no set bit).  If maxBit <= w nothing moves; otherwise digit i is multiplied by
    2^(gamma - maxBit + i w), i.e. bit maxBit lands on bit gamma: a left shift (capped at gamma - 1) for a non-negative
    exponent, a truncating right shift otherwise.  Y is the sum of the moved digits and shift = maxBit - gamma.
    Returns Y, shift and (maxBit, left shifts, right shifts) per digit position."""
    Xd = np.asarray(Xd, dtype=np.int64)
    k = Xd.shape[0]
    weight = (w * np.arange(k, dtype=np.int64)).reshape((k,) + (1,) * (Xd.ndim - 1))
    top = np.where(Xd > 0, bit_position(Xd) + weight, 0)
    max_bit = int(top.max()) if top.size else 0
    exponent = (gamma - max_bit + w * np.arange(k, dtype=np.int64)) if max_bit > w else np.zeros(k, dtype=np.int64)
    lshift = np.clip(exponent, 0, gamma - 1)
    rshift = np.clip(-exponent, 0, None)
    moved = [(Xd[i] << int(lshift[i])) >> int(rshift[i]) for i in range(k)]
    return np.sum(moved, axis=0), max_bit - gamma, (max_bit, lshift, rshift)


def shift2msbs_plus_clear(X, m, w: int, gamma: int):
    """"Shift2MSBs^+" on residues X (k, ...) of non-negative numbers."""
    Y, shift, _ = shift2msbs_plus_digits_clear(rns2mrns_clear(X, m), w, gamma)
    return Y, shift


def shift2msbs_pm_clear(X, m, w: int, Gamma: int):
    """"Shift2MSBs^+-" on residues X (k, ...) of signed numbers (negatives in the upper half of Z_M)."""
    m = [int(q) for q in m]
    s = sign_rns_clear(X, m, -1, 1, 1)
    Xp = np.stack([np.mod(s * np.asarray(X[i], dtype=np.int64), q) for i, q in enumerate(m)])
    Yp, shift = shift2msbs_plus_clear(Xp, m, w, Gamma - 1)
    return s * Yp, shift


def shift_tables(p, m, w: int, gamma: int):
    """Tables of Shift2MSBs^+ over Z_t: [0, k) digit -> bit position + i w (R6); [k] a - b + 32 -> ReLU(a - b) (R7);
    [k+1, 2k+1) maxBit -> shift code of digit i (R8); [2k+1] 16 code + digit -> shifted digit (R8)."""
    t = 1 << p.msg_bits
    if t < 256:
        raise ValueError("the RNS gadgets need an 8-bit message space")
    k = len(m)
    v = np.arange(t, dtype=np.int64)
    pos = [np.where((v > 0) & (v < 16), bit_position(v) + i * w, 0) for i in range(k)]
    relu = [np.maximum(v - MAX_OFFSET, 0) * (v < 2 * MAX_OFFSET)]
    code = [np.where(v <= k * w, shift_code(v, i, w, gamma), 0) for i in range(k)]
    app = [np.where(v < 256, apply_shift_code(v >> 4, v & 15) % t, 0)]
    return np.stack(pos + relu + code + app).astype(np.uint64)


def pm_tables(p, m):
    """Extra tables of Shift2MSBs^+-: [0, k) 16 flag + residue -> |x| mod m_i; [k] 128 flag + y -> s y, signed in Z_t (R9)."""
    t = 1 << p.msg_bits
    v = np.arange(t, dtype=np.int64)
    ab = [np.where(v < 16, v % int(q), np.where(v < 32, (-(v - 16)) % int(q), 0)) for q in m]
    sg = [np.where(v < 128, v, signed_encode(-(v - 128), t))]
    return np.stack(ab + sg).astype(np.uint64)


def _max_tree(p, vals, relu_table, bsk, ksk) -> np.ndarray:
    """Maximum of the ciphertexts vals (n, n+1 words) by levels of pairwise maxima (R7).  Returns one ciphertext."""
    cur = np.array(vals, dtype=np.uint64)
    while cur.shape[0] > 1:
        h = cur.shape[0] // 2
        a, b = cur[0:2 * h:2], cur[1:2 * h:2]
        with np.errstate(over="ignore"):
            d = _lookup(p, _add_const(p, a - b, MAX_OFFSET), relu_table, np.zeros(h, dtype=np.uint32), bsk, ksk)
            nxt = b + d
        cur = np.concatenate([nxt, cur[2 * h:]]) if cur.shape[0] % 2 else nxt
    return cur[0]


def shift2msbs_plus_encrypted(p, x_cts, m, w: int, gamma: int, bsk, ksk):
    """"Shift2MSBs^+" on ciphertexts: residues k x count x (n+1) -> (Y: count x (n+1), shift: (n+1,), signed in Z_t)."""
    m = [int(q) for q in m]
    k = len(m)
    st = shift_tables(p, m, w, gamma)
    y = rns2mrns_encrypted(p, x_cts, m, bsk, ksk)                                   # Step 1
    count = y.shape[1]
    idx = np.repeat(np.arange(k, dtype=np.uint32), count).reshape(k, count)
    u = _lookup(p, y, st[:k], idx, bsk, ksk)                                        # Step 2
    max_bit = _max_tree(p, u.reshape(k * count, p.n + 1), st[k:k + 1], bsk, ksk)
    codes = _lookup(p, np.broadcast_to(max_bit, (k, p.n + 1)), st[k + 1:2 * k + 1], np.arange(k, dtype=np.uint32), bsk, ksk)   # Step 3
    with np.errstate(over="ignore"):
        packed = codes[:, None, :] * np.uint64(16) + y                              # Step 4
        ys = _lookup(p, packed, st[2 * k + 1:], np.zeros((k, count), dtype=np.uint32), bsk, ksk)
        Y = ys.sum(axis=0, dtype=np.uint64)                                         # Step 5
    shift = _add_const(p, max_bit, -gamma)                                          # Step 6
    return Y, shift


def shift2msbs_pm_encrypted(p, x_cts, m, w: int, Gamma: int, bsk, ksk):
    """"Shift2MSBs^+-" on ciphertexts: residues k x count x (n+1) of signed numbers -> (Y signed in Z_t, shift)."""
    m = [int(q) for q in m]
    k = len(m)
    count = x_cts.shape[1]
    flag = sign_rns_encrypted(p, x_cts, m, 1, 0, 0, bsk, ksk)                       # [x < 0]
    pt = pm_tables(p, m)
    idx = np.repeat(np.arange(k, dtype=np.uint32), count).reshape(k, count)
    with np.errstate(over="ignore"):
        xp = _lookup(p, flag[None] * np.uint64(16) + x_cts, pt[:k], idx, bsk, ksk)  # |x| in RNS
    Yp, shift = shift2msbs_plus_encrypted(p, xp, m, w, Gamma - 1, bsk, ksk)
    with np.errstate(over="ignore"):
        Y = _lookup(p, flag * np.uint64(128) + Yp, pt[k:], np.zeros(count, dtype=np.uint32), bsk, ksk)
    return Y, shift


# ---------------------------------------------------------------------------------------------------------------------
# MatmulHighRes^RNS (Algorithm "MatmulHighRes^RNS", appendix "Low-bitwidth high-resolution MatMul"): the product modulo a base
# of 5-bit moduli, every intermediate still within 8 bits.
#
# Readings of points the paper leaves open:
#   R15 extractBits(X', [3, 4]) is (X' >> 3) & 3 and extractBits(X', [0, 2]) is X' & 7, one lookup each on the residue (the
#       paper uses the bit extraction as a black box).  The two expandDims lines of step 3 are read as acting on X_1' and X_2'.
#   R16 Y_1* = X_1' W' mod m'' is one two-input lookup on 32 x_1 + w (3 + 5 bits); Y_2* = X_2' W' is one two-input lookup on
#       32 x_2 + w returning the plain product (at most 3 * 31 = 93), followed by the custom lookup v -> 8 v mod m_i the paper
#       names; step 4 reduces Y_1* + Y_2* (at most 2 * 30) by one more lookup.
#   R17 Step 5 as R3: the slices summed are those of Y*, and Y + Y' <= 30 + 7 * 30 = 240 is reduced by one lookup.
RNS_BASES_5BIT = {2: (31, 30), 3: (29, 31, 30), 4: (27, 29, 31, 28), 5: (25, 27, 29, 31, 28), 6: (23, 25, 27, 29, 31, 28)}
BLOCK_HIGHRES = 7


def matmul_highres_clear(X, W, m) -> np.ndarray:
    """Algorithm "MatmulHighRes^RNS" on clear integers.  X: a x b, W: b x c (signed), m: k moduli below 32.  Returns k x a x c."""
    X = np.asarray(X, dtype=np.int64)
    W = np.asarray(W, dtype=np.int64)
    m = np.asarray(m, dtype=np.int64)
    b = X.shape[1]
    mp, mpp = m[:, None, None], m[:, None, None, None]
    # Step 1: inputs to RNS representation
    Xr = np.mod(X[None], mp)
    Wr = np.mod(W[None], mp)
    # Step 2: bit chunks of X'
    X2 = (Xr >> 3) & 3
    X1 = Xr & 7
    # Step 3: partial products
    Y1 = np.mod(X1[:, :, :, None] * Wr[:, None, :, :], mpp)
    Y2 = X2[:, :, :, None] * Wr[:, None, :, :]
    assert int(Y2.max()) < 128
    Y2 = np.mod(Y2 * 8, mpp)
    # Step 4: add the partial products
    Ys = np.mod(Y1 + Y2, mpp)
    # Step 5: block-wise summation
    n = min(BLOCK_HIGHRES, b)
    Y = np.mod(Ys[:, :, :n, :].sum(axis=2), mp)
    i = n
    while i < b:
        j = min(i + n, b)
        Yp = Ys[:, :, i:j, :].sum(axis=2)
        assert int((Y + Yp).max()) < 256
        Y = np.mod(Y + Yp, mp)
        i += n
    return Y


def highres_tables(p, m) -> np.ndarray:
    """The 4k + 3 lookup tables over Z_t (t >= 256): k of v -> signed(v) mod m_i, k of u -> (u >> 5)(u & 31) mod m_i, k of
    v -> 8 v mod m_i, k of v -> v mod m_i, then v -> (v >> 3) & 3, v -> v & 7 and u -> (u >> 5)(u & 31)."""
    t = 1 << p.msg_bits
    if t < 256:
        raise ValueError("MatmulHighRes^RNS needs an 8-bit message space")
    v = np.arange(t, dtype=np.int64)
    inside = v < 256
    prod = np.where(inside, (v >> 5) * (v & 31), 0)
    tabs = [np.mod(signed_decode(v, t), q) for q in m]
    tabs += [np.where(inside, np.mod(prod, q), 0) for q in m]
    tabs += [np.mod(8 * v, q) for q in m]
    tabs += [np.mod(v, q) for q in m]
    tabs += [(v >> 3) & 3, v & 7, prod]
    return np.stack(tabs).astype(np.uint64)


def matmul_highres_encrypted(p, x_cts, w_cts, m, bsk, ksk) -> np.ndarray:
    """Algorithm "MatmulHighRes^RNS" on ciphertexts.  x_cts: a x b x (n+1), w_cts: b x c x (n+1), encryptions of signed 8-bit values
    (R1).  Returns k x a x c x (n+1) encryptions of the residues of X W."""
    m = [int(q) for q in m]
    k = len(m)
    a, b = x_cts.shape[:2]
    c = w_cts.shape[1]
    tabs = highres_tables(p, m)
    kk = np.arange(k, dtype=np.uint32)
    one = lambda shape, i: np.full(shape, i, dtype=np.uint32)
    # Step 1
    Xr = _lookup(p, np.broadcast_to(x_cts[None], (k, a, b, p.n + 1)), tabs, np.broadcast_to(kk[:, None, None], (k, a, b)), bsk, ksk)
    Wr = _lookup(p, np.broadcast_to(w_cts[None], (k, b, c, p.n + 1)), tabs, np.broadcast_to(kk[:, None, None], (k, b, c)), bsk, ksk)
    # Step 2 (R15)
    X2 = _lookup(p, Xr, tabs, one((k, a, b), 4 * k), bsk, ksk)
    X1 = _lookup(p, Xr, tabs, one((k, a, b), 4 * k + 1), bsk, ksk)
    # Step 3 (R16)
    per_mod = np.broadcast_to(kk[:, None, None, None], (k, a, b, c))
    with np.errstate(over="ignore"):
        Y1 = _lookup(p, X1[:, :, :, None, :] * np.uint64(32) + Wr[:, None, :, :, :], tabs, k + per_mod, bsk, ksk)
        Y2 = _lookup(p, X2[:, :, :, None, :] * np.uint64(32) + Wr[:, None, :, :, :], tabs, one((k, a, b, c), 4 * k + 2), bsk, ksk)
    Y2 = _lookup(p, Y2, tabs, 2 * k + per_mod, bsk, ksk)
    # Step 4
    with np.errstate(over="ignore"):
        Ys = _lookup(p, Y1 + Y2, tabs, 3 * k + per_mod, bsk, ksk)
    # Step 5 (R17)
    idx = 3 * k + np.broadcast_to(kk[:, None, None], (k, a, c))
    n = min(BLOCK_HIGHRES, b)
    with np.errstate(over="ignore"):
        Y = _lookup(p, Ys[:, :, :n, :, :].sum(axis=2, dtype=np.uint64), tabs, idx, bsk, ksk)
        i = n
        while i < b:
            j = min(i + n, b)
            Y = _lookup(p, Y + Ys[:, :, i:j, :, :].sum(axis=2, dtype=np.uint64), tabs, idx, bsk, ksk)
            i += n
    return Y
