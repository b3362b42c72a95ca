"""Pins of the Matmul^RNS oracle (oracle/gadgets.py): the paper's printed table and example, the plain definition
(integer matrix product reduced modulo each modulus), brute force in Python integers, and decryption of the encrypted
pipeline.  CPU only."""
import math
import os

import numpy as np
import pytest

import synth
from synth import Params

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def gd(orc):
    from oracle import gadgets
    return gadgets


def _rows(name):
    return [l.strip() for l in open(os.path.join(GOLDEN, name)) if l.strip() and not l.startswith("#")]


def test_rns_bases_match_the_printed_table(gd):
    rows = _rows("rns_bases.txt")
    assert len(rows) == len(gd.RNS_BASES) == 5
    for row in rows:
        k, base, bits = [f.strip() for f in row.split("|")]
        base = tuple(int(x) for x in base.split())
        assert gd.RNS_BASES[int(k)] == base and len(base) == int(k)
        # the printed bitwidth is log2 of the product of the moduli (printed to two decimals, truncated or rounded)
        assert abs(gd.rns_base_bitwidth(base) - float(bits)) < 0.011
        # what the gadgets rely on: 4-bit moduli, pairwise coprime, the most significant (last) one even
        assert all(2 <= q <= 16 for q in base)
        assert all(math.gcd(p, q) == 1 for i, p in enumerate(base) for q in base[i + 1:])
        assert base[-1] % 2 == 0


def test_get_rns_base_picks_the_smallest_sufficient_base(gd):
    assert gd.get_rns_base(7.0) == (15, 14)
    assert gd.get_rns_base(7.72) == (13, 15, 14)          # log2(210) = 7.714 < 7.72
    assert gd.get_rns_base(11.0) == (13, 15, 14)
    assert gd.get_rns_base(14.5) == (11, 13, 15, 14)
    assert gd.get_rns_base(16.0) == (7, 11, 13, 15, 8)
    assert gd.get_rns_base(18.0) == (5, 7, 9, 11, 13, 8)
    with pytest.raises(ValueError):
        gd.get_rns_base(19.0)


def test_signed_encoding_matches_the_printed_example(gd):
    signed, enc = [[int(x) for x in r.split()] for r in _rows("signed_encoding.txt")]
    assert gd.signed_encode(signed, 5).tolist() == enc
    assert gd.signed_decode(enc, 5).tolist() == signed
    v = np.arange(256)
    assert np.array_equal(gd.signed_decode(v, 256), v.astype(np.uint8).view(np.int8).astype(np.int64))   # two's complement
    for M in (5, 14, 210, 2730):
        u = np.arange(M)
        assert np.array_equal(gd.signed_encode(gd.signed_decode(u, M), M), u)
        d = gd.signed_decode(u, M)
        assert d.max() == (M - 1) // 2 and d.min() == -(M // 2)


def _rand_int8(seed, stream, shape, lo=-128, hi=127):
    n = int(np.prod(shape))
    return (synth.uniform_below(seed, stream, n, hi - lo + 1).astype(np.int64) + lo).reshape(shape)


@pytest.mark.parametrize("a,b,c,k", [(1, 1, 1, 2), (3, 14, 2, 3), (2, 15, 3, 2), (2, 16, 2, 4), (4, 31, 5, 5), (2, 45, 3, 6), (1, 784, 2, 5)])
def test_clear_clone_is_the_integer_product_modulo_each_modulus(gd, a, b, c, k):
    m = gd.RNS_BASES[k]
    X = _rand_int8(7, "lin_inputs", (a, b))
    W = _rand_int8(7, "weights", (b, c))
    Y = gd.matmul_rns_clear(X, W, m)
    Z = X @ W
    assert Y.shape == (k, a, c)
    for i, q in enumerate(m):
        assert np.array_equal(Y[i], np.mod(Z, q))
    # values the base can hold come back exactly through the Chinese remainder theorem
    M = math.prod(m)
    small = np.abs(Z) <= (M - 1) // 2 - 1
    assert np.array_equal(gd.crt_reconstruct(Y, m)[small], Z[small])


def test_clear_clone_against_brute_force_python_integers(gd):
    m = (7, 11, 13)
    X = [[-128, 127, 5], [0, -1, 100]]
    W = [[127, -128], [3, 0], [-77, 9]]
    Y = gd.matmul_rns_clear(X, W, m)
    for i, q in enumerate(m):
        for r in range(2):
            for s in range(2):
                tot = 0
                for j in range(3):
                    tot += ((X[r][j] % q) * (W[j][s] % q)) % q       # Python's % is the mathematical residue
                assert int(Y[i, r, s]) == tot % q


def test_extreme_inputs_keep_every_intermediate_within_eight_bits(gd):
    # all residues at their maximum: the clone's own assertion checks Y + Y' < 256 in every block
    for k in (2, 6):
        m = gd.RNS_BASES[k]
        X = np.full((2, 61), -1)       # -1 = m_i - 1 modulo every modulus
        W = np.full((61, 2), -1)
        Y = gd.matmul_rns_clear(X, W, m)
        assert np.array_equal(Y[:, 0, 0], np.mod(61, m))


def test_lookup_tables(gd):
    p = Params(name="t", n=4, k=1, N=2048, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8, msg_bits=8,
               sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1, seed=99)
    m = (7, 11, 13, 15, 8)
    red_s, prod, red = gd.lookup_tables(p, m)
    assert red_s.shape == prod.shape == red.shape == (5, 256)
    for i, q in enumerate(m):
        for x in range(16):
            for w in range(16):
                assert int(prod[i, 16 * x + w]) == (x * w) % q
        assert int(red_s[i, 255]) == (-1) % q and int(red_s[i, 128]) == (-128) % q and int(red_s[i, 127]) == 127 % q
        assert [int(v) for v in red[i, :2 * q]] == [v % q for v in range(2 * q)]
    with pytest.raises(ValueError):
        gd.lookup_tables(p.with_(msg_bits=4), m)


def test_encrypted_pipeline_decrypts_to_the_clear_clone(orc, gd):
    # insecure toy parameters (4 key bits) with an 8-bit message space: one lookup is 7e7 multiply-adds in the oracle
    p = Params(name="gadget_toy", n=4, k=1, N=2048, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8, msg_bits=8,
               sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1, seed=0x6AD6E7)
    keys = orc.Keys(p, synth)
    m = (13, 15, 14)
    a, b, c = 2, 17, 1                                      # two blocks in step 3: 15 + 2
    X = _rand_int8(p.seed, "lin_inputs", (a, b))
    W = _rand_int8(p.seed, "weights", (b, c))
    X[0, 0], W[0, 0], X[1, 1], W[1, 0] = -128, -128, 127, -1
    x_cts = orc.encrypt_messages(p, synth, keys.lwe_sk, gd.signed_encode(X, 256).reshape(-1).astype(np.uint64)).reshape(a, b, p.n + 1)
    w_cts = orc.encrypt_messages(p, synth, keys.lwe_sk, gd.signed_encode(W, 256).reshape(-1).astype(np.uint64), offset=a * b).reshape(b, c, p.n + 1)
    Y = gd.matmul_rns_encrypted(p, x_cts, w_cts, m, keys.bsk, keys.ksk)
    got, err = orc.decode(orc.lwe_phase(keys.lwe_sk, Y.reshape(-1, p.n + 1)), p.msg_bits)
    want = gd.matmul_rns_clear(X, W, m)
    assert np.array_equal(got.reshape(want.shape).astype(np.int64), want)
    assert np.array_equal(gd.crt_reconstruct(want, m), gd.signed_decode(np.mod(X @ W, 13 * 15 * 14), 13 * 15 * 14))
    assert float(np.abs(err).max()) < 2.0 ** -12           # far from the 2^-10 decision boundary


# ---- RNS-to-MRNS conversion and sign determination -------------------------------------------------------------------
def test_rns2mrns_reproduces_the_printed_example(gd):
    rows = {r.split("|")[0].strip(): [int(v) for v in r.split("|")[1].split()] for r in _rows("rns_to_mrns_example.txt")}
    m = rows["moduli"]
    x = rows["value"][0]
    assert [x % q for q in m] == rows["rns"]
    y = gd.rns2mrns_clear(np.array(rows["rns"]).reshape(3, 1), m)
    assert y[:, 0].tolist() == rows["mrns"]
    assert int(gd.mrns_value(y, m)[0]) == x == rows["mrns"][0] + rows["mrns"][1] * 5 + rows["mrns"][2] * 35
    # the printed intermediate rows: subtract the finished digit, multiply by the inverse of its modulus
    r = rows["rns"]
    s1 = [r[0], (r[1] - r[0]) % 7, (r[2] - r[0]) % 8]
    assert s1 == rows["after_subtract_1"]
    m1 = [s1[0], s1[1] * pow(5, -1, 7) % 7, s1[2] * pow(5, -1, 8) % 8]
    assert m1 == rows["after_multiply_1"]
    s2 = [m1[0], m1[1], (m1[2] - m1[1]) % 8]
    assert s2 == rows["after_subtract_2"]
    assert [s2[0], s2[1], s2[2] * pow(7, -1, 8) % 8] == rows["after_multiply_2"]


def test_rns2mrns_and_sign_exhaustively_over_every_base_of_the_table(gd):
    for k, m in gd.RNS_BASES.items():
        M = math.prod(m)
        x = np.arange(M, dtype=np.int64)
        res = gd.rns_encode(x, m)
        y = gd.rns2mrns_clear(res, m)
        assert all(int(y[i].max()) < m[i] and int(y[i].min()) >= 0 for i in range(k))
        assert np.array_equal(gd.mrns_value(y, m), x)                       # the digits are the number
        s = gd.sign_rns_clear(res, m, -1, 0, 1)
        assert np.array_equal(s, np.sign(gd.signed_decode(x, M)))           # true sign of the signed value
        assert np.array_equal(gd.sign_rns_clear(res, m, -1, 1, 1), np.where(gd.signed_decode(x, M) < 0, -1, 1))


def test_sign_needs_an_even_top_modulus(gd):
    with pytest.raises(ValueError):
        gd.sign_rns_clear(np.zeros((2, 1), dtype=np.int64), (14, 15), -1, 0, 1)


def test_rns_gadget_tables(gd):
    p = Params(name="t", n=4, k=1, N=2048, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8, msg_bits=8,
               sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1, seed=99)
    m = (7, 11, 13, 15, 8)
    tabs = gd.rns2mrns_tables(p, m)
    assert tabs.shape == (10, 256)
    for i in range(4):
        for j in range(i + 1, 5):
            row = tabs[gd.pair_index(5, i, j)]
            for a in range(m[j]):
                for b in range(m[i]):
                    assert int(row[a - b + gd.OFFSET]) == ((a - b) * pow(m[i], -1, m[j])) % m[j]
    st = gd.sign_tables(p, m, -1, 0, 1)
    assert st[0, :8].tolist() == [0, 0, 0, 0, 1, 1, 1, 1]
    assert int(st[1, 0]) == 0 and int(st[1, 1]) == 1 and int(st[1, 127]) == 1 and int(st[1, 128]) == 255 and int(st[1, 218]) == 255


def test_encrypted_rns2mrns_and_sign_decrypt_to_the_clear_clone(orc, gd):
    p = Params(name="gadget_toy", n=4, k=1, N=2048, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8, msg_bits=8,
               sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1, seed=0x6AD6E7)
    keys = orc.Keys(p, synth)
    m = (13, 15, 14)
    M = math.prod(m)
    vals = np.array([0, 1, -1, 99, -99, M // 2 - 1, -(M // 2), 7, -1364, 1363, 2, -2], dtype=np.int64)
    res = gd.rns_encode(vals, m)                                            # 3 x 12
    cts = orc.encrypt_messages(p, synth, keys.lwe_sk, res.reshape(-1).astype(np.uint64)).reshape(3, len(vals), p.n + 1)
    y = gd.rns2mrns_encrypted(p, cts, m, keys.bsk, keys.ksk)
    got, _ = orc.decode(orc.lwe_phase(keys.lwe_sk, y.reshape(-1, p.n + 1)), p.msg_bits)
    assert np.array_equal(got.reshape(3, -1).astype(np.int64), gd.rns2mrns_clear(res, m))
    s = gd.sign_rns_encrypted(p, cts, m, -1, 0, 1, keys.bsk, keys.ksk)
    got, _ = orc.decode(orc.lwe_phase(keys.lwe_sk, s), p.msg_bits)
    assert np.array_equal(gd.signed_decode(got.astype(np.int64), 256), np.sign(vals))


# ---- Shift2MSBs ---------------------------------------------------------------------------------------------------------
def test_shift2msbs_plus_reproduces_the_printed_example(gd):
    rows = {r.split("|")[0].strip(): [int(v) for v in r.split("|")[1].split()] for r in _rows("shift2msbs_example.txt")}
    Xd = np.array([rows["digits_0"], rows["digits_1"], rows["digits_2"]]).T.reshape(3, 1, 3)      # k x a x b
    Y, shift, (max_bit, lshift, rshift) = gd.shift2msbs_plus_digits_clear(Xd, rows["w"][0], rows["gamma"][0])
    assert max_bit == rows["max_bit"][0]
    assert lshift.tolist() == rows["lshift"] and rshift.tolist() == rows["rshift"]
    assert Y.reshape(-1).tolist() == rows["y"] and shift == rows["shift"][0]
    # the same through the single-number shift code the encrypted pipeline uses
    for i in range(3):
        code = gd.shift_code(max_bit, i, 4, 5)
        assert np.array_equal(gd.apply_shift_code(code, Xd[i]), (Xd[i] << lshift[i]) >> rshift[i])


def test_shift2msbs_zero_digit_reading_is_visible(gd):
    # The reading of step 2 for a zero digit (position 0, not i w as the printed formula ceil(log2(x + 1)) + i w would give)
    # is not settled by the printed worked example: there the top digit of one element is non-zero, so maxBit = 10 under
    # both readings.  On a tensor whose upper digits are all zero the two readings part: digits (5, 0, 0) with w = 4,
    # gamma = 5.  This reading: maxBit = 3 <= w, nothing moves, Y = 5, shift = -2.  The printed formula: the zero digits
    # would report positions 4 and 8, maxBit = 8, digit 0 moves right by 3, Y = 0, shift = 3 -- a small number wiped
    # out although "only shift down, never up" needs no shift at all.  The pin fixes the choice made here.
    Xd = np.array([[5], [0], [0]])
    Y, shift, (max_bit, lshift, rshift) = gd.shift2msbs_plus_digits_clear(Xd, 4, 5)
    assert (int(Y[0]), shift, max_bit) == (5, -2, 3)
    assert list(lshift) == [0, 0, 0] and list(rshift) == [0, 0, 0]
    # the printed formula, evaluated by hand for this input
    printed_positions = [math.ceil(math.log2(5 + 1)) + 0, math.ceil(math.log2(0 + 1)) + 4, math.ceil(math.log2(0 + 1)) + 8]
    printed_max = max(printed_positions)
    assert printed_positions == [3, 4, 8] and printed_max > 4
    assert (5 >> -(5 - (printed_max - 0)), printed_max - 5) == (0, 3)
    # same through the lookup tables the encrypted pipeline uses: a zero digit's table entry is 0 at every position
    p = Params(name="t", n=4, k=1, N=2048, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8, msg_bits=8,
               sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1, seed=99)
    tabs = gd.shift_tables(p, (13, 15, 14), 4, 5)
    assert [int(tabs[i][0]) for i in range(3)] == [0, 0, 0]
    assert [int(tabs[i][1]) for i in range(3)] == [1, 5, 9]


def test_shift2msbs_properties(gd):
    m, w = (13, 15, 14), 4
    M = math.prod(m)
    for gamma in (5, 7):
        x = synth.uniform_below(11 + gamma, "misc", 64, M // 2).astype(np.int64)
        Y, shift = gd.shift2msbs_plus_clear(gd.rns_encode(x, m), m, w, gamma)
        assert int(Y.max()) < (1 << gamma) and int(Y.min()) >= 0
        d = gd.rns2mrns_clear(gd.rns_encode(x, m), m)
        top = max(int(np.where(d[i] > 0, gd.bit_position(d[i]) + 4 * i, 0).max()) for i in range(3))
        assert shift == top - gamma
        # the largest element keeps its leading bit at position gamma
        assert int(Y.max()) >= (1 << (gamma - 1))
    # small inputs (highest bit within the first digit) are not shifted at all
    x = np.array([0, 1, 5, 12], dtype=np.int64)
    Y, shift = gd.shift2msbs_plus_clear(gd.rns_encode(x, m), m, w, 7)
    assert Y.tolist() == x.tolist() and shift == 4 - 7
    # signed variant: odd symmetry, and the sign of every non-zero output
    x = np.concatenate([synth.uniform_below(5, "misc", 40, M // 2).astype(np.int64), [0, 1, -1, M // 2 - 1, -(M // 2)]])
    Yp, s1 = gd.shift2msbs_pm_clear(gd.rns_encode(x, m), m, w, 8)
    Yn, s2 = gd.shift2msbs_pm_clear(gd.rns_encode(-x[:-1], m), m, w, 8)
    assert np.array_equal(Yp[:-1], -Yn) and int(np.abs(Yp).max()) < 128
    assert np.all(np.sign(Yp[Yp != 0]) == np.sign(x[Yp != 0]))


def test_shift_tables(gd):
    p = Params(name="t", n=4, k=1, N=2048, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8, msg_bits=8,
               sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1, seed=99)
    m, w, gamma = (13, 15, 14), 4, 5
    st = gd.shift_tables(p, m, w, gamma)
    assert st.shape == (2 * 3 + 2, 256)
    assert st[0, :16].tolist() == [0, 1, 2, 2, 3, 3, 3, 3, 4, 4, 4, 4, 4, 4, 4, 4]
    assert st[2, :16].tolist() == [0] + [v + 8 for v in [1, 2, 2, 3, 3, 3, 3, 4, 4, 4, 4, 4, 4, 4, 4]]
    for a in range(25):
        for b in range(25):
            assert int(st[3, a - b + gd.MAX_OFFSET]) == max(a - b, 0)
    # codes at the printed example's maxBit = 10: lshift 3 for the top digit, rshift 1 and 5 (clamped to 4) below
    assert [int(st[4 + i, 10]) for i in range(3)] == [8 + 4, 8 + 1, 3]
    assert int(st[7, 16 * 3 + 3]) == 24 and int(st[7, 16 * 9 + 12]) == 6 and int(st[7, 16 * 12 + 6]) == 0
    pt = gd.pm_tables(p, m)
    for i, q in enumerate(m):
        assert [int(pt[i, 16 + x]) for x in range(q)] == [(-x) % q for x in range(q)]
        assert [int(pt[i, x]) for x in range(q)] == list(range(q))
    assert int(pt[3, 5]) == 5 and int(pt[3, 128 + 5]) == 251 and int(pt[3, 128]) == 0


def test_encrypted_shift2msbs_decrypts_to_the_clear_clone(orc, gd):
    p = Params(name="gadget_toy", n=4, k=1, N=2048, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8, msg_bits=8,
               sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1, seed=0x6AD6E7)
    keys = orc.Keys(p, synth)
    m, w = (13, 15, 14), 4
    # the printed example's three inputs (from their digits) plus two more
    vals = np.array([0 + 2 * 13 + 3 * 195, 2 + 12 * 13 + 1 * 195, 6 + 1 * 13, 1000, 3], dtype=np.int64)
    res = gd.rns_encode(vals, m)
    cts = orc.encrypt_messages(p, synth, keys.lwe_sk, res.reshape(-1).astype(np.uint64), offset=777).reshape(3, len(vals), p.n + 1)
    Y, shift = gd.shift2msbs_plus_encrypted(p, cts, m, w, 5, keys.bsk, keys.ksk)
    got, _ = orc.decode(orc.lwe_phase(keys.lwe_sk, Y), p.msg_bits)
    want, want_shift = gd.shift2msbs_plus_clear(res, m, w, 5)
    assert np.array_equal(got.astype(np.int64), want)
    sh, _ = orc.decode(orc.lwe_phase(keys.lwe_sk, shift[None]), p.msg_bits)
    assert int(gd.signed_decode(sh.astype(np.int64), 256)[0]) == want_shift
    # signed variant
    svals = np.array([vals[0], -vals[1], vals[2], -1000, 0, -3], dtype=np.int64)
    sres = gd.rns_encode(svals, m)
    scts = orc.encrypt_messages(p, synth, keys.lwe_sk, sres.reshape(-1).astype(np.uint64), offset=999).reshape(3, len(svals), p.n + 1)
    Y, shift = gd.shift2msbs_pm_encrypted(p, scts, m, w, 6, keys.bsk, keys.ksk)
    got, _ = orc.decode(orc.lwe_phase(keys.lwe_sk, Y), p.msg_bits)
    want, want_shift = gd.shift2msbs_pm_clear(sres, m, w, 6)
    assert np.array_equal(gd.signed_decode(got.astype(np.int64), 256), want)
    sh, _ = orc.decode(orc.lwe_phase(keys.lwe_sk, shift[None]), p.msg_bits)
    assert int(gd.signed_decode(sh.astype(np.int64), 256)[0]) == want_shift


# ---- MatmulHighRes^RNS -------------------------------------------------------------------------------------------------
def test_5bit_rns_bases_match_the_printed_table(gd):
    rows = _rows("rns_bases_5bit.txt")
    assert len(rows) == len(gd.RNS_BASES_5BIT) == 5
    for row in rows:
        k, base, bits = [f.strip() for f in row.split("|")]
        base = tuple(int(x) for x in base.split())
        assert gd.RNS_BASES_5BIT[int(k)] == base and len(base) == int(k)
        assert abs(gd.rns_base_bitwidth(base) - float(bits)) < 0.011
        assert all(16 < q < 32 for q in base)
        assert all(math.gcd(p, q) == 1 for i, p in enumerate(base) for q in base[i + 1:])
        assert base[-1] % 2 == 0


@pytest.mark.parametrize("a,b,c,k", [(2, 3, 2, 2), (3, 7, 2, 3), (2, 8, 3, 4), (1, 40, 2, 6), (4, 15, 1, 5)])
def test_highres_clear_clone_is_the_integer_product_modulo_each_modulus(gd, a, b, c, k):
    m = gd.RNS_BASES_5BIT[k]
    X = _rand_int8(7 * a + b, "lin_inputs", (a, b))
    W = _rand_int8(7 * a + b, "weights", (b, c))
    Y = gd.matmul_highres_clear(X, W, m)
    assert Y.shape == (k, a, c)
    for i, q in enumerate(m):
        assert np.array_equal(Y[i], np.mod(X @ W, q))
    M = math.prod(m)
    assert np.array_equal(gd.crt_reconstruct(Y, m), gd.signed_decode(np.mod(X @ W, M), M))


def test_highres_against_brute_force_and_at_the_extremes(gd):
    m = (29, 31, 30)
    X = _rand_int8(3, "lin_inputs", (2, 9))
    W = _rand_int8(3, "weights", (9, 2))
    Y = gd.matmul_highres_clear(X, W, m)
    for i, q in enumerate(m):
        for r in range(2):
            for s in range(2):
                assert int(Y[i, r, s]) == sum(int(X[r, j]) * int(W[j, s]) for j in range(9)) % q
    # all-extreme inputs: the clone's own asserts check that no intermediate leaves 8 bits
    for xv, wv in ((-128, -128), (127, 127), (-1, -1), (127, -128)):
        X = np.full((1, 30), xv); W = np.full((30, 1), wv)
        for base in gd.RNS_BASES_5BIT.values():
            Y = gd.matmul_highres_clear(X, W, base)
            assert [int(v) for v in Y[:, 0, 0]] == [(30 * xv * wv) % q for q in base]


def test_highres_tables(gd):
    p = Params(name="gadget_toy", n=4, k=1, N=2048, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8, msg_bits=8,
               sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1, seed=99)
    m = (29, 31, 30)
    tabs = gd.highres_tables(p, m).astype(np.int64)
    assert tabs.shape == (15, 256)
    for i, q in enumerate(m):
        assert tabs[i, 255] == (-1) % q and tabs[i, 128] == (-128) % q and tabs[i, 127] == 127 % q
        for x in range(8):
            for w in range(32):
                assert tabs[3 + i, 32 * x + w] == (x * w) % q
        assert [int(v) for v in tabs[6 + i, :100]] == [(8 * v) % q for v in range(100)]
        assert [int(v) for v in tabs[9 + i]] == [v % q for v in range(256)]
    for v in range(32):
        assert tabs[12, v] == v >> 3 and tabs[13, v] == v % 8 and 8 * tabs[12, v] + tabs[13, v] == v
    for x in range(4):
        for w in range(32):
            assert tabs[14, 32 * x + w] == x * w


def test_encrypted_highres_decrypts_to_the_clear_clone(orc, gd):
    p = Params(name="gadget_toy", n=4, k=1, N=2048, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8, msg_bits=8,
               sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1, seed=0x6AD6E7)
    keys = orc.Keys(p, synth)
    m = (29, 31, 30)
    a, b, c = 2, 9, 1                                       # two blocks in step 5: 7 + 2
    X = _rand_int8(p.seed, "lin_inputs", (a, b))
    W = _rand_int8(p.seed, "weights", (b, c))
    X[0, 0], W[0, 0], X[1, 1], W[1, 0] = -128, -128, 127, -1
    x_cts = orc.encrypt_messages(p, synth, keys.lwe_sk, gd.signed_encode(X, 256).reshape(-1).astype(np.uint64)).reshape(a, b, p.n + 1)
    w_cts = orc.encrypt_messages(p, synth, keys.lwe_sk, gd.signed_encode(W, 256).reshape(-1).astype(np.uint64), offset=a * b).reshape(b, c, p.n + 1)
    Y = gd.matmul_highres_encrypted(p, x_cts, w_cts, m, keys.bsk, keys.ksk)
    got, err = orc.decode(orc.lwe_phase(keys.lwe_sk, Y.reshape(-1, p.n + 1)), p.msg_bits)
    want = gd.matmul_highres_clear(X, W, m)
    assert np.array_equal(got.reshape(want.shape).astype(np.int64), want)
    assert np.array_equal(want, np.mod((X @ W)[None], np.array(m)[:, None, None]))
    assert float(np.abs(err).max()) < 2.0 ** -12
