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
