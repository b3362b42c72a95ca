"""Pins for the CPU oracle (no GPU): the oracle is checked against what the scheme and the mathematics fix.

The paper treats the bootstrapping as a black box (Sec. "TFHE & Concrete"), so there are no printed
ciphertext values; the pins are the invariants of the CGGI scheme: ring identities, the decomposition
identity, decrypt(PBS(Enc(m))) = f(m) for every message, the negacyclic law, linearity, special cases
with zero keys / zero noise, closed-form noise variances, and bit-for-bit agreement with a second
definition in Python integers on tiny parameters.
"""
import math

import numpy as np
import pytest

import synth
from synth import Params
from tests import bigint_ref as ref

MASK = (1 << 64) - 1


def tiny(**kw):
    base = dict(name="tiny", n=8, k=1, N=32, pbs_base_log=8, pbs_level=2, ks_base_log=4, ks_level=3,
                msg_bits=2, sigma_lwe=2.0 ** -24, sigma_bsk=2.0 ** -44, batch=8, n_luts=1, seed=77)
    base.update(kw)
    return Params(**base)


def rng_words(seed, count):
    return synth.words(seed, "misc", count)


# ---------------------------------------------------------------- ring product

@pytest.mark.parametrize("N", [2, 4, 8, 16, 64])
def test_schoolbook_equals_matrix_definition(orc, N):
    P = rng_words(N, N)
    Qp = rng_words(N + 1000, N)
    want = ref.polymul([int(v) for v in P], [int(v) for v in Qp])
    got = orc.negacyclic_mul(P, Qp)
    assert [int(v) for v in got] == want


@pytest.mark.parametrize("N", [128, 512, 2048])
def test_schoolbook_equals_linear_convolution_folded(orc, N):
    # independent route: full linear convolution in exact integers, then fold with X^N = -1
    P = rng_words(3 * N, N)
    d = synth.uniform_below(N, "misc", N, 1 << 23, offset=7).astype(np.int64) - (1 << 22)   # signed digits
    full = np.convolve(np.array([int(v) for v in P], dtype=object), np.array([int(v) for v in d], dtype=object))
    want = [(int(full[c]) - (int(full[c + N]) if c + N < len(full) else 0)) % (1 << 64) for c in range(N)]
    got = orc.negacyclic_mul(d.astype(np.uint64), P)
    assert [int(v) for v in got] == want
    assert np.array_equal(got, orc.negacyclic_mul(P, d.astype(np.uint64)))       # commutative


def test_x_to_the_n_is_minus_one_and_monomials(orc):
    N = 64
    P = rng_words(5, N)
    assert np.array_equal(orc.monomial_mul(P, N), (~P + np.uint64(1)))           # X^N P = -P
    assert np.array_equal(orc.monomial_mul(P, 0), P)
    for r in [1, 5, N - 1, N, N + 3, 2 * N - 1]:
        mono = np.zeros(N, dtype=np.uint64)
        if r < N:
            mono[r] = 1
        else:
            mono[r - N] = MASK                                                   # -1
        assert np.array_equal(orc.monomial_mul(P, r), orc.negacyclic_mul(mono, P)), r
    # X^a X^b = X^(a+b mod 2N)
    assert np.array_equal(orc.monomial_mul(orc.monomial_mul(P, 37), 100), orc.monomial_mul(P, 137 % (2 * N)))


def test_ring_product_is_bilinear(orc):
    N = 32
    A, B, C = rng_words(1, N), rng_words(2, N), rng_words(3, N)
    with np.errstate(over="ignore"):
        assert np.array_equal(orc.negacyclic_mul(A + B, C), orc.negacyclic_mul(A, C) + orc.negacyclic_mul(B, C))


# ---------------------------------------------------------------- decomposition, modswitch

@pytest.mark.parametrize("beta,level", [(4, 3), (8, 2), (2, 5), (3, 5), (16, 1), (5, 3)])
def test_decomposition_identity_exhaustive_top_bits(orc, beta, level):
    bits = beta * level
    B = 1 << beta
    low = [0, 1, (1 << (63 - bits)) - 1, 1 << (63 - bits), (1 << (63 - bits)) + 1, (1 << (64 - bits)) - 1]
    step = 1 if bits <= 12 else 5
    for top in range(0, 1 << bits, step):
        for lo in low:
            x = ((top << (64 - bits)) | lo) & MASK
            d = [int(v) for v in orc.decompose(x, beta, level)]
            assert all(-B // 2 <= v < B // 2 for v in d)
            recomposed = sum(v << (64 - (j + 1) * beta) for j, v in enumerate(d)) & MASK
            rounded = (((x + (1 << (63 - bits))) >> (64 - bits)) << (64 - bits)) & MASK
            assert recomposed == rounded
            diff = (x - recomposed) & MASK
            diff = diff - (1 << 64) if diff >= (1 << 63) else diff
            assert -(1 << (63 - bits)) <= diff < (1 << (63 - bits)) + 1
            assert d == ref.digits(x, beta, level)


@pytest.mark.parametrize("beta,level", [(23, 1), (15, 2), (8, 8), (32, 2), (21, 3)])
def test_decomposition_identity_random(orc, beta, level):
    bits = beta * level
    xs = [int(v) for v in rng_words(beta * 100 + level, 2000)] + [0, MASK, 1 << 63, (1 << 63) - 1]
    for x in xs:
        d = [int(v) for v in orc.decompose(x, beta, level)]
        assert d == ref.digits(x, beta, level)
        recomposed = sum(v << (64 - (j + 1) * beta) for j, v in enumerate(d)) & MASK
        if bits < 64:
            rounded = (((x + (1 << (63 - bits))) >> (64 - bits)) << (64 - bits)) & MASK
        else:
            rounded = x
        assert recomposed == rounded


def test_modswitch_rounds_to_nearest_and_wraps(orc):
    for N in [8, 512, 2048, 32768]:
        w = 64 - int(math.log2(2 * N))
        assert orc.modswitch(0, N) == 0
        assert orc.modswitch((1 << (w - 1)) - 1, N) == 0
        assert orc.modswitch(1 << (w - 1), N) == 1                   # tie rounds up
        assert orc.modswitch(MASK, N) == 0                           # wraps to 0
        assert orc.modswitch(1 << 63, N) == N
        for x in [int(v) for v in rng_words(N, 200)]:
            assert orc.modswitch(x, N) == ref.modswitch(x, N)
            # nearest multiple of 2^64/2N in exact integers
            k = orc.modswitch(x, N)
            dist = min((x - (k << w)) % (1 << 64), ((k << w) - x) % (1 << 64))
            assert dist <= 1 << (w - 1)


# ---------------------------------------------------------------- LUT encoding

def test_lut_encode_boxes(orc):
    p = tiny(N=64, msg_bits=3)
    table = np.array([3, 1, 4, 1, 5, 2, 6, 7], dtype=np.uint64)
    V = orc.lut_encode(p, table)[0]
    box, h, delta = p.N // p.t, p.N // p.t // 2, p.delta
    # unrotated polynomial V0[j] = delta f(j div box); V = X^{-h} V0
    V0 = np.array([delta * int(table[j // box]) for j in range(p.N)], dtype=object)
    want = orc.monomial_mul(np.array([int(v) & MASK for v in V0], dtype=np.uint64), 2 * p.N - h)
    assert np.array_equal(V, want)
    # every mod-switched phase within half a box of m*box reads f(m)
    for m in range(p.t):
        for off in range(-h, box - h):
            j = m * box + off
            val = int(V[j]) if j >= 0 else (-int(V[j + p.N])) & MASK
            assert val == (delta * int(table[m])) & MASK


def test_signed_encoding_relu_table_matches_paper_example():
    # tests/golden/signed_encoding.txt: the paper's example (0,1,2,-2,-1) -> (0,1,2,3,4) on Z_5:
    # non-negative values occupy the lower half, negative ones the upper half.
    import os
    rows = [l.split() for l in open(os.path.join(os.path.dirname(__file__), "golden", "signed_encoding.txt"))
            if l.strip() and not l.startswith("#")]
    signed = [int(v) for v in rows[0]]
    encoded = [int(v) for v in rows[1]]
    M = len(signed)
    assert [v % M for v in signed] == encoded
    p = synth.CONFIGS[2]
    relu = synth.relu_table(p)
    for v in range(p.t):
        sv = v if v < p.t // 2 else v - p.t           # decode: upper half is negative
        assert int(relu[v]) == max(sv, 0)


# ---------------------------------------------------------------- LWE / GLWE linearity and round trips

def test_lwe_roundtrip_and_linearity(orc):
    p = tiny(n=64, msg_bits=3)
    sk = synth.lwe_secret(p)
    m1 = synth.messages(p, 32)
    m2 = synth.messages(p.with_(seed=5), 32)
    c1 = orc.encrypt_messages(p, synth, sk, m1)
    c2 = orc.encrypt_messages(p, synth, sk, m2, offset=1000)
    d1, e1 = orc.decode(orc.lwe_phase(sk, c1), p.msg_bits)
    assert np.array_equal(d1, m1)
    assert np.abs(e1).max() < 8 * p.sigma_lwe
    with np.errstate(over="ignore"):
        s, _ = orc.decode(orc.lwe_phase(sk, c1 + c2), p.msg_bits)
        assert np.array_equal(s, (m1 + m2) % np.uint64(2 * p.t))
        t3, _ = orc.decode(orc.lwe_phase(sk, c1 * np.uint64(3)), p.msg_bits)
        assert np.array_equal(t3, (m1 * np.uint64(3)) % np.uint64(2 * p.t))
        neg, _ = orc.decode(orc.lwe_phase(sk, (~c1) + np.uint64(1)), p.msg_bits)
        assert np.array_equal(neg, (np.uint64(2 * p.t) - m1) % np.uint64(2 * p.t))


def test_glwe_roundtrip_and_linearity(orc):
    p = tiny(N=64)
    S = synth.glwe_secret(p)
    M1 = rng_words(11, p.N) & ~np.uint64((1 << 40) - 1)
    M2 = rng_words(12, p.N) & ~np.uint64((1 << 40) - 1)
    A1, A2 = rng_words(13, p.N).reshape(1, p.N), rng_words(14, p.N).reshape(1, p.N)
    E1 = synth.gaussian_ints(1, "misc", p.N, 2.0 ** -40)
    E2 = synth.gaussian_ints(2, "misc", p.N, 2.0 ** -40)
    C1, C2 = orc.glwe_encrypt(S, A1, E1, M1), orc.glwe_encrypt(S, A2, E2, M2)
    with np.errstate(over="ignore"):
        assert np.array_equal(orc.glwe_phase(S, C1), M1 + E1.astype(np.uint64))
        assert np.array_equal(orc.glwe_phase(S, C1 + C2), M1 + M2 + (E1 + E2).astype(np.uint64))
        # multiplying a GLWE ciphertext by a monomial rotates its phase
        rot = np.stack([orc.monomial_mul(C1[r], 5) for r in range(2)])
        assert np.array_equal(orc.glwe_phase(S, rot), orc.monomial_mul(M1 + E1.astype(np.uint64), 5))


def test_sample_extract_phase_is_constant_coefficient(orc):
    p = tiny(N=64, k=2)
    S = synth.glwe_secret(p)
    ct = rng_words(21, 3 * p.N).reshape(3, p.N)
    lwe = orc.sample_extract(p, ct)
    assert int(orc.lwe_phase(S.reshape(-1), lwe)) == int(orc.glwe_phase(S, ct)[0])


# ---------------------------------------------------------------- special cases of the bootstrapping

def test_zero_bsk_leaves_rotated_lut(orc):
    # all-zero secret keys, masks and noise: the bootstrapping key is all zeros, the accumulator is never
    # changed, and the output is the trivial ciphertext (0,..,0, +-V[b~ mod N]).
    p = tiny(n=6, N=32, msg_bits=2)
    bsk = np.zeros((p.n, 2, p.pbs_level, 2, p.N), dtype=np.uint64)
    V = orc.lut_encode(p, np.array([1, 3, 0, 2], dtype=np.uint64))
    for bt in [0, 1, 7, p.N - 1, p.N, p.N + 1, 2 * p.N - 1]:
        lwe = rng_words(bt, p.n + 1).copy()
        lwe[p.n] = np.uint64(bt << (64 - 6))                    # 2N = 64 = 2^6
        out = orc.pbs_batch(p, lwe.reshape(1, -1), V, None, bsk)[0]
        assert not out[:-1].any()
        want = int(V[0][bt]) if bt < p.N else (-int(V[0][bt - p.N])) & MASK
        assert int(out[-1]) == want


def test_zero_mask_input_leaves_accumulator_unchanged(orc):
    # a~_i = 0 for all i: X^0 ACC - ACC = 0, Dec(0) = 0, nothing is added, whatever the key is.
    p = tiny()
    keys = orc.Keys(p, synth, with_ksk=False)
    V = orc.lut_encode(p, synth.random_tables(p, 1))
    lwe = np.zeros((1, p.n + 1), dtype=np.uint64)
    lwe[0, p.n] = np.uint64(5 << (64 - 6))
    acc = orc.blind_rotate_batch(p, lwe, V, None, keys.bsk, p.n)[0]
    assert not acc[0].any()
    assert np.array_equal(acc[1], orc.monomial_mul(V[0], 2 * p.N - 5))


def test_noiseless_bsk_rotates_exactly_up_to_rounding(orc):
    # zero-noise bootstrapping key: after all n steps the accumulator's phase is X^{-mu~} V with
    # mu~ = b~ - sum a~_i s_i, up to the decomposition rounding only:
    # |error| <= (#ones in s) * (1 + k N) * 2^(63 - beta*l) per coefficient.
    p = tiny(n=12, N=64, sigma_bsk=0.0, pbs_base_log=10, pbs_level=3, msg_bits=3)
    keys = orc.Keys(p, synth, with_ksk=False)
    V = orc.lut_encode(p, synth.random_tables(p, 1))
    cts = rng_words(99, 6 * (p.n + 1)).reshape(6, p.n + 1)
    accs = orc.blind_rotate_batch(p, cts, V, None, keys.bsk, p.n)
    bound = int(keys.lwe_sk.sum()) * (1 + p.N) * (1 << (63 - 30))
    for c in range(6):
        mu = orc.modswitch(int(cts[c, p.n]), p.N)
        for i in range(p.n):
            mu -= orc.modswitch(int(cts[c, i]), p.N) * int(keys.lwe_sk[i])
        want = orc.monomial_mul(V[0], (-mu) % (2 * p.N))
        got = orc.glwe_phase(keys.glwe_sk, accs[c])
        err = (got - want).astype(np.int64)
        assert np.abs(err).max() <= bound
        assert np.abs(err).max() > 0          # rounding error is really there (not a trivial pass)


def test_cmux_selects(orc):
    # one CMux with a noiseless GGSW of bit s: s=0 keeps ACC, s=1 gives X^a ACC (up to rounding)
    p = tiny(n=2, N=32, sigma_bsk=0.0, pbs_base_log=16, pbs_level=3)
    S = synth.glwe_secret(p)
    acc_msg = rng_words(7, p.N) & ~np.uint64((1 << 30) - 1)
    acc = orc.glwe_encrypt(S, rng_words(8, p.N).reshape(1, -1), np.zeros(p.N, dtype=np.int64), acc_msg)
    for s in (0, 1):
        mask, noise = synth.bsk_randomness(p)
        bsk = orc.bsk_gen(p, np.array([s, s], dtype=np.uint64), S, mask, noise)
        out = orc.cmux(p, acc, bsk[0], 9)
        want = orc.monomial_mul(acc_msg, 9) if s else acc_msg
        err = (orc.glwe_phase(S, out) - want).astype(np.int64)
        assert np.abs(err).max() <= (1 + p.N) * (1 << 15)


# ---------------------------------------------------------------- functional: every message, negacyclic law

@pytest.mark.parametrize("case", [
    dict(n=16, N=64, msg_bits=2, pbs_base_log=8, pbs_level=3, ks_base_log=4, ks_level=4),
    dict(n=24, N=128, msg_bits=3, pbs_base_log=12, pbs_level=2, ks_base_log=3, ks_level=5, k=1),
    dict(n=12, N=32, msg_bits=2, pbs_base_log=10, pbs_level=2, ks_base_log=4, ks_level=4, k=2),
])
def test_pbs_keyswitch_evaluates_the_table_for_every_message(orc, case):
    p = tiny(sigma_lwe=2.0 ** -30, sigma_bsk=2.0 ** -50, **case)
    keys = orc.Keys(p, synth)
    tables = np.concatenate([synth.random_tables(p, 2), synth.identity_table(p).reshape(1, -1)])
    V = orc.lut_encode(p, tables)
    reps = 3
    msgs = np.tile(np.arange(2 * p.t, dtype=np.uint64), reps)            # includes padding bit set
    lut_idx = (np.arange(msgs.size) % 3).astype(np.uint32)
    cts = orc.encrypt_messages(p, synth, keys.lwe_sk, msgs)
    big = orc.pbs_batch(p, cts, V, lut_idx, keys.bsk)
    small = orc.keyswitch_batch(p, big, keys.ksk)
    got_big, err_big = orc.decode(orc.lwe_phase(keys.big_sk, big), p.msg_bits)
    got_small, err_small = orc.decode(orc.lwe_phase(keys.lwe_sk, small), p.msg_bits)
    for c, m in enumerate(msgs):
        f = int(tables[lut_idx[c]][int(m) % p.t])
        want = f if m < p.t else (-f) % (2 * p.t)                            # negacyclic law: m + t -> -f(m)
        assert int(got_big[c]) == want, (c, m)
        assert int(got_small[c]) == want, (c, m)
    assert np.abs(err_big).max() < 2.0 ** -10 and np.abs(err_small).max() < 2.0 ** -6


def test_keyswitch_is_linear_and_exact_on_trivial_keys(orc):
    p = tiny(n=16, N=64, ks_base_log=4, ks_level=4)
    keys = orc.Keys(p, synth, with_bsk=False)
    m1, m2 = synth.messages(p, 16), synth.messages(p.with_(seed=3), 16)
    c1 = orc.encrypt_messages(p, synth, keys.big_sk, m1)
    c2 = orc.encrypt_messages(p, synth, keys.big_sk, m2, offset=500)
    with np.errstate(over="ignore"):
        ks = orc.keyswitch_batch(p, c1 + c2, keys.ksk)
    got, _ = orc.decode(orc.lwe_phase(keys.lwe_sk, ks), p.msg_bits)
    assert np.array_equal(got, (m1 + m2) % np.uint64(2 * p.t))
    # all-zero key-switching key: the output is exactly (0,...,0, b')
    out = orc.keyswitch_batch(p, c1, np.zeros_like(keys.ksk))
    assert not out[:, :-1].any() and np.array_equal(out[:, -1], c1[:, -1])


def test_lwe_lincomb_matches_integer_matmul(orc):
    G, J, O, width = 3, 20, 5, 9
    cts = rng_words(31, G * J * width).reshape(G, J, width)
    w = (synth.uniform_below(31, "misc", J * O, 13, offset=999).astype(np.int64) - 6).astype(np.int32).reshape(J, O)
    got = orc.lwe_lincomb_batch(cts, w)
    want = np.zeros((G, O, width), dtype=object)
    for g in range(G):
        for o in range(O):
            for x in range(width):
                want[g, o, x] = sum(int(w[j, o]) * int(cts[g, j, x]) for j in range(J)) % (1 << 64)
    assert np.array_equal(got.astype(object), want)


# ---------------------------------------------------------------- brute force against the Python-integer definition

@pytest.mark.parametrize("k,level,beta", [(1, 2, 8), (2, 1, 16), (1, 4, 4)])
def test_tiny_pbs_bit_exact_against_python_integers(orc, k, level, beta):
    p = tiny(n=4, N=8, k=k, pbs_base_log=beta, pbs_level=level, msg_bits=1, ks_base_log=4, ks_level=2,
             sigma_lwe=2.0 ** -20, sigma_bsk=2.0 ** -30, seed=1000 + k * 10 + level)
    keys = orc.Keys(p, synth)
    V = orc.lut_encode(p, np.array([[1, 0], [1, 1]], dtype=np.uint64))
    msgs = np.arange(4, dtype=np.uint64)
    cts = orc.encrypt_messages(p, synth, keys.lwe_sk, msgs)
    lut_idx = np.array([0, 1, 1, 0], dtype=np.uint32)
    params = (p.n, p.k, p.N, beta, level)
    bsk_l = keys.bsk.astype(object).tolist()
    ksk_l = keys.ksk.astype(object).tolist()
    for steps in (0, 1, 3, p.n):
        accs = orc.blind_rotate_batch(p, cts, V, lut_idx, keys.bsk, steps)
        for c in range(4):
            want = ref.blind_rotate(params, [int(v) for v in cts[c]], [int(v) for v in V[lut_idx[c]]], bsk_l, steps)
            assert accs[c].astype(object).tolist() == want, (steps, c)
    big = orc.pbs_batch(p, cts, V, lut_idx, keys.bsk)
    small = orc.keyswitch_batch(p, big, keys.ksk)
    for c in range(4):
        acc = ref.blind_rotate(params, [int(v) for v in cts[c]], [int(v) for v in V[lut_idx[c]]], bsk_l, p.n)
        ext = ref.sample_extract(params, acc)
        assert [int(v) for v in big[c]] == ext
        assert [int(v) for v in small[c]] == ref.keyswitch(ext, ksk_l, p.ks_base_log, p.ks_level, p.n)


# ---------------------------------------------------------------- closed-form noise variances

def test_modswitch_drift_variance(orc):
    # Var of (mu~/2N - phase/2^64) = (1 + hw(s)) / (12 (2N)^2) for a binary key of Hamming weight hw
    p = tiny(n=64, N=256, sigma_lwe=0.0)
    sk = synth.lwe_secret(p)
    cts = rng_words(41, 4096 * (p.n + 1)).reshape(4096, p.n + 1)
    phases = orc.lwe_phase(sk, cts)
    drift = []
    for c in range(cts.shape[0]):
        mu = orc.modswitch(int(cts[c, p.n]), p.N) - sum(orc.modswitch(int(cts[c, i]), p.N) for i in range(p.n) if sk[i])
        d = (mu / (2 * p.N) - int(phases[c]) / 2.0 ** 64) % 1.0
        drift.append(d - 1.0 if d >= 0.5 else d)
    var = float(np.var(drift))
    want = (1 + int(sk.sum())) / (12.0 * (2 * p.N) ** 2)
    assert abs(var / want - 1.0) < 0.10
    assert abs(float(np.mean(drift))) < 4 * math.sqrt(want / len(drift))


@pytest.mark.parametrize("sigma", [2.0 ** -30, 2.0 ** -13])
def test_keyswitch_noise_variance(orc, sigma):
    # Averaged over keys: Var_KS = kN * l * ((B^2+2)/12) * sigma^2 + kN / (24 B^(2l)).  For ONE key, over random
    # inputs, the digits (uniform on [-B/2, B/2), variance (B^2-1)/12, mean -1/2) multiply the key's fixed noise
    # values e_ij, so the variance over inputs is ((B^2-1)/12) * sum e_ij^2 + hw(s') / (12 B^(2l)), and the mean
    # is -(1/2) sum e_ij.  The two cases make the rounding term, respectively the key-noise term, dominant.
    p = tiny(n=32, N=256, ks_base_log=3, ks_level=3, sigma_lwe=sigma)
    keys = orc.Keys(p, synth, with_bsk=False)
    _, ksk_noise = synth.ksk_randomness(p)
    e = ksk_noise.astype(np.float64) / 2.0 ** 64
    count = 4096
    cts = rng_words(51, count * (p.N + 1)).reshape(count, p.N + 1)
    out = orc.keyswitch_batch(p, cts, keys.ksk)
    err = (orc.lwe_phase(keys.lwe_sk, out) - orc.lwe_phase(keys.big_sk, cts)).astype(np.int64) / 2.0 ** 64
    B = 2.0 ** p.ks_base_log
    round_term = int(keys.big_sk.sum()) / (12.0 * B ** (2 * p.ks_level))
    want = ((B * B - 1) / 12.0) * float((e * e).sum()) + round_term
    assert abs(float(np.var(err)) / want - 1.0) < 0.08
    # the sign convention of the subtraction shows in the mean: out = (0, b') - sum d * KSK
    assert abs(float(np.mean(err)) - 0.5 * float(e.sum())) < 5 * math.sqrt(want / count)
    # and the realised key noise is itself close to its nominal variance
    nominal = p.N * p.ks_level * sigma ** 2
    assert abs(float((e * e).sum()) / nominal - 1.0) < 0.2


@pytest.mark.parametrize("sigma_bsk,beta,level", [(2.0 ** -26, 6, 2), (2.0 ** -50, 4, 2)])
def test_blind_rotation_noise_variance(orc, sigma_bsk, beta, level):
    # Var_BR = n (k+1) l N ((B^2+2)/12) sigma_bsk^2  +  hw(s) (1 + hw(S)) / (12 B^(2l)); the two cases make
    # the key-noise term, respectively the rounding term, the dominant one.
    p = tiny(n=16, N=64, pbs_base_log=beta, pbs_level=level, sigma_bsk=sigma_bsk, msg_bits=2)
    keys = orc.Keys(p, synth, with_ksk=False)
    V = orc.lut_encode(p, synth.random_tables(p, 1))
    count = 128
    cts = rng_words(61, count * (p.n + 1)).reshape(count, p.n + 1)
    accs = orc.blind_rotate_batch(p, cts, V, None, keys.bsk, p.n)
    errs = []
    for c in range(count):
        mu = orc.modswitch(int(cts[c, p.n]), p.N)
        mu -= sum(orc.modswitch(int(cts[c, i]), p.N) for i in range(p.n) if keys.lwe_sk[i])
        want = orc.monomial_mul(V[0], (-mu) % (2 * p.N))
        errs.append((orc.glwe_phase(keys.glwe_sk, accs[c]) - want).astype(np.int64) / 2.0 ** 64)
    var = float(np.var(np.concatenate(errs)))
    B = 2.0 ** beta
    key_term = p.n * 2 * level * p.N * ((B * B + 2) / 12.0) * sigma_bsk ** 2
    round_term = int(keys.lwe_sk.sum()) * (1 + int(keys.glwe_sk.sum())) / (12.0 * B ** (2 * level))
    assert abs(var / (key_term + round_term) - 1.0) < 0.12
    assert max(key_term, round_term) / (key_term + round_term) > 0.9


def test_config1_as_written_would_not_decrypt(orc):
    # Configuration 1 as written gives sigma = 2^-20 to the bootstrapping key as well.  The oracle run with such a key:
    # the measured blind-rotation noise has the closed form's variance (std 2^-4.8 > Delta/2 = 2^-5), and the share of
    # wrong decryptions is the Gaussian tail the closed form predicts (about 39 %), which is why the library's
    # configuration 1 uses sigma_bsk = 2^-40 (closed-form std below 2^-10).
    p = synth.CONFIGS[1]
    keys = orc.Keys(p, synth, with_ksk=False, sigma_bsk=2.0 ** -20)
    count = 192
    msgs = synth.messages(p, count, "ramp")
    cts = orc.encrypt_messages(p, synth, keys.lwe_sk, msgs)
    tables = synth.config_tables(1)
    big = orc.pbs_batch(p, cts, orc.lut_encode(p, tables), None, keys.bsk)
    phase = orc.lwe_phase(keys.big_sk, big)
    want = tables[0, msgs.astype(np.int64)]
    got, _ = orc.decode(phase, p.msg_bits)
    with np.errstate(over="ignore"):
        err = (phase - want * np.uint64(p.delta)).astype(np.int64).astype(np.float64) / 2.0 ** 64      # against the true value
    B = 2.0 ** p.pbs_base_log
    var = p.n * 2 * p.pbs_level * p.N * ((B * B + 2) / 12.0) * (2.0 ** -20) ** 2
    assert math.sqrt(var) > 2.0 ** -5
    assert abs(float(np.mean(err ** 2)) / var - 1.0) < 0.25
    half = 2.0 ** -(p.msg_bits + 2)                                       # Delta / 2 in torus units
    tail = math.erfc(half / math.sqrt(2.0 * var))                         # P(|e| > Delta/2), 0.385 here
    assert 0.37 < tail < 0.40
    wrong = float(np.mean(got != want))
    assert abs(wrong - tail) < 4.0 * math.sqrt(tail * (1 - tail) / count)  # 0.14 at 192 samples
    var_fixed = p.n * 2 * p.pbs_level * p.N * ((B * B + 2) / 12.0) * p.sigma_bsk ** 2 \
        + p.n * (1 + p.N / 2) / (24.0 * B ** (2 * p.pbs_level))
    assert math.sqrt(var_fixed) < 2.0 ** -10
