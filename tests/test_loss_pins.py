"""Pins of the oracle of the two-input lookup, IntCELossDeriv and the clipped weight update (oracle/loss.py): values worked
out by hand from the formulas, the softmax definition the algorithm approximates, exact rational rounding, brute force,
invariants, and decryption of the encrypted pipelines.  CPU only."""
import math
from fractions import Fraction

import numpy as np
import pytest

import synth
from synth import Params


@pytest.fixture(scope="module")
def ls(orc):
    from oracle import loss
    return loss


TOY = dict(n=4, k=1, N=2048, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8, msg_bits=8,
           sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1)


def test_exponential_values_worked_out_by_hand(ls):
    # Gamma = 7: round(2^kappa e^(v - 63)); e^-1 = 0.3679, e^-2 = 0.1353, e^-3 = 0.0498, e^-4 = 0.0183
    assert ls.exp_value([63, 62, 61, 60, 59, 58, 0], 7, 4).tolist() == [16, 6, 2, 1, 0, 0, 0]      # 16, 5.89, 2.17, 0.80, 0.29
    assert ls.exp_value([63, 62, 61, 60, 59], 7, 2).tolist() == [4, 1, 1, 0, 0]                    # 4, 1.47, 0.54, 0.20
    assert ls.exp_value([63, 62, 61], 7, 1).tolist() == [2, 1, 0]                                  # 2, 0.74, 0.27
    assert ls.exp_value([7, 6, 5, 4], 4, 3).tolist() == [8, 3, 1, 0]                               # 8, 2.94, 1.08, 0.40
    # the largest logit maps to 2^kappa, and the table never decreases
    for Gamma in (4, 6, 7, 8):
        for kappa in (1, 2, 4):
            vals = ls.exp_value(np.arange(1 << (Gamma - 1)), Gamma, kappa)
            assert int(vals[-1]) == 1 << kappa and np.all(np.diff(vals) >= 0) and int(vals.min()) >= 0
            # against the definition evaluated with Python floats
            for v in range(max(0, (1 << (Gamma - 1)) - 8), 1 << (Gamma - 1)):
                assert int(vals[v]) == round(math.exp(v - ((1 << (Gamma - 1)) - 1)) * (1 << kappa))


def test_rounding_is_to_nearest_with_ties_to_even(ls):
    assert ls.round_half_even_div([5, 7, 9, 1, 3, 10, 0], [2, 2, 2, 2, 2, 4, 9]).tolist() == [2, 4, 4, 0, 2, 2, 0]
    # against exact rationals: Python's round() of a Fraction is ties-to-even
    for num in range(0, 70):
        for den in range(1, 40):
            assert int(ls.round_half_even_div(num, den)) == round(Fraction(num, den))


def test_clear_loss_derivative_on_rows_worked_out_by_hand(ls):
    # kappa = 4, Gamma = 7.  Row 0: one dominant logit -> exponentials (16, 0, 0), S = 16, shares round(257/17) = 15, round(1/17) = 0,
    # sum 15.  Label on the dominant class: error (0, 0, 0).  Row 1: label elsewhere: error (15, -15, 0).
    # Row 2: all logits small -> exponentials 0, S = 0, shares 1 each, sum 3; error (1, 1, -2).
    # Row 3: logits 63, 62, 61 -> exponentials (16, 6, 2), S = 24, shares round(257/25) = 10, round(97/25) = 4, round(33/25) = 1, sum 15;
    # label on class 1: error (10, 4 - 15, 1).
    Yhat = np.array([[63, 10, -64], [63, 10, -64], [-5, 0, 12], [63, 62, 61]])
    Y = np.array([[1, 0, 0], [0, 1, 0], [0, 0, 1], [0, 1, 0]])
    err = ls.int_ce_loss_deriv_clear(Yhat, Y, 7, 4, return_error=True)
    assert err.tolist() == [[0, 0, 0], [15, -15, 0], [1, 1, -2], [10, -11, 1]]
    assert ls.int_ce_loss_deriv_clear(Yhat, Y, 7, 4).tolist() == [[0, 0, 0], [1, -1, 0], [1, 1, -1], [1, -1, 1]]


def test_clear_loss_derivative_invariants_and_agreement_with_softmax(ls):
    rng = np.random.default_rng(20250417)
    for kappa, b in ((4, 3), (2, 7), (1, 16), (4, 2)):
        a = 800
        # logits near the top of the range, where the approximated exponential is not flat
        Yhat = rng.integers(52, 64, size=(a, b))
        Yhat[::7] = rng.integers(-64, 64, size=Yhat[::7].shape)
        lab = rng.integers(0, b, size=a)
        Y = np.eye(b, dtype=np.int64)[lab]
        err = ls.int_ce_loss_deriv_clear(Yhat, Y, 7, kappa, return_error=True)
        sgn = ls.int_ce_loss_deriv_clear(Yhat, Y, 7, kappa)
        assert np.all(err.sum(axis=1) == 0)                        # the label's share is the whole row sum
        assert np.array_equal(sgn, np.sign(err))
        assert int(np.abs(err).max()) <= (b << kappa)              # the output width the algorithm states
        assert np.all(err[np.arange(a), lab] <= 0)                 # the labelled class never gets a positive error
        others = np.ones_like(Y, dtype=bool)
        others[np.arange(a), lab] = False
        assert np.all(err[others] >= 0)
        # rows whose largest logit sits at the top of the range (below it the approximated exponential is flat): where the true
        # softmax error is away from 0, the integer version has its sign
        soft = np.exp(Yhat - Yhat.max(axis=1, keepdims=True))
        soft = soft / soft.sum(axis=1, keepdims=True) - Y
        if kappa == 4:
            clear = (np.abs(soft) > 0.1) & (Yhat.max(axis=1) >= 62)[:, None]
            assert int(clear.sum()) > 100
            assert np.array_equal(sgn[clear], np.sign(soft[clear]).astype(np.int64))
    with pytest.raises(ValueError):
        ls.int_ce_loss_deriv_clear(np.zeros((1, 17)), np.zeros((1, 17)), 7, 1)


def test_loss_tables(ls):
    p = Params(name="toy", seed=1, **TOY)
    tabs = ls.loss_tables(p, 7, 7, 2)
    assert tabs.shape == (5, 256)
    relu, ex, share, prod, sgn = [t.astype(np.int64) for t in tabs]
    assert relu[5] == 5 and relu[127] == 127 and relu[128] == 0 and relu[255] == 0
    assert ex[63] == 4 and ex[62] == 1 and ex[61] == 1 and ex[60] == 0 and ex[64] == 0 and ex[200] == 0
    eb, sb = ls.loss_widths(7, 2)
    assert (eb, sb) == (3, 5)                                       # values 0..4 and 0..28
    for e in range(8):
        for s in range(32):
            assert share[(e << sb) + s] == round(Fraction(4 * e + 1, s + 1))
    for s in range(32):
        assert prod[s] == 0 and prod[32 + s] == s
    assert sgn[128] == 0 and sgn[129] == 1 and sgn[255] == 1 and sgn[127] == 255 and sgn[0] == 255      # the sign of v - 128
    # kappa = 4 with three classes needs 5 + 6 bits: does not fit 8
    with pytest.raises(ValueError):
        ls.loss_tables(p, 3, 7, 4)
    with pytest.raises(ValueError):
        ls.loss_tables(p, 3, 9, 2)


def test_bivariate_table_and_weight_update_brute_force(ls):
    p = Params(name="toy", seed=1, **TOY)
    tab = ls.bivariate_table(p, lambda x, y: x * y + 1, 3, 5).astype(np.int64)
    for x in range(8):
        for y in range(32):
            assert tab[32 * x + y] == (x * y + 1) % 256
    with pytest.raises(ValueError):
        ls.bivariate_table(p, lambda x, y: 0, 5, 4)
    for alpha in (2, 4, 6):
        t = ls.weight_update_table(p, alpha)[0].astype(np.int64)
        half = 1 << (alpha - 1)
        for w in range(-half, half):
            for g in (-1, 0, 1):
                want = max(-half, min(half - 1, w - g))
                assert int(ls.weight_update_clear(w, g, alpha)) == want
                assert t[4 * (w + half) + g + 1] == want % 256
    with pytest.raises(ValueError):
        ls.weight_update_table(p, 7)


def test_encrypted_loss_derivative_and_weight_update_decrypt_to_the_clear_clones(orc, ls):
    from oracle import gadgets as gd
    p = Params(name="loss_toy", seed=0x10552, **TOY)
    keys = orc.Keys(p, synth)
    Gamma, kappa = 7, 2
    Yhat = np.array([[63, 62, -3, 10, 61], [-64, 5, 0, -1, 20], [63, 63, 63, 63, 63]])
    Y = np.eye(5, dtype=np.int64)[[1, 4, 0]]
    a, b = Yhat.shape
    enc = lambda vals, off: orc.encrypt_messages(p, synth, keys.lwe_sk, gd.signed_encode(vals, 256).reshape(-1).astype(np.uint64),
                                                 offset=off)
    yh = enc(Yhat, 0).reshape(a, b, p.n + 1)
    yl = enc(Y, a * b).reshape(a, b, p.n + 1)
    out = ls.int_ce_loss_deriv_encrypted(p, yh, yl, Gamma, kappa, keys.bsk, keys.ksk)
    got, err = orc.decode(orc.lwe_phase(keys.lwe_sk, out.reshape(-1, p.n + 1)), p.msg_bits)
    want = ls.int_ce_loss_deriv_clear(Yhat, Y, Gamma, kappa)
    assert np.array_equal(gd.signed_decode(got.astype(np.int64), 256).reshape(a, b), want)
    assert float(np.abs(err).max()) < 2.0 ** -12
    assert want.tolist()[1] == [1, 1, 1, 1, -1]                     # the flat row: every class the same share

    alpha = 6
    W = np.array([-32, -32, -31, 0, 5, 31, 31, 30, -1])
    G = np.array([1, -1, 1, 0, -1, -1, 1, -1, 1])
    wc, gc = enc(W, 100), enc(G + 1, 200)
    upd = ls.weight_update_encrypted(p, wc, gc, alpha, keys.bsk, keys.ksk)
    got, err = orc.decode(orc.lwe_phase(keys.lwe_sk, upd), p.msg_bits)
    assert gd.signed_decode(got.astype(np.int64), 256).tolist() == [-32, -31, -32, 0, 6, 31, 30, 31, -2]
    assert gd.signed_decode(got.astype(np.int64), 256).tolist() == ls.weight_update_clear(W, G, alpha).tolist()

    # a free-standing two-input lookup: (x, y) -> max(x, y) on 4 + 4 bits
    x = np.array([0, 3, 15, 9, 7]); y = np.array([0, 12, 1, 9, 8])
    tab = ls.bivariate_table(p, max, 4, 4)[None]
    out = ls.bivariate_lookup_encrypted(p, enc(x, 300), enc(y, 400), 4, tab, np.zeros(5, dtype=np.uint32), keys.bsk, keys.ksk)
    got, _ = orc.decode(orc.lwe_phase(keys.lwe_sk, out), p.msg_bits)
    assert got.astype(np.int64).tolist() == np.maximum(x, y).tolist()


# ---- the paper's own settings: kappa = 4 and alpha = 8 (Sec. "Evaluation") ----------------------------------------------
# They need lookups on 11 and 10 bits: the same algorithms in a wider message space (one padding bit above it), which the
# polynomial size must carry (N >= 2 t, and boxes wide enough for the modulus-switch drift).  Toy sets (insecure on purpose,
# so that an oracle lookup stays near 1e9 multiply-adds): the drift of the rotation is sqrt((1 + n/2) / 12) = 0.41 positions
# at n = 2 against half-boxes of 2 positions.
WIDE11 = dict(n=2, k=1, N=8192, pbs_base_log=15, pbs_level=2, ks_base_log=4, ks_level=8, msg_bits=11,
              sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1)
WIDE10 = dict(n=2, k=1, N=4096, pbs_base_log=22, pbs_level=1, ks_base_log=4, ks_level=8, msg_bits=10,
              sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1)


def _through_tables(ls, p, Yhat, Y, Gamma, kappa):
    """IntCELossDeriv evaluated through the five lookup tables and the packed indices of the encrypted pipeline, on clear
    integers modulo 2t (what the ciphertexts carry when nothing goes wrong)."""
    t = 1 << p.msg_bits
    a, b = Yhat.shape
    relu, ex, share, prod, sgn = [x.astype(np.int64) for x in ls.loss_tables(p, b, Gamma, kappa)]
    _, sb = ls.loss_widths(b, kappa)
    E = ex[relu[np.mod(Yhat, t)]]
    S = E.sum(axis=1, keepdims=True)
    Q = share[(E << sb) + S]
    T = Q.sum(axis=1, keepdims=True)
    P = prod[(Y << sb) + T]
    return sgn[Q - P + t // 2]


def test_loss_tables_at_kappa_4_on_an_11_bit_message_space(ls):
    from oracle import gadgets as gd
    p = Params(name="wide11", seed=3, **WIDE11)
    b, Gamma, kappa = 3, 7, 4
    eb, sb = ls.loss_widths(b, kappa)
    assert (eb, sb) == (5, 6) and eb + sb == p.msg_bits             # exponentials 0..16, row sums 0..48
    relu, ex, share, prod, sgn = [x.astype(np.int64) for x in ls.loss_tables(p, b, Gamma, kappa)]
    assert [int(ex[v]) for v in (63, 62, 61, 60, 59, 0)] == [16, 6, 2, 1, 0, 0] and int(ex[64]) == 0
    for e in range(17):
        for s in range(49):
            assert share[(e << sb) + s] == round(Fraction(16 * e + 1, s + 1))
    assert share[(16 << sb) + 16] == 15 and share[(6 << sb) + 24] == 4 and share[0] == 1        # the hand-worked rows' shares
    for s in range(49):
        assert prod[s] == 0 and prod[64 + s] == s
    assert sgn[1024] == 0 and sgn[1025] == 1 and sgn[1023] == 2047 and relu[1023] == 1023 and relu[1024] == 0
    # the rows worked out by hand above, through the tables and packed indices
    Yhat = np.array([[63, 10, -64], [63, 10, -64], [-5, 0, 12], [63, 62, 61]])
    Y = np.array([[1, 0, 0], [0, 1, 0], [0, 0, 1], [0, 1, 0]])
    got = gd.signed_decode(_through_tables(ls, p, Yhat, Y, Gamma, kappa), 2048)
    assert got.tolist() == [[0, 0, 0], [1, -1, 0], [1, 1, -1], [1, -1, 1]]
    # and on random rows against the clone
    rng = np.random.default_rng(404)
    Yhat = rng.integers(54, 64, size=(300, 3))
    Yhat[::5] = rng.integers(-64, 64, size=Yhat[::5].shape)
    Y = np.eye(3, dtype=np.int64)[rng.integers(0, 3, size=300)]
    assert np.array_equal(gd.signed_decode(_through_tables(ls, p, Yhat, Y, Gamma, kappa), 2048), ls.int_ce_loss_deriv_clear(Yhat, Y, Gamma, kappa))


def test_weight_update_brute_force_at_alpha_8(ls):
    # clip(w - g) to [-128, 127] over every signed 8-bit weight and every g, through the table on 4 (w + 128) + g + 1
    p = Params(name="wide10", seed=3, **WIDE10)
    t = ls.weight_update_table(p, 8)[0].astype(np.int64)
    assert t.shape == (1024,)
    seen = 0
    for w in range(-128, 128):
        for g in (-1, 0, 1):
            want = max(-128, min(127, w - g))
            assert int(ls.weight_update_clear(w, g, 8)) == want
            assert t[4 * (w + 128) + g + 1] == want % 1024
            seen += 1
    assert seen == 768
    assert t[4 * 0 + 2] == (-128) % 1024 and t[4 * 255 + 0] == 127                              # the two clipped corners
    with pytest.raises(ValueError):
        ls.weight_update_table(Params(name="toy", seed=1, **TOY), 8)                            # 10 bits do not fit 8


def test_encrypted_pipelines_decrypt_at_kappa_4_and_alpha_8(orc, ls):
    from oracle import gadgets as gd
    p = Params(name="wide11", seed=0x11B17, **WIDE11)
    keys = orc.Keys(p, synth)
    t = 1 << p.msg_bits
    enc = lambda q, k, vals, off: orc.encrypt_messages(q, synth, k.lwe_sk, gd.signed_encode(vals, 1 << q.msg_bits).reshape(-1).astype(np.uint64),
                                                       offset=off)
    Yhat = np.array([[63, 62, 61], [63, 10, -64], [-5, 0, 12]])
    Y = np.eye(3, dtype=np.int64)[[1, 1, 2]]
    a, b = Yhat.shape
    yh = enc(p, keys, Yhat, 0).reshape(a, b, p.n + 1)
    yl = enc(p, keys, Y, a * b).reshape(a, b, p.n + 1)
    out = ls.int_ce_loss_deriv_encrypted(p, yh, yl, 7, 4, keys.bsk, keys.ksk)
    got, err = orc.decode(orc.lwe_phase(keys.lwe_sk, out.reshape(-1, p.n + 1)), p.msg_bits)
    assert gd.signed_decode(got.astype(np.int64), t).reshape(a, b).tolist() == [[1, -1, 1], [1, -1, 0], [1, 1, -1]]
    assert float(np.abs(err).max()) < 2.0 ** -15                    # against Delta / 2 = 2^-13

    p10 = Params(name="wide10", seed=0x10B17, **WIDE10)
    k10 = orc.Keys(p10, synth)
    W = np.array([-128, -128, -127, 0, 5, 127, 127, 126, -1, 64])
    G = np.array([1, -1, 1, 0, -1, -1, 1, -1, 1, 0])
    upd = ls.weight_update_encrypted(p10, enc(p10, k10, W, 100), enc(p10, k10, G + 1, 200), 8, k10.bsk, k10.ksk)
    got, err = orc.decode(orc.lwe_phase(k10.lwe_sk, upd), p10.msg_bits)
    assert gd.signed_decode(got.astype(np.int64), 1024).tolist() == [-128, -127, -128, 0, 6, 127, 126, 127, -2, 64]
    assert float(np.abs(err).max()) < 2.0 ** -14
