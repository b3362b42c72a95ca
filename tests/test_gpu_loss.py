"""GPU parity of the two-input lookup, IntCELossDeriv and the clipped weight update: the library against the oracle's
encrypted pipelines, bit for bit, and decryption against the clear-integer clones.  Toy (insecure) parameters with an 8-bit
message space keep the oracle's lookups at 7e7 multiply-adds each; the paper's own settings (kappa = 4, alpha = 8) run on toy
sets with 11- and 10-bit message spaces."""
import ctypes

import numpy as np
import pytest

import synth
from synth import Params

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def slz():
    if not torch.cuda.is_available():
        pytest.fail("the gpu tests need a GPU: torch.cuda.is_available() is False")
    import paper_2504_17785_amd as m
    m.lib()
    return m


@pytest.fixture(scope="module")
def toy(orc):
    p = Params(name="loss_toy", n=4, k=1, N=2048, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8, msg_bits=8,
               sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1, seed=0x10552)
    return p, orc.Keys(p, synth)


def _enc(orc, p, keys, vals, offset):
    from oracle import gadgets as gd
    return orc.encrypt_messages(p, synth, keys.lwe_sk, gd.signed_encode(vals, 1 << p.msg_bits).reshape(-1).astype(np.uint64),
                                offset=offset)


def _logits(p, a, b, offset):
    """Signed 7-bit logits: most near the top of the range (where the approximated exponential moves), some anywhere."""
    top = 63 - synth.uniform_below(p.seed, "messages", a * b, 6, offset).astype(np.int64)
    wide = synth.uniform_below(p.seed, "messages", a * b, 128, offset + a * b).astype(np.int64) - 64
    pick = synth.uniform_below(p.seed, "messages", a * b, 4, offset + 2 * a * b)
    Yhat = np.where(pick == 0, wide, top).reshape(a, b)
    labels = np.eye(b, dtype=np.int64)[synth.uniform_below(p.seed, "lut_idx", a, b, offset).astype(np.int64)]
    return Yhat, labels


@pytest.mark.parametrize("a,b,kappa,max_batch", [(3, 5, 2, 64), (2, 7, 2, 5), (4, 16, 1, 64), (1, 1, 2, 1), (5, 2, 2, 3)])
def test_int_ce_loss_deriv_matches_oracle_and_decrypts(slz, orc, toy, a, b, kappa, max_batch):
    from oracle import gadgets as gd
    from oracle import loss
    p, keys = toy
    Gamma = 7
    Yhat, Y = _logits(p, a, b, offset=100 * a + b)
    Yhat.flat[0] = 63
    if a * b > 2:
        Yhat.flat[1], Yhat.flat[-1] = -64, 0
    yh = _enc(orc, p, keys, Yhat, 0).reshape(a, b, p.n + 1)
    yl = _enc(orc, p, keys, Y, a * b).reshape(a, b, p.n + 1)
    ctx = slz.Context(p, max_batch)                      # lookups larger than max_batch go through in chunks
    d_bsk = ctx.bsk_prepare(slz.to_device_u64(keys.bsk))
    d_luts = slz.to_device_u64(slz.loss_luts(p, b, Gamma, kappa))
    got = slz.to_host_u64(ctx.int_ce_loss_deriv(slz.to_device_u64(yh), slz.to_device_u64(yl), Gamma, kappa, d_luts, d_bsk,
                                                slz.to_device_u64(keys.ksk)))
    want = loss.int_ce_loss_deriv_encrypted(p, yh, yl, Gamma, kappa, keys.bsk, keys.ksk)
    assert np.array_equal(got, want)
    dec, _ = orc.decode(orc.lwe_phase(keys.lwe_sk, got.reshape(-1, p.n + 1)), p.msg_bits)
    assert np.array_equal(gd.signed_decode(dec.astype(np.int64), 256).reshape(a, b), loss.int_ce_loss_deriv_clear(Yhat, Y, Gamma, kappa))


@pytest.mark.parametrize("alpha,count,max_batch", [(6, 70, 64), (4, 16, 64), (2, 5, 2)])
def test_weight_update_matches_oracle_and_decrypts(slz, orc, toy, alpha, count, max_batch):
    from oracle import gadgets as gd
    from oracle import loss
    p, keys = toy
    half = 1 << (alpha - 1)
    W = synth.uniform_below(p.seed, "weights", count, 2 * half, alpha).astype(np.int64) - half
    G = synth.uniform_below(p.seed, "lut_idx", count, 3, alpha).astype(np.int64) - 1
    W[:4] = [-half, -half, half - 1, half - 1]
    G[:4] = [1, -1, -1, 1]                               # both clipped ends and their free neighbours
    wc, gc = _enc(orc, p, keys, W, 0), _enc(orc, p, keys, G + 1, count)
    ctx = slz.Context(p, max_batch)
    d_bsk = ctx.bsk_prepare(slz.to_device_u64(keys.bsk))
    d_luts = slz.to_device_u64(slz.weight_update_luts(p, alpha))
    got = slz.to_host_u64(ctx.weight_update(slz.to_device_u64(wc), slz.to_device_u64(gc), alpha, d_luts, d_bsk, slz.to_device_u64(keys.ksk)))
    want = loss.weight_update_encrypted(p, wc, gc, alpha, keys.bsk, keys.ksk)
    assert np.array_equal(got, want)
    dec, _ = orc.decode(orc.lwe_phase(keys.lwe_sk, got), p.msg_bits)
    assert np.array_equal(gd.signed_decode(dec.astype(np.int64), 256), np.clip(W - G, -half, half - 1))


# ---- the paper's own settings (Sec. "Evaluation"): kappa = 4 and weights clipped to the signed 8-bit range -----------------
# 11- and 10-bit lookups: the same entry points on parameter sets with a wider message space (toy sizes for the oracle's sake).
@pytest.fixture(scope="module")
def wide11(orc):
    p = Params(name="wide11", n=2, k=1, N=8192, pbs_base_log=15, pbs_level=2, ks_base_log=4, ks_level=8, msg_bits=11,
               sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1, seed=0x11B17)
    return p, orc.Keys(p, synth)


@pytest.fixture(scope="module")
def wide10(orc):
    p = Params(name="wide10", n=2, k=1, N=4096, pbs_base_log=22, pbs_level=1, ks_base_log=4, ks_level=8, msg_bits=10,
               sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1, seed=0x10B17)
    return p, orc.Keys(p, synth)


@pytest.mark.parametrize("a,b,max_batch", [(4, 3, 64), (3, 2, 4)])
def test_int_ce_loss_deriv_at_kappa_4(slz, orc, wide11, a, b, max_batch):
    from oracle import gadgets as gd
    from oracle import loss
    p, keys = wide11
    Gamma, kappa = 7, 4
    Yhat, Y = _logits(p, a, b, offset=100 * a + b)
    Yhat[0] = [63, 62, 61][:b]                           # a row whose exponentials are 16, 6, 2
    Yhat.flat[-1] = -64
    yh = _enc(orc, p, keys, Yhat, 0).reshape(a, b, p.n + 1)
    yl = _enc(orc, p, keys, Y, a * b).reshape(a, b, p.n + 1)
    ctx = slz.Context(p, max_batch)
    assert ctx.path == "three_pass_large_n"
    d_bsk = ctx.bsk_prepare(slz.to_device_u64(keys.bsk))
    d_luts = slz.to_device_u64(slz.loss_luts(p, b, Gamma, kappa))
    assert np.array_equal(slz.loss_luts(p, b, Gamma, kappa), orc.lut_encode(p, loss.loss_tables(p, b, Gamma, kappa)))
    got = slz.to_host_u64(ctx.int_ce_loss_deriv(slz.to_device_u64(yh), slz.to_device_u64(yl), Gamma, kappa, d_luts, d_bsk,
                                                slz.to_device_u64(keys.ksk)))
    want = loss.int_ce_loss_deriv_encrypted(p, yh, yl, Gamma, kappa, keys.bsk, keys.ksk)
    assert np.array_equal(got, want)
    dec, _ = orc.decode(orc.lwe_phase(keys.lwe_sk, got.reshape(-1, p.n + 1)), p.msg_bits)
    assert np.array_equal(gd.signed_decode(dec.astype(np.int64), 1 << p.msg_bits).reshape(a, b),
                          loss.int_ce_loss_deriv_clear(Yhat, Y, Gamma, kappa))


@pytest.mark.parametrize("count,max_batch", [(40, 64), (9, 4)])
def test_weight_update_at_alpha_8(slz, orc, wide10, count, max_batch):
    from oracle import gadgets as gd
    from oracle import loss
    p, keys = wide10
    alpha = 8
    W = synth.uniform_below(p.seed, "weights", count, 256, alpha).astype(np.int64) - 128
    G = synth.uniform_below(p.seed, "lut_idx", count, 3, alpha).astype(np.int64) - 1
    W[:4] = [-128, -128, 127, 127]
    G[:4] = [1, -1, -1, 1]                               # both clipped ends and their free neighbours
    wc, gc = _enc(orc, p, keys, W, 0), _enc(orc, p, keys, G + 1, count)
    ctx = slz.Context(p, max_batch)
    assert ctx.path == "fused_n4096"
    d_bsk = ctx.bsk_prepare(slz.to_device_u64(keys.bsk))
    assert np.array_equal(slz.weight_update_luts(p, alpha), orc.lut_encode(p, loss.weight_update_table(p, alpha)))
    d_luts = slz.to_device_u64(slz.weight_update_luts(p, alpha))
    got = slz.to_host_u64(ctx.weight_update(slz.to_device_u64(wc), slz.to_device_u64(gc), alpha, d_luts, d_bsk, slz.to_device_u64(keys.ksk)))
    want = loss.weight_update_encrypted(p, wc, gc, alpha, keys.bsk, keys.ksk)
    assert np.array_equal(got, want)
    dec, _ = orc.decode(orc.lwe_phase(keys.lwe_sk, got), p.msg_bits)
    assert np.array_equal(gd.signed_decode(dec.astype(np.int64), 1024), np.clip(W - G, -128, 127))


def test_bivariate_lookup_matches_oracle_with_several_tables(slz, orc, toy):
    from oracle import loss
    p, keys = toy
    count, bx, by = 37, 3, 5
    x = synth.uniform_below(p.seed, "messages", count, 1 << bx, 7).astype(np.int64)
    y = synth.uniform_below(p.seed, "messages", count, 1 << by, 8).astype(np.int64)
    x[:2], y[:2] = [0, 7], [0, 31]
    tabs = np.stack([loss.bivariate_table(p, lambda u, v: u * v, bx, by), loss.bivariate_table(p, lambda u, v: max(4 * u, v), bx, by),
                     loss.bivariate_table(p, lambda u, v: (u + v) % 7, bx, by)])
    idx = (np.arange(count) % 3).astype(np.uint32)
    xc, yc = _enc(orc, p, keys, x, 0), _enc(orc, p, keys, y, count)
    ctx = slz.Context(p, 16)
    d_bsk = ctx.bsk_prepare(slz.to_device_u64(keys.bsk))
    d_luts = slz.to_device_u64(slz.lut_encode(p, tabs))
    d_idx = torch.from_numpy(idx.astype(np.int32)).cuda()
    got = slz.to_host_u64(ctx.bivariate_lookup(slz.to_device_u64(xc), slz.to_device_u64(yc), by, d_luts, d_bsk, slz.to_device_u64(keys.ksk),
                                               lut_index=d_idx))
    want = loss.bivariate_lookup_encrypted(p, xc, yc, by, tabs, idx, keys.bsk, keys.ksk)
    assert np.array_equal(got, want)
    dec, _ = orc.decode(orc.lwe_phase(keys.lwe_sk, got), p.msg_bits)
    f = [lambda u, v: u * v, lambda u, v: max(4 * u, v), lambda u, v: (u + v) % 7]
    assert dec.astype(np.int64).tolist() == [f[i % 3](int(x[i]), int(y[i])) % 256 for i in range(count)]
    # without an index every pair uses table 0
    got0 = slz.to_host_u64(ctx.bivariate_lookup(slz.to_device_u64(xc), slz.to_device_u64(yc), by, d_luts, d_bsk, slz.to_device_u64(keys.ksk)))
    assert np.array_equal(got0, loss.bivariate_lookup_encrypted(p, xc, yc, by, tabs, np.zeros(count, dtype=np.uint32), keys.bsk, keys.ksk))


def test_loss_error_codes(slz, toy):
    p, keys = toy
    ctx = slz.Context(p, 8)
    L = slz.lib()
    sh = slz.SlzLossShape(2, 3, 7, 2)
    need = ctypes.c_size_t(0)
    assert L.slz_loss_workspace(ctx._h, ctypes.byref(sh), ctypes.byref(need)) == 0 and need.value > 0
    buf = torch.zeros(need.value + 4096, dtype=torch.uint8, device="cuda")
    ptr = buf.data_ptr()
    cts = torch.zeros((6, p.n + 1), dtype=torch.int64, device="cuda")
    luts = torch.zeros((5, p.N), dtype=torch.int64, device="cuda")
    key = torch.zeros(64, dtype=torch.int64, device="cuda")          # never read: every call below is rejected before any launch
    c, l, k = cts.data_ptr(), luts.data_ptr(), key.data_ptr()
    INVALID = slz.SLZ_E_INVALID_ARG
    call = lambda shape, ws, nbytes, x=c: L.slz_int_ce_loss_deriv(ctx._h, ctypes.byref(shape), x, c, l, k, k, c, ws, nbytes, None)
    assert call(sh, ptr, need.value - 1) == INVALID                  # workspace too small
    assert call(sh, ptr + 8, need.value) == INVALID                  # workspace not 256-byte aligned
    assert call(sh, ptr, need.value, x=c + 4) == INVALID             # ciphertexts not 8-byte aligned
    assert call(slz.SlzLossShape(2, 3, 7, 4), ptr, need.value) == INVALID      # 5 + 6 bits do not fit 8
    assert call(slz.SlzLossShape(2, 17, 7, 1), ptr, need.value) == INVALID     # more than 16 classes
    assert call(slz.SlzLossShape(0, 3, 7, 2), ptr, need.value) == INVALID
    assert L.slz_int_ce_loss_deriv(ctx._h, ctypes.byref(sh), c, None, l, k, k, c, ptr, need.value, None) == INVALID
    bneed = ctypes.c_size_t(0)
    assert L.slz_bivariate_workspace(ctx._h, 6, ctypes.byref(bneed)) == 0 and 0 < bneed.value <= need.value
    assert L.slz_bivariate_workspace(ctx._h, 0, ctypes.byref(bneed)) == INVALID
    assert L.slz_bivariate_lookup(ctx._h, c, c, 8, l, None, 1, k, k, c, 6, ptr, need.value, None) == INVALID     # y_bits >= msg_bits
    assert L.slz_bivariate_lookup(ctx._h, c, c, 4, l, None, 0, k, k, c, 6, ptr, need.value, None) == INVALID     # no table
    assert L.slz_bivariate_lookup(ctx._h, c, c, 4, l, None, 1, k, k, c, 6, ptr, 16, None) == INVALID
    assert L.slz_weight_update(ctx._h, 7, c, c, l, k, k, c, 6, ptr, need.value, None) == INVALID                 # alpha + 2 > 8
    assert L.slz_weight_update(ctx._h, 6, c, c, l, k, k, c, 0, ptr, need.value, None) == INVALID
    torch.cuda.synchronize()
