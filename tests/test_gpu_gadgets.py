"""GPU parity of the Matmul^RNS gadget: slz_matmul_rns against the oracle's encrypted pipeline, bit for bit, and
decryption against the clear-integer clone.  Toy (insecure) parameters with an 8-bit message space keep the oracle's
lookups at 7e7 multiply-adds each; the N = 2048, l = 1 shape runs the fused blind-rotation kernel."""
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
    p = Params(name="gadget_toy", n=4, k=1, N=2048, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8, msg_bits=8,
               sigma_lwe=2.0 ** -40, sigma_bsk=2.0 ** -50, batch=1, n_luts=1, seed=0x6AD6E7)
    return p, orc.Keys(p, synth)


def _inputs(orc, gd, p, keys, a, b, c, offset):
    X = (synth.uniform_below(p.seed, "lin_inputs", a * b, 256, offset).astype(np.int64) - 128).reshape(a, b)
    W = (synth.uniform_below(p.seed, "weights", b * c, 256, offset).astype(np.int64) - 128).reshape(b, c)
    X.flat[0], W.flat[0] = -128, -128
    X.flat[-1], W.flat[-1] = 127, -1
    x_cts = orc.encrypt_messages(p, synth, keys.lwe_sk, gd.signed_encode(X, 256).reshape(-1).astype(np.uint64), offset=offset)
    w_cts = orc.encrypt_messages(p, synth, keys.lwe_sk, gd.signed_encode(W, 256).reshape(-1).astype(np.uint64), offset=offset + a * b)
    return X, W, x_cts.reshape(a, b, p.n + 1), w_cts.reshape(b, c, p.n + 1)


@pytest.mark.parametrize("a,b,c,m,max_batch", [(2, 3, 2, (15, 14), 64), (2, 17, 1, (13, 15, 14), 512), (1, 31, 2, (7, 11, 13, 15, 8), 37),
                                                (3, 1, 1, (5, 7, 9, 11, 13, 8), 1)])
def test_matmul_rns_matches_oracle_and_decrypts(slz, orc, toy, a, b, c, m, max_batch):
    from oracle import gadgets as gd
    p, keys = toy
    X, W, x_cts, w_cts = _inputs(orc, gd, p, keys, a, b, c, offset=1000 * a + b)
    ctx = slz.Context(p, max_batch)                       # lookups larger than max_batch go through in chunks
    assert ctx.path == "fused_n2048"
    d_bsk = ctx.bsk_prepare(slz.to_device_u64(keys.bsk))
    d_luts = slz.to_device_u64(slz.matmul_rns_luts(p, m, a, b, c))
    got = slz.to_host_u64(ctx.matmul_rns(slz.to_device_u64(x_cts), slz.to_device_u64(w_cts), m, d_luts, d_bsk, slz.to_device_u64(keys.ksk)))
    want = gd.matmul_rns_encrypted(p, x_cts, w_cts, m, keys.bsk, keys.ksk)
    assert np.array_equal(got, want)
    dec, err = orc.decode(orc.lwe_phase(keys.lwe_sk, got.reshape(-1, p.n + 1)), p.msg_bits)
    clear = gd.matmul_rns_clear(X, W, m)
    assert np.array_equal(dec.reshape(clear.shape).astype(np.int64), clear)
    for i, q in enumerate(m):
        assert np.array_equal(clear[i], np.mod(X @ W, q))


@pytest.mark.parametrize("a,b,c,m,max_batch", [(2, 3, 2, (31, 30), 64), (2, 9, 1, (29, 31, 30), 512), (1, 15, 2, (25, 27, 29, 31, 28), 37),
                                                (2, 1, 1, (23, 25, 27, 29, 31, 28), 1)])
def test_matmul_highres_matches_oracle_and_decrypts(slz, orc, toy, a, b, c, m, max_batch):
    from oracle import gadgets as gd
    p, keys = toy
    X, W, x_cts, w_cts = _inputs(orc, gd, p, keys, a, b, c, offset=2000 * a + b)
    ctx = slz.Context(p, max_batch)
    d_bsk = ctx.bsk_prepare(slz.to_device_u64(keys.bsk))
    d_luts = slz.to_device_u64(slz.matmul_highres_luts(p, m, a, b, c))
    got = slz.to_host_u64(ctx.matmul_rns(slz.to_device_u64(x_cts), slz.to_device_u64(w_cts), m, d_luts, d_bsk, slz.to_device_u64(keys.ksk),
                                         highres=True))
    want = gd.matmul_highres_encrypted(p, x_cts, w_cts, m, keys.bsk, keys.ksk)
    assert np.array_equal(got, want)
    dec, err = orc.decode(orc.lwe_phase(keys.lwe_sk, got.reshape(-1, p.n + 1)), p.msg_bits)
    for i, q in enumerate(m):
        assert np.array_equal(dec.reshape(len(m), a, c)[i].astype(np.int64), np.mod(X @ W, q))


def test_matmul_highres_error_codes(slz, toy):
    import ctypes
    p, keys = toy
    ctx = slz.Context(p, 8)
    L = slz.lib()
    sh = slz.make_matmul_rns_shape((31, 30), 2, 2, 2)
    need = ctypes.c_size_t(0)
    assert L.slz_matmul_highres_workspace(ctx._h, ctypes.byref(sh), ctypes.byref(need)) == 0 and need.value > 0
    buf = torch.zeros(need.value + 4096, dtype=torch.uint8, device="cuda")
    ptr = buf.data_ptr()
    cts = torch.zeros((8, p.n + 1), dtype=torch.int64, device="cuda")
    c = cts.data_ptr()
    call = lambda shape, ws, nbytes, x=c: L.slz_matmul_highres(ctx._h, ctypes.byref(shape), x, c, c, c, c, c, ws, nbytes, None)
    assert call(sh, ptr, need.value - 1) == slz.SLZ_E_INVALID_ARG
    assert call(sh, ptr + 8, need.value) == slz.SLZ_E_INVALID_ARG
    assert call(sh, ptr, need.value, x=c + 4) == slz.SLZ_E_INVALID_ARG
    assert call(slz.make_matmul_rns_shape((33, 31), 2, 2, 2), ptr, need.value) == slz.SLZ_E_INVALID_ARG
    assert call(slz.make_matmul_rns_shape((31, 30), 2, 0, 2), ptr, need.value) == slz.SLZ_E_INVALID_ARG
    torch.cuda.synchronize()


def test_matmul_rns_error_codes(slz, toy):
    import ctypes
    p, keys = toy
    ctx = slz.Context(p, 8)
    L = slz.lib()
    sh = slz.make_matmul_rns_shape((15, 14), 2, 2, 2)
    need = ctypes.c_size_t(0)
    assert L.slz_matmul_rns_workspace(ctx._h, ctypes.byref(sh), ctypes.byref(need)) == 0 and need.value > 0
    buf = torch.zeros(need.value + 4096, dtype=torch.uint8, device="cuda")
    ptr = buf.data_ptr()
    args = lambda ws, nbytes: (ctx._h, ctypes.byref(sh), ptr, ptr, ptr, ptr, ptr, ptr, ws, nbytes, None)
    assert L.slz_matmul_rns(*args(ptr, need.value - 1)) == slz.SLZ_E_INVALID_ARG        # workspace too small
    assert L.slz_matmul_rns(*args(ptr + 8, need.value)) == slz.SLZ_E_INVALID_ARG        # workspace not 256-byte aligned
    assert L.slz_matmul_rns(*args(None, need.value)) == slz.SLZ_E_INVALID_ARG
    bad = slz.make_matmul_rns_shape((15, 33), 2, 2, 2)
    assert L.slz_matmul_rns_workspace(ctx._h, ctypes.byref(bad), ctypes.byref(need)) == slz.SLZ_E_INVALID_ARG
    ctx4 = slz.Context(p.with_(msg_bits=4), 8)
    assert L.slz_matmul_rns_workspace(ctx4._h, ctypes.byref(sh), ctypes.byref(need)) == slz.SLZ_E_INVALID_ARG


@pytest.mark.parametrize("m,max_batch", [((5, 7, 8), 64), ((13, 15, 14), 7), ((7, 11, 13, 15, 8), 256), ((15, 14), 1)])
def test_rns2mrns_and_sign_match_oracle_and_decrypt(slz, orc, toy, m, max_batch):
    import math
    from oracle import gadgets as gd
    p, keys = toy
    M = math.prod(m)
    vals = np.array([0, 1, -1, 99 % (M // 2), -(99 % (M // 2)), (M - 1) // 2, -(M // 2), 2, -2, 7, -7], dtype=np.int64)
    res = gd.rns_encode(vals, m)
    cts = orc.encrypt_messages(p, synth, keys.lwe_sk, res.reshape(-1).astype(np.uint64), offset=5000).reshape(len(m), len(vals), p.n + 1)
    ctx = slz.Context(p, max_batch)
    d_bsk = ctx.bsk_prepare(slz.to_device_u64(keys.bsk))
    d_ksk = slz.to_device_u64(keys.ksk)
    d_cts = slz.to_device_u64(cts)
    nzp = (-1, 0, 1)
    d_luts = slz.to_device_u64(slz.rns_luts(p, m, *nzp))
    # conversion: bit for bit against the oracle pipeline, and the digits are the number
    y = slz.to_host_u64(ctx.rns2mrns(d_cts, m, d_luts, d_bsk, d_ksk))
    assert np.array_equal(y, gd.rns2mrns_encrypted(p, cts, m, keys.bsk, keys.ksk))
    dec, _ = orc.decode(orc.lwe_phase(keys.lwe_sk, y.reshape(-1, p.n + 1)), p.msg_bits)
    digits = dec.reshape(len(m), -1).astype(np.int64)
    assert np.array_equal(digits, gd.rns2mrns_clear(res, m))
    assert np.array_equal(gd.mrns_value(digits, m), np.mod(vals, M))
    if m[-1] % 2 == 0:
        s = slz.to_host_u64(ctx.sign_rns(d_cts, m, d_luts, d_bsk, d_ksk))
        assert np.array_equal(s, gd.sign_rns_encrypted(p, cts, m, *nzp, keys.bsk, keys.ksk))
        dec, _ = orc.decode(orc.lwe_phase(keys.lwe_sk, s), p.msg_bits)
        assert np.array_equal(gd.signed_decode(dec.astype(np.int64), 256), np.sign(vals))


def test_sign_rns_rejects_an_odd_top_modulus(slz, toy):
    import ctypes
    p, keys = toy
    ctx = slz.Context(p, 8)
    L = slz.lib()
    sh = slz.make_rns_shape((14, 15), 4)
    need = ctypes.c_size_t(0)
    assert L.slz_rns_workspace(ctx._h, ctypes.byref(sh), ctypes.byref(need)) == 0
    buf = torch.zeros(need.value, dtype=torch.uint8, device="cuda")
    ptr = buf.data_ptr()
    assert L.slz_sign_rns(ctx._h, ctypes.byref(sh), ptr, ptr, ptr, ptr, ptr, ptr, need.value, None) == slz.SLZ_E_INVALID_ARG
    bad = slz.make_rns_shape((6, 15), 4)
    assert L.slz_rns_workspace(ctx._h, ctypes.byref(bad), ctypes.byref(need)) == slz.SLZ_E_INVALID_ARG


@pytest.mark.parametrize("m,gamma,max_batch", [((13, 15, 14), 5, 64), ((15, 14), 7, 5), ((7, 11, 13, 15, 8), 6, 256)])
def test_shift2msbs_matches_oracle_and_decrypts(slz, orc, toy, m, gamma, max_batch):
    import math
    from oracle import gadgets as gd
    p, keys = toy
    M, w = math.prod(m), 4
    # non-negative inputs: the printed example's three numbers (reduced into the base's positive range) and edge cases
    vals = np.array([2 * 13 + 3 * 195, 2 + 12 * 13 + 195, 6 + 13, 1000, 3, 0, (M - 1) // 2], dtype=np.int64) % (M // 2)
    ctx = slz.Context(p, max_batch)
    d_bsk = ctx.bsk_prepare(slz.to_device_u64(keys.bsk))
    d_ksk = slz.to_device_u64(keys.ksk)
    d_luts = slz.to_device_u64(slz.shift2msbs_luts(p, m, w, gamma))

    def run(values, signed):
        res = gd.rns_encode(values, m)
        cts = orc.encrypt_messages(p, synth, keys.lwe_sk, res.reshape(-1).astype(np.uint64), offset=31337).reshape(len(m), len(values), p.n + 1)
        y, shift = ctx.shift2msbs(slz.to_device_u64(cts), m, w, gamma, d_luts, d_bsk, d_ksk, signed=signed)
        y, shift = slz.to_host_u64(y), slz.to_host_u64(shift)
        if signed:
            want_y, want_shift = gd.shift2msbs_pm_encrypted(p, cts, m, w, gamma + 1, keys.bsk, keys.ksk)
            clear_y, clear_shift = gd.shift2msbs_pm_clear(res, m, w, gamma + 1)
        else:
            want_y, want_shift = gd.shift2msbs_plus_encrypted(p, cts, m, w, gamma, keys.bsk, keys.ksk)
            clear_y, clear_shift = gd.shift2msbs_plus_clear(res, m, w, gamma)
        assert np.array_equal(y, want_y) and np.array_equal(shift, want_shift)          # bit for bit
        dec, _ = orc.decode(orc.lwe_phase(keys.lwe_sk, y), p.msg_bits)
        assert np.array_equal(gd.signed_decode(dec.astype(np.int64), 256), clear_y)
        dec, _ = orc.decode(orc.lwe_phase(keys.lwe_sk, shift[None]), p.msg_bits)
        assert int(gd.signed_decode(dec.astype(np.int64), 256)[0]) == clear_shift

    run(vals, signed=False)
    if m[-1] % 2 == 0:
        svals = vals * np.array([1, -1, 1, -1, -1, 1, -1])
        run(svals, signed=True)
