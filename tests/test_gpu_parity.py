"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle, bit for bit, on the
same seeded keys and inputs.  All integer work: the bar is exact equality of every output word."""
import ctypes

import numpy as np
import pytest

import synth
from synth import Params

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def tiny(**kw):
    base = dict(name="tiny", n=10, k=1, N=64, pbs_base_log=8, pbs_level=2, ks_base_log=4, ks_level=3,
                msg_bits=2, sigma_lwe=2.0 ** -30, sigma_bsk=2.0 ** -50, batch=8, n_luts=2, seed=4242)
    base.update(kw)
    return Params(**base)


@pytest.fixture(scope="module")
def slz():
    if not torch.cuda.is_available():
        pytest.fail("the gpu tests need a GPU: torch.cuda.is_available() is False")
    import paper_2504_17785_amd as m
    m.lib()
    return m


class Case:
    """Keys, LUTs and input ciphertexts of one parameter set, on host (oracle side) and device."""

    def __init__(self, slz, orc, p, batch, n_tables=2, msgs=None, raw_inputs=False, force_generic=False):
        self.p, self.batch = p, batch
        self.keys = orc.Keys(p, synth)
        self.tables = synth.random_tables(p, n_tables)
        self.luts = orc.lut_encode(p, self.tables)
        self.lut_idx = synth.uniform_below(p.seed, "lut_idx", batch, n_tables).astype(np.uint32)
        if raw_inputs:
            self.msgs = None
            self.cts = synth.raw_words(p, "raw_ct", batch * (p.n + 1)).reshape(batch, p.n + 1)
        else:
            self.msgs = synth.messages(p, batch) if msgs is None else np.asarray(msgs, dtype=np.uint64)
            self.cts = orc.encrypt_messages(p, synth, self.keys.lwe_sk, self.msgs)
        self.ctx = slz.Context(p, batch)
        if force_generic:
            self.ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
        self.d_bsk = self.ctx.bsk_prepare(slz.to_device_u64(self.keys.bsk))
        self.d_ksk = slz.to_device_u64(self.keys.ksk)
        self.d_luts = slz.to_device_u64(self.luts)
        self.d_idx = torch.from_numpy(self.lut_idx.astype(np.int32)).cuda()
        self.d_cts = slz.to_device_u64(self.cts)


SHAPES = [
    dict(n=6, N=8, k=1, pbs_base_log=8, pbs_level=2),
    dict(n=7, N=16, k=2, pbs_base_log=6, pbs_level=3),
    dict(n=10, N=64, k=1, pbs_base_log=23, pbs_level=1),
    dict(n=5, N=256, k=1, pbs_base_log=12, pbs_level=2),
    dict(n=4, N=1024, k=3, pbs_base_log=15, pbs_level=1),
    dict(n=3, N=2048, k=1, pbs_base_log=23, pbs_level=1),
    dict(n=3, N=4096, k=1, pbs_base_log=11, pbs_level=2),     # larger than one LDS chunk: HBM stages
    dict(n=2, N=8192, k=1, pbs_base_log=15, pbs_level=2),
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "N%d_k%d_l%d" % (s["N"], s["k"], s["pbs_level"]))
def test_blind_rotation_states_match_oracle(slz, orc, shape):
    p = tiny(**shape)
    batch = 5
    case = Case(slz, orc, p, batch, raw_inputs=True, force_generic=True)
    for steps in sorted({0, 1, 2, p.n}):
        want = orc.blind_rotate_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk, steps)
        got = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk, steps))
        assert np.array_equal(got, want), "accumulators differ after %d steps" % steps
    want = orc.pbs_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk)
    got = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    assert np.array_equal(got, want)
    # lut_idx == NULL: every ciphertext uses LUT 0
    want0 = orc.pbs_batch(p, case.cts, case.luts, None, case.keys.bsk)
    got0 = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, None, case.d_bsk))
    assert np.array_equal(got0, want0)


def test_worst_case_magnitudes_stay_exact(slz, orc):
    # key words and accumulator words at the extremes of the signed range, digits at +-B/2: the largest
    # sums the exactness bound allows for this shape
    p = tiny(n=3, N=2048, k=1, pbs_base_log=23, pbs_level=1)
    case = Case(slz, orc, p, 3, raw_inputs=True, force_generic=True)
    bsk = case.keys.bsk.copy()
    flat = bsk.reshape(-1)
    flat[0::3] = np.uint64(1 << 63)                       # -2^63
    flat[1::3] = np.uint64((1 << 63) - 1)                 # 2^63 - 1
    luts = case.luts.copy()
    luts[:, 0::2] = np.uint64((1 << 63) - (1 << 40))      # decomposes to digit +-2^22
    luts[:, 1::2] = np.uint64(1 << 63)
    d_bsk = case.ctx.bsk_prepare(slz.to_device_u64(bsk))
    want = orc.blind_rotate_batch(p, case.cts, luts, case.lut_idx, bsk, p.n)
    got = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, slz.to_device_u64(luts), case.d_idx, d_bsk, p.n))
    assert np.array_equal(got, want)


@pytest.mark.parametrize("batch,kN,n,beta,l", [(1, 64, 10, 4, 3), (13, 128, 33, 3, 5), (8, 256, 255, 2, 8),
                                               (37, 2048, 742, 3, 5), (3, 32, 300, 5, 2), (5, 64, 20, 12, 5), (21, 16, 9, 4, 4)])
def test_keyswitch_matches_oracle(slz, orc, batch, kN, n, beta, l):
    p = tiny(n=n, N=kN, k=1, ks_base_log=beta, ks_level=l)
    ksk = synth.raw_words(p, "raw_ksk", kN * l * (n + 1)).reshape(kN, l, n + 1)
    cts = synth.raw_words(p, "raw_ct", batch * (kN + 1)).reshape(batch, kN + 1)
    ctx = slz.Context(p, batch)
    got = slz.to_host_u64(ctx.keyswitch_batch(slz.to_device_u64(cts), slz.to_device_u64(ksk)))
    assert np.array_equal(got, orc.keyswitch_batch(p, cts, ksk))


@pytest.mark.parametrize("batch,k,N,n,beta,l", [(16, 1, 32, 5, 8, 8), (300, 3, 32, 100, 1, 7), (65, 1, 512, 31, 7, 9),
                                                 (257, 1, 256, 32, 4, 16), (1024, 1, 1024, 63, 2, 3), (33, 2, 64, 64, 6, 1)])
def test_matrix_core_keyswitch_matches_oracle_and_scalar_path(slz, orc, batch, k, N, n, beta, l):
    # digits of at most a byte and 16 or more ciphertexts: the int8 matrix-core contraction.  Ragged ciphertext tiles,
    # ragged output-word tiles, several workgroup groups, 64-bit decompositions, k > 1.
    p = tiny(n=n, N=N, k=k, ks_base_log=beta, ks_level=l)
    kN = k * N
    ksk = synth.raw_words(p, "raw_ksk", kN * l * (n + 1)).reshape(kN, l, n + 1)
    cts = synth.raw_words(p, "raw_ct", batch * (kN + 1)).reshape(batch, kN + 1)
    want = orc.keyswitch_batch(p, cts, ksk)
    d_cts, d_ksk = slz.to_device_u64(cts), slz.to_device_u64(ksk)
    ctx = slz.Context(p, batch)
    assert np.array_equal(slz.to_host_u64(ctx.keyswitch_batch(d_cts, d_ksk)), want)
    ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
    assert np.array_equal(slz.to_host_u64(ctx.keyswitch_batch(d_cts, d_ksk)), want)
    # a context made for fewer ciphertexts takes the batch in chunks
    ctx_small = slz.Context(p, 40)
    assert np.array_equal(slz.to_host_u64(ctx_small.keyswitch_batch(d_cts, d_ksk)), want)


def test_matrix_core_keyswitch_extreme_bytes_and_digits(slz, orc):
    # key words whose bytes sit at the edges of the signed-byte recoding (0x7f / 0x80 / 0xff / 0x00 with and without carry
    # into the next byte) against mask words whose digits are all -B/2, all B/2 - 1, or carry through every level
    p = tiny(n=70, N=256, k=1, ks_base_log=8, ks_level=8)
    kN, l, n, batch = 256, 8, 70, 48
    pats = np.array([0x8080808080808080, 0x7f7f7f7f7f7f7f7f, 0xffffffffffffffff, 0x0000000000000000, 0x807f807f807f807f,
                     0x7f807f807f807f80, 0xff7fff80007f0080, 0x0100000000000080], dtype=np.uint64)
    ksk = pats[(np.arange(kN * l * (n + 1)) * 5 // 3) % len(pats)].reshape(kN, l, n + 1)
    cts = pats[(np.arange(batch * (kN + 1)) // 7) % len(pats)].reshape(batch, kN + 1)
    cts[0, :] = np.uint64(0x8080808080808080)
    cts[1, :] = np.uint64(0x7f7f7f7f7f7f7f7f)
    ksk[:, :, 0] = np.uint64(0x8080808080808080)
    ksk[:, :, 1] = np.uint64(0x7f7f7f7f7f7f7f7f)
    ctx = slz.Context(p, batch)
    got = slz.to_host_u64(ctx.keyswitch_batch(slz.to_device_u64(cts), slz.to_device_u64(ksk)))
    assert np.array_equal(got, orc.keyswitch_batch(p, cts, ksk))


@pytest.mark.parametrize("batch,k,N,n,beta,l", [(16, 1, 32, 5, 8, 8), (300, 3, 32, 100, 1, 7), (65, 1, 512, 31, 7, 9),
                                                 (257, 1, 256, 32, 4, 16), (1024, 1, 1024, 63, 2, 3), (33, 2, 64, 64, 6, 1),
                                                 (1, 1, 64, 10, 4, 3), (37, 1, 2048, 742, 3, 5), (70, 3, 32, 40, 3, 5)])
def test_keyswitch_with_prepared_key_matches_oracle(slz, orc, batch, k, N, n, beta, l):
    # the key recoded once into the contraction's operands: row-block counts that are and are not multiples of eight
    # (the prepared key is zero-padded), ragged word and ciphertext tiles, one ciphertext, chunks of a smaller context
    p = tiny(n=n, N=N, k=k, ks_base_log=beta, ks_level=l)
    kN = k * N
    ksk = synth.raw_words(p, "raw_ksk", kN * l * (n + 1)).reshape(kN, l, n + 1)
    cts = synth.raw_words(p, "raw_ct", batch * (kN + 1)).reshape(batch, kN + 1)
    want = orc.keyswitch_batch(p, cts, ksk)
    d_cts, d_ksk = slz.to_device_u64(cts), slz.to_device_u64(ksk)
    ctx = slz.Context(p, batch)
    kskp = ctx.ksk_prepare(d_ksk)
    assert kskp.numel() == ctx.ksk_prepared_bytes() and ctx.ksk_prepared_bytes() % 8192 == 0
    got = ctx.keyswitch_batch_prepared(d_cts, kskp)
    assert np.array_equal(slz.to_host_u64(got), want)
    assert torch.equal(got, ctx.keyswitch_batch(d_cts, d_ksk))
    ctx_small = slz.Context(p, 40)
    assert np.array_equal(slz.to_host_u64(ctx_small.keyswitch_batch_prepared(d_cts, kskp)), want)


def test_keyswitch_with_prepared_key_extreme_bytes_and_errors(slz, orc):
    p = tiny(n=70, N=256, k=1, ks_base_log=8, ks_level=8)
    kN, l, n, batch = 256, 8, 70, 48
    pats = np.array([0x8080808080808080, 0x7f7f7f7f7f7f7f7f, 0xffffffffffffffff, 0x0000000000000000, 0x807f807f807f807f,
                     0x7f807f807f807f80, 0xff7fff80007f0080, 0x0100000000000080], dtype=np.uint64)
    ksk = pats[(np.arange(kN * l * (n + 1)) * 5 // 3) % len(pats)].reshape(kN, l, n + 1)
    cts = pats[(np.arange(batch * (kN + 1)) // 7) % len(pats)].reshape(batch, kN + 1)
    ksk[:, :, 0] = np.uint64(0x8080808080808080)
    ksk[:, :, 1] = np.uint64(0x7f7f7f7f7f7f7f7f)
    ctx = slz.Context(p, batch)
    d_cts, d_ksk = slz.to_device_u64(cts), slz.to_device_u64(ksk)
    kskp = ctx.ksk_prepare(d_ksk)
    assert np.array_equal(slz.to_host_u64(ctx.keyswitch_batch_prepared(d_cts, kskp)), orc.keyswitch_batch(p, cts, ksk))
    L = slz.lib()
    out = torch.zeros((batch, n + 1), dtype=torch.int64, device="cuda")
    import ctypes
    small = ctypes.c_size_t(ctx.ksk_prepared_bytes() - 1)
    assert L.slz_ksk_prepare(ctx._h, d_ksk.data_ptr(), kskp.data_ptr(), ctypes.byref(small), None) == slz.SLZ_E_INVALID_ARG
    assert L.slz_ksk_prepare(ctx._h, d_ksk.data_ptr(), kskp.data_ptr(), None, None) == slz.SLZ_E_INVALID_ARG
    assert L.slz_keyswitch_batch_prepared(ctx._h, d_cts.data_ptr(), None, out.data_ptr(), batch, None) == slz.SLZ_E_INVALID_ARG
    assert L.slz_keyswitch_batch_prepared(ctx._h, d_cts.data_ptr(), kskp.data_ptr() + 8, out.data_ptr(), batch, None) == slz.SLZ_E_INVALID_ARG
    assert L.slz_keyswitch_batch_prepared(ctx._h, d_cts.data_ptr(), kskp.data_ptr(), out.data_ptr(), 0, None) == slz.SLZ_E_INVALID_ARG
    # a keyswitch base above 2^8 has no matrix-core form
    wide = slz.Context(tiny(n=20, N=64, k=1, ks_base_log=12, ks_level=5), 4)
    need = ctypes.c_size_t(0)
    assert L.slz_ksk_prepare(wide._h, None, None, ctypes.byref(need), None) == slz.SLZ_E_UNSUPPORTED
    assert L.slz_keyswitch_batch_prepared(wide._h, d_cts.data_ptr(), kskp.data_ptr(), out.data_ptr(), 4, None) == slz.SLZ_E_UNSUPPORTED
    torch.cuda.synchronize()


def _lincomb_weights(p, J, O, kind):
    raw = synth.words(p.seed, "weights", J * O).view(np.int64)
    if kind == "small":          # residue-sized, as in the matmul gadget: one byte plane
        return (raw % 13).astype(np.int32).reshape(J, O)
    if kind == "int8":           # the whole signed-byte range, edges included
        w = (raw % 256 - 128).astype(np.int32)
        edge = np.array([-128, 127, 0, -1], dtype=np.int32)
        w[:len(edge)] = edge[:len(w)]
        return w.reshape(J, O)
    if kind == "int16":          # two or three byte planes
        return (raw % 65536 - 32768).astype(np.int32).reshape(J, O)
    w = (raw >> 32).astype(np.int32)                      # full int32 range: five byte planes
    edge = np.array([-2**31, 2**31 - 1, 0x7f7f7f7f, -0x7f7f7f80, 0x7fffff80, 128, -129, 0x00800000], dtype=np.int64).astype(np.int32)
    w[:len(edge)] = edge[:len(w)]
    return w.reshape(J, O)


@pytest.mark.parametrize("G,J,O,n,kind", [(5, 37, 19, 42, "small"), (2, 784, 128, 742, "small"), (3, 100, 33, 70, "int8"),
                                           (2, 65, 130, 31, "int16"), (2, 40, 257, 9, "int32"), (1, 1, 1, 5, "int32"),
                                           (4, 32, 64, 63, "int32")])
def test_lincomb_matches_oracle(slz, orc, G, J, O, n, kind):
    # ragged output tiles, ragged word tiles, ragged row blocks, 2/4/8-wave workgroups, one to five weight byte planes
    p = tiny(n=n)
    cts = synth.raw_words(p, "raw_ct", G * J * (n + 1)).reshape(G, J, n + 1)
    w = _lincomb_weights(p, J, O, kind)
    want = orc.lwe_lincomb_batch(cts, w)
    d_cts, d_w = slz.to_device_u64(cts), torch.from_numpy(w).cuda()
    ctx = slz.Context(p, 1)
    assert np.array_equal(slz.to_host_u64(ctx.lwe_lincomb_batch(d_cts, d_w)), want)
    # a second call on the same context with fewer byte planes must not see the first call's plane count
    w2 = _lincomb_weights(p, J, O, "small")
    assert np.array_equal(slz.to_host_u64(ctx.lwe_lincomb_batch(d_cts, torch.from_numpy(w2).cuda())), orc.lwe_lincomb_batch(cts, w2))
    ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)           # the scalar kernel
    assert np.array_equal(slz.to_host_u64(ctx.lwe_lincomb_batch(d_cts, d_w)), want)


def test_config1_full_pipeline_bit_exact_and_decrypts(slz, orc):
    p = synth.CONFIGS[1]
    case = Case(slz, orc, p, p.batch, n_tables=1, msgs=synth.config_messages(1))
    case.tables = synth.config_tables(1)
    case.luts = orc.lut_encode(p, case.tables)
    case.d_luts = slz.to_device_u64(slz.lut_encode(p, case.tables))
    big = case.ctx.pbs_batch(case.d_cts, case.d_luts, None, case.d_bsk)
    small = case.ctx.keyswitch_batch(big, case.d_ksk)
    want_big = orc.pbs_batch(p, case.cts, case.luts, None, case.keys.bsk)
    want_small = orc.keyswitch_batch(p, want_big, case.keys.ksk)
    assert np.array_equal(slz.to_host_u64(big), want_big)
    assert np.array_equal(slz.to_host_u64(small), want_small)
    got, err = orc.decode(orc.lwe_phase(case.keys.lwe_sk, slz.to_host_u64(small)), p.msg_bits)
    assert np.array_equal(got, case.tables[0][case.msgs.astype(np.int64)])
    assert np.abs(err).max() < 2.0 ** -6


def test_results_do_not_depend_on_batch_composition_or_repetition(slz, orc):
    p = tiny(n=12, N=512, pbs_base_log=8, pbs_level=2)
    case = Case(slz, orc, p, 9, raw_inputs=True)
    full = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    again = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    assert np.array_equal(full, again)
    perm = np.array([4, 0, 8, 2, 6, 1, 7, 3, 5])
    d_cts = slz.to_device_u64(case.cts[perm])
    d_idx = torch.from_numpy(case.lut_idx[perm].astype(np.int32)).cuda()
    shuffled = slz.to_host_u64(case.ctx.pbs_batch(d_cts, case.d_luts, d_idx, case.d_bsk))
    assert np.array_equal(shuffled, full[perm])
    part = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts[2:5].contiguous(), case.d_luts, case.d_idx[2:5].contiguous(), case.d_bsk))
    assert np.array_equal(part, full[2:5])


def test_error_codes(slz):
    L = slz.lib()
    p = tiny()
    h = ctypes.c_void_p()
    cp = slz.make_params(p)
    assert L.slz_ctx_create(ctypes.byref(cp), 0, ctypes.byref(h)) == -1                     # batch 0
    bad = slz.make_params(p.with_(pbs_base_log=33, pbs_level=2))
    assert L.slz_ctx_create(ctypes.byref(bad), 4, ctypes.byref(h)) == -1                    # base*level > 64
    big = slz.make_params(p.with_(N=2048, pbs_base_log=30, pbs_level=2))
    assert L.slz_ctx_create(ctypes.byref(big), 4, ctypes.byref(h)) == -2                    # exactness bound
    ctx = slz.Context(p, 4)
    x = torch.zeros(64, dtype=torch.int64, device="cuda")
    assert L.slz_pbs_batch(ctx._h, x.data_ptr(), x.data_ptr(), None, 1, x.data_ptr(), x.data_ptr(), 5, None) == -5
    assert L.slz_pbs_batch(ctx._h, x.data_ptr(), x.data_ptr(), None, 1, x.data_ptr(), x.data_ptr(), 0, None) == -1
    # ciphertext arrays need word alignment (any sub-batch of an array is a valid argument), tables and keys 16 bytes
    assert L.slz_pbs_batch(ctx._h, x.data_ptr() + 4, x.data_ptr(), None, 1, x.data_ptr(), x.data_ptr(), 1, None) == -1
    assert L.slz_pbs_batch(ctx._h, x.data_ptr(), x.data_ptr() + 8, None, 1, x.data_ptr(), x.data_ptr(), 1, None) == -1
    assert L.slz_pbs_batch(ctx._h, x.data_ptr(), x.data_ptr(), None, 1, x.data_ptr() + 8, x.data_ptr(), 1, None) == -1
    assert L.slz_blind_rotate_batch(ctx._h, x.data_ptr(), x.data_ptr(), None, 1, x.data_ptr(), p.n + 1, x.data_ptr(), 1, None) == -1
    need = ctypes.c_size_t(0)
    assert L.slz_bsk_prepare(ctx._h, None, None, ctypes.byref(need), None) == 0
    assert need.value == p.n * 2 * 2 * p.pbs_level * 2 * p.N * 8
    short = ctypes.c_size_t(need.value - 8)
    assert L.slz_bsk_prepare(ctx._h, x.data_ptr(), x.data_ptr(), ctypes.byref(short), None) == -1
    torch.cuda.synchronize()


def test_binding_rejects_wrong_sizes_on_the_host(slz, orc):
    # a tensor of the wrong width or a short output is a Python error before any kernel sees the pointer
    p = tiny()
    case = Case(slz, orc, p, 4)
    c = case.ctx
    with pytest.raises(ValueError):
        c.pbs_batch(case.d_cts[:, :-1].contiguous(), case.d_luts, case.d_idx, case.d_bsk)
    with pytest.raises(ValueError):
        c.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk, out=torch.empty((3, p.k * p.N + 1), dtype=torch.int64, device="cuda"))
    with pytest.raises(ValueError):
        c.pbs_batch(case.d_cts, case.d_luts.reshape(-1)[:-1], case.d_idx, case.d_bsk)
    with pytest.raises(ValueError):
        c.pbs_batch(case.d_cts, case.d_luts, case.d_idx[:2], case.d_bsk)
    with pytest.raises(ValueError):
        c.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk[:-1])
    with pytest.raises(ValueError):
        c.blind_rotate_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk, p.n + 1)
    big = c.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)
    with pytest.raises(ValueError):
        c.keyswitch_batch(big, case.d_ksk.reshape(-1)[:-1])
    with pytest.raises(ValueError):
        c.keyswitch_batch(big[:, :-1].contiguous(), case.d_ksk)
    with pytest.raises(ValueError):
        c.ks_pbs_batch(case.d_cts, case.d_ksk, case.d_luts, case.d_idx, case.d_bsk)      # small ciphertexts where big ones belong
    with pytest.raises(ValueError):
        c.bsk_prepare(slz.to_device_u64(case.keys.bsk.reshape(-1)[:-1]))
    with pytest.raises(ValueError):
        c.lwe_lincomb_batch(case.d_cts.reshape(1, 4, p.n + 1), torch.zeros((3, 2), dtype=torch.int32, device="cuda"))
    assert np.array_equal(slz.to_host_u64(c.keyswitch_batch(big, case.d_ksk)),
                          orc.keyswitch_batch(p, slz.to_host_u64(big), case.keys.ksk))


@pytest.mark.parametrize("shape", [dict(n=3, N=256, k=1, pbs_base_log=12, pbs_level=2),        # generic path: four buffers
                                   dict(n=2, N=4096, k=1, pbs_base_log=11, pbs_level=2)],      # large-N path: three
                         ids=["generic", "large_n"])
def test_out_of_memory_in_scratch_allocation_leaves_the_context_usable(slz, orc, shape):
    # the n-th scratch allocation of a first call fails (forced from the host, no device involved): the call reports
    # SLZ_E_NOMEM, keeps nothing half-allocated, and the next call on the same context allocates everything and is exact
    p = tiny(**shape)
    case = Case(slz, orc, p, 3, raw_inputs=True)
    if shape["N"] == 4096:
        case.ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 0)
        assert case.ctx.path in ("three_pass_large_n", "fused_n4096")
    want = orc.pbs_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk)
    for nth in (2, 1, 0):
        case.ctx.set_option(slz.SLZ_OPT_FAIL_ALLOC_AFTER, nth)
        with pytest.raises(slz.SlzError) as e:
            case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)
        assert e.value.code == slz.SLZ_E_NOMEM
    case.ctx.set_option(slz.SLZ_OPT_FAIL_ALLOC_AFTER, -1)
    got = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    assert np.array_equal(got, want)
    # the keyswitch scratch and the keyswitch-first buffer go through the same allocator
    p2 = tiny(n=20, N=64, k=1, ks_base_log=4, ks_level=3)
    case2 = Case(slz, orc, p2, 16, raw_inputs=True)
    big = case2.ctx.pbs_batch(case2.d_cts, case2.d_luts, case2.d_idx, case2.d_bsk)
    case2.ctx.set_option(slz.SLZ_OPT_FAIL_ALLOC_AFTER, 0)
    with pytest.raises(slz.SlzError) as e:
        case2.ctx.keyswitch_batch(big, case2.d_ksk)
    assert e.value.code == slz.SLZ_E_NOMEM
    small = slz.to_host_u64(case2.ctx.keyswitch_batch(big, case2.d_ksk))
    assert np.array_equal(small, orc.keyswitch_batch(p2, slz.to_host_u64(big), case2.keys.ksk))


# ---------------------------------------------------------------- fused kernel (N = 2048, k = 1, l = 1, base 2^23)

def _fused_case(slz, orc, n, batch, **kw):
    p = synth.CONFIGS[2].with_(n=n, name="cfg2_n%d" % n, **kw)
    case = Case(slz, orc, p, batch, n_tables=3, raw_inputs=True)
    assert case.ctx.path == "fused_n2048"
    return p, case


def test_fused_blind_rotation_states_match_oracle(slz, orc):
    p, case = _fused_case(slz, orc, 6, 5)
    for steps in (0, 1, 2, 3, p.n):
        want = orc.blind_rotate_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk, steps)
        got = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk, steps))
        assert np.array_equal(got, want), "accumulators differ after %d steps" % steps
    want = orc.pbs_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk)
    got = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    assert np.array_equal(got, want)
    got0 = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, None, case.d_bsk))
    assert np.array_equal(got0, orc.pbs_batch(p, case.cts, case.luts, None, case.keys.bsk))


def test_fused_rotation_amounts_cover_every_wrap_case(slz, orc):
    # a~ = 0, 1, N-1, N, N+1, 2N-1 and lane/register boundaries, for the body rotation and the step rotations
    p, case = _fused_case(slz, orc, 2, 12)
    N = p.N
    amounts = [0, 1, 63, 64, 1023, 1024, N - 1, N, N + 1, N + 1025, 2 * N - 64, 2 * N - 1]
    cts = case.cts.copy()
    for c, a in enumerate(amounts):
        cts[c, 0] = np.uint64(a << (64 - 12))
        cts[c, 1] = np.uint64(amounts[(c + 5) % 12] << (64 - 12))
        cts[c, 2] = np.uint64(amounts[(c + 7) % 12] << (64 - 12))     # body
    d_cts = slz.to_device_u64(cts)
    for steps in (0, 1, 2):
        want = orc.blind_rotate_batch(p, cts, case.luts, case.lut_idx, case.keys.bsk, steps)
        got = slz.to_host_u64(case.ctx.blind_rotate_batch(d_cts, case.d_luts, case.d_idx, case.d_bsk, steps))
        assert np.array_equal(got, want), "accumulators differ after %d steps" % steps


def test_fused_worst_case_magnitudes_and_generic_agreement(slz, orc):
    p, case = _fused_case(slz, orc, 4, 3)
    bsk = case.keys.bsk.copy()
    flat = bsk.reshape(-1)
    flat[0::3] = np.uint64(1 << 63)
    flat[1::3] = np.uint64((1 << 63) - 1)
    luts = case.luts.copy()
    luts[:, 0::2] = np.uint64((1 << 63) - (1 << 40))
    luts[:, 1::2] = np.uint64(1 << 63)
    d_bsk = case.ctx.bsk_prepare(slz.to_device_u64(bsk))
    d_luts = slz.to_device_u64(luts)
    want = orc.blind_rotate_batch(p, case.cts, luts, case.lut_idx, bsk, p.n)
    got = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, d_luts, case.d_idx, d_bsk, p.n))
    assert np.array_equal(got, want)
    case.ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
    gen = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, d_luts, case.d_idx, d_bsk, p.n))
    assert np.array_equal(gen, want)


def test_fused_other_gadget_bases(slz, orc):
    for beta in (8, 16, 21):
        p, case = _fused_case(slz, orc, 3, 4, pbs_base_log=beta)
        want = orc.pbs_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk)
        got = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
        assert np.array_equal(got, want), beta


def test_fused_more_ciphertexts_than_resident_workgroups(slz, orc):
    # 600 ciphertexts > 512 resident workgroups: some workgroups process two; compare the fused path with the
    # generic path on all, and with the oracle on a sample
    p, case = _fused_case(slz, orc, 3, 600)
    fused = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    case.ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
    gen = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    assert np.array_equal(fused, gen)
    idx = np.array([0, 1, 255, 511, 512, 513, 599])
    want = orc.pbs_batch(p, case.cts[idx], case.luts, case.lut_idx[idx], case.keys.bsk)
    assert np.array_equal(fused[idx], want)


def test_fused_pacing_between_ciphertexts_changes_nothing(slz, orc):
    # 1100 ciphertexts on 512 workgroups: three rounds, the last one ragged (76 workgroups).  Between rounds the workgroups wait
    # for each other (a timing hint with a bounded wait); with it off they run free.  Same bits either way, on repeated
    # launches (the arrival counters are cleared per launch), and with a batch that needs no pacing in between.
    p, case = _fused_case(slz, orc, 2, 1100)
    ctx = case.ctx
    paced = slz.to_host_u64(ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    small = slz.to_host_u64(ctx.pbs_batch(case.d_cts[:300], case.d_luts, case.d_idx[:300], case.d_bsk))
    again = slz.to_host_u64(ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    ctx.set_option(slz.SLZ_OPT_FUSED_PACING, 0)
    free = slz.to_host_u64(ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    assert np.array_equal(paced, free) and np.array_equal(again, free) and np.array_equal(small, free[:300])
    idx = np.array([0, 511, 512, 1023, 1024, 1099])
    assert np.array_equal(paced[idx], orc.pbs_batch(p, case.cts[idx], case.luts, case.lut_idx[idx], case.keys.bsk))
    # the give-up path: paced, but the first wait that is not satisfied at once switches the pacing off for the launch
    ctx.set_option(slz.SLZ_OPT_FUSED_PACING, 2)
    gave_up = slz.to_host_u64(ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    ctx.set_option(slz.SLZ_OPT_FUSED_PACING, 1)
    after = slz.to_host_u64(ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    assert np.array_equal(gave_up, free) and np.array_equal(after, free)
    with pytest.raises(slz.SlzError):
        ctx.set_option(slz.SLZ_OPT_FUSED_PACING, 3)
    with pytest.raises(slz.SlzError):
        slz.Context(tiny(), 4).set_option(slz.SLZ_OPT_FUSED_PACING, 1)      # not the N = 2048 fused path


# ---------------------------------------------------------------- fused kernel for N = 512 (k = 1 or 3, l = 1)

@pytest.mark.parametrize("k,beta", [(3, 18), (3, 7), (1, 23), (1, 10)])
def test_fused_n512_states_and_outputs_match_oracle(slz, orc, k, beta):
    p = tiny(n=4, N=512, k=k, pbs_base_log=beta, pbs_level=1)
    case = Case(slz, orc, p, 7, raw_inputs=True)
    assert case.ctx.path == "fused_n512"
    for steps in sorted({0, 1, 2, p.n}):
        want = orc.blind_rotate_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk, steps)
        got = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk, steps))
        assert np.array_equal(got, want), "accumulators differ after %d steps" % steps
    want = orc.pbs_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk)
    assert np.array_equal(slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)), want)
    want0 = orc.pbs_batch(p, case.cts, case.luts, None, case.keys.bsk)
    assert np.array_equal(slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, None, case.d_bsk)), want0)
    case.ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
    assert np.array_equal(slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)), want)


@pytest.mark.parametrize("k,beta", [(3, 24), (1, 25)])
def test_fused_n512_worst_case_and_many_ciphertexts(slz, orc, k, beta):
    # (k + 1) * 512 * 2^(beta - 1) * 2^63 = 2^97: the largest sums allowed
    p = tiny(n=3, N=512, k=k, pbs_base_log=beta, pbs_level=1, ks_base_log=4, ks_level=4, msg_bits=2, sigma_lwe=2.0 ** -30,
             sigma_bsk=2.0 ** -50)
    case = Case(slz, orc, p, 3, raw_inputs=True)
    assert case.ctx.path == "fused_n512"
    bsk = case.keys.bsk.copy()
    flat = bsk.reshape(-1)
    flat[0::3] = np.uint64(1 << 63)
    flat[1::3] = np.uint64((1 << 63) - 1)
    luts = case.luts.copy()
    luts[:, 0::2] = np.uint64((1 << 63) - (1 << (63 - beta)))
    luts[:, 1::2] = np.uint64(1 << 63)
    d_bsk = case.ctx.bsk_prepare(slz.to_device_u64(bsk))
    want = orc.blind_rotate_batch(p, case.cts, luts, case.lut_idx, bsk, p.n)
    got = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, slz.to_device_u64(luts), case.d_idx, d_bsk, p.n))
    assert np.array_equal(got, want)
    # 1100 real encryptions: more than the resident workgroups of either variant; decryption of all, oracle on a sample
    many = Case(slz, orc, p.with_(n=12, pbs_base_log=18), 1100)
    big = many.ctx.pbs_batch(many.d_cts, many.d_luts, many.d_idx, many.d_bsk)
    fused = slz.to_host_u64(big)
    small = slz.to_host_u64(many.ctx.keyswitch_batch(big, many.d_ksk))
    dec, _ = orc.decode(orc.lwe_phase(many.keys.lwe_sk, small), p.msg_bits)
    assert np.array_equal(dec, many.tables[many.lut_idx.astype(np.int64), many.msgs.astype(np.int64)])
    idx = np.array([0, 511, 512, 1023, 1024, 1099])
    assert np.array_equal(fused[idx], orc.pbs_batch(many.p, many.cts[idx], many.luts, many.lut_idx[idx], many.keys.bsk))
    many.ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
    assert np.array_equal(slz.to_host_u64(many.ctx.pbs_batch(many.d_cts, many.d_luts, many.d_idx, many.d_bsk)), fused)


@pytest.mark.parametrize("beta", [8, 12, 3])
def test_fused_n512_two_levels_states_and_outputs_match_oracle(slz, orc, beta):
    p = tiny(n=5, N=512, k=1, pbs_base_log=beta, pbs_level=2)
    case = Case(slz, orc, p, 7, raw_inputs=True)
    assert case.ctx.path == "fused_n512"
    for steps in sorted({0, 1, 2, p.n}):
        want = orc.blind_rotate_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk, steps)
        got = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk, steps))
        assert np.array_equal(got, want), "accumulators differ after %d steps" % steps
    want = orc.pbs_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk)
    assert np.array_equal(slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)), want)
    case.ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
    assert np.array_equal(slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)), want)


def test_fused_n512_two_levels_worst_case_and_many_ciphertexts(slz, orc):
    p = tiny(n=3, N=512, k=1, pbs_base_log=24, pbs_level=2)       # 4 * 512 * 2^23 * 2^63 = 2^97: the largest sums allowed
    case = Case(slz, orc, p, 3, raw_inputs=True)
    assert case.ctx.path == "fused_n512"
    bsk = case.keys.bsk.copy()
    flat = bsk.reshape(-1)
    flat[0::3] = np.uint64(1 << 63)
    flat[1::3] = np.uint64((1 << 63) - 1)
    luts = case.luts.copy()
    luts[:, 0::2] = np.uint64((1 << 63) - (1 << 15) - (1 << 39))  # both digits at -2^23 or 2^23 - 1
    luts[:, 1::2] = np.uint64(1 << 63)
    d_bsk = case.ctx.bsk_prepare(slz.to_device_u64(bsk))
    want = orc.blind_rotate_batch(p, case.cts, luts, case.lut_idx, bsk, p.n)
    got = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, slz.to_device_u64(luts), case.d_idx, d_bsk, p.n))
    assert np.array_equal(got, want)
    many = Case(slz, orc, tiny(n=4, N=512, k=1, pbs_base_log=8, pbs_level=2), 600, raw_inputs=True)
    fused = slz.to_host_u64(many.ctx.pbs_batch(many.d_cts, many.d_luts, many.d_idx, many.d_bsk))
    idx = np.array([0, 511, 512, 599])
    assert np.array_equal(fused[idx], orc.pbs_batch(many.p, many.cts[idx], many.luts, many.lut_idx[idx], many.keys.bsk))
    many.ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
    assert np.array_equal(slz.to_host_u64(many.ctx.pbs_batch(many.d_cts, many.d_luts, many.d_idx, many.d_bsk)), fused)


# ---------------------------------------------------------------- fused kernel for N = 1024 (k = 1, l = 1)

@pytest.mark.parametrize("beta", [23, 8, 16, 24])
def test_fused_n1024_states_and_outputs_match_oracle(slz, orc, beta):
    p = tiny(n=4, N=1024, k=1, pbs_base_log=beta, pbs_level=1)
    case = Case(slz, orc, p, 7, raw_inputs=True)
    assert case.ctx.path == "fused_n1024"
    for steps in sorted({0, 1, 2, p.n}):
        want = orc.blind_rotate_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk, steps)
        got = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk, steps))
        assert np.array_equal(got, want), "accumulators differ after %d steps" % steps
    want = orc.pbs_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk)
    assert np.array_equal(slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)), want)
    want0 = orc.pbs_batch(p, case.cts, case.luts, None, case.keys.bsk)
    assert np.array_equal(slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, None, case.d_bsk)), want0)
    case.ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
    assert case.ctx.path == "generic"
    assert np.array_equal(slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)), want)


def test_fused_n1024_worst_case_magnitudes(slz, orc):
    p = tiny(n=3, N=1024, k=1, pbs_base_log=24, pbs_level=1)      # 2 * 1024 * 2^23 * 2^63 = 2^97: the largest sums allowed
    case = Case(slz, orc, p, 3, raw_inputs=True)
    assert case.ctx.path == "fused_n1024"
    bsk = case.keys.bsk.copy()
    flat = bsk.reshape(-1)
    flat[0::3] = np.uint64(1 << 63)
    flat[1::3] = np.uint64((1 << 63) - 1)
    luts = case.luts.copy()
    luts[:, 0::2] = np.uint64((1 << 63) - (1 << 39))      # decomposes to digit +-2^23
    luts[:, 1::2] = np.uint64(1 << 63)
    d_bsk = case.ctx.bsk_prepare(slz.to_device_u64(bsk))
    want = orc.blind_rotate_batch(p, case.cts, luts, case.lut_idx, bsk, p.n)
    got = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, slz.to_device_u64(luts), case.d_idx, d_bsk, p.n))
    assert np.array_equal(got, want)


def test_fused_n1024_more_ciphertexts_than_resident_workgroups_and_decryption(slz, orc):
    # 600 ciphertexts > 512 resident workgroups; real encryptions: the whole batch decrypts to the tables
    p = tiny(n=16, N=1024, k=1, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=4, msg_bits=3, sigma_lwe=2.0 ** -30,
             sigma_bsk=2.0 ** -50)
    case = Case(slz, orc, p, 600)
    assert case.ctx.path == "fused_n1024"
    big = case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)
    fused = slz.to_host_u64(big)
    small = slz.to_host_u64(case.ctx.keyswitch_batch(big, case.d_ksk))
    got, _ = orc.decode(orc.lwe_phase(case.keys.lwe_sk, small), p.msg_bits)
    assert np.array_equal(got, case.tables[case.lut_idx.astype(np.int64), case.msgs.astype(np.int64)])
    idx = np.array([0, 1, 255, 511, 512, 513, 599])
    want = orc.pbs_batch(p, case.cts[idx], case.luts, case.lut_idx[idx], case.keys.bsk)
    assert np.array_equal(fused[idx], want)
    case.ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
    assert np.array_equal(slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)), fused)


@pytest.mark.parametrize("beta", [23, 9])
def test_fused_n1024_k2_states_and_outputs_match_oracle(slz, orc, beta):
    p = tiny(n=4, N=1024, k=2, pbs_base_log=beta, pbs_level=1)
    case = Case(slz, orc, p, 7, raw_inputs=True)
    assert case.ctx.path == "fused_n1024"
    for steps in sorted({0, 1, 2, p.n}):
        want = orc.blind_rotate_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk, steps)
        got = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk, steps))
        assert np.array_equal(got, want), "accumulators differ after %d steps" % steps
    want = orc.pbs_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk)
    assert np.array_equal(slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)), want)
    case.ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
    assert np.array_equal(slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)), want)


def test_fused_n1024_k2_worst_case_and_many_ciphertexts(slz, orc):
    p = tiny(n=3, N=1024, k=2, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=4, msg_bits=3, sigma_lwe=2.0 ** -30,
             sigma_bsk=2.0 ** -50)
    case = Case(slz, orc, p, 3, raw_inputs=True)
    assert case.ctx.path == "fused_n1024"
    bsk = case.keys.bsk.copy()
    flat = bsk.reshape(-1)
    flat[0::3] = np.uint64(1 << 63)
    flat[1::3] = np.uint64((1 << 63) - 1)
    luts = case.luts.copy()
    luts[:, 0::2] = np.uint64((1 << 63) - (1 << 40))
    luts[:, 1::2] = np.uint64(1 << 63)
    d_bsk = case.ctx.bsk_prepare(slz.to_device_u64(bsk))
    want = orc.blind_rotate_batch(p, case.cts, luts, case.lut_idx, bsk, p.n)
    got = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, slz.to_device_u64(luts), case.d_idx, d_bsk, p.n))
    assert np.array_equal(got, want)
    # 600 real encryptions > 512 resident workgroups: decryption of the whole batch, oracle on a sample, generic path on all
    many = Case(slz, orc, p.with_(n=12), 600)
    big = many.ctx.pbs_batch(many.d_cts, many.d_luts, many.d_idx, many.d_bsk)
    fused = slz.to_host_u64(big)
    small = slz.to_host_u64(many.ctx.keyswitch_batch(big, many.d_ksk))
    dec, _ = orc.decode(orc.lwe_phase(many.keys.lwe_sk, small), p.msg_bits)
    assert np.array_equal(dec, many.tables[many.lut_idx.astype(np.int64), many.msgs.astype(np.int64)])
    idx = np.array([0, 511, 512, 599])
    assert np.array_equal(fused[idx], orc.pbs_batch(many.p, many.cts[idx], many.luts, many.lut_idx[idx], many.keys.bsk))
    many.ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
    assert np.array_equal(slz.to_host_u64(many.ctx.pbs_batch(many.d_cts, many.d_luts, many.d_idx, many.d_bsk)), fused)


# ---------------------------------------------------------------- fused kernel for N = 4096 (k = 1, l = 1)

@pytest.mark.parametrize("beta", [22, 8, 16])
def test_fused_n4096_states_and_outputs_match_oracle(slz, orc, beta):
    p = tiny(n=3, N=4096, k=1, pbs_base_log=beta, pbs_level=1)
    case = Case(slz, orc, p, 5, raw_inputs=True)
    assert case.ctx.path == "fused_n4096"
    for steps in sorted({0, 1, 2, p.n}):
        want = orc.blind_rotate_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk, steps)
        got = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk, steps))
        assert np.array_equal(got, want), "accumulators differ after %d steps" % steps
    want = orc.pbs_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk)
    assert np.array_equal(slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)), want)
    want0 = orc.pbs_batch(p, case.cts, case.luts, None, case.keys.bsk)
    assert np.array_equal(slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, None, case.d_bsk)), want0)
    case.ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
    assert np.array_equal(slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)), want)


def test_fused_n4096_worst_case_magnitudes(slz, orc):
    p = tiny(n=2, N=4096, k=1, pbs_base_log=22, pbs_level=1)      # 2 * 4096 * 2^21 * 2^63 = 2^97: the largest sums allowed
    case = Case(slz, orc, p, 3, raw_inputs=True)
    assert case.ctx.path == "fused_n4096"
    bsk = case.keys.bsk.copy()
    flat = bsk.reshape(-1)
    flat[0::3] = np.uint64(1 << 63)
    flat[1::3] = np.uint64((1 << 63) - 1)
    luts = case.luts.copy()
    luts[:, 0::2] = np.uint64((1 << 63) - (1 << 41))      # decomposes to digit +-2^21
    luts[:, 1::2] = np.uint64(1 << 63)
    d_bsk = case.ctx.bsk_prepare(slz.to_device_u64(bsk))
    want = orc.blind_rotate_batch(p, case.cts, luts, case.lut_idx, bsk, p.n)
    got = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, slz.to_device_u64(luts), case.d_idx, d_bsk, p.n))
    assert np.array_equal(got, want)


def test_fused_n4096_more_ciphertexts_than_resident_workgroups(slz, orc):
    # 300 ciphertexts > 256 resident workgroups; all against the generic path, a sample against the oracle
    p = tiny(n=3, N=4096, k=1, pbs_base_log=22, pbs_level=1)
    case = Case(slz, orc, p, 300, raw_inputs=True)
    assert case.ctx.path == "fused_n4096"
    fused = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    idx = np.array([0, 1, 255, 256, 257, 299])
    want = orc.pbs_batch(p, case.cts[idx], case.luts, case.lut_idx[idx], case.keys.bsk)
    assert np.array_equal(fused[idx], want)
    case.ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
    assert np.array_equal(slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)), fused)


# ---------------------------------------------------------------- large-N three-pass path (N = 2048 G, k = 1)

@pytest.mark.parametrize("shape", [
    dict(n=3, N=4096, k=1, pbs_base_log=11, pbs_level=2),
    dict(n=3, N=8192, k=1, pbs_base_log=15, pbs_level=1),
    dict(n=2, N=16384, k=1, pbs_base_log=7, pbs_level=4),
    dict(n=2, N=32768, k=1, pbs_base_log=15, pbs_level=2),
], ids=lambda s: "N%d_l%d" % (s["N"], s["pbs_level"]))
@pytest.mark.parametrize("block", [1024, 2048])
def test_large_n_path_matches_oracle_and_generic(slz, orc, shape, block):
    p = tiny(**shape)
    batch = 5
    case = Case(slz, orc, p, batch, raw_inputs=True)
    assert case.ctx.path == "three_pass_large_n"
    case.ctx.set_option(slz.SLZ_OPT_LARGE_N_BLOCK, block)       # row pass on 1024-blocks (16 coefficients per lane) or 2048-blocks
    for steps in sorted({0, 1, p.n}):
        want = orc.blind_rotate_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk, steps)
        got = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk, steps))
        assert np.array_equal(got, want), "accumulators differ after %d steps" % steps
    want = orc.pbs_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk)
    got = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    assert np.array_equal(got, want)
    # five ciphertexts on 1024-blocks took the latency-oriented kernels (four launches per step); the same call on the
    # throughput kernels, after one more step count on them
    case.ctx.set_option(slz.SLZ_OPT_LARGE_N_LATENCY, 0)
    assert np.array_equal(slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)), want)
    one = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk, 1))
    assert np.array_equal(one, orc.blind_rotate_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk, 1))
    case.ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
    gen = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    assert np.array_equal(gen, want)


def test_large_n_latency_kernels_at_their_largest_batch_and_one_past_it(slz, orc):
    # N = 8192 on 1024-blocks: up to 1024 / 16 = 64 ciphertexts take the latency-oriented kernels (up to 16 with the row pass
    # in two launches, above that in one launch of one-component tasks), 65 the throughput ones; a ciphertext's result must
    # not depend on which
    p = tiny(n=2, N=8192, k=1, pbs_base_log=15, pbs_level=2)
    case = Case(slz, orc, p, 65, raw_inputs=True)
    assert case.ctx.path == "three_pass_large_n"
    all65 = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    for count in (64, 17, 16, 1):
        part = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts[:count], case.d_luts, case.d_idx[:count], case.d_bsk))
        assert np.array_equal(part, all65[:count]), count
    idx = np.array([0, 15, 16, 63, 64])
    assert np.array_equal(all65[idx], orc.pbs_batch(p, case.cts[idx], case.luts, case.lut_idx[idx], case.keys.bsk))
    with pytest.raises(slz.SlzError):
        case.ctx.set_option(slz.SLZ_OPT_LARGE_N_LATENCY, 2)


def test_large_n_path_takes_n2048_with_two_levels(slz, orc):
    # N = 2048 with more than one level has no fused kernel; it runs the large-N path as two 1024-blocks
    p = tiny(n=3, N=2048, k=1, pbs_base_log=12, pbs_level=2)
    case = Case(slz, orc, p, 5, raw_inputs=True)
    assert case.ctx.path == "three_pass_large_n"
    with pytest.raises(slz.SlzError):
        case.ctx.set_option(slz.SLZ_OPT_LARGE_N_BLOCK, 2048)    # a single 2048-block is not a large-N shape
    want = orc.pbs_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk)
    got = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    assert np.array_equal(got, want)
    case.ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
    assert np.array_equal(slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)), want)


@pytest.mark.parametrize("block", [1024, 2048])
def test_large_n_worst_case_magnitudes(slz, orc, block):
    p = tiny(n=2, N=8192, k=1, pbs_base_log=21, pbs_level=1)      # 2 * 8192 * 2^20 * 2^63 = 2^97: the largest sums allowed
    case = Case(slz, orc, p, 3, raw_inputs=True)
    assert case.ctx.path == "three_pass_large_n"
    case.ctx.set_option(slz.SLZ_OPT_LARGE_N_BLOCK, block)
    bsk = case.keys.bsk.copy()
    flat = bsk.reshape(-1)
    flat[0::3] = np.uint64(1 << 63)
    flat[1::3] = np.uint64((1 << 63) - 1)
    luts = case.luts.copy()
    luts[:, 0::2] = np.uint64((1 << 63) - (1 << 42))
    luts[:, 1::2] = np.uint64(1 << 63)
    d_bsk = case.ctx.bsk_prepare(slz.to_device_u64(bsk))
    want = orc.blind_rotate_batch(p, case.cts, luts, case.lut_idx, bsk, p.n)
    got = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, slz.to_device_u64(luts), case.d_idx, d_bsk, p.n))
    assert np.array_equal(got, want)
    case.ctx.set_option(slz.SLZ_OPT_LARGE_N_LATENCY, 0)           # three ciphertexts: the throughput kernels as well
    got = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, slz.to_device_u64(luts), case.d_idx, d_bsk, p.n))
    assert np.array_equal(got, want)


def test_largest_polynomial_size_matches_oracle(slz, orc):
    # N = 65536 = 32 blocks of 2048: the largest polynomial the library takes (the 11-bit lookups of the loss gadgets run at
    # it).  One oracle CMux of this size is 3.4e10 multiply-adds, so: two steps (the second one on dense accumulators),
    # three ciphertexts, uniform key words.
    p = tiny(n=2, N=65536, k=1, pbs_base_log=15, pbs_level=2, msg_bits=11)
    batch = 3
    R, C = (p.k + 1) * p.pbs_level, p.k + 1
    bsk = synth.raw_words(p, "raw_bsk", p.n * R * C * p.N).reshape(p.n, p.k + 1, p.pbs_level, C, p.N)
    cts = synth.raw_words(p, "raw_ct", batch * (p.n + 1)).reshape(batch, p.n + 1)
    luts = orc.lut_encode(p, synth.random_tables(p, 2))
    lut_idx = np.array([0, 1, 0], dtype=np.uint32)
    ctx = slz.Context(p, batch)
    assert ctx.path == "three_pass_large_n"
    d_bsk = ctx.bsk_prepare(slz.to_device_u64(bsk))
    d_cts, d_luts = slz.to_device_u64(cts), slz.to_device_u64(luts)
    d_idx = torch.from_numpy(lut_idx.astype(np.int32)).cuda()
    want = orc.blind_rotate_batch(p, cts, luts, lut_idx, bsk, 2)
    got = slz.to_host_u64(ctx.blind_rotate_batch(d_cts, d_luts, d_idx, d_bsk, 2))
    assert np.array_equal(got, want)
    big = slz.to_host_u64(ctx.pbs_batch(d_cts, d_luts, d_idx, d_bsk))
    assert np.array_equal(big, np.stack([orc.sample_extract(p, a) for a in want]))
    assert slz.Context(tiny(n=2, N=131072, k=1, pbs_base_log=15, pbs_level=2), 1).path == "generic"     # one size up


def test_large_n_two_lanes_match_one_lane_and_oracle(slz, orc):
    # 70 ciphertexts at N = 16384: chunks of 64 + 6 on two internal streams (the default) against one chunk at a time
    p = tiny(n=2, N=16384, k=1, pbs_base_log=15, pbs_level=1)
    case = Case(slz, orc, p, 70, raw_inputs=True)
    assert case.ctx.path == "three_pass_large_n"
    two = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    again = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    case.ctx.set_option(slz.SLZ_OPT_LARGE_N_LANES, 1)
    one = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))
    assert np.array_equal(two, one) and np.array_equal(again, one)
    idx = np.array([0, 63, 64, 69])
    want = orc.pbs_batch(p, case.cts[idx], case.luts, case.lut_idx[idx], case.keys.bsk)
    assert np.array_equal(two[idx], want)
    case.ctx.set_option(slz.SLZ_OPT_LARGE_N_LANES, 2)
    acc2 = slz.to_host_u64(case.ctx.blind_rotate_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk, 1))
    want_acc = orc.blind_rotate_batch(p, case.cts[idx], case.luts, case.lut_idx[idx], case.keys.bsk, 1)
    assert np.array_equal(acc2[idx], want_acc)
    with pytest.raises(slz.SlzError):
        case.ctx.set_option(slz.SLZ_OPT_LARGE_N_LANES, 3)


def test_work_is_enqueued_on_the_callers_stream(slz, orc):
    # a non-default torch stream: the library must launch on the hipStream_t it is given (same HIP runtime as torch)
    p, case = _fused_case(slz, orc, 3, 7)
    want = orc.pbs_batch(p, case.cts, case.luts, case.lut_idx, case.keys.bsk)
    want_small = orc.keyswitch_batch(p, want, case.keys.ksk)
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        big = case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)
        small = case.ctx.keyswitch_batch(big, case.d_ksk)
        case.ctx.set_option(slz.SLZ_OPT_FORCE_GENERIC, 1)
        big_gen = case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk)
    stream.synchronize()
    assert np.array_equal(slz.to_host_u64(big), want)
    assert np.array_equal(slz.to_host_u64(big_gen), want)
    assert np.array_equal(slz.to_host_u64(small), want_small)


# ---- keyswitch-first order -------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("shape,batch", [(dict(n=7, N=16, k=2, pbs_base_log=6, pbs_level=3), 5),
                                         (dict(n=5, N=2048, k=1, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8), 70),
                                         (dict(n=3, N=4096, k=1, pbs_base_log=11, pbs_level=2, ks_base_log=2, ks_level=9), 3)],
                         ids=["generic_k2", "fused_mfma_ks", "large_n"])
def test_keyswitch_first_order_matches_oracle(slz, orc, shape, batch):
    p = tiny(**shape)
    case = Case(slz, orc, p, batch, raw_inputs=True)
    big_in = synth.raw_words(p, "raw_ct", batch * (p.k * p.N + 1), offset=77).reshape(batch, p.k * p.N + 1)
    want = orc.pbs_batch(p, orc.keyswitch_batch(p, big_in, case.keys.ksk), case.luts, case.lut_idx, case.keys.bsk)
    d_in = slz.to_device_u64(big_in)
    got = case.ctx.ks_pbs_batch(d_in, case.d_ksk, case.d_luts, case.d_idx, case.d_bsk)
    assert np.array_equal(slz.to_host_u64(got), want)
    # identical to the two calls one after the other, and usable in place
    two = case.ctx.pbs_batch(case.ctx.keyswitch_batch(d_in, case.d_ksk), case.d_luts, case.d_idx, case.d_bsk)
    assert torch.equal(got, two)
    case.ctx.ks_pbs_batch(d_in, case.d_ksk, case.d_luts, case.d_idx, case.d_bsk, out=d_in)
    assert np.array_equal(slz.to_host_u64(d_in), want)
    # a smaller batch through the same scratch
    part = case.ctx.ks_pbs_batch(slz.to_device_u64(big_in[1:3]), case.d_ksk, case.d_luts, case.d_idx[1:3].contiguous(), case.d_bsk)
    assert np.array_equal(slz.to_host_u64(part), want[1:3])


def test_keyswitch_first_chain_decrypts_at_config1(slz, orc):
    """Two lookups in keyswitch-first order at a real parameter set: f, then g on the result, read under the big key."""
    p = synth.CONFIGS[1]
    case = Case(slz, orc, p, p.batch, n_tables=2, msgs=synth.config_messages(1))
    t = 1 << p.msg_bits
    first = slz.to_host_u64(case.ctx.pbs_batch(case.d_cts, case.d_luts, case.d_idx, case.d_bsk))       # brings the inputs under the big key
    chained = case.ctx.ks_pbs_batch(slz.to_device_u64(first), case.d_ksk, case.d_luts, case.d_idx, case.d_bsk)
    want = orc.pbs_batch(p, orc.keyswitch_batch(p, first, case.keys.ksk), case.luts, case.lut_idx, case.keys.bsk)
    assert np.array_equal(slz.to_host_u64(chained), want)
    got, err = orc.decode(orc.lwe_phase(case.keys.big_sk, want), p.msg_bits)
    idx = case.lut_idx.astype(np.int64)
    inner = case.tables[idx, case.msgs.astype(np.int64)].astype(np.int64) % t
    assert np.array_equal(got.astype(np.int64), case.tables[idx, inner].astype(np.int64))
    assert np.abs(err).max() < 2.0 ** -6


def test_keyswitch_first_error_codes(slz, orc):
    p = tiny(n=6, N=64, pbs_base_log=8, pbs_level=2)
    case = Case(slz, orc, p, 4, raw_inputs=True)
    L = slz.lib()
    big = torch.zeros((5, p.k * p.N + 1), dtype=torch.int64, device="cuda")
    b, k, l, q = big.data_ptr(), case.d_ksk.data_ptr(), case.d_luts.data_ptr(), case.d_bsk.data_ptr()
    call = lambda *a: L.slz_ks_pbs_batch(case.ctx._h, *a, None)
    assert call(b, k, l, None, 2, q, b, 5) == slz.SLZ_E_TOO_LARGE
    assert call(b, k, l, None, 2, q, b, 0) == slz.SLZ_E_INVALID_ARG
    assert call(b, k, l, None, 0, q, b, 4) == slz.SLZ_E_INVALID_ARG
    assert call(None, k, l, None, 2, q, b, 4) == slz.SLZ_E_INVALID_ARG
    assert call(b + 4, k, l, None, 2, q, b, 4) == slz.SLZ_E_INVALID_ARG
    assert call(b, k + 8, l, None, 2, q, b, 4) == slz.SLZ_E_INVALID_ARG
    torch.cuda.synchronize()


# ---- HIP graph capture -----------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("shape,batch", [(dict(n=5, N=2048, k=1, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8), 40),
                                         (dict(n=3, N=1024, k=1, pbs_base_log=23, pbs_level=1), 9),
                                         (dict(n=6, N=256, k=2, pbs_base_log=8, pbs_level=2), 7),
                                         (dict(n=2, N=16384, k=1, pbs_base_log=15, pbs_level=1), 70),
                                         (dict(n=2, N=2048, k=1, pbs_base_log=23, pbs_level=1, ks_base_log=4, ks_level=8), 1100),
                                         (dict(n=2, N=8192, k=1, pbs_base_log=15, pbs_level=2), 3)],
                         ids=["fused_n2048", "fused_n1024", "generic_k2", "large_n_two_lanes", "fused_n2048_paced_rounds",
                              "large_n_latency_kernels"])
def test_lookup_replays_from_a_hip_graph(slz, orc, shape, batch):
    """A serving loop captures one lookup (bootstrapping + keyswitch) once and replays it: after a warm-up call (which makes
    the library's lazy allocations) the calls record nothing but kernels and event edges, and every replay on new inputs
    matches the eager result."""
    p = tiny(**shape)
    case = Case(slz, orc, p, batch, raw_inputs=True)
    d_in = case.d_cts.clone()
    big = torch.empty((batch, p.k * p.N + 1), dtype=torch.int64, device="cuda")
    small = torch.empty((batch, p.n + 1), dtype=torch.int64, device="cuda")

    def lookup():
        case.ctx.pbs_batch(d_in, case.d_luts, case.d_idx, case.d_bsk, out=big)
        case.ctx.keyswitch_batch(big, case.d_ksk, out=small)

    lookup()                                             # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lookup()
    for rep in range(3):
        cts = synth.raw_words(p, "raw_ct", batch * (p.n + 1), offset=1000 * (rep + 1)).reshape(batch, p.n + 1)
        d_in.copy_(slz.to_device_u64(cts))
        big.zero_(); small.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got_big, got_small = slz.to_host_u64(big), slz.to_host_u64(small)
        lookup()                                         # the program's own eager work between replays
        torch.cuda.synchronize()
        assert np.array_equal(got_big, slz.to_host_u64(big)) and np.array_equal(got_small, slz.to_host_u64(small)), rep
        if rep == 0:
            idx = np.array([0, batch - 1])
            want = orc.pbs_batch(p, cts[idx], case.luts, case.lut_idx[idx], case.keys.bsk)
            assert np.array_equal(got_big[idx], want)
            assert np.array_equal(got_small[idx], orc.keyswitch_batch(p, want, case.keys.ksk))
