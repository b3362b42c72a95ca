"""The keyswitch entry point that allocates nothing (scratch in a fixed device array of the library), through the C ABI:
bit for bit against slz_keyswitch_batch and the CPU oracle, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def slz():
    if not torch.cuda.is_available():
        pytest.fail("the gpu tests need a GPU: torch.cuda.is_available() is False")
    import paper_2504_17785_amd as m
    m.lib()
    return m


def test_static_scratch_keyswitch_matches_the_allocating_entry_point(slz, orc):
    p = synth.CONFIGS[2]                      # kN = 2048 -> n = 742, base 2^3, 5 levels: the matrix-core keyswitch
    kN = p.k * p.N
    ksk = synth.raw_words(p, "raw_ksk", kN * p.ks_level * (p.n + 1)).reshape(kN, p.ks_level, p.n + 1)
    d_ksk = slz.to_device_u64(ksk)
    ctx = slz.Context(p, 200)
    first = None
    for batch, offset in ((200, 0), (70, 1 << 20)):     # seven tiles (the last ragged), then three
        cts = synth.raw_words(p, "raw_ct", batch * (kN + 1), offset=offset).reshape(batch, kN + 1)
        d_cts = slz.to_device_u64(cts)
        out = torch.full((batch, p.n + 1), -1, dtype=torch.int64, device="cuda")
        ctx.keyswitch_batch_static(d_cts, d_ksk, out)
        got = slz.to_host_u64(out)
        want = slz.to_host_u64(ctx.keyswitch_batch(d_cts, d_ksk))
        assert np.array_equal(got, want), batch
        idx = np.array([0, batch // 2, batch - 1])
        assert np.array_equal(got[idx], orc.keyswitch_batch(p, cts[idx], ksk)), batch
        if first is None:
            first = (d_cts, got)
    # the first input once more: the smaller call in between has left nothing behind that is read
    out = torch.empty((200, p.n + 1), dtype=torch.int64, device="cuda")
    ctx.keyswitch_batch_static(first[0], d_ksk, out)
    assert np.array_equal(slz.to_host_u64(out), first[1])


def test_static_scratch_keyswitch_limits(slz):
    p = synth.CONFIGS[2]
    kN = p.k * p.N
    ctx = slz.Context(p, 64)
    d_ksk = torch.zeros((kN, p.ks_level, p.n + 1), dtype=torch.int64, device="cuda")
    too_many = 1632 + 32                       # one tile past the 16 MiB array at this shape
    d_cts = torch.zeros((too_many, kN + 1), dtype=torch.int64, device="cuda")
    out = torch.empty((too_many, p.n + 1), dtype=torch.int64, device="cuda")
    with pytest.raises(slz.SlzError) as e:
        ctx.keyswitch_batch_static(d_cts, d_ksk, out)
    assert e.value.code == slz.SLZ_E_TOO_LARGE
    ctx.keyswitch_batch_static(d_cts[:1632], d_ksk, out[:1632])      # the largest batch that fits
    torch.cuda.synchronize()
    assert int(out[:1632, : p.n].abs().max()) == 0
    big_base = slz.Context(p.with_(ks_base_log=16, ks_level=2), 8)    # digits wider than a byte: no matrix-core path
    with pytest.raises(slz.SlzError) as e:
        big_base.keyswitch_batch_static(d_cts[:8], torch.zeros((kN, 2, p.n + 1), dtype=torch.int64, device="cuda"), out[:8])
    assert e.value.code == slz.SLZ_E_UNSUPPORTED
