"""Seeded synthetic inputs shared by the tests, the CPU oracle's callers and bench.py.

This module holds NO arithmetic of the TFHE method itself: it only produces raw
randomness (secret-key bits, uniform mask words, rounded Gaussian noise integers,
messages, lookup tables, LUT indices, clear weights) as pure functions of
(config seed, stream name, index), plus the five parameter sets as plain data.
Encryption, key generation and every step of the bootstrapping live elsewhere
(the CPU oracle for the tests, the HIP library for the product) and take these
arrays as inputs, so both sides see identical bytes.

Generator: SplitMix64 in counter mode.  word(i) of a stream with key K is
mix64(K + (i+1) * 0x9E3779B97F4A7C15).  Stream keys are derived from the config
seed and a fixed stream id.  Gaussian noise is Box-Muller in double precision on
two 53-bit uniforms, scaled by sigma * 2^64 and rounded to the nearest integer.
"""
from __future__ import annotations

import dataclasses
import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

STREAMS = {
    "lwe_sk": 1, "glwe_sk": 2, "bsk_mask": 3, "bsk_noise": 4, "ksk_mask": 5,
    "ksk_noise": 6, "messages": 7, "ct_mask": 8, "ct_noise": 9, "lut_tables": 10,
    "lut_idx": 11, "weights": 12, "raw_bsk": 13, "raw_ksk": 14, "raw_ct": 15,
    "lin_inputs": 16, "lin_mask": 17, "lin_noise": 18, "misc": 19,
}


def _mix64(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def stream_key(seed: int, stream: str | int) -> np.uint64:
    sid = STREAMS[stream] if isinstance(stream, str) else int(stream)
    a = _mix64(np.uint64(seed & 0xFFFFFFFFFFFFFFFF))
    with np.errstate(over="ignore"):
        b = _mix64(np.uint64(sid) * _GOLDEN + np.uint64(0x1234567))
    return np.uint64(_mix64(a ^ b))


_CHUNK = 1 << 22      # large requests are generated in pieces of this many values on a few threads (counter mode:
_THREADS = 8          # the result does not depend on how the range is cut)


def _in_chunks(fn, count: int, dtype) -> np.ndarray:
    if count <= 2 * _CHUNK:
        return fn(0, count)
    import concurrent.futures
    out = np.empty(count, dtype=dtype)

    def piece(start):
        stop = min(count, start + _CHUNK)
        out[start:stop] = fn(start, stop - start)

    with concurrent.futures.ThreadPoolExecutor(_THREADS) as ex:
        list(ex.map(piece, range(0, count, _CHUNK)))
    return out


def _words(key: np.uint64, count: int, offset: int) -> np.ndarray:
    idx = np.arange(offset + 1, offset + count + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix64(key + idx * _GOLDEN)


def words(seed: int, stream: str | int, count: int, offset: int = 0) -> np.ndarray:
    """`count` uniform u64 words of the stream, starting at index `offset`."""
    key = stream_key(seed, stream)
    return _in_chunks(lambda start, cnt: _words(key, cnt, offset + start), count, np.uint64)


def bits(seed: int, stream: str | int, count: int, offset: int = 0) -> np.ndarray:
    """Uniform bits (one per generated word, taken from bit 63) as uint64 0/1."""
    return words(seed, stream, count, offset) >> np.uint64(63)


def uniform_below(seed: int, stream: str | int, count: int, bound: int, offset: int = 0) -> np.ndarray:
    """Uniform integers in [0, bound) for bound <= 2^32 (multiply-shift on the top 32 bits)."""
    assert 0 < bound <= (1 << 32)
    hi = words(seed, stream, count, offset) >> np.uint64(32)
    return ((hi * np.uint64(bound)) >> np.uint64(32)).astype(np.uint64)


def gaussian_ints(seed: int, stream: str | int, count: int, sigma: float, offset: int = 0) -> np.ndarray:
    """Rounded Gaussian noise on the 2^64 torus: round(z * sigma * 2^64) as int64 (two's complement)."""
    if sigma == 0.0:
        return np.zeros(count, dtype=np.int64)
    key = stream_key(seed, stream)

    def piece(start, cnt):
        w = _words(key, 2 * cnt, 2 * (offset + start))
        u1 = ((w[0::2] >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)  # (0,1]
        u2 = (w[1::2] >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)          # [0,1)
        z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        return np.rint(z * (sigma * 18446744073709551616.0)).astype(np.int64)

    return _in_chunks(piece, count, np.int64)


@dataclasses.dataclass(frozen=True)
class Params:
    """A TFHE parameter set (plain data).  One padding bit is implied: Delta = 2^(63 - msg_bits)."""
    name: str
    n: int            # small LWE dimension
    k: int            # GLWE dimension
    N: int            # polynomial size (power of two)
    pbs_base_log: int
    pbs_level: int
    ks_base_log: int
    ks_level: int
    msg_bits: int
    sigma_lwe: float  # noise of LWE encryptions and of the key-switching key (torus units)
    sigma_bsk: float  # noise of the bootstrapping key (GLWE)
    batch: int
    n_luts: int
    seed: int

    @property
    def delta(self) -> int:
        return 1 << (63 - self.msg_bits)

    @property
    def t(self) -> int:
        return 1 << self.msg_bits

    @property
    def big_n(self) -> int:
        return self.k * self.N

    def with_(self, **kw) -> "Params":
        return dataclasses.replace(self, **kw)


_SEED0 = 0x51E20000

# The five workloads, as parameter sets.  Where the configuration text is loose the
# reading is: config 1 keeps sigma = 2^-20 for LWE/KSK noise and uses 2^-40 for the
# bootstrapping key (2^-20 there gives blind-rotation noise above Delta/2); config 3
# uses sigma_lwe = 2^-24; configs 4 and 5 carry 4-bit messages.
CONFIGS = {
    1: Params("cfg1_tiny", 128, 1, 512, 8, 2, 4, 3, 3, 2.0 ** -20, 2.0 ** -40, 8, 1, _SEED0 + 1),
    2: Params("cfg2_n742_N2048", 742, 1, 2048, 23, 1, 3, 5, 3, 2.0 ** -17, 2.0 ** -51, 1024, 3, _SEED0 + 2),
    3: Params("cfg3_n1024_N32768", 1024, 1, 32768, 15, 2, 4, 5, 8, 2.0 ** -24, 2.0 ** -62, 256, 16, _SEED0 + 3),
    4: Params("cfg4_gadget", 742, 1, 2048, 23, 1, 3, 5, 4, 2.0 ** -17, 2.0 ** -51, 3 * 32 * 128, 3, _SEED0 + 4),
    5: Params("cfg5_batch16384", 742, 1, 2048, 23, 1, 3, 5, 4, 2.0 ** -17, 2.0 ** -51, 16384, 64, _SEED0 + 5),
}

CFG4_MODULI = (7, 11, 13)
CFG4_BATCH, CFG4_IN, CFG4_OUT = 32, 784, 128


# ---- raw material for keys and ciphertexts (arrays of randomness only) -------------------------

def lwe_secret(p: Params) -> np.ndarray:
    return bits(p.seed, "lwe_sk", p.n)


def glwe_secret(p: Params) -> np.ndarray:
    return bits(p.seed, "glwe_sk", p.k * p.N).reshape(p.k, p.N)


def bsk_randomness(p: Params):
    """Mask polynomials [n][k+1][l][k][N] (u64) and noise polynomials [n][k+1][l][N] (i64)."""
    rows = p.n * (p.k + 1) * p.pbs_level
    mask = words(p.seed, "bsk_mask", rows * p.k * p.N).reshape(p.n, p.k + 1, p.pbs_level, p.k, p.N)
    noise = gaussian_ints(p.seed, "bsk_noise", rows * p.N, p.sigma_bsk).reshape(p.n, p.k + 1, p.pbs_level, p.N)
    return mask, noise


def bsk_randomness_sparse(p: Params, nnz: int):
    """As bsk_randomness, but every mask polynomial has only `nnz` non-zero words (uniform words at seeded positions;
    positions may coincide).  A test device: a key built from it is a valid encryption of the same key bits with real
    noise, useless for security, and a schoolbook key generation costs nnz N instead of N^2 per row."""
    rows = p.n * (p.k + 1) * p.pbs_level
    polys = rows * p.k
    mask = np.zeros((polys, p.N), dtype=np.uint64)
    pos = uniform_below(p.seed, "misc", polys * nnz, p.N, offset=1 << 20).reshape(polys, nnz).astype(np.int64)
    val = words(p.seed, "bsk_mask", polys * nnz).reshape(polys, nnz)
    for q in range(nnz):
        mask[np.arange(polys), pos[:, q]] = val[:, q]
    noise = gaussian_ints(p.seed, "bsk_noise", rows * p.N, p.sigma_bsk).reshape(p.n, p.k + 1, p.pbs_level, p.N)
    return mask.reshape(p.n, p.k + 1, p.pbs_level, p.k, p.N), noise


def ksk_randomness(p: Params):
    """Mask words [kN][l_ks][n] (u64) and noise [kN][l_ks] (i64)."""
    rows = p.k * p.N * p.ks_level
    mask = words(p.seed, "ksk_mask", rows * p.n).reshape(p.k * p.N, p.ks_level, p.n)
    noise = gaussian_ints(p.seed, "ksk_noise", rows, p.sigma_lwe).reshape(p.k * p.N, p.ks_level)
    return mask, noise


def ct_randomness(p: Params, count: int, dim: int | None = None, sigma: float | None = None, offset: int = 0):
    """Mask words [count][dim] and noise [count] for fresh LWE encryptions (dim defaults to n)."""
    dim = p.n if dim is None else dim
    sigma = p.sigma_lwe if sigma is None else sigma
    mask = words(p.seed, "ct_mask", count * dim, offset * dim).reshape(count, dim)
    noise = gaussian_ints(p.seed, "ct_noise", count, sigma, offset)
    return mask, noise


def messages(p: Params, count: int, mode: str = "uniform") -> np.ndarray:
    if mode == "ramp":
        return (np.arange(count, dtype=np.uint64) % np.uint64(p.t)).astype(np.uint64)
    return uniform_below(p.seed, "messages", count, p.t)


def random_tables(p: Params, count: int, offset: int = 0) -> np.ndarray:
    """`count` seeded random maps Z_t -> Z_t as u64 [count][t]."""
    return uniform_below(p.seed, "lut_tables", count * p.t, p.t, offset * p.t).reshape(count, p.t)


def identity_table(p: Params) -> np.ndarray:
    return np.arange(p.t, dtype=np.uint64)


def relu_table(p: Params) -> np.ndarray:
    """ReLU under the signed encoding of Z_t (lower half non-negative, upper half negative)."""
    v = np.arange(p.t, dtype=np.uint64)
    return np.where(v < np.uint64(p.t // 2), v, np.uint64(0)).astype(np.uint64)


def mod_table(p: Params, r: int) -> np.ndarray:
    return (np.arange(p.t, dtype=np.uint64) % np.uint64(r)).astype(np.uint64)


def config_tables(cfg: int) -> np.ndarray:
    """The lookup tables of a configuration, u64 [n_luts][t]."""
    p = CONFIGS[cfg]
    if cfg == 1:
        return random_tables(p, 1)
    if cfg == 2:
        return np.stack([identity_table(p), relu_table(p), random_tables(p, 1)[0]])
    if cfg == 3:
        return random_tables(p, 16)
    if cfg == 4:
        return np.stack([mod_table(p, r) for r in CFG4_MODULI])
    if cfg == 5:
        return random_tables(p, 64)
    raise KeyError(cfg)


def config_lut_idx(cfg: int, count: int | None = None) -> np.ndarray:
    p = CONFIGS[cfg]
    count = p.batch if count is None else count
    if cfg == 1:
        return np.zeros(count, dtype=np.uint32)
    if cfg == 2:
        return (np.arange(count) % 3).astype(np.uint32)
    if cfg == 4:
        per = count // 3
        return np.repeat(np.arange(3, dtype=np.uint32), per)
    return uniform_below(p.seed, "lut_idx", count, p.n_luts).astype(np.uint32)


def config_messages(cfg: int, count: int | None = None) -> np.ndarray:
    p = CONFIGS[cfg]
    count = p.batch if count is None else count
    if cfg in (1, 3):
        return messages(p, count, "ramp")
    return messages(p, count)


def raw_words(p: Params, stream: str, count: int, offset: int = 0) -> np.ndarray:
    """Uniform words standing in for key or ciphertext material where only its distribution matters
    (throughput runs: TFHE keys and ciphertexts are uniform-looking u64 words)."""
    return words(p.seed, stream, count, offset)


def cfg4_clear_inputs():
    """Config 4 linear part: residues x[r][b][j] uniform in [0, m_r) and clear weights w[r][j][o] in [0, m_r)."""
    p = CONFIGS[4]
    xs, ws = [], []
    for i, r in enumerate(CFG4_MODULI):
        xs.append(uniform_below(p.seed, "lin_inputs", CFG4_BATCH * CFG4_IN, r, i * CFG4_BATCH * CFG4_IN)
                  .reshape(CFG4_BATCH, CFG4_IN))
        ws.append(uniform_below(p.seed, "weights", CFG4_IN * CFG4_OUT, r, i * CFG4_IN * CFG4_OUT)
                  .reshape(CFG4_IN, CFG4_OUT))
    return np.stack(xs), np.stack(ws).astype(np.int32)
