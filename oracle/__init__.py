"""ctypes front end of the CPU oracle (oracle/tfhe_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  The GPU library never imports this package and this package
never imports the GPU library.  Every function here marshals numpy arrays into the C oracle;
the arithmetic is all in the C file.  Randomness (key bits, masks, noise) is passed in.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tfhe_oracle.c")
_LIB = os.path.join(_HERE, "libtfhe_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over ciphertexts only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


class _P(ctypes.Structure):
    _fields_ = [(f, ctypes.c_uint32) for f in
                ("n", "k", "N", "pbs_base_log", "pbs_level", "ks_base_log", "ks_level", "msg_bits")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        # TFHE_ORACLE_LIB lets the mutation tests load a deliberately broken build of the oracle
        _lib = ctypes.CDLL(os.environ.get("TFHE_ORACLE_LIB") or build())
        _lib.orc_modswitch.restype = ctypes.c_uint32
        _lib.orc_modswitch.argtypes = [ctypes.c_uint64, ctypes.c_uint32]
        _lib.orc_lwe_phase.restype = ctypes.c_uint64
        _lib.orc_lut_encode.restype = ctypes.c_int
        _lib.orc_num_threads.restype = ctypes.c_int
    return _lib


def _cp(p) -> _P:
    return _P(p.n, p.k, p.N, p.pbs_base_log, p.pbs_level, p.ks_base_log, p.ks_level, p.msg_bits)


def _u64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint64)


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int64)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(lib().orc_num_threads())


# ---- ring and scalar steps ------------------------------------------------------------------

def negacyclic_mul(P, Q) -> np.ndarray:
    P, Q = _u64(P), _u64(Q)
    out = np.empty_like(P)
    lib().orc_negacyclic_mul(_ptr(P), _ptr(Q), ctypes.c_uint32(P.size), _ptr(out))
    return out


def monomial_mul(P, r: int) -> np.ndarray:
    P = _u64(P)
    out = np.empty_like(P)
    lib().orc_monomial_mul(_ptr(P), ctypes.c_uint32(P.size), ctypes.c_uint32(r), _ptr(out))
    return out


def decompose(x: int, beta: int, level: int) -> np.ndarray:
    d = np.zeros(level, dtype=np.int64)
    lib().orc_decompose(ctypes.c_uint64(int(x) & 0xFFFFFFFFFFFFFFFF), ctypes.c_uint32(beta),
                        ctypes.c_uint32(level), _ptr(d))
    return d


def modswitch(x: int, N: int) -> int:
    return int(lib().orc_modswitch(ctypes.c_uint64(int(x) & 0xFFFFFFFFFFFFFFFF), ctypes.c_uint32(N)))


def lut_encode(p, tables) -> np.ndarray:
    tables = _u64(tables).reshape(-1, p.t)
    out = np.empty((tables.shape[0], p.N), dtype=np.uint64)
    cp = _cp(p)
    rc = lib().orc_lut_encode(ctypes.byref(cp), _ptr(tables), ctypes.c_uint32(tables.shape[0]), _ptr(out))
    if rc != 0:
        raise ValueError("lut_encode: N must be at least 2t")
    return out


# ---- encryption / decryption / keys ---------------------------------------------------------

def lwe_encrypt(sk, mask, noise, pt) -> np.ndarray:
    """Batch of LWE encryptions: mask [count][dim], noise [count] (int64), pt [count] (u64 plaintexts)."""
    sk, mask, noise, pt = _u64(sk), _u64(mask), _i64(noise), _u64(pt)
    count, dim = mask.shape
    out = np.empty((count, dim + 1), dtype=np.uint64)
    L = lib()
    for c in range(count):
        L.orc_lwe_encrypt(_ptr(sk), ctypes.c_uint32(dim), _ptr(mask[c]), ctypes.c_int64(int(noise[c])),
                          ctypes.c_uint64(int(pt[c])), _ptr(out[c]))
    return out


def lwe_phase(sk, cts) -> np.ndarray:
    sk, cts = _u64(sk), _u64(cts)
    cts2 = cts.reshape(-1, cts.shape[-1])
    L = lib()
    out = np.array([L.orc_lwe_phase(_ptr(sk), ctypes.c_uint32(sk.size), _ptr(cts2[c]))
                    for c in range(cts2.shape[0])], dtype=np.uint64)
    return out.reshape(cts.shape[:-1])


def decode(phase, msg_bits: int):
    """Round a phase to the message grid with one padding bit: returns (m in Z_{2t}, noise as float torus units)."""
    phase = _u64(phase)
    shift = np.uint64(63 - msg_bits)
    delta = np.uint64(1) << shift
    with np.errstate(over="ignore"):
        m = ((phase + (delta >> np.uint64(1))) >> shift) & np.uint64((1 << (msg_bits + 1)) - 1)
        err = (phase - m * delta).astype(np.int64).astype(np.float64) / 18446744073709551616.0
    return m, err


def glwe_encrypt(sk, mask, noise, M) -> np.ndarray:
    sk, mask, noise, M = _u64(sk), _u64(mask), _i64(noise), _u64(M)
    k, N = sk.shape
    ct = np.empty((k + 1, N), dtype=np.uint64)
    lib().orc_glwe_encrypt(_ptr(sk), ctypes.c_uint32(k), ctypes.c_uint32(N), _ptr(mask), _ptr(noise), _ptr(M), _ptr(ct))
    return ct


def glwe_phase(sk, ct) -> np.ndarray:
    sk, ct = _u64(sk), _u64(ct)
    k, N = sk.shape
    ph = np.empty(N, dtype=np.uint64)
    lib().orc_glwe_phase(_ptr(sk), ctypes.c_uint32(k), ctypes.c_uint32(N), _ptr(ct), _ptr(ph))
    return ph


def bsk_gen(p, lwe_sk, glwe_sk, mask, noise) -> np.ndarray:
    lwe_sk, glwe_sk, mask, noise = _u64(lwe_sk), _u64(glwe_sk), _u64(mask), _i64(noise)
    bsk = np.empty((p.n, p.k + 1, p.pbs_level, p.k + 1, p.N), dtype=np.uint64)
    cp = _cp(p)
    lib().orc_bsk_gen(ctypes.byref(cp), _ptr(lwe_sk), _ptr(glwe_sk), _ptr(mask), _ptr(noise), _ptr(bsk))
    return bsk


def ksk_gen(p, big_sk, lwe_sk, mask, noise) -> np.ndarray:
    big_sk, lwe_sk, mask, noise = _u64(big_sk), _u64(lwe_sk), _u64(mask), _i64(noise)
    ksk = np.empty((p.k * p.N, p.ks_level, p.n + 1), dtype=np.uint64)
    cp = _cp(p)
    lib().orc_ksk_gen(ctypes.byref(cp), _ptr(big_sk), _ptr(lwe_sk), _ptr(mask), _ptr(noise), _ptr(ksk))
    return ksk


# ---- bootstrapping --------------------------------------------------------------------------

def cmux(p, acc, bsk_i, a_tilde: int) -> np.ndarray:
    acc = _u64(acc).copy()
    bsk_i = _u64(bsk_i)
    cp = _cp(p)
    lib().orc_cmux(ctypes.byref(cp), _ptr(acc), _ptr(bsk_i), ctypes.c_uint32(a_tilde))
    return acc


def _idx(lut_idx):
    if lut_idx is None:
        return None, None
    a = np.ascontiguousarray(lut_idx, dtype=np.uint32)
    return a, _ptr(a)


def blind_rotate_batch(p, lwe_in, luts, lut_idx, bsk, n_steps: int) -> np.ndarray:
    lwe_in, luts, bsk = _u64(lwe_in), _u64(luts), _u64(bsk)
    batch = lwe_in.shape[0]
    keep, ip = _idx(lut_idx)
    out = np.empty((batch, p.k + 1, p.N), dtype=np.uint64)
    cp = _cp(p)
    lib().orc_blind_rotate_batch(ctypes.byref(cp), _ptr(lwe_in), _ptr(luts), ip, _ptr(bsk),
                                 ctypes.c_uint32(n_steps), _ptr(out), ctypes.c_uint32(batch))
    return out


def sample_extract(p, acc) -> np.ndarray:
    acc = _u64(acc)
    out = np.empty(p.k * p.N + 1, dtype=np.uint64)
    cp = _cp(p)
    lib().orc_sample_extract(ctypes.byref(cp), _ptr(acc), _ptr(out))
    return out


def pbs_batch(p, lwe_in, luts, lut_idx, bsk) -> np.ndarray:
    lwe_in, luts, bsk = _u64(lwe_in), _u64(luts), _u64(bsk)
    batch = lwe_in.shape[0]
    keep, ip = _idx(lut_idx)
    out = np.empty((batch, p.k * p.N + 1), dtype=np.uint64)
    cp = _cp(p)
    lib().orc_pbs_batch(ctypes.byref(cp), _ptr(lwe_in), _ptr(luts), ip, _ptr(bsk), _ptr(out), ctypes.c_uint32(batch))
    return out


def keyswitch_batch(p, lwe_in, ksk) -> np.ndarray:
    lwe_in, ksk = _u64(lwe_in), _u64(ksk)
    batch = lwe_in.shape[0]
    out = np.empty((batch, p.n + 1), dtype=np.uint64)
    cp = _cp(p)
    lib().orc_keyswitch_batch(ctypes.byref(cp), _ptr(lwe_in), _ptr(ksk), _ptr(out), ctypes.c_uint32(batch))
    return out


def lwe_lincomb_batch(cts, w) -> np.ndarray:
    cts = _u64(cts)
    w = np.ascontiguousarray(w, dtype=np.int32)
    G, J, width = cts.shape
    O = w.shape[1]
    out = np.empty((G, O, width), dtype=np.uint64)
    lib().orc_lwe_lincomb_batch(_ptr(cts), _ptr(w), _ptr(out), ctypes.c_uint32(G), ctypes.c_uint32(J),
                                ctypes.c_uint32(O), ctypes.c_uint32(width))
    return out


# ---- convenience built only from the calls above ------------------------------------------------

class Keys:
    """Secret keys and public evaluation keys of one parameter set, generated from the seeded streams."""

    def __init__(self, p, synth, with_bsk=True, with_ksk=True, sigma_bsk=None, sigma_ksk=None):
        self.p = p
        self.lwe_sk = synth.lwe_secret(p)
        self.glwe_sk = synth.glwe_secret(p)
        self.big_sk = self.glwe_sk.reshape(-1)
        self.bsk = None
        self.ksk = None
        if with_bsk:
            pp = p if sigma_bsk is None else p.with_(sigma_bsk=sigma_bsk)
            mask, noise = synth.bsk_randomness(pp)
            self.bsk = bsk_gen(p, self.lwe_sk, self.glwe_sk, mask, noise)
        if with_ksk:
            pp = p if sigma_ksk is None else p.with_(sigma_lwe=sigma_ksk)
            mask, noise = synth.ksk_randomness(pp)
            self.ksk = ksk_gen(p, self.big_sk, self.lwe_sk, mask, noise)


def encrypt_messages(p, synth, lwe_sk, msgs, sigma=None, offset=0) -> np.ndarray:
    msgs = _u64(msgs)
    mask, noise = synth.ct_randomness(p, msgs.size, dim=len(lwe_sk), sigma=sigma, offset=offset)
    with np.errstate(over="ignore"):
        pt = msgs * np.uint64(p.delta)
    return lwe_encrypt(lwe_sk, mask, noise, pt)
