"""Python binding of libsilenzio_pbs (batched TFHE PBS + LWE keyswitch on MI355X / gfx950).

Argument marshalling only: every step runs in the HIP kernels of the shared library.  PyTorch is
used for device memory and streams.  The functions mirror the C ABI in include/silenzio_pbs.h
one to one.  There is no CPU fallback: if the library is missing and cannot be built, importing
a function raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SILENZIO_PBS_LIB") or os.path.join(_HERE, "libsilenzio_pbs.so")

SLZ_OPT_FORCE_GENERIC = 1
SLZ_OPT_LARGE_N_BLOCK = 2
SLZ_OPT_LARGE_N_LANES = 3
SLZ_OPT_FAIL_ALLOC_AFTER = 4
SLZ_OPT_LARGE_N_LATENCY = 5
SLZ_OPT_FUSED_PACING = 6
SLZ_OK, SLZ_E_INVALID_ARG, SLZ_E_UNSUPPORTED, SLZ_E_HIP, SLZ_E_NOMEM, SLZ_E_TOO_LARGE = 0, -1, -2, -3, -4, -5


class SlzParams(ctypes.Structure):
    _fields_ = [(f, ctypes.c_uint32) for f in
                ("n", "k", "N", "pbs_base_log", "pbs_level", "ks_base_log", "ks_level", "msg_bits")]


class SlzError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (where, lib().slz_strerror(code).decode(), code))


_lib = None

EXPORTS = ("slz_ctx_create", "slz_ctx_destroy", "slz_ctx_set_option", "slz_lut_encode", "slz_bsk_prepare",
           "slz_pbs_batch", "slz_blind_rotate_batch", "slz_keyswitch_batch", "slz_keyswitch_batch_static", "slz_ksk_prepare", "slz_keyswitch_batch_prepared",
           "slz_ks_pbs_batch", "slz_lwe_lincomb_batch",
           "slz_pbs_path", "slz_strerror", "slz_matmul_rns_luts", "slz_matmul_rns_workspace", "slz_matmul_rns",
           "slz_rns_luts", "slz_rns_workspace", "slz_rns2mrns", "slz_sign_rns",
           "slz_shift2msbs_luts", "slz_shift2msbs_workspace", "slz_shift2msbs_plus", "slz_shift2msbs_pm",
           "slz_bivariate_workspace", "slz_bivariate_lookup", "slz_loss_luts", "slz_loss_workspace", "slz_int_ce_loss_deriv",
           "slz_weight_update_luts", "slz_weight_update",
           "slz_matmul_highres_luts", "slz_matmul_highres_workspace", "slz_matmul_highres")


def lib():
    """Loads the built library (building it first only if no built library exists)."""
    global _lib
    if _lib is None:
        # PyTorch must be loaded first: its wheel bundles the HIP runtime under the same soname the library
        # links against, and a process must hold exactly one HIP runtime (torch's streams and allocations
        # are only valid in the runtime that made them).
        import torch  # noqa: F401
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build()
        L = ctypes.CDLL(LIB_PATH)
        vp, u32, sz = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_size_t
        L.slz_ctx_create.argtypes = [ctypes.POINTER(SlzParams), u32, ctypes.POINTER(vp)]
        L.slz_ctx_destroy.argtypes = [vp]
        L.slz_ctx_set_option.argtypes = [vp, ctypes.c_int, ctypes.c_int]
        L.slz_lut_encode.argtypes = [ctypes.POINTER(SlzParams), vp, u32, vp]
        L.slz_bsk_prepare.argtypes = [vp, vp, vp, ctypes.POINTER(sz), vp]
        L.slz_pbs_batch.argtypes = [vp, vp, vp, vp, u32, vp, vp, u32, vp]
        L.slz_blind_rotate_batch.argtypes = [vp, vp, vp, vp, u32, vp, u32, vp, u32, vp]
        L.slz_keyswitch_batch.argtypes = [vp, vp, vp, vp, u32, vp]
        L.slz_keyswitch_batch_static.argtypes = [vp, vp, vp, vp, u32, vp]
        L.slz_ksk_prepare.argtypes = [vp, vp, vp, ctypes.POINTER(sz), vp]
        L.slz_keyswitch_batch_prepared.argtypes = [vp, vp, vp, vp, u32, vp]
        L.slz_ks_pbs_batch.argtypes = [vp, vp, vp, vp, vp, u32, vp, vp, u32, vp]
        L.slz_lwe_lincomb_batch.argtypes = [vp, vp, vp, vp, u32, u32, u32, vp]
        L.slz_pbs_path.argtypes = [vp]
        L.slz_pbs_path.restype = ctypes.c_char_p
        L.slz_matmul_rns_luts.argtypes = [ctypes.POINTER(SlzParams), ctypes.POINTER(SlzMatmulRnsShape), vp]
        L.slz_matmul_rns_workspace.argtypes = [vp, ctypes.POINTER(SlzMatmulRnsShape), ctypes.POINTER(sz)]
        L.slz_matmul_rns.argtypes = [vp, ctypes.POINTER(SlzMatmulRnsShape), vp, vp, vp, vp, vp, vp, vp, sz, vp]
        i32 = ctypes.c_int32
        L.slz_matmul_highres_luts.argtypes = L.slz_matmul_rns_luts.argtypes
        L.slz_matmul_highres_workspace.argtypes = L.slz_matmul_rns_workspace.argtypes
        L.slz_matmul_highres.argtypes = L.slz_matmul_rns.argtypes
        L.slz_rns_luts.argtypes = [ctypes.POINTER(SlzParams), ctypes.POINTER(SlzRnsShape), i32, i32, i32, vp]
        L.slz_rns_workspace.argtypes = [vp, ctypes.POINTER(SlzRnsShape), ctypes.POINTER(sz)]
        L.slz_rns2mrns.argtypes = [vp, ctypes.POINTER(SlzRnsShape), vp, vp, vp, vp, vp, vp, sz, vp]
        L.slz_sign_rns.argtypes = [vp, ctypes.POINTER(SlzRnsShape), vp, vp, vp, vp, vp, vp, sz, vp]
        L.slz_shift2msbs_luts.argtypes = [ctypes.POINTER(SlzParams), ctypes.POINTER(SlzShiftShape), vp]
        L.slz_shift2msbs_workspace.argtypes = [vp, ctypes.POINTER(SlzShiftShape), ctypes.POINTER(sz)]
        L.slz_shift2msbs_plus.argtypes = [vp, ctypes.POINTER(SlzShiftShape), vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.slz_shift2msbs_pm.argtypes = [vp, ctypes.POINTER(SlzShiftShape), vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.slz_bivariate_workspace.argtypes = [vp, u32, ctypes.POINTER(sz)]
        L.slz_bivariate_lookup.argtypes = [vp, vp, vp, u32, vp, vp, u32, vp, vp, vp, u32, vp, sz, vp]
        L.slz_loss_luts.argtypes = [ctypes.POINTER(SlzParams), ctypes.POINTER(SlzLossShape), vp]
        L.slz_loss_workspace.argtypes = [vp, ctypes.POINTER(SlzLossShape), ctypes.POINTER(sz)]
        L.slz_int_ce_loss_deriv.argtypes = [vp, ctypes.POINTER(SlzLossShape), vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.slz_weight_update_luts.argtypes = [ctypes.POINTER(SlzParams), u32, vp]
        L.slz_weight_update.argtypes = [vp, u32, vp, vp, vp, vp, vp, vp, u32, vp, sz, vp]
        L.slz_strerror.argtypes = [ctypes.c_int]
        L.slz_strerror.restype = ctypes.c_char_p
        for name in EXPORTS:
            if name not in ("slz_pbs_path", "slz_strerror"):
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


class SlzMatmulRnsShape(ctypes.Structure):
    """slz_matmul_rns_shape of include/silenzio_gadgets.h."""
    _fields_ = [("k", ctypes.c_uint32), ("m", ctypes.c_uint32 * 8), ("a", ctypes.c_uint32), ("b", ctypes.c_uint32),
                ("c", ctypes.c_uint32)]


def make_matmul_rns_shape(m, a: int, b: int, c: int) -> SlzMatmulRnsShape:
    m = [int(q) for q in m]
    if not 1 <= len(m) <= 8:
        raise ValueError("1 to 8 moduli")
    return SlzMatmulRnsShape(len(m), (ctypes.c_uint32 * 8)(*m), a, b, c)


def matmul_rns_luts(p, m, a: int, b: int, c: int) -> np.ndarray:
    """slz_matmul_rns_luts: the 3k lookup polynomials of Matmul^RNS, u64 [3k][N] (host)."""
    cp = make_params(p)
    sh = make_matmul_rns_shape(m, a, b, c)
    out = np.empty((3 * sh.k, p.N), dtype=np.uint64)
    _check(lib().slz_matmul_rns_luts(ctypes.byref(cp), ctypes.byref(sh), out.ctypes.data), "slz_matmul_rns_luts")
    return out


def matmul_highres_luts(p, m, a: int, b: int, c: int) -> np.ndarray:
    """slz_matmul_highres_luts: the 4k + 3 lookup polynomials of MatmulHighRes^RNS, u64 [4k + 3][N] (host)."""
    cp = make_params(p)
    sh = make_matmul_rns_shape(m, a, b, c)
    out = np.empty((4 * sh.k + 3, p.N), dtype=np.uint64)
    _check(lib().slz_matmul_highres_luts(ctypes.byref(cp), ctypes.byref(sh), out.ctypes.data), "slz_matmul_highres_luts")
    return out


class SlzRnsShape(ctypes.Structure):
    """slz_rns_shape of include/silenzio_gadgets.h."""
    _fields_ = [("k", ctypes.c_uint32), ("m", ctypes.c_uint32 * 8), ("count", ctypes.c_uint32)]


def make_rns_shape(m, count: int) -> SlzRnsShape:
    m = [int(q) for q in m]
    if not 1 <= len(m) <= 8:
        raise ValueError("1 to 8 moduli")
    return SlzRnsShape(len(m), (ctypes.c_uint32 * 8)(*m), count)


def rns_luts(p, m, neg: int = -1, zero: int = 0, pos: int = 1) -> np.ndarray:
    """slz_rns_luts: conversion tables of RNS2MRNS plus the two tables of Sign_(neg,zero,pos), u64 [k(k-1)/2 + 2][N] (host)."""
    cp = make_params(p)
    sh = make_rns_shape(m, 1)
    out = np.empty((sh.k * (sh.k - 1) // 2 + 2, p.N), dtype=np.uint64)
    _check(lib().slz_rns_luts(ctypes.byref(cp), ctypes.byref(sh), neg, zero, pos, out.ctypes.data), "slz_rns_luts")
    return out


class SlzShiftShape(ctypes.Structure):
    """slz_shift_shape of include/silenzio_gadgets.h."""
    _fields_ = [("k", ctypes.c_uint32), ("m", ctypes.c_uint32 * 8), ("count", ctypes.c_uint32), ("w", ctypes.c_uint32),
                ("gamma", ctypes.c_uint32)]


def make_shift_shape(m, count: int, w: int, gamma: int) -> SlzShiftShape:
    m = [int(q) for q in m]
    if not 1 <= len(m) <= 8:
        raise ValueError("1 to 8 moduli")
    return SlzShiftShape(len(m), (ctypes.c_uint32 * 8)(*m), count, w, gamma)


def shift2msbs_luts(p, m, w: int, gamma: int) -> np.ndarray:
    """slz_shift2msbs_luts: every table of Shift2MSBs^+ / ^+- for unsigned output bitwidth gamma, u64 [k(k-1)/2 + 3k + 5][N] (host)."""
    cp = make_params(p)
    sh = make_shift_shape(m, 1, w, gamma)
    out = np.empty((sh.k * (sh.k - 1) // 2 + 3 * sh.k + 5, p.N), dtype=np.uint64)
    _check(lib().slz_shift2msbs_luts(ctypes.byref(cp), ctypes.byref(sh), out.ctypes.data), "slz_shift2msbs_luts")
    return out


class SlzLossShape(ctypes.Structure):
    """slz_loss_shape of include/silenzio_gadgets.h."""
    _fields_ = [("a", ctypes.c_uint32), ("b", ctypes.c_uint32), ("big_gamma", ctypes.c_uint32), ("kappa", ctypes.c_uint32)]


def loss_luts(p, b: int, big_gamma: int, kappa: int) -> np.ndarray:
    """slz_loss_luts: the five lookup polynomials of IntCELossDeriv, u64 [5][N] (host)."""
    cp = make_params(p)
    sh = SlzLossShape(1, b, big_gamma, kappa)
    out = np.empty((5, p.N), dtype=np.uint64)
    _check(lib().slz_loss_luts(ctypes.byref(cp), ctypes.byref(sh), out.ctypes.data), "slz_loss_luts")
    return out


def weight_update_luts(p, alpha: int) -> np.ndarray:
    """slz_weight_update_luts: the lookup polynomial of the clipped weight update, u64 [1][N] (host)."""
    cp = make_params(p)
    out = np.empty((1, p.N), dtype=np.uint64)
    _check(lib().slz_weight_update_luts(ctypes.byref(cp), alpha, out.ctypes.data), "slz_weight_update_luts")
    return out


def make_params(p) -> SlzParams:
    """From any object with the fields n, k, N, pbs_base_log, pbs_level, ks_base_log, ks_level, msg_bits."""
    return SlzParams(p.n, p.k, p.N, p.pbs_base_log, p.pbs_level, p.ks_base_log, p.ks_level, p.msg_bits)


def _check(rc: int, where: str):
    if rc != 0:
        raise SlzError(rc, where)


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _dev_u64(t, what: str) -> int:
    """Device address of a contiguous int64/uint64 CUDA tensor (the bits are the u64 words)."""
    import torch
    if not t.is_cuda or not t.is_contiguous() or t.dtype not in (torch.int64, torch.uint64, torch.float64):
        raise TypeError("%s: need a contiguous 64-bit CUDA tensor" % what)
    return t.data_ptr()


def _need(t, count: int, what: str, exact: bool = True):
    """Host-side size check of a device buffer: a wrong width or a short output must be a Python error, not a device fault."""
    have = t.numel()
    if (have != count) if exact else (have < count):
        raise ValueError("%s: %d elements, need %s%d" % (what, have, "" if exact else "at least ", count))


def to_device_u64(a: np.ndarray):
    """numpy uint64 array -> CUDA int64 tensor with the same bits."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint64).view(np.int64)).cuda()


def to_host_u64(t) -> np.ndarray:
    return t.cpu().numpy().view(np.uint64)


def lut_encode(p, tables: np.ndarray) -> np.ndarray:
    """slz_lut_encode: tables u64 [n_tables][t] (host) -> LUT polynomials u64 [n_tables][N] (host)."""
    cp = make_params(p)
    tables = np.ascontiguousarray(tables, dtype=np.uint64).reshape(-1, 1 << p.msg_bits)
    out = np.empty((tables.shape[0], p.N), dtype=np.uint64)
    _check(lib().slz_lut_encode(ctypes.byref(cp), tables.ctypes.data, tables.shape[0], out.ctypes.data), "slz_lut_encode")
    return out


class Context:
    """slz_ctx wrapper.  Owns the context handle; tensors passed in stay owned by the caller."""

    def __init__(self, p, max_batch: int):
        self.p = p
        self.cp = make_params(p)
        self.max_batch = int(max_batch)
        self._h = ctypes.c_void_p()
        _check(lib().slz_ctx_create(ctypes.byref(self.cp), self.max_batch, ctypes.byref(self._h)), "slz_ctx_create")

    def close(self):
        if self._h:
            lib().slz_ctx_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def path(self) -> str:
        return lib().slz_pbs_path(self._h).decode()

    def set_option(self, option: int, value: int):
        _check(lib().slz_ctx_set_option(self._h, option, value), "slz_ctx_set_option")

    def bsk_prepared_bytes(self) -> int:
        need = ctypes.c_size_t(0)
        _check(lib().slz_bsk_prepare(self._h, None, None, ctypes.byref(need), None), "slz_bsk_prepare(size)")
        return need.value

    def bsk_prepare(self, bsk_dev):
        """Standard-domain BSK (CUDA tensor, u64 bits) -> prepared key (CUDA float64 tensor, library-private layout)."""
        import torch
        _need(bsk_dev, self.p.n * (self.p.k + 1) ** 2 * self.p.pbs_level * self.p.N, "bsk")
        need = self.bsk_prepared_bytes()
        dst = torch.empty(need // 8, dtype=torch.float64, device=bsk_dev.device)
        nb = ctypes.c_size_t(need)
        _check(lib().slz_bsk_prepare(self._h, _dev_u64(bsk_dev, "bsk"), dst.data_ptr(), ctypes.byref(nb), _stream()),
               "slz_bsk_prepare")
        return dst

    def _lut_args(self, luts_dev, lut_idx_dev, batch: int):
        import torch
        n_luts = luts_dev.numel() // self.p.N
        if n_luts == 0 or luts_dev.numel() != n_luts * self.p.N:
            raise ValueError("luts: %d elements, need a positive multiple of N = %d" % (luts_dev.numel(), self.p.N))
        idx_ptr = None
        if lut_idx_dev is not None:
            if lut_idx_dev.dtype != torch.int32 or not lut_idx_dev.is_cuda or not lut_idx_dev.is_contiguous():
                raise TypeError("lut_idx: need a contiguous int32 CUDA tensor")
            _need(lut_idx_dev, batch, "lut_idx", exact=False)
            idx_ptr = lut_idx_dev.data_ptr()
        return n_luts, idx_ptr

    def _check_keys(self, bsk_prepared=None, ksk=None):
        if bsk_prepared is not None and bsk_prepared.numel() * bsk_prepared.element_size() < self.bsk_prepared_bytes():
            raise ValueError("bsk_prepared: %d bytes, need %d" % (bsk_prepared.numel() * bsk_prepared.element_size(),
                                                                  self.bsk_prepared_bytes()))
        if ksk is not None:
            _need(ksk, self.p.k * self.p.N * self.p.ks_level * (self.p.n + 1), "ksk")

    def _small(self, t, what: str, rows: int = None):
        """A ciphertext array under the small key: [..][n+1]."""
        if t.shape[-1] != self.p.n + 1:
            raise ValueError("%s: rows of %d words, need n + 1 = %d" % (what, t.shape[-1], self.p.n + 1))
        if rows is not None:
            _need(t, rows * (self.p.n + 1), what)

    def _big(self, t, what: str, rows: int = None):
        """A ciphertext array under the big key: [..][kN+1]."""
        w = self.p.k * self.p.N + 1
        if t.shape[-1] != w:
            raise ValueError("%s: rows of %d words, need kN + 1 = %d" % (what, t.shape[-1], w))
        if rows is not None:
            _need(t, rows * w, what)

    def pbs_batch(self, lwe_in, luts, lut_idx, bsk_prepared, out=None):
        import torch
        batch = lwe_in.shape[0]
        if out is None:
            out = torch.empty((batch, self.p.k * self.p.N + 1), dtype=torch.int64, device=lwe_in.device)
        n_luts, idx_ptr = self._lut_args(luts, lut_idx, batch)
        self._small(lwe_in, "lwe_in")
        self._big(out, "out", batch)
        self._check_keys(bsk_prepared)
        _check(lib().slz_pbs_batch(self._h, _dev_u64(lwe_in, "lwe_in"), _dev_u64(luts, "luts"), idx_ptr, n_luts,
                                   bsk_prepared.data_ptr(), _dev_u64(out, "out"), batch, _stream()), "slz_pbs_batch")
        return out

    def blind_rotate_batch(self, lwe_in, luts, lut_idx, bsk_prepared, n_steps: int, out=None):
        import torch
        batch = lwe_in.shape[0]
        if out is None:
            out = torch.empty((batch, self.p.k + 1, self.p.N), dtype=torch.int64, device=lwe_in.device)
        n_luts, idx_ptr = self._lut_args(luts, lut_idx, batch)
        self._small(lwe_in, "lwe_in")
        _need(out, batch * (self.p.k + 1) * self.p.N, "out")
        self._check_keys(bsk_prepared)
        if not 0 <= int(n_steps) <= self.p.n:
            raise ValueError("n_steps: %d, need 0 .. n = %d" % (n_steps, self.p.n))
        _check(lib().slz_blind_rotate_batch(self._h, _dev_u64(lwe_in, "lwe_in"), _dev_u64(luts, "luts"), idx_ptr, n_luts,
                                            bsk_prepared.data_ptr(), int(n_steps), _dev_u64(out, "out"), batch, _stream()),
               "slz_blind_rotate_batch")
        return out

    def keyswitch_batch(self, lwe_in, ksk, out=None):
        import torch
        batch = lwe_in.shape[0]
        if out is None:
            out = torch.empty((batch, self.p.n + 1), dtype=torch.int64, device=lwe_in.device)
        self._big(lwe_in, "lwe_in")
        self._small(out, "out", batch)
        self._check_keys(ksk=ksk)
        _check(lib().slz_keyswitch_batch(self._h, _dev_u64(lwe_in, "lwe_in"), _dev_u64(ksk, "ksk"), _dev_u64(out, "out"),
                                         batch, _stream()), "slz_keyswitch_batch")
        return out

    def ksk_prepared_bytes(self) -> int:
        need = ctypes.c_size_t(0)
        _check(lib().slz_ksk_prepare(self._h, None, None, ctypes.byref(need), None), "slz_ksk_prepare(size)")
        return need.value

    def ksk_prepare(self, ksk):
        """Standard keyswitching key (CUDA tensor, u64 bits) -> the key as operands of the matrix-core contraction (CUDA
        uint8 tensor, library-private layout)."""
        import torch
        self._check_keys(ksk=ksk)
        need = self.ksk_prepared_bytes()
        dst = torch.empty(need, dtype=torch.uint8, device=ksk.device)
        nb = ctypes.c_size_t(need)
        _check(lib().slz_ksk_prepare(self._h, _dev_u64(ksk, "ksk"), dst.data_ptr(), ctypes.byref(nb), _stream()), "slz_ksk_prepare")
        return dst

    def keyswitch_batch_prepared(self, lwe_in, ksk_prepared, out=None):
        import torch
        batch = lwe_in.shape[0]
        if out is None:
            out = torch.empty((batch, self.p.n + 1), dtype=torch.int64, device=lwe_in.device)
        self._big(lwe_in, "lwe_in")
        self._small(out, "out", batch)
        if not ksk_prepared.is_cuda or not ksk_prepared.is_contiguous() or \
                ksk_prepared.numel() * ksk_prepared.element_size() < self.ksk_prepared_bytes():
            raise ValueError("ksk_prepared: need the contiguous CUDA tensor that ksk_prepare returned")
        _check(lib().slz_keyswitch_batch_prepared(self._h, _dev_u64(lwe_in, "lwe_in"), ksk_prepared.data_ptr(), _dev_u64(out, "out"),
                                                  batch, _stream()), "slz_keyswitch_batch_prepared")
        return out

    def keyswitch_batch_static(self, lwe_in, ksk, out):
        """slz_keyswitch_batch_static: the keyswitch with its scratch in a fixed device array of the library; `out`
        ([batch][n+1]) comes from the caller, so that nothing is allocated on the way."""
        self._big(lwe_in, "lwe_in")
        self._small(out, "out", lwe_in.shape[0])
        self._check_keys(ksk=ksk)
        _check(lib().slz_keyswitch_batch_static(self._h, _dev_u64(lwe_in, "lwe_in"), _dev_u64(ksk, "ksk"), _dev_u64(out, "out"),
                                                lwe_in.shape[0], _stream()), "slz_keyswitch_batch_static")
        return out

    def ks_pbs_batch(self, lwe_in, ksk, luts, lut_idx, bsk_prepared, out=None):
        """slz_ks_pbs_batch: keyswitch, then bootstrapping; [batch][kN+1] -> [batch][kN+1] (out may be lwe_in)."""
        import torch
        batch = lwe_in.shape[0]
        if out is None:
            out = torch.empty((batch, self.p.k * self.p.N + 1), dtype=torch.int64, device=lwe_in.device)
        n_luts, idx_ptr = self._lut_args(luts, lut_idx, batch)
        self._big(lwe_in, "lwe_in")
        self._big(out, "out", batch)
        self._check_keys(bsk_prepared, ksk)
        _check(lib().slz_ks_pbs_batch(self._h, _dev_u64(lwe_in, "lwe_in"), _dev_u64(ksk, "ksk"), _dev_u64(luts, "luts"), idx_ptr, n_luts,
                                      bsk_prepared.data_ptr(), _dev_u64(out, "out"), batch, _stream()), "slz_ks_pbs_batch")
        return out

    def matmul_rns(self, x_cts, w_cts, m, luts, bsk_prepared, ksk, out=None, highres: bool = False):
        """slz_matmul_rns (highres: slz_matmul_highres, 5-bit moduli): x_cts [a][b][n+1], w_cts [b][c][n+1] -> [k][a][c][n+1];
        allocates the workspace the call needs."""
        import torch
        a, b = x_cts.shape[:2]
        c = w_cts.shape[1]
        sh = make_matmul_rns_shape(m, a, b, c)
        need = ctypes.c_size_t(0)
        L = lib()
        ws_fn, fn, name = (L.slz_matmul_highres_workspace, L.slz_matmul_highres, "slz_matmul_highres") if highres else \
            (L.slz_matmul_rns_workspace, L.slz_matmul_rns, "slz_matmul_rns")
        _check(ws_fn(self._h, ctypes.byref(sh), ctypes.byref(need)), name + "_workspace")
        ws = torch.empty(need.value, dtype=torch.uint8, device=x_cts.device)
        if out is None:
            out = torch.empty((sh.k, a, c, self.p.n + 1), dtype=torch.int64, device=x_cts.device)
        self._small(x_cts, "x_cts", a * b)
        self._small(w_cts, "w_cts", b * c)
        self._small(out, "out", sh.k * a * c)
        _need(luts, ((4 * sh.k + 3) if highres else 3 * sh.k) * self.p.N, "luts")
        self._check_keys(bsk_prepared, ksk)
        _check(fn(self._h, ctypes.byref(sh), _dev_u64(x_cts, "x_cts"), _dev_u64(w_cts, "w_cts"), _dev_u64(luts, "luts"),
                  bsk_prepared.data_ptr(), _dev_u64(ksk, "ksk"), _dev_u64(out, "out"), ws.data_ptr(), need.value, _stream()), name)
        torch.cuda.current_stream().synchronize()     # the workspace is released when this returns
        return out

    def _rns_call(self, fn, name, x_cts, m, luts, bsk_prepared, ksk, out):
        import torch
        sh = make_rns_shape(m, x_cts.shape[1])
        self._small(x_cts, "x_cts", sh.k * sh.count)
        self._small(out, "out", out.numel() // (self.p.n + 1))
        _need(out, (sh.k if name == "slz_rns2mrns" else 1) * sh.count * (self.p.n + 1), "out")
        _need(luts, (sh.k * (sh.k - 1) // 2 + 2) * self.p.N, "luts")
        self._check_keys(bsk_prepared, ksk)
        need = ctypes.c_size_t(0)
        _check(lib().slz_rns_workspace(self._h, ctypes.byref(sh), ctypes.byref(need)), "slz_rns_workspace")
        ws = torch.empty(need.value, dtype=torch.uint8, device=x_cts.device)
        _check(fn(self._h, ctypes.byref(sh), _dev_u64(x_cts, "x_cts"), _dev_u64(luts, "luts"), bsk_prepared.data_ptr(),
                  _dev_u64(ksk, "ksk"), _dev_u64(out, "out"), ws.data_ptr(), need.value, _stream()), name)
        torch.cuda.current_stream().synchronize()     # the workspace is released when this returns
        return out

    def rns2mrns(self, x_cts, m, luts, bsk_prepared, ksk, out=None):
        """slz_rns2mrns: residues [k][count][n+1] -> mixed-radix digits [k][count][n+1]."""
        import torch
        if out is None:
            out = torch.empty_like(x_cts)
        return self._rns_call(lib().slz_rns2mrns, "slz_rns2mrns", x_cts, m, luts, bsk_prepared, ksk, out)

    def sign_rns(self, x_cts, m, luts, bsk_prepared, ksk, out=None):
        """slz_sign_rns: residues [k][count][n+1] -> [count][n+1] encryptions of the neg / zero / pos values of the tables."""
        import torch
        if out is None:
            out = torch.empty((x_cts.shape[1], self.p.n + 1), dtype=torch.int64, device=x_cts.device)
        return self._rns_call(lib().slz_sign_rns, "slz_sign_rns", x_cts, m, luts, bsk_prepared, ksk, out)

    def shift2msbs(self, x_cts, m, w: int, gamma: int, luts, bsk_prepared, ksk, signed: bool = False):
        """slz_shift2msbs_plus / slz_shift2msbs_pm: residues [k][count][n+1] -> (Y [count][n+1], shift [n+1]); gamma is the
        unsigned output bitwidth (for signed inputs: Gamma - 1)."""
        import torch
        count = x_cts.shape[1]
        sh = make_shift_shape(m, count, w, gamma)
        self._small(x_cts, "x_cts", sh.k * count)
        _need(luts, (sh.k * (sh.k - 1) // 2 + 3 * sh.k + 5) * self.p.N, "luts")
        self._check_keys(bsk_prepared, ksk)
        need = ctypes.c_size_t(0)
        _check(lib().slz_shift2msbs_workspace(self._h, ctypes.byref(sh), ctypes.byref(need)), "slz_shift2msbs_workspace")
        ws = torch.empty(need.value, dtype=torch.uint8, device=x_cts.device)
        y = torch.empty((count, self.p.n + 1), dtype=torch.int64, device=x_cts.device)
        shift = torch.empty((self.p.n + 1,), dtype=torch.int64, device=x_cts.device)
        fn = lib().slz_shift2msbs_pm if signed else lib().slz_shift2msbs_plus
        _check(fn(self._h, ctypes.byref(sh), _dev_u64(x_cts, "x_cts"), _dev_u64(luts, "luts"), bsk_prepared.data_ptr(),
                  _dev_u64(ksk, "ksk"), _dev_u64(y, "y"), _dev_u64(shift, "shift"), ws.data_ptr(), need.value, _stream()),
               "slz_shift2msbs")
        torch.cuda.current_stream().synchronize()     # the workspace is released when this returns
        return y, shift

    def _bivariate_ws(self, count: int, device):
        import torch
        need = ctypes.c_size_t(0)
        _check(lib().slz_bivariate_workspace(self._h, count, ctypes.byref(need)), "slz_bivariate_workspace")
        return torch.empty(need.value, dtype=torch.uint8, device=device), need.value

    def bivariate_lookup(self, x_cts, y_cts, y_bits: int, luts, bsk_prepared, ksk, lut_index=None):
        """slz_bivariate_lookup: [count][n+1] pairs -> [count][n+1], one lookup each on 2^y_bits x + y."""
        import torch
        count = x_cts.shape[0]
        self._small(x_cts, "x_cts", count)
        self._small(y_cts, "y_cts", count)
        if luts.numel() == 0 or luts.numel() % self.p.N:
            raise ValueError("luts: need a positive multiple of N elements")
        if lut_index is not None:
            _need(lut_index, count, "lut_index", exact=False)
        self._check_keys(bsk_prepared, ksk)
        ws, need = self._bivariate_ws(count, x_cts.device)
        out = torch.empty((count, self.p.n + 1), dtype=torch.int64, device=x_cts.device)
        if lut_index is not None and (lut_index.dtype != torch.int32 or not lut_index.is_cuda or not lut_index.is_contiguous()):
            raise TypeError("lut_index: need a contiguous int32 CUDA tensor")
        _check(lib().slz_bivariate_lookup(self._h, _dev_u64(x_cts, "x_cts"), _dev_u64(y_cts, "y_cts"), y_bits, _dev_u64(luts, "luts"),
                                          None if lut_index is None else lut_index.data_ptr(), luts.shape[0],
                                          bsk_prepared.data_ptr(), _dev_u64(ksk, "ksk"), _dev_u64(out, "out"), count, ws.data_ptr(),
                                          need, _stream()), "slz_bivariate_lookup")
        torch.cuda.current_stream().synchronize()     # the workspace is released when this returns
        return out

    def int_ce_loss_deriv(self, logits, labels, big_gamma: int, kappa: int, luts, bsk_prepared, ksk):
        """slz_int_ce_loss_deriv: logits and one-hot labels [a][b][n+1] -> the sign of the error [a][b][n+1]."""
        import torch
        a, b = logits.shape[:2]
        sh = SlzLossShape(a, b, big_gamma, kappa)
        self._small(logits, "logits", a * b)
        self._small(labels, "labels", a * b)
        _need(luts, 5 * self.p.N, "luts")
        self._check_keys(bsk_prepared, ksk)
        need = ctypes.c_size_t(0)
        _check(lib().slz_loss_workspace(self._h, ctypes.byref(sh), ctypes.byref(need)), "slz_loss_workspace")
        ws = torch.empty(need.value, dtype=torch.uint8, device=logits.device)
        out = torch.empty((a, b, self.p.n + 1), dtype=torch.int64, device=logits.device)
        _check(lib().slz_int_ce_loss_deriv(self._h, ctypes.byref(sh), _dev_u64(logits, "logits"), _dev_u64(labels, "labels"),
                                           _dev_u64(luts, "luts"), bsk_prepared.data_ptr(), _dev_u64(ksk, "ksk"), _dev_u64(out, "out"),
                                           ws.data_ptr(), need.value, _stream()), "slz_int_ce_loss_deriv")
        torch.cuda.current_stream().synchronize()     # the workspace is released when this returns
        return out

    def weight_update(self, w_cts, gcode_cts, alpha: int, luts, bsk_prepared, ksk):
        """slz_weight_update: weights and codes G + 1, [count][n+1] each -> clip(W - G), [count][n+1]."""
        import torch
        count = w_cts.shape[0]
        self._small(w_cts, "w_cts", count)
        self._small(gcode_cts, "gcode_cts", count)
        _need(luts, self.p.N, "luts")
        self._check_keys(bsk_prepared, ksk)
        ws, need = self._bivariate_ws(count, w_cts.device)
        out = torch.empty((count, self.p.n + 1), dtype=torch.int64, device=w_cts.device)
        _check(lib().slz_weight_update(self._h, alpha, _dev_u64(w_cts, "w_cts"), _dev_u64(gcode_cts, "gcode_cts"), _dev_u64(luts, "luts"),
                                       bsk_prepared.data_ptr(), _dev_u64(ksk, "ksk"), _dev_u64(out, "out"), count, ws.data_ptr(), need,
                                       _stream()), "slz_weight_update")
        torch.cuda.current_stream().synchronize()     # the workspace is released when this returns
        return out

    def lwe_lincomb_batch(self, cts, w, out=None):
        import torch
        G, J, width = cts.shape
        O = w.shape[1]
        if w.dtype != torch.int32 or not w.is_cuda or not w.is_contiguous():
            raise TypeError("w: need a contiguous int32 CUDA tensor")
        if out is None:
            out = torch.empty((G, O, width), dtype=torch.int64, device=cts.device)
        self._small(cts, "cts")
        _need(w, J * O, "w")
        self._small(out, "out", G * O)
        _check(lib().slz_lwe_lincomb_batch(self._h, _dev_u64(cts, "cts"), w.data_ptr(), _dev_u64(out, "out"), G, J, O,
                                           _stream()), "slz_lwe_lincomb_batch")
        return out
