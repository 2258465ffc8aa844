"""CPU oracle for the CompactFusion residual codec.  TEST INFRASTRUCTURE ONLY.

ctypes binding over ``cf_oracle.c`` (plain single-threaded C written from
arxiv 2507.17511: Sec. 3.1, Sec. 3.2, App. D, App. H).  Only the tests, the
smoke check and the benchmark's cpu-baseline leg may import this package; the
HIP library and its Python binding never do, and share no code with it.

Arrays are numpy; bf16 tensors travel as ``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cf_oracle.c")
_LIB = os.path.join(_HERE, "libcf_oracle.so")

F32, BF16 = 0, 1
SCALE_CHANNEL, SCALE_GROUP, SCALE_RANK1, SPARSE_NM = 0, 1, 2, 3
EF_RECON, EF_LITERAL, EF_OFF = 0, 1, 2

CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict fp32: no contraction, no fast-math)."""
    newest_src = max(os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "cf_oracle.h")))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest_src:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Cfg(ctypes.Structure):
    _fields_ = [
        ("n_tokens", ctypes.c_int64),
        ("n_channels", ctypes.c_int64),
        ("dtype", ctypes.c_int32),
        ("bits", ctypes.c_int32),
        ("scale", ctypes.c_int32),
        ("group", ctypes.c_int32),
        ("ef", ctypes.c_int32),
        ("err_dtype", ctypes.c_int32),
    ]


@dataclass(frozen=True)
class Config:
    n_tokens: int
    n_channels: int
    dtype: int = BF16
    bits: int = 2
    scale: int = SCALE_CHANNEL
    group: int = 128
    ef: int = EF_RECON
    err_dtype: int = F32

    def c(self) -> _Cfg:
        return _Cfg(self.n_tokens, self.n_channels, self.dtype, self.bits, self.scale,
                    self.group, self.ef, self.err_dtype)

    @property
    def shape(self):
        return (self.n_tokens, self.n_channels)

    @property
    def np_dtype(self):
        return np.uint16 if self.dtype == BF16 else np.float32

    @property
    def np_err_dtype(self):
        return np.uint16 if self.err_dtype == BF16 else np.float32


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        vp, cp = ctypes.c_void_p, ctypes.POINTER(_Cfg)
        L.cfo_bf16_to_f32.restype = ctypes.c_float
        L.cfo_bf16_to_f32.argtypes = [ctypes.c_uint16]
        L.cfo_f32_to_bf16.restype = ctypes.c_uint16
        L.cfo_f32_to_bf16.argtypes = [ctypes.c_float]
        L.cfo_f32_to_bf16_array.restype = None
        L.cfo_f32_to_bf16_array.argtypes = [vp, vp, ctypes.c_int64]
        L.cfo_treesum.restype = ctypes.c_float
        L.cfo_treesum.argtypes = [vp, ctypes.c_int64, ctypes.c_int64]
        L.cfo_codes_bytes.restype = ctypes.c_int64
        L.cfo_codes_bytes.argtypes = [cp]
        L.cfo_scales_count.restype = ctypes.c_int64
        L.cfo_scales_count.argtypes = [cp]
        L.cfo_nm_values_offset.restype = ctypes.c_int64
        L.cfo_nm_values_offset.argtypes = [cp]
        L.cfo_check.argtypes = [cp]
        for name, n in [("cfo_residual", 4), ("cfo_scales", 2), ("cfo_select", 3), ("cfo_pack", 2),
                        ("cfo_unpack", 2), ("cfo_decode", 3), ("cfo_nm_select", 2), ("cfo_nm_pack", 3), ("cfo_nm_unpack", 2)]:
            getattr(L, name).restype = None
            getattr(L, name).argtypes = [cp] + [vp] * n
        for name, n in [("cfo_warmup", 3), ("cfo_compress", 5), ("cfo_decompress", 3), ("cfo_step", 5),
                        ("cfo_naive", 4)]:
            getattr(L, name).restype = ctypes.c_int
            getattr(L, name).argtypes = [cp] + [vp] * n
        _lib = L
    return _lib


def _p(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"], "oracle arrays must be dense row-major"
    return a.ctypes.data_as(ctypes.c_void_p)


def _chk(a: np.ndarray, dtype, size: int, what: str):
    if a.dtype != dtype or a.size != size:
        raise ValueError(f"{what}: expected {size} x {np.dtype(dtype).name}, got {a.size} x {a.dtype.name}")


# ---------------------------------------------------------------- elements

def bf16_to_f32(h: np.ndarray) -> np.ndarray:
    """Element-wise through the oracle's own widening."""
    L = lib()
    flat = np.ascontiguousarray(h, dtype=np.uint16).ravel()
    return np.array([L.cfo_bf16_to_f32(int(v)) for v in flat], dtype=np.float32).reshape(np.shape(h))


def f32_to_bf16(f: np.ndarray) -> np.ndarray:
    """Element-wise through the oracle's own round-to-nearest-even narrowing."""
    L = lib()
    flat = np.ascontiguousarray(f, dtype=np.float32).ravel()
    out = np.empty(flat.shape, dtype=np.uint16)
    L.cfo_f32_to_bf16_array(_p(flat), _p(out), flat.size)
    return out.reshape(np.shape(f))


def treesum(v: np.ndarray) -> np.float32:
    v = np.ascontiguousarray(v, dtype=np.float32)
    return np.float32(lib().cfo_treesum(_p(v), v.size, 1))


# ---------------------------------------------------------------- stages

def codes_bytes(cfg: Config) -> int:
    return int(lib().cfo_codes_bytes(ctypes.byref(cfg.c())))


def alloc_codes(cfg: Config) -> np.ndarray:
    if cfg.scale == SPARSE_NM:          # masks, then values: not a [tokens, bytes] matrix
        return np.zeros(codes_bytes(cfg), dtype=np.uint8)
    return np.zeros((cfg.n_tokens, cfg.n_channels * cfg.bits // 8), dtype=np.uint8)


def alloc_scales(cfg: Config) -> np.ndarray:
    return np.zeros(int(lib().cfo_scales_count(ctypes.byref(cfg.c()))), dtype=np.float32)


def residual(cfg: Config, x, recon, err) -> np.ndarray:
    n = cfg.n_tokens * cfg.n_channels
    _chk(x, cfg.np_dtype, n, "x"); _chk(recon, cfg.np_dtype, n, "recon"); _chk(err, cfg.np_err_dtype, n, "err")
    z = np.empty(cfg.shape, dtype=np.float32)
    lib().cfo_residual(ctypes.byref(cfg.c()), _p(x), _p(recon), _p(err), _p(z))
    return z


def scales(cfg: Config, z) -> np.ndarray:
    _chk(z, np.float32, cfg.n_tokens * cfg.n_channels, "z")
    s = alloc_scales(cfg)
    lib().cfo_scales(ctypes.byref(cfg.c()), _p(z), _p(s))
    return s


def select(cfg: Config, z, s) -> np.ndarray:
    _chk(z, np.float32, cfg.n_tokens * cfg.n_channels, "z")
    code = np.empty(cfg.shape, dtype=np.uint8)
    lib().cfo_select(ctypes.byref(cfg.c()), _p(z), _p(s), _p(code))
    return code


def pack(cfg: Config, code) -> np.ndarray:
    _chk(code, np.uint8, cfg.n_tokens * cfg.n_channels, "code")
    out = alloc_codes(cfg)
    lib().cfo_pack(ctypes.byref(cfg.c()), _p(code), _p(out))
    return out


def unpack(cfg: Config, packed) -> np.ndarray:
    _chk(packed, np.uint8, cfg.n_tokens * cfg.n_channels * cfg.bits // 8, "packed")
    code = np.empty(cfg.shape, dtype=np.uint8)
    lib().cfo_unpack(ctypes.byref(cfg.c()), _p(packed), _p(code))
    return code


def decode(cfg: Config, code, s) -> np.ndarray:
    _chk(code, np.uint8, cfg.n_tokens * cfg.n_channels, "code")
    d = np.empty(cfg.shape, dtype=np.float32)
    lib().cfo_decode(ctypes.byref(cfg.c()), _p(code), _p(s), _p(d))
    return d


# ---------------------------------------------------------------- N:M block sparsifier stages

def nm_select(cfg: Config, z) -> np.ndarray:
    _chk(z, np.float32, cfg.n_tokens * cfg.n_channels, "z")
    keep = np.empty(cfg.shape, dtype=np.uint8)
    lib().cfo_nm_select(ctypes.byref(cfg.c()), _p(z), _p(keep))
    return keep


def nm_pack(cfg: Config, z, keep) -> np.ndarray:
    _chk(z, np.float32, cfg.n_tokens * cfg.n_channels, "z")
    _chk(keep, np.uint8, cfg.n_tokens * cfg.n_channels, "keep")
    wire = alloc_codes(cfg)
    lib().cfo_nm_pack(ctypes.byref(cfg.c()), _p(z), _p(keep), _p(wire))
    return wire


def nm_unpack(cfg: Config, wire) -> np.ndarray:
    _chk(wire, np.uint8, codes_bytes(cfg), "wire")
    d = np.empty(cfg.shape, dtype=np.float32)
    lib().cfo_nm_unpack(ctypes.byref(cfg.c()), _p(wire), _p(d))
    return d


def nm_values_offset(cfg: Config) -> int:
    return int(lib().cfo_nm_values_offset(ctypes.byref(cfg.c())))


# ---------------------------------------------------------------- whole operations

def _state_chk(cfg, x=None, recon=None, err=None):
    n = cfg.n_tokens * cfg.n_channels
    if x is not None: _chk(x, cfg.np_dtype, n, "x")
    if recon is not None: _chk(recon, cfg.np_dtype, n, "recon")
    if err is not None: _chk(err, cfg.np_err_dtype, n, "err")


def _rc(rc):
    if rc != 0:
        raise ValueError("oracle rejected the configuration")


def warmup(cfg: Config, x0):
    """recon_0 = x_0, e_0 = 0.  Returns (recon, err) as new arrays."""
    _state_chk(cfg, x=x0)
    recon = np.empty(cfg.shape, dtype=cfg.np_dtype)
    err = np.empty(cfg.shape, dtype=cfg.np_err_dtype)
    _rc(lib().cfo_warmup(ctypes.byref(cfg.c()), _p(x0), _p(recon), _p(err)))
    return recon, err


def compress(cfg: Config, x, recon, err):
    """Sender half; updates ``err`` in place, returns (codes, scales)."""
    _state_chk(cfg, x, recon, err)
    codes, s = alloc_codes(cfg), alloc_scales(cfg)
    _rc(lib().cfo_compress(ctypes.byref(cfg.c()), _p(x), _p(recon), _p(err), _p(codes), _p(s)))
    return codes, s


def decompress(cfg: Config, codes, s, recon):
    """Receiver half; updates ``recon`` in place."""
    _state_chk(cfg, recon=recon)
    _chk(codes, np.uint8, codes_bytes(cfg), "codes")
    _rc(lib().cfo_decompress(ctypes.byref(cfg.c()), _p(codes), _p(s), _p(recon)))


def step(cfg: Config, x, recon, err):
    """One codec step; updates ``recon`` and ``err`` in place, returns (codes, scales)."""
    _state_chk(cfg, x, recon, err)
    codes, s = alloc_codes(cfg), alloc_scales(cfg)
    _rc(lib().cfo_step(ctypes.byref(cfg.c()), _p(x), _p(recon), _p(err), _p(codes), _p(s)))
    return codes, s


def naive(cfg: Config, x):
    """Naive compression of x itself; returns (recon, codes, scales)."""
    _state_chk(cfg, x=x)
    recon = np.empty(cfg.shape, dtype=cfg.np_dtype)
    codes, s = alloc_codes(cfg), alloc_scales(cfg)
    _rc(lib().cfo_naive(ctypes.byref(cfg.c()), _p(x), _p(recon), _p(codes), _p(s)))
    return recon, codes, s
