"""MI355X-native residual codec of CompactFusion (arxiv 2507.17511).

Thin ctypes binding over ``libcompactfusion.so`` (HIP, gfx950): the functions
here have the names and argument order of ``include/compactfusion.h`` and only
marshal arguments -- every step of the codec runs in the library's kernels.
There is no CPU fallback: if the library is not built, importing it raises.

Device pointers may be given as ints, as objects with ``data_ptr()`` (torch
tensors), or as a ready ``PtrArray`` built once with :func:`ptr_array`.
"""
from __future__ import annotations

import ctypes
import os
from typing import Iterable, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("CF_LIBRARY") or os.path.join(_HERE, "libcompactfusion.so")   # override: developer builds

# cf_status
CF_OK, CF_ERR_INVALID_ARG, CF_ERR_SHAPE, CF_ERR_UNSUPPORTED, CF_ERR_STATE, CF_ERR_WORKSPACE, CF_ERR_DEVICE = range(7)
# cf_dtype
CF_F32, CF_BF16 = 0, 1
# cf_scale_kind
CF_SCALE_CHANNEL, CF_SCALE_GROUP, CF_SCALE_RANK1, CF_SPARSE_NM, CF_LOWRANK = 0, 1, 2, 3, 4
# cf_ef_mode
CF_EF_RECON, CF_EF_LITERAL, CF_EF_OFF, CF_EF_NAIVE = 0, 1, 2, 3
CF_FLAG_SINGLE_PASS = 0x1
CF_FLAG_TWO_KERNEL = 0x2
CF_FLAG_LOWRANK_INT4 = 0x4
CF_FLAG_FIXED_GRID = 0x8
CF_FLAG_TEST_NO_WAIT = 0x100

EXPORTS = ["cf_sizes", "cf_workspace_bytes", "cf_init", "cf_warmup", "cf_set_warm", "cf_compress",
           "cf_decompress", "cf_step_fused", "cf_destroy", "cf_status_string", "cf_last_hip_error",
           "cf_profile_next_call", "cf_profile_launch_count", "cf_profile_kernel_name", "cf_check_device",
           "cf_step_fused_static", "cf_given_up_items"]


class cf_tensor_desc(ctypes.Structure):
    _fields_ = [("n_tokens", ctypes.c_int64), ("n_channels", ctypes.c_int64), ("dtype", ctypes.c_int32),
                ("bits", ctypes.c_int32), ("scale", ctypes.c_int32), ("group", ctypes.c_int32)]


class cf_options(ctypes.Structure):
    _fields_ = [("ef", ctypes.c_int32), ("err_dtype", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("tile_rows", ctypes.c_int32), ("encode_rows", ctypes.c_int32)]


class CFError(RuntimeError):
    def __init__(self, status: int, where: str, hip: int = 0):
        self.status = status
        self.hip_error = hip
        msg = cf_status_string(status)
        super().__init__(f"{where}: {msg} (cf_status {status}" + (f", hipError {hip})" if hip else ")"))


_lib = None


def lib() -> ctypes.CDLL:
    """Loads the built library; never builds and never falls back."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2507_17511_amd.build` "
                              "(or __graft_entry__.build()) first; there is no CPU fallback")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        dp, op = ctypes.POINTER(cf_tensor_desc), ctypes.POINTER(cf_options)
        pp = ctypes.POINTER(ctypes.c_void_p)
        szp = ctypes.POINTER(sz)
        L.cf_sizes.restype = i32
        L.cf_sizes.argtypes = [dp, op, szp, szp, szp, szp]
        L.cf_workspace_bytes.restype = sz
        L.cf_workspace_bytes.argtypes = [dp, i32, op]
        L.cf_init.restype = i32
        L.cf_init.argtypes = [pp, dp, i32, op, vp, sz, vp]
        L.cf_warmup.restype = i32
        L.cf_warmup.argtypes = [vp, i32, i32, pp, pp, pp, vp]
        L.cf_set_warm.restype = i32
        L.cf_set_warm.argtypes = [vp, i32, i32, i32]
        L.cf_compress.restype = i32
        L.cf_compress.argtypes = [vp, i32, i32, pp, pp, pp, pp, pp, vp]
        L.cf_decompress.restype = i32
        L.cf_decompress.argtypes = [vp, i32, i32, pp, pp, pp, vp]
        L.cf_step_fused.restype = i32
        L.cf_step_fused.argtypes = [vp, i32, i32, pp, pp, pp, pp, pp, vp]
        L.cf_destroy.restype = None
        L.cf_destroy.argtypes = [vp]
        L.cf_status_string.restype = ctypes.c_char_p
        L.cf_status_string.argtypes = [i32]
        L.cf_last_hip_error.restype = i32
        L.cf_last_hip_error.argtypes = [vp]
        L.cf_check_device.restype = i32
        L.cf_check_device.argtypes = [vp, vp]
        L.cf_profile_next_call.restype = i32
        L.cf_profile_next_call.argtypes = [vp, pp, i32]
        L.cf_profile_launch_count.restype = i32
        L.cf_profile_launch_count.argtypes = [vp]
        L.cf_profile_kernel_name.restype = ctypes.c_char_p
        L.cf_profile_kernel_name.argtypes = [vp, i32]
        L.cf_given_up_items.restype = i32
        L.cf_given_up_items.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_uint32)]
        L.cf_step_fused_static.restype = i32
        L.cf_step_fused_static.argtypes = [dp, i32, op, pp, pp, pp, pp, pp, vp]
        _lib = L
    return _lib


# ---------------------------------------------------------------- marshalling

def _addr(p) -> Optional[int]:
    if p is None:
        return None
    if hasattr(p, "data_ptr"):
        return p.data_ptr()
    return int(p)


def ptr_array(ptrs: Iterable):
    """A host array of device pointers, reusable across calls."""
    addrs = [_addr(p) for p in ptrs]
    return (ctypes.c_void_p * len(addrs))(*addrs)


def _pa(ptrs):
    if ptrs is None:
        return None
    if isinstance(ptrs, ctypes.Array):
        return ptrs
    return ptr_array(ptrs)


def _descs(descs: Sequence[cf_tensor_desc]):
    if isinstance(descs, ctypes.Array):
        return descs
    return (cf_tensor_desc * len(descs))(*descs)


def _check(status: int, where: str, ctx=None):
    if status != CF_OK:
        hip = lib().cf_last_hip_error(ctx) if (ctx and status == CF_ERR_DEVICE) else 0
        raise CFError(status, where, hip)


def desc(n_tokens: int, n_channels: int, dtype: int = CF_BF16, bits: int = 2, scale: int = CF_SCALE_CHANNEL,
         group: int = 128) -> cf_tensor_desc:
    return cf_tensor_desc(n_tokens, n_channels, dtype, bits, scale, group)


def options(ef: int = CF_EF_RECON, err_dtype: int = CF_F32, flags: int = 0, tile_rows: int = 0,
            encode_rows: int = 0) -> cf_options:
    return cf_options(ef, err_dtype, flags, tile_rows, encode_rows)


# ---------------------------------------------------------------- the C entry points

def cf_status_string(status: int) -> str:
    return lib().cf_status_string(status).decode()


def cf_sizes(d: cf_tensor_desc, opts: Optional[cf_options] = None):
    """-> (codes_bytes, scales_bytes, recon_bytes, err_bytes)"""
    out = [ctypes.c_size_t() for _ in range(4)]
    st = lib().cf_sizes(ctypes.byref(d), ctypes.byref(opts) if opts else None, *[ctypes.byref(o) for o in out])
    _check(st, "cf_sizes")
    return tuple(o.value for o in out)


def cf_workspace_bytes(descs, opts: Optional[cf_options] = None) -> int:
    arr = _descs(descs)
    return int(lib().cf_workspace_bytes(arr, len(arr), ctypes.byref(opts) if opts else None))


def cf_init(descs, opts: Optional[cf_options], workspace, workspace_bytes: int, stream=None):
    """-> opaque context handle (release with cf_destroy)"""
    arr = _descs(descs)
    ctx = ctypes.c_void_p()
    st = lib().cf_init(ctypes.byref(ctx), arr, len(arr), ctypes.byref(opts) if opts else None,
                       _addr(workspace), workspace_bytes, _addr(stream))
    _check(st, "cf_init")
    return ctx


def cf_destroy(ctx) -> None:
    lib().cf_destroy(ctx)


def cf_last_hip_error(ctx) -> int:
    return int(lib().cf_last_hip_error(ctx))


def cf_set_warm(ctx, first: int, count: int, warm: bool = True) -> None:
    _check(lib().cf_set_warm(ctx, first, count, 1 if warm else 0), "cf_set_warm", ctx)


def cf_warmup(ctx, first: int, count: int, x0, recon, err, stream=None) -> None:
    _check(lib().cf_warmup(ctx, first, count, _pa(x0), _pa(recon), _pa(err), _addr(stream)), "cf_warmup", ctx)


def cf_compress(ctx, first: int, count: int, x, recon, err, codes, scales, stream=None) -> None:
    _check(lib().cf_compress(ctx, first, count, _pa(x), _pa(recon), _pa(err), _pa(codes), _pa(scales),
                             _addr(stream)), "cf_compress", ctx)


def cf_decompress(ctx, first: int, count: int, codes, scales, recon, stream=None) -> None:
    _check(lib().cf_decompress(ctx, first, count, _pa(codes), _pa(scales), _pa(recon), _addr(stream)),
           "cf_decompress", ctx)


def cf_step_fused(ctx, first: int, count: int, x, recon, err, codes, scales, stream=None) -> None:
    _check(lib().cf_step_fused(ctx, first, count, _pa(x), _pa(recon), _pa(err), _pa(codes), _pa(scales),
                               _addr(stream)), "cf_step_fused", ctx)


CF_STATIC_SCRATCH_BYTES = 16 << 20


def cf_step_fused_static(descs, opts: Optional[cf_options], x, recon, err, codes, scales, stream=None) -> None:
    """One whole codec step over all tensors with the library's own static scratch: no context, no workspace,
    no allocation."""
    arr = _descs(descs)
    _check(lib().cf_step_fused_static(arr, len(arr), ctypes.byref(opts) if opts else None, _pa(x), _pa(recon), _pa(err),
                                      _pa(codes), _pa(scales), _addr(stream)), "cf_step_fused_static")


def cf_profile_next_call(ctx, events, n_pairs: int) -> None:
    """events: sequence of 2*n_pairs hipEvent_t handles (ints) or None to switch off."""
    _check(lib().cf_profile_next_call(ctx, _pa(events) if events is not None else None, n_pairs),
           "cf_profile_next_call", ctx)


def cf_profile_launch_count(ctx) -> int:
    return int(lib().cf_profile_launch_count(ctx))


def cf_profile_kernel_name(ctx, k: int) -> Optional[str]:
    name = lib().cf_profile_kernel_name(ctx, k)
    return name.decode() if name else None


def cf_check_device(ctx, stream=None) -> None:
    """Synchronises the stream; raises if that fails or the device-side consistency check tripped."""
    _check(lib().cf_check_device(ctx, _addr(stream)), "cf_check_device", ctx)


def cf_given_up_items(ctx, stream=None) -> int:
    """Synchronises the stream; -> items of the last single pass that were given up and done by the second launch."""
    n = ctypes.c_uint32()
    _check(lib().cf_given_up_items(ctx, _addr(stream), ctypes.byref(n)), "cf_given_up_items", ctx)
    return int(n.value)
