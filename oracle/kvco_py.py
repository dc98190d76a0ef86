"""ctypes binding of the CPU oracle (oracle/kvco.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's CPU-baseline leg.  Works on numpy arrays in host memory; 16-bit
floating point tensors travel as uint16 bit patterns.
"""
import ctypes as C
import os

import numpy as np

from . import build_oracle

_lib = None


class Layout(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("L", "H", "D", "dtype", "T", "th", "tw", "TX", "TY", "k_mode", "v_mode", "seg")]


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build_oracle.ensure_current())  # rebuilt when stale: see build_oracle
        i64, p = C.c_int64, C.c_void_p
        LP = C.POINTER(Layout)
        _lib.kvco_check.argtypes = [LP]
        for f in ("kvco_frames_per_group", "kvco_frame_bytes", "kvco_meta_floats"):
            getattr(_lib, f).argtypes = [LP]
            getattr(_lib, f).restype = i64
        _lib.kvco_meta_kind_offset.argtypes = [LP, C.c_int]
        _lib.kvco_meta_kind_offset.restype = i64
        _lib.kvco_frame_offset.argtypes = [LP, C.c_int, C.c_int, i64, C.c_int, C.c_int]
        _lib.kvco_frame_offset.restype = i64
        _lib.kvco_meta_offset.argtypes = [LP, C.c_int, C.c_int, i64, C.c_int, C.c_int]
        _lib.kvco_meta_offset.restype = i64
        _lib.kvco_widen.argtypes = [C.c_uint16, C.c_int]
        _lib.kvco_widen.restype = C.c_float
        _lib.kvco_narrow.argtypes = [C.c_float, C.c_int]
        _lib.kvco_narrow.restype = C.c_uint16
        _lib.kvco_group_params.argtypes = [p, i64, p, p, p]
        _lib.kvco_group_params.restype = None
        _lib.kvco_quantize.argtypes = [C.c_float, C.c_float, C.c_float]
        _lib.kvco_quantize.restype = C.c_uint8
        _lib.kvco_dequantize.argtypes = [C.c_uint8, C.c_float, C.c_float]
        _lib.kvco_dequantize.restype = C.c_float
        _lib.kvco_pack.argtypes = [LP, p, i64, i64, i64, i64, p, p]
        _lib.kvco_restore.argtypes = [LP, p, p, i64, p, i64, i64, i64]
        _lib.kvco_restore_paged.argtypes = [LP, p, p, i64, i64, p, i64, C.c_int32, p, i64, p]
        _lib.kvco_restore_paged_frame.argtypes = [LP, p, p, C.c_int, C.c_int, C.c_int, i64, i64, p, i64, C.c_int32, p, i64, p]
        _lib.kvco_threads.restype = C.c_int
    return _lib


def make_layout(L, H, D, dtype, T, th, tw, TX, TY, k_mode=0, v_mode=1, seg=0):
    """seg = d2 of the two-level tiling of Sec. 3.2.2 (0: the row-major retile)."""
    return Layout(L, H, D, dtype, T, th, tw, TX, TY, k_mode, v_mode, seg)


def frames_per_group(lo):
    return lib().kvco_frames_per_group(C.byref(lo))


def frame_bytes(lo):
    return lib().kvco_frame_bytes(C.byref(lo))


def meta_floats(lo):
    return lib().kvco_meta_floats(C.byref(lo))


def meta_kind_offset(lo, kind):
    return lib().kvco_meta_kind_offset(C.byref(lo), kind)


def frame_offset(lo, kind, l, t, h, d):
    return lib().kvco_frame_offset(C.byref(lo), kind, l, t, h, d)


def meta_offset(lo, kind, l, t, h, d):
    return lib().kvco_meta_offset(C.byref(lo), kind, l, t, h, d)


def widen(bits, dtype):
    return lib().kvco_widen(int(bits), dtype)


def narrow(x, dtype):
    return lib().kvco_narrow(float(np.float32(x)), dtype)


def group_params(xs):
    xs = np.ascontiguousarray(xs, dtype=np.float32)
    out = (C.c_float * 3)()
    base = C.addressof(out)
    lib().kvco_group_params(xs.ctypes.data, xs.size, base, base + 4, base + 8)
    return np.float32(out[0]), np.float32(out[1]), np.float32(out[2])  # scale, mn, inv


def quantize(x, mn, inv):
    return lib().kvco_quantize(float(np.float32(x)), float(np.float32(mn)), float(np.float32(inv)))


def dequantize(code, scale, mn):
    return np.float32(lib().kvco_dequantize(int(code), float(np.float32(scale)), float(np.float32(mn))))


def threads():
    return lib().kvco_threads()


def n_chunks(lo, n_tokens):
    return (n_tokens + lo.T - 1) // lo.T


def _contig_strides(lo, n_tokens):
    Cc = lo.H * lo.D
    return 2 * n_tokens * Cc, n_tokens * Cc, Cc


def pack(lo, kv_u16, n_tokens, strides=None):
    """kv_u16: uint16 array holding [L][2][n_tokens][H][D] (contiguous unless strides given).
    Returns (frames uint8 [n_chunks*frame_bytes], meta float32 [n_chunks*meta_floats])."""
    assert kv_u16.dtype == np.uint16 and kv_u16.flags.c_contiguous
    ls, ks, ts = strides if strides is not None else _contig_strides(lo, n_tokens)
    nc = n_chunks(lo, n_tokens)
    frames = np.full(nc * frame_bytes(lo), 0xA5, dtype=np.uint8)  # the oracle must overwrite every byte
    meta = np.full(nc * meta_floats(lo), np.float32(np.nan), dtype=np.float32)
    rc = lib().kvco_pack(C.byref(lo), kv_u16.ctypes.data, ls, ks, ts, n_tokens, frames.ctypes.data, meta.ctypes.data)
    if rc:
        raise ValueError("kvco_pack rejected its arguments")
    return frames, meta


def restore(lo, frames, meta, n_tokens, out=None, strides=None):
    assert frames.dtype == np.uint8 and meta.dtype == np.float32
    ls, ks, ts = strides if strides is not None else _contig_strides(lo, n_tokens)
    if out is None:
        out = np.zeros(lo.L * 2 * n_tokens * lo.H * lo.D, dtype=np.uint16)
    rc = lib().kvco_restore(C.byref(lo), frames.ctypes.data, meta.ctypes.data, n_tokens, out.ctypes.data, ls, ks, ts)
    if rc:
        raise ValueError("kvco_restore rejected its arguments")
    return out


def restore_paged(lo, frames, meta, first_token, n_tokens, caches, num_blocks, block_size, block_table):
    """caches: list of L uint16 arrays, each [2][num_blocks][block_size][H][D]; written in place.
    Returns the error word (bit 0: a block id was out of range)."""
    assert len(caches) == lo.L
    for c in caches:
        assert c.dtype == np.uint16 and c.flags.c_contiguous and c.size == 2 * num_blocks * block_size * lo.H * lo.D
    ptrs = (C.c_void_p * lo.L)(*[c.ctypes.data for c in caches])
    bt = np.ascontiguousarray(block_table, dtype=np.int32)
    err = C.c_uint32(0)
    rc = lib().kvco_restore_paged(C.byref(lo), frames.ctypes.data, meta.ctypes.data, first_token, n_tokens, ptrs,
                                  num_blocks, block_size, bt.ctypes.data, bt.size, C.byref(err))
    if rc:
        raise ValueError("kvco_restore_paged rejected its arguments")
    return err.value


def frame_size(lo):
    """bytes of one frame: three planes"""
    return 3 * lo.TY * lo.th * lo.TX * lo.tw


def frame_start(lo, kind, lg, f):
    """offset of frame (kind, lg, f) inside a chunk's frame section"""
    return frame_offset(lo, kind, 3 * lg, f, 0, 0)


def restore_paged_frame(lo, frame, meta, kind, lg, f, first_token, n_tokens, caches, num_blocks, block_size, block_table):
    assert frame.dtype == np.uint8 and frame.size == frame_size(lo) and meta.dtype == np.float32
    ptrs = (C.c_void_p * lo.L)(*[c.ctypes.data for c in caches])
    bt = np.ascontiguousarray(block_table, dtype=np.int32)
    err = C.c_uint32(0)
    frame = np.ascontiguousarray(frame)
    rc = lib().kvco_restore_paged_frame(C.byref(lo), frame.ctypes.data, meta.ctypes.data, kind, lg, f, first_token,
                                        n_tokens, ptrs, num_blocks, block_size, bt.ctypes.data, bt.size, C.byref(err))
    if rc:
        raise ValueError("kvco_restore_paged_frame rejected its arguments")
    return err.value
