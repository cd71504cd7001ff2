"""ctypes front end of the CPU oracle (oracle/fcv2_oracle.cpp).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by __graft_entry__.smoke() and by the cpu_baseline leg of
bench.py; never by the product package.  Works on numpy arrays; bf16 tensors travel as uint16 bit patterns.
"""
import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build

F_SPIKE = 1
F_META_FP32 = 2
F_META_INT = 4
F_IDX_BF16 = 8
DT_BF16 = 0
DT_FP32 = 1
ABSENT = 2**64 - 1


class _Fmt(C.Structure):
    _fields_ = [("bits", C.c_uint32), ("group", C.c_uint32), ("flags", C.c_uint32)]


class _Layout(C.Structure):
    _fields_ = [(k, C.c_uint64) for k in (
        "n", "n_groups", "total_bytes", "off_plane8", "off_plane4", "off_plane2", "off_plane1",
        "off_scale", "off_zero", "off_spike_val", "off_spike_idx")]


@dataclass(frozen=True)
class Layout:
    n: int
    n_groups: int
    total_bytes: int
    off_plane8: int
    off_plane4: int
    off_plane2: int
    off_plane1: int
    off_scale: int
    off_zero: int
    off_spike_val: int
    off_spike_idx: int


_lib = None


def lib():
    global _lib
    if _lib is None:
        # FCV2_ORACLE_SANITIZE=1: the build with AddressSanitizer and UndefinedBehaviorSanitizer (the process must have
        # been started with the sanitizer runtime preloaded; tests/test_sanitizers.py does that in a child process)
        L = C.CDLL(_build.build(sanitize=os.environ.get("FCV2_ORACLE_SANITIZE") == "1"))
        u8p, u16p, f32p, i32p = (C.POINTER(t) for t in (C.c_uint8, C.c_uint16, C.c_float, C.c_int32))
        fmtp = C.POINTER(_Fmt)
        L.orc_get_layout.argtypes = [C.c_uint64, fmtp, C.c_uint32, C.POINTER(_Layout)]
        L.orc_key.argtypes = [C.c_uint16]
        L.orc_key.restype = C.c_uint32
        L.orc_bf16_rne.argtypes = [C.c_float]
        L.orc_bf16_rne.restype = C.c_uint16
        L.orc_quantize_group.argtypes = [u16p, fmtp, u8p, f32p, f32p, u16p, u8p]
        L.orc_split_pack.argtypes = [u8p, C.c_uint64, fmtp, C.c_uint32, u8p]
        L.orc_unpack_codes.argtypes = [u8p, C.c_uint64, fmtp, C.c_uint32, u8p]
        L.orc_quantize_pack.argtypes = [u16p, C.c_uint64, fmtp, C.c_uint32, u8p]
        L.orc_unpack_dequant.argtypes = [u8p, C.c_uint64, fmtp, C.c_uint32, C.c_void_p, C.c_int]
        L.orc_reduce_requant.argtypes = [C.POINTER(u8p), C.c_int, C.c_uint64, fmtp, fmtp, C.c_uint32, u8p, f32p]
        L.orc_dispatch_quant.argtypes = [u16p, i32p, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, fmtp, u8p,
                                         i32p, i32p]
        L.orc_scale_int.argtypes = [C.c_float]
        L.orc_scale_int.restype = C.c_int
        L.orc_scale_of_int.argtypes = [C.c_int]
        L.orc_scale_of_int.restype = C.c_float
        L.orc_meta_int.argtypes = [C.c_float, C.c_float, C.c_uint32, C.POINTER(C.c_int8), u8p, f32p, f32p]
        _lib = L
    return _lib


def _fmt(bits, group, flags):
    return _Fmt(int(bits), int(group), int(flags))


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def _chk(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with status {rc}")


def get_layout(n, bits, group, flags, align=256) -> Layout:
    out = _Layout()
    _chk(lib().orc_get_layout(n, C.byref(_fmt(bits, group, flags)), align, C.byref(out)), "get_layout")
    return Layout(*(getattr(out, k) for k, _ in _Layout._fields_))


def key(u16) -> int:
    return int(lib().orc_key(int(u16)))


def bf16_rne(v: float) -> int:
    return int(lib().orc_bf16_rne(float(v)))


def scale_int(scale: float) -> int:
    """Eq. 1 with theta = 10, clamped to a signed byte."""
    return int(lib().orc_scale_int(float(scale)))


def scale_of_int(k: int):
    return np.float32(lib().orc_scale_of_int(int(k)))


def meta_int(lo: float, hi: float, bits: int):
    """Integer metadata of a group whose values to quantize span [lo, hi]: (scale_int, zero_int, scale, offset)."""
    k, z, s, zf = C.c_int8(), C.c_uint8(), C.c_float(), C.c_float()
    _chk(lib().orc_meta_int(float(lo), float(hi), bits, C.byref(k), C.byref(z), C.byref(s), C.byref(zf)), "meta_int")
    return int(k.value), int(z.value), np.float32(s.value), np.float32(zf.value)


def quantize_group(x_u16, bits, flags):
    """One group (len(x) = G).  Returns codes, scale, zero, spike_val[2], spike_idx[2]."""
    x = np.ascontiguousarray(x_u16, dtype=np.uint16)
    G = x.size
    codes = np.zeros(G, np.uint8)
    s, z = C.c_float(), C.c_float()
    sv, si = np.zeros(2, np.uint16), np.zeros(2, np.uint8)
    _chk(lib().orc_quantize_group(_p(x, C.c_uint16), C.byref(_fmt(bits, G, flags)), _p(codes, C.c_uint8),
                                  C.byref(s), C.byref(z), _p(sv, C.c_uint16), _p(si, C.c_uint8)), "quantize_group")
    return codes, np.float32(s.value), np.float32(z.value), sv, si


def split_pack(codes, bits, group, flags, align=256):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    L = get_layout(codes.size, bits, group, flags, align)
    out = np.zeros(L.total_bytes, np.uint8)
    _chk(lib().orc_split_pack(_p(codes, C.c_uint8), codes.size, C.byref(_fmt(bits, group, flags)), align,
                              _p(out, C.c_uint8)), "split_pack")
    return out


def unpack_codes(packed, n, bits, group, flags, align=256):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    codes = np.zeros(n, np.uint8)
    _chk(lib().orc_unpack_codes(_p(packed, C.c_uint8), n, C.byref(_fmt(bits, group, flags)), align,
                                _p(codes, C.c_uint8)), "unpack_codes")
    return codes


def quantize_pack(x_u16, bits, group, flags, align=256):
    x = np.ascontiguousarray(x_u16, dtype=np.uint16).reshape(-1)
    L = get_layout(x.size, bits, group, flags, align)
    out = np.zeros(L.total_bytes, np.uint8)
    _chk(lib().orc_quantize_pack(_p(x, C.c_uint16), x.size, C.byref(_fmt(bits, group, flags)), align,
                                 _p(out, C.c_uint8)), "quantize_pack")
    return out


def unpack_dequant(packed, n, bits, group, flags, out_dtype=DT_FP32, align=256):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    L = get_layout(n, bits, group, flags, align)
    if packed.size < L.total_bytes:
        raise ValueError("packed buffer too small")
    out = np.zeros(n, np.float32 if out_dtype == DT_FP32 else np.uint16)
    _chk(lib().orc_unpack_dequant(_p(packed, C.c_uint8), n, C.byref(_fmt(bits, group, flags)), align,
                                  out.ctypes.data_as(C.c_void_p), out_dtype), "unpack_dequant")
    return out


def reduce_requant(peers, n, fmt_in, fmt_out=None, want_sum=False, align=256):
    """peers: list of packed uint8 arrays; fmt_* = (bits, group, flags).  Returns packed_out[, sum fp32]."""
    fmt_out = fmt_out or fmt_in
    peers = [np.ascontiguousarray(p, dtype=np.uint8) for p in peers]
    Lin = get_layout(n, *fmt_in, align)
    for p in peers:
        if p.size < Lin.total_bytes:
            raise ValueError("peer buffer too small")
    Lout = get_layout(n, *fmt_out, align)
    out = np.zeros(Lout.total_bytes, np.uint8)
    arr = (C.POINTER(C.c_uint8) * len(peers))(*[_p(p, C.c_uint8) for p in peers])
    s = np.zeros(n, np.float32) if want_sum else None
    _chk(lib().orc_reduce_requant(arr, len(peers), n, C.byref(_fmt(*fmt_in)), C.byref(_fmt(*fmt_out)), align,
                                  _p(out, C.c_uint8), _p(s, C.c_float) if want_sum else None), "reduce_requant")
    return (out, s) if want_sum else out


def dispatch_quant(x_u16, topk_ids, E, bits, group, flags):
    """x: [T, H] uint16, topk_ids: [T, K] int32 (-1 = dropped).  Returns send_buf[R, row_bytes],
    expert_offsets[E+1], row_src[R]."""
    x = np.ascontiguousarray(x_u16, dtype=np.uint16)
    ids = np.ascontiguousarray(topk_ids, dtype=np.int32)
    T, H = x.shape
    K = ids.shape[1]
    L = get_layout(H, bits, group, flags, 16)
    R = int((ids != -1).sum())
    send = np.zeros((max(R, 1), L.total_bytes), np.uint8)
    offs = np.zeros(E + 1, np.int32)
    src = np.zeros(max(R, 1), np.int32)
    _chk(lib().orc_dispatch_quant(_p(x, C.c_uint16), _p(ids, C.c_int32), T, H, K, E,
                                  C.byref(_fmt(bits, group, flags)), _p(send, C.c_uint8), _p(offs, C.c_int32),
                                  _p(src, C.c_int32)), "dispatch_quant")
    return send[:R], offs, src[:R]
