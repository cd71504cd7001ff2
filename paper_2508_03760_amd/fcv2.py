"""Thin ctypes binding of the C-ABI library libfcv2 (include/fcv2.h).  Same names as the C entry points.

Argument marshalling only: torch supplies device memory and the current HIP stream, every step of the codec
runs in the library's kernels.  There is no CPU fallback: if the library cannot be loaded, calls raise.
"""
import ctypes as C
import os
from dataclasses import dataclass

import torch

from . import build as _build

F_SPIKE = 1
F_META_FP32 = 2
F_META_INT = 4
F_IDX_BF16 = 8
DT_BF16 = 0
DT_FP32 = 1
ABSENT = 2**64 - 1
TENSOR_ALIGN = 256
ROW_ALIGN = 16
MAX_PEERS = 16
STATIC_SCRATCH_BYTES = 2 << 20


class Fcv2Error(RuntimeError):
    pass


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
    """Load libfcv2.so.  A built library that matches the sources is loaded as it is; a missing one, or one built from
    other sources than the tree now holds (an edit since the last build), is compiled first.  A failing compile raises:
    there is no other path."""
    global _lib
    if _lib is None:
        path = _build.lib_path()
        if not os.path.exists(path) or not _build.is_current():
            _build.build()
        L = C.CDLL(path)
        fmtp, vp = C.POINTER(_Fmt), C.c_void_p
        L.fcv2_get_layout.argtypes = [C.c_uint64, fmtp, C.c_uint32, C.POINTER(_Layout)]
        L.fcv2_quantize_pack.argtypes = [vp, C.c_uint64, fmtp, vp, vp]
        L.fcv2_unpack_dequant.argtypes = [vp, C.c_uint64, fmtp, vp, C.c_int, vp]
        L.fcv2_quantize_pack_slices.argtypes = [vp, C.c_uint64, C.c_uint32, fmtp, vp, C.c_uint64, vp]
        L.fcv2_unpack_dequant_slices.argtypes = [C.POINTER(vp), C.c_uint32, C.c_uint64, fmtp, vp, C.c_int, vp]
        L.fcv2_stream_copy.argtypes = [vp, vp, C.c_uint64, vp]  # include/fcv2_diag.h
        L.fcv2_reduce_requant.argtypes = [C.POINTER(vp), C.c_int, C.c_uint64, fmtp, fmtp, vp, vp, vp]
        L.fcv2_dispatch_workspace_bytes.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32, C.POINTER(C.c_size_t)]
        L.fcv2_dispatch_quant.argtypes = [vp, vp, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, fmtp, vp, vp, vp,
                                          vp, C.c_size_t, vp]
        L.fcv2_dispatch_quant_noalloc.argtypes = [vp, vp, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, fmtp, vp, vp, vp, vp]
        L.fcv2_status_string.argtypes = [C.c_int]
        L.fcv2_status_string.restype = C.c_char_p
        L.fcv2_version.restype = C.c_int
        _lib = L
    return _lib


def _check(rc, what):
    if rc != 0:
        raise Fcv2Error(f"{what}: {lib().fcv2_status_string(rc).decode()} ({rc})")


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t: torch.Tensor, what: str):
    if not t.is_cuda or not t.is_contiguous():
        raise Fcv2Error(f"{what} must be a contiguous device tensor")
    return C.c_void_p(t.data_ptr())


def version() -> int:
    return lib().fcv2_version()


def get_layout(n, bits, group, flags, section_align=TENSOR_ALIGN) -> Layout:
    out = _Layout()
    _check(lib().fcv2_get_layout(n, C.byref(_Fmt(bits, group, flags)), section_align, C.byref(out)), "fcv2_get_layout")
    return Layout(*(getattr(out, k) for k, _ in _Layout._fields_))


def quantize_pack(x: torch.Tensor, bits, group, flags, out: torch.Tensor = None) -> torch.Tensor:
    """x: bf16 device tensor (any shape, contiguous).  Returns the packed record as a uint8 device tensor."""
    if x.dtype != torch.bfloat16:
        raise Fcv2Error("x must be bfloat16")
    n = x.numel()
    L = get_layout(n, bits, group, flags)
    if out is None:
        out = torch.zeros(L.total_bytes, dtype=torch.uint8, device=x.device)
    elif out.numel() < L.total_bytes or out.dtype != torch.uint8:
        raise Fcv2Error("out must be a uint8 tensor of at least total_bytes")
    _check(lib().fcv2_quantize_pack(_dev(x, "x"), n, C.byref(_Fmt(bits, group, flags)), _dev(out, "out"), _stream()),
           "fcv2_quantize_pack")
    return out


def unpack_dequant(packed: torch.Tensor, n, bits, group, flags, out_dtype=torch.float32,
                   out: torch.Tensor = None) -> torch.Tensor:
    L = get_layout(n, bits, group, flags)
    if packed.dtype != torch.uint8 or packed.numel() < L.total_bytes:
        raise Fcv2Error("packed must be a uint8 tensor of at least total_bytes")
    if out_dtype not in (torch.float32, torch.bfloat16):
        raise Fcv2Error("out_dtype must be float32 or bfloat16")
    if out is None:
        out = torch.empty(n, dtype=out_dtype, device=packed.device)
    elif out.numel() != n or out.dtype != out_dtype:
        raise Fcv2Error("out has the wrong size or dtype")
    _check(lib().fcv2_unpack_dequant(_dev(packed, "packed"), n, C.byref(_Fmt(bits, group, flags)), _dev(out, "out"),
                                     DT_FP32 if out_dtype == torch.float32 else DT_BF16, _stream()),
           "fcv2_unpack_dequant")
    return out


def quantize_pack_slices(x: torch.Tensor, n_slices, bits, group, flags, out: torch.Tensor = None) -> torch.Tensor:
    """Cut x into n_slices equal slices and pack each into a record of its own.  Returns a uint8 tensor
    [n_slices, record_stride]; row j is the record of slice j."""
    if x.dtype != torch.bfloat16:
        raise Fcv2Error("x must be bfloat16")
    n = x.numel()
    if n_slices < 1 or n % n_slices:
        raise Fcv2Error("n must be a multiple of n_slices")
    L = get_layout(n // n_slices, bits, group, flags)
    if out is None:
        out = torch.zeros((n_slices, L.total_bytes), dtype=torch.uint8, device=x.device)
    elif out.dtype != torch.uint8 or out.dim() != 2 or out.shape[0] != n_slices or out.shape[1] < L.total_bytes:
        raise Fcv2Error("out must be a uint8 tensor [n_slices, >= total_bytes]")
    _check(lib().fcv2_quantize_pack_slices(_dev(x, "x"), n, n_slices, C.byref(_Fmt(bits, group, flags)), _dev(out, "out"),
                                           out.shape[1], _stream()), "fcv2_quantize_pack_slices")
    return out


def unpack_dequant_slices(records, n, bits, group, flags, out_dtype=torch.float32, out: torch.Tensor = None) -> torch.Tensor:
    """records: list of packed uint8 device tensors, record j = slice j of the output of n elements."""
    k = len(records)
    if k < 1 or n % k:
        raise Fcv2Error("n must be a multiple of the number of records")
    L = get_layout(n // k, bits, group, flags)
    for r in records:
        if r.dtype != torch.uint8 or r.numel() < L.total_bytes:
            raise Fcv2Error("every record must be a uint8 tensor of at least total_bytes")
    if out is None:
        out = torch.empty(n, dtype=out_dtype, device=records[0].device)
    arr = (C.c_void_p * k)(*[_dev(r, "record").value for r in records])
    _check(lib().fcv2_unpack_dequant_slices(arr, k, n, C.byref(_Fmt(bits, group, flags)), _dev(out, "out"),
                                            DT_FP32 if out_dtype == torch.float32 else DT_BF16, _stream()),
           "fcv2_unpack_dequant_slices")
    return out


def stream_copy(src: torch.Tensor, dst: torch.Tensor):
    """Diagnostic: plain streaming copy of src into dst (same byte size, a multiple of 16)."""
    nbytes = src.numel() * src.element_size()
    if nbytes != dst.numel() * dst.element_size():
        raise Fcv2Error("src and dst differ in size")
    _check(lib().fcv2_stream_copy(_dev(src, "src"), _dev(dst, "dst"), nbytes, _stream()), "fcv2_stream_copy")


def reduce_requant(peers, n, fmt_in, fmt_out=None, want_sum=False, out: torch.Tensor = None,
                   sum_out: torch.Tensor = None):
    """peers: list of packed uint8 device tensors of format fmt_in = (bits, group, flags).
    Returns packed_out, or (packed_out, fp32 sums) with want_sum."""
    fmt_out = fmt_out or fmt_in
    Lin = get_layout(n, *fmt_in)
    Lout = get_layout(n, *fmt_out)
    if not 1 <= len(peers) <= MAX_PEERS:
        raise Fcv2Error("1..16 peers")
    for p in peers:
        if p.dtype != torch.uint8 or p.numel() < Lin.total_bytes:
            raise Fcv2Error("every peer must be a uint8 tensor of at least total_bytes")
    if out is None:
        out = torch.zeros(Lout.total_bytes, dtype=torch.uint8, device=peers[0].device)
    if want_sum and sum_out is None:
        sum_out = torch.empty(n, dtype=torch.float32, device=peers[0].device)
    arr = (C.c_void_p * len(peers))(*[_dev(p, "peer").value for p in peers])
    _check(lib().fcv2_reduce_requant(arr, len(peers), n, C.byref(_Fmt(*fmt_in)), C.byref(_Fmt(*fmt_out)),
                                     _dev(out, "out"), _dev(sum_out, "sum_out") if sum_out is not None else None,
                                     _stream()), "fcv2_reduce_requant")
    return (out, sum_out) if want_sum else out


def dispatch_workspace_bytes(T, K, E) -> int:
    out = C.c_size_t()
    _check(lib().fcv2_dispatch_workspace_bytes(T, K, E, C.byref(out)), "fcv2_dispatch_workspace_bytes")
    return out.value


def dispatch_quant(x: torch.Tensor, topk_ids: torch.Tensor, E, bits, group, flags, send_buf=None,
                   expert_offsets=None, row_src=None, workspace=None):
    """x: [T, H] bf16, topk_ids: [T, K] int32 (device).  Returns send_buf [T*K, row_bytes] uint8,
    expert_offsets [E+1] int32, row_src [T*K] int32 (first expert_offsets[E] entries valid)."""
    T, H = x.shape
    K = topk_ids.shape[1]
    if x.dtype != torch.bfloat16 or topk_ids.dtype != torch.int32 or topk_ids.shape[0] != T:
        raise Fcv2Error("x must be [T,H] bfloat16 and topk_ids [T,K] int32")
    L = get_layout(H, bits, group, flags, ROW_ALIGN)
    dev = x.device
    if send_buf is None:
        send_buf = torch.zeros((T * K, L.total_bytes), dtype=torch.uint8, device=dev)
    if expert_offsets is None:
        expert_offsets = torch.zeros(E + 1, dtype=torch.int32, device=dev)
    if row_src is None:
        row_src = torch.full((T * K,), -1, dtype=torch.int32, device=dev)
    need = dispatch_workspace_bytes(T, K, E)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    _check(lib().fcv2_dispatch_quant(_dev(x, "x"), _dev(topk_ids, "topk_ids"), T, H, K, E,
                                     C.byref(_Fmt(bits, group, flags)), _dev(send_buf, "send_buf"),
                                     _dev(expert_offsets, "expert_offsets"), _dev(row_src, "row_src"),
                                     _dev(workspace, "workspace"), workspace.numel(), _stream()), "fcv2_dispatch_quant")
    return send_buf, expert_offsets, row_src


def dispatch_quant_noalloc(x: torch.Tensor, topk_ids: torch.Tensor, E, bits, group, flags, send_buf: torch.Tensor,
                           expert_offsets: torch.Tensor, row_src: torch.Tensor):
    """fcv2_dispatch_quant_noalloc: as dispatch_quant, but the planning scratch is the library's static device array.
    The caller passes every output; this binding allocates nothing either."""
    T, H = x.shape
    K = topk_ids.shape[1]
    if x.dtype != torch.bfloat16 or topk_ids.dtype != torch.int32 or topk_ids.shape[0] != T:
        raise Fcv2Error("x must be [T,H] bfloat16 and topk_ids [T,K] int32")
    _check(lib().fcv2_dispatch_quant_noalloc(_dev(x, "x"), _dev(topk_ids, "topk_ids"), T, H, K, E,
                                             C.byref(_Fmt(bits, group, flags)), _dev(send_buf, "send_buf"),
                                             _dev(expert_offsets, "expert_offsets"), _dev(row_src, "row_src"), _stream()),
           "fcv2_dispatch_quant_noalloc")
    return send_buf, expert_offsets, row_src
