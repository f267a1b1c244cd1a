"""ctypes binding of libqesgd.so: the same entry points as include/qesgd.h.

Argument marshalling only.  Tensors are torch tensors on the GPU (torch is used
for device memory and streams, nothing else); every step of the path runs in
the library's kernels.  There is no fallback: if the library has not been built
the first call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqesgd.so")

NORM_L2 = 0
NORM_MAX = 1

OK = 0
ERR_NULL, ERR_DIM, ERR_LEVELS, ERR_BUCKET, ERR_WORKERS = -1, -2, -3, -4, -5
ERR_NORM_KIND, ERR_ALIGN, ERR_STRIDE, ERR_WORKSPACE, ERR_HIP = -6, -7, -8, -9, -10
ERR_BITS, ERR_DELTA, ERR_ROUNDS, ERR_SCRATCH = -11, -12, -13, -14
NOALLOC_SCRATCH_BYTES = 4 << 20


class QesgdError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (code {code})")


class _Layout(C.Structure):
    _fields_ = [("n_buckets", C.c_uint64), ("level_bits", C.c_uint32), ("reserved", C.c_uint32),
                ("sign_words", C.c_uint64), ("level_words", C.c_uint64),
                ("norms_off", C.c_uint64), ("signs_off", C.c_uint64), ("levels_off", C.c_uint64),
                ("bytes_per_worker", C.c_uint64), ("payload_bytes", C.c_uint64)]


@dataclass(frozen=True)
class Layout:
    n_buckets: int
    level_bits: int
    sign_words: int
    level_words: int
    norms_off: int
    signs_off: int
    levels_off: int
    bytes_per_worker: int
    payload_bytes: int


_lib = None


def lib():
    """Loads libqesgd.so once; raises if it is missing (there is no other path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: build it with "
                               "`python -m paper_1901_03040_amd.build` (hipcc, gfx950)")
        L = C.CDLL(LIB_PATH)
        u32, u64, vp, sz = C.c_uint32, C.c_uint64, C.c_void_p, C.c_size_t
        L.qesgd_layout_query.argtypes = [u64, u32, u64, C.POINTER(_Layout)]
        L.qesgd_layout_query.restype = C.c_int
        L.qesgd_workspace_bytes.argtypes = [u64, u32, u64, u32]
        L.qesgd_workspace_bytes.restype = sz
        L.qesgd_quantize_pack.argtypes = [vp, vp, u64, u32, u64, u32, u64, u32, u32, vp, vp, sz, vp]
        L.qesgd_quantize_pack.restype = C.c_int
        L.qesgd_quantize_pack_batched.argtypes = [vp, u64, vp, u64, u32, u64, u32, u64, u32, u32,
                                                  vp, u64, vp, sz, vp]
        L.qesgd_quantize_pack_batched.restype = C.c_int
        L.qesgd_quantize_pack_batched_noalloc.argtypes = [vp, u64, vp, u64, u32, u64, u32, u64, u32, u32,
                                                          vp, u64, vp]
        L.qesgd_quantize_pack_batched_noalloc.restype = C.c_int
        L.qesgd_unpack_aggregate.argtypes = [vp, u64, u32, u64, u32, u64, vp, vp]
        L.qesgd_unpack_aggregate.restype = C.c_int
        L.qesgd_apply_update.argtypes = [vp, vp, vp, vp, u64, vp]
        L.qesgd_apply_update.restype = C.c_int
        L.qesgd_unpack_aggregate_update.argtypes = [vp, u64, u32, u64, u32, u64, vp, vp, vp, vp, vp]
        L.qesgd_unpack_aggregate_update.restype = C.c_int
        L.qesgd_round.argtypes = [vp, u64, vp, u64, u32, u64, u32, u64, u32, u32, vp, u64, vp, sz, vp, vp, vp, vp, vp]
        L.qesgd_round.restype = C.c_int
        L.qesgd_quantize_fixed.argtypes = [vp, vp, u64, C.c_float, u32, u64, u32, u32, vp, vp]
        L.qesgd_quantize_fixed.restype = C.c_int
        L.qesgd_dequantize_fixed_update.argtypes = [vp, u64, C.c_float, u32, vp, vp, vp, vp, vp]
        L.qesgd_dequantize_fixed_update.restype = C.c_int
        L.qesgd_epoch_commit.argtypes = [vp, vp, u32, u64, vp]
        L.qesgd_epoch_commit.restype = C.c_int
        L.qesgd_strerror.argtypes = [C.c_int]
        L.qesgd_strerror.restype = C.c_char_p
        L.qesgd_last_hip_error.argtypes = []
        L.qesgd_last_hip_error.restype = C.c_int
        L.qesgd_abi_version.argtypes = []
        L.qesgd_abi_version.restype = u32
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().qesgd_strerror(int(code)).decode()


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream) -> Optional[C.c_void_p]:
    """torch stream, raw hipStream_t handle (int), or None = torch's current stream."""
    if isinstance(stream, int):
        return C.c_void_p(stream)
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check(rc: int, where: str):
    if rc != OK:
        raise QesgdError(rc, where)


def qesgd_layout_query(d: int, s: int, bucket: int) -> Layout:
    out = _Layout()
    _check(lib().qesgd_layout_query(int(d), int(s), int(bucket), C.byref(out)), "qesgd_layout_query")
    return Layout(out.n_buckets, out.level_bits, out.sign_words, out.level_words, out.norms_off,
                  out.signs_off, out.levels_off, out.bytes_per_worker, out.payload_bytes)


def qesgd_workspace_bytes(d: int, s: int, bucket: int, K: int) -> int:
    return int(lib().qesgd_workspace_bytes(int(d), int(s), int(bucket), int(K)))


def qesgd_quantize_pack(x, center, d, s, bucket, norm_kind, seed, rnd, worker, packed,
                        workspace=None, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().qesgd_quantize_pack(_ptr(x), _ptr(center), int(d), int(s), int(bucket), int(norm_kind),
                                     int(seed), int(rnd), int(worker), _ptr(packed), _ptr(workspace),
                                     ws_bytes, _stream(stream)), "qesgd_quantize_pack")


def qesgd_quantize_pack_batched(x_slab, x_stride, center, d, s, bucket, norm_kind, seed, rnd, K,
                                packed_slab, packed_stride, workspace=None, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().qesgd_quantize_pack_batched(_ptr(x_slab), int(x_stride), _ptr(center), int(d), int(s),
                                             int(bucket), int(norm_kind), int(seed), int(rnd), int(K),
                                             _ptr(packed_slab), int(packed_stride), _ptr(workspace),
                                             ws_bytes, _stream(stream)), "qesgd_quantize_pack_batched")


def qesgd_quantize_pack_batched_noalloc(x_slab, x_stride, center, d, s, bucket, norm_kind, seed, rnd, K,
                                        packed_slab, packed_stride, stream=None):
    _check(lib().qesgd_quantize_pack_batched_noalloc(_ptr(x_slab), int(x_stride), _ptr(center), int(d), int(s),
                                                     int(bucket), int(norm_kind), int(seed), int(rnd), int(K),
                                                     _ptr(packed_slab), int(packed_stride), _stream(stream)),
           "qesgd_quantize_pack_batched_noalloc")


def qesgd_unpack_aggregate(packed_slab, packed_stride, K, d, s, bucket, zbar, stream=None):
    _check(lib().qesgd_unpack_aggregate(_ptr(packed_slab), int(packed_stride), int(K), int(d), int(s),
                                        int(bucket), _ptr(zbar), _stream(stream)), "qesgd_unpack_aggregate")


def qesgd_apply_update(w_snap, zbar, u_out, zsum_inout, d, stream=None):
    _check(lib().qesgd_apply_update(_ptr(w_snap), _ptr(zbar), _ptr(u_out), _ptr(zsum_inout), int(d),
                                    _stream(stream)), "qesgd_apply_update")


def qesgd_unpack_aggregate_update(packed_slab, packed_stride, K, d, s, bucket, w_snap, zbar_out, u_out,
                                  zsum_inout, stream=None):
    _check(lib().qesgd_unpack_aggregate_update(_ptr(packed_slab), int(packed_stride), int(K), int(d),
                                               int(s), int(bucket), _ptr(w_snap), _ptr(zbar_out),
                                               _ptr(u_out), _ptr(zsum_inout), _stream(stream)),
           "qesgd_unpack_aggregate_update")


def qesgd_round(x_slab, x_stride, center, d, s, bucket, norm_kind, seed, rnd, K, packed_slab, packed_stride,
                w_snap, zbar_out, u_out, zsum_inout, workspace=None, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().qesgd_round(_ptr(x_slab), int(x_stride), _ptr(center), int(d), int(s), int(bucket), int(norm_kind),
                             int(seed), int(rnd), int(K), _ptr(packed_slab), int(packed_stride), _ptr(workspace),
                             ws_bytes, _ptr(w_snap), _ptr(zbar_out), _ptr(u_out), _ptr(zsum_inout), _stream(stream)),
           "qesgd_round")


def qesgd_quantize_fixed(x, center, d, delta, b, seed, rnd, worker, codes, stream=None):
    _check(lib().qesgd_quantize_fixed(_ptr(x), _ptr(center), int(d), float(delta), int(b), int(seed), int(rnd),
                                      int(worker), _ptr(codes), _stream(stream)), "qesgd_quantize_fixed")


def qesgd_dequantize_fixed_update(codes, d, delta, b, w_snap, z_out, u_out, zsum_inout, stream=None):
    _check(lib().qesgd_dequantize_fixed_update(_ptr(codes), int(d), float(delta), int(b), _ptr(w_snap), _ptr(z_out),
                                               _ptr(u_out), _ptr(zsum_inout), _stream(stream)),
           "qesgd_dequantize_fixed_update")


def qesgd_epoch_commit(w_inout, zsum_inout, rounds, d, stream=None):
    _check(lib().qesgd_epoch_commit(_ptr(w_inout), _ptr(zsum_inout), int(rounds), int(d), _stream(stream)),
           "qesgd_epoch_commit")


def qesgd_abi_version() -> int:
    return int(lib().qesgd_abi_version())


def qesgd_last_hip_error() -> int:
    return int(lib().qesgd_last_hip_error())


# ---- allocation helpers (torch is the allocator) ---------------------------

def alloc_packed(lay: Layout, K: int, device="cuda") -> torch.Tensor:
    """[K, bytes_per_worker] uint8, 256-byte aligned rows (torch's allocator aligns to 512)."""
    t = torch.empty((K, lay.bytes_per_worker), dtype=torch.uint8, device=device)
    assert t.data_ptr() % 256 == 0
    return t


def planes(packed_row: torch.Tensor, lay: Layout):
    """Views (norms f32[nb], signs i32[sign_words], levels i32[level_words]) of one packed block."""
    norms = packed_row[lay.norms_off: lay.norms_off + 4 * lay.n_buckets].view(torch.float32)
    signs = packed_row[lay.signs_off: lay.signs_off + 4 * lay.sign_words].view(torch.int32)
    levels = packed_row[lay.levels_off: lay.levels_off + 4 * lay.level_words].view(torch.int32)
    return norms, signs, levels
