"""ctypes front end of the CPU oracle (test infrastructure, not product code).

Only tests, the smoke check and the benchmark's cpu_baseline leg import this.
It compiles ``qesgd_oracle.cpp`` with g++ (no fast-math, no FMA contraction) and
passes numpy arrays straight through; no arithmetic of the method lives here.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qesgd_oracle.cpp")
_SO = os.path.join(_HERE, "libqesgd_oracle.so")

CXXFLAGS = ["-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
            "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    """Compile the oracle; returns the path of the shared object."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.run(["g++", *CXXFLAGS, "-o", _SO, _SRC], check=True)
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = C.CDLL(_SO)
        u32, u64, f32, vp = C.c_uint32, C.c_uint64, C.c_float, C.c_void_p
        L.qo_philox4x32_10.argtypes = [vp, vp, vp]
        L.qo_philox4x32_10.restype = None
        L.qo_uniform16.argtypes = [u64, u32, u32, u64]
        L.qo_uniform16.restype = u32
        L.qo_level_bits.argtypes = [u32]
        L.qo_level_bits.restype = C.c_int
        L.qo_shape.argtypes = [u64, u32, u64, vp, vp, vp, vp]
        L.qo_shape.restype = C.c_int
        L.qo_bucket_norm.argtypes = [vp, u64, u64, u32]
        L.qo_bucket_norm.restype = f32
        L.qo_bucket_sumsq.argtypes = [vp, u64, u64]
        L.qo_bucket_sumsq.restype = f32
        L.qo_inverse_step.argtypes = [f32, u32]
        L.qo_inverse_step.restype = f32
        L.qo_round_level.argtypes = [f32, u32]
        L.qo_round_level.restype = u32
        L.qo_quantize_bucket.argtypes = [vp, u64, u64, u64, u32, u32, u64, u32, u32, vp, vp, vp]
        L.qo_quantize_bucket.restype = None
        L.qo_pack.argtypes = [vp, vp, u64, u32, vp, vp]
        L.qo_pack.restype = None
        L.qo_unpack.argtypes = [vp, vp, u64, u32, vp, vp]
        L.qo_unpack.restype = None
        L.qo_quantize_pack.argtypes = [vp, vp, u64, u32, u64, u32, u64, u32, u32, vp, vp, vp]
        L.qo_quantize_pack.restype = C.c_int
        L.qo_unpack_aggregate_range.argtypes = [vp, vp, vp, u32, u64, u32, u64, u64, u64, vp]
        L.qo_unpack_aggregate_range.restype = C.c_int
        L.qo_unpack_aggregate.argtypes = [vp, vp, vp, u32, u64, u32, u64, vp]
        L.qo_unpack_aggregate.restype = C.c_int
        L.qo_apply_update.argtypes = [vp, vp, vp, vp, u64]
        L.qo_apply_update.restype = None
        L.qo_epoch_commit.argtypes = [vp, vp, u32, u64]
        L.qo_epoch_commit.restype = None
        L.qo_fixed_round.argtypes = [f32, f32, u32, u32]
        L.qo_fixed_round.restype = C.c_int32
        L.qo_quantize_fixed.argtypes = [vp, vp, u64, f32, u32, u64, u32, u32, vp]
        L.qo_quantize_fixed.restype = C.c_int
        L.qo_dequantize_fixed_update.argtypes = [vp, u64, f32, u32, vp, vp, vp, vp]
        L.qo_dequantize_fixed_update.restype = C.c_int
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def philox4x32_10(counter, key):
    c = np.ascontiguousarray(counter, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().qo_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def uniform16(seed, rnd, worker, i):
    return int(lib().qo_uniform16(int(seed), int(rnd), int(worker), int(i)))


def shape(d, s, bucket):
    """-> (n_buckets, sign_words, level_words, padded_n, level_bits)."""
    nb, nsw, nlw, N = (C.c_uint64() for _ in range(4))
    rc = lib().qo_shape(int(d), int(s), int(bucket), C.byref(nb), C.byref(nsw), C.byref(nlw), C.byref(N))
    if rc != 0:
        raise ValueError(f"unsupported shape d={d} s={s} bucket={bucket}")
    return nb.value, nsw.value, nlw.value, N.value, lib().qo_level_bits(int(s))


def bucket_norm(v, padded_n, norm_kind=0):
    v = _f32(v)
    return float(lib().qo_bucket_norm(_p(v), v.size, int(padded_n), int(norm_kind)))


def bucket_sumsq(v, padded_n):
    v = _f32(v)
    return float(lib().qo_bucket_sumsq(_p(v), v.size, int(padded_n)))


def inverse_step(norm, s):
    return float(lib().qo_inverse_step(float(np.float32(norm)), int(s)))


def round_level(a, r16):
    return int(lib().qo_round_level(float(np.float32(a)), int(r16)))


def quantize_bucket(v, padded_n, i0, s, seed, rnd, worker, norm_kind=0):
    """-> (norm, level[len] uint32, sign[len] uint8) for one bucket starting at coordinate i0."""
    v = _f32(v)
    level = np.zeros(v.size, dtype=np.uint32)
    sign = np.zeros(v.size, dtype=np.uint8)
    norm = C.c_float()
    lib().qo_quantize_bucket(_p(v), v.size, int(padded_n), int(i0), int(s), int(norm_kind),
                             int(seed), int(rnd), int(worker), C.byref(norm), _p(level), _p(sign))
    return float(norm.value), level, sign


def pack(level, sign, s):
    level = np.ascontiguousarray(level, dtype=np.uint32)
    sign = np.ascontiguousarray(sign, dtype=np.uint8)
    d = level.size
    m = lib().qo_level_bits(int(s))
    sw = np.empty((d + 31) // 32, dtype=np.uint32)
    lw = np.empty((d * m + 31) // 32, dtype=np.uint32)
    lib().qo_pack(_p(level), _p(sign), d, int(s), _p(sw), _p(lw))
    return sw, lw


def unpack(sign_words, level_words, d, s):
    sw = np.ascontiguousarray(sign_words, dtype=np.uint32)
    lw = np.ascontiguousarray(level_words, dtype=np.uint32)
    level = np.empty(d, dtype=np.uint32)
    sign = np.empty(d, dtype=np.uint8)
    lib().qo_unpack(_p(sw), _p(lw), int(d), int(s), _p(level), _p(sign))
    return level, sign


def quantize_pack(x, s, bucket, seed, rnd, worker, center=None, norm_kind=0):
    """-> (norms[nb] f32, sign_words u32, level_words u32) for one worker."""
    x = _f32(x)
    c = None if center is None else _f32(center)
    d = x.size
    assert c is None or c.size >= d, "center is shorter than x"
    nb, nsw, nlw, _, _ = shape(d, s, bucket)
    norms = np.empty(nb, dtype=np.float32)
    sw = np.empty(nsw, dtype=np.uint32)
    lw = np.empty(nlw, dtype=np.uint32)
    rc = lib().qo_quantize_pack(_p(x), _p(c), d, int(s), int(bucket), int(norm_kind),
                                int(seed), int(rnd), int(worker), _p(norms), _p(sw), _p(lw))
    if rc != 0:
        raise ValueError("qo_quantize_pack rejected its arguments")
    return norms, sw, lw


def unpack_aggregate(norms, sign_words, level_words, d, s, bucket, i_begin=0, i_end=None):
    """norms[K,nb], sign_words[K,nsw], level_words[K,nlw] -> zbar[i_begin:i_end]."""
    norms = np.ascontiguousarray(norms, dtype=np.float32)
    sw = np.ascontiguousarray(sign_words, dtype=np.uint32)
    lw = np.ascontiguousarray(level_words, dtype=np.uint32)
    K = norms.shape[0]
    nb, nsw, nlw, _, _ = shape(d, s, bucket)
    assert norms.shape == (K, nb) and sw.shape == (K, nsw) and lw.shape == (K, nlw)
    if i_end is None:
        i_end = d
    zbar = np.empty(i_end - i_begin, dtype=np.float32)
    rc = lib().qo_unpack_aggregate_range(_p(norms), _p(sw), _p(lw), K, int(d), int(s), int(bucket),
                                         int(i_begin), int(i_end), _p(zbar))
    if rc != 0:
        raise ValueError("qo_unpack_aggregate_range rejected its arguments")
    return zbar


def apply_update(w_snap, zbar, zsum=None):
    """-> (u, zsum_new or None); zsum is not modified in place."""
    w = _f32(w_snap)
    z = _f32(zbar)
    assert z.size == w.size, "zbar and w_snap differ in length"
    u = np.empty_like(w)
    zs = None if zsum is None else _f32(zsum).copy()
    assert zs is None or zs.size == w.size, "zsum and w_snap differ in length"
    lib().qo_apply_update(_p(w), _p(z), _p(u), _p(zs), w.size)
    return u, zs


def epoch_commit(w, zsum, rounds):
    """-> (w_next, zsum_reset): w + zsum / rounds, and the zeroed running sum."""
    w = _f32(w).copy()
    zs = _f32(zsum).copy()
    assert zs.size == w.size, "zsum and w differ in length"
    lib().qo_epoch_commit(_p(w), _p(zs), int(rounds), w.size)
    return w, zs


def fixed_round(v, delta, b, r16):
    return int(lib().qo_fixed_round(float(np.float32(v)), float(np.float32(delta)), int(b), int(r16)))


def quantize_fixed(x, delta, b, seed, rnd, worker, center=None):
    """Fixed-grid quantiser of Eq. (1)-(2): -> codes, ceil(d*b/32) uint32 words."""
    x = _f32(x)
    c = None if center is None else _f32(center)
    assert c is None or c.size >= x.size, "center is shorter than x"
    codes = np.empty((x.size * b + 31) // 32, dtype=np.uint32)
    rc = lib().qo_quantize_fixed(_p(x), _p(c), x.size, float(np.float32(delta)), int(b), int(seed), int(rnd),
                                 int(worker), _p(codes))
    if rc != 0:
        raise ValueError("qo_quantize_fixed rejected its arguments")
    return codes


def dequantize_fixed_update(codes, d, delta, b, w_snap=None, zsum=None):
    """-> (z, u or None, zsum_new or None)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint32)
    assert codes.size >= (d * b + 31) // 32, "codes is shorter than ceil(d*b/32) words"
    z = np.empty(d, dtype=np.float32)
    w = None if w_snap is None else _f32(w_snap)
    u = None if w is None else np.empty(d, dtype=np.float32)
    zs = None if zsum is None else _f32(zsum).copy()
    assert (w is None or w.size == d) and (zs is None or zs.size == d), "w_snap / zsum length differs from d"
    rc = lib().qo_dequantize_fixed_update(_p(codes), int(d), float(np.float32(delta)), int(b), _p(w), _p(z), _p(u), _p(zs))
    if rc != 0:
        raise ValueError("qo_dequantize_fixed_update rejected its arguments")
    return z, u, zs
