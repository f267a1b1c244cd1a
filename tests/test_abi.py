"""Host-side checks of the C ABI that need no GPU: the library loads, exports what the
header declares, computes the packed layout, and rejects bad arguments before any HIP call."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "qesgd.h")


@pytest.fixture(scope="module")
def B():
    from paper_1901_03040_amd import binding
    binding.lib()
    return binding


def test_exports_every_declared_symbol(B):
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(qesgd_[a-z_0-9]+)\s*\(", text))
    assert {"qesgd_quantize_pack", "qesgd_unpack_aggregate", "qesgd_apply_update"} <= names
    assert len(names) >= 10
    for n in names:
        assert hasattr(B.lib(), n), n
    assert B.qesgd_abi_version() == 2
    assert B.qesgd_last_hip_error() == 0


def test_error_strings(B):
    for code in range(0, -15, -1):
        assert B.strerror(code) and "unknown" not in B.strerror(code)
    assert "unknown" in B.strerror(-99)


@pytest.mark.parametrize("d,s,bucket,nb,m", [
    (16_384, 4, 16_384, 1, 2), (1_048_576, 16, 512, 2048, 4), (11_173_962, 4, 2048, 5457, 2),
    (25_557_032, 256, 8192, 3120, 8), (138_357_544, 2, 4096, 33_779, 1), (1000, 65536, 96, 11, 16),
    (5, 2, 4096, 1, 1), (1001, 8, 96, 11, 3), (1001, 32, 96, 11, 5), (77, 64, 4096, 1, 6), (33, 128, 32, 2, 7)])
def test_layout(B, d, s, bucket, nb, m):
    lay = B.qesgd_layout_query(d, s, bucket)
    assert (lay.n_buckets, lay.level_bits) == (nb, m)
    assert lay.sign_words == (d + 31) // 32 and lay.level_words == (d * m + 31) // 32
    assert lay.payload_bytes == 4 * (nb + lay.sign_words + lay.level_words)
    offs = [lay.norms_off, lay.signs_off, lay.levels_off, lay.bytes_per_worker]
    assert all(o % 256 == 0 for o in offs) and offs == sorted(offs)
    assert lay.signs_off >= 4 * nb and lay.levels_off - lay.signs_off >= 4 * lay.sign_words
    assert lay.bytes_per_worker - lay.levels_off >= 4 * lay.level_words
    assert lay.bytes_per_worker - lay.payload_bytes < 3 * 256


def test_payload_matches_table(B):
    """Packed bytes per worker of the five configurations (4*nb + 4*ceil(d/32) + 4*ceil(d*m/32))."""
    want = {(16_384, 4, 16_384): 6_148, (1_048_576, 16, 512): 663_552, (11_173_962, 4, 2048): 4_212_068,
            (25_557_032, 256, 8192): 28_764_144, (138_357_544, 2, 4096): 34_724_508}
    for (d, s, b), p in want.items():
        assert B.qesgd_layout_query(d, s, b).payload_bytes == p


def test_layout_errors(B):
    for args, code in [((0, 4, 32), B.ERR_DIM), ((1 << 40, 4, 32), B.ERR_DIM), ((100, 3, 32), B.ERR_LEVELS),
                       ((100, 1, 32), B.ERR_LEVELS), ((100, 4, 0), B.ERR_BUCKET), ((100, 4, 48), B.ERR_BUCKET)]:
        with pytest.raises(B.QesgdError) as e:
            B.qesgd_layout_query(*args)
        assert e.value.code == code
    B.qesgd_layout_query(100, 4, 100)      # bucket >= d needs no multiple of 32
    B.qesgd_layout_query(100, 4, 1000)
    assert B.lib().qesgd_layout_query(100, 4, 32, None) == B.ERR_NULL


def test_workspace_bytes(B):
    assert B.qesgd_workspace_bytes(138_357_544, 2, 4096, 8) == 0
    assert B.qesgd_workspace_bytes(1 << 20, 4, 32768, 8) == 0
    # one bucket of 2^20 coordinates: 2^20 / 4096 partial sums per worker
    assert B.qesgd_workspace_bytes(1 << 20, 4, 1 << 20, 3) == 3 * 256 * 4
    assert B.qesgd_workspace_bytes(100_000, 4, 100_000, 1) == (131_072 // 4096) * 4
    assert B.qesgd_workspace_bytes(0, 4, 32, 1) == 0


def _rc_quant(B, x=0x10000, center=None, d=4096, s=4, bucket=512, kind=0, packed=0x20000,
              ws=None, ws_bytes=0):
    return B.lib().qesgd_quantize_pack(x, center, d, s, bucket, kind, 1, 0, 0, packed, ws, ws_bytes, None)


def _rc_quant_b(B, x=0x10000, stride=4096, d=4096, s=4, bucket=512, K=2, packed=0x20000, pstride=1 << 20):
    return B.lib().qesgd_quantize_pack_batched(x, stride, None, d, s, bucket, 0, 1, 0, K, packed, pstride,
                                               None, 0, None)


def test_quantize_argument_errors(B):
    """Fake device addresses: every call below must be rejected before a launch is attempted."""
    assert _rc_quant(B, x=None) == B.ERR_NULL
    assert _rc_quant(B, packed=None) == B.ERR_NULL
    assert _rc_quant(B, d=0) == B.ERR_DIM
    assert _rc_quant(B, s=3) == B.ERR_LEVELS
    assert _rc_quant(B, bucket=0) == B.ERR_BUCKET
    assert _rc_quant(B, bucket=100) == B.ERR_BUCKET
    assert _rc_quant(B, kind=2) == B.ERR_NORM_KIND
    assert _rc_quant(B, x=0x10004) == B.ERR_ALIGN
    assert _rc_quant(B, center=0x10008) == B.ERR_ALIGN
    assert _rc_quant(B, packed=0x20010) == B.ERR_ALIGN
    assert _rc_quant(B, d=100_000, bucket=100_000) == B.ERR_WORKSPACE
    assert _rc_quant(B, d=100_000, bucket=100_000, ws=0x30000, ws_bytes=64) == B.ERR_WORKSPACE
    assert _rc_quant_b(B, K=0) == B.ERR_WORKERS
    assert _rc_quant_b(B, K=65) == B.ERR_WORKERS
    assert _rc_quant_b(B, stride=4000) == B.ERR_STRIDE
    assert _rc_quant_b(B, stride=4098) == B.ERR_STRIDE
    assert _rc_quant_b(B, pstride=256) == B.ERR_STRIDE
    assert _rc_quant_b(B, pstride=(1 << 20) + 16) == B.ERR_STRIDE


def test_noalloc_argument_errors(B):
    """The no-allocation form rejects bad arguments and shapes beyond its scratch before any HIP call."""
    L = B.lib()
    x, pk = 0x10000, 0x20000
    f = L.qesgd_quantize_pack_batched_noalloc
    assert f(None, 4096, None, 4096, 4, 512, 0, 1, 0, 2, pk, 1 << 20, None) == B.ERR_NULL
    assert f(x, 4096, None, 4096, 4, 512, 0, 1, 0, 0, pk, 1 << 20, None) == B.ERR_WORKERS
    assert f(x, 4000, None, 4096, 4, 512, 0, 1, 0, 2, pk, 1 << 20, None) == B.ERR_STRIDE
    assert f(x, 4096, None, 4096, 4, 512, 2, 1, 0, 2, pk, 1 << 20, None) == B.ERR_NORM_KIND
    d = 1 << 31                                      # one bucket: 2^31 / 4096 partial sums per worker
    assert B.qesgd_workspace_bytes(d, 2, d, 2) == B.NOALLOC_SCRATCH_BYTES
    assert B.qesgd_workspace_bytes(d, 2, d, 3) > B.NOALLOC_SCRATCH_BYTES
    assert f(x, d, None, d, 2, d, 0, 1, 0, 3, pk, 1 << 33, None) == B.ERR_SCRATCH
    assert "scratch" in B.strerror(B.ERR_SCRATCH)


def test_round_argument_errors(B):
    L = B.lib()
    x, pk, w, z, u = 0x10000, 0x20000, 0x30000, 0x40000, 0x50000
    f = L.qesgd_round
    assert f(None, 4096, None, 4096, 4, 512, 0, 1, 0, 2, pk, 1 << 20, None, 0, w, z, u, None, None) == B.ERR_NULL
    assert f(x, 4096, None, 4096, 4, 512, 0, 1, 0, 2, pk, 1 << 20, None, 0, None, z, u, None, None) == B.ERR_NULL
    assert f(x, 4096, None, 4096, 4, 512, 0, 1, 0, 0, pk, 1 << 20, None, 0, w, z, u, None, None) == B.ERR_WORKERS
    assert f(x, 4096, None, 4096, 3, 512, 0, 1, 0, 2, pk, 1 << 20, None, 0, w, z, u, None, None) == B.ERR_LEVELS
    assert f(x, 4000, None, 4096, 4, 512, 0, 1, 0, 2, pk, 1 << 20, None, 0, w, z, u, None, None) == B.ERR_STRIDE
    assert f(x, 100_000, None, 100_000, 4, 100_000, 0, 1, 0, 2, pk, 1 << 20, None, 0, w, z, u, None, None) == B.ERR_WORKSPACE
    assert f(x, 4096, None, 4096, 4, 512, 0, 1, 0, 2, pk, 1 << 20, None, 0, w, z, u + 4, None, None) == B.ERR_ALIGN


def test_aggregate_argument_errors(B):
    L = B.lib()
    pk, z, w, u = 0x20000, 0x30000, 0x40000, 0x50000
    assert L.qesgd_unpack_aggregate(None, 1 << 20, 2, 4096, 4, 512, z, None) == B.ERR_NULL
    assert L.qesgd_unpack_aggregate(pk, 1 << 20, 2, 4096, 4, 512, None, None) == B.ERR_NULL
    assert L.qesgd_unpack_aggregate(pk, 1 << 20, 0, 4096, 4, 512, z, None) == B.ERR_WORKERS
    assert L.qesgd_unpack_aggregate(pk, 1 << 20, 2, 4096, 5, 512, z, None) == B.ERR_LEVELS
    assert L.qesgd_unpack_aggregate(pk, 128, 2, 4096, 4, 512, z, None) == B.ERR_STRIDE
    assert L.qesgd_unpack_aggregate(pk, 1 << 20, 2, 4096, 4, 512, z + 4, None) == B.ERR_ALIGN
    assert L.qesgd_unpack_aggregate(pk + 64, 1 << 20, 2, 4096, 4, 512, z, None) == B.ERR_ALIGN
    assert L.qesgd_unpack_aggregate_update(pk, 1 << 20, 2, 4096, 4, 512, None, z, u, None, None) == B.ERR_NULL
    assert L.qesgd_unpack_aggregate_update(pk, 1 << 20, 2, 4096, 4, 512, w, z, None, None, None) == B.ERR_NULL
    assert L.qesgd_unpack_aggregate_update(pk, 1 << 20, 2, 0, 4, 512, w, z, u, None, None) == B.ERR_DIM
    assert L.qesgd_unpack_aggregate_update(pk, 1 << 20, 2, 4096, 4, 512, w, z, u, 0x60008, None) == B.ERR_ALIGN
    assert L.qesgd_apply_update(None, z, u, None, 10, None) == B.ERR_NULL
    assert L.qesgd_apply_update(w, z, u, None, 0, None) == B.ERR_DIM
    assert L.qesgd_apply_update(w, z, u + 8, None, 10, None) == B.ERR_ALIGN


def test_missing_library_is_loud(monkeypatch):
    from paper_1901_03040_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libqesgd.so")
    with pytest.raises(RuntimeError, match="not found"):
        binding.qesgd_layout_query(10, 4, 32)


def test_fixed_grid_and_epoch_commit_argument_errors(B):
    L = B.lib()
    x, c, w, z, u, zs = 0x10000, 0x20000, 0x30000, 0x40000, 0x50000, 0x60000
    assert L.qesgd_quantize_fixed(None, None, 100, 0.1, 8, 1, 0, 0, c, None) == B.ERR_NULL
    assert L.qesgd_quantize_fixed(x, None, 100, 0.1, 8, 1, 0, 0, None, None) == B.ERR_NULL
    assert L.qesgd_quantize_fixed(x, None, 0, 0.1, 8, 1, 0, 0, c, None) == B.ERR_DIM
    assert L.qesgd_quantize_fixed(x, None, 100, 0.1, 3, 1, 0, 0, c, None) == B.ERR_BITS
    assert L.qesgd_quantize_fixed(x, None, 100, 0.1, 32, 1, 0, 0, c, None) == B.ERR_BITS
    assert L.qesgd_quantize_fixed(x, None, 100, 0.0, 8, 1, 0, 0, c, None) == B.ERR_DELTA
    assert L.qesgd_quantize_fixed(x, None, 100, -1.0, 8, 1, 0, 0, c, None) == B.ERR_DELTA
    assert L.qesgd_quantize_fixed(x, None, 100, float("inf"), 8, 1, 0, 0, c, None) == B.ERR_DELTA
    assert L.qesgd_quantize_fixed(x, None, 100, float("nan"), 8, 1, 0, 0, c, None) == B.ERR_DELTA
    assert L.qesgd_quantize_fixed(x + 4, None, 100, 0.1, 8, 1, 0, 0, c, None) == B.ERR_ALIGN
    assert L.qesgd_dequantize_fixed_update(None, 100, 0.1, 8, w, z, u, zs, None) == B.ERR_NULL
    assert L.qesgd_dequantize_fixed_update(c, 100, 0.1, 8, None, None, None, None, None) == B.ERR_NULL
    assert L.qesgd_dequantize_fixed_update(c, 100, 0.1, 8, None, z, u, None, None) == B.ERR_NULL   # u needs w
    assert L.qesgd_dequantize_fixed_update(c, 100, 0.1, 5, w, z, u, zs, None) == B.ERR_BITS
    assert L.qesgd_dequantize_fixed_update(c, 100, 0.0, 8, w, z, u, zs, None) == B.ERR_DELTA
    assert L.qesgd_dequantize_fixed_update(c, 100, 0.1, 8, w, z + 8, u, zs, None) == B.ERR_ALIGN
    assert L.qesgd_epoch_commit(None, zs, 3, 100, None) == B.ERR_NULL
    assert L.qesgd_epoch_commit(w, zs, 0, 100, None) == B.ERR_ROUNDS
    assert L.qesgd_epoch_commit(w, zs, 3, 0, None) == B.ERR_DIM
    assert L.qesgd_epoch_commit(w, zs + 4, 3, 100, None) == B.ERR_ALIGN
    for code in (B.ERR_BITS, B.ERR_DELTA, B.ERR_ROUNDS):
        assert "unknown" not in B.strerror(code)


def test_header_is_plain_c(tmp_path):
    """include/qesgd.h compiles as C99 (no C++ in the boundary) and a C program links against the
    library's host-only calls."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("gcc not available")
    from paper_1901_03040_amd import binding
    src = tmp_path / "use_header.c"
    src.write_text("""
#include "qesgd.h"
#include <stdio.h>
int main(void) {
    qesgd_layout lay;
    int rc = qesgd_layout_query(138357544ull, 2u, 4096ull, &lay);
    if (rc != QESGD_OK || lay.payload_bytes != 34724508ull) return 1;
    if (qesgd_quantize_pack(0, 0, 10, 4, 32, QESGD_NORM_L2, 1, 0, 0, 0, 0, 0, 0) != QESGD_ERR_NULL) return 2;
    if (qesgd_abi_version() != QESGD_ABI_VERSION) return 3;
    puts(qesgd_strerror(QESGD_ERR_SCRATCH));
    return 0;
}
""")
    exe = tmp_path / "use_header"
    lib_dir = os.path.dirname(binding.LIB_PATH)
    built = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", f"-I{os.path.join(ROOT, 'include')}",
                            str(src), "-o", str(exe), f"-L{lib_dir}", "-lqesgd", f"-Wl,-rpath,{lib_dir}"],
                           capture_output=True, text=True)
    assert built.returncode == 0, built.stderr[-2000:]
    run = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, (run.returncode, run.stderr[-1000:])
    assert "scratch" in run.stdout
