"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only, g++).

1. The oracle, driven from a small C++ program over exactly-sized heap buffers at ragged sizes,
   every level width, both norms, wide buckets and the fixed grid: any read or write past a buffer,
   any signed overflow or bad shift aborts the program.
2. The library's host side (shape arithmetic and argument validation of the C ABI) with the kernel
   launchers replaced by stubs: layouts at the extremes of the accepted range (d up to 2^40 - 1,
   every level width) and every rejection path, under the same sanitizers.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
# the sanitizer runtimes are linked statically, so the program does not depend on the order of preloaded libraries
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1",
       "-static-libasan", "-static-libubsan"]

ORACLE_DRIVER = r"""
#include "ORACLE_CPP"
#include <cstdio>
#include <cstdlib>
#include <memory>

template <class T> std::unique_ptr<T[]> buf(uint64_t n) { return std::unique_ptr<T[]>(new T[n ? n : 1]); }

int main() {
    const uint32_t levels[] = {2, 4, 8, 16, 32, 64, 128, 256, 65536};
    const uint64_t dims[] = {1, 7, 31, 32, 33, 511, 1001, 5000, 70003};
    const uint64_t buckets[] = {32, 96, 512, 4096, 1u << 20};
    uint64_t cases = 0;
    for (uint32_t s : levels) for (uint64_t d : dims) for (uint64_t bucket : buckets) for (uint32_t kind = 0; kind < 2; ++kind) {
        uint64_t nb, nsw, nlw, N;
        if (qo_shape(d, s, bucket, &nb, &nsw, &nlw, &N) != 0) return 2;
        const uint32_t K = 3;
        auto x = buf<float>(d); auto c = buf<float>(d);
        for (uint64_t i = 0; i < d; ++i) { x[i] = 1e-3f * (float)((int)((i * 2654435761u) % 2001) - 1000); c[i] = 0.5f * x[i]; }
        auto norms = buf<float>(K * nb); auto sw = buf<uint32_t>(K * nsw); auto lw = buf<uint32_t>(K * nlw);
        for (uint32_t k = 0; k < K; ++k)
            if (qo_quantize_pack(x.get(), (k & 1) ? c.get() : nullptr, d, s, bucket, kind, 77 + k, 3, k,
                                 norms.get() + k * nb, sw.get() + k * nsw, lw.get() + k * nlw) != 0) return 3;
        auto level = buf<uint32_t>(d); auto sign = buf<uint8_t>(d);
        qo_unpack(sw.get(), lw.get(), d, s, level.get(), sign.get());
        auto sw2 = buf<uint32_t>(nsw); auto lw2 = buf<uint32_t>(nlw);
        qo_pack(level.get(), sign.get(), d, s, sw2.get(), lw2.get());
        for (uint64_t j = 0; j < nsw; ++j) if (sw2[j] != sw[j]) return 4;
        for (uint64_t j = 0; j < nlw; ++j) if (lw2[j] != lw[j]) return 5;
        auto zbar = buf<float>(d); auto u = buf<float>(d); auto zsum = buf<float>(d);
        for (uint64_t i = 0; i < d; ++i) zsum[i] = 0.0f;
        if (qo_unpack_aggregate(norms.get(), sw.get(), lw.get(), K, d, s, bucket, zbar.get()) != 0) return 6;
        const uint64_t a = d / 3, e = d - d / 4;
        auto part = buf<float>(e - a);
        if (qo_unpack_aggregate_range(norms.get(), sw.get(), lw.get(), K, d, s, bucket, a, e, part.get()) != 0) return 7;
        for (uint64_t i = a; i < e; ++i) if (part[i - a] != zbar[i]) return 8;
        qo_apply_update(x.get(), zbar.get(), u.get(), zsum.get(), d);
        qo_apply_update(x.get(), zbar.get(), u.get(), nullptr, d);
        qo_epoch_commit(u.get(), zsum.get(), 3, d);
        ++cases;
    }
    const uint32_t bits[] = {2, 4, 8, 16};
    for (uint32_t b : bits) for (uint64_t d : dims) {
        const uint64_t nw = (d * b + 31) / 32;
        auto x = buf<float>(d); auto c = buf<float>(d);
        for (uint64_t i = 0; i < d; ++i) { x[i] = 1e-2f * (float)((int)((i * 40503u) % 4001) - 2000); c[i] = -x[i]; }
        auto codes = buf<uint32_t>(nw);
        if (qo_quantize_fixed(x.get(), (d & 1) ? c.get() : nullptr, d, 3.1e-3f, b, 5, 1, 2, codes.get()) != 0) return 9;
        auto z = buf<float>(d); auto u = buf<float>(d); auto zs = buf<float>(d);
        for (uint64_t i = 0; i < d; ++i) zs[i] = 1.0f;
        if (qo_dequantize_fixed_update(codes.get(), d, 3.1e-3f, b, x.get(), z.get(), u.get(), zs.get()) != 0) return 10;
        if (qo_dequantize_fixed_update(codes.get(), d, 3.1e-3f, b, nullptr, z.get(), nullptr, nullptr) != 0) return 11;
        ++cases;
    }
    std::printf("oracle sanitizer cases: %llu\n", (unsigned long long)cases);
    return 0;
}
"""

API_STUBS = r"""
#include "qesgd_internal.h"
namespace qesgd {
static int launches = 0;
int launch_quantize(const Shape&, const QuantizeArgs&) { ++launches; return QESGD_OK; }
int static_scratch(float** out) { static float dummy[4]; *out = dummy; return QESGD_OK; }
int launch_aggregate(const Shape&, const AggregateArgs&) { ++launches; return QESGD_OK; }
bool round_fused_covers(const Shape& sh, uint32_t) { return sh.N == sh.B; }
int launch_round_fused(const Shape&, const QuantizeArgs&, const AggregateArgs&) { ++launches; return QESGD_OK; }
int launch_apply_update(const float*, const float*, float*, float*, uint64_t, hipStream_t) { ++launches; return QESGD_OK; }
int launch_quantize_fixed(const float*, const float*, uint64_t, float, uint32_t, uint64_t, uint32_t, uint32_t, void*, hipStream_t) { ++launches; return QESGD_OK; }
int launch_dequantize_fixed_update(const void*, uint64_t, float, uint32_t, const float*, float*, float*, float*, hipStream_t) { ++launches; return QESGD_OK; }
int launch_epoch_commit(float*, float*, uint32_t, uint64_t, hipStream_t) { ++launches; return QESGD_OK; }
}
#include <cstdio>
int main() {
    const uint32_t levels[] = {2, 4, 8, 16, 32, 64, 128, 256, 65536};
    const uint64_t dims[] = {1, 31, 32, 33, 4097, 138357544ull, (1ull << 32) + 5, (1ull << 40) - 1};
    const uint64_t buckets[] = {32, 96, 512, 4096, 32768, 65536, 48000, 1ull << 41};
    unsigned long long ok = 0;
    for (uint32_t s : levels) for (uint64_t d : dims) for (uint64_t b : buckets) {
        qesgd_layout L;
        if (qesgd_layout_query(d, s, b, &L) != QESGD_OK) return 2;
        if (L.payload_bytes != 4 * (L.n_buckets + L.sign_words + L.level_words)) return 3;
        if (L.bytes_per_worker < L.payload_bytes || L.bytes_per_worker % 256) return 4;
        for (uint32_t K = 1; K <= 64; K += 21) (void)qesgd_workspace_bytes(d, s, b, K);
        ++ok;
    }
    float* x = (float*)0x10000; void* pk = (void*)0x20000; float* z = (float*)0x30000;
    // accepted calls reach the (stubbed) launchers; rejected ones must not
    if (qesgd_quantize_pack(x, nullptr, 4096, 4, 512, 0, 1, 0, 0, pk, nullptr, 0, nullptr) != QESGD_OK) return 5;
    if (qesgd_quantize_pack_batched(x, 4096, nullptr, 4096, 4, 512, 0, 1, 0, 64, pk, 1 << 20, nullptr, 0, nullptr) != QESGD_OK) return 6;
    if (qesgd_quantize_pack_batched_noalloc(x, 1 << 20, nullptr, 1 << 20, 4, 1 << 20, 0, 1, 0, 3, pk, 1 << 22, nullptr) != QESGD_OK) return 7;
    if (qesgd_unpack_aggregate_update(pk, 1 << 20, 2, 4096, 4, 512, x, z, z, nullptr, nullptr) != QESGD_OK) return 8;
    if (qesgd_round(x, 4096, nullptr, 4096, 4, 512, 0, 1, 0, 2, pk, 1 << 20, nullptr, 0, x, z, z, nullptr, nullptr) != QESGD_OK) return 17;
    if (qesgd_round(x, 4096, nullptr, 4096, 4, 96, 0, 1, 0, 2, pk, 1 << 20, nullptr, 0, x, z, z, nullptr, nullptr) != QESGD_OK) return 18;
    const int before = qesgd::launches;
    if (qesgd_round(x, 4096, nullptr, 4096, 4, 512, 0, 1, 0, 2, pk, 1 << 20, nullptr, 0, nullptr, z, z, nullptr, nullptr) != QESGD_ERR_NULL) return 19;
    if (qesgd_quantize_pack(x, nullptr, 0, 4, 512, 0, 1, 0, 0, pk, nullptr, 0, nullptr) != QESGD_ERR_DIM) return 9;
    if (qesgd_quantize_pack(x, nullptr, 1ull << 40, 4, 512, 0, 1, 0, 0, pk, nullptr, 0, nullptr) != QESGD_ERR_DIM) return 10;
    if (qesgd_quantize_pack(x, nullptr, 100000, 4, 100000, 0, 1, 0, 0, pk, nullptr, 0, nullptr) != QESGD_ERR_WORKSPACE) return 11;
    if (qesgd_quantize_pack_batched_noalloc(x, 1ull << 31, nullptr, 1ull << 31, 2, 1ull << 31, 0, 1, 0, 3, pk, 1ull << 33, nullptr) != QESGD_ERR_SCRATCH) return 12;
    if (qesgd_quantize_fixed(x, nullptr, 100, 0.0f, 8, 1, 0, 0, pk, nullptr) != QESGD_ERR_DELTA) return 13;
    if (qesgd_epoch_commit(x, z, 0, 100, nullptr) != QESGD_ERR_ROUNDS) return 14;
    if (qesgd::launches != before) return 15;
    for (int code = 0; code >= -20; --code) if (!qesgd_strerror(code)) return 16;
    std::printf("api sanitizer shapes: %llu\n", ok);
    return 0;
}
"""


def _build_and_run(tmp_path, name, source, extra):
    if shutil.which("g++") is None:
        pytest.skip("g++ not available")
    src = tmp_path / f"{name}.cpp"
    src.write_text(source)
    exe = tmp_path / name
    cmd = ["g++", "-std=c++17", *SAN, "-ffp-contract=off", *extra, str(src), "-o", str(exe)]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "asan" in built.stderr.lower() and "cannot find" in built.stderr.lower():
        pytest.skip("sanitizer runtime not installed")
    assert built.returncode == 0, built.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, (run.returncode, run.stdout[-1000:], run.stderr[-3000:])
    return run.stdout


def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    out = _build_and_run(tmp_path, "oracle_san",
                         ORACLE_DRIVER.replace("ORACLE_CPP", os.path.join(ROOT, "oracle", "qesgd_oracle.cpp")), [])
    assert "oracle sanitizer cases" in out


def test_api_host_side_under_address_and_ub_sanitizers(tmp_path):
    """Shape arithmetic and validation of the C ABI; the launchers are stubs, no HIP call is made."""
    inc = ["-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", f"-I{os.path.join(ROOT, 'include')}",
           f"-I{os.path.join(ROOT, 'paper_1901_03040_amd', 'csrc')}", "-Wno-deprecated-declarations",
           os.path.join(ROOT, "paper_1901_03040_amd", "csrc", "qesgd_api.cpp")]
    if not os.path.exists("/opt/rocm/include/hip/hip_runtime.h"):
        pytest.skip("HIP headers not available")
    out = _build_and_run(tmp_path, "api_san", API_STUBS, inc)
    assert "api sanitizer shapes" in out
