// Benchmark aid, not part of the method and not part of libqesgd: plain streaming kernels with
// the memory-access mixes of the hot kernels and no arithmetic to speak of, so that a benchmark
// can set the kernels' throughput against what the same machine reaches on the same footprint.
// Built into its own shared object (libqesgd_bench_probe.so) that only bench.py loads.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr uint32_t kChunk = 512;       // 64 lanes x 8 floats, the quantiser's wave chunk

// The quantiser's read pattern: a workgroup owns 4096 floats, a wave two chunks
// of 512, a lane 8 consecutive floats of each chunk (two 128-bit loads).
__device__ __forceinline__ void load_like_quantiser(const float* __restrict__ a, uint64_t base, uint32_t lane_off,
                                                    float& s0, float& s1) {
    const float4 a0 = *reinterpret_cast<const float4*>(a + base + lane_off);
    const float4 a1 = *reinterpret_cast<const float4*>(a + base + lane_off + 4);
    const float4 b0 = *reinterpret_cast<const float4*>(a + base + lane_off + kChunk);
    const float4 b1 = *reinterpret_cast<const float4*>(a + base + lane_off + kChunk + 4);
    s0 = ((a0.x + a0.y) + (a0.z + a0.w)) + ((a1.x + a1.y) + (a1.z + a1.w));
    s1 = ((b0.x + b0.y) + (b0.z + b0.w)) + ((b1.x + b1.y) + (b1.z + b1.w));
}

__global__ void __launch_bounds__(256) k_probe_read(const float* __restrict__ a, float* __restrict__ b) {
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t lane_off = wave * (2u * kChunk) + lane * 8u;
    const uint64_t base = (uint64_t)blockIdx.x * 4096u;
    float s0, s1;
    load_like_quantiser(a, base, lane_off, s0, s1);
    if (s0 + s1 == 1.2345e38f) b[base + lane_off] = s0;   // keeps the loads; not taken for ordinary data
}

// Reads like the quantiser and writes one word per 32 floats into each of two
// planes from every fourth lane: the sign and level planes at one level bit.
__global__ void __launch_bounds__(256) k_probe_quantize_mix(const float* __restrict__ a, uint32_t* __restrict__ p0,
                                                            uint32_t* __restrict__ p1) {
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t lane_off = wave * (2u * kChunk) + lane * 8u;
    const uint64_t base = (uint64_t)blockIdx.x * 4096u;
    float s0, s1;
    load_like_quantiser(a, base, lane_off, s0, s1);
    if ((lane & 3u) == 0u) {
        const uint64_t w = (base + lane_off) >> 5;
        p0[w] = __float_as_uint(s0);
        p1[w] = __float_as_uint(s0) ^ 1u;
        p0[w + (kChunk >> 5)] = __float_as_uint(s1);
        p1[w + (kChunk >> 5)] = __float_as_uint(s1) ^ 1u;
    }
}

// Reads like the quantiser and writes one byte per float, 8 bytes per lane and chunk: the
// fixed-grid quantiser at b = 8 (4 bytes in, 1 byte out per coordinate).
__global__ void __launch_bounds__(256) k_probe_byte_codes_mix(const float* __restrict__ a, uint2* __restrict__ codes) {
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t lane_off = wave * (2u * kChunk) + lane * 8u;
    const uint64_t base = (uint64_t)blockIdx.x * 4096u;
    float s0, s1;
    load_like_quantiser(a, base, lane_off, s0, s1);
    codes[(base + lane_off) >> 3] = make_uint2(__float_as_uint(s0), __float_as_uint(s1));
    codes[(base + lane_off + kChunk) >> 3] = make_uint2(__float_as_uint(s1), __float_as_uint(s0));
}

__global__ void __launch_bounds__(256) k_probe_copy(const float4* __restrict__ a, float4* __restrict__ b) {
    const uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    b[i] = a[i];
}

// Two fp32 streams in, three out, one float4 per lane: the vector traffic of the update.
__global__ void __launch_bounds__(256) k_probe_update_mix(const float4* __restrict__ a, const float4* __restrict__ b,
                                                          float4* __restrict__ c, float4* __restrict__ d,
                                                          float4* __restrict__ e) {
    const uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    const float4 x = a[i], y = b[i];
    c[i] = x;
    d[i] = make_float4(x.x + y.x, x.y + y.y, x.z + y.z, x.w + y.w);
    e[i] = y;
}

bool aligned16(const void* p) { return ((uintptr_t)p % 16u) == 0; }

}  // namespace

extern "C" {

enum { PROBE_READ = 0, PROBE_COPY = 1, PROBE_QUANTIZE_MIX = 2, PROBE_UPDATE_MIX = 3, PROBE_BYTE_CODES_MIX = 4 };

// n floats, a multiple of 4096; all pointers device memory, 16-byte aligned; unused ones NULL.
//   PROBE_READ            reads a[n] like the quantiser (a lane owns 32 bytes); b (n floats) is
//                         not written for ordinary data.
//   PROBE_COPY            b[n] = a[n], 16 bytes per lane.
//   PROBE_QUANTIZE_MIX    reads a[n] like the quantiser, writes n/32 words to each of b and c.
//   PROBE_UPDATE_MIX      reads a[n], b[n]; writes c[n], d[n], e[n], 16 bytes per lane.
//   PROBE_BYTE_CODES_MIX  reads a[n] like the quantiser, writes n bytes to b.
// Returns 0, -1 for a bad argument, or the hipError_t of a failed launch.
int qesgd_bench_probe(uint32_t pattern, const float* a, float* b, float* c, float* d, float* e, uint64_t n,
                      void* stream) {
    if (pattern > PROBE_BYTE_CODES_MIX || !a || !b) return -1;
    if ((pattern == PROBE_QUANTIZE_MIX || pattern == PROBE_UPDATE_MIX) && !c) return -1;
    if (pattern == PROBE_UPDATE_MIX && (!d || !e)) return -1;
    if (n == 0 || n % 4096u != 0 || n >= (1ull << 40)) return -1;
    if (!aligned16(a) || !aligned16(b) || !aligned16(c) || !aligned16(d) || !aligned16(e)) return -1;
    const uint64_t tiles = n / 4096u;
    if (tiles * 4u >= (1ull << 31)) return -1;
    hipStream_t st = (hipStream_t)stream;
    switch (pattern) {
        case PROBE_READ:
            hipLaunchKernelGGL(k_probe_read, dim3((uint32_t)tiles), dim3(256), 0, st, a, b);
            break;
        case PROBE_COPY:
            hipLaunchKernelGGL(k_probe_copy, dim3((uint32_t)(tiles * 4u)), dim3(256), 0, st,
                               reinterpret_cast<const float4*>(a), reinterpret_cast<float4*>(b));
            break;
        case PROBE_QUANTIZE_MIX:
            hipLaunchKernelGGL(k_probe_quantize_mix, dim3((uint32_t)tiles), dim3(256), 0, st, a,
                               reinterpret_cast<uint32_t*>(b), reinterpret_cast<uint32_t*>(c));
            break;
        case PROBE_BYTE_CODES_MIX:
            hipLaunchKernelGGL(k_probe_byte_codes_mix, dim3((uint32_t)tiles), dim3(256), 0, st, a,
                               reinterpret_cast<uint2*>(b));
            break;
        default:
            hipLaunchKernelGGL(k_probe_update_mix, dim3((uint32_t)(tiles * 4u)), dim3(256), 0, st,
                               reinterpret_cast<const float4*>(a), reinterpret_cast<const float4*>(b),
                               reinterpret_cast<float4*>(c), reinterpret_cast<float4*>(d),
                               reinterpret_cast<float4*>(e));
            break;
    }
    return (int)hipGetLastError();
}

}  // extern "C"
