// The quantiser exactly as the paper writes it, Q_{delta,b} of Sec. 2.1, Eq. (1)-(2): a fixed
// grid {delta*k : -2^(b-1) <= k <= 2^(b-1)-1} with a caller-chosen step, clamping outside the
// range, stochastic floor/ceil inside; its inverse fused with u = w_t + z (Alg. 2); and the
// end-of-epoch commit w_{t+1} = w_t + (1/K_t) sum_k z_{t,k} (Alg. 3, last step).
// No reduction is needed, so these are plain streaming kernels.
#include "qesgd_device.h"
#include "qesgd_internal.h"

namespace qesgd {
namespace {

struct FParams {
    const float* x;
    const float* center;
    uint32_t* codes;
    uint64_t d;
    uint64_t code_words;
    float delta;
    float lo, hi;          // -2^(b-1), 2^(b-1)-1 as floats
    uint32_t key0, key1, round, worker;
};

// Eq. (2) for one coordinate: a = v/delta clamped to [lo, hi] (the clamp reproduces the first
// and last case: at an end of the range the value is on the grid and never moves), then
// floor + [r + trunc(frac * 2^16) >= 2^16].  Returns k.
__device__ __forceinline__ int32_t fixed_round(float v, float delta, float lo, float hi, uint32_t r16) {
    const float a = fminf(fmaxf(v / delta, lo), hi);
    const float l = floorf(a);
    const float f = a - l;
    const uint32_t T = (uint32_t)(f * 65536.0f);
    return (int32_t)l + (int32_t)((r16 + T) >> 16);
}

template <int B>
__global__ void __launch_bounds__(256) k_quantize_fixed(const FParams p) {
    constexpr uint32_t mask = (1u << B) - 1u;
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t i = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) * kLaneElems;
    // whole waves leave together: the cross-lane step below needs every lane of a pair
    const uint64_t wave_base = i - lane * kLaneElems;
    if (wave_base >= p.d) return;
    const uint32_t nvalid = i >= p.d ? 0u : (p.d - i < 8 ? (uint32_t)(p.d - i) : 8u);

    float v[8];
    if (nvalid == 8) {
        const float4 a = *reinterpret_cast<const float4*>(p.x + i);
        const float4 b = *reinterpret_cast<const float4*>(p.x + i + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
        if (p.center) {
            const float4 ca = *reinterpret_cast<const float4*>(p.center + i);
            const float4 cb = *reinterpret_cast<const float4*>(p.center + i + 4);
            v[0] -= ca.x; v[1] -= ca.y; v[2] -= ca.z; v[3] -= ca.w;
            v[4] -= cb.x; v[5] -= cb.y; v[6] -= cb.z; v[7] -= cb.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float t = 0.0f;
            if ((uint32_t)e < nvalid) {
                t = p.x[i + e];
                if (p.center) t -= p.center[i + e];
            }
            v[e] = t;
        }
    }

    const uint64_t g = i >> 3;
    uint32_t rnd[4];
    philox4x32_10((uint32_t)g, (uint32_t)(g >> 32), p.worker, p.round, p.key0, p.key1, rnd);

    uint32_t code[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t r16 = variate16(rnd, e);
        const int32_t k = fixed_round(v[e], p.delta, p.lo, p.hi, r16);
        code[e] = ((uint32_t)e < nvalid) ? ((uint32_t)k & mask) : 0u;     // padding bits stay 0
    }

    uint32_t* __restrict__ out = p.codes;
    if (B == 2) {
        uint32_t h = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) h |= code[e] << (2 * e);
        uint32_t w = h << (16u * (lane & 1u));
        w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0xB1, 0xF, 0xF, false);   // the other lane of the pair
        if ((lane & 1u) == 0u && nvalid > 0) out[i >> 4] = w;
    } else if (B == 4) {
        uint32_t w = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) w |= code[e] << (4 * e);
        if (nvalid > 0) out[i >> 3] = w;
    } else if (B == 8) {
        const uint32_t w0 = code[0] | (code[1] << 8) | (code[2] << 16) | (code[3] << 24);
        const uint32_t w1 = code[4] | (code[5] << 8) | (code[6] << 16) | (code[7] << 24);
        if (nvalid == 8) {
            *reinterpret_cast<uint2*>(out + (i >> 2)) = make_uint2(w0, w1);
        } else {
            if (nvalid > 0) out[i >> 2] = w0;
            if (nvalid > 4) out[(i >> 2) + 1] = w1;
        }
    } else {
        const uint32_t w0 = code[0] | (code[1] << 16), w1 = code[2] | (code[3] << 16);
        const uint32_t w2 = code[4] | (code[5] << 16), w3 = code[6] | (code[7] << 16);
        if (nvalid == 8) {
            *reinterpret_cast<uint4*>(out + (i >> 1)) = make_uint4(w0, w1, w2, w3);
        } else {
            if (nvalid > 0) out[i >> 1] = w0;
            if (nvalid > 2) out[(i >> 1) + 1] = w1;
            if (nvalid > 4) out[(i >> 1) + 2] = w2;
            if (nvalid > 6) out[(i >> 1) + 3] = w3;
        }
    }
}

struct DParams {
    const uint32_t* codes;
    const float* w;
    float* z;
    float* u;
    float* zsum;
    uint64_t d;
    uint64_t code_words;
    float delta;
};

__device__ __forceinline__ float decode(uint32_t field, int bits, float delta) {
    const int32_t k = ((int32_t)(field << (32 - bits))) >> (32 - bits);     // sign extension
    return (float)k * delta;
}

// One float4 per lane for the vectors, 4*B code bits per lane.
template <int B>
__global__ void __launch_bounds__(256) k_dequantize_fixed_update(const DParams p) {
    constexpr uint32_t mask = (1u << B) - 1u;
    const uint64_t i = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4u;
    if (i >= p.d) return;
    const uint32_t nvalid = p.d - i < 4 ? (uint32_t)(p.d - i) : 4u;
    const unsigned char* bytes = reinterpret_cast<const unsigned char*>(p.codes);
    uint32_t f[4];
    if (B == 2) {
        const uint32_t c = bytes[i >> 2];
#pragma unroll
        for (int e = 0; e < 4; ++e) f[e] = (c >> (2 * e)) & mask;
    } else if (B == 4) {
        const uint32_t c = *reinterpret_cast<const unsigned short*>(bytes + (i >> 1));
#pragma unroll
        for (int e = 0; e < 4; ++e) f[e] = (c >> (4 * e)) & mask;
    } else if (B == 8) {
        const uint32_t c = p.codes[i >> 2];
#pragma unroll
        for (int e = 0; e < 4; ++e) f[e] = (c >> (8 * e)) & mask;
    } else {
        const uint32_t c0 = p.codes[i >> 1];
        const uint32_t c1 = ((i >> 1) + 1 < p.code_words) ? p.codes[(i >> 1) + 1] : 0u;
        f[0] = c0 & mask; f[1] = c0 >> 16; f[2] = c1 & mask; f[3] = c1 >> 16;
    }
    float z[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) z[e] = decode(f[e], B, p.delta);

    if (nvalid == 4) {
        if (p.z) *reinterpret_cast<float4*>(p.z + i) = make_float4(z[0], z[1], z[2], z[3]);
        if (p.u) {
            const float4 a = *reinterpret_cast<const float4*>(p.w + i);
            *reinterpret_cast<float4*>(p.u + i) = make_float4(a.x + z[0], a.y + z[1], a.z + z[2], a.w + z[3]);
        }
        if (p.zsum) {
            const float4 s = *reinterpret_cast<const float4*>(p.zsum + i);
            *reinterpret_cast<float4*>(p.zsum + i) = make_float4(s.x + z[0], s.y + z[1], s.z + z[2], s.w + z[3]);
        }
    } else {
        for (uint32_t e = 0; e < nvalid; ++e) {
            const float ze = e == 0 ? z[0] : (e == 1 ? z[1] : z[2]);
            if (p.z) p.z[i + e] = ze;
            if (p.u) p.u[i + e] = p.w[i + e] + ze;
            if (p.zsum) p.zsum[i + e] = p.zsum[i + e] + ze;
        }
    }
}

__global__ void __launch_bounds__(256) k_epoch_commit(float* w, float* zsum, float kt, float rcp_kt, uint64_t d) {
    const uint64_t i = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4u;
    if (i >= d) return;
    if (i + 4 <= d) {
        const float4 a = *reinterpret_cast<const float4*>(w + i);
        const float4 s = *reinterpret_cast<const float4*>(zsum + i);
        float4 m;
        if (rcp_kt != 0.0f) m = make_float4(s.x * rcp_kt, s.y * rcp_kt, s.z * rcp_kt, s.w * rcp_kt);   // exact for 2^j
        else m = make_float4(s.x / kt, s.y / kt, s.z / kt, s.w / kt);
        *reinterpret_cast<float4*>(w + i) = make_float4(a.x + m.x, a.y + m.y, a.z + m.z, a.w + m.w);
        *reinterpret_cast<float4*>(zsum + i) = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    } else {
        for (uint64_t j = i; j < d; ++j) {
            const float m = rcp_kt != 0.0f ? zsum[j] * rcp_kt : zsum[j] / kt;
            w[j] = w[j] + m;
            zsum[j] = 0.0f;
        }
    }
}

int check_launch() {
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_last_hip_error((int)e);
        return QESGD_ERR_HIP;
    }
    return QESGD_OK;
}

}  // namespace

int launch_quantize_fixed(const float* x, const float* center, uint64_t d, float delta, uint32_t b,
                          uint64_t seed, uint32_t round, uint32_t worker, void* codes, hipStream_t stream) {
    FParams p{};
    p.x = x;
    p.center = center;
    p.codes = (uint32_t*)codes;
    p.d = d;
    p.code_words = (d * b + 31) / 32;
    p.delta = delta;
    p.lo = -(float)(1u << (b - 1));
    p.hi = (float)((1u << (b - 1)) - 1u);
    p.key0 = (uint32_t)seed;
    p.key1 = (uint32_t)(seed >> 32);
    p.round = round;
    p.worker = worker;
    const uint64_t lanes = (d + kLaneElems - 1) / kLaneElems;
    const uint64_t blocks = (lanes + 255) / 256;
    if (blocks >= (1ull << 31)) return QESGD_ERR_DIM;
    const dim3 grid((uint32_t)blocks), block(256);
    switch (b) {
        case 2: hipLaunchKernelGGL(k_quantize_fixed<2>, grid, block, 0, stream, p); break;
        case 4: hipLaunchKernelGGL(k_quantize_fixed<4>, grid, block, 0, stream, p); break;
        case 8: hipLaunchKernelGGL(k_quantize_fixed<8>, grid, block, 0, stream, p); break;
        default: hipLaunchKernelGGL(k_quantize_fixed<16>, grid, block, 0, stream, p); break;
    }
    return check_launch();
}

int launch_dequantize_fixed_update(const void* codes, uint64_t d, float delta, uint32_t b, const float* w,
                                   float* z, float* u, float* zsum, hipStream_t stream) {
    DParams p{};
    p.codes = (const uint32_t*)codes;
    p.w = w;
    p.z = z;
    p.u = u;
    p.zsum = zsum;
    p.d = d;
    p.code_words = (d * b + 31) / 32;
    p.delta = delta;
    const uint64_t lanes = (d + 3) / 4;
    const uint64_t blocks = (lanes + 255) / 256;
    if (blocks >= (1ull << 31)) return QESGD_ERR_DIM;
    const dim3 grid((uint32_t)blocks), block(256);
    switch (b) {
        case 2: hipLaunchKernelGGL(k_dequantize_fixed_update<2>, grid, block, 0, stream, p); break;
        case 4: hipLaunchKernelGGL(k_dequantize_fixed_update<4>, grid, block, 0, stream, p); break;
        case 8: hipLaunchKernelGGL(k_dequantize_fixed_update<8>, grid, block, 0, stream, p); break;
        default: hipLaunchKernelGGL(k_dequantize_fixed_update<16>, grid, block, 0, stream, p); break;
    }
    return check_launch();
}

int launch_epoch_commit(float* w, float* zsum, uint32_t rounds, uint64_t d, hipStream_t stream) {
    const uint64_t lanes = (d + 3) / 4;
    const uint64_t blocks = (lanes + 255) / 256;
    if (blocks >= (1ull << 31)) return QESGD_ERR_DIM;
    const float kt = (float)rounds;
    const float rcp = ((rounds & (rounds - 1)) == 0) ? 1.0f / kt : 0.0f;
    hipLaunchKernelGGL(k_epoch_commit, dim3((uint32_t)blocks), dim3(256), 0, stream, w, zsum, kt, rcp, d);
    return check_launch();
}

}  // namespace qesgd
