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
    uint32_t full_tiles;   // tiles that lie wholly inside the vector
    float delta;
    float lo, hi;          // -2^(b-1), 2^(b-1)-1 as floats
    uint32_t key0, key1, round, worker;
};

// Eq. (2) for one coordinate: a = v/delta clamped to [lo, hi] (the clamp reproduces the first
// and last case: at an end of the range the value is on the grid and never moves), then
// floor + [r + trunc(frac * 2^16) >= 2^16].  Returns k.
__device__ __forceinline__ int32_t round_on_grid(float a, uint32_t r16) {
    const float l = floorf(a);
    const float f = a - l;
    const uint32_t T = (uint32_t)(f * 65536.0f);
    return (int32_t)l + (int32_t)((r16 + T) >> 16);
}

// The quotient v / delta for a step that is the same for every coordinate.
//   EXACT_DIV: the IEEE division as the compiler expands it (scaling of extreme operands, a
//   reciprocal refined once, two corrections of the quotient, fix-up of special cases).
//   otherwise: the same reciprocal and the same two corrections with the reciprocal computed once
//   per lane instead of once per coordinate and without the scaling and fix-up steps.  The host
//   selects this form only for 2^-60 <= delta <= 2^60, where those steps change nothing for any v
//   whose quotient can influence the code: v is first limited to +-2^b * delta (twice the range of
//   the grid, so the limited value still clamps to the same end code), which rules out overflow,
//   and a quotient below 2^-44 in magnitude (the only place where the hardware would rescale a
//   tiny numerator) gives k = 0 whatever its exact bits are.  The result is then the correctly
//   rounded quotient, bit for bit what EXACT_DIV gives.
template <bool EXACT_DIV>
struct Divider {
    float delta, rcp, vmax, lo, hi;
    __device__ __forceinline__ Divider(float delta_, float lo_, float hi_) : delta(delta_), lo(lo_), hi(hi_) {
        rcp = 0.0f;
        vmax = 0.0f;
        if (!EXACT_DIV) {
            const float r0 = __builtin_amdgcn_rcpf(delta);
            rcp = __builtin_fmaf(__builtin_fmaf(-delta, r0, 1.0f), r0, r0);
            vmax = -2.0f * lo * delta;                     // 2^b * delta
        }
    }
    // a = clamp(v / delta, lo, hi); inputs are finite
    __device__ __forceinline__ float operator()(float v) const {
        if (EXACT_DIV) return fminf(fmaxf(v / delta, lo), hi);
        const float vc = __builtin_amdgcn_fmed3f(v, -vmax, vmax);
        float q = vc * rcp;
        q = __builtin_fmaf(__builtin_fmaf(-delta, q, vc), rcp, q);
        q = __builtin_fmaf(__builtin_fmaf(-delta, q, vc), rcp, q);
        return __builtin_amdgcn_fmed3f(q, lo, hi);
    }
};

// Variates, rounding and the stores for the 8 coordinates of a lane that start at coordinate i
// (a multiple of 8), of which nvalid (0..8) exist.  Whole waves call this together: the 2-bit
// form combines the two lanes of a pair.
template <int B, bool EXACT_DIV>
__device__ __forceinline__ void fixed_chunk(const FParams& p, const Divider<EXACT_DIV>& div, const float (&v)[8],
                                            uint64_t i, uint32_t nvalid, uint32_t lane) {
    constexpr uint32_t mask = (1u << B) - 1u;
    const uint64_t g = i >> 3;
    uint32_t rnd[4];
    philox4x32_10((uint32_t)g, (uint32_t)(g >> 32), p.worker, p.round, p.key0, p.key1, rnd);

    uint32_t code[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t r16 = variate16(rnd, e);
        const int32_t k = round_on_grid(div(v[e]), r16);
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

// A workgroup owns a tile of kFixedWaves waves x kFixedChunks chunks x 512 coordinates; a lane
// owns 8 consecutive coordinates of each of its wave's chunks (two 128-bit loads, one Philox call).
// All loads of a tile are issued before the first variate is drawn.  Tiles wholly inside the
// vector run without guards; the ragged last tile guards every access per lane.  The waves share
// nothing, and the smallest unit measured fastest: at d = 138 M, b = 8, one wave x one chunk 0.144 ms,
// four waves x one chunk 0.148 ms, four waves x two / four chunks 0.155 / 0.158 ms, persistent
// workgroups that keep the next tile's loads in flight 0.165 ms or more.
constexpr int kFixedChunks = 1;
constexpr uint32_t kFixedWaves = 1;
constexpr uint32_t kFixedTile = kFixedWaves * kFixedChunks * kChunk;

template <int B, bool CENTER, bool EXACT_DIV>
__global__ void __launch_bounds__(kFixedWaves * 64) k_quantize_fixed(const FParams p) {
    constexpr int CH = kFixedChunks;
    const Divider<EXACT_DIV> div(p.delta, p.lo, p.hi);
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint64_t base = (uint64_t)blockIdx.x * kFixedTile + wave * (uint32_t)(CH * kChunk) + lane * kLaneElems;
    float v[CH][8];
    if (blockIdx.x < p.full_tiles) {
        float4 a[CH], b[CH], ca[CH], cb[CH];
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const uint64_t i = base + (uint32_t)c * kChunk;
            a[c] = *reinterpret_cast<const float4*>(p.x + i);
            b[c] = *reinterpret_cast<const float4*>(p.x + i + 4);
            if (CENTER) {
                ca[c] = *reinterpret_cast<const float4*>(p.center + i);
                cb[c] = *reinterpret_cast<const float4*>(p.center + i + 4);
            }
        }
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            v[c][0] = a[c].x; v[c][1] = a[c].y; v[c][2] = a[c].z; v[c][3] = a[c].w;
            v[c][4] = b[c].x; v[c][5] = b[c].y; v[c][6] = b[c].z; v[c][7] = b[c].w;
            if (CENTER) {
                v[c][0] -= ca[c].x; v[c][1] -= ca[c].y; v[c][2] -= ca[c].z; v[c][3] -= ca[c].w;
                v[c][4] -= cb[c].x; v[c][5] -= cb[c].y; v[c][6] -= cb[c].z; v[c][7] -= cb[c].w;
            }
        }
#pragma unroll
        for (int c = 0; c < CH; ++c) fixed_chunk<B, EXACT_DIV>(p, div, v[c], base + (uint32_t)c * kChunk, 8u, lane);
        return;
    }
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const uint64_t i = base + (uint32_t)c * kChunk;
        // whole waves stay together: the cross-lane step of the 2-bit form needs both lanes of a pair
        const uint32_t nvalid = i >= p.d ? 0u : (p.d - i < 8 ? (uint32_t)(p.d - i) : 8u);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float t = 0.0f;
            if ((uint32_t)e < nvalid) {
                t = p.x[i + e];
                if (CENTER) t -= p.center[i + e];
            }
            v[c][e] = t;
        }
        fixed_chunk<B, EXACT_DIV>(p, div, v[c], i, nvalid, lane);
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
    const uint64_t blocks = (d + kFixedTile - 1) / kFixedTile;
    if (blocks >= (1ull << 31)) return QESGD_ERR_DIM;
    p.full_tiles = (uint32_t)(d / kFixedTile);
    const dim3 grid((uint32_t)blocks), block(kFixedWaves * 64);
    // the short division is used where its scaling-free form is exact (see Divider)
    const bool exact_div = !(delta >= 0x1p-60f && delta <= 0x1p60f);
#define QESGD_LAUNCH_FIXED(BB)                                                                                      \
    do {                                                                                                            \
        if (center && exact_div) hipLaunchKernelGGL((k_quantize_fixed<BB, true, true>), grid, block, 0, stream, p);  \
        else if (center) hipLaunchKernelGGL((k_quantize_fixed<BB, true, false>), grid, block, 0, stream, p);         \
        else if (exact_div) hipLaunchKernelGGL((k_quantize_fixed<BB, false, true>), grid, block, 0, stream, p);      \
        else hipLaunchKernelGGL((k_quantize_fixed<BB, false, false>), grid, block, 0, stream, p);                    \
    } while (0)
    switch (b) {
        case 2: QESGD_LAUNCH_FIXED(2); break;
        case 4: QESGD_LAUNCH_FIXED(4); break;
        case 8: QESGD_LAUNCH_FIXED(8); break;
        default: QESGD_LAUNCH_FIXED(16); break;
    }
#undef QESGD_LAUNCH_FIXED
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
