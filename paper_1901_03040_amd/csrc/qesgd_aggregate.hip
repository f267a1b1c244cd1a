// Server side of a QESGD round on gfx950: unpack + dequantise the K workers'
// codes, average them in worker order (Alg. 3, server task), and apply
// u = w_t + z with the running sum of z (Alg. 2; last step of Alg. 2 / Alg. 3).
//
// A lane owns 8 consecutive coordinates: per worker it reads one sign byte, m
// level bytes and the bucket scale, per vector two 128-bit words.  All the fp32
// traffic (w, zsum in; zbar, u, zsum out) is touched exactly once.
#include "qesgd_internal.h"

namespace qesgd {
namespace {

struct AParams {
    const unsigned char* packed;
    const float* w;
    float* zbar;
    float* u;
    float* zsum;
    uint64_t packed_stride;
    uint64_t d;
    uint64_t B;
    uint64_t norms_off, signs_off, levels_off;
    uint64_t level_words;
    uint32_t K;
    int32_t log2B;          // >= 0 when B is a power of two, else -1
    float smax;
    float rcpK;             // exact 1/K when K is a power of two, else 0
};

__device__ __forceinline__ void store8(float* __restrict__ dst, uint64_t i, uint32_t nvalid, const float (&r)[8]) {
    if (nvalid == 8) {
        *reinterpret_cast<float4*>(dst + i) = make_float4(r[0], r[1], r[2], r[3]);
        *reinterpret_cast<float4*>(dst + i + 4) = make_float4(r[4], r[5], r[6], r[7]);
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if ((uint32_t)e < nvalid) dst[i + e] = r[e];
    }
}

__device__ __forceinline__ void load8(const float* __restrict__ src, uint64_t i, uint32_t nvalid, float (&r)[8]) {
    if (nvalid == 8) {
        const float4 a = *reinterpret_cast<const float4*>(src + i);
        const float4 b = *reinterpret_cast<const float4*>(src + i + 4);
        r[0] = a.x; r[1] = a.y; r[2] = a.z; r[3] = a.w;
        r[4] = b.x; r[5] = b.y; r[6] = b.z; r[7] = b.w;
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) r[e] = ((uint32_t)e < nvalid) ? src[i + e] : 0.0f;
    }
}

// The 8*M level bits of the lane's coordinates, as up to four words.
template <int M>
__device__ __forceinline__ void load_level_bits(const uint32_t* __restrict__ levels, uint64_t i, uint32_t nvalid,
                                                uint64_t level_words, uint32_t (&w)[4]) {
    w[0] = w[1] = w[2] = w[3] = 0;
    const unsigned char* bytes = reinterpret_cast<const unsigned char*>(levels);
    if (M == 1) {
        w[0] = bytes[i >> 3];
    } else if (M == 2) {
        w[0] = *reinterpret_cast<const unsigned short*>(bytes + (i >> 2));
    } else if (M == 4) {
        w[0] = levels[i >> 3];
    } else if (M == 8) {
        if (nvalid == 8) {
            const uint2 t = *reinterpret_cast<const uint2*>(levels + (i >> 2));
            w[0] = t.x; w[1] = t.y;
        } else {
            w[0] = levels[i >> 2];
            if ((i >> 2) + 1 < level_words) w[1] = levels[(i >> 2) + 1];
        }
    } else {
        if (nvalid == 8) {
            const uint4 t = *reinterpret_cast<const uint4*>(levels + (i >> 1));
            w[0] = t.x; w[1] = t.y; w[2] = t.z; w[3] = t.w;
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if ((i >> 1) + q < level_words) w[q] = levels[(i >> 1) + q];
        }
    }
}

template <int M>
__device__ __forceinline__ uint32_t level_of(const uint32_t (&w)[4], int e) {
    constexpr uint32_t mask = (1u << M) - 1u;
    const int bit = e * M;
    return (w[bit >> 5] >> (bit & 31)) & mask;
}

template <int M>
__global__ void __launch_bounds__(256) k_unpack_aggregate_update(const AParams p) {
    const uint64_t i = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) * kLaneElems;
    if (i >= p.d) return;
    const uint64_t rem = p.d - i;
    const uint32_t nvalid = rem < 8 ? (uint32_t)rem : 8u;
    const uint64_t b = p.log2B >= 0 ? (i >> p.log2B) : (i / p.B);

    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0f;

#pragma unroll 4
    for (uint32_t k = 0; k < p.K; ++k) {
        const unsigned char* __restrict__ blk = p.packed + (uint64_t)k * p.packed_stride;
        const float norm = reinterpret_cast<const float*>(blk + p.norms_off)[b];
        const uint32_t sbyte = (blk + p.signs_off)[i >> 3];
        uint32_t w[4];
        load_level_bits<M>(reinterpret_cast<const uint32_t*>(blk + p.levels_off), i, nvalid, p.level_words, w);
        const float step = norm / p.smax;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float q = (float)level_of<M>(w, e) * step;
            const uint32_t flip = ((sbyte >> e) & 1u) << 31;
            acc[e] = acc[e] + __uint_as_float(__float_as_uint(q) ^ flip);
        }
    }

    float z[8];
    if (p.rcpK != 0.0f) {
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = acc[e] * p.rcpK;      // exact scaling by 2^-j == the division
    } else {
        const float fk = (float)p.K;
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = acc[e] / fk;
    }
    if (p.zbar) store8(p.zbar, i, nvalid, z);
    if (p.w) {
        float w8[8], u8[8];
        load8(p.w, i, nvalid, w8);
#pragma unroll
        for (int e = 0; e < 8; ++e) u8[e] = w8[e] + z[e];
        store8(p.u, i, nvalid, u8);
    }
    if (p.zsum) {
        float s8[8];
        load8(p.zsum, i, nvalid, s8);
#pragma unroll
        for (int e = 0; e < 8; ++e) s8[e] = s8[e] + z[e];
        store8(p.zsum, i, nvalid, s8);
    }
}

__global__ void __launch_bounds__(256) k_apply_update(const float* w, const float* zbar,
                                                      float* u, float* zsum, uint64_t d) {
    const uint64_t i = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) * kLaneElems;
    if (i >= d) return;
    const uint64_t rem = d - i;
    const uint32_t nvalid = rem < 8 ? (uint32_t)rem : 8u;
    float z[8], w8[8], u8[8];
    load8(zbar, i, nvalid, z);
    load8(w, i, nvalid, w8);
#pragma unroll
    for (int e = 0; e < 8; ++e) u8[e] = w8[e] + z[e];
    if (zsum) {
        float s8[8];
        load8(zsum, i, nvalid, s8);
#pragma unroll
        for (int e = 0; e < 8; ++e) s8[e] = s8[e] + z[e];
        store8(zsum, i, nvalid, s8);
    }
    store8(u, i, nvalid, u8);
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

int launch_aggregate(const Shape& sh, const AggregateArgs& a) {
    AParams p{};
    p.packed = a.packed;
    p.w = a.w_snap;
    p.zbar = a.zbar_out;
    p.u = a.u_out;
    p.zsum = a.zsum;
    p.packed_stride = a.packed_stride;
    p.d = sh.d;
    p.B = sh.B;
    p.norms_off = sh.lay.norms_off;
    p.signs_off = sh.lay.signs_off;
    p.levels_off = sh.lay.levels_off;
    p.level_words = sh.lay.level_words;
    p.K = a.K;
    p.log2B = -1;
    if ((sh.B & (sh.B - 1)) == 0) {
        int lg = 0;
        while ((1ull << lg) < sh.B) ++lg;
        p.log2B = lg;
    }
    p.smax = (float)(sh.s - 1);
    p.rcpK = ((a.K & (a.K - 1)) == 0) ? 1.0f / (float)a.K : 0.0f;

    const uint64_t lanes = (sh.d + kLaneElems - 1) / kLaneElems;
    const uint64_t blocks = (lanes + 255) / 256;
    if (blocks >= (1ull << 31)) return QESGD_ERR_DIM;
    const dim3 grid((uint32_t)blocks), block(256);
    switch (sh.m) {
        case 1: hipLaunchKernelGGL(k_unpack_aggregate_update<1>, grid, block, 0, a.stream, p); break;
        case 2: hipLaunchKernelGGL(k_unpack_aggregate_update<2>, grid, block, 0, a.stream, p); break;
        case 4: hipLaunchKernelGGL(k_unpack_aggregate_update<4>, grid, block, 0, a.stream, p); break;
        case 8: hipLaunchKernelGGL(k_unpack_aggregate_update<8>, grid, block, 0, a.stream, p); break;
        default: hipLaunchKernelGGL(k_unpack_aggregate_update<16>, grid, block, 0, a.stream, p); break;
    }
    return check_launch();
}

int launch_apply_update(const float* w, const float* zbar, float* u, float* zsum, uint64_t d,
                        hipStream_t stream) {
    const uint64_t lanes = (d + kLaneElems - 1) / kLaneElems;
    const uint64_t blocks = (lanes + 255) / 256;
    if (blocks >= (1ull << 31)) return QESGD_ERR_DIM;
    hipLaunchKernelGGL(k_apply_update, dim3((uint32_t)blocks), dim3(256), 0, stream, w, zbar, u, zsum, d);
    return check_launch();
}

}  // namespace qesgd
