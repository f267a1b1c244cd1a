// Device code of the server side shared by the translation units that launch it (not installed):
// the kernel parameter block, reading a lane's level bits from a packed plane, one worker's
// contribution to a lane's 8 coordinates, and the per-lane guarded form of the whole step.
#pragma once

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
    uint32_t wave_uniform_bucket;   // 1 when every 512-aligned chunk lies inside one bucket
    uint32_t wave_two_buckets;      // else 1 when a 512-aligned chunk touches at most two buckets and K <= 32
    float smax;
    float rcpK;             // exact 1/K when K is a power of two, else 0
};

// Bucket of coordinate i (a multiple of 8).  Bucket sizes are multiples of 32 unless there is a
// single bucket, so the quotient can be taken in units of 32 coordinates: a 32-bit division for
// every vector below 2^37 coordinates instead of a 64-bit one (which costs more vector
// instructions than the rest of a lane's work).
__device__ __forceinline__ uint64_t bucket_of(uint64_t i, const AParams& p) {
    if (p.log2B >= 0) return i >> p.log2B;
    if (p.B >= p.d) return 0;
    if ((p.d >> 37) == 0) return (uint32_t)(i >> 5) / (uint32_t)(p.B >> 5);
    return i / p.B;
}

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

// The 8*M level bits of the lane's coordinates, as up to four words.  For a
// width that does not divide 32 the lane's M bytes start at byte (i/8)*M of the
// plane, at any alignment: the two or three words that hold them are read and
// shifted down so that coordinate i's field starts at bit 0 of w[0].
template <int M>
__device__ __forceinline__ void load_level_bits(const uint32_t* __restrict__ levels, uint64_t i, uint32_t nvalid,
                                                uint64_t level_words, uint32_t (&w)[4]) {
    w[0] = w[1] = w[2] = w[3] = 0;
    const unsigned char* bytes = reinterpret_cast<const unsigned char*>(levels);
    if (M == 3 || M == 5 || M == 6 || M == 7) {
        const uint64_t byte0 = (i >> 3) * (uint64_t)M;
        const uint64_t a = byte0 >> 2;
        const uint32_t sh = 8u * (uint32_t)(byte0 & 3u);
        const uint32_t t0 = a < level_words ? levels[a] : 0u;
        const uint32_t t1 = a + 1 < level_words ? levels[a + 1] : 0u;
        const uint32_t t2 = (M == 7 && a + 2 < level_words) ? levels[a + 2] : 0u;   // 7 bytes from byte 2 or 3 reach a third word
        const uint64_t lo = (uint64_t)t0 | ((uint64_t)t1 << 32);
        uint64_t v = lo >> sh;
        if (M == 7 && sh != 0u) v |= (uint64_t)t2 << (64u - sh);
        w[0] = (uint32_t)v;
        w[1] = (uint32_t)(v >> 32);
    } else if (M == 1) {
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
    if ((bit & 31) + M > 32) {                            // the field continues in the next word
        const uint64_t both = (uint64_t)w[bit >> 5] | ((uint64_t)w[(bit >> 5) + 1] << 32);
        return (uint32_t)(both >> (bit & 31)) & mask;
    }
    return (w[bit >> 5] >> (bit & 31)) & mask;
}

// Sign flip without a branch: q ^ (shifted_sign & 0x80000000) in one v_bitop3
// (truth table of a ^ (b & c) with a = 0xF0, b = 0xCC, c = 0xAA: 0x78).
__device__ __forceinline__ float apply_sign(float q, uint32_t sign_in_bit31) {
    return __uint_as_float(__builtin_amdgcn_bitop3_b32(__float_as_uint(q), sign_in_bit31, 0x80000000u, 0x78));
}

// One worker's contribution to the 8 coordinates of a lane: acc[e] += +-level_e * step.
template <int M>
__device__ __forceinline__ void accumulate8(float (&acc)[8], uint32_t sbyte, const uint32_t (&w)[4], float step) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float q = (float)level_of<M>(w, e) * step;
        acc[e] = acc[e] + apply_sign(q, sbyte << (31 - e));
    }
}

// Ragged end of the vector (and shapes the wave-uniform path below does not cover): every
// access guarded per lane, 8 consecutive coordinates per lane for all streams.
template <int M>
__device__ __forceinline__ void aggregate_lane_guarded(const AParams& p, uint64_t i) {
    if (i >= p.d) return;
    const uint64_t rem = p.d - i;
    const uint32_t nvalid = rem < 8 ? (uint32_t)rem : 8u;
    const uint64_t b = bucket_of(i, p);

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
        accumulate8<M>(acc, sbyte, w, norm / p.smax);
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

}  // namespace
}  // namespace qesgd
