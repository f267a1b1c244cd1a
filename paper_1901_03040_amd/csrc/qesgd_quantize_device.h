// Device code of the quantiser shared by the translation units that launch it (not installed):
// the kernel parameter block, the cross-lane tree, rounding and packing of a lane's 8 coordinates,
// the guarded tile and the straight-line tile of the power-of-two-bucket kernels.
#pragma once

#include "qesgd_aggregate_device.h"
#include "qesgd_device.h"
#include "qesgd_internal.h"

namespace qesgd {
namespace {

struct QParams {
    const float* x;
    const float* center;
    unsigned char* packed;
    float* workspace;
    uint64_t x_stride;
    uint64_t packed_stride;
    uint64_t d;
    uint64_t B;
    uint64_t nb;
    uint64_t norms_off, signs_off, levels_off;
    uint32_t log2N;
    uint32_t tile0;              // generic kernel: first tile it covers
    uint32_t tiles_per_worker;   // generic kernel: tiles it covers per worker
    uint32_t full_tiles;         // fast kernels: tiles per worker that lie wholly inside the vector
    uint32_t tail_tiles;         // fast quantize kernel: ragged tiles per worker after those (0 or 1)
    uint32_t group_workers;      // workers covered by this launch
    uint32_t ws_tiles_per_worker;  // partial sums: workspace entries per worker (nb * N / 4096)
    uint64_t data_tiles;         // partial sums: 4096-slot tiles of a worker that hold coordinates
    uint32_t key0, key1;
    uint32_t round;
    uint32_t worker0;
    float smax;
};


// ---------------------------------------------------------------------------
// Cross-lane helpers.
// ---------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
    return __uint_as_float(dpp_u32<CTRL>(__float_as_uint(x)));
}
constexpr int kDppXor1 = 0xB1;          // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;          // quad_perm [2,3,0,1]
constexpr int kDppQuadLane0 = 0x00;     // quad_perm [0,0,0,0]: lane 0 of the quad to all four
constexpr int kDppHalfMirror = 0x141;   // lane l -> 7 - l inside each 8: the other quad
constexpr int kDppRowMirror = 0x140;    // lane l -> 15 - l inside each 16: the other 8

template <int KIND>
__device__ __forceinline__ float combine(float a, float b) {
    if (KIND == QESGD_NORM_L2) return a + b;
    return fmaxf(a, b);
}

// The two halves of an exchange between 16-lane rows (lanes l and l ^ 16) or
// between wave halves (l and l ^ 32): v_permlane16_swap / v_permlane32_swap hand
// every lane its own row's value and the partner row's value, in some order;
// the combine is commutative, so the order does not matter.
template <int KIND>
__device__ __forceinline__ float combine_xor16(float t) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(t), __float_as_uint(t), false, false);
    return combine<KIND>(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
template <int KIND>
__device__ __forceinline__ float combine_xor32(float t) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(t), __float_as_uint(t), false, false);
    return combine<KIND>(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Butterfly over the lanes that share a bucket (lanes_per_bucket = 1..64, a power
// of two, wave-uniform).  The mirror steps fetch "the other half" because after
// the previous steps all lanes of a half hold the same value; a + b == b + a, so
// every lane ends with the tree sum.
template <int KIND>
__device__ __forceinline__ float lane_butterfly(float t, uint32_t lanes_per_bucket) {
    if (lanes_per_bucket > 1) t = combine<KIND>(t, dpp_f32<kDppXor1>(t));
    if (lanes_per_bucket > 2) t = combine<KIND>(t, dpp_f32<kDppXor2>(t));
    if (lanes_per_bucket > 4) t = combine<KIND>(t, dpp_f32<kDppHalfMirror>(t));
    if (lanes_per_bucket > 8) t = combine<KIND>(t, dpp_f32<kDppRowMirror>(t));
    if (lanes_per_bucket > 16) t = combine_xor16<KIND>(t);
    if (lanes_per_bucket > 32) t = combine_xor32<KIND>(t);
    return t;
}

template <int KIND>
__device__ __forceinline__ float lane_tree(const float (&v)[8]) {
    if (KIND == QESGD_NORM_L2) {
        const float q0 = v[0] * v[0], q1 = v[1] * v[1], q2 = v[2] * v[2], q3 = v[3] * v[3];
        const float q4 = v[4] * v[4], q5 = v[5] * v[5], q6 = v[6] * v[6], q7 = v[7] * v[7];
        return ((q0 + q1) + (q2 + q3)) + ((q4 + q5) + (q6 + q7));
    }
    return fmaxf(fmaxf(fmaxf(fabsf(v[0]), fabsf(v[1])), fmaxf(fabsf(v[2]), fabsf(v[3]))),
                 fmaxf(fmaxf(fabsf(v[4]), fabsf(v[5])), fmaxf(fabsf(v[6]), fabsf(v[7]))));
}

// The same in-lane tree over 8 values that are already partial results (no squaring).
template <int KIND>
__device__ __forceinline__ float lane_tree_of_partials(const float (&q)[8]) {
    return combine<KIND>(combine<KIND>(combine<KIND>(q[0], q[1]), combine<KIND>(q[2], q[3])),
                         combine<KIND>(combine<KIND>(q[4], q[5]), combine<KIND>(q[6], q[7])));
}

// Pairwise tree over up to 16 wave totals parked in LDS; entries beyond `count`
// are +0 (adding +0 is exact, so the padded tree equals the tree over `count`).
// `sm` must have 32 readable floats: a hoisted read of sm[base + r] stays inside.
template <int KIND>
__device__ __forceinline__ float lds_tree16(const float* sm, uint32_t base, uint32_t count) {
    float a[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) a[r] = ((uint32_t)r < count) ? sm[base + r] : 0.0f;
#pragma unroll
    for (int w = 1; w < 16; w <<= 1) {
#pragma unroll
        for (int r = 0; r < 16; r += 2 * w) a[r] = combine<KIND>(a[r], a[r + w]);
    }
    return a[0];
}

// ---------------------------------------------------------------------------
// Rounding and in-lane packing of the 8 coordinates of a lane.
//   fixed = trunc(min(|v| * inv, smax) * 2^16) = floor(a) * 2^16 + trunc(frac(a) * 2^16)
//   level = (fixed + r16) >> 16        (the carry out of the low half rounds up)
// inv * 2^16 is folded into the scale when it is finite: scaling by a power of
// two commutes with rounding, and a product that underflows truncates to 0
// either way.  bits[] receives the 8*M level bits (M = 1: low byte, M = 2: low
// half, M = 4: one word, M = 8: two words, M = 16: four words; M = 3, 5, 6, 7:
// the low 8*M bits of bits[0..1] read as one 64-bit string).
// ---------------------------------------------------------------------------
template <int M>
__device__ __forceinline__ void round_and_pack(const float (&v)[8], const uint32_t (&rnd)[4], float inv,
                                               float smax, uint32_t& sign_byte, uint32_t (&bits)[4]) {
    uint32_t y[8];
    const float inv16 = inv * 65536.0f;
    if (inv16 < INFINITY) {
        const float smax16 = smax * 65536.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t r16 = variate16(rnd, e);
            y[e] = (uint32_t)fminf(fabsf(v[e]) * inv16, smax16) + r16;
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t r16 = variate16(rnd, e);
            y[e] = (uint32_t)(fminf(fabsf(v[e]) * inv, smax) * 65536.0f) + r16;
        }
    }
    uint32_t sb = 0;
#pragma unroll
    for (int e = 7; e >= 0; --e) sb = sb + sb + (v[e] < 0.0f ? 1u : 0u);   // v_cmp + v_addc
    sign_byte = sb;
    bits[0] = bits[1] = bits[2] = bits[3] = 0;
    if (M == 1 || M == 2 || M == 4) {
        uint32_t w = y[0] >> 16;
#pragma unroll
        for (int e = 1; e < 8; ++e) w |= (y[e] >> 16) << (M * e);
        bits[0] = w;
    } else if (M == 3 || M == 5 || M == 6 || M == 7) {       // 8*M <= 56 bits: one 64-bit string
        uint64_t w = y[0] >> 16;
#pragma unroll
        for (int e = 1; e < 8; ++e) w |= (uint64_t)(y[e] >> 16) << (M * e);
        bits[0] = (uint32_t)w;
        bits[1] = (uint32_t)(w >> 32);
    } else if (M == 8) {
        bits[0] = (y[0] >> 16) | ((y[1] >> 16) << 8) | ((y[2] >> 16) << 16) | ((y[3] >> 16) << 24);
        bits[1] = (y[4] >> 16) | ((y[5] >> 16) << 8) | ((y[6] >> 16) << 16) | ((y[7] >> 16) << 24);
    } else {
        bits[0] = (y[0] >> 16) | (y[1] & 0xFFFF0000u);
        bits[1] = (y[2] >> 16) | (y[3] & 0xFFFF0000u);
        bits[2] = (y[4] >> 16) | (y[5] & 0xFFFF0000u);
        bits[3] = (y[6] >> 16) | (y[7] & 0xFFFF0000u);
    }
}

__device__ __forceinline__ float inverse_step(float norm, float smax) {
    float inv = smax / norm;
    if (!(inv < INFINITY)) inv = 0.0f;     // norm 0 (or reciprocal overflow): every level is 0
    return inv;
}

// Cross-lane assembly of words and the stores, for a lane whose 8 coordinates
// start at coordinate i (a multiple of 8) of which nvalid (0..8) exist.
// sign_words / level_words point at word 0 of the planes.
template <int M>
__device__ __forceinline__ void store_codes(uint32_t* __restrict__ sign_words, uint32_t* __restrict__ level_words,
                                            uint64_t i, uint32_t nvalid, uint32_t lane,
                                            uint32_t sign_byte, const uint32_t (&bits)[4]) {
    {
        uint32_t w = sign_byte << (8u * (lane & 3u));
        w |= dpp_u32<kDppXor1>(w);
        w |= dpp_u32<kDppXor2>(w);
        if ((lane & 3u) == 0u && nvalid > 0) sign_words[i >> 5] = w;
    }
    if (M == 1) {
        uint32_t w = bits[0] << (8u * (lane & 3u));
        w |= dpp_u32<kDppXor1>(w);
        w |= dpp_u32<kDppXor2>(w);
        if ((lane & 3u) == 0u && nvalid > 0) level_words[i >> 5] = w;
    } else if (M == 2) {
        uint32_t w = bits[0] << (16u * (lane & 1u));
        w |= dpp_u32<kDppXor1>(w);
        if ((lane & 1u) == 0u && nvalid > 0) level_words[i >> 4] = w;
    } else if (M == 4) {
        if (nvalid > 0) level_words[i >> 3] = bits[0];
    } else if (M == 3 || M == 5 || M == 6 || M == 7) {
        // The 32 coordinates of a quad fill M whole words; lane j's 8*M bits start at bit
        // 8*M*j of that block.  Every lane shifts its string into each of the M words, the
        // quad ORs them, and lane j stores words j and j+4 of the block (those that hold a
        // coordinate of the vector).
        const uint32_t j = lane & 3u;
        uint32_t nq = nvalid;
        nq += dpp_u32<kDppXor1>(nq);
        nq += dpp_u32<kDppXor2>(nq);
        const uint32_t nwords = (nq * (uint32_t)M + 31u) >> 5;
        const uint64_t i_quad = (uint64_t)dpp_u32<kDppQuadLane0>((uint32_t)i) |
                                ((uint64_t)dpp_u32<kDppQuadLane0>((uint32_t)(i >> 32)) << 32);
        const uint64_t v = (uint64_t)bits[0] | ((uint64_t)bits[1] << 32);
        const int at = 8 * M * (int)j;
        uint32_t first = 0, second = 0;
#pragma unroll
        for (int q = 0; q < M; ++q) {
            const int sh = at - 32 * q;                   // where the string starts relative to word q
            uint32_t c = 0;
            if (sh >= 0 && sh < 32) c = (uint32_t)v << sh;
            else if (sh < 0 && sh > -64) c = (uint32_t)(v >> (-sh));
            c |= dpp_u32<kDppXor1>(c);
            c |= dpp_u32<kDppXor2>(c);
            if (q < 4) { if (j == (uint32_t)q) first = c; }
            else { if (j == (uint32_t)(q - 4)) second = c; }
        }
        uint32_t* __restrict__ dst = level_words + (i_quad >> 5) * (uint64_t)M;
        if (j < nwords) dst[j] = first;
        if (M > 4 && j + 4u < nwords) dst[j + 4u] = second;
    } else if (M == 8) {
        if (nvalid == 8) {
            *reinterpret_cast<uint2*>(level_words + (i >> 2)) = make_uint2(bits[0], bits[1]);
        } else {
            if (nvalid > 0) level_words[i >> 2] = bits[0];
            if (nvalid > 4) level_words[(i >> 2) + 1] = bits[1];
        }
    } else {
        if (nvalid == 8) {
            *reinterpret_cast<uint4*>(level_words + (i >> 1)) = make_uint4(bits[0], bits[1], bits[2], bits[3]);
        } else {
            if (nvalid > 0) level_words[i >> 1] = bits[0];
            if (nvalid > 2) level_words[(i >> 1) + 1] = bits[1];
            if (nvalid > 4) level_words[(i >> 1) + 2] = bits[2];
            if (nvalid > 6) level_words[(i >> 1) + 3] = bits[3];
        }
    }
}

// ---------------------------------------------------------------------------
// Guarded tile: the shared body of the generic kernel and of the ragged last tile.
// ---------------------------------------------------------------------------
// Where the 8 slots of this lane fall: bucket, first coordinate, how many of
// them are real coordinates (0..8), and whether they open the bucket.
struct LaneSpan {
    uint64_t bucket;
    uint64_t i;        // first coordinate (a multiple of 8)
    uint32_t nvalid;
    bool opens_bucket;
};

__device__ __forceinline__ LaneSpan lane_span(uint64_t slot, const QParams& p) {
    LaneSpan s;
    const uint64_t N = 1ull << p.log2N;
    s.bucket = slot >> p.log2N;
    const uint64_t j = slot & (N - 1);
    uint64_t len = 0;
    if (s.bucket < p.nb) {
        const uint64_t rem = p.d - s.bucket * p.B;
        len = rem < p.B ? rem : p.B;
    }
    s.nvalid = j < len ? (uint32_t)((len - j) < 8 ? (len - j) : 8) : 0u;
    s.i = s.bucket * p.B + j;
    s.opens_bucket = (j == 0) && (s.bucket < p.nb);
    return s;
}

__device__ __forceinline__ void load_lane(const float* __restrict__ x, const float* __restrict__ center,
                                          const LaneSpan& s, float (&v)[8]) {
    if (s.nvalid == 8) {
        const float4 a = *reinterpret_cast<const float4*>(x + s.i);
        const float4 b = *reinterpret_cast<const float4*>(x + s.i + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
        if (center) {
            const float4 ca = *reinterpret_cast<const float4*>(center + s.i);
            const float4 cb = *reinterpret_cast<const float4*>(center + s.i + 4);
            v[0] -= ca.x; v[1] -= ca.y; v[2] -= ca.z; v[3] -= ca.w;
            v[4] -= cb.x; v[5] -= cb.y; v[6] -= cb.z; v[7] -= cb.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float t = 0.0f;
            if ((uint32_t)e < s.nvalid) {
                t = x[s.i + e];
                if (center) t -= center[s.i + e];
            }
            v[e] = t;
        }
    }
}

// One tile of worker k with every access guarded per lane.  PRE = true: the scales were
// computed by the partial-sum passes and are read from the norms plane.  sm: 32 floats of LDS.
// ACC = true: the dequantised codes are also added to acc[chunk][0..8) (the server's sum over
// workers, for the launch that runs a whole round).
template <int M, int CH, int KIND, bool PRE, bool ACC = false>
__device__ __forceinline__ void guarded_tile(const QParams& p, uint32_t k, uint32_t tile, float* sm,
                                             float (*acc)[8] = nullptr) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t nwaves = blockDim.x >> 6;
    const float* __restrict__ x = p.x + (uint64_t)k * p.x_stride;
    unsigned char* __restrict__ out = p.packed + (uint64_t)k * p.packed_stride;
    float* __restrict__ norms = reinterpret_cast<float*>(out + p.norms_off);
    uint32_t* __restrict__ signs = reinterpret_cast<uint32_t*>(out + p.signs_off);
    uint32_t* __restrict__ levels = reinterpret_cast<uint32_t*>(out + p.levels_off);
    const uint64_t N = 1ull << p.log2N;
    const uint64_t slot0 = ((uint64_t)tile * nwaves + wave) * (uint64_t)(CH * kChunk) + lane * kLaneElems;

    LaneSpan span[CH];
    float v[CH][8];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        span[c] = lane_span(slot0 + (uint64_t)c * kChunk, p);
        load_lane(x, p.center, span[c], v[c]);
    }

    float norm[CH];
    if (PRE) {
#pragma unroll
        for (int c = 0; c < CH; ++c) norm[c] = span[c].bucket < p.nb ? norms[span[c].bucket] : 0.0f;
    } else {
        float t[CH];
        const uint32_t lanes_per_bucket = (uint32_t)((N < kChunk ? N : kChunk) / kLaneElems);
#pragma unroll
        for (int c = 0; c < CH; ++c) t[c] = lane_butterfly<KIND>(lane_tree<KIND>(v[c]), lanes_per_bucket);
        if (N > kChunk) {
            const uint32_t chunks_per_bucket = (uint32_t)(N / kChunk < (uint64_t)CH ? N / kChunk : (uint64_t)CH);
#pragma unroll
            for (int w = 1; w < CH; w <<= 1) {
                if (chunks_per_bucket > (uint32_t)w) {
#pragma unroll
                    for (int c = 0; c < CH; c += 2 * w) t[c] = combine<KIND>(t[c], t[c + w]);
                }
            }
            if (N > (uint64_t)(CH * kChunk)) {          // the bucket spans several waves
                const uint32_t waves_per_bucket = (uint32_t)(N / (CH * kChunk));
                if (lane == 0) sm[wave] = t[0];
                __syncthreads();
                t[0] = lds_tree16<KIND>(sm, wave & ~(waves_per_bucket - 1u), waves_per_bucket);
            }
#pragma unroll
            for (int w = CH / 2; w >= 1; w >>= 1) {
                if (chunks_per_bucket > (uint32_t)w) {
#pragma unroll
                    for (int c = 0; c < CH; c += 2 * w) t[c + w] = t[c];
                }
            }
        }
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            norm[c] = (KIND == QESGD_NORM_L2) ? sqrtf(t[c]) : t[c];
            if (span[c].opens_bucket) norms[span[c].bucket] = norm[c];
        }
    }

#pragma unroll
    for (int c = 0; c < CH; ++c) {
        // Lanes are in slot order, so a chunk whose first lane holds no coordinate is all padding
        // (the tail of a bucket that is not a power of two, or of the vector): nothing to encode.
        if (__builtin_amdgcn_readfirstlane(span[c].nvalid) == 0u) continue;
        const uint64_t g = span[c].i >> 3;
        uint32_t rnd[4];
        philox4x32_10((uint32_t)g, (uint32_t)(g >> 32), p.worker0 + k, p.round, p.key0, p.key1, rnd);
        uint32_t sign_byte, bits[4];
        round_and_pack<M>(v[c], rnd, inverse_step(norm[c], p.smax), p.smax, sign_byte, bits);
        store_codes<M>(signs, levels, span[c].i, span[c].nvalid, lane, sign_byte, bits);
        if (ACC) accumulate8<M>(acc[c], sign_byte, bits, norm[c] / p.smax);
    }
}

// ---------------------------------------------------------------------------
// Fast kernel.  Geometry per bucket size: tile = NW waves x CH chunks x 512.
// ---------------------------------------------------------------------------
template <int LOG2N>
struct Geo {
    // Buckets up to 2048: one chunk per wave (2048-coordinate tiles measured faster than 4096: 80
    // against 84 us at d = 11 M), and two waves instead of four up to 1024 (0.84 against 0.86 ms at
    // d = 138 M, K = 8, bucket 512 or 1024; one wave is slower again); 4096 / 8192: two chunks per
    // wave (one chunk and twice the waves is as fast at 4096 and much slower at 8192: 0.46 against
    // 0.38 ms at d = 25.6 M, K = 16).
    static constexpr int CH = (LOG2N == 15) ? 4 : (LOG2N <= 11 ? 1 : 2);
    static constexpr int NW = (LOG2N <= 10) ? 2 : ((LOG2N <= 12) ? 4 : (LOG2N == 13 ? 8 : 16));
    static constexpr uint32_t TILE = (uint32_t)NW * CH * kChunk;
};

// Geo<log2 N> for a run-time N (host side): chunks per wave and waves per workgroup.
inline void fast_geometry(uint64_t N, uint32_t* ch, uint32_t* nwaves) {
    *ch = N == 32768 ? 4u : (N <= 2048 ? 1u : 2u);
    *nwaves = N <= 1024 ? 2u : (N <= 4096 ? 4u : (N == 8192 ? 8u : 16u));
}

template <int CH, bool CENTER>
__device__ __forceinline__ void load_tile(const float* __restrict__ xt, const float* __restrict__ ct,
                                          uint32_t lane_off, float (&v)[CH][8]) {
    float4 a[CH], b[CH], ca[CH], cb[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const uint32_t o = lane_off + (uint32_t)c * kChunk;
        a[c] = *reinterpret_cast<const float4*>(xt + o);
        b[c] = *reinterpret_cast<const float4*>(xt + o + 4);
        if (CENTER) {
            ca[c] = *reinterpret_cast<const float4*>(ct + o);
            cb[c] = *reinterpret_cast<const float4*>(ct + o + 4);
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
}

// Everything a workgroup needs to know about its worker, in registers.
struct FastCtx {
    float* __restrict__ norms;
    uint32_t* __restrict__ signs;
    uint32_t* __restrict__ levels;
    uint32_t lane, wave, lane_off, worker, round, key0, key1;
    float smax;
};

// One tile: bucket totals, scales, variates, rounding, packing, stores.  ACC as in guarded_tile.
template <int M, int LOG2N, bool ACC = false>
__device__ __forceinline__ void process_tile(const FastCtx& cx, float (&v)[Geo<LOG2N>::CH][8], uint32_t t, float* sm,
                                             float (*acc)[8] = nullptr) {
    constexpr int CH = Geo<LOG2N>::CH;
    constexpr uint32_t N = 1u << LOG2N;
    constexpr uint32_t TILE = Geo<LOG2N>::TILE;
    constexpr uint32_t LPB = (N < kChunk ? N : kChunk) / kLaneElems;                       // lanes per bucket
    constexpr int CPB = N <= kChunk ? 1 : (int)(N / kChunk < (uint32_t)CH ? N / kChunk : (uint32_t)CH);  // chunks per bucket in a wave
    constexpr uint32_t WPB = N <= CH * kChunk ? 1u : N / (CH * kChunk);                     // waves per bucket
    constexpr int KIND = QESGD_NORM_L2;
    const uint64_t e0 = (uint64_t)t * TILE;                      // first coordinate of the tile

    float tot[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) tot[c] = lane_butterfly<KIND>(lane_tree<KIND>(v[c]), LPB);
    if (CPB > 1) {
#pragma unroll
        for (int w = 1; w < CPB; w <<= 1) {
#pragma unroll
            for (int c = 0; c < CH; c += 2 * w) tot[c] = combine<KIND>(tot[c], tot[c + w]);
        }
    }
    if (WPB > 1) {
        if (cx.lane == 0) sm[cx.wave] = tot[0];
        __syncthreads();
        tot[0] = lds_tree16<KIND>(sm, cx.wave & ~(WPB - 1u), WPB);
    }

    float inv = 0.0f, step = 0.0f;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const uint32_t off = cx.lane_off + (uint32_t)c * kChunk;
        if (c % CPB == 0) {                                       // first chunk of a bucket (or of its part in this wave)
            const float norm = sqrtf(tot[c]);
            inv = inverse_step(norm, cx.smax);
            if (ACC) step = norm / cx.smax;
            if ((off & (N - 1u)) == 0u) cx.norms[(e0 >> LOG2N) + (off >> LOG2N)] = norm;
        }
        const uint64_t i = e0 + off;
        const uint64_t g = i >> 3;
        uint32_t rnd[4];
        philox4x32_10((uint32_t)g, (uint32_t)(g >> 32), cx.worker, cx.round, cx.key0, cx.key1, rnd);
        uint32_t sign_byte, bits[4];
        round_and_pack<M>(v[c], rnd, inv, cx.smax, sign_byte, bits);
        store_codes<M>(cx.signs, cx.levels, i, 8u, cx.lane, sign_byte, bits);
        if (ACC) accumulate8<M>(acc[c], sign_byte, bits, step);
    }
}

}  // namespace
}  // namespace qesgd
