// Worker side of a QESGD round on gfx950: bucket scale, stochastic rounding
// (Sec. 2.1, Eq. (2)) and bit packing, one pass over the input.
//
// Mapping.  The coordinates are laid out in "slot space": bucket b owns the N
// slots [b*N, (b+1)*N), N = bucket size zero-padded to a power of two, so that
// every bucket starts on a power-of-two boundary whatever its length.  A lane
// owns 8 consecutive slots (two 128-bit loads, one Philox call, one sign byte),
// a wavefront owns CH chunks of 64 x 8 = 512 slots, a workgroup owns
// nwaves x CH x 512 slots.  The fp32 sum of squares is the balanced binary tree
// over slot index bits: bits 0-2 inside the lane, bits 3-8 as an xor butterfly
// over lanes (DPP for masks 1,2,4,8; cross-row exchange for 16,32), then the
// chunks of a wave, then the waves of a workgroup through LDS.  Every lane ends
// with its bucket's total, so the scale never goes through memory.
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
    uint32_t tiles_per_worker;
    uint32_t key0, key1;
    uint32_t round;
    uint32_t worker0;
    float smax;
};

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  The key is wave-uniform, so its Weyl
// sequence lives in scalar registers.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&o)[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t pa = (uint64_t)0xD2511F53u * c0;
        const uint64_t pb = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)pb;
        c3 = (uint32_t)pa;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    o[0] = c0; o[1] = c1; o[2] = c2; o[3] = c3;
}

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
constexpr int kDppHalfMirror = 0x141;   // lane l -> 7 - l inside each 8: the other quad
constexpr int kDppRowMirror = 0x140;    // lane l -> 15 - l inside each 16: the other 8

template <int KIND>
__device__ __forceinline__ float combine(float a, float b) {
    if (KIND == QESGD_NORM_L2) return a + b;
    return fmaxf(a, b);
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
    if (lanes_per_bucket > 16) t = combine<KIND>(t, __shfl_xor(t, 16, 64));
    if (lanes_per_bucket > 32) t = combine<KIND>(t, __shfl_xor(t, 32, 64));
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

// Pairwise tree over up to 16 wave totals parked in LDS; entries beyond `count`
// are +0 (adding +0 is exact, so the padded tree equals the tree over `count`).
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
// The fused kernel.  PRE = true: the scales were computed by the partial-sum
// passes below and are read from the norms plane.
// ---------------------------------------------------------------------------
template <int M, int CH, int KIND, bool PRE>
__global__ void k_quantize_pack(const QParams p) {
    __shared__ float sm[32];   // 16 wave totals; the upper half stays unused so a hoisted read of sm[base + r] stays inside
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t nwaves = blockDim.x >> 6;
    const uint32_t k = blockIdx.x / p.tiles_per_worker;
    const uint32_t tile = blockIdx.x - k * p.tiles_per_worker;
    const float* __restrict__ x = p.x + (uint64_t)k * p.x_stride;
    unsigned char* __restrict__ out = p.packed + (uint64_t)k * p.packed_stride;
    float* __restrict__ norms = reinterpret_cast<float*>(out + p.norms_off);
    uint32_t* __restrict__ signs = reinterpret_cast<uint32_t*>(out + p.signs_off);
    uint32_t* __restrict__ levels = reinterpret_cast<uint32_t*>(out + p.levels_off);
    const uint64_t N = 1ull << p.log2N;
    const uint64_t slot0 = ((uint64_t)tile * nwaves + wave) * (uint64_t)(CH * kChunk) + lane * kLaneElems;

    LaneSpan span[CH];
    float v[CH][8];
    uint32_t rnd[CH][4];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        span[c] = lane_span(slot0 + (uint64_t)c * kChunk, p);
        load_lane(x, p.center, span[c], v[c]);
    }
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const uint64_t g = span[c].i >> 3;
        philox4x32_10((uint32_t)g, (uint32_t)(g >> 32), p.worker0 + k, p.round, p.key0, p.key1, rnd[c]);
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

    const float smax = p.smax;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        float inv = smax / norm[c];
        if (!(inv < INFINITY)) inv = 0.0f;
        uint32_t lvl[8];
        uint32_t sbyte = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float a = fminf(fabsf(v[c][e]) * inv, smax);
            const uint32_t fixed = (uint32_t)(a * 65536.0f);           // floor(a)*2^16 + trunc(frac(a)*2^16)
            const uint32_t word = rnd[c][e >> 1];
            const uint32_t r16 = (e & 1) ? (word >> 16) : (word & 0xFFFFu);
            lvl[e] = (fixed + r16) >> 16;                              // carry out of the low half = round up
            sbyte |= (v[c][e] < 0.0f ? 1u : 0u) << e;
        }
        const uint32_t nvalid = span[c].nvalid;
        const uint64_t i = span[c].i;
        // sign plane: 4 lanes make a word
        {
            uint32_t w = sbyte << (8u * (lane & 3u));
            w |= dpp_u32<kDppXor1>(w);
            w |= dpp_u32<kDppXor2>(w);
            if ((lane & 3u) == 0u && nvalid > 0) signs[i >> 5] = w;
        }
        if (M == 1) {
            uint32_t lb = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) lb |= lvl[e] << e;
            uint32_t w = lb << (8u * (lane & 3u));
            w |= dpp_u32<kDppXor1>(w);
            w |= dpp_u32<kDppXor2>(w);
            if ((lane & 3u) == 0u && nvalid > 0) levels[i >> 5] = w;
        } else if (M == 2) {
            uint32_t lb = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) lb |= lvl[e] << (2 * e);
            uint32_t w = lb << (16u * (lane & 1u));
            w |= dpp_u32<kDppXor1>(w);
            if ((lane & 1u) == 0u && nvalid > 0) levels[i >> 4] = w;
        } else if (M == 4) {
            uint32_t w = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) w |= lvl[e] << (4 * e);
            if (nvalid > 0) levels[i >> 3] = w;
        } else if (M == 8) {
            const uint32_t w0 = lvl[0] | (lvl[1] << 8) | (lvl[2] << 16) | (lvl[3] << 24);
            const uint32_t w1 = lvl[4] | (lvl[5] << 8) | (lvl[6] << 16) | (lvl[7] << 24);
            if (nvalid == 8) {
                *reinterpret_cast<uint2*>(levels + (i >> 2)) = make_uint2(w0, w1);
            } else {
                if (nvalid > 0) levels[i >> 2] = w0;
                if (nvalid > 4) levels[(i >> 2) + 1] = w1;
            }
        } else {  // M == 16
            const uint32_t w0 = lvl[0] | (lvl[1] << 16), w1 = lvl[2] | (lvl[3] << 16);
            const uint32_t w2 = lvl[4] | (lvl[5] << 16), w3 = lvl[6] | (lvl[7] << 16);
            if (nvalid == 8) {
                *reinterpret_cast<uint4*>(levels + (i >> 1)) = make_uint4(w0, w1, w2, w3);
            } else {
                if (nvalid > 0) levels[i >> 1] = w0;
                if (nvalid > 2) levels[(i >> 1) + 1] = w1;
                if (nvalid > 4) levels[(i >> 1) + 2] = w2;
                if (nvalid > 6) levels[(i >> 1) + 3] = w3;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Buckets wider than kMaxSinglePassBucket: pass A leaves the tree sum of every
// 4096-slot tile in the workspace, pass B finishes the tree per bucket and
// writes the scale, then k_quantize_pack<.., PRE = true> reads it.
// workspace[(k*nb + b)*P + t], P = N / 4096.
// ---------------------------------------------------------------------------
template <int KIND>
__global__ void k_tile_partials(const QParams p) {
    constexpr int CH = 2;
    __shared__ float sm[32];   // 16 wave totals; the upper half stays unused so a hoisted read of sm[base + r] stays inside
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t k = blockIdx.x / p.tiles_per_worker;
    const uint32_t tile = blockIdx.x - k * p.tiles_per_worker;
    const float* __restrict__ x = p.x + (uint64_t)k * p.x_stride;
    const uint64_t slot0 = ((uint64_t)tile * 4 + wave) * (uint64_t)(CH * kChunk) + lane * kLaneElems;
    float t[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        float v[8];
        const LaneSpan s = lane_span(slot0 + (uint64_t)c * kChunk, p);
        load_lane(x, p.center, s, v);
        t[c] = lane_butterfly<KIND>(lane_tree<KIND>(v), 64);
    }
    t[0] = combine<KIND>(t[0], t[1]);
    if (lane == 0) sm[wave] = t[0];
    __syncthreads();
    if (threadIdx.x == 0) {
        const float total = combine<KIND>(combine<KIND>(sm[0], sm[1]), combine<KIND>(sm[2], sm[3]));
        // tiles of a bucket are consecutive in slot space, so (bucket, tile in bucket) = tile index
        p.workspace[(uint64_t)k * p.tiles_per_worker + tile] = total;
    }
}

template <int KIND>
__global__ void k_finish_norms(const QParams p, uint64_t P) {
    const uint64_t kb = blockIdx.x;                     // k*nb + b
    const uint32_t k = (uint32_t)(kb / p.nb);
    const uint64_t b = kb - (uint64_t)k * p.nb;
    float* ws = p.workspace + kb * P;
    for (uint64_t h = 1; h < P; h <<= 1) {
        for (uint64_t r = (uint64_t)threadIdx.x * 2 * h; r < P; r += (uint64_t)blockDim.x * 2 * h)
            ws[r] = combine<KIND>(ws[r], ws[r + h]);
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        float* norms = reinterpret_cast<float*>(p.packed + (uint64_t)k * p.packed_stride + p.norms_off);
        norms[b] = (KIND == QESGD_NORM_L2) ? sqrtf(ws[0]) : ws[0];
    }
}

template <int M, int CH, bool PRE>
int launch_kind(const QParams& p, uint32_t norm_kind, dim3 grid, dim3 block, hipStream_t st) {
    if (norm_kind == QESGD_NORM_L2)
        hipLaunchKernelGGL((k_quantize_pack<M, CH, QESGD_NORM_L2, PRE>), grid, block, 0, st, p);
    else
        hipLaunchKernelGGL((k_quantize_pack<M, CH, QESGD_NORM_MAX, PRE>), grid, block, 0, st, p);
    return 0;
}

template <int CH, bool PRE>
int launch_m(const QParams& p, uint32_t m, uint32_t norm_kind, dim3 grid, dim3 block, hipStream_t st) {
    switch (m) {
        case 1: return launch_kind<1, CH, PRE>(p, norm_kind, grid, block, st);
        case 2: return launch_kind<2, CH, PRE>(p, norm_kind, grid, block, st);
        case 4: return launch_kind<4, CH, PRE>(p, norm_kind, grid, block, st);
        case 8: return launch_kind<8, CH, PRE>(p, norm_kind, grid, block, st);
        default: return launch_kind<16, CH, PRE>(p, norm_kind, grid, block, st);
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

int launch_quantize(const Shape& sh, const QuantizeArgs& a) {
    QParams p{};
    p.x = a.x;
    p.center = a.center;
    p.packed = a.packed;
    p.workspace = a.workspace;
    p.x_stride = a.x_stride;
    p.packed_stride = a.packed_stride;
    p.d = sh.d;
    p.B = sh.B;
    p.nb = sh.nb;
    p.norms_off = sh.lay.norms_off;
    p.signs_off = sh.lay.signs_off;
    p.levels_off = sh.lay.levels_off;
    p.log2N = sh.log2N;
    p.key0 = (uint32_t)a.seed;
    p.key1 = (uint32_t)(a.seed >> 32);
    p.round = a.round;
    p.worker0 = a.worker0;
    p.smax = (float)(sh.s - 1);

    const uint64_t slots = sh.nb * sh.N;                 // slot space of one worker
    const bool two_pass = sh.N > kMaxSinglePassBucket;
    uint32_t ch = 2, nwaves = 4;
    if (!two_pass) {
        if (sh.N == 8192) nwaves = 8;
        else if (sh.N == 16384) nwaves = 16;
        else if (sh.N == 32768) { ch = 4; nwaves = 16; }
    }
    const uint64_t tile = (uint64_t)nwaves * ch * kChunk;
    const uint64_t tiles = (slots + tile - 1) / tile;
    if (tiles * a.K >= (1ull << 31)) return QESGD_ERR_DIM;
    p.tiles_per_worker = (uint32_t)tiles;
    const dim3 grid((uint32_t)(tiles * a.K));
    const dim3 block(nwaves * kWaveSize);

    if (two_pass) {
        const uint64_t P = sh.N / kPartialTile;          // tiles == nb * P
        if (a.norm_kind == QESGD_NORM_L2) {
            hipLaunchKernelGGL(k_tile_partials<QESGD_NORM_L2>, grid, block, 0, a.stream, p);
            hipLaunchKernelGGL(k_finish_norms<QESGD_NORM_L2>, dim3((uint32_t)(sh.nb * a.K)), dim3(256), 0, a.stream, p, P);
        } else {
            hipLaunchKernelGGL(k_tile_partials<QESGD_NORM_MAX>, grid, block, 0, a.stream, p);
            hipLaunchKernelGGL(k_finish_norms<QESGD_NORM_MAX>, dim3((uint32_t)(sh.nb * a.K)), dim3(256), 0, a.stream, p, P);
        }
        const int rc = check_launch();
        if (rc != QESGD_OK) return rc;
        launch_m<2, true>(p, sh.m, a.norm_kind, grid, block, a.stream);
    } else if (ch == 2) {
        launch_m<2, false>(p, sh.m, a.norm_kind, grid, block, a.stream);
    } else {
        launch_m<4, false>(p, sh.m, a.norm_kind, grid, block, a.stream);
    }
    return check_launch();
}

}  // namespace qesgd
