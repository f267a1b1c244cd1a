// Worker side of a QESGD round on gfx950: bucket scale, stochastic rounding
// (Sec. 2.1, Eq. (2)) and bit packing, one pass over the input.
//
// Mapping.  The coordinates are laid out in "slot space": bucket b owns the N
// slots [b*N, (b+1)*N), N = bucket size zero-padded to a power of two, so that
// every bucket starts on a power-of-two boundary whatever its length.  A lane
// owns 8 consecutive slots (two 128-bit loads, one Philox call, one sign byte),
// a wavefront owns CH chunks of 64 x 8 = 512 slots, a workgroup owns a tile of
// nwaves x CH x 512 slots.  The fp32 sum of squares is the balanced binary tree
// over slot index bits: bits 0-2 inside the lane, bits 3-8 as an xor butterfly
// over lanes (DPP for masks 1,2,4,8; row / half swaps for 16,32), then the
// chunks of a wave, then the waves of a workgroup through LDS.  Every lane ends
// with its bucket's total, so the scale never goes through memory.
//
// The kernels share the arithmetic:
//   k_quantize_pack_fast  power-of-two buckets, L2 scale, level width dividing
//                         32, tiles that lie wholly inside the vector.  N is a
//                         template parameter, so the whole tile is straight-line
//                         code without guards; the ragged last tile of a worker
//                         runs the guarded body in the same launch.
//   k_quantize_pack       everything else: buckets that are not a power of two,
//                         max-norm, level widths 3/5/6/7, tiny vectors, and the
//                         last pass of buckets too wide for one workgroup.
//   k_tile_partials(_fast), k_finish_norms, k_quantize_pack_pre_fast
//                         buckets wider than kMaxSinglePassBucket: per-tile tree
//                         sums into the workspace, the rest of each bucket's
//                         tree, then the quantiser with the scale read back.
#include <mutex>

#include "qesgd_quantize_device.h"

// Scratch of the entry point that allocates nothing: the partial sums of the two-pass path for
// callers that cannot bring a workspace.  One copy per GPU, held until the process ends; every
// call on a GPU shares it.  In host code this name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) float scratch[qesgd::kStaticScratchFloats];

namespace qesgd {
namespace {

// PRE (second pass of a wide bucket): workers and tiles are walked backwards, so that the launch
// starts with what the partial-sum pass read last and most of it is still in the memory-side cache.
template <int M, int CH, int KIND, bool PRE>
__global__ void k_quantize_pack(const QParams p) {
    __shared__ float sm[32];
    uint32_t k = blockIdx.x / p.tiles_per_worker;
    uint32_t local = blockIdx.x - k * p.tiles_per_worker;
    if (PRE) {
        k = p.group_workers - 1u - k;
        local = p.tiles_per_worker - 1u - local;
    }
    guarded_tile<M, CH, KIND, PRE>(p, k, p.tile0 + local, sm);
}

// One tile per workgroup; the ragged last tile of a worker, if any, runs the guarded code in
// the same launch.  (Walking several tiles per workgroup with the next tile's loads
// in flight was measured and is slower: the packed stores of a long-lived workgroup spread
// out in time and the mixed read/write stream to HBM loses more than the prefetch gains.)
template <int M, int LOG2N, bool CENTER>
__global__ void __launch_bounds__(Geo<LOG2N>::NW * 64) k_quantize_pack_fast(const QParams p) {
    constexpr int CH = Geo<LOG2N>::CH;
    constexpr uint32_t TILE = Geo<LOG2N>::TILE;
    __shared__ float sm[32];

    const uint32_t per_worker = p.full_tiles + p.tail_tiles;
    uint32_t k, t;
    if (CENTER) {
        // All workers read the same `center`.  Workgroups are handed to the 8 XCDs round-robin by
        // id, so the K workgroups of one tile get ids 8 apart: they run on one XCD one after the
        // other, and all but the first find the tile of `center` in that XCD's L2.
        const uint32_t K = p.group_workers;
        const uint32_t tiles8 = p.full_tiles & ~7u;
        const uint32_t span = 8u * K;
        if (blockIdx.x < (tiles8 >> 3) * span) {
            const uint32_t g = blockIdx.x / span, r = blockIdx.x - g * span;
            k = r >> 3;
            t = g * 8u + (r & 7u);
        } else {                                          // fewer than 8 tiles left, and the ragged one
            const uint32_t rest = per_worker - tiles8;
            const uint32_t r = blockIdx.x - (tiles8 >> 3) * span;
            k = r / rest;
            t = tiles8 + (r - k * rest);
        }
    } else {
        k = blockIdx.x / per_worker;
        t = blockIdx.x - k * per_worker;
    }
    if (t >= p.full_tiles) {                              // the ragged last tile of the worker (at most one)
        guarded_tile<M, CH, QESGD_NORM_L2, false>(p, k, t, sm);
        return;
    }
    const float* __restrict__ xk = p.x + (uint64_t)k * p.x_stride;
    const float* __restrict__ ck = p.center;
    unsigned char* __restrict__ out = p.packed + (uint64_t)k * p.packed_stride;
    FastCtx cx;
    cx.norms = reinterpret_cast<float*>(out + p.norms_off);
    cx.signs = reinterpret_cast<uint32_t*>(out + p.signs_off);
    cx.levels = reinterpret_cast<uint32_t*>(out + p.levels_off);
    cx.lane = threadIdx.x & 63u;
    cx.wave = threadIdx.x >> 6;
    cx.lane_off = cx.wave * (uint32_t)(CH * kChunk) + cx.lane * kLaneElems;   // coordinate offset inside a tile
    cx.worker = p.worker0 + k;
    cx.round = p.round;
    cx.key0 = p.key0;
    cx.key1 = p.key1;
    cx.smax = p.smax;

    float buf[CH][8];
    load_tile<CH, CENTER>(xk + (uint64_t)t * TILE, ck + (uint64_t)t * TILE, cx.lane_off, buf);
    process_tile<M, LOG2N>(cx, buf, t, sm);
}

// The center form for several workers: a workgroup owns one tile of every worker, keeps the tile
// of `center` in registers and takes the workers one after the other with the next worker's loads
// in flight, so `center` is read once per tile instead of once per tile and worker.
template <int M, int LOG2N>
__global__ void __launch_bounds__(Geo<LOG2N>::NW * 64) k_quantize_pack_center(const QParams p) {
    constexpr int CH = Geo<LOG2N>::CH;
    constexpr uint32_t TILE = Geo<LOG2N>::TILE;
    __shared__ float sm[2][32];             // alternate per worker: one barrier per tile suffices
    const uint32_t t = blockIdx.x;
    const uint32_t K = p.group_workers;
    if (t >= p.full_tiles) {                              // the ragged last tile
        for (uint32_t k = 0; k < K; ++k) guarded_tile<M, CH, QESGD_NORM_L2, false>(p, k, t, sm[k & 1u]);
        return;
    }
    FastCtx cx;
    cx.lane = threadIdx.x & 63u;
    cx.wave = threadIdx.x >> 6;
    cx.lane_off = cx.wave * (uint32_t)(CH * kChunk) + cx.lane * kLaneElems;
    cx.round = p.round;
    cx.key0 = p.key0;
    cx.key1 = p.key1;
    cx.smax = p.smax;
    const uint64_t e0 = (uint64_t)t * TILE;
    float4 ca[CH], cb[CH], a[CH], b[CH], na[CH], nb2[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const uint32_t o = cx.lane_off + (uint32_t)c * kChunk;
        ca[c] = *reinterpret_cast<const float4*>(p.center + e0 + o);
        cb[c] = *reinterpret_cast<const float4*>(p.center + e0 + o + 4);
        a[c] = *reinterpret_cast<const float4*>(p.x + e0 + o);
        b[c] = *reinterpret_cast<const float4*>(p.x + e0 + o + 4);
    }
    for (uint32_t k = 0; k < K; ++k) {
        if (k + 1 < K) {
            const float* __restrict__ xn = p.x + (uint64_t)(k + 1) * p.x_stride + e0;
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const uint32_t o = cx.lane_off + (uint32_t)c * kChunk;
                na[c] = *reinterpret_cast<const float4*>(xn + o);
                nb2[c] = *reinterpret_cast<const float4*>(xn + o + 4);
            }
        }
        float v[CH][8];
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            v[c][0] = a[c].x - ca[c].x; v[c][1] = a[c].y - ca[c].y; v[c][2] = a[c].z - ca[c].z; v[c][3] = a[c].w - ca[c].w;
            v[c][4] = b[c].x - cb[c].x; v[c][5] = b[c].y - cb[c].y; v[c][6] = b[c].z - cb[c].z; v[c][7] = b[c].w - cb[c].w;
        }
        unsigned char* __restrict__ out = p.packed + (uint64_t)k * p.packed_stride;
        cx.norms = reinterpret_cast<float*>(out + p.norms_off);
        cx.signs = reinterpret_cast<uint32_t*>(out + p.signs_off);
        cx.levels = reinterpret_cast<uint32_t*>(out + p.levels_off);
        cx.worker = p.worker0 + k;
        process_tile<M, LOG2N>(cx, v, t, sm[k & 1u]);
        if (k + 1 < K) {
#pragma unroll
            for (int c = 0; c < CH; ++c) { a[c] = na[c]; b[c] = nb2[c]; }
        }
    }
}

// Tree sum (or max) of one 4096-slot tile of worker k with every access guarded per lane, left in
// the workspace.  Tiles of a bucket are consecutive in slot space, so the workspace index of
// (bucket, tile in bucket) is the tile index.  sm: 4 floats of LDS.
template <int KIND>
__device__ __forceinline__ void guarded_partial_tile(const QParams& p, uint32_t k, uint32_t tile, float* sm) {
    constexpr int CH = 2;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = threadIdx.x >> 6;
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
        p.workspace[(uint64_t)k * p.ws_tiles_per_worker + tile] = total;
    }
}

// Buckets wider than kMaxSinglePassBucket, tiles wholly inside the vector (slot == coordinate:
// power-of-two bucket, or a single bucket).  First pass: tree sum of one 4096-coordinate tile into
// the workspace.  Last pass: the quantiser with the bucket scale read from the norms plane; a tile
// never straddles two such buckets, so the scale is one scalar per workgroup.
template <bool CENTER>
__global__ void __launch_bounds__(256) k_tile_partials_fast(const QParams p) {
    constexpr int KIND = QESGD_NORM_L2;
    __shared__ float sm[4];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t per_worker = p.full_tiles + p.tail_tiles;
    const uint32_t k = blockIdx.x / per_worker;
    const uint32_t t = blockIdx.x - k * per_worker;
    if (t >= p.full_tiles) {                              // the ragged last tile of the worker (at most one)
        guarded_partial_tile<KIND>(p, k, t, sm);
        return;
    }
    const uint32_t lane_off = wave * (2u * kChunk) + lane * kLaneElems;
    float v[2][8];
    load_tile<2, CENTER>(p.x + (uint64_t)k * p.x_stride + (uint64_t)t * kPartialTile,
                         p.center + (uint64_t)t * kPartialTile, lane_off, v);
    const float t0 = lane_butterfly<KIND>(lane_tree<KIND>(v[0]), 64);
    const float t1 = lane_butterfly<KIND>(lane_tree<KIND>(v[1]), 64);
    if (lane == 0) sm[wave] = t0 + t1;
    __syncthreads();
    if (threadIdx.x == 0) p.workspace[(uint64_t)k * p.ws_tiles_per_worker + t] = (sm[0] + sm[1]) + (sm[2] + sm[3]);
}

template <int M, bool CENTER>
__global__ void __launch_bounds__(256) k_quantize_pack_pre_fast(const QParams p) {
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t per_worker = p.full_tiles + p.tail_tiles;
    const uint32_t kf = blockIdx.x / per_worker;
    const uint32_t k = p.group_workers - 1u - kf;                       // backwards: see k_quantize_pack
    const uint32_t t = per_worker - 1u - (blockIdx.x - kf * per_worker);
    if (t >= p.full_tiles) {                              // the ragged last tile of the worker (at most one)
        guarded_tile<M, 2, QESGD_NORM_L2, true>(p, k, t, nullptr);
        return;
    }
    unsigned char* __restrict__ out = p.packed + (uint64_t)k * p.packed_stride;
    const float* __restrict__ norms = reinterpret_cast<const float*>(out + p.norms_off);
    uint32_t* __restrict__ signs = reinterpret_cast<uint32_t*>(out + p.signs_off);
    uint32_t* __restrict__ levels = reinterpret_cast<uint32_t*>(out + p.levels_off);
    const uint32_t lane_off = wave * (2u * kChunk) + lane * kLaneElems;
    const uint64_t e0 = (uint64_t)t * kPartialTile;
    float v[2][8];
    load_tile<2, CENTER>(p.x + (uint64_t)k * p.x_stride + e0, p.center + e0, lane_off, v);
    const float inv = inverse_step(norms[e0 >> p.log2N], p.smax);
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const uint64_t i = e0 + lane_off + (uint32_t)c * kChunk;
        const uint64_t g = i >> 3;
        uint32_t rnd[4];
        philox4x32_10((uint32_t)g, (uint32_t)(g >> 32), p.worker0 + k, p.round, p.key0, p.key1, rnd);
        uint32_t sign_byte, bits[4];
        round_and_pack<M>(v[c], rnd, inv, p.smax, sign_byte, bits);
        store_codes<M>(signs, levels, i, 8u, lane, sign_byte, bits);
    }
}

// ---------------------------------------------------------------------------
// Buckets wider than kMaxSinglePassBucket, guarded versions: pass A leaves the
// tree sum of a 4096-slot tile in the workspace, pass B finishes the tree per
// bucket and writes the scale, then k_quantize_pack<.., PRE = true> reads it.
// workspace[(k*nb + b)*P + t], P = N / 4096.
// ---------------------------------------------------------------------------
template <int KIND>
__global__ void k_tile_partials(const QParams p) {
    __shared__ float sm[4];
    const uint32_t k = blockIdx.x / p.tiles_per_worker;
    const uint32_t tile = p.tile0 + (blockIdx.x - k * p.tiles_per_worker);
    guarded_partial_tile<KIND>(p, k, tile, sm);
}

// Finishes the tree of one bucket: P leaves (a power of two, >= 16), of which only the first
// `valid` were written (the rest of the padded bucket is +0, the identity of both combines, and is
// never read).  One workgroup of W = 1..16 waves per (worker, bucket) walks the leaves in tiles of
// W x 2 chunks x 512, each reduced like a tile of the first pass (leaf index bits 0-2 in the
// lane, 3-8 across lanes, 9 across the two chunks, then the waves); the tile totals are joined by
// a binary counter: stack[l] holds the finished subtree of 2^l tiles that waits for its right
// sibling.  W is the largest power of two with W x 1024 <= max(P, 1024).
template <int KIND>
__global__ void __launch_bounds__(1024) k_finish_norms(const QParams p, uint64_t P, uint32_t dense) {
    __shared__ float sm[2][16];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t nwaves = blockDim.x >> 6;
    const uint64_t tile = (uint64_t)nwaves * 1024u;
    const uint64_t kb = blockIdx.x;                     // k*nb + b
    const uint32_t k = (uint32_t)(kb / p.nb);
    const uint64_t b = kb - (uint64_t)k * p.nb;
    const float* __restrict__ ws = p.workspace + kb * P;
    uint64_t valid = P;
    if (dense) {
        const uint64_t left = p.data_tiles - b * P;     // buckets before the last are full
        valid = left < P ? left : P;
    }
    const uint64_t iters = (P + tile - 1) / tile;                         // a power of two
    float stack[16];
#pragma unroll
    for (int l = 0; l < 16; ++l) stack[l] = 0.0f;
    for (uint64_t it = 0; it < iters; ++it) {
        float total = 0.0f;
        const uint64_t base = it * tile;
        if (base < valid) {                              // uniform: tiles beyond `valid` are all +0
            float t2[2];
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const uint64_t j = base + wave * 1024u + (uint32_t)c * kChunk + lane * kLaneElems;
                float q[8];
                if (j + 8 <= valid) {
                    const float4 a0 = *reinterpret_cast<const float4*>(ws + j);
                    const float4 a1 = *reinterpret_cast<const float4*>(ws + j + 4);
                    q[0] = a0.x; q[1] = a0.y; q[2] = a0.z; q[3] = a0.w;
                    q[4] = a1.x; q[5] = a1.y; q[6] = a1.z; q[7] = a1.w;
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) q[e] = (j + e < valid) ? ws[j + e] : 0.0f;
                }
                t2[c] = lane_butterfly<KIND>(lane_tree_of_partials<KIND>(q), 64);
            }
            float* buf = sm[it & 1u];
            if (lane == 0) buf[wave] = combine<KIND>(t2[0], t2[1]);
            __syncthreads();                             // one barrier per tile: the buffers alternate
            total = lds_tree16<KIND>(buf, 0, nwaves);
        }
#pragma unroll
        for (int l = 0; l < 16; ++l) {                   // 16 waves whenever P > 16384: iters <= 2^40 / 4096 / 16384 = 2^14
            if (((it >> l) & 1u) == 0u) { stack[l] = total; break; }
            total = combine<KIND>(stack[l], total);
        }
    }
    if (threadIdx.x == 0) {
        float result = stack[0];
#pragma unroll
        for (int l = 1; l < 16; ++l)
            if ((iters >> l) & 1u) result = stack[l];
        float* norms = reinterpret_cast<float*>(p.packed + (uint64_t)k * p.packed_stride + p.norms_off);
        norms[b] = (KIND == QESGD_NORM_L2) ? sqrtf(result) : result;
    }
}

// ---------------------------------------------------------------------------
// Launch plumbing.
// ---------------------------------------------------------------------------
template <int M, int CH, bool PRE>
void launch_kind(const QParams& p, uint32_t norm_kind, dim3 grid, dim3 block, hipStream_t st) {
    if (norm_kind == QESGD_NORM_L2)
        hipLaunchKernelGGL((k_quantize_pack<M, CH, QESGD_NORM_L2, PRE>), grid, block, 0, st, p);
    else
        hipLaunchKernelGGL((k_quantize_pack<M, CH, QESGD_NORM_MAX, PRE>), grid, block, 0, st, p);
}

template <int CH, bool PRE>
void launch_m(const QParams& p, uint32_t m, uint32_t norm_kind, dim3 grid, dim3 block, hipStream_t st) {
    switch (m) {
        case 1: launch_kind<1, CH, PRE>(p, norm_kind, grid, block, st); break;
        case 2: launch_kind<2, CH, PRE>(p, norm_kind, grid, block, st); break;
        case 3: launch_kind<3, CH, PRE>(p, norm_kind, grid, block, st); break;
        case 4: launch_kind<4, CH, PRE>(p, norm_kind, grid, block, st); break;
        case 5: launch_kind<5, CH, PRE>(p, norm_kind, grid, block, st); break;
        case 6: launch_kind<6, CH, PRE>(p, norm_kind, grid, block, st); break;
        case 7: launch_kind<7, CH, PRE>(p, norm_kind, grid, block, st); break;
        case 8: launch_kind<8, CH, PRE>(p, norm_kind, grid, block, st); break;
        default: launch_kind<16, CH, PRE>(p, norm_kind, grid, block, st); break;
    }
}

template <int M, int LOG2N>
void launch_fast_one(const QParams& p, uint32_t blocks, hipStream_t st) {
    // With a center and enough tiles to fill the chip many times over (measured: it pays from about
    // 64 waves per SIMD on), a workgroup takes one tile of every worker and reads `center` once.
    if (p.center && p.group_workers > 1 && (uint64_t)p.full_tiles * Geo<LOG2N>::NW >= 65536u) {
        hipLaunchKernelGGL((k_quantize_pack_center<M, LOG2N>), dim3(p.full_tiles + p.tail_tiles),
                           dim3(Geo<LOG2N>::NW * 64), 0, st, p);
        return;
    }
    if (p.center)
        hipLaunchKernelGGL((k_quantize_pack_fast<M, LOG2N, true>), dim3(blocks), dim3(Geo<LOG2N>::NW * 64), 0, st, p);
    else
        hipLaunchKernelGGL((k_quantize_pack_fast<M, LOG2N, false>), dim3(blocks), dim3(Geo<LOG2N>::NW * 64), 0, st, p);
}

template <int M>
void launch_fast_n(const QParams& p, uint32_t blocks, hipStream_t st) {
    switch (p.log2N) {
        case 5: launch_fast_one<M, 5>(p, blocks, st); break;
        case 6: launch_fast_one<M, 6>(p, blocks, st); break;
        case 7: launch_fast_one<M, 7>(p, blocks, st); break;
        case 8: launch_fast_one<M, 8>(p, blocks, st); break;
        case 9: launch_fast_one<M, 9>(p, blocks, st); break;
        case 10: launch_fast_one<M, 10>(p, blocks, st); break;
        case 11: launch_fast_one<M, 11>(p, blocks, st); break;
        case 12: launch_fast_one<M, 12>(p, blocks, st); break;
        case 13: launch_fast_one<M, 13>(p, blocks, st); break;
        case 14: launch_fast_one<M, 14>(p, blocks, st); break;
        default: launch_fast_one<M, 15>(p, blocks, st); break;
    }
}

void launch_fast(const QParams& p, uint32_t m, uint32_t blocks, hipStream_t st) {
    switch (m) {
        case 1: launch_fast_n<1>(p, blocks, st); break;
        case 2: launch_fast_n<2>(p, blocks, st); break;
        case 4: launch_fast_n<4>(p, blocks, st); break;
        case 8: launch_fast_n<8>(p, blocks, st); break;
        default: launch_fast_n<16>(p, blocks, st); break;
    }
}

template <int M>
void launch_pre_fast_m(const QParams& p, uint32_t blocks, hipStream_t st) {
    if (p.center) hipLaunchKernelGGL((k_quantize_pack_pre_fast<M, true>), dim3(blocks), dim3(256), 0, st, p);
    else hipLaunchKernelGGL((k_quantize_pack_pre_fast<M, false>), dim3(blocks), dim3(256), 0, st, p);
}

void launch_pre_fast(const QParams& p, uint32_t m, uint32_t blocks, hipStream_t st) {
    switch (m) {
        case 1: launch_pre_fast_m<1>(p, blocks, st); break;
        case 2: launch_pre_fast_m<2>(p, blocks, st); break;
        case 3: launch_pre_fast_m<3>(p, blocks, st); break;
        case 4: launch_pre_fast_m<4>(p, blocks, st); break;
        case 5: launch_pre_fast_m<5>(p, blocks, st); break;
        case 6: launch_pre_fast_m<6>(p, blocks, st); break;
        case 7: launch_pre_fast_m<7>(p, blocks, st); break;
        case 8: launch_pre_fast_m<8>(p, blocks, st); break;
        default: launch_pre_fast_m<16>(p, blocks, st); break;
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

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices] = {};     // device address of `scratch` on each GPU, looked up once

}  // namespace

// Device address of the current GPU's copy of `scratch`.  The first call on a device asks the
// runtime for the address (each GPU holds its own copy at its own address); later calls read
// the table.
int static_scratch(float** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && (dev < 0 || dev >= kMaxDevices)) e = hipErrorInvalidDevice;
    if (e != hipSuccess) {
        set_last_hip_error((int)e);
        return QESGD_ERR_HIP;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            set_last_hip_error((int)(e != hipSuccess ? e : hipErrorInvalidSymbol));
            return QESGD_ERR_HIP;
        }
        g_scratch_ptr[dev] = static_cast<float*>(ptr);
    }
    *out = g_scratch_ptr[dev];
    return QESGD_OK;
}

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
    p.group_workers = a.K;

    const uint64_t slots = sh.nb * sh.N;                 // slot space of one worker
    const bool two_pass = sh.N > kMaxSinglePassBucket;
    // Tiles that lie wholly inside the vector go to the fast kernel when the bucket is a
    // power of two (slot == coordinate), the scale is the L2 norm and the level width
    // divides a word (the other widths are served by the generic kernel alone).
    const bool fast = !two_pass && a.norm_kind == QESGD_NORM_L2 && sh.N == sh.B && sh.log2N >= 5 &&
                      32u % sh.m == 0u;
    uint32_t ch = 2, nwaves = 4;                         // generic kernel: 2 chunks per wave, 4..16 waves
    if (fast) {
        fast_geometry(sh.N, &ch, &nwaves);
    } else if (!two_pass) {
        if (sh.N == 8192) nwaves = 8;
        else if (sh.N == 16384) nwaves = 16;
        else if (sh.N == 32768) { ch = 4; nwaves = 16; }
    }
    const uint64_t tile = (uint64_t)nwaves * ch * kChunk;
    const uint64_t tiles = (slots + tile - 1) / tile;
    if (tiles * a.K >= (1ull << 31)) return QESGD_ERR_DIM;
    const dim3 block(nwaves * kWaveSize);

    if (two_pass) {
        // Slot space equals coordinate space when the bucket is a power of two or there is a single
        // bucket; then only the tiles that hold coordinates are visited, and the ones wholly inside
        // the vector take the unguarded kernels.
        const uint64_t P = sh.N / kPartialTile;          // tiles == nb * P
        uint32_t finish_waves = 1;
        while (finish_waves < 16 && (uint64_t)finish_waves * 1024u < P) finish_waves <<= 1;
        const dim3 finish_block(finish_waves * kWaveSize);
        const bool dense = sh.N == sh.B || sh.nb == 1;
        const uint64_t data_tiles = dense ? (sh.d + kPartialTile - 1) / kPartialTile : tiles;
        const uint64_t full_tiles = (dense && a.norm_kind == QESGD_NORM_L2) ? sh.d / kPartialTile : 0;
        p.ws_tiles_per_worker = (uint32_t)tiles;
        p.data_tiles = data_tiles;
        p.full_tiles = (uint32_t)full_tiles;
        p.tile0 = (uint32_t)full_tiles;
        p.tiles_per_worker = (uint32_t)(data_tiles - full_tiles);
        // The second pass re-reads what the first read.  Workers are taken in groups whose input
        // fits the memory-side cache (all of them at once when everything fits), the partial sums,
        // the rest of the tree and the quantiser one group after the other, and the quantiser walks
        // its group backwards: what the first pass read last is read first.
        const uint64_t worker_bytes = 4u * sh.d;
        uint32_t group = a.K;
        if ((uint64_t)a.K * worker_bytes > kCacheBudgetBytes) {
            const uint64_t fit = kCacheBudgetBytes / worker_bytes;
            group = fit < 1 ? 1u : (uint32_t)fit;
        }
        for (uint32_t k0 = 0; k0 < a.K; k0 += group) {
            const uint32_t kg = a.K - k0 < group ? a.K - k0 : group;
            p.x = a.x + (uint64_t)k0 * a.x_stride;
            p.packed = a.packed + (uint64_t)k0 * a.packed_stride;
            p.workspace = a.workspace + (uint64_t)k0 * tiles;
            p.worker0 = a.worker0 + k0;
            p.group_workers = kg;
            const dim3 finish_grid((uint32_t)(sh.nb * kg));
            int rc;
            if (full_tiles > 0) {
                // dense tiles unguarded, the ragged last tile of each worker guarded in the same launches
                p.tail_tiles = (uint32_t)(data_tiles - full_tiles);
                const dim3 grid((uint32_t)(data_tiles * kg));
                if (p.center) hipLaunchKernelGGL(k_tile_partials_fast<true>, grid, block, 0, a.stream, p);
                else hipLaunchKernelGGL(k_tile_partials_fast<false>, grid, block, 0, a.stream, p);
                hipLaunchKernelGGL(k_finish_norms<QESGD_NORM_L2>, finish_grid, finish_block, 0, a.stream, p, P, 1u);
                rc = check_launch();
                if (rc != QESGD_OK) return rc;
                launch_pre_fast(p, sh.m, (uint32_t)(data_tiles * kg), a.stream);
            } else {
                const dim3 grid((uint32_t)(data_tiles * kg));
                if (a.norm_kind == QESGD_NORM_L2) {
                    hipLaunchKernelGGL(k_tile_partials<QESGD_NORM_L2>, grid, block, 0, a.stream, p);
                    hipLaunchKernelGGL(k_finish_norms<QESGD_NORM_L2>, finish_grid, finish_block, 0, a.stream, p, P, dense ? 1u : 0u);
                } else {
                    hipLaunchKernelGGL(k_tile_partials<QESGD_NORM_MAX>, grid, block, 0, a.stream, p);
                    hipLaunchKernelGGL(k_finish_norms<QESGD_NORM_MAX>, finish_grid, finish_block, 0, a.stream, p, P, dense ? 1u : 0u);
                }
                rc = check_launch();
                if (rc != QESGD_OK) return rc;
                launch_m<2, true>(p, sh.m, a.norm_kind, grid, block, a.stream);
            }
            rc = check_launch();
            if (rc != QESGD_OK) return rc;
        }
        return QESGD_OK;
    }

    if (fast) {
        // full_tiles may be 0 (a vector shorter than a tile): the launch is then one guarded tile per worker
        p.full_tiles = (uint32_t)(sh.d / tile);
        p.tail_tiles = (uint32_t)(tiles - p.full_tiles);
        launch_fast(p, sh.m, (uint32_t)(tiles * a.K), a.stream);
        return check_launch();
    }
    p.tile0 = 0;
    p.tiles_per_worker = (uint32_t)tiles;
    const dim3 grid((uint32_t)(tiles * a.K));
    if (ch == 2) launch_m<2, false>(p, sh.m, a.norm_kind, grid, block, a.stream);
    else launch_m<4, false>(p, sh.m, a.norm_kind, grid, block, a.stream);
    return check_launch();
}

}  // namespace qesgd
