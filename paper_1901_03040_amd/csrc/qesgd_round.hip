// A whole round in one launch, for one GPU that holds the K workers and the server: every
// worker's quantise + pack (Sec. 2.1, Eq. (2); Sec. 3) and the server's sum over workers and
// update (Alg. 3, server task; Alg. 2: u = w_t + z) with the results of the two-call form, bit
// for bit, including the packed blocks.
//
// No grid-wide wait is needed: buckets are independent on the worker side and coordinates on the
// server side, so a workgroup that owns one tile of every worker has all it needs for that tile of
// z.  It takes the workers one after the other (the next worker's loads in flight while the
// current one is rounded), keeps the running sum of the dequantised codes in registers, and writes
// z, u and the running sum of z at the end.  The packed codes are written but never read back.
// What this saves is one dependent launch per round and K*P bytes of reads; it exists for sizes at
// which a round is launch-bound.
#include "qesgd_aggregate_device.h"
#include "qesgd_quantize_device.h"

namespace qesgd {
namespace {

struct RParams {
    QParams q;
    const float* w;
    float* zbar;
    float* u;
    float* zsum;
    float rcpK;      // exact 1/K when K is a power of two, else 0
    uint32_t K;
};

template <int CH>
__device__ __forceinline__ void load_raw(const float* __restrict__ xt, uint32_t lane_off, float4 (&a)[CH], float4 (&b)[CH]) {
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const uint32_t o = lane_off + (uint32_t)c * kChunk;
        a[c] = *reinterpret_cast<const float4*>(xt + o);
        b[c] = *reinterpret_cast<const float4*>(xt + o + 4);
    }
}

template <int M, int LOG2N, bool CENTER>
__global__ void __launch_bounds__(Geo<LOG2N>::NW * 64) k_round_fused(const RParams r) {
    constexpr int CH = Geo<LOG2N>::CH;
    constexpr uint32_t TILE = Geo<LOG2N>::TILE;
    __shared__ float sm[2][32];             // alternate per worker: one barrier per tile suffices
    __shared__ float4 stage[Geo<LOG2N>::NW][128];
    const QParams& p = r.q;
    const uint32_t t = blockIdx.x;
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t lane_off = wave * (uint32_t)(CH * kChunk) + lane * kLaneElems;

    float acc[CH][8];
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[c][e] = 0.0f;

    if (t < p.full_tiles) {
        const uint64_t e0 = (uint64_t)t * TILE;
        float4 ca[CH], cb[CH], a[CH], b[CH], na[CH], nbuf[CH];
        if (CENTER) load_raw<CH>(p.center + e0, lane_off, ca, cb);
        load_raw<CH>(p.x + e0, lane_off, a, b);
        for (uint32_t k = 0; k < r.K; ++k) {
            if (k + 1 < r.K) load_raw<CH>(p.x + (uint64_t)(k + 1) * p.x_stride + e0, lane_off, na, nbuf);
            float v[CH][8];
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                v[c][0] = a[c].x; v[c][1] = a[c].y; v[c][2] = a[c].z; v[c][3] = a[c].w;
                v[c][4] = b[c].x; v[c][5] = b[c].y; v[c][6] = b[c].z; v[c][7] = b[c].w;
                if (CENTER) {
                    v[c][0] -= ca[c].x; v[c][1] -= ca[c].y; v[c][2] -= ca[c].z; v[c][3] -= ca[c].w;
                    v[c][4] -= cb[c].x; v[c][5] -= cb[c].y; v[c][6] -= cb[c].z; v[c][7] -= cb[c].w;
                }
            }
            unsigned char* __restrict__ out = p.packed + (uint64_t)k * p.packed_stride;
            FastCtx cx;
            cx.norms = reinterpret_cast<float*>(out + p.norms_off);
            cx.signs = reinterpret_cast<uint32_t*>(out + p.signs_off);
            cx.levels = reinterpret_cast<uint32_t*>(out + p.levels_off);
            cx.lane = lane;
            cx.wave = wave;
            cx.lane_off = lane_off;
            cx.worker = p.worker0 + k;
            cx.round = p.round;
            cx.key0 = p.key0;
            cx.key1 = p.key1;
            cx.smax = p.smax;
            process_tile<M, LOG2N, true>(cx, v, t, sm[k & 1u], acc);
            if (k + 1 < r.K) {
#pragma unroll
                for (int c = 0; c < CH; ++c) { a[c] = na[c]; b[c] = nbuf[c]; }
            }
        }
    } else {                                              // the ragged last tile
        for (uint32_t k = 0; k < r.K; ++k)
            guarded_tile<M, CH, QESGD_NORM_L2, false, true>(p, k, t, sm[k & 1u], acc);
    }

    const float fk = (float)r.K;
    if (t < p.full_tiles) {
        // z moves from the lane-of-8 layout of the codes to one float4 of each 256-coordinate half
        // per lane, so that every 128-bit access of a wave covers a contiguous KiB, through 2 KiB
        // of LDS private to the wave (same wave on both sides: LDS keeps program order).
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            float z[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) z[e] = (r.rcpK != 0.0f) ? acc[c][e] * r.rcpK : acc[c][e] / fk;
            stage[wave][2 * lane] = make_float4(z[0], z[1], z[2], z[3]);
            stage[wave][2 * lane + 1] = make_float4(z[4], z[5], z[6], z[7]);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const float4 za = stage[wave][lane];
            const float4 zb = stage[wave][64 + lane];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();                       // the next chunk overwrites the staging area
            const uint64_t ia = (uint64_t)t * TILE + wave * (uint32_t)(CH * kChunk) + (uint32_t)c * kChunk + lane * 4u;
            const uint64_t ib = ia + 256u;
            const float4 wa = *reinterpret_cast<const float4*>(r.w + ia);
            const float4 wb = *reinterpret_cast<const float4*>(r.w + ib);
            if (r.zbar) {
                *reinterpret_cast<float4*>(r.zbar + ia) = za;
                *reinterpret_cast<float4*>(r.zbar + ib) = zb;
            }
            *reinterpret_cast<float4*>(r.u + ia) = make_float4(wa.x + za.x, wa.y + za.y, wa.z + za.z, wa.w + za.w);
            *reinterpret_cast<float4*>(r.u + ib) = make_float4(wb.x + zb.x, wb.y + zb.y, wb.z + zb.z, wb.w + zb.w);
            if (r.zsum) {
                const float4 sa = *reinterpret_cast<const float4*>(r.zsum + ia);
                const float4 sb = *reinterpret_cast<const float4*>(r.zsum + ib);
                *reinterpret_cast<float4*>(r.zsum + ia) = make_float4(sa.x + za.x, sa.y + za.y, sa.z + za.z, sa.w + za.w);
                *reinterpret_cast<float4*>(r.zsum + ib) = make_float4(sb.x + zb.x, sb.y + zb.y, sb.z + zb.z, sb.w + zb.w);
            }
        }
        return;
    }
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        // the ragged tile, lane by lane (power-of-two buckets: slot == coordinate)
        const uint64_t i = (uint64_t)t * TILE + lane_off + (uint32_t)c * kChunk;
        if (i >= p.d) continue;
        const uint64_t rem = p.d - i;
        const uint32_t nvalid = rem < 8 ? (uint32_t)rem : 8u;
        float z[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = (r.rcpK != 0.0f) ? acc[c][e] * r.rcpK : acc[c][e] / fk;
        if (r.zbar) store8(r.zbar, i, nvalid, z);
        float w8[8], u8[8];
        load8(r.w, i, nvalid, w8);
#pragma unroll
        for (int e = 0; e < 8; ++e) u8[e] = w8[e] + z[e];
        store8(r.u, i, nvalid, u8);
        if (r.zsum) {
            float s8[8];
            load8(r.zsum, i, nvalid, s8);
#pragma unroll
            for (int e = 0; e < 8; ++e) s8[e] = s8[e] + z[e];
            store8(r.zsum, i, nvalid, s8);
        }
    }
}

template <int M, int LOG2N>
void launch_one(const RParams& r, uint32_t blocks, hipStream_t st) {
    if (r.q.center)
        hipLaunchKernelGGL((k_round_fused<M, LOG2N, true>), dim3(blocks), dim3(Geo<LOG2N>::NW * 64), 0, st, r);
    else
        hipLaunchKernelGGL((k_round_fused<M, LOG2N, false>), dim3(blocks), dim3(Geo<LOG2N>::NW * 64), 0, st, r);
}

template <int M>
void launch_n(const RParams& r, uint32_t blocks, hipStream_t st) {
    switch (r.q.log2N) {
        case 5: launch_one<M, 5>(r, blocks, st); break;
        case 6: launch_one<M, 6>(r, blocks, st); break;
        case 7: launch_one<M, 7>(r, blocks, st); break;
        case 8: launch_one<M, 8>(r, blocks, st); break;
        case 9: launch_one<M, 9>(r, blocks, st); break;
        case 10: launch_one<M, 10>(r, blocks, st); break;
        case 11: launch_one<M, 11>(r, blocks, st); break;
        case 12: launch_one<M, 12>(r, blocks, st); break;
        case 13: launch_one<M, 13>(r, blocks, st); break;
        case 14: launch_one<M, 14>(r, blocks, st); break;
        default: launch_one<M, 15>(r, blocks, st); break;
    }
}

}  // namespace

bool round_fused_covers(const Shape& sh, uint32_t norm_kind) {
    return norm_kind == QESGD_NORM_L2 && sh.N == sh.B && sh.log2N >= 5 && sh.N <= kMaxSinglePassBucket &&
           32u % sh.m == 0u;
}

int launch_round_fused(const Shape& sh, const QuantizeArgs& a, const AggregateArgs& g) {
    RParams r{};
    QParams& p = r.q;
    p.x = a.x;
    p.center = a.center;
    p.packed = a.packed;
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
    uint32_t ch, nwaves;
    fast_geometry(sh.N, &ch, &nwaves);
    const uint64_t tile = (uint64_t)nwaves * ch * kChunk;
    const uint64_t tiles = (sh.nb * sh.N + tile - 1) / tile;
    if (tiles >= (1ull << 31)) return QESGD_ERR_DIM;
    p.full_tiles = (uint32_t)(sh.d / tile);
    p.tail_tiles = (uint32_t)(tiles - p.full_tiles);
    r.w = g.w_snap;
    r.zbar = g.zbar_out;
    r.u = g.u_out;
    r.zsum = g.zsum;
    r.K = a.K;
    r.rcpK = ((a.K & (a.K - 1)) == 0) ? 1.0f / (float)a.K : 0.0f;
    switch (sh.m) {
        case 1: launch_n<1>(r, (uint32_t)tiles, a.stream); break;
        case 2: launch_n<2>(r, (uint32_t)tiles, a.stream); break;
        case 4: launch_n<4>(r, (uint32_t)tiles, a.stream); break;
        case 8: launch_n<8>(r, (uint32_t)tiles, a.stream); break;
        default: launch_n<16>(r, (uint32_t)tiles, a.stream); break;
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_last_hip_error((int)e);
        return QESGD_ERR_HIP;
    }
    return QESGD_OK;
}

}  // namespace qesgd
