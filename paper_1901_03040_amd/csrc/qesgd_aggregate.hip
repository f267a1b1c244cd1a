// Server side of a QESGD round on gfx950: unpack + dequantise the K workers'
// codes, average them in worker order (Alg. 3, server task), and apply
// u = w_t + z with the running sum of z (Alg. 2; last step of Alg. 2 / Alg. 3).
//
// A lane owns 8 consecutive coordinates: per worker it reads one sign byte, m
// level bytes and the bucket scale, per vector two 128-bit words.  All the fp32
// traffic (w, zsum in; zbar, u, zsum out) is touched exactly once.
#include "qesgd_aggregate_device.h"

namespace qesgd {
namespace {

// A wave owns 512 consecutive coordinates.  The codes are read with a lane owning 8
// consecutive coordinates (one sign byte, 8*M level bits per worker); the fp32 vectors are
// read and written with a lane owning one float4 of each 256-coordinate half, so that every
// 128-bit access of a wave covers a contiguous KiB (a 32-byte lane stride would split every
// store into half-filled requests).  z crosses from one layout to the other through 2 KiB of
// LDS private to the wave.  UPDATE: w, u present.  When the bucket size is a multiple of 512
// the whole wave shares a bucket: lane k divides worker k's scale once and the loop reads it
// back as a scalar.
// Waves per workgroup; the waves share nothing.  Two measured 1-2% faster than four or eight at
// d = 11 M .. 138 M (0.532 against 0.539 ms at d = 138 M, K = 8), one the same as two.
constexpr uint32_t kAggWaves = 2;
template <int M, bool UPDATE, bool ZSUM, bool ZBAR>
__global__ void __launch_bounds__(kAggWaves * 64) k_unpack_aggregate_update(const AParams p) {
    __shared__ float4 stage[kAggWaves][128];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint64_t wave_base = ((uint64_t)blockIdx.x * kAggWaves + wave) * kChunk;
    if (wave_base >= p.d) return;
    if (wave_base + kChunk > p.d) {                       // ragged last wave
        aggregate_lane_guarded<M>(p, wave_base + lane * kLaneElems);
        return;
    }
    const uint64_t i = wave_base + lane * kLaneElems;     // code layout: 8 consecutive coordinates
    const uint64_t ia = wave_base + lane * 4u;            // vector layout: float4 #lane of each half
    const uint64_t ib = ia + 256u;

    float4 wa, wb, sa, sb;
    if (UPDATE) {
        wa = *reinterpret_cast<const float4*>(p.w + ia);
        wb = *reinterpret_cast<const float4*>(p.w + ib);
    }
    if (ZSUM) {
        sa = *reinterpret_cast<const float4*>(p.zsum + ia);
        sb = *reinterpret_cast<const float4*>(p.zsum + ib);
    }

    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0f;

    if (p.wave_uniform_bucket) {
        const uint64_t b = bucket_of(wave_base, p);
        float my_step = 0.0f;
        if (lane < p.K) {
            const float norm = reinterpret_cast<const float*>(p.packed + (uint64_t)lane * p.packed_stride + p.norms_off)[b];
            my_step = norm / p.smax;
        }
        uint32_t k = 0;
        for (; k + 4 <= p.K; k += 4) {                    // four workers' codes in flight at a time
            uint32_t sbyte[4], w[4][4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const unsigned char* __restrict__ blk = p.packed + (uint64_t)(k + j) * p.packed_stride;
                sbyte[j] = (blk + p.signs_off)[i >> 3];
                load_level_bits<M>(reinterpret_cast<const uint32_t*>(blk + p.levels_off), i, 8u, p.level_words, w[j]);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float step = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_step), k + j));
                accumulate8<M>(acc, sbyte[j], w[j], step);
            }
        }
        for (; k < p.K; ++k) {
            const unsigned char* __restrict__ blk = p.packed + (uint64_t)k * p.packed_stride;
            const uint32_t sbyte = (blk + p.signs_off)[i >> 3];
            uint32_t w[4];
            load_level_bits<M>(reinterpret_cast<const uint32_t*>(blk + p.levels_off), i, 8u, p.level_words, w);
            const float step = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_step), k));
            accumulate8<M>(acc, sbyte, w, step);
        }
    } else if (p.wave_two_buckets) {
        // Buckets of at least 512 coordinates that do not line up with the waves: a wave touches at
        // most two of them.  Lane k divides worker k's scale of the first, lane 32 + k of the second.
        const uint64_t b0 = bucket_of(wave_base, p);
        const uint64_t boundary = (b0 + 1) * p.B;           // first coordinate of the second bucket
        float my_step = 0.0f;
        const uint32_t kk = lane & 31u;
        const uint64_t bb = b0 + (lane >> 5);
        if (kk < p.K && bb * p.B < p.d) {
            const float norm = reinterpret_cast<const float*>(p.packed + (uint64_t)kk * p.packed_stride + p.norms_off)[bb];
            my_step = norm / p.smax;
        }
        const bool second = i >= boundary;
        uint32_t k = 0;
        for (; k + 4 <= p.K; k += 4) {                    // four workers' codes in flight at a time
            uint32_t sbyte[4], w[4][4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const unsigned char* __restrict__ blk = p.packed + (uint64_t)(k + j) * p.packed_stride;
                sbyte[j] = (blk + p.signs_off)[i >> 3];
                load_level_bits<M>(reinterpret_cast<const uint32_t*>(blk + p.levels_off), i, 8u, p.level_words, w[j]);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float s0 = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_step), k + j));
                const float s1 = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_step), 32u + k + j));
                accumulate8<M>(acc, sbyte[j], w[j], second ? s1 : s0);
            }
        }
        for (; k < p.K; ++k) {
            const unsigned char* __restrict__ blk = p.packed + (uint64_t)k * p.packed_stride;
            const uint32_t sbyte = (blk + p.signs_off)[i >> 3];
            uint32_t w[4];
            load_level_bits<M>(reinterpret_cast<const uint32_t*>(blk + p.levels_off), i, 8u, p.level_words, w);
            const float s0 = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_step), k));
            const float s1 = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_step), 32u + k));
            accumulate8<M>(acc, sbyte, w, second ? s1 : s0);
        }
    } else {
        const uint64_t b = bucket_of(i, p);
#pragma unroll 4
        for (uint32_t k = 0; k < p.K; ++k) {
            const unsigned char* __restrict__ blk = p.packed + (uint64_t)k * p.packed_stride;
            const float norm = reinterpret_cast<const float*>(blk + p.norms_off)[b];
            const uint32_t sbyte = (blk + p.signs_off)[i >> 3];
            uint32_t w[4];
            load_level_bits<M>(reinterpret_cast<const uint32_t*>(blk + p.levels_off), i, 8u, p.level_words, w);
            accumulate8<M>(acc, sbyte, w, norm / p.smax);
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

    // lane-of-8 layout -> float4-per-half layout (same wave on both sides: LDS keeps program order)
    stage[wave][2 * lane] = make_float4(z[0], z[1], z[2], z[3]);
    stage[wave][2 * lane + 1] = make_float4(z[4], z[5], z[6], z[7]);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const float4 za = stage[wave][lane];
    const float4 zb = stage[wave][64 + lane];

    if (ZBAR) {
        *reinterpret_cast<float4*>(p.zbar + ia) = za;
        *reinterpret_cast<float4*>(p.zbar + ib) = zb;
    }
    if (UPDATE) {
        *reinterpret_cast<float4*>(p.u + ia) = make_float4(wa.x + za.x, wa.y + za.y, wa.z + za.z, wa.w + za.w);
        *reinterpret_cast<float4*>(p.u + ib) = make_float4(wb.x + zb.x, wb.y + zb.y, wb.z + zb.z, wb.w + zb.w);
    }
    if (ZSUM) {
        *reinterpret_cast<float4*>(p.zsum + ia) = make_float4(sa.x + za.x, sa.y + za.y, sa.z + za.z, sa.w + za.w);
        *reinterpret_cast<float4*>(p.zsum + ib) = make_float4(sb.x + zb.x, sb.y + zb.y, sb.z + zb.z, sb.w + zb.w);
    }
}

// u = w + z, zsum += z: one float4 per lane so that every access of a wave is a contiguous KiB.
__global__ void __launch_bounds__(256) k_apply_update(const float* w, const float* zbar,
                                                      float* u, float* zsum, uint64_t d) {
    const uint64_t i = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4u;
    if (i >= d) return;
    if (i + 4 <= d) {
        const float4 z = *reinterpret_cast<const float4*>(zbar + i);
        const float4 a = *reinterpret_cast<const float4*>(w + i);
        if (zsum) {
            const float4 s = *reinterpret_cast<const float4*>(zsum + i);
            *reinterpret_cast<float4*>(zsum + i) = make_float4(s.x + z.x, s.y + z.y, s.z + z.z, s.w + z.w);
        }
        *reinterpret_cast<float4*>(u + i) = make_float4(a.x + z.x, a.y + z.y, a.z + z.z, a.w + z.w);
    } else {
        for (uint64_t j = i; j < d; ++j) {
            const float z = zbar[j];
            const float a = w[j];
            if (zsum) zsum[j] = zsum[j] + z;
            u[j] = a + z;
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

    p.wave_uniform_bucket = (sh.B % kChunk == 0 || sh.nb == 1) ? 1u : 0u;
    p.wave_two_buckets = (!p.wave_uniform_bucket && sh.B >= kChunk && a.K <= 32u) ? 1u : 0u;

    const uint64_t lanes = (sh.d + kLaneElems - 1) / kLaneElems;
    const uint64_t blocks = (lanes + kAggWaves * 64 - 1) / (kAggWaves * 64);
    if (blocks >= (1ull << 31)) return QESGD_ERR_DIM;
    const dim3 grid((uint32_t)blocks), block(kAggWaves * 64);
    const bool upd = a.w_snap != nullptr, zs = a.zsum != nullptr, zb = a.zbar_out != nullptr;
#define QESGD_LAUNCH_AGG(MM)                                                                              \
    do {                                                                                                 \
        if (upd && zs && zb) hipLaunchKernelGGL((k_unpack_aggregate_update<MM, true, true, true>), grid, block, 0, a.stream, p);        \
        else if (upd && zs) hipLaunchKernelGGL((k_unpack_aggregate_update<MM, true, true, false>), grid, block, 0, a.stream, p);        \
        else if (upd && zb) hipLaunchKernelGGL((k_unpack_aggregate_update<MM, true, false, true>), grid, block, 0, a.stream, p);        \
        else if (upd) hipLaunchKernelGGL((k_unpack_aggregate_update<MM, true, false, false>), grid, block, 0, a.stream, p);             \
        else hipLaunchKernelGGL((k_unpack_aggregate_update<MM, false, false, true>), grid, block, 0, a.stream, p);                      \
    } while (0)
    switch (sh.m) {
        case 1: QESGD_LAUNCH_AGG(1); break;
        case 2: QESGD_LAUNCH_AGG(2); break;
        case 3: QESGD_LAUNCH_AGG(3); break;
        case 4: QESGD_LAUNCH_AGG(4); break;
        case 5: QESGD_LAUNCH_AGG(5); break;
        case 6: QESGD_LAUNCH_AGG(6); break;
        case 7: QESGD_LAUNCH_AGG(7); break;
        case 8: QESGD_LAUNCH_AGG(8); break;
        default: QESGD_LAUNCH_AGG(16); break;
    }
#undef QESGD_LAUNCH_AGG
    return check_launch();
}

int launch_apply_update(const float* w, const float* zbar, float* u, float* zsum, uint64_t d,
                        hipStream_t stream) {
    const uint64_t lanes = (d + 3) / 4;
    const uint64_t blocks = (lanes + 255) / 256;
    if (blocks >= (1ull << 31)) return QESGD_ERR_DIM;
    hipLaunchKernelGGL(k_apply_update, dim3((uint32_t)blocks), dim3(256), 0, stream, w, zbar, u, zsum, d);
    return check_launch();
}

}  // namespace qesgd
