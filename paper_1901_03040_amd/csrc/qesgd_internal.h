// Internal declarations shared by the translation units of libqesgd (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qesgd.h"

namespace qesgd {

// Coordinates handled by one lane per chunk, lanes per wavefront, and the
// resulting wave chunk: 64 lanes x 8 consecutive coordinates.
constexpr uint32_t kLaneElems = 8;
constexpr uint32_t kWaveSize = 64;
constexpr uint32_t kChunk = kLaneElems * kWaveSize;   // 512

// Largest zero-padded bucket whose scale is found in the same pass that
// quantises it (16 waves x 4 chunks x 512 coordinates held in registers).
constexpr uint64_t kMaxSinglePassBucket = 32768;
// Tile of the partial-sum pass used for larger buckets.
constexpr uint64_t kPartialTile = 4096;
// Input bytes that the two-pass path lets the first pass read before the second pass re-reads
// them: well inside the 256 MB memory-side cache, which also has to take the packed output.
constexpr uint64_t kCacheBudgetBytes = 160ull << 20;
// Floats of the per-GPU static scratch behind qesgd_quantize_pack_batched_noalloc (4 MiB): one
// partial sum per 4096 padded coordinates, i.e. K * n_buckets * padded_bucket <= 2^32.
constexpr size_t kStaticScratchFloats = QESGD_NOALLOC_SCRATCH_BYTES / sizeof(float);

struct Shape {
    uint64_t d;
    uint32_t s;
    uint32_t m;          // level bits
    uint64_t B;          // effective bucket = min(bucket, d)
    uint64_t nb;         // buckets
    uint64_t N;          // B zero-padded to a power of two, at least 8
    uint32_t log2N;
    qesgd_layout lay;
};

// Validates (d, s, bucket) and fills the shape; returns QESGD_OK or an error.
int make_shape(uint64_t d, uint32_t s, uint64_t bucket, Shape* out);

struct QuantizeArgs {
    const float* x;
    uint64_t x_stride;       // floats between workers
    const float* center;     // nullable
    uint32_t norm_kind;
    uint64_t seed;
    uint32_t round;
    uint32_t worker0;        // worker id of slab row 0
    uint32_t K;              // rows
    unsigned char* packed;
    uint64_t packed_stride;  // bytes between workers
    float* workspace;        // two-pass path only
    hipStream_t stream;
};

struct AggregateArgs {
    const unsigned char* packed;
    uint64_t packed_stride;
    uint32_t K;
    const float* w_snap;     // nullable: no update
    float* zbar_out;         // nullable
    float* u_out;            // nullable iff w_snap is
    float* zsum;             // nullable
    hipStream_t stream;
};

int launch_quantize(const Shape& sh, const QuantizeArgs& a);
// Device address of the current GPU's static scratch (kStaticScratchFloats floats).
int static_scratch(float** out);
int launch_aggregate(const Shape& sh, const AggregateArgs& a);
// One launch for a whole round (quantise K workers, sum, update) where the shape allows it:
// power-of-two bucket of 32..32768 coordinates, L2 scale, level width dividing 32.
bool round_fused_covers(const Shape& sh, uint32_t norm_kind);
int launch_round_fused(const Shape& sh, const QuantizeArgs& a, const AggregateArgs& g);
int launch_apply_update(const float* w, const float* zbar, float* u, float* zsum, uint64_t d,
                        hipStream_t stream);

int launch_quantize_fixed(const float* x, const float* center, uint64_t d, float delta, uint32_t b,
                          uint64_t seed, uint32_t round, uint32_t worker, void* codes, hipStream_t stream);
int launch_dequantize_fixed_update(const void* codes, uint64_t d, float delta, uint32_t b, const float* w,
                                   float* z, float* u, float* zsum, hipStream_t stream);
int launch_epoch_commit(float* w, float* zsum, uint32_t rounds, uint64_t d, hipStream_t stream);

void set_last_hip_error(int e);

}  // namespace qesgd
