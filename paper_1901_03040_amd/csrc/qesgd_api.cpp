// Host side of the C ABI: shape arithmetic, argument validation, dispatch.
// Every check here runs before the first HIP call of an entry point.
#include "qesgd_internal.h"

namespace qesgd {

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(int e) { g_last_hip_error = e; }

static int level_bits(uint32_t s) {
    switch (s) {
        case 2u: return 1;
        case 4u: return 2;
        case 8u: return 3;
        case 16u: return 4;
        case 32u: return 5;
        case 64u: return 6;
        case 128u: return 7;
        case 256u: return 8;
        case 65536u: return 16;
        default: return -1;
    }
}

static uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

int make_shape(uint64_t d, uint32_t s, uint64_t bucket, Shape* out) {
    if (d == 0 || d >= (1ull << 40)) return QESGD_ERR_DIM;
    const int m = level_bits(s);
    if (m < 0) return QESGD_ERR_LEVELS;
    if (bucket == 0) return QESGD_ERR_BUCKET;
    const uint64_t B = bucket < d ? bucket : d;
    if (B < d && (B % 32) != 0) return QESGD_ERR_BUCKET;
    Shape sh{};
    sh.d = d;
    sh.s = s;
    sh.m = (uint32_t)m;
    sh.B = B;
    sh.nb = (d + B - 1) / B;
    uint64_t N = 8;                       // padding with +0 beyond the bucket does not change the tree sum
    uint32_t lg = 3;
    while (N < B) { N <<= 1; ++lg; }
    sh.N = N;
    sh.log2N = lg;
    qesgd_layout& L = sh.lay;
    L.n_buckets = sh.nb;
    L.level_bits = (uint32_t)m;
    L.reserved = 0;
    L.sign_words = (d + 31) / 32;
    L.level_words = (d * (uint64_t)m + 31) / 32;
    L.norms_off = 0;
    L.signs_off = round_up(4 * L.n_buckets, 256);
    L.levels_off = L.signs_off + round_up(4 * L.sign_words, 256);
    L.bytes_per_worker = L.levels_off + round_up(4 * L.level_words, 256);
    L.payload_bytes = 4 * (L.n_buckets + L.sign_words + L.level_words);
    *out = sh;
    return QESGD_OK;
}

static bool aligned(const void* p, uintptr_t a) { return ((uintptr_t)p % a) == 0; }

static size_t workspace_floats(const Shape& sh, uint32_t K) {
    if (sh.N <= kMaxSinglePassBucket) return 0;
    return (size_t)K * sh.nb * (sh.N / kPartialTile);
}

// Validates a quantise call and fills the shape and the launch arguments; launches nothing.
static int quantize_check(const float* x, uint64_t x_stride, const float* center, uint64_t d,
                          uint32_t s, uint64_t bucket, uint32_t norm_kind, uint64_t seed,
                          uint32_t round, uint32_t worker0, uint32_t K, void* packed,
                          uint64_t packed_stride, void* workspace, size_t workspace_bytes,
                          void* stream, bool static_workspace, Shape* shape, QuantizeArgs* args) {
    if (!x || !packed) return QESGD_ERR_NULL;
    Shape& sh = *shape;
    const int rc = make_shape(d, s, bucket, &sh);
    if (rc != QESGD_OK) return rc;
    if (K == 0 || K > QESGD_MAX_WORKERS) return QESGD_ERR_WORKERS;
    if (norm_kind != QESGD_NORM_L2 && norm_kind != QESGD_NORM_MAX) return QESGD_ERR_NORM_KIND;
    if (!aligned(x, 16) || !aligned(center, 16) || !aligned(packed, 256) || !aligned(workspace, 16))
        return QESGD_ERR_ALIGN;
    if (K > 1) {
        if (x_stride < d || (x_stride % 4) != 0) return QESGD_ERR_STRIDE;
        if (packed_stride < sh.lay.bytes_per_worker || (packed_stride % 256) != 0) return QESGD_ERR_STRIDE;
    }
    const size_t need = workspace_floats(sh, K) * sizeof(float);
    if (static_workspace) {
        if (need > QESGD_NOALLOC_SCRATCH_BYTES) return QESGD_ERR_SCRATCH;
        if (need > 0) {
            float* ptr = nullptr;
            const int src = static_scratch(&ptr);
            if (src != QESGD_OK) return src;
            workspace = ptr;
        }
    } else if (need > 0 && (!workspace || workspace_bytes < need)) {
        return QESGD_ERR_WORKSPACE;
    }
    QuantizeArgs& a = *args;
    a = QuantizeArgs{};
    a.x = x;
    a.x_stride = x_stride;
    a.center = center;
    a.norm_kind = norm_kind;
    a.seed = seed;
    a.round = round;
    a.worker0 = worker0;
    a.K = K;
    a.packed = (unsigned char*)packed;
    a.packed_stride = packed_stride;
    a.workspace = (float*)workspace;
    a.stream = (hipStream_t)stream;
    return QESGD_OK;
}

static int quantize_common(const float* x, uint64_t x_stride, const float* center, uint64_t d,
                           uint32_t s, uint64_t bucket, uint32_t norm_kind, uint64_t seed,
                           uint32_t round, uint32_t worker0, uint32_t K, void* packed,
                           uint64_t packed_stride, void* workspace, size_t workspace_bytes,
                           void* stream, bool static_workspace = false) {
    Shape sh;
    QuantizeArgs a;
    const int rc = quantize_check(x, x_stride, center, d, s, bucket, norm_kind, seed, round, worker0, K, packed,
                                  packed_stride, workspace, workspace_bytes, stream, static_workspace, &sh, &a);
    return rc != QESGD_OK ? rc : launch_quantize(sh, a);
}

static int aggregate_check(const void* packed, uint64_t packed_stride, uint32_t K, uint64_t d,
                           uint32_t s, uint64_t bucket, const float* w, float* zbar, float* u,
                           float* zsum, bool fused, void* stream, Shape* shape, AggregateArgs* args) {
    if (!packed) return QESGD_ERR_NULL;
    if (fused ? (!w || !u) : !zbar) return QESGD_ERR_NULL;
    Shape& sh = *shape;
    const int rc = make_shape(d, s, bucket, &sh);
    if (rc != QESGD_OK) return rc;
    if (K == 0 || K > QESGD_MAX_WORKERS) return QESGD_ERR_WORKERS;
    if (!aligned(packed, 256) || !aligned(w, 16) || !aligned(zbar, 16) || !aligned(u, 16) || !aligned(zsum, 16))
        return QESGD_ERR_ALIGN;
    if (K > 1 && (packed_stride < sh.lay.bytes_per_worker || (packed_stride % 256) != 0)) return QESGD_ERR_STRIDE;
    AggregateArgs& a = *args;
    a = AggregateArgs{};
    a.packed = (const unsigned char*)packed;
    a.packed_stride = packed_stride;
    a.K = K;
    a.w_snap = w;
    a.zbar_out = zbar;
    a.u_out = u;
    a.zsum = zsum;
    a.stream = (hipStream_t)stream;
    return QESGD_OK;
}

static int aggregate_common(const void* packed, uint64_t packed_stride, uint32_t K, uint64_t d,
                            uint32_t s, uint64_t bucket, const float* w, float* zbar, float* u,
                            float* zsum, bool fused, void* stream) {
    Shape sh;
    AggregateArgs a;
    const int rc = aggregate_check(packed, packed_stride, K, d, s, bucket, w, zbar, u, zsum, fused, stream, &sh, &a);
    return rc != QESGD_OK ? rc : launch_aggregate(sh, a);
}

}  // namespace qesgd

using namespace qesgd;

extern "C" {

int qesgd_layout_query(uint64_t d, uint32_t s, uint64_t bucket, qesgd_layout* out) {
    if (!out) return QESGD_ERR_NULL;
    Shape sh;
    const int rc = make_shape(d, s, bucket, &sh);
    if (rc != QESGD_OK) return rc;
    *out = sh.lay;
    return QESGD_OK;
}

size_t qesgd_workspace_bytes(uint64_t d, uint32_t s, uint64_t bucket, uint32_t K) {
    Shape sh;
    if (make_shape(d, s, bucket, &sh) != QESGD_OK || K == 0 || K > QESGD_MAX_WORKERS) return 0;
    return workspace_floats(sh, K) * sizeof(float);
}

int qesgd_quantize_pack(const float* x, const float* center, uint64_t d, uint32_t s, uint64_t bucket,
                        uint32_t norm_kind, uint64_t seed, uint32_t round, uint32_t worker,
                        void* packed, void* workspace, size_t workspace_bytes, void* stream) {
    return quantize_common(x, 0, center, d, s, bucket, norm_kind, seed, round, worker, 1, packed, 0,
                           workspace, workspace_bytes, stream);
}

int qesgd_quantize_pack_batched(const float* x_slab, uint64_t x_stride, const float* center,
                                uint64_t d, uint32_t s, uint64_t bucket, uint32_t norm_kind,
                                uint64_t seed, uint32_t round, uint32_t K, void* packed_slab,
                                uint64_t packed_stride, void* workspace, size_t workspace_bytes,
                                void* stream) {
    return quantize_common(x_slab, x_stride, center, d, s, bucket, norm_kind, seed, round, 0, K,
                           packed_slab, packed_stride, workspace, workspace_bytes, stream);
}

int qesgd_quantize_pack_batched_noalloc(const float* x_slab, uint64_t x_stride, const float* center,
                                        uint64_t d, uint32_t s, uint64_t bucket, uint32_t norm_kind,
                                        uint64_t seed, uint32_t round, uint32_t K, void* packed_slab,
                                        uint64_t packed_stride, void* stream) {
    return quantize_common(x_slab, x_stride, center, d, s, bucket, norm_kind, seed, round, 0, K,
                           packed_slab, packed_stride, nullptr, 0, stream, true);
}

int qesgd_unpack_aggregate(const void* packed_slab, uint64_t packed_stride, uint32_t K, uint64_t d,
                           uint32_t s, uint64_t bucket, float* zbar, void* stream) {
    return aggregate_common(packed_slab, packed_stride, K, d, s, bucket, nullptr, zbar, nullptr,
                            nullptr, false, stream);
}

int qesgd_apply_update(const float* w_snap, const float* zbar, float* u_out, float* zsum_inout,
                       uint64_t d, void* stream) {
    if (!w_snap || !zbar || !u_out) return QESGD_ERR_NULL;
    if (d == 0 || d >= (1ull << 40)) return QESGD_ERR_DIM;
    if (!aligned(w_snap, 16) || !aligned(zbar, 16) || !aligned(u_out, 16) || !aligned(zsum_inout, 16))
        return QESGD_ERR_ALIGN;
    return launch_apply_update(w_snap, zbar, u_out, zsum_inout, d, (hipStream_t)stream);
}

int qesgd_unpack_aggregate_update(const void* packed_slab, uint64_t packed_stride, uint32_t K,
                                  uint64_t d, uint32_t s, uint64_t bucket, const float* w_snap,
                                  float* zbar_out, float* u_out, float* zsum_inout, void* stream) {
    return aggregate_common(packed_slab, packed_stride, K, d, s, bucket, w_snap, zbar_out, u_out,
                            zsum_inout, true, stream);
}

int qesgd_round(const float* x_slab, uint64_t x_stride, const float* center, uint64_t d, uint32_t s,
                uint64_t bucket, uint32_t norm_kind, uint64_t seed, uint32_t round, uint32_t K,
                void* packed_slab, uint64_t packed_stride, void* workspace, size_t workspace_bytes,
                const float* w_snap, float* zbar_out, float* u_out, float* zsum_inout, void* stream) {
    Shape sh, sh2;
    QuantizeArgs q;
    AggregateArgs g;
    int rc = quantize_check(x_slab, x_stride, center, d, s, bucket, norm_kind, seed, round, 0, K, packed_slab,
                            packed_stride, workspace, workspace_bytes, stream, false, &sh, &q);
    if (rc != QESGD_OK) return rc;
    rc = aggregate_check(packed_slab, packed_stride, K, d, s, bucket, w_snap, zbar_out, u_out, zsum_inout, true,
                         stream, &sh2, &g);
    if (rc != QESGD_OK) return rc;
    if (round_fused_covers(sh, norm_kind)) return launch_round_fused(sh, q, g);
    rc = launch_quantize(sh, q);
    return rc != QESGD_OK ? rc : launch_aggregate(sh, g);
}

static bool fixed_bits_ok(uint32_t b) { return b == 2 || b == 4 || b == 8 || b == 16; }

int qesgd_quantize_fixed(const float* x, const float* center, uint64_t d, float delta, uint32_t b,
                         uint64_t seed, uint32_t round, uint32_t worker, void* codes, void* stream) {
    if (!x || !codes) return QESGD_ERR_NULL;
    if (d == 0 || d >= (1ull << 40)) return QESGD_ERR_DIM;
    if (!fixed_bits_ok(b)) return QESGD_ERR_BITS;
    if (!(delta > 0.0f) || !(delta < __builtin_inff())) return QESGD_ERR_DELTA;
    if (!aligned(x, 16) || !aligned(center, 16) || !aligned(codes, 16)) return QESGD_ERR_ALIGN;
    return launch_quantize_fixed(x, center, d, delta, b, seed, round, worker, codes, (hipStream_t)stream);
}

int qesgd_dequantize_fixed_update(const void* codes, uint64_t d, float delta, uint32_t b,
                                  const float* w_snap, float* z_out, float* u_out, float* zsum_inout,
                                  void* stream) {
    if (!codes || (!z_out && !u_out && !zsum_inout)) return QESGD_ERR_NULL;
    if ((u_out != nullptr) != (w_snap != nullptr)) return QESGD_ERR_NULL;
    if (d == 0 || d >= (1ull << 40)) return QESGD_ERR_DIM;
    if (!fixed_bits_ok(b)) return QESGD_ERR_BITS;
    if (!(delta > 0.0f) || !(delta < __builtin_inff())) return QESGD_ERR_DELTA;
    if (!aligned(codes, 16) || !aligned(w_snap, 16) || !aligned(z_out, 16) || !aligned(u_out, 16) ||
        !aligned(zsum_inout, 16))
        return QESGD_ERR_ALIGN;
    return launch_dequantize_fixed_update(codes, d, delta, b, w_snap, z_out, u_out, zsum_inout, (hipStream_t)stream);
}

int qesgd_epoch_commit(float* w_inout, float* zsum_inout, uint32_t rounds, uint64_t d, void* stream) {
    if (!w_inout || !zsum_inout) return QESGD_ERR_NULL;
    if (d == 0 || d >= (1ull << 40)) return QESGD_ERR_DIM;
    if (rounds == 0) return QESGD_ERR_ROUNDS;
    if (!aligned(w_inout, 16) || !aligned(zsum_inout, 16)) return QESGD_ERR_ALIGN;
    return launch_epoch_commit(w_inout, zsum_inout, rounds, d, (hipStream_t)stream);
}

const char* qesgd_strerror(int code) {
    switch (code) {
        case QESGD_OK: return "ok";
        case QESGD_ERR_NULL: return "a required pointer is NULL";
        case QESGD_ERR_DIM: return "d must be in [1, 2^40)";
        case QESGD_ERR_LEVELS: return "s must be one of 2, 4, 8, 16, 32, 64, 128, 256, 65536";
        case QESGD_ERR_BUCKET: return "bucket must be > 0 and, when smaller than d, a multiple of 32";
        case QESGD_ERR_WORKERS: return "K must be in [1, 64]";
        case QESGD_ERR_NORM_KIND: return "norm_kind must be 0 (L2) or 1 (max)";
        case QESGD_ERR_ALIGN: return "pointer alignment: 16 bytes for vectors, 256 for packed blocks";
        case QESGD_ERR_STRIDE: return "slab stride too small or not a multiple of 16 bytes (packed: 256)";
        case QESGD_ERR_WORKSPACE: return "workspace missing or smaller than qesgd_workspace_bytes()";
        case QESGD_ERR_HIP: return "kernel launch failed (see qesgd_last_hip_error)";
        case QESGD_ERR_BITS: return "b must be one of 2, 4, 8, 16";
        case QESGD_ERR_DELTA: return "delta must be a positive finite number";
        case QESGD_ERR_ROUNDS: return "rounds must be at least 1";
        case QESGD_ERR_SCRATCH: return "shape needs more scratch than the no-allocation entry point holds (4 MiB)";
        default: return "unknown error code";
    }
}

int qesgd_last_hip_error(void) { return g_last_hip_error; }

uint32_t qesgd_abi_version(void) { return QESGD_ABI_VERSION; }

}  // extern "C"
