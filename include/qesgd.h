/* qesgd.h -- C ABI of the MI355X (gfx950) QESGD hot path.
 *
 * One synchronous-SGD round of Quantized Epoch-SGD, compress-on-push form:
 * every worker k holds the deviation z_hat_k of its parameters from the epoch
 * snapshot w_t (Alg. 2: z_hat = z - eta * grad f(u)), sends Q(z_hat_k), and the
 * server forms z = (1/K) sum_k Q(z_hat_k), u = w_t + z and the running sum of
 * z that the epoch mean needs (Alg. 2 / Alg. 3, last step).  Q is the
 * coordinate-wise stochastic rounding of Sec. 2.1, Eq. (2), applied bucket by
 * bucket with the bucket's own scale (Sec. 3, bucket remark).
 *
 * Conventions
 *   - Every data pointer is DEVICE memory owned by the caller; the library
 *     neither allocates nor frees nor keeps pointers after a call returns.
 *   - Data pointers must be 16-byte aligned (packed blocks: 256-byte aligned).
 *   - Calls validate their arguments on the host, enqueue kernels on `stream`
 *     (a hipStream_t passed as void*, NULL = the default stream) and return
 *     without synchronising.  Argument errors are detected before any HIP call,
 *     so they can be exercised on a machine without a GPU.
 *   - Return value: QESGD_OK (0) or a negative QESGD_ERR_* code.  Nothing has
 *     been enqueued when an argument error is returned; QESGD_ERR_HIP reports a
 *     failed launch, and the launches of the same call that preceded it (the
 *     partial-sum passes of wide buckets) may already be in the stream.
 *   - Inputs must be finite; NaN / Inf give unspecified codes.
 *   - Arithmetic is IEEE binary32, round to nearest even, no fused multiply-add,
 *     subnormals kept; results do not depend on the launch geometry.
 *
 * Quantiser (one reading of what the paper leaves open)
 *   - s magnitude levels {0..s-1}, s in {2,4,8,16,32,64,128,256,65536}; m =
 *     log2(s) level bits plus one sign bit per coordinate; grid step delta_b =
 *     norm_b/(s-1).  (The widths that divide 32 take the specialised kernels.)
 *   - bucket b covers coordinates [b*bucket, min((b+1)*bucket, d)); bucket >= d
 *     means a single bucket; otherwise bucket must be a multiple of 32.
 *   - norm_b: L2 norm (fp32 sum of squares added as a balanced binary tree over
 *     the bucket zero-padded to a power of two, then sqrt) or max |v_i|.
 *   - coordinate i: a = min(|v_i|*(s-1)/norm_b, s-1); level = floor(a) +
 *     [r + trunc(frac(a)*2^16) >= 2^16] with r the 16-bit uniform variate of i;
 *     sign = [v_i < 0].
 *   - r: Philox4x32-10, key = seed, counter = (i>>3 low, i>>3 high, worker,
 *     round); coordinate i takes output word (i&7)>>1, low half if i is even,
 *     high half if odd.
 *
 * Packed block of one worker (byte offsets from qesgd_layout_query, each a
 * multiple of 256):
 *     float    norms [n_buckets]              at norms_off
 *     uint32_t signs [ceil(d/32)]             at signs_off   bit (i&31) of word i>>5
 *     uint32_t levels[ceil(d*m/32)]           at levels_off  bits [i*m, i*m+m) of the plane read as
 *                                                            one little-endian bit string (bit t = bit
 *                                                            t&31 of word t>>5; for m = 3,5,6,7 a
 *                                                            field may continue in the next word)
 *   Unused high bits of the last word of a plane are written as 0; bytes
 *   between the planes are never written.
 */
#ifndef QESGD_H
#define QESGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QESGD_ABI_VERSION 2u
#define QESGD_MAX_WORKERS 64u
#define QESGD_NOALLOC_SCRATCH_BYTES (4u << 20)

enum {
    QESGD_OK = 0,
    QESGD_ERR_NULL = -1,       /* a required pointer is NULL                          */
    QESGD_ERR_DIM = -2,        /* d == 0 or d >= 2^40, or the launch would need 2^31
                                  workgroups or more (one per 1024..65536 coordinates
                                  and worker: e.g. d = 2^38 with K = 64)              */
    QESGD_ERR_LEVELS = -3,     /* s not 2,4,8,16,32,64,128,256 or 65536                */
    QESGD_ERR_BUCKET = -4,     /* bucket == 0, or bucket < d and bucket % 32 != 0      */
    QESGD_ERR_WORKERS = -5,    /* K == 0 or K > QESGD_MAX_WORKERS                      */
    QESGD_ERR_NORM_KIND = -6,  /* norm_kind not QESGD_NORM_L2 / QESGD_NORM_MAX         */
    QESGD_ERR_ALIGN = -7,      /* a pointer is not aligned as required                 */
    QESGD_ERR_STRIDE = -8,     /* a slab stride is too small or not a 16-byte multiple */
    QESGD_ERR_WORKSPACE = -9,  /* workspace NULL or smaller than qesgd_workspace_bytes */
    QESGD_ERR_HIP = -10,       /* a launch failed; see qesgd_last_hip_error()          */
    QESGD_ERR_BITS = -11,      /* b not in {2,4,8,16}                                  */
    QESGD_ERR_DELTA = -12,     /* delta not a positive finite number                   */
    QESGD_ERR_ROUNDS = -13,    /* rounds == 0                                          */
    QESGD_ERR_SCRATCH = -14    /* the shape needs more than QESGD_NOALLOC_SCRATCH_BYTES */
};

enum { QESGD_NORM_L2 = 0, QESGD_NORM_MAX = 1 };

typedef struct qesgd_layout {
    uint64_t n_buckets;        /* ceil(d / min(bucket, d))                              */
    uint32_t level_bits;       /* m = log2(s)                                           */
    uint32_t reserved;
    uint64_t sign_words;       /* ceil(d / 32)                                          */
    uint64_t level_words;      /* ceil(d * m / 32)                                      */
    uint64_t norms_off;        /* byte offsets inside a worker's packed block           */
    uint64_t signs_off;
    uint64_t levels_off;
    uint64_t bytes_per_worker; /* size of a packed block, a multiple of 256            */
    uint64_t payload_bytes;    /* 4*(n_buckets + sign_words + level_words): what a
                                  worker would put on the wire                          */
} qesgd_layout;

/* Shape of the packed form for (d, s, bucket).  Host only.  (Sec. 3, bucket
 * remark; Sec. 5 accounts the traffic in bits per coordinate.) */
int qesgd_layout_query(uint64_t d, uint32_t s, uint64_t bucket, qesgd_layout* out);

/* Bytes of device scratch that qesgd_quantize_pack[_batched] needs for
 * (d, s, bucket, K).  0 whenever the zero-padded bucket has at most 32,768
 * coordinates (the scale is then found in one pass over the input); larger
 * buckets take a second pass and park partial sums here.  Returns 0 on invalid
 * arguments as well (the quantize call reports them). */
size_t qesgd_workspace_bytes(uint64_t d, uint32_t s, uint64_t bucket, uint32_t K);

/* Worker side: z = Q(z_hat) of Alg. 2, per bucket (Sec. 2.1 Eq. (2); Sec. 3).
 *   x       [d] fp32, device.  The vector to quantise ...
 *   center  [d] fp32, device, or NULL.  ... or, when given, v = x - center is
 *           quantised (x = current parameters, center = w_t: the deviation from
 *           the snapshot of Sec. 2.2 is formed on the fly).
 *   seed, round, worker  select the variates; equal triples give equal codes.
 *   packed  device, 256-byte aligned, qesgd_layout.bytes_per_worker bytes, written.
 *   workspace / workspace_bytes  device scratch, see qesgd_workspace_bytes; may
 *           be NULL / 0 when that returns 0. */
int qesgd_quantize_pack(const float* x, const float* center,
                        uint64_t d, uint32_t s, uint64_t bucket, uint32_t norm_kind,
                        uint64_t seed, uint32_t round, uint32_t worker,
                        void* packed, void* workspace, size_t workspace_bytes, void* stream);

/* The same for K simulated workers in one launch: worker k reads
 * x_slab + k*x_stride (stride in floats, a multiple of 4, >= d), uses variates
 * (seed, round, worker = k) and writes packed_slab + k*packed_stride (bytes, a
 * multiple of 256, >= bytes_per_worker).  center (shared, [d]) may be NULL. */
int qesgd_quantize_pack_batched(const float* x_slab, uint64_t x_stride, const float* center,
                                uint64_t d, uint32_t s, uint64_t bucket, uint32_t norm_kind,
                                uint64_t seed, uint32_t round, uint32_t K,
                                void* packed_slab, uint64_t packed_stride,
                                void* workspace, size_t workspace_bytes, void* stream);

/* qesgd_quantize_pack_batched for callers that can neither allocate nor bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same results bit for bit, no workspace: the partial sums of wide buckets go to a
 * QESGD_NOALLOC_SCRATCH_BYTES array that lives in the library's device image, one copy per GPU,
 * held until the process ends.  The call allocates and frees nothing.
 *   - Shapes with qesgd_workspace_bytes(d, s, bucket, K) > QESGD_NOALLOC_SCRATCH_BYTES are rejected
 *     with QESGD_ERR_SCRATCH before any HIP call (the limit is K * n_buckets * padded bucket
 *     <= 2^32 coordinates; shapes that need no workspace are never rejected for it).
 *   - The device that is current at the call must be the one `stream` belongs to; the first call
 *     on a device that needs the scratch looks its address up (hipGetSymbolAddress), so make that
 *     call once before capturing a graph.
 *   - All calls on one GPU share the array: calls that overlap in time on one GPU (two streams,
 *     two threads) race on it.  Nothing in it has to be cleared between calls: every partial sum
 *     a call reads was written by that call. */
int qesgd_quantize_pack_batched_noalloc(const float* x_slab, uint64_t x_stride, const float* center,
                                        uint64_t d, uint32_t s, uint64_t bucket, uint32_t norm_kind,
                                        uint64_t seed, uint32_t round, uint32_t K,
                                        void* packed_slab, uint64_t packed_stride, void* stream);

/* Server side (Alg. 3, server task: the sum over the p workers and its scaling):
 *   zbar[i] = ( sum_{k=0}^{K-1} +-level_{k,i} * (norm_{k,b(i)}/(s-1)) ) / K,
 * workers added in the order k = 0..K-1 starting from +0.
 *   packed_slab  K packed blocks, packed_stride bytes apart.   zbar [d] fp32, written. */
int qesgd_unpack_aggregate(const void* packed_slab, uint64_t packed_stride, uint32_t K,
                           uint64_t d, uint32_t s, uint64_t bucket, float* zbar, void* stream);

/* u = w_t + z (Alg. 2) and, when zsum is given, zsum += z (the sum behind the
 * epoch mean w_{t+1} = w_t + (1/K_t) sum_k z_{t,k}, Alg. 3 last step).
 *   w_snap [d], zbar [d] read; u_out [d] written; zsum_inout [d] or NULL.
 *   u_out may alias w_snap or zbar. */
int qesgd_apply_update(const float* w_snap, const float* zbar,
                       float* u_out, float* zsum_inout, uint64_t d, void* stream);

/* qesgd_unpack_aggregate followed by qesgd_apply_update in one pass, with
 * bit-identical results.  zbar_out and zsum_inout may be NULL. */
int qesgd_unpack_aggregate_update(const void* packed_slab, uint64_t packed_stride, uint32_t K,
                                  uint64_t d, uint32_t s, uint64_t bucket,
                                  const float* w_snap, float* zbar_out, float* u_out,
                                  float* zsum_inout, void* stream);

/* A whole round on a GPU that holds the K workers and the server: qesgd_quantize_pack_batched
 * followed by qesgd_unpack_aggregate_update, same arguments, same results bit for bit (the packed
 * blocks are written too).  Buckets are independent on the worker side (Sec. 3) and coordinates
 * on the server side (Alg. 3, server task), so one workgroup can own one tile of every worker and
 * of z: for a power-of-two bucket of 32..32768 coordinates, the L2 scale and a level width that
 * divides 32 the round is a single launch that never reads the packed codes back; every other
 * shape runs the two calls one after the other.  It exists for sizes at which a round is bound by
 * its launches; in the method the two halves run on different machines. */
int qesgd_round(const float* x_slab, uint64_t x_stride, const float* center,
                uint64_t d, uint32_t s, uint64_t bucket, uint32_t norm_kind,
                uint64_t seed, uint32_t round, uint32_t K,
                void* packed_slab, uint64_t packed_stride, void* workspace, size_t workspace_bytes,
                const float* w_snap, float* zbar_out, float* u_out, float* zsum_inout, void* stream);

/* The quantiser exactly as the paper writes it (Sec. 2.1, Eq. (1)-(2)): fixed grid
 * {delta*k : -2^(b-1) <= k <= 2^(b-1)-1}, b in {2,4,8,16}, step delta chosen by the caller
 * (e.g. the schedule delta_t = O(1/(sqrt(t) 2^(b-1))) of Sec. 4).  Per coordinate:
 * a = fl(v/delta); a >= 2^(b-1)-1 gives the top code, a <= -2^(b-1) the bottom code (the two
 * clamp cases); otherwise k = floor(a) + [r + trunc(fl(a - floor(a))*2^16) >= 2^16] with the same
 * variates r as qesgd_quantize_pack.  v = x, or x - center when center is given.
 *   codes  device, 16-byte aligned, ceil(d*b/32) uint32 words, written: coordinate i is the
 *          b-bit two's complement of k at bit (i*b)&31 of word (i*b)>>5; unused high bits 0. */
int qesgd_quantize_fixed(const float* x, const float* center, uint64_t d, float delta, uint32_t b,
                         uint64_t seed, uint32_t round, uint32_t worker, void* codes, void* stream);

/* Inverse of the above fused with Alg. 2's u = w_t + z: z_i = fl(k_i * delta),
 * u_i = w_i + z_i, zsum_i += z_i.  z_out, (w_snap, u_out) and zsum_inout are each optional
 * (NULL), at least one output must be given; u_out needs w_snap. */
int qesgd_dequantize_fixed_update(const void* codes, uint64_t d, float delta, uint32_t b,
                                  const float* w_snap, float* z_out, float* u_out, float* zsum_inout,
                                  void* stream);

/* End of an epoch (Alg. 3, last step; equal to Alg. 2's mean of the iterates u_{t,k}):
 * w_i += zsum_i / rounds, then zsum_i = 0 for the next epoch (z starts again at 0). */
int qesgd_epoch_commit(float* w_inout, float* zsum_inout, uint32_t rounds, uint64_t d, void* stream);

const char* qesgd_strerror(int code);
/* hipError_t (as int) of the last failed launch on the calling thread, 0 if none. */
int qesgd_last_hip_error(void);
uint32_t qesgd_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* QESGD_H */
