// QESGD hot-path ORACLE -- test infrastructure, not product code.
//
// A plain, single-threaded, deliberately slow CPU statement of what the
// quantize / pack / unpack / aggregate / update path computes.  Only tests,
// the smoke check and the benchmark's cpu_baseline leg may call it.  It shares
// no source, header, table or helper with the HIP library.
//
// What is written here, and where the paper fixes it:
//   * stochastic rounding to a uniform grid, floor/ceil with probability
//     proportional to the distance to the other neighbour   (Sec. 2.1, Eq. (2))
//   * every coordinate rounded independently                (Sec. 2.1, after Eq. (2))
//   * the vector is split into buckets, each compressed on its own with its
//     own scale                                             (Sec. 3, bucket remark)
//   * the quantised variable is the deviation z from the epoch snapshot w_t,
//     and the working parameter is u = w_t + z              (Sec. 2.2; Alg. 2)
//   * the server sums what the p workers sent and scales it (Alg. 3, server task)
//   * the epoch mean is w_t plus the mean of the z iterates (Alg. 2 / Alg. 3, last step)
//   * the norm is the L2 norm                               (Sec. 2, notation)
//
// What the paper leaves open and this file fixes (one reading each):
//   * "s levels": magnitudes {0, ..., s-1}, grid step delta = norm / (s-1),
//     one sign bit plus m = log2(s) magnitude bits per coordinate
//     (s = 2, 4, 8, 16, 32, 64, 128, 256, 65536).
//   * the packed form: a plane of sign bits and a plane of m-bit levels, each
//     one little-endian bit string cut into 32-bit words.
//   * the uniform variate has 16 bits: with a = |v| / delta, l = floor(a),
//     f = a - l, T = trunc(f * 2^16), the value is rounded up iff
//     r + T >= 2^16 for a 16-bit uniform r, so P(up) = T / 2^16 in (f - 2^-16, f].
//   * the uniform variates come from Philox4x32-10 (Salmon, Moraes, Dror, Shaw,
//     SC'11), key = seed, counter = (element group, worker, round); one call
//     serves 8 consecutive coordinates.
//   * the sum of squares is a pairwise binary tree in fp32 over the bucket
//     zero-padded to a power of two (floating-point addition is not
//     associative, so the order is part of the definition).
//   * all arithmetic is IEEE-754 binary32 with round-to-nearest-even, no fused
//     multiply-add, subnormals kept.  (Build: -O2 -ffp-contract=off, no fast-math.)
//
// Parity pins (tests/, CPU only): Philox against an independent library
// engine; rounding probabilities by exhaustive enumeration of the 16-bit
// variate; unbiasedness and the variance bound of Lemma 1 by enumeration and by
// Monte Carlo; the summation order on rounding-sensitive hand cases; pack /
// unpack round trips and a hand-written word example; aggregate / update against
// double precision and the epoch-mean identity; the fixed-grid quantiser of
// Eq. (1)-(2) by enumeration of the variate (probabilities, clamp cases, both
// halves of Lemma 1) and a hand-written code word.
// Parity unpinned: none of the functions below; the convergence behaviour of
// the full method (Theorem 1) is outside this path.

#include <cmath>
#include <cstddef>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

// ---------------------------------------------------------------------------
// Philox4x32-10.  One round: two 32x32->64 products, the high halves are mixed
// with the other two counter words and the key; the key is advanced by the
// Weyl constants between rounds.
// ---------------------------------------------------------------------------
const uint32_t PHILOX_MUL_A = 0xD2511F53u;  // multiplies counter word 0
const uint32_t PHILOX_MUL_B = 0xCD9E8D57u;  // multiplies counter word 2
const uint32_t PHILOX_WEYL_0 = 0x9E3779B9u;
const uint32_t PHILOX_WEYL_1 = 0xBB67AE85u;

void philox_round(uint32_t c[4], const uint32_t k[2]) {
    const uint64_t prod_a = (uint64_t)PHILOX_MUL_A * (uint64_t)c[0];
    const uint64_t prod_b = (uint64_t)PHILOX_MUL_B * (uint64_t)c[2];
    const uint32_t n0 = (uint32_t)(prod_b >> 32) ^ c[1] ^ k[0];
    const uint32_t n1 = (uint32_t)prod_b;
    const uint32_t n2 = (uint32_t)(prod_a >> 32) ^ c[3] ^ k[1];
    const uint32_t n3 = (uint32_t)prod_a;
    c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
}

void philox4x32_10(const uint32_t counter[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c[4] = {counter[0], counter[1], counter[2], counter[3]};
    uint32_t k[2] = {key[0], key[1]};
    for (int round = 0; round < 10; ++round) {
        if (round > 0) { k[0] += PHILOX_WEYL_0; k[1] += PHILOX_WEYL_1; }
        philox_round(c, k);
    }
    out[0] = c[0]; out[1] = c[1]; out[2] = c[2]; out[3] = c[3];
}

// The 16-bit uniform variate of coordinate i for (seed, round, worker).
// Coordinates 8g .. 8g+7 share Philox call g; coordinate i takes output word
// (i mod 8) / 2, low half if i is even and high half if i is odd.
uint32_t uniform16(uint64_t seed, uint32_t round, uint32_t worker, uint64_t i) {
    const uint64_t g = i >> 3;
    const uint32_t counter[4] = {(uint32_t)g, (uint32_t)(g >> 32), worker, round};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t o[4];
    philox4x32_10(counter, key, o);
    const uint32_t word = o[(i & 7) >> 1];
    return (i & 1) ? (word >> 16) : (word & 0xFFFFu);
}

// ---------------------------------------------------------------------------
// Problem shape.
// ---------------------------------------------------------------------------
int level_bits_of(uint32_t s) {          // m = log2(s) for the supported s
    switch (s) {
        case 2: return 1;
        case 4: return 2;
        case 8: return 3;
        case 16: return 4;
        case 32: return 5;
        case 64: return 6;
        case 128: return 7;
        case 256: return 8;
        case 65536: return 16;
        default: return -1;
    }
}

// The level plane is one little-endian bit string: coordinate i owns bits
// [i*m, i*m+m), bit t of the string being bit (t mod 32) of word t/32.  A field
// whose width does not divide 32 may continue into the next word.
void put_level(uint32_t* words, uint64_t i, uint64_t m, uint32_t level) {
    for (uint64_t j = 0; j < m; ++j) {
        const uint64_t t = i * m + j;
        if ((level >> j) & 1u) words[t >> 5] |= 1u << (t & 31);
    }
}

uint32_t get_level(const uint32_t* words, uint64_t i, uint64_t m) {
    uint32_t level = 0;
    for (uint64_t j = 0; j < m; ++j) {
        const uint64_t t = i * m + j;
        level |= ((words[t >> 5] >> (t & 31)) & 1u) << j;
    }
    return level;
}

uint64_t effective_bucket(uint64_t d, uint64_t bucket) { return bucket < d ? bucket : d; }

uint64_t pow2_at_least(uint64_t n) { uint64_t p = 1; while (p < n) p <<= 1; return p; }

// ---------------------------------------------------------------------------
// Bucket scale.  L2: square every coordinate in fp32, pad with +0 to N (a power
// of two), and add in a balanced binary tree: a node over [lo, lo+n) is the
// fp32 sum of its two halves.
// ---------------------------------------------------------------------------
float tree_sum_squares(const float* v, uint64_t len, uint64_t lo, uint64_t n) {
    if (n == 1) {
        if (lo >= len) return 0.0f;
        const float sq = v[lo] * v[lo];
        return sq;
    }
    const float left = tree_sum_squares(v, len, lo, n / 2);
    const float right = tree_sum_squares(v, len, lo + n / 2, n / 2);
    const float sum = left + right;
    return sum;
}

float bucket_norm(const float* v, uint64_t len, uint64_t padded_n, uint32_t norm_kind) {
    if (norm_kind == 0) return sqrtf(tree_sum_squares(v, len, 0, padded_n));
    float mx = 0.0f;
    for (uint64_t j = 0; j < len; ++j) { const float a = fabsf(v[j]); if (a > mx) mx = a; }
    return mx;
}

// (s-1)/norm, or 0 when that is not a finite number (empty or all-zero bucket,
// or a norm so small that the reciprocal overflows): such a bucket encodes as
// all-zero levels.
float inverse_step(float norm, float smax) {
    float inv = smax / norm;
    if (!(inv < INFINITY)) inv = 0.0f;
    return inv;
}

// Eq. (2) for one coordinate on the grid {0, delta, ..., (s-1) delta} of its
// magnitude: returns the level in [0, s-1].  r16 is the 16-bit uniform variate.
uint32_t round_level(float a, uint32_t r16) {
    const float l = floorf(a);
    const float f = a - l;                               // exact in fp32
    const uint32_t T = (uint32_t)(f * 65536.0f);         // exact product, truncated
    const uint32_t up = (r16 + T) >> 16;                 // 1 iff r16 + T >= 2^16
    return (uint32_t)l + up;
}

void quantize_coordinate(float v, float inv, float smax, uint32_t r16,
                         uint32_t* level, uint32_t* sign) {
    const float a = fminf(fabsf(v) * inv, smax);
    *level = round_level(a, r16);
    *sign = (v < 0.0f) ? 1u : 0u;
}

}  // namespace

extern "C" {

// ---- exposed pieces (so that each can be pinned on its own) ----------------

void qo_philox4x32_10(const uint32_t* counter, const uint32_t* key, uint32_t* out) {
    philox4x32_10(counter, key, out);
}

uint32_t qo_uniform16(uint64_t seed, uint32_t round, uint32_t worker, uint64_t i) {
    return uniform16(seed, round, worker, i);
}

int qo_level_bits(uint32_t s) { return level_bits_of(s); }

// Shape of the packed form of one worker's vector: buckets, 32-bit words in the
// sign plane, 32-bit words in the level plane, padded tree width.
int qo_shape(uint64_t d, uint32_t s, uint64_t bucket, uint64_t* n_buckets,
             uint64_t* sign_words, uint64_t* level_words, uint64_t* padded_n) {
    const int m = level_bits_of(s);
    if (m < 0 || d == 0 || bucket == 0) return -1;
    const uint64_t B = effective_bucket(d, bucket);
    if (B < d && (B % 32) != 0) return -1;
    *n_buckets = (d + B - 1) / B;
    *sign_words = (d + 31) / 32;
    *level_words = (d * (uint64_t)m + 31) / 32;
    *padded_n = pow2_at_least(B);
    return 0;
}

float qo_bucket_norm(const float* v, uint64_t len, uint64_t padded_n, uint32_t norm_kind) {
    return bucket_norm(v, len, padded_n, norm_kind);
}

// The fp32 tree sum of squares alone (the L2 scale before its square root).
float qo_bucket_sumsq(const float* v, uint64_t len, uint64_t padded_n) {
    return tree_sum_squares(v, len, 0, padded_n);
}

float qo_inverse_step(float norm, uint32_t s) { return inverse_step(norm, (float)(s - 1)); }

uint32_t qo_round_level(float a, uint32_t r16) { return round_level(a, r16); }

// One bucket: v[0..len) are its coordinates, the first of which is coordinate
// i0 of the whole vector (the variates are keyed on the global index).
// Writes the bucket scale and one level / sign per coordinate.
void qo_quantize_bucket(const float* v, uint64_t len, uint64_t padded_n, uint64_t i0,
                        uint32_t s, uint32_t norm_kind,
                        uint64_t seed, uint32_t round, uint32_t worker,
                        float* norm_out, uint32_t* level_out, uint8_t* sign_out) {
    const float smax = (float)(s - 1);
    const float norm = bucket_norm(v, len, padded_n, norm_kind);
    const float inv = inverse_step(norm, smax);
    for (uint64_t j = 0; j < len; ++j) {
        uint32_t level, sign;
        quantize_coordinate(v[j], inv, smax, uniform16(seed, round, worker, i0 + j), &level, &sign);
        level_out[j] = level;
        sign_out[j] = (uint8_t)sign;
    }
    *norm_out = norm;
}

// Codes -> words.  Coordinate i puts its sign in bit (i mod 32) of sign word
// i/32 and its level in the m bits starting at bit i*m of the level plane's bit
// string.  Unused high bits of the last word of a plane are 0.
void qo_pack(const uint32_t* level, const uint8_t* sign, uint64_t d, uint32_t s,
             uint32_t* sign_words, uint32_t* level_words) {
    const uint64_t m = (uint64_t)level_bits_of(s);
    const uint64_t nsw = (d + 31) / 32, nlw = (d * m + 31) / 32;
    for (uint64_t w = 0; w < nsw; ++w) sign_words[w] = 0;
    for (uint64_t w = 0; w < nlw; ++w) level_words[w] = 0;
    for (uint64_t i = 0; i < d; ++i) {
        sign_words[i >> 5] |= (uint32_t)(sign[i] & 1u) << (i & 31);
        put_level(level_words, i, m, level[i]);
    }
}

void qo_unpack(const uint32_t* sign_words, const uint32_t* level_words, uint64_t d, uint32_t s,
               uint32_t* level, uint8_t* sign) {
    const uint64_t m = (uint64_t)level_bits_of(s);
    for (uint64_t i = 0; i < d; ++i) {
        sign[i] = (uint8_t)((sign_words[i >> 5] >> (i & 31)) & 1u);
        level[i] = get_level(level_words, i, m);
    }
}

// ---- the three steps of a round -------------------------------------------

// Worker side (Alg. 2, the step z = Q(z_hat), per bucket): v = x, or x - center
// when center is given; norms[nb], sign_words, level_words as sized by qo_shape.
int qo_quantize_pack(const float* x, const float* center, uint64_t d, uint32_t s,
                     uint64_t bucket, uint32_t norm_kind,
                     uint64_t seed, uint32_t round, uint32_t worker,
                     float* norms, uint32_t* sign_words, uint32_t* level_words) {
    uint64_t nb, nsw, nlw, N;
    if (qo_shape(d, s, bucket, &nb, &nsw, &nlw, &N) != 0 || norm_kind > 1) return -1;
    const uint64_t B = effective_bucket(d, bucket);
    std::vector<float> v(d);
    for (uint64_t i = 0; i < d; ++i) {
        if (center) { const float diff = x[i] - center[i]; v[i] = diff; }
        else v[i] = x[i];
    }
    std::vector<uint32_t> level(d);
    std::vector<uint8_t> sign(d);
    for (uint64_t b = 0; b < nb; ++b) {
        const uint64_t i0 = b * B;
        const uint64_t len = (i0 + B <= d) ? B : (d - i0);
        qo_quantize_bucket(&v[i0], len, N, i0, s, norm_kind, seed, round, worker,
                           &norms[b], &level[i0], &sign[i0]);
    }
    qo_pack(level.data(), sign.data(), d, s, sign_words, level_words);
    return 0;
}

// Server side (Alg. 3, the sum over the p workers and its scaling), for the
// coordinates [i_begin, i_end): worker k's planes start at norms + k*nb,
// sign_words + k*nsw, level_words + k*nlw.  Workers are added in the order
// k = 0, 1, ..., K-1 starting from +0, then the sum is divided by K.
int qo_unpack_aggregate_range(const float* norms, const uint32_t* sign_words,
                              const uint32_t* level_words, uint32_t K,
                              uint64_t d, uint32_t s, uint64_t bucket,
                              uint64_t i_begin, uint64_t i_end, float* zbar /*[i_end-i_begin]*/) {
    uint64_t nb, nsw, nlw, N;
    if (qo_shape(d, s, bucket, &nb, &nsw, &nlw, &N) != 0 || K == 0 || i_end > d) return -1;
    const uint64_t B = effective_bucket(d, bucket);
    const uint64_t m = (uint64_t)level_bits_of(s);
    const float smax = (float)(s - 1);
    for (uint64_t i = i_begin; i < i_end; ++i) {
        const uint64_t b = i / B;
        float acc = 0.0f;
        for (uint32_t k = 0; k < K; ++k) {
            const float step = norms[(uint64_t)k * nb + b] / smax;
            const uint32_t level = get_level(level_words + (uint64_t)k * nlw, i, m);
            const uint32_t sign = (sign_words[(uint64_t)k * nsw + (i >> 5)] >> (i & 31)) & 1u;
            float q = (float)level * step;
            if (sign) q = -q;
            const float sum = acc + q;
            acc = sum;
        }
        zbar[i - i_begin] = acc / (float)K;
    }
    return 0;
}

int qo_unpack_aggregate(const float* norms, const uint32_t* sign_words, const uint32_t* level_words,
                        uint32_t K, uint64_t d, uint32_t s, uint64_t bucket, float* zbar) {
    return qo_unpack_aggregate_range(norms, sign_words, level_words, K, d, s, bucket, 0, d, zbar);
}

// u = w_t + z (Alg. 2), and the running sum of the z iterates that the epoch
// mean needs (last step of Alg. 2 / Alg. 3).  zsum may be null.
void qo_apply_update(const float* w_snap, const float* zbar, float* u, float* zsum, uint64_t d) {
    for (uint64_t i = 0; i < d; ++i) {
        const float ui = w_snap[i] + zbar[i];
        u[i] = ui;
        if (zsum) { const float zs = zsum[i] + zbar[i]; zsum[i] = zs; }
    }
}

// End of an epoch (last step of Alg. 3): w_{t+1} = w_t + (1/K_t) * sum_k z_{t,k}; the
// running sum restarts at 0 for the next epoch (z starts at 0 again, Alg. 2 first step).
void qo_epoch_commit(float* w, float* zsum, uint32_t rounds, uint64_t d) {
    const float kt = (float)rounds;
    for (uint64_t i = 0; i < d; ++i) {
        const float mean = zsum[i] / kt;
        const float wi = w[i] + mean;
        w[i] = wi;
        zsum[i] = 0.0f;
    }
}

// ---------------------------------------------------------------------------
// The quantiser exactly as the paper writes it (Sec. 2.1, Eq. (1)-(2)): a fixed
// grid {delta * k : -2^(b-1) <= k <= 2^(b-1) - 1} with a caller-chosen step
// delta (the schedule delta_t of Sec. 4 / Sec. 5 is the caller's), values outside
// the range are clamped to its ends, values inside are rounded down or up with
// probability proportional to the distance to the other neighbour.
// Readings: a = fl(v / delta) is formed in fp32; the variate has 16 bits and
// rounds up iff r + trunc(frac(a) * 2^16) >= 2^16 (as above); the code of k is its
// b-bit two's complement, b in {2, 4, 8, 16}, packed like the level plane
// (coordinate i at bit (i*b) mod 32 of word (i*b)/32).
// ---------------------------------------------------------------------------
int32_t qo_fixed_round(float v, float delta, uint32_t b, uint32_t r16) {
    const float lo = -(float)(1u << (b - 1));            // -2^(b-1)
    const float hi = (float)((1u << (b - 1)) - 1u);      //  2^(b-1) - 1
    float a = v / delta;
    if (a >= hi) return (int32_t)hi;                     // Eq. (2), first case
    if (a <= lo) return (int32_t)lo;                     // Eq. (2), last case
    const float l = floorf(a);
    const float f = a - l;                               // fp32: exact for a >= 0; a tiny negative a gives 1
    const uint32_t T = (uint32_t)(f * 65536.0f);         // 0 .. 65536
    const uint32_t up = (r16 + T) >> 16;                 // 0 or 1
    return (int32_t)l + (int32_t)up;
}

int qo_fixed_code_bits_ok(uint32_t b) { return (b == 2 || b == 4 || b == 8 || b == 16) ? 1 : 0; }

// codes: ceil(d*b/32) words.  v = x, or x - center when center is given.
int qo_quantize_fixed(const float* x, const float* center, uint64_t d, float delta, uint32_t b,
                      uint64_t seed, uint32_t round, uint32_t worker, uint32_t* codes) {
    if (!qo_fixed_code_bits_ok(b) || d == 0 || !(delta > 0.0f) || !(delta < INFINITY)) return -1;
    const uint64_t nw = (d * (uint64_t)b + 31) / 32;
    const uint32_t mask = (b == 32) ? 0xFFFFFFFFu : ((1u << b) - 1u);
    for (uint64_t w = 0; w < nw; ++w) codes[w] = 0;
    for (uint64_t i = 0; i < d; ++i) {
        float v = x[i];
        if (center) { const float diff = x[i] - center[i]; v = diff; }
        const int32_t k = qo_fixed_round(v, delta, b, uniform16(seed, round, worker, i));
        const uint64_t bit = i * (uint64_t)b;
        codes[bit >> 5] |= ((uint32_t)k & mask) << (bit & 31);
    }
    return 0;
}

// z = delta * k, u = w + z, zsum += z (zsum, z_out may be null).
int qo_dequantize_fixed_update(const uint32_t* codes, uint64_t d, float delta, uint32_t b,
                               const float* w_snap, float* z_out, float* u, float* zsum) {
    if (!qo_fixed_code_bits_ok(b) || d == 0) return -1;
    const uint32_t mask = (1u << b) - 1u;
    for (uint64_t i = 0; i < d; ++i) {
        const uint64_t bit = i * (uint64_t)b;
        uint32_t c = (codes[bit >> 5] >> (bit & 31)) & mask;
        int32_t k = (int32_t)c;
        if (c & (1u << (b - 1))) k -= (int32_t)(1u << b);            // sign extension
        const float z = (float)k * delta;
        if (z_out) z_out[i] = z;
        if (u) { const float ui = w_snap[i] + z; u[i] = ui; }
        if (zsum) { const float zs = zsum[i] + z; zsum[i] = zs; }
    }
    return 0;
}

}  // extern "C"
