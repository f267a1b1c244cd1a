// Device-side pieces shared by the kernels of libqesgd (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qesgd {

// Three-way xor in one v_bitop3 (truth table of a ^ b ^ c).
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11).  counter = (c0, c1, c2, c3), key = (k0, k1).
// One round: two 32x32->64 products; the high halves are mixed with the other two counter words
// and the key, the key advances by the Weyl constants.  The key is wave-uniform in every kernel
// here, so its schedule lives in scalar registers; the 64-bit products are single v_mad_u64_u32.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&o)[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t pa = (uint64_t)0xD2511F53u * c0;
        const uint64_t pb = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = xor3((uint32_t)(pb >> 32), c1, k0);
        const uint32_t n2 = xor3((uint32_t)(pa >> 32), c3, k1);
        c1 = (uint32_t)pb;
        c3 = (uint32_t)pa;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    o[0] = c0; o[1] = c1; o[2] = c2; o[3] = c3;
}

// The 16-bit variate of the e-th of the 8 coordinates served by one call: word e/2, low half
// for even e, high half for odd e.
__device__ __forceinline__ uint32_t variate16(const uint32_t (&o)[4], int e) {
    const uint32_t word = o[e >> 1];
    return (e & 1) ? (word >> 16) : (word & 0xFFFFu);
}

}  // namespace qesgd
