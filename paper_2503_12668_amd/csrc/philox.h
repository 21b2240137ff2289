// Counter-based random direction z (replaces the saved generator states of Alg. 2, Sec. 5.1):
// Philox4x32-10 keyed by the step seed, counter = (element index / 8, tensor id), followed by
// Box-Muller on 16-bit uniforms (each 32-bit output word yields one pair of elements).  z[p, e] is a pure function of (seed, p, e).
#pragma once
#include "common.h"

namespace zo2 {

struct PhiloxKeys {   // the ten round keys of one seed, wave-uniform (live in SGPRs)
    uint32_t k0[10], k1[10];
};

__host__ __device__ __forceinline__ PhiloxKeys philox_keys(uint64_t seed) {
    PhiloxKeys k;
    uint32_t a = (uint32_t)seed, b = (uint32_t)(seed >> 32);
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        k.k0[r] = a;
        k.k1[r] = b;
        a += 0x9E3779B9u;
        b += 0xBB67AE85u;
    }
    return k;
}

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              const PhiloxKeys& k, uint32_t out[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        // three-input exclusive or in one instruction (truth table 0x96): left as two ^ the compiler emits two v_xor
        const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), c1, k.k0[r], 0x96);
        const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), c3, k.k1[r], 0x96);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// One Box-Muller pair from one word: u1 = ((x >> 16) + 1) / 2^16 in (0, 1],
// u2 = (x & 0xffff) / 2^16 in [0, 1); (rho cos 2 pi u2, rho sin 2 pi u2), rho = sqrt(-2 ln u1) <= 4.71.
// u1 and u2 are exact in fp32.  The hardware log2 / sqrt are 1-ulp operations; the
// hardware sin / cos take their argument in revolutions, which u2 already is.
__device__ __forceinline__ void box_muller(uint32_t x, float& za, float& zb) {
    const float u1 = (float)((x >> 16) + 1u) * 1.52587890625e-05f;
    const float u2 = (float)(x & 0xffffu) * 1.52587890625e-05f;
    // -2 ln u1 = (-2 ln 2) log2 u1
    const float t = -1.3862943611198906f * __builtin_amdgcn_logf(u1);
    const float rho = __builtin_amdgcn_sqrtf(t);
    za = rho * __builtin_amdgcn_cosf(u2);
    zb = rho * __builtin_amdgcn_sinf(u2);
}

// z of elements 8q .. 8q+7 of tensor `tensor_id`: one Philox call, output word i gives elements 8q+2i, 8q+2i+1.
__device__ __forceinline__ void gaussian8(const PhiloxKeys& k, uint32_t tensor_id, uint64_t q, float z[8]) {
    uint32_t w[4];
    philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), tensor_id, 0u, k, w);
#pragma unroll
    for (int i = 0; i < 4; ++i) box_muller(w[i], z[2 * i], z[2 * i + 1]);
}

// z of elements e .. e+3, e a multiple of 4 (half of a Philox call).
__device__ __forceinline__ void gaussian4(const PhiloxKeys& k, uint32_t tensor_id, uint64_t e, float z[4]) {
    const uint64_t q = e >> 3;
    uint32_t w[4];
    philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), tensor_id, 0u, k, w);
    const bool hi = (e & 4) != 0;
    box_muller(hi ? w[2] : w[0], z[0], z[1]);
    box_muller(hi ? w[3] : w[1], z[2], z[3]);
}

// 16 rounding bits for each of the elements 8q .. 8q+7 (stochastic rounding of the stored theta'): a second
// stream of the same generator, told apart by the last counter word (1; z uses 0).  Element 8q + j takes the
// low (j even) or high (j odd) half of output word j >> 1.
__device__ __forceinline__ void rounding_words(const PhiloxKeys& k, uint32_t tensor_id, uint64_t q, uint32_t w[4]) {
    philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), tensor_id, 1u, k, w);
}
__device__ __forceinline__ uint32_t rounding_bits_of(const uint32_t w[4], int j) { return (w[j >> 1] >> (16 * (j & 1))) & 0xffffu; }

}  // namespace zo2
