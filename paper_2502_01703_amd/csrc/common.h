// Shared host/device helpers of the HIP library (status handling, the R generator).
// The generator is specified in prose in the design notes; this is the library's own
// implementation of that specification (the CPU oracle has a separate one).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "qless.h"

namespace qless {

constexpr uint32_t kGold = 0x9E3779B1u;       // word-counter stride
constexpr uint32_t kSaltStride = 0x68E31DA4u; // separates the Rademacher and Gaussian streams
constexpr uint32_t kMulA = 0x85EBCA6Bu;
constexpr uint32_t kMulB = 0xC2B2AE35u;

__host__ __device__ inline uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= kMulA; x ^= x >> 13; x *= kMulB; x ^= x >> 16;
    return x;
}

struct SeedKeys { uint32_t s0, s1; };
struct RowKey { uint32_t a, b; };

__host__ __device__ inline SeedKeys seed_keys(uint64_t seed) {
    SeedKeys k;
    k.s0 = mix32((uint32_t)seed + 0x9E3779B9u);
    k.s1 = mix32((uint32_t)(seed >> 32) ^ k.s0 ^ 0x7F4A7C15u);
    return k;
}
__host__ __device__ inline RowKey row_key(SeedKeys sk, uint32_t m) {
    RowKey r;
    r.a = mix32(sk.s1 + m * kGold);
    r.b = mix32(r.a ^ sk.s0 ^ 0x5BD1E995u);
    return r;
}
// counter = w * kGold + salt * kSaltStride (mod 2^32), formed by the caller
__host__ __device__ inline uint32_t key_word(RowKey key, uint32_t counter) {
    uint32_t x = key.a + counter;
    x ^= x >> 16; x *= kMulA; x ^= key.b;
    x ^= x >> 13; x *= kMulB; x ^= x >> 16;
    return x;
}

inline qless_status launch_status() {
    return hipGetLastError() == hipSuccess ? QLESS_OK : QLESS_ERR_DEVICE;
}
inline bool valid_bits(int bits) { return bits == 1 || bits == 2 || bits == 4 || bits == 8; }

// Gaussian table (bf16 bit patterns), built once on the host
const uint16_t *gaussian_table_bf16();

}  // namespace qless
