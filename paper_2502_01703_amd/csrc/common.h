// Shared host/device helpers of the HIP library: status handling, asynchronous LDS copies and
// the generator of the projection matrix R (paper Eq.(1): a random Rademacher or Gaussian map,
// Sec. 2.4; the paper fixes no generator).  R is never stored; entry (m, j) is a pure function
// of (seed, m, j):
//   mix(x):  x ^= x>>16; x *= 0x85EBCA6B; x ^= x>>13; x *= 0xC2B2AE35; x ^= x>>16      (mod 2^32)
//   s0 = mix(seed_lo + 0x9E3779B9),  s1 = mix(seed_hi ^ s0 ^ 0x7F4A7C15)
//   keyA(m) = mix(s1 + m*0x9E3779B1),  keyB(m) = mix(keyA(m) ^ s0 ^ 0x5BD1E995)
//   word(m, w, salt): x = keyA(m) + w*0x9E3779B1 + salt*0x68E31DA4;
//                     x ^= x>>16; x *= 0x85EBCA6B; x ^= keyB(m); x ^= x>>13; x *= 0xC2B2AE35; x ^= x>>16
//   Rademacher: R[m][j] = -1 iff bit beta(j%32) of word(m, j/32, 0) is set, beta(c) = 4*(c%8) + 3 - c/8
//   Gaussian:   R[m][j] = T[byte (j%4) of word(m, j/4, 1)], T[i] = bf16(Phi^-1((i + 1/2)/256))
// This file is the library's own implementation of that specification.
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

// Asynchronous 16-byte global -> LDS copy (no VGPR staging): lane L of the wavefront writes LDS
// bytes [lds_addr + 16 L, +16) with the 16 bytes at its own global address.  lds_addr must be
// wave-uniform.  Completion is tracked by vmcnt like any vector load; wait_vmcnt<N> blocks until
// at most N of the wavefront's vector memory operations are outstanding (they retire in order).
__device__ inline void global_to_lds16(const void *gptr, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(lds_addr), "v"(gptr) : "memory");
}
// Same with a wave-uniform base address (SGPR pair) plus an unsigned 32-bit lane offset.
__device__ inline void global_to_lds16(const void *base, unsigned lane_off, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(lane_off), "s"(base) : "memory");
}
template <int N> __device__ inline void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// Kernels that ask for more dynamic LDS than the 64 KB a launch may use by default.  Each such
// kernel is entered in a list while the library is loaded (no HIP call is made then);
// device_ready() raises the limit of every listed kernel on the current device, once per device,
// and is called by qless_init() and at the top of every entry point that launches one of them.
bool register_lds_kernel(const void *fn, int bytes);
qless_status device_ready();
template <auto Fn, int BYTES> struct LdsKernel {
    static inline const bool listed = register_lds_kernel((const void *)Fn, BYTES);
};
// names a kernel's list entry so that the entry exists in the loaded library
#define QLESS_LDS_KERNEL(fn, bytes) ((void)qless::LdsKernel<&fn, (bytes)>::listed)

// topk.hip: device address of the current GPU's scratch array of qless_topk_noalloc (looked up once
// per device)
qless_status topk_scratch_address(void **out);

inline qless_status launch_status() {
    return hipGetLastError() == hipSuccess ? QLESS_OK : QLESS_ERR_DEVICE;
}
inline bool valid_bits(int bits) { return bits == 1 || bits == 2 || bits == 4 || bits == 8; }

// quantize.hip: Eq.(4),(5) over n rows whose value at (row, m) is the sum, in ascending s, of
// src[s * plane + row * ld + m] for s < nsplit; `keep` (or null) receives the summed rows in fp32.
// With `accum` the value is accum[row * ldA + m] + (that sum), and `other[row * ldO + m]` is added last
// (accum may be the same memory as keep; rows of at most 16384 elements then).
qless_status quantize_rows(const float *src, int64_t ld, int nsplit, size_t plane, float *keep, int64_t ldK,
                           int64_t n, int32_t k, int bits, void *codes, float *S, float *rnorm,
                           hipStream_t st, const float *accum = nullptr, int64_t ldA = 0,
                           const float *other = nullptr, int64_t ldO = 0);

// Groups of consecutive validation columns: group t is [end[t-1], end[t]), end[-1] = 0.
struct GroupEnds { int32_t end[QLESS_MAX_GROUPS]; };
// misc.hip: out[z][t] = maximum (mean == 0) or left-to-right fp32 mean of full[z][group t], enqueued on st
qless_status aggregate_rows(const float *full, int64_t N, int32_t M, const GroupEnds &ge, int T, int mean,
                            float *out, hipStream_t st);

// Gaussian table (bf16 bit patterns)
const uint16_t *gaussian_table_bf16();

}  // namespace qless
