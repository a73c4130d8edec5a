// qless_quantize: absmax b-bit quantisation and packing of projected gradients
// (paper Eq.(4),(5), Sec. 2.3 / 3.1; the 1-bit sign code of Table 3 / Sec. 5).
//
// One workgroup of 256 threads per row.  The row is read once into registers (k <= 16384) or
// twice (longer rows; the second read is served by L2), reduced to its absolute maximum with
// wavefront shuffles, quantised with the canonical fp32 sequence
//     scale = alpha / S (IEEE division),  q = clamp(rne(P * scale))
// and written as packed codes with coalesced stores.  HBM-bound: 4k bytes in, k*bits/8 + 8 out.
#include "common.h"

namespace qless {

constexpr int kQThreads = 256;
constexpr int kQMaxRegs = 64;   // floats cached per thread: rows up to 256*64 = 16384 elements

__device__ inline float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ inline unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ inline int quant1(float p, float scale, float alpha) {
    float t = __fmul_rn(p, scale);
    float r = rintf(t);
    r = fminf(fmaxf(r, -alpha), alpha);
    return (int)r;
}

// Element ownership: thread t owns, for each group g, the E consecutive elements starting at
// g * 256 * E + t * E, where E = 4 (8-bit: one dword of codes), 8 (4-bit: one dword) or
// 1 (2-/1-bit: a wavefront ballot yields 64 plane bits).  k is a multiple of 64, so a thread's
// E elements are all inside the row or all outside, and so is a whole wavefront for E = 1.
template <int E>
__device__ inline void load_elems(const float *p, int base, int32_t k, bool vec, float (&v)[E]) {
    if (base >= k) {
#pragma unroll
        for (int e = 0; e < E; ++e) v[e] = 0.0f;
        return;
    }
    if (E >= 4 && vec) {
#pragma unroll
        for (int e = 0; e < E; e += 4) {
            const float4 f = *(const float4 *)(p + base + e);
            v[e] = f.x; v[e + 1] = f.y; v[e + 2] = f.z; v[e + 3] = f.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < E; ++e) v[e] = p[base + e];
    }
}

template <int BITS, int E>
__device__ inline void emit_elems(const float (&v)[E], int base, int32_t k, float scale, float alpha,
                                  unsigned char *crow, int lane, unsigned long long &n2) {
    const bool in = base < k;
    if (BITS == 8) {
        uint32_t w = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int q = quant1(v[e], scale, alpha);
            n2 += (unsigned)(q * q);
            w |= ((uint32_t)q & 0xFFu) << (8 * e);
        }
        if (in) *(uint32_t *)(crow + base) = w;
    } else if (BITS == 4) {
        uint32_t w = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int q = quant1(v[e], scale, alpha);
            n2 += (unsigned)(q * q);
            w |= ((uint32_t)q & 0xFu) << (4 * e);
        }
        if (in) *(uint32_t *)(crow + base / 2) = w;
    } else if (BITS == 2) {
        const int q = quant1(v[0], scale, alpha);
        const unsigned long long nz = __ballot(in && q != 0);
        const unsigned long long sg = __ballot(in && q < 0);
        if (lane == 0 && in) {
            *(unsigned long long *)(crow + base / 8) = nz;
            *(unsigned long long *)(crow + k / 8 + base / 8) = sg;
            n2 += (unsigned)__popcll(nz);
        }
    } else {
        const unsigned long long sg = __ballot(in && v[0] < 0.0f);
        if (lane == 0 && in) *(unsigned long long *)(crow + base / 8) = sg;
    }
}

template <int BITS, bool CACHED>
__global__ void __launch_bounds__(kQThreads)
quantize_kernel(const float *__restrict__ P, int64_t ldP, int32_t k, unsigned char *__restrict__ codes,
                float *__restrict__ S_out, float *__restrict__ rnorm_out, int vec) {
    constexpr int E = BITS == 8 ? 4 : (BITS == 4 ? 8 : 1);
    constexpr int GROUP = kQThreads * E;
    constexpr int MAXG = CACHED ? kQMaxRegs / E : 1;
    __shared__ float s_max[4];
    __shared__ unsigned long long s_sum[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const float *p = P + row * ldP;
    unsigned char *crow = codes + row * ((int64_t)k * BITS / 8);
    const int ngroups = (k + GROUP - 1) / GROUP;

    float reg[MAXG][E];
    float amax = 0.0f;
    if (CACHED) {
#pragma unroll
        for (int g = 0; g < MAXG; ++g) {
            if (g < ngroups) {
                load_elems<E>(p, g * GROUP + tid * E, k, vec != 0, reg[g]);
#pragma unroll
                for (int e = 0; e < E; ++e) amax = fmaxf(amax, fabsf(reg[g][e]));
            }
        }
    } else {
        for (int g = 0; g < ngroups; ++g) {
            load_elems<E>(p, g * GROUP + tid * E, k, vec != 0, reg[0]);
#pragma unroll
            for (int e = 0; e < E; ++e) amax = fmaxf(amax, fabsf(reg[0][e]));
        }
    }
    amax = wave_max(amax);
    if (lane == 0) s_max[wave] = amax;
    __syncthreads();
    const float S = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
    const float alpha = (float)((1 << (BITS - 1)) - 1);
    const float scale = (BITS > 1 && S > 0.0f) ? __fdiv_rn(alpha, S) : 0.0f;

    unsigned long long n2 = 0;
    if (CACHED) {
#pragma unroll
        for (int g = 0; g < MAXG; ++g)
            if (g < ngroups) emit_elems<BITS, E>(reg[g], g * GROUP + tid * E, k, scale, alpha, crow, lane, n2);
    } else {
        for (int g = 0; g < ngroups; ++g) {
            load_elems<E>(p, g * GROUP + tid * E, k, vec != 0, reg[0]);
            emit_elems<BITS, E>(reg[0], g * GROUP + tid * E, k, scale, alpha, crow, lane, n2);
        }
    }
    if (BITS == 1) {
        if (tid == 0) {
            S_out[row] = S;
            rnorm_out[row] = (float)(1.0 / sqrt((double)k));
        }
        return;
    }
    n2 = wave_sum_u64(n2);
    if (lane == 0) s_sum[wave] = n2;
    __syncthreads();
    if (tid == 0) {
        const unsigned long long tot = s_sum[0] + s_sum[1] + s_sum[2] + s_sum[3];
        S_out[row] = S;
        rnorm_out[row] = tot ? (float)(1.0 / sqrt((double)tot)) : 0.0f;
    }
}

template <int BITS>
static void launch_quantize(const float *P, int64_t ldP, int64_t n, int32_t k, void *codes, float *S,
                            float *rnorm, hipStream_t st) {
    constexpr int E = BITS == 8 ? 4 : (BITS == 4 ? 8 : 1);
    const bool cached = ((k + kQThreads * E - 1) / (kQThreads * E)) * E <= kQMaxRegs;
    const int vec = ((uintptr_t)P % 16 == 0 && ldP % 4 == 0) ? 1 : 0;
    // grid.x is limited to 2^31-1 rows per launch
    for (int64_t r0 = 0; r0 < n; r0 += 0x40000000) {
        const int64_t rows = n - r0 < 0x40000000 ? n - r0 : 0x40000000;
        const float *p = P + r0 * ldP;
        unsigned char *c = (unsigned char *)codes + r0 * ((int64_t)k * BITS / 8);
        if (cached)
            hipLaunchKernelGGL((quantize_kernel<BITS, true>), dim3((unsigned)rows), dim3(kQThreads), 0, st,
                               p, ldP, k, c, S + r0, rnorm + r0, vec);
        else
            hipLaunchKernelGGL((quantize_kernel<BITS, false>), dim3((unsigned)rows), dim3(kQThreads), 0, st,
                               p, ldP, k, c, S + r0, rnorm + r0, vec);
    }
}

}  // namespace qless

using namespace qless;

extern "C" qless_status qless_quantize(const float *P, int64_t ldP, int64_t n, int32_t k, int bits,
                                       void *codes, float *S, float *rnorm, void *stream) {
    if (n < 0 || k <= 0 || ldP < k) return QLESS_ERR_INVALID_ARG;
    if (n > 0 && (!P || !codes || !S || !rnorm)) return QLESS_ERR_INVALID_ARG;
    if (!valid_bits(bits) || k % 64 != 0) return QLESS_ERR_UNSUPPORTED;
    if (n == 0) return QLESS_OK;
    hipStream_t st = (hipStream_t)stream;
    switch (bits) {
        case 8: launch_quantize<8>(P, ldP, n, k, codes, S, rnorm, st); break;
        case 4: launch_quantize<4>(P, ldP, n, k, codes, S, rnorm, st); break;
        case 2: launch_quantize<2>(P, ldP, n, k, codes, S, rnorm, st); break;
        default: launch_quantize<1>(P, ldP, n, k, codes, S, rnorm, st); break;
    }
    return launch_status();
}
