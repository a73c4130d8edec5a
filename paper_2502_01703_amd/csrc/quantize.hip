// qless_quantize: absmax b-bit quantisation and packing of projected gradients
// (paper Eq.(4),(5), Sec. 2.3 / 3.1; the 1-bit sign code of Table 3 / Sec. 5).
//
// Rows up to 8192 elements: one wavefront per row (four rows per workgroup), the whole row held
// in registers (128 floats per lane at k = 8192), absolute maximum and sum of squares reduced
// with DPP row shifts and broadcasts -- no LDS, no barrier, so every wavefront keeps its loads
// in flight independently.  Longer rows: one workgroup per row, cached in registers up to
// k = 16384, re-read (from L2) above that.  Canonical fp32 sequence on both paths:
//     scale = alpha / S (IEEE division),  q = clamp(rne(P * scale))
// Codes leave as packed words with coalesced stores.  HBM-bound: 4k bytes in, k*bits/8 + 8 out.
#include "common.h"

namespace qless {

constexpr int kQThreads = 256;

// Wavefront reductions on DPP: row_shr 1/2/4/8 build the totals of the four 16-lane rows in
// their last lanes, row_bcast15 / row_bcast31 carry them into lane 63.  Lanes without a source
// read 0, the identity of both uses (max of absolute values, unsigned sum).
template <int CTRL, int ROWMASK>
__device__ inline uint32_t dpp0(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROWMASK, 0xF, false);
}
__device__ inline float wave_max(float v) {          // v >= 0; result uniform
    uint32_t x = __float_as_uint(v);                 // non-negative floats order like their bits
    x = max(x, dpp0<0x111, 0xF>(x)); x = max(x, dpp0<0x112, 0xF>(x));
    x = max(x, dpp0<0x114, 0xF>(x)); x = max(x, dpp0<0x118, 0xF>(x));
    x = max(x, dpp0<0x142, 0xA>(x)); x = max(x, dpp0<0x143, 0xC>(x));
    return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)x, 63));
}
__device__ inline uint32_t wave_sum_u32(uint32_t x) {   // result uniform
    x += dpp0<0x111, 0xF>(x); x += dpp0<0x112, 0xF>(x);
    x += dpp0<0x114, 0xF>(x); x += dpp0<0x118, 0xF>(x);
    x += dpp0<0x142, 0xA>(x); x += dpp0<0x143, 0xC>(x);
    return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}

// OR of a value over each aligned group of 8 lanes, valid in the group's first lane
// (three v_or_b32 with DPP row_shl:1/2/4; lanes shifted in from outside a row read 0).
__device__ inline uint32_t or_reduce8(uint32_t v) {
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x101, 0xF, 0xF, true);
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x102, 0xF, 0xF, true);
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x104, 0xF, 0xF, true);
    return v;
}

__device__ inline int quant1(float p, float scale, float alpha) {
    float t = __fmul_rn(p, scale);
    float r = rintf(t);
    r = fminf(fmaxf(r, -alpha), alpha);
    return (int)r;
}

// Element ownership: thread t owns, for each group g, the E consecutive elements starting at
// g * 256 * E + t * E with E = 4: one dword of codes (8-bit), one 16-bit word (4-bit) or one
// nibble of plane bits OR-combined over 8 neighbouring lanes into a 32-bit plane word (2-/1-bit).
// k is a multiple of 64, so a thread's E elements are all inside the row or all outside, and so
// is every aligned group of 8 lanes for the bit planes.
// Branch-free load of a thread's E elements: the address is clamped into the row, elements past
// the row end become 0 by a select (so all of a thread's loads can be issued back to back).
// The row's value at element m is p[m] + p[plane + m] + ... over nsplit planes, added in that
// order (nsplit = 1 for an ordinary matrix; the fused projection passes its split-d partial sums).
// SUM = false is the plain matrix (one plane): no loop, so a thread's loads go out back to back.
// With an accumulator row `acc` the value is acc[m] + (that sum), and with a second one, `oth`, oth[m] is
// added last (the sliced datastore build: slices accumulated in call order, two accumulators joined).
template <int E, bool SUM>
__device__ inline void load_elems(const float *p, int base, int32_t k, bool vec, int nsplit, size_t plane,
                                  float (&v)[E], const float *acc = nullptr, const float *oth = nullptr) {
    const bool in = base < k;
    const int b = in ? base : k - E;
    if (!SUM) nsplit = 1;
    if (E >= 4 && vec) {
#pragma unroll
        for (int e = 0; e < E; e += 4) {
            float4 f = *(const float4 *)(p + b + e);
            int s = 1;
            for (; s + 4 <= nsplit; s += 4) {          // four planes in flight, added in plane order
                float4 t[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) t[u] = *(const float4 *)(p + (size_t)(s + u) * plane + b + e);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    f.x = __fadd_rn(f.x, t[u].x); f.y = __fadd_rn(f.y, t[u].y);
                    f.z = __fadd_rn(f.z, t[u].z); f.w = __fadd_rn(f.w, t[u].w);
                }
            }
            for (; s < nsplit; ++s) {
                const float4 t = *(const float4 *)(p + (size_t)s * plane + b + e);
                f.x = __fadd_rn(f.x, t.x); f.y = __fadd_rn(f.y, t.y);
                f.z = __fadd_rn(f.z, t.z); f.w = __fadd_rn(f.w, t.w);
            }
            if (SUM && acc) {
                const float4 t = *(const float4 *)(acc + b + e);
                f.x = __fadd_rn(t.x, f.x); f.y = __fadd_rn(t.y, f.y);
                f.z = __fadd_rn(t.z, f.z); f.w = __fadd_rn(t.w, f.w);
            }
            if (SUM && oth) {
                const float4 t = *(const float4 *)(oth + b + e);
                f.x = __fadd_rn(f.x, t.x); f.y = __fadd_rn(f.y, t.y);
                f.z = __fadd_rn(f.z, t.z); f.w = __fadd_rn(f.w, t.w);
            }
            v[e] = in ? f.x : 0.0f; v[e + 1] = in ? f.y : 0.0f;
            v[e + 2] = in ? f.z : 0.0f; v[e + 3] = in ? f.w : 0.0f;
        }
    } else {
#pragma unroll
        for (int e = 0; e < E; ++e) {
            float f = p[b + e];
            for (int s = 1; s < nsplit; ++s) f = __fadd_rn(f, p[(size_t)s * plane + b + e]);
            if (SUM && acc) f = __fadd_rn(acc[b + e], f);
            if (SUM && oth) f = __fadd_rn(f, oth[b + e]);
            v[e] = in ? f : 0.0f;
        }
    }
}

// Optional fp32 copy of the (summed) row, written while it is in registers.
template <int E>
__device__ inline void keep_elems(float *dst, int base, int32_t k, bool vec, const float (&v)[E]) {
    if (!dst || base >= k) return;
    if (E >= 4 && vec) {
#pragma unroll
        for (int e = 0; e < E; e += 4) *(float4 *)(dst + base + e) = make_float4(v[e], v[e + 1], v[e + 2], v[e + 3]);
    } else {
#pragma unroll
        for (int e = 0; e < E; ++e) dst[base + e] = v[e];
    }
}

template <int BITS, int E>
__device__ inline void emit_elems(const float (&v)[E], int base, int32_t k, float scale, float alpha,
                                  unsigned char *crow, int lane, uint32_t &n2) {
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
        if (in) *(uint16_t *)(crow + base / 2) = (uint16_t)w;
    } else {
        // plane bits of this thread's 4 elements, placed at bit 4*(lane%8) .. +3 of a 32-bit word
        uint32_t sg = 0, nz = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            if (BITS == 2) {
                const int q = quant1(v[e], scale, alpha);
                nz |= (uint32_t)(q != 0) << e;
                sg |= (uint32_t)(q < 0) << e;
            } else {
                sg |= (uint32_t)(v[e] < 0.0f) << e;
            }
        }
        const int sh = 4 * (lane & 7);
        sg <<= sh;
        sg = or_reduce8(sg);
        if (BITS == 2) {
            n2 += (unsigned)__popc(nz);
            nz <<= sh;
            nz = or_reduce8(nz);
        }
        if (in && (lane & 7) == 0) {
            if (BITS == 2) {
                *(uint32_t *)(crow + base / 8) = nz;
                *(uint32_t *)(crow + k / 8 + base / 8) = sg;
            } else {
                *(uint32_t *)(crow + base / 8) = sg;
            }
        }
    }
}

// MEAN selects the absmean variant (Sec. 5): the scale is 1 / mean|g| instead of alpha / max|g|, with
// the mean taken in fixed point (32 fractional bits below the binary exponent of the row maximum), so
// that it does not depend on the order of the additions.
template <int BITS, int NG, bool SUM, bool MEAN = false>   // NG > 0: the row fits NG register groups per thread; NG == 0: re-read it
__global__ void __launch_bounds__(kQThreads)
quantize_kernel(const float *__restrict__ P, int64_t ldP, int32_t k, unsigned char *__restrict__ codes,
                float *__restrict__ S_out, float *__restrict__ rnorm_out, int vec, int nsplit, size_t plane,
                float *keep, int64_t ldK, const float *accum = nullptr, int64_t ldA = 0,
                const float *other = nullptr, int64_t ldO = 0) {
    constexpr int E = 4;
    constexpr int GROUP = kQThreads * E;
    constexpr bool CACHED = NG > 0;
    constexpr int MAXG = CACHED ? NG : 1;
    __shared__ float s_max[4];
    __shared__ uint32_t s_sum[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const float *p = P + row * ldP;
    unsigned char *crow = codes + row * ((int64_t)k * BITS / 8);
    float *krow = keep ? keep + row * ldK : nullptr;
    const float *arow = accum ? accum + row * ldA : nullptr, *orow = other ? other + row * ldO : nullptr;
    const int ngroups = (k + GROUP - 1) / GROUP;

    float reg[MAXG][E];
    float amax = 0.0f;
    if (CACHED) {
#pragma unroll
        for (int g = 0; g < MAXG; ++g) {
            if (g < ngroups) {
                load_elems<E, SUM>(p, g * GROUP + tid * E, k, vec != 0, nsplit, plane, reg[g], arow, orow);
                if (SUM) keep_elems<E>(krow, g * GROUP + tid * E, k, vec != 0, reg[g]);
#pragma unroll
                for (int e = 0; e < E; ++e) amax = fmaxf(amax, fabsf(reg[g][e]));
            }
        }
    } else {
        for (int g = 0; g < ngroups; ++g) {
            load_elems<E, SUM>(p, g * GROUP + tid * E, k, vec != 0, nsplit, plane, reg[0], arow, orow);
            if (SUM) keep_elems<E>(krow, g * GROUP + tid * E, k, vec != 0, reg[0]);
#pragma unroll
            for (int e = 0; e < E; ++e) amax = fmaxf(amax, fabsf(reg[0][e]));
        }
    }
    amax = wave_max(amax);
    if (lane == 0) s_max[wave] = amax;
    __syncthreads();
    float S = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
    const float alpha = (float)((1 << (BITS - 1)) - 1);
    float scale = (BITS > 1 && S > 0.0f) ? __fdiv_rn(alpha, S) : 0.0f;
    if (MEAN) {
        __shared__ unsigned long long s_abs[4];
        int ex = 0;
        (void)frexpf(S, &ex);                                  // max|g| = f 2^ex, f in [0.5, 1)
        unsigned long long u = 0;                             // sum of trunc(|g| 2^(32-ex)), each below 2^32
        if (S > 0.0f) {
            if (CACHED) {
#pragma unroll
                for (int g = 0; g < MAXG; ++g)
                    if (g < ngroups) {
#pragma unroll
                        for (int e = 0; e < E; ++e) u += (uint32_t)ldexpf(fabsf(reg[g][e]), 32 - ex);
                    }
            } else {
                for (int g = 0; g < ngroups; ++g) {
                    load_elems<E, SUM>(p, g * GROUP + tid * E, k, vec != 0, nsplit, plane, reg[0], arow, orow);
#pragma unroll
                    for (int e = 0; e < E; ++e) u += (uint32_t)ldexpf(fabsf(reg[0][e]), 32 - ex);
                }
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) u += __shfl_xor(u, o, 64);
        if (lane == 0) s_abs[wave] = u;
        __syncthreads();
        const unsigned long long U = s_abs[0] + s_abs[1] + s_abs[2] + s_abs[3];
        S = S > 0.0f ? (float)ldexp((double)U / (double)k, ex - 32) : 0.0f;
        scale = (BITS > 1 && S > 0.0f) ? __fdiv_rn(1.0f, S) : 0.0f;
    }

    uint32_t n2 = 0;        // per-thread partial: < 2^32 for rows up to 2^26 elements
    if (CACHED) {
#pragma unroll
        for (int g = 0; g < MAXG; ++g)
            if (g < ngroups) emit_elems<BITS, E>(reg[g], g * GROUP + tid * E, k, scale, alpha, crow, lane, n2);
    } else {
        for (int g = 0; g < ngroups; ++g) {
            load_elems<E, SUM>(p, g * GROUP + tid * E, k, vec != 0, nsplit, plane, reg[0], arow, orow);
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
    n2 = wave_sum_u32(n2);   // a wavefront's share: < 2^32 for rows up to 2^20 elements
    if (lane == 0) s_sum[wave] = n2;
    __syncthreads();
    if (tid == 0) {
        const unsigned long long tot = (unsigned long long)s_sum[0] + s_sum[1] + s_sum[2] + s_sum[3];
        S_out[row] = S;
        rnorm_out[row] = tot ? (float)(1.0 / sqrt((double)tot)) : 0.0f;
    }
}

// One wavefront per row, k <= 256 * NG * ... : lane L owns, for each group g < NG, the four
// elements starting at 256 g + 4 L.
template <int BITS, int NG, bool VEC, bool SUM>
__global__ void __launch_bounds__(kQThreads)
quantize_wave_kernel(const float *__restrict__ P, int64_t ldP, int64_t n, int32_t k,
                     unsigned char *__restrict__ codes, float *__restrict__ S_out,
                     float *__restrict__ rnorm_out, int nsplit, size_t plane,
                     float *keep, int64_t ldK, const float *accum = nullptr, int64_t ldA = 0,
                     const float *other = nullptr, int64_t ldO = 0) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n) return;                       // whole wavefront; nothing below synchronises
    const float *p = P + row * ldP;
    unsigned char *crow = codes + row * ((int64_t)k * BITS / 8);
    float reg[NG][4];
    float amax = 0.0f;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        load_elems<4, SUM>(p, g * 256 + lane * 4, k, VEC, nsplit, plane, reg[g], accum ? accum + row * ldA : nullptr,
                           other ? other + row * ldO : nullptr);
        if (SUM) keep_elems<4>(keep ? keep + row * ldK : nullptr, g * 256 + lane * 4, k, VEC, reg[g]);
#pragma unroll
        for (int e = 0; e < 4; ++e) amax = fmaxf(amax, fabsf(reg[g][e]));
    }
    const float S = wave_max(amax);
    const float alpha = (float)((1 << (BITS - 1)) - 1);
    const float scale = (BITS > 1 && S > 0.0f) ? __fdiv_rn(alpha, S) : 0.0f;
    uint32_t n2 = 0;
#pragma unroll
    for (int g = 0; g < NG; ++g)
        emit_elems<BITS, 4>(reg[g], g * 256 + lane * 4, k, scale, alpha, crow, lane, n2);
    const uint32_t tot = BITS == 1 ? (uint32_t)k : wave_sum_u32(n2);
    if (lane == 0) {
        S_out[row] = S;
        rnorm_out[row] = tot ? (float)(1.0 / sqrt((double)tot)) : 0.0f;
    }
}

// Source rows: value(row, m) = sum over s < nsplit of P[s * plane + row * ldP + m].  A wavefront per
// row when there are many short rows; a workgroup per row when rows are long, or when few rows
// each sum many planes (more loads in flight per row).
template <int BITS>
static void launch_quantize(const float *P, int64_t ldP, int nsplit, size_t plane, float *keep, int64_t ldK,
                            int64_t n, int32_t k, void *codes, float *S, float *rnorm, hipStream_t st,
                            const float *accum = nullptr, int64_t ldA = 0, const float *other = nullptr, int64_t ldO = 0) {
    constexpr int E = 4;
    const int groups = (k + kQThreads * E - 1) / (kQThreads * E);
    const int vec = ((uintptr_t)P % 16 == 0 && ldP % 4 == 0 && plane % 4 == 0 &&
                     (!keep || ((uintptr_t)keep % 16 == 0 && ldK % 4 == 0)) &&
                     (!accum || ((uintptr_t)accum % 16 == 0 && ldA % 4 == 0)) &&
                     (!other || ((uintptr_t)other % 16 == 0 && ldO % 4 == 0))) ? 1 : 0;
    // summing kernels exist for 16-byte aligned planes only (the projection workspace always is)
    const bool sum = nsplit > 1 || keep != nullptr || accum != nullptr || other != nullptr;
    if (k <= 8192 && (!sum || (n >= 2048 && vec))) {
        // wavefront per row; 4 rows per workgroup
        for (int64_t r0 = 0; r0 < n; r0 += 0x40000000) {
            const int64_t rows = n - r0 < 0x40000000 ? n - r0 : 0x40000000;
            const float *p = P + r0 * ldP;
            float *kp = keep ? keep + r0 * ldK : nullptr;
            const float *ap = accum ? accum + r0 * ldA : nullptr, *op = other ? other + r0 * ldO : nullptr;
            unsigned char *c = (unsigned char *)codes + r0 * ((int64_t)k * BITS / 8);
            const dim3 grid((unsigned)((rows + 3) / 4)), block(kQThreads);
#define QLESS_QW(NG) do { \
                if (sum) hipLaunchKernelGGL((quantize_wave_kernel<BITS, NG, true, true>), grid, block, 0, st, p, ldP, rows, k, c, S + r0, rnorm + r0, nsplit, plane, kp, ldK, ap, ldA, op, ldO); \
                else if (vec) hipLaunchKernelGGL((quantize_wave_kernel<BITS, NG, true, false>), grid, block, 0, st, p, ldP, rows, k, c, S + r0, rnorm + r0, nsplit, plane, kp, ldK); \
                else hipLaunchKernelGGL((quantize_wave_kernel<BITS, NG, false, false>), grid, block, 0, st, p, ldP, rows, k, c, S + r0, rnorm + r0, nsplit, plane, kp, ldK); } while (0)
            if (k <= 2048) QLESS_QW(8);
            else if (k <= 4096) QLESS_QW(16);
            else QLESS_QW(32);
#undef QLESS_QW
        }
        return;
    }
    // grid.x is limited to 2^31-1 rows per launch
    for (int64_t r0 = 0; r0 < n; r0 += 0x40000000) {
        const int64_t rows = n - r0 < 0x40000000 ? n - r0 : 0x40000000;
        const float *p = P + r0 * ldP;
        float *kp = keep ? keep + r0 * ldK : nullptr;
        const float *ap = accum ? accum + r0 * ldA : nullptr, *op = other ? other + r0 * ldO : nullptr;
        unsigned char *c = (unsigned char *)codes + r0 * ((int64_t)k * BITS / 8);
#define QLESS_QB(NG) do { \
            if (sum) hipLaunchKernelGGL((quantize_kernel<BITS, NG, true>), dim3((unsigned)rows), dim3(kQThreads), 0, st, \
                                        p, ldP, k, c, S + r0, rnorm + r0, vec, nsplit, plane, kp, ldK, ap, ldA, op, ldO); \
            else hipLaunchKernelGGL((quantize_kernel<BITS, NG, false>), dim3((unsigned)rows), dim3(kQThreads), 0, st, \
                                    p, ldP, k, c, S + r0, rnorm + r0, vec, nsplit, plane, kp, ldK); } while (0)
        if (groups <= 4) QLESS_QB(4);
        else if (groups <= 8) QLESS_QB(8);
        else if (groups <= 16) QLESS_QB(16);
        else QLESS_QB(0);
#undef QLESS_QB
    }
}

// Absmean variant: workgroup-per-row kernels only (an HBM-bound comparator, not the datastore path).
template <int BITS>
static void launch_quantize_absmean(const float *P, int64_t ldP, int64_t n, int32_t k, void *codes, float *S,
                                    float *rnorm, hipStream_t st) {
    const int groups = (k + kQThreads * 4 - 1) / (kQThreads * 4);
    const int vec = ((uintptr_t)P % 16 == 0 && ldP % 4 == 0) ? 1 : 0;
    for (int64_t r0 = 0; r0 < n; r0 += 0x40000000) {
        const int64_t rows = n - r0 < 0x40000000 ? n - r0 : 0x40000000;
        const float *p = P + r0 * ldP;
        unsigned char *c = (unsigned char *)codes + r0 * ((int64_t)k * BITS / 8);
#define QLESS_QM(NG) hipLaunchKernelGGL((quantize_kernel<BITS, NG, false, true>), dim3((unsigned)rows), dim3(kQThreads), 0, st, \
                                        p, ldP, k, c, S + r0, rnorm + r0, vec, 1, (size_t)0, (float *)nullptr, (int64_t)0)
        if (groups <= 4) QLESS_QM(4);
        else if (groups <= 8) QLESS_QM(8);
        else if (groups <= 16) QLESS_QM(16);
        else QLESS_QM(0);
#undef QLESS_QM
    }
}

qless_status quantize_rows(const float *src, int64_t ld, int nsplit, size_t plane, float *keep, int64_t ldK,
                           int64_t n, int32_t k, int bits, void *codes, float *S, float *rnorm,
                           hipStream_t st, const float *accum, int64_t ldA, const float *other, int64_t ldO) {
    // rows too long for registers are read twice: an accumulator that the kept copy overwrites cannot be
    if ((accum || other) && k > kQThreads * 4 * 16) return QLESS_ERR_UNSUPPORTED;
    switch (bits) {
        case 8: launch_quantize<8>(src, ld, nsplit, plane, keep, ldK, n, k, codes, S, rnorm, st, accum, ldA, other, ldO); break;
        case 4: launch_quantize<4>(src, ld, nsplit, plane, keep, ldK, n, k, codes, S, rnorm, st, accum, ldA, other, ldO); break;
        case 2: launch_quantize<2>(src, ld, nsplit, plane, keep, ldK, n, k, codes, S, rnorm, st, accum, ldA, other, ldO); break;
        default: launch_quantize<1>(src, ld, nsplit, plane, keep, ldK, n, k, codes, S, rnorm, st, accum, ldA, other, ldO); break;
    }
    return launch_status();
}

// 16-bit LESS comparator store (Sec. 2.2, Table 1 baseline): rows normalised to unit length and
// rounded to bfloat16.  One workgroup per row; the squared norm is summed in fp64, the row is read
// a second time (from L2) for the scaling pass.  HBM-bound: 4k bytes in, 2k out.
__device__ inline uint16_t bf16_rne_bits(float f) {
    const uint32_t u = __float_as_uint(f);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);        // finite inputs
}
__global__ void __launch_bounds__(kQThreads)
normalize16_kernel(const float *__restrict__ P, int64_t ldP, int32_t k, uint16_t *__restrict__ out, int vec) {
    __shared__ double s_ss[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const float *p = P + row * ldP;
    uint16_t *o = out + row * (int64_t)k;
    double ss = 0.0;
    if (vec) {
        for (int m = tid * 4; m < k; m += kQThreads * 4) {
            const float4 f = *(const float4 *)(p + m);
            ss += (double)f.x * f.x + (double)f.y * f.y + (double)f.z * f.z + (double)f.w * f.w;
        }
    } else {
        for (int m = tid; m < k; m += kQThreads) ss += (double)p[m] * p[m];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if (lane == 0) s_ss[wave] = ss;
    __syncthreads();
    const double tot = (s_ss[0] + s_ss[1]) + (s_ss[2] + s_ss[3]);
    const float inv = tot > 0.0 ? (float)(1.0 / sqrt(tot)) : 0.0f;
    if (vec) {
        for (int m = tid * 4; m < k; m += kQThreads * 4) {
            const float4 f = *(const float4 *)(p + m);
            const uint32_t lo = bf16_rne_bits(__fmul_rn(f.x, inv)) | ((uint32_t)bf16_rne_bits(__fmul_rn(f.y, inv)) << 16);
            const uint32_t hi = bf16_rne_bits(__fmul_rn(f.z, inv)) | ((uint32_t)bf16_rne_bits(__fmul_rn(f.w, inv)) << 16);
            *(uint2 *)(o + m) = make_uint2(lo, hi);
        }
    } else {
        for (int m = tid; m < k; m += kQThreads) o[m] = bf16_rne_bits(__fmul_rn(p[m], inv));
    }
}

}  // namespace qless

using namespace qless;

extern "C" qless_status qless_normalize16(const float *P, int64_t ldP, int64_t n, int32_t k, void *out,
                                          void *stream) {
    if (n < 0 || k <= 0 || ldP < k) return QLESS_ERR_INVALID_ARG;
    if (n > 0 && (!P || !out)) return QLESS_ERR_INVALID_ARG;
    if (k % 64 != 0) return QLESS_ERR_UNSUPPORTED;
    if (n == 0) return QLESS_OK;
    const int vec = ((uintptr_t)P % 16 == 0 && ldP % 4 == 0 && (uintptr_t)out % 8 == 0) ? 1 : 0;
    for (int64_t r0 = 0; r0 < n; r0 += 0x40000000) {
        const int64_t rows = n - r0 < 0x40000000 ? n - r0 : 0x40000000;
        hipLaunchKernelGGL(normalize16_kernel, dim3((unsigned)rows), dim3(kQThreads), 0, (hipStream_t)stream,
                           P + r0 * ldP, ldP, k, (uint16_t *)out + r0 * (int64_t)k, vec);
    }
    return launch_status();
}

extern "C" qless_status qless_quantize(const float *P, int64_t ldP, int64_t n, int32_t k, int bits,
                                       void *codes, float *S, float *rnorm, void *stream) {
    if (n < 0 || k <= 0 || ldP < k) return QLESS_ERR_INVALID_ARG;
    if (n > 0 && (!P || !codes || !S || !rnorm)) return QLESS_ERR_INVALID_ARG;
    if ((uintptr_t)codes % 4) return QLESS_ERR_INVALID_ARG;            // the packed codes are stored as 32-bit words
    if (!valid_bits(bits) || k % 64 != 0) return QLESS_ERR_UNSUPPORTED;
    if (n == 0) return QLESS_OK;
    return quantize_rows(P, ldP, 1, 0, nullptr, 0, n, k, bits, codes, S, rnorm, (hipStream_t)stream);
}

extern "C" qless_status qless_quantize_absmean(const float *P, int64_t ldP, int64_t n, int32_t k, int bits,
                                               void *codes, float *S, float *rnorm, void *stream) {
    if (n < 0 || k <= 0 || ldP < k) return QLESS_ERR_INVALID_ARG;
    if (n > 0 && (!P || !codes || !S || !rnorm)) return QLESS_ERR_INVALID_ARG;
    if ((uintptr_t)codes % 4) return QLESS_ERR_INVALID_ARG;            // the packed codes are stored as 32-bit words
    if (!valid_bits(bits) || k % 64 != 0) return QLESS_ERR_UNSUPPORTED;
    if (n == 0) return QLESS_OK;
    hipStream_t st = (hipStream_t)stream;
    switch (bits) {
        case 8: launch_quantize_absmean<8>(P, ldP, n, k, codes, S, rnorm, st); break;
        case 4: launch_quantize_absmean<4>(P, ldP, n, k, codes, S, rnorm, st); break;
        case 2: launch_quantize_absmean<2>(P, ldP, n, k, codes, S, rnorm, st); break;
        default: launch_quantize_absmean<1>(P, ldP, n, k, codes, S, rnorm, st); break;
    }
    return launch_status();
}
