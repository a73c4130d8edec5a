// Status strings, the aggregation over groups of validation examples, and the host-side Gaussian
// quantile table of the projection
// (paper Sec. 2.4 allows a Gaussian random matrix; entries are the 256 standard-normal
// quantiles Phi^-1((i + 1/2)/256), each rounded to the nearest bfloat16).
#include "common.h"
#include <cmath>
#include <cstring>
#include <mutex>

namespace qless {

// Phi^-1 by Newton's iteration on Phi(x) - p with Phi from erfc, started at 0 and safeguarded
// by a shrinking bracket.
static double normal_quantile(double p) {
    double lo = -12.0, hi = 12.0, x = 0.0;
    for (int it = 0; it < 100; ++it) {
        const double cdf = 0.5 * std::erfc(-x * 0.70710678118654752440);
        const double err = cdf - p;
        if (err > 0) hi = x; else lo = x;
        const double pdf = 0.39894228040143267794 * std::exp(-0.5 * x * x);
        double nx = x - err / pdf;
        if (!(nx > lo && nx < hi)) nx = 0.5 * (lo + hi);
        if (std::fabs(nx - x) < 1e-15 * (1.0 + std::fabs(x))) { x = nx; break; }
        x = nx;
    }
    return x;
}

static uint16_t to_bf16_rne(double v) {
    const float f = (float)v;
    uint32_t u;
    std::memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

const uint16_t *gaussian_table_bf16() {
    static uint16_t table[256];
    static std::once_flag once;
    std::call_once(once, [] {
        for (int i = 0; i < 256; ++i) table[i] = to_bf16_rne(normal_quantile((i + 0.5) / 256.0));
    });
    return table;
}

struct GroupEnds { int32_t end[QLESS_MAX_GROUPS]; };

// one thread per (train example, group): the group's entries are visited in column order, so the
// mean is the same sequence of fp32 additions for every launch shape
__global__ void __launch_bounds__(256)
aggregate_kernel(const float *full, int64_t N, int32_t M, GroupEnds ge, int T, int mean, float *out) {
    const int64_t total = N * (int64_t)T;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t z = i / T;
        const int t = (int)(i - z * T);
        const int32_t g0 = t ? ge.end[t - 1] : 0, g1 = ge.end[t];
        const float *row = full + z * (int64_t)M;
        float r;
        if (mean) {
            float s = 0.0f;
            for (int32_t j = g0; j < g1; ++j) s = __fadd_rn(s, row[j]);
            r = __fdiv_rn(s, (float)(g1 - g0));
        } else {
            r = row[g0];
            for (int32_t j = g0 + 1; j < g1; ++j) { const float v = row[j]; if (v > r) r = v; }
        }
        out[i] = r;
    }
}

}  // namespace qless

extern "C" qless_status qless_aggregate(const float *full, int64_t N, int32_t M, const int32_t *group_end, int T,
                                        qless_agg mode, float *out, void *stream) {
    if (N < 0 || M < 1 || !group_end || T < 1) return QLESS_ERR_INVALID_ARG;
    if (mode != QLESS_AGG_MAX && mode != QLESS_AGG_MEAN) return QLESS_ERR_UNSUPPORTED;
    if (T > QLESS_MAX_GROUPS) return QLESS_ERR_UNSUPPORTED;
    qless::GroupEnds ge{};
    for (int t = 0; t < T; ++t) {
        const int32_t g0 = t ? group_end[t - 1] : 0;
        if (group_end[t] <= g0 || group_end[t] > M) return QLESS_ERR_INVALID_ARG;
        ge.end[t] = group_end[t];
    }
    if (group_end[T - 1] != M) return QLESS_ERR_INVALID_ARG;
    if (N == 0) return QLESS_OK;
    if (!full || !out) return QLESS_ERR_INVALID_ARG;
    int64_t blocks = (N * (int64_t)T + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(qless::aggregate_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, full, N, M, ge, T,
                       mode == QLESS_AGG_MEAN ? 1 : 0, out);
    return qless::launch_status();
}

extern "C" const char *qless_status_string(qless_status s) {
    switch (s) {
        case QLESS_OK: return "ok";
        case QLESS_ERR_INVALID_ARG: return "invalid argument";
        case QLESS_ERR_UNSUPPORTED: return "unsupported configuration";
        case QLESS_ERR_WORKSPACE: return "workspace missing or too small";
        case QLESS_ERR_DEVICE: return "HIP runtime error";
    }
    return "unknown status";
}

extern "C" qless_status qless_gaussian_table(float *host_out256) {
    if (!host_out256) return QLESS_ERR_INVALID_ARG;
    const uint16_t *t = qless::gaussian_table_bf16();
    for (int i = 0; i < 256; ++i) {
        const uint32_t u = (uint32_t)t[i] << 16;
        std::memcpy(&host_out256[i], &u, 4);
    }
    return QLESS_OK;
}
