// Status strings and the host-side Gaussian quantile table of the projection
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

}  // namespace qless

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
