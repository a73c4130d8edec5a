// Status strings, one-time device set-up, the aggregation over groups of validation examples, and the
// Gaussian quantile table of the projection
// (paper Sec. 2.4 allows a Gaussian random matrix; entries are the 256 standard-normal
// quantiles Phi^-1((i + 1/2)/256), each rounded to the nearest bfloat16).
#include "common.h"
#include <atomic>
#include <cstring>
#include <mutex>
#include <vector>

namespace qless {

// The table is a constant of the library (bfloat16 bit patterns), so that every host builds the same
// R whatever its math library; T[255 - i] = -T[i].
static const uint16_t kGaussianTable[256] = {
    0xC039, 0xC021, 0xC015, 0xC00D, 0xC007, 0xC002, 0xBFFA, 0xBFF2, 0xBFEB, 0xBFE5, 0xBFDF, 0xBFD9,
    0xBFD4, 0xBFCF, 0xBFCB, 0xBFC6, 0xBFC2, 0xBFBE, 0xBFBB, 0xBFB7, 0xBFB4, 0xBFB0, 0xBFAD, 0xBFAA,
    0xBFA7, 0xBFA4, 0xBFA2, 0xBF9F, 0xBF9C, 0xBF99, 0xBF97, 0xBF94, 0xBF92, 0xBF90, 0xBF8D, 0xBF8B,
    0xBF89, 0xBF87, 0xBF84, 0xBF82, 0xBF80, 0xBF7C, 0xBF78, 0xBF74, 0xBF70, 0xBF6D, 0xBF69, 0xBF65,
    0xBF61, 0xBF5E, 0xBF5A, 0xBF56, 0xBF53, 0xBF4F, 0xBF4C, 0xBF48, 0xBF45, 0xBF42, 0xBF3E, 0xBF3B,
    0xBF38, 0xBF35, 0xBF31, 0xBF2E, 0xBF2B, 0xBF28, 0xBF25, 0xBF22, 0xBF1F, 0xBF1C, 0xBF19, 0xBF16,
    0xBF13, 0xBF10, 0xBF0D, 0xBF0A, 0xBF07, 0xBF04, 0xBF01, 0xBEFD, 0xBEF7, 0xBEF2, 0xBEEC, 0xBEE7,
    0xBEE1, 0xBEDC, 0xBED6, 0xBED1, 0xBECB, 0xBEC6, 0xBEC0, 0xBEBB, 0xBEB6, 0xBEB0, 0xBEAB, 0xBEA6,
    0xBEA1, 0xBE9B, 0xBE96, 0xBE91, 0xBE8C, 0xBE86, 0xBE81, 0xBE78, 0xBE6E, 0xBE63, 0xBE59, 0xBE4F,
    0xBE45, 0xBE3B, 0xBE30, 0xBE26, 0xBE1C, 0xBE12, 0xBE08, 0xBDFB, 0xBDE7, 0xBDD3, 0xBDBF, 0xBDAB,
    0xBD97, 0xBD82, 0xBD5D, 0xBD35, 0xBD0C, 0xBCC9, 0xBC71, 0xBBA0, 0x3BA0, 0x3C71, 0x3CC9, 0x3D0C,
    0x3D35, 0x3D5D, 0x3D82, 0x3D97, 0x3DAB, 0x3DBF, 0x3DD3, 0x3DE7, 0x3DFB, 0x3E08, 0x3E12, 0x3E1C,
    0x3E26, 0x3E30, 0x3E3B, 0x3E45, 0x3E4F, 0x3E59, 0x3E63, 0x3E6E, 0x3E78, 0x3E81, 0x3E86, 0x3E8C,
    0x3E91, 0x3E96, 0x3E9B, 0x3EA1, 0x3EA6, 0x3EAB, 0x3EB0, 0x3EB6, 0x3EBB, 0x3EC0, 0x3EC6, 0x3ECB,
    0x3ED1, 0x3ED6, 0x3EDC, 0x3EE1, 0x3EE7, 0x3EEC, 0x3EF2, 0x3EF7, 0x3EFD, 0x3F01, 0x3F04, 0x3F07,
    0x3F0A, 0x3F0D, 0x3F10, 0x3F13, 0x3F16, 0x3F19, 0x3F1C, 0x3F1F, 0x3F22, 0x3F25, 0x3F28, 0x3F2B,
    0x3F2E, 0x3F31, 0x3F35, 0x3F38, 0x3F3B, 0x3F3E, 0x3F42, 0x3F45, 0x3F48, 0x3F4C, 0x3F4F, 0x3F53,
    0x3F56, 0x3F5A, 0x3F5E, 0x3F61, 0x3F65, 0x3F69, 0x3F6D, 0x3F70, 0x3F74, 0x3F78, 0x3F7C, 0x3F80,
    0x3F82, 0x3F84, 0x3F87, 0x3F89, 0x3F8B, 0x3F8D, 0x3F90, 0x3F92, 0x3F94, 0x3F97, 0x3F99, 0x3F9C,
    0x3F9F, 0x3FA2, 0x3FA4, 0x3FA7, 0x3FAA, 0x3FAD, 0x3FB0, 0x3FB4, 0x3FB7, 0x3FBB, 0x3FBE, 0x3FC2,
    0x3FC6, 0x3FCB, 0x3FCF, 0x3FD4, 0x3FD9, 0x3FDF, 0x3FE5, 0x3FEB, 0x3FF2, 0x3FFA, 0x4002, 0x4007,
    0x400D, 0x4015, 0x4021, 0x4039,
};

const uint16_t *gaussian_table_bf16() { return kGaussianTable; }

struct LdsEntry { const void *fn; int bytes; };
static std::vector<LdsEntry> &lds_kernels() {
    static std::vector<LdsEntry> list;            // built by static initialisers of the other files
    return list;
}
static std::mutex &ready_mutex() {
    static std::mutex m;
    return m;
}
bool register_lds_kernel(const void *fn, int bytes) {
    std::lock_guard<std::mutex> lock(ready_mutex());
    for (LdsEntry &e : lds_kernels())
        if (e.fn == fn) { if (bytes > e.bytes) e.bytes = bytes; return true; }
    lds_kernels().push_back(LdsEntry{fn, bytes});
    return true;
}

constexpr int kMaxReadyDevices = 64;
static std::atomic<bool> ready[kMaxReadyDevices];

qless_status device_ready() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxReadyDevices) return QLESS_ERR_DEVICE;
    if (ready[dev].load(std::memory_order_acquire)) return QLESS_OK;
    std::lock_guard<std::mutex> lock(ready_mutex());
    if (ready[dev].load(std::memory_order_relaxed)) return QLESS_OK;
    for (const LdsEntry &e : lds_kernels())
        if (hipFuncSetAttribute(e.fn, hipFuncAttributeMaxDynamicSharedMemorySize, e.bytes) != hipSuccess) {
            (void)hipGetLastError();
            return QLESS_ERR_DEVICE;
        }
    void *scratch = nullptr;
    const qless_status rs = topk_scratch_address(&scratch);
    if (rs != QLESS_OK) return rs;
    ready[dev].store(true, std::memory_order_release);
    return QLESS_OK;
}

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

qless_status aggregate_rows(const float *full, int64_t N, int32_t M, const GroupEnds &ge, int T, int mean,
                            float *out, hipStream_t st) {
    int64_t blocks = (N * (int64_t)T + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(aggregate_kernel, dim3((unsigned)blocks), dim3(256), 0, st, full, N, M, ge, T, mean, out);
    return launch_status();
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
    return qless::aggregate_rows(full, N, M, ge, T, mode == QLESS_AGG_MEAN ? 1 : 0, out, (hipStream_t)stream);
}

extern "C" qless_status qless_init(void) { return qless::device_ready(); }

extern "C" const char *qless_status_string(qless_status s) {
    switch (s) {
        case QLESS_OK: return "ok";
        case QLESS_ERR_INVALID_ARG: return "invalid argument";
        case QLESS_ERR_UNSUPPORTED: return "unsupported configuration";
        case QLESS_ERR_WORKSPACE: return "workspace missing, too small or misaligned";
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
