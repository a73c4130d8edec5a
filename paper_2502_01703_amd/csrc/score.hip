// qless_score: influence of every train example on every validation example from the packed
// datastore (paper Eq.(6),(7), Sec. 3.2), summed over checkpoints with learning-rate weights and
// reduced by max over validation examples.
//
// Integer dot products are exact; how they are formed depends on the code width:
//   1-bit   D = k - 2 popcount(a ^ b)                                   (XOR + V_BCNT)
//   2-bit   D = popcount(nz_a & nz_b) - 2 popcount(nz_a & nz_b & (sg_a ^ sg_b))   (bit planes)
//   8-bit   int8 x int8 -> int32 MFMA (v_mfma_i32_32x32x32_i8)
//   4-bit   nibbles moved to the high half of a byte ((w<<4)&0xF0F0F0F0, w&0xF0F0F0F0) give int8
//           operands 16 q; the MFMA accumulates 256 D, shifted back exactly.
// The fp32 epilogue is a fixed sequence of single operations (compiled without contraction):
//   acc += ((float)D * rnorm_train) * (eta * rnorm_val), checkpoints in order, starting from +0.
//
// A workgroup owns a block of train rows and walks over all validation tiles, keeping the
// running row maximum in registers, so every train code is read from HBM once per val tile
// (and from L2 after the first) and `score` is written exactly once.
#include "common.h"

namespace qless {

struct ScoreArgs {
    const unsigned char *tc[QLESS_MAX_CHECKPOINTS];
    const unsigned char *vc[QLESS_MAX_CHECKPOINTS];
    const float *tr[QLESS_MAX_CHECKPOINTS];
    const float *vr[QLESS_MAX_CHECKPOINTS];
    float eta[QLESS_MAX_CHECKPOINTS];
    int C;
    int64_t N;
    int32_t M, k;
    float *score, *full;
};

__device__ inline float neg_inf() { return __uint_as_float(0xFF800000u); }

// ------------------------------------------------------------------------------------------
// 1-bit / 2-bit: popcount kernel.  Thread grid TY x TX; thread (ty, tx) owns train rows
// ty + TY*i (i < RT) and val rows tx + TX*j (j < CT) of the tile.  Rows past the end of the
// train or val set are read from the last valid row (clamped) and masked in the epilogue.
// ------------------------------------------------------------------------------------------
template <int BITS, int RT, int CT, int TY, int TX>
__global__ void __launch_bounds__(256, 2)
score_popcount_kernel(ScoreArgs a) {
    static_assert(TY * TX == 256, "256 threads");
    constexpr int KC = 16;                      // words per plane per stage
    constexpr int PL = BITS;                    // bit planes per row
    constexpr int SW = PL * KC + 4;             // LDS row stride in words (pad: conflict-free b128)
    constexpr int TN = RT * TY, TM = CT * TX;
    constexpr int RSTEP = 256 / (8 * PL);       // rows covered by one pass of 8-byte loads
    constexpr int TMP = ((TM + RSTEP - 1) / RSTEP) * RSTEP;
    constexpr int ROWS = TN + TMP;
    constexpr int UT = TN / RSTEP, UV = TMP / RSTEP;
    static_assert(TN % RSTEP == 0, "train tile is a multiple of the load pass");
    extern __shared__ __attribute__((aligned(16))) uint32_t lds[];

    const int tid = threadIdx.x;
    const int tx = tid % TX, ty = tid / TX;
    const int64_t row0 = (int64_t)blockIdx.x * TN;
    const int kw = a.k / 32;                    // words per plane
    const int nstages = (kw + KC - 1) / KC;
    const int64_t cb = (int64_t)a.k * BITS / 8;
    // staging role of this thread: 8-byte chunk q of plane pl of rows rloc + RSTEP*u
    const int q = tid & 7;
    const int pl = PL == 2 ? ((tid >> 3) & 1) : 0;
    const int rloc = tid / (8 * PL);
    const int lds_slot = rloc * SW + pl * KC + q * 2;

    float rmax[RT];
#pragma unroll
    for (int i = 0; i < RT; ++i) rmax[i] = neg_inf();

    for (int v0 = 0; v0 < a.M; v0 += TM) {
        float facc[RT][CT];
#pragma unroll
        for (int i = 0; i < RT; ++i)
#pragma unroll
            for (int j = 0; j < CT; ++j) facc[i][j] = 0.0f;

        for (int ci = 0; ci < a.C; ++ci) {
            const unsigned char *tcp = a.tc[ci] + (int64_t)pl * (a.k / 8);
            const unsigned char *vcp = a.vc[ci] + (int64_t)pl * (a.k / 8);
            int accP[RT][CT], accN[BITS == 2 ? RT : 1][BITS == 2 ? CT : 1];
#pragma unroll
            for (int i = 0; i < RT; ++i)
#pragma unroll
                for (int j = 0; j < CT; ++j) { accP[i][j] = 0; if (BITS == 2) accN[i][j] = 0; }

            uint2 st[UT + UV];
            auto fetch = [&](int s) {
                int w = s * KC + q * 2;
                const bool live = w < kw;
                if (!live) w = kw - 2;
#pragma unroll
                for (int u = 0; u < UT; ++u) {
                    int64_t r = row0 + rloc + RSTEP * u;
                    if (r > a.N - 1) r = a.N - 1;
                    const uint2 val = *(const uint2 *)(tcp + r * cb + (int64_t)w * 4);
                    st[u] = live ? val : make_uint2(0, 0);
                }
#pragma unroll
                for (int u = 0; u < UV; ++u) {
                    int r = v0 + rloc + RSTEP * u;
                    if (r > a.M - 1) r = a.M - 1;
                    const uint2 val = *(const uint2 *)(vcp + (int64_t)r * cb + (int64_t)w * 4);
                    st[UT + u] = live ? val : make_uint2(0, 0);
                }
            };
            auto commit = [&](int buf) {
                uint32_t *dst = lds + buf * ROWS * SW + lds_slot;
#pragma unroll
                for (int u = 0; u < UT + UV; ++u) *(uint2 *)(dst + u * RSTEP * SW) = st[u];
            };
            fetch(0);
            commit(0);
            __syncthreads();
            for (int s = 0; s < nstages; ++s) {
                const int buf = s & 1;
                if (s + 1 < nstages) fetch(s + 1);
                const uint32_t *ta = lds + buf * ROWS * SW + ty * SW;
                const uint32_t *va = lds + buf * ROWS * SW + (TN + tx) * SW;
#pragma unroll 1
                for (int g = 0; g < KC / 4; ++g) {
                    uint4 an[RT], as[BITS == 2 ? RT : 1];
#pragma unroll
                    for (int i = 0; i < RT; ++i) {
                        an[i] = *(const uint4 *)(ta + TY * i * SW + g * 4);
                        if (BITS == 2) as[i] = *(const uint4 *)(ta + TY * i * SW + KC + g * 4);
                    }
#pragma unroll
                    for (int j = 0; j < CT; ++j) {
                        const uint4 bn = *(const uint4 *)(va + TX * j * SW + g * 4);
                        if (BITS == 1) {
#pragma unroll
                            for (int i = 0; i < RT; ++i) {
                                accP[i][j] += __popc(an[i].x ^ bn.x);
                                accP[i][j] += __popc(an[i].y ^ bn.y);
                                accP[i][j] += __popc(an[i].z ^ bn.z);
                                accP[i][j] += __popc(an[i].w ^ bn.w);
                            }
                        } else {
                            const uint4 bs = *(const uint4 *)(va + TX * j * SW + KC + g * 4);
#pragma unroll
                            for (int i = 0; i < RT; ++i) {
                                uint32_t t;
                                t = an[i].x & bn.x; accP[i][j] += __popc(t); accN[i][j] += __popc(t & (as[i].x ^ bs.x));
                                t = an[i].y & bn.y; accP[i][j] += __popc(t); accN[i][j] += __popc(t & (as[i].y ^ bs.y));
                                t = an[i].z & bn.z; accP[i][j] += __popc(t); accN[i][j] += __popc(t & (as[i].z ^ bs.z));
                                t = an[i].w & bn.w; accP[i][j] += __popc(t); accN[i][j] += __popc(t & (as[i].w ^ bs.w));
                            }
                        }
                    }
                }
                if (s + 1 < nstages) commit(buf ^ 1);
                __syncthreads();
            }
            // checkpoint epilogue
            float rt[RT], wv[CT];
#pragma unroll
            for (int i = 0; i < RT; ++i) {
                int64_t r = row0 + ty + TY * i;
                if (r > a.N - 1) r = a.N - 1;
                rt[i] = a.tr[ci][r];
            }
#pragma unroll
            for (int j = 0; j < CT; ++j) {
                int c = v0 + tx + TX * j;
                if (c > a.M - 1) c = a.M - 1;
                wv[j] = __fmul_rn(a.eta[ci], a.vr[ci][c]);
            }
#pragma unroll
            for (int i = 0; i < RT; ++i)
#pragma unroll
                for (int j = 0; j < CT; ++j) {
                    const int D = BITS == 1 ? a.k - 2 * accP[i][j] : accP[i][j] - 2 * accN[i][j];
                    const float t = __fmul_rn(__fmul_rn((float)D, rt[i]), wv[j]);
                    facc[i][j] = __fadd_rn(facc[i][j], t);
                }
        }
        // val-tile epilogue
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            const int64_t r = row0 + ty + TY * i;
#pragma unroll
            for (int j = 0; j < CT; ++j) {
                const int c = v0 + tx + TX * j;
                if (c < a.M) {
                    rmax[i] = fmaxf(rmax[i], facc[i][j]);
                    if (a.full && r < a.N) a.full[r * a.M + c] = facc[i][j];
                }
            }
        }
    }
    if (a.score) {
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            float m = rmax[i];
#pragma unroll
            for (int o = TX / 2; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
            const int64_t r = row0 + ty + TY * i;
            if (tx == 0 && r < a.N) a.score[r] = m;
        }
    }
}

// ------------------------------------------------------------------------------------------
// 8-bit / 4-bit: int8 MFMA kernel.  Workgroup tile 256 train rows x 64 val rows; each of the
// four waves owns 64 x 64 as 2 x 2 accumulators of 32 x 32.
// ------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(16))) int i32x16;

template <int BITS>
__global__ void __launch_bounds__(256)
score_mfma_kernel(ScoreArgs a) {
    constexpr int TN = 256, TM = 64, ROWS = TN + TM;
    constexpr int KE = BITS == 8 ? 64 : 128;        // code elements per stage
    constexpr int SB = KE * BITS / 8;               // stage bytes per row: 64
    constexpr int STRIDE = SB + 16;
    constexpr int CHUNKS = ROWS * (SB / 16);        // 16-byte chunks per stage
    constexpr int CPT = (CHUNKS + 255) / 256;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int64_t row0 = (int64_t)blockIdx.x * TN;
    const int64_t cb = (int64_t)a.k * BITS / 8;
    const int nstages = (a.k + KE - 1) / KE;

    float rmax[2][16];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) rmax[b][v] = neg_inf();

    for (int v0 = 0; v0 < a.M; v0 += TM) {
        float facc[2][2][16];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int v = 0; v < 16; ++v) facc[b][c][v] = 0.0f;

        for (int ci = 0; ci < a.C; ++ci) {
            const unsigned char *tcp = a.tc[ci], *vcp = a.vc[ci];
            i32x16 acc[2][2];
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int c = 0; c < 2; ++c)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[b][c][v] = 0;

            uint4 st[CPT];
            auto fetch = [&](int s) {
#pragma unroll
                for (int u = 0; u < CPT; ++u) {
                    const int c = tid + 256 * u;
                    uint4 val = make_uint4(0, 0, 0, 0);
                    if (c < CHUNKS) {
                        const int r = c / (SB / 16), q = c % (SB / 16);
                        const int64_t byte = (int64_t)s * SB + q * 16;
                        if (byte < cb) {
                            if (r < TN) { if (row0 + r < a.N) val = *(const uint4 *)(tcp + (row0 + r) * cb + byte); }
                            else { if (v0 + (r - TN) < a.M) val = *(const uint4 *)(vcp + (int64_t)(v0 + r - TN) * cb + byte); }
                        }
                    }
                    st[u] = val;
                }
            };
            auto commit = [&](int buf) {
#pragma unroll
                for (int u = 0; u < CPT; ++u) {
                    const int c = tid + 256 * u;
                    if (c < CHUNKS) {
                        const int r = c / (SB / 16), q = c % (SB / 16);
                        *(uint4 *)(smem + buf * ROWS * STRIDE + r * STRIDE + q * 16) = st[u];
                    }
                }
            };
            __syncthreads();
            fetch(0);
            commit(0);
            __syncthreads();
            for (int s = 0; s < nstages; ++s) {
                const int buf = s & 1;
                if (s + 1 < nstages) fetch(s + 1);
                const unsigned char *ta = smem + buf * ROWS * STRIDE + (wave * 64) * STRIDE;
                const unsigned char *va = smem + buf * ROWS * STRIDE + TN * STRIDE;
#pragma unroll
                for (int ks = 0; ks < KE / 32; ++ks) {
                    i32x4 af[2], bf[2];
#pragma unroll
                    for (int b = 0; b < 2; ++b) {
                        if (BITS == 8) {
                            af[b] = *(const i32x4 *)(ta + (32 * b + l32) * STRIDE + 32 * ks + 16 * half);
                            bf[b] = *(const i32x4 *)(va + (32 * b + l32) * STRIDE + 32 * ks + 16 * half);
                        } else {
                            const uint2 pa = *(const uint2 *)(ta + (32 * b + l32) * STRIDE + 16 * ks + 8 * half);
                            const uint2 pb = *(const uint2 *)(va + (32 * b + l32) * STRIDE + 16 * ks + 8 * half);
                            af[b][0] = (int)((pa.x << 4) & 0xF0F0F0F0u); af[b][1] = (int)(pa.x & 0xF0F0F0F0u);
                            af[b][2] = (int)((pa.y << 4) & 0xF0F0F0F0u); af[b][3] = (int)(pa.y & 0xF0F0F0F0u);
                            bf[b][0] = (int)((pb.x << 4) & 0xF0F0F0F0u); bf[b][1] = (int)(pb.x & 0xF0F0F0F0u);
                            bf[b][2] = (int)((pb.y << 4) & 0xF0F0F0F0u); bf[b][3] = (int)(pb.y & 0xF0F0F0F0u);
                        }
                    }
#pragma unroll
                    for (int b = 0; b < 2; ++b)
#pragma unroll
                        for (int c = 0; c < 2; ++c)
                            acc[b][c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[b], bf[c], acc[b][c], 0, 0, 0);
                }
                if (s + 1 < nstages) commit(buf ^ 1);
                __syncthreads();
            }
            // checkpoint epilogue.  acc[b][c][v]: train row 32b + 8(v/4) + 4 half + v%4, val col 32c + l32
            // lane L of the wave holds rnorm of train row (wave*64 + L); rows are fetched by shuffle
            int64_t myrow = row0 + wave * 64 + lane;
            if (myrow > a.N - 1) myrow = a.N - 1;
            const float rt_lane = a.tr[ci][myrow];
            float wv[2];
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                int col = v0 + 32 * c + l32;
                if (col > a.M - 1) col = a.M - 1;
                wv[c] = __fmul_rn(a.eta[ci], a.vr[ci][col]);
            }
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float rt = __shfl(rt_lane, 32 * b + 8 * (v >> 2) + 4 * half + (v & 3), 64);
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        const int D = BITS == 8 ? acc[b][c][v] : (acc[b][c][v] >> 8);
                        const float t = __fmul_rn(__fmul_rn((float)D, rt), wv[c]);
                        facc[b][c][v] = __fadd_rn(facc[b][c][v], t);
                    }
                }
        }
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int col = v0 + 32 * c + l32;
            if (col < a.M) {
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        rmax[b][v] = fmaxf(rmax[b][v], facc[b][c][v]);
                        const int64_t r = row0 + wave * 64 + 32 * b + 8 * (v >> 2) + 4 * half + (v & 3);
                        if (a.full && r < a.N) a.full[r * a.M + col] = facc[b][c][v];
                    }
            }
        }
    }
    if (a.score) {
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float m = rmax[b][v];
#pragma unroll
                for (int o = 16; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
                const int64_t r = row0 + wave * 64 + 32 * b + 8 * (v >> 2) + 4 * half + (v & 3);
                if (l32 == 0 && r < a.N) a.score[r] = m;
            }
    }
}

template <int BITS, int RT, int CT, int TY, int TX>
static void launch_popcount(const ScoreArgs &a, hipStream_t st) {
    constexpr int TN = RT * TY, TM = CT * TX, SW = BITS * 16 + 4, RSTEP = 256 / (8 * BITS);
    constexpr int TMP = ((TM + RSTEP - 1) / RSTEP) * RSTEP;
    const size_t lds = 2 * (size_t)(TN + TMP) * SW * 4;
    const unsigned grid = (unsigned)((a.N + TN - 1) / TN);
    hipLaunchKernelGGL((score_popcount_kernel<BITS, RT, CT, TY, TX>), dim3(grid), dim3(256), lds, st, a);
}

}  // namespace qless

using namespace qless;

extern "C" size_t qless_score_workspace(int64_t N, int32_t M, int32_t k, int bits, int C) {
    (void)N; (void)M; (void)k; (void)bits; (void)C;
    return 0;
}

extern "C" qless_status qless_score(const void *const *train_codes, const float *const *train_rnorm,
                                    const void *const *val_codes, const float *const *val_rnorm,
                                    const float *eta, int C, int64_t N, int32_t M, int32_t k, int bits,
                                    float *score, float *full, void *ws, size_t ws_bytes, void *stream) {
    (void)ws; (void)ws_bytes;
    if (!train_codes || !train_rnorm || !val_codes || !val_rnorm || !eta) return QLESS_ERR_INVALID_ARG;
    if (C < 1 || N < 0 || M < 1 || k <= 0) return QLESS_ERR_INVALID_ARG;
    if (!score && !full) return QLESS_ERR_INVALID_ARG;
    if (C > QLESS_MAX_CHECKPOINTS || !valid_bits(bits) || k % 64 != 0 || k > 65536) return QLESS_ERR_UNSUPPORTED;
    if (N > (int64_t)0x7FFFFFFF * 64) return QLESS_ERR_UNSUPPORTED;
    ScoreArgs a{};
    for (int i = 0; i < C; ++i) {
        if (!val_codes[i] || !val_rnorm[i] || (N > 0 && (!train_codes[i] || !train_rnorm[i]))) return QLESS_ERR_INVALID_ARG;
        if ((uintptr_t)val_codes[i] % 16 || (uintptr_t)train_codes[i] % 16) return QLESS_ERR_INVALID_ARG;
        a.tc[i] = (const unsigned char *)train_codes[i]; a.vc[i] = (const unsigned char *)val_codes[i];
        a.tr[i] = train_rnorm[i]; a.vr[i] = val_rnorm[i]; a.eta[i] = eta[i];
    }
    a.C = C; a.N = N; a.M = M; a.k = k; a.score = score; a.full = full;
    if (N == 0) return QLESS_OK;
    hipStream_t st = (hipStream_t)stream;
    if (bits == 1) {
        if (M > 32) launch_popcount<1, 8, 4, 16, 16>(a, st);
        else if (M > 8) launch_popcount<1, 8, 4, 32, 8>(a, st);
        else launch_popcount<1, 8, 1, 32, 8>(a, st);
    } else if (bits == 2) {
        if (M > 32) launch_popcount<2, 4, 4, 16, 16>(a, st);
        else if (M > 8) launch_popcount<2, 4, 4, 32, 8>(a, st);
        else launch_popcount<2, 8, 1, 32, 8>(a, st);
    } else {
        const size_t lds = 2 * (size_t)(256 + 64) * (64 + 16);
        const unsigned grid = (unsigned)((N + 255) / 256);
        if (bits == 8) hipLaunchKernelGGL((score_mfma_kernel<8>), dim3(grid), dim3(256), lds, st, a);
        else hipLaunchKernelGGL((score_mfma_kernel<4>), dim3(grid), dim3(256), lds, st, a);
    }
    return launch_status();
}
