// qless_project: P = R G^T-style random projection (paper Eq.(1); matrix families of Sec. 2.4)
// as a bf16 MFMA GEMM whose B operand (the random matrix) is generated in registers.
//
// Shape of the problem: M-dimension = batch rows n (small), N-dimension = k projected
// coordinates, contraction over the gradient dimension d (huge).  One workgroup of 8 waves
// owns a 64 (rows) x 1024 (coordinates) output tile for one slice of d; each wave owns
// 64 x 128 of it as 2 x 4 MFMA 32x32 accumulators.  Gaussian projections of batches that
// fill 128-row tiles take 128 x 512 tiles instead (4 x 2 accumulators per wave): every
// generated fragment of the random operand then feeds four matrix instructions instead of two.  The gradient tile is staged through LDS; partial tiles of
// the d-slices go to the workspace and are summed in a fixed order by a second kernel, so
// results are run-to-run identical.
//
// Random operand: lanes 0..31 of a wave take one 32-column word of R for their row m, lanes
// 32..63 the next word; the 32 sign bits of a word feed four MFMA K-steps of 8 columns each.
// Column c of a word reads hash bit 4*(c%8) + 3 - c/8, which is exactly what
// ((h << s) & 0x88888888) | 0x22222222 places in the sign position of eight FP4 (E2M1) codes
// of +-1.0 for K-step s; V_CVT_SCALEF32_PK_BF16_FP4 expands them to packed bf16 +-1.0, two
// elements per instruction.
#include "common.h"

namespace qless {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kWaves = 8;
constexpr int kStageD = 128;                   // gradient columns per LDS stage
constexpr int kLdsStride = kStageD * 2 + 16;   // bytes per staged row (+16: conflict-free b128 reads)
// NB = 32-row blocks per workgroup tile (2 or 4); a wave owns NB x (8 / NB) accumulators
template <int NB> struct ProjShape {
    static_assert(NB == 2 || NB == 4, "64- or 128-row tiles");
    static constexpr int KB = 8 / NB;                   // 32-coordinate blocks per wave
    static constexpr int kTileRows = 32 * NB;           // batch rows per workgroup
    static constexpr int kWaveCols = 32 * KB;           // projected coordinates per wave
    static constexpr int kTileCols = kWaves * kWaveCols;   // 1024 or 512 per workgroup
    static constexpr int kStageBytes = kTileRows * kLdsStride;
    static constexpr int kDirectStageBytes = kTileRows * kStageD * 2;
};
// 128-row tiles for the Gaussian family (whose operand generation, one table look-up per element,
// is what bounds the kernel) when they cover the batch with no more padding rows than 64-row tiles
// would.  The Rademacher kernel gains nothing from them: it already runs at the matrix-core rate the
// chip sustains.
static int tile_row_blocks(int64_t n, bool gauss) {
    return (gauss && n > 64 && (n + 127) / 128 * 128 <= (n + 63) / 64 * 64) ? 4 : 2;
}

struct ProjectPlan {
    int64_t ntiles, ktiles, nsplit, stages_per_split, slices, grid;
    size_t ws_bytes;
};

static ProjectPlan make_plan(int64_t n, int64_t d_len, int32_t k, bool gauss) {
    ProjectPlan p{};
    const int nb = tile_row_blocks(n, gauss);
    const int kTileRows = 32 * nb, kTileCols = kWaves * 32 * (8 / nb);
    p.ntiles = (n + kTileRows - 1) / kTileRows;
    p.ktiles = (k + kTileCols - 1) / kTileCols;
    int64_t stages = (d_len + kStageD - 1) / kStageD;
    if (n <= 0 || d_len <= 0) { p.nsplit = 0; p.ws_bytes = 0; return p; }
    int64_t tiles = p.ntiles * p.ktiles;
    int64_t want = (2048 / kWaves + tiles - 1) / tiles;   // about eight waves per CU
    if (want > stages) want = stages;
    if (want < 1) want = 1;
    p.stages_per_split = (stages + want - 1) / want;
    p.nsplit = (stages + p.stages_per_split - 1) / p.stages_per_split;
    p.slices = p.ntiles * p.nsplit;
    p.grid = p.ktiles * 8 * ((p.slices + 7) / 8);
    p.ws_bytes = (size_t)p.nsplit * (size_t)n * (size_t)k * sizeof(float);
    return p;
}

struct ProjectArgs {
    const void *G;
    float *ws;
    int64_t n, d_len, ldG;
    uint32_t wbase;          // d_offset / 32
    int32_t k;
    SeedKeys sk;
    int32_t ktiles, nsplit;
    int64_t slices, stages_per_split;
};

struct GaussTable { uint16_t v[256]; };

__device__ inline uint32_t pack_bf16_rne(float a, float b) {
    uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
    ua += 0x7FFFu + ((ua >> 16) & 1u);
    ub += 0x7FFFu + ((ub >> 16) & 1u);
    return (ua >> 16) | (ub & 0xFFFF0000u);
}

// Loads 8 consecutive gradient elements (row, col..col+7) as packed bf16; elements outside
// [0, n) x [0, c_end) read as zero.
template <bool IN_F32, bool ALIGNED>
__device__ inline uint4 load_chunk(const ProjectArgs &a, int64_t row, int64_t col, int64_t c_end) {
    uint4 out = make_uint4(0, 0, 0, 0);
    if (row >= a.n || col >= c_end) return out;
    if (IN_F32) {
        const float *p = (const float *)a.G + row * a.ldG + col;
        float f[8];
        if (ALIGNED && col + 8 <= c_end) {
            float4 lo = *(const float4 *)p, hi = *(const float4 *)(p + 4);
            f[0] = lo.x; f[1] = lo.y; f[2] = lo.z; f[3] = lo.w;
            f[4] = hi.x; f[5] = hi.y; f[6] = hi.z; f[7] = hi.w;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = (col + e < c_end) ? p[e] : 0.0f;
        }
        out.x = pack_bf16_rne(f[0], f[1]); out.y = pack_bf16_rne(f[2], f[3]);
        out.z = pack_bf16_rne(f[4], f[5]); out.w = pack_bf16_rne(f[6], f[7]);
    } else {
        const uint16_t *p = (const uint16_t *)a.G + row * a.ldG + col;
        if (ALIGNED && col + 8 <= c_end) {
            out = *(const uint4 *)p;
        } else {
            uint32_t h[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) h[e] = (col + e < c_end) ? p[e] : 0u;
            out.x = h[0] | (h[1] << 16); out.y = h[2] | (h[3] << 16);
            out.z = h[4] | (h[5] << 16); out.w = h[6] | (h[7] << 16);
        }
    }
    return out;
}

union Frag { bf16x8 v; bf16x2 p[4]; uint4 u; uint32_t w[4]; uint16_t h[8]; };

// DIRECT: gradient tiles go global -> LDS asynchronously (no VGPR staging) into a ring of kRing
// unpadded, XOR-swizzled stage buffers, three stages ahead of the MFMAs.  It needs bf16 input,
// 16-byte aligned rows and a gradient length that is a multiple of the stage width; every other
// case stages through registers into two padded buffers.
constexpr int kRing = 4;
constexpr int kGaussCopies = 32;                // copies of the Gaussian table in LDS
constexpr int kProjectMaxLds = kRing * 128 * kStageD * 2 + 256 * kGaussCopies * 2;   // largest request of any shape (128-row tiles)

template <bool IN_F32, bool ALIGNED, bool GAUSS, bool DIRECT, int NB>
__global__ void __launch_bounds__(kWaves * 64, 2)
project_kernel(ProjectArgs a, GaussTable gt) {
    static_assert(!DIRECT || (!IN_F32 && ALIGNED), "direct LDS copies move bf16 rows as they are");
    using Sh = ProjShape<NB>;
    constexpr int KB = Sh::KB, kTileRows = Sh::kTileRows, kWaveCols = Sh::kWaveCols, kTileCols = Sh::kTileCols;
    constexpr int kStageBytes = Sh::kStageBytes, kDirectStageBytes = Sh::kDirectStageBytes;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // XCD-aware decode: consecutive workgroup ids land on different XCDs, so the ktiles
    // workgroups that share one gradient slice are given ids 8 apart (same XCD, same L2).
    const int64_t id = blockIdx.x;
    const int xcd = (int)(id & 7);
    const int64_t t = id >> 3;
    const int kt = (int)(t % a.ktiles);
    const int64_t slice = (t / a.ktiles) * 8 + xcd;
    if (slice >= a.slices) return;
    const int64_t ntile = slice / a.nsplit;
    const int split = (int)(slice % a.nsplit);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int64_t row0 = ntile * kTileRows;
    const int64_t c_begin = (int64_t)split * a.stages_per_split * kStageD;
    int64_t c_end = c_begin + a.stages_per_split * kStageD;
    if (c_end > a.d_len) c_end = a.d_len;
    const int nstages = (int)((c_end - c_begin + kStageD - 1) / kStageD);

    uint16_t *gtab = (uint16_t *)(smem + (DIRECT ? kRing * kDirectStageBytes : 2 * kStageBytes));
    // Gaussian table in LDS, 32 copies side by side: entry i for lane l at halfword 32 i + l % 32, so
    // the 32 lanes that look up together use 16 different banks whatever their indices are (a single
    // copy makes them collide on the 128 dwords of the table)
    if (GAUSS) {
        for (int i = tid; i < 256 * kGaussCopies; i += kWaves * 64) gtab[i] = gt.v[i / kGaussCopies];
    }

    // row keys of this lane's KB 32-row blocks of the random matrix
    const int mbase = kt * kTileCols + wave * kWaveCols;
    RowKey key[KB];
    bool live[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        int m = mbase + 32 * kb + l32;
        live[kb] = (mbase + 32 * kb) < a.k;            // wave-uniform (k is a multiple of 64)
        key[kb] = row_key(a.sk, (uint32_t)m);
        if (!GAUSS) key[kb].a += (uint32_t)half * kGold;   // upper half-wave reads the next word
    }

    f32x16 acc[NB][KB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[nb][kb][v] = 0.0f;

    // staging (register path): kTileRows rows x 16 chunks of 8 columns; thread handles chunks tid + kThreads*i
    constexpr int kThreads = kWaves * 64;
    constexpr int kChunksPerThread = kTileRows * (kStageD / 8) / kThreads;
    uint4 stage_regs[DIRECT ? 1 : kChunksPerThread];
    auto fetch = [&](int s) {
        const int64_t cs = c_begin + (int64_t)s * kStageD;
#pragma unroll
        for (int i = 0; i < kChunksPerThread; ++i) {
            int c = tid + kThreads * i;
            int r = c >> 4, cc = c & 15;
            stage_regs[DIRECT ? 0 : i] = load_chunk<IN_F32, ALIGNED>(a, row0 + r, cs + cc * 8, c_end);
        }
    };
    auto commit = [&](int buf) {
#pragma unroll
        for (int i = 0; i < kChunksPerThread; ++i) {
            int c = tid + kThreads * i;
            int r = c >> 4, cc = c & 15;
            *(uint4 *)(smem + buf * kStageBytes + r * kLdsStride + cc * 16) = stage_regs[DIRECT ? 0 : i];
        }
    };

    // staging (direct path): a stage is kTileRows rows x 256 bytes = 16 or 32 wavefront copies of 1 KB,
    // two or four per wave.  Copy q fills LDS chunks 64 q .. 64 q + 63 (rows 4 q .. 4 q + 3); chunk `pos` of row r
    // holds gradient chunk pos ^ (r & 15), so 16 consecutive rows read the same gradient chunk
    // from 16 different bank groups.  Rows past n re-read row n-1 (never stored).
    constexpr int kCopies = kDirectStageBytes / 1024 / kWaves;
    const unsigned char *cptr[kCopies];
    unsigned cdst[kCopies];
    const unsigned lds0 = (unsigned)(uintptr_t)((__attribute__((address_space(3))) unsigned char *)smem);
    const int uwave = __builtin_amdgcn_readfirstlane(wave);
    if (DIRECT) {
#pragma unroll
        for (int u = 0; u < kCopies; ++u) {
            const int q = uwave * kCopies + u;
            const int r = 4 * q + (lane >> 4), pos = lane & 15;
            int64_t grow = row0 + r;
            if (grow > a.n - 1) grow = a.n - 1;
            cptr[u] = (const unsigned char *)a.G + (grow * a.ldG + c_begin) * 2 + ((pos ^ (r & 15)) << 4);
            cdst[u] = (unsigned)q * 1024u;
        }
    }
    auto issue = [&](int s) {                      // start the copies of stage s (ring slot s % kRing)
        const unsigned buf = lds0 + (unsigned)(s % kRing) * kDirectStageBytes;
#pragma unroll
        for (int u = 0; u < kCopies; ++u) {
            global_to_lds16(cptr[u], buf + cdst[u]);
            cptr[u] += kStageD * 2;
        }
    };
    // A fragment (rows 32 nb + l32, columns 64 bp + 32 half + 8 ks .. +7) of the stage in `slot`
    const unsigned a_sw = (unsigned)(((4 * half) ^ (l32 & 15)) << 4);
    auto read_a = [&](int slot, int nb, int bp, int ks) -> uint4 {
        if (DIRECT)
            return *(const uint4 *)(smem + slot * kDirectStageBytes + (32 * nb + l32) * (kStageD * 2) +
                                    (a_sw ^ (unsigned)((8 * bp + ks) << 4)));
        return *(const uint4 *)(smem + slot * kStageBytes + (32 * nb + l32) * kLdsStride +
                                (64 * bp + 32 * half + 8 * ks) * 2);
    };

    if (DIRECT) {
#pragma unroll
        for (int s = 0; s < kRing - 1; ++s)
            if (s < nstages) issue(s);
    } else {
        fetch(0);
        commit(0);
        __syncthreads();
    }

    const uint16_t *gl = gtab + (lane & (kGaussCopies - 1));   // this lane's copy of the table
    uint32_t fp4_one = 0x22222222u;                // eight FP4 codes of +1.0
    asm volatile("" : "+v"(fp4_one));              // keep it in a vector register
    for (int s = 0; s < nstages; ++s) {
        const int buf = DIRECT ? s % kRing : (s & 1);
        if (DIRECT) {
            // stage s is the oldest copy group in flight; two younger ones may stay outstanding
            if (s + kRing - 2 < nstages) wait_vmcnt<(kRing - 2) * kCopies>(); else wait_vmcnt<0>();
            __syncthreads();                       // stage s visible to all waves; slot of stage s-1 free
            if (s + kRing - 1 < nstages) issue(s + kRing - 1);
        } else {
            if (s + 1 < nstages) fetch(s + 1);
        }
        const int64_t cs = c_begin + (int64_t)s * kStageD;       // multiple of 128
        const uint32_t wstage = a.wbase + (uint32_t)(cs >> 5);
#pragma unroll
        for (int bp = 0; bp < 2; ++bp) {
            // A fragments: rows 32*nb + l32, columns 64*bp + 32*half + 8*ks .. +7
            Frag af[NB][4];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    af[nb][ks].u = read_a(buf, nb, bp, ks);
            const uint32_t wpair = wstage + 2u * bp;             // word index of lanes 0..31
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                // row blocks past k (last k-tile only) are computed and dropped in the epilogue
                if (!GAUSS) {
                    const uint32_t h = key_word(key[kb], wpair * kGold);
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) {
                        // (h << ks) & 0x88888888 | 0x22222222 in two instructions: the fused and-or takes one
                        // literal only, so the second constant is held in a register
                        uint32_t x;
                        asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(x) : "v"(h << ks), "s"(0x88888888u), "v"(fp4_one));
                        Frag bf;
                        bf.p[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(x, 1.0f, 0);
                        bf.p[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(x, 1.0f, 1);
                        bf.p[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(x, 1.0f, 2);
                        bf.p[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(x, 1.0f, 3);
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb)
                            acc[nb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[nb][ks].v, bf.v, acc[nb][kb], 0, 0, 0);
                    }
                } else {
                    // Gaussian-like entries: 4 columns per word, one table byte per column
                    const uint32_t w4 = (wpair + (uint32_t)half) * 8u;   // word of column 32*(...)
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) {
                        const uint32_t h0 = key_word(key[kb], (w4 + 2u * ks) * kGold + kSaltStride);
                        const uint32_t h1 = key_word(key[kb], (w4 + 2u * ks + 1u) * kGold + kSaltStride);
                        Frag bf;
                        bf.h[0] = gl[(h0 & 0xFF) * kGaussCopies];         bf.h[1] = gl[((h0 >> 8) & 0xFF) * kGaussCopies];
                        bf.h[2] = gl[((h0 >> 16) & 0xFF) * kGaussCopies]; bf.h[3] = gl[(h0 >> 24) * kGaussCopies];
                        bf.h[4] = gl[(h1 & 0xFF) * kGaussCopies];         bf.h[5] = gl[((h1 >> 8) & 0xFF) * kGaussCopies];
                        bf.h[6] = gl[((h1 >> 16) & 0xFF) * kGaussCopies]; bf.h[7] = gl[(h1 >> 24) * kGaussCopies];
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb)
                            acc[nb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[nb][ks].v, bf.v, acc[nb][kb], 0, 0, 0);
                    }
                }
            }
        }
        if (!DIRECT) {
            if (s + 1 < nstages) commit(buf ^ 1);
            __syncthreads();
        }
    }

    // partial tile -> workspace [split][n][k];  D[i][j]: j = lane%32, i = 8*(v/4) + 4*(lane/32) + v%4
    float *wsp = a.ws + (size_t)split * (size_t)a.n * (size_t)a.k;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            if (!live[kb]) continue;
            const int m = mbase + 32 * kb + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = row0 + 32 * nb + 8 * (v >> 2) + 4 * half + (v & 3);
                if (row < a.n) wsp[(size_t)row * a.k + m] = acc[nb][kb][v];
            }
        }
}

// P = (accumulate ? P : 0) + ((p_0 + p_1) + p_2) + ...   fixed order over the d-slices
__global__ void __launch_bounds__(256)
project_reduce_kernel(const float *ws, int nsplit, int64_t n, int32_t k, int accumulate,
                      float *P, int64_t ldP) {
    const int64_t total = n * (int64_t)k;
    const size_t plane = (size_t)total;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        float s = 0.0f;
        for (int sp = 0; sp < nsplit; ++sp) s += ws[(size_t)sp * plane + (size_t)i];
        const int64_t row = i / k, m = i - row * k;
        float *dst = P + row * ldP + m;
        *dst = accumulate ? (*dst + s) : s;
    }
}

__global__ void generator_words_kernel(SeedKeys sk, uint32_t m0, int32_t nrows, uint32_t w0,
                                       int32_t nwords, uint32_t salt, uint32_t *out) {
    const int64_t total = (int64_t)nrows * nwords;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t r = (uint32_t)(i / nwords), t = (uint32_t)(i % nwords);
        out[i] = key_word(row_key(sk, m0 + r), (w0 + t) * kGold + salt * kSaltStride);
    }
}

}  // namespace qless

using namespace qless;

extern "C" size_t qless_project_workspace(int64_t n, int64_t d_len, int32_t k) {
    if (n <= 0 || d_len <= 0 || k <= 0) return 0;
    // enough for either matrix family (their tile shapes, hence their d-splits, may differ)
    const size_t r = make_plan(n, d_len, k, false).ws_bytes, g = make_plan(n, d_len, k, true).ws_bytes;
    return r > g ? r : g;
}

// Validates the projection arguments shared by both entry points and launches the split-d
// partial sums into ws ([nsplit][n][k]).  *nsplit_out = 0 when there is nothing to launch.
static qless_status project_partials(const void *G, qless_dtype dt, int64_t n, int64_t d_len, int64_t ldG,
                                     int64_t d_offset, int32_t k, qless_proj kind, uint64_t seed,
                                     void *ws, size_t ws_bytes, hipStream_t st, int *nsplit_out) {
    *nsplit_out = 0;
    if (n < 0 || d_len < 0 || d_offset < 0 || k <= 0 || ldG < d_len) return QLESS_ERR_INVALID_ARG;
    if (n > 0 && d_len > 0 && !G) return QLESS_ERR_INVALID_ARG;
    if (dt != QLESS_F32 && dt != QLESS_BF16) return QLESS_ERR_UNSUPPORTED;
    if (kind != QLESS_RADEMACHER && kind != QLESS_GAUSSIAN) return QLESS_ERR_UNSUPPORTED;
    if (k % 64 != 0 || d_offset % 32 != 0) return QLESS_ERR_UNSUPPORTED;
    if (d_offset + d_len > ((int64_t)1 << 36)) return QLESS_ERR_UNSUPPORTED;
    // the Gaussian stream numbers its words with 32 bits, four columns to a word
    if (kind == QLESS_GAUSSIAN && d_offset + d_len > ((int64_t)1 << 34)) return QLESS_ERR_UNSUPPORTED;
    if (n > ((int64_t)1 << 31)) return QLESS_ERR_UNSUPPORTED;
    if (n == 0) return QLESS_OK;
    ProjectPlan plan = make_plan(n, d_len, k, kind == QLESS_GAUSSIAN);
    if (plan.ws_bytes > 0 && (!ws || ws_bytes < plan.ws_bytes || (uintptr_t)ws % 16 != 0)) return QLESS_ERR_WORKSPACE;
    if (plan.grid > 0x7FFFFFFF) return QLESS_ERR_UNSUPPORTED;
    if (plan.nsplit == 0) return QLESS_OK;

    ProjectArgs a{};
    a.G = G; a.ws = (float *)ws; a.n = n; a.d_len = d_len; a.ldG = ldG;
    a.wbase = (uint32_t)(d_offset >> 5); a.k = k; a.sk = seed_keys(seed);
    a.ktiles = (int32_t)plan.ktiles; a.nsplit = (int32_t)plan.nsplit;
    a.slices = plan.slices; a.stages_per_split = plan.stages_per_split;
    GaussTable gt{};
    const bool gauss = kind == QLESS_GAUSSIAN;
    if (gauss) { const uint16_t *t = gaussian_table_bf16(); for (int i = 0; i < 256; ++i) gt.v[i] = t[i]; }
    const size_t esz = dt == QLESS_F32 ? 4 : 2;
    const bool aligned = ((uintptr_t)G % 16 == 0) && ((ldG * esz) % 16 == 0);
    const bool direct = dt == QLESS_BF16 && aligned && d_len % kStageD == 0;
    const int nb = tile_row_blocks(n, gauss);
    const size_t lds = (direct ? (size_t)kRing * (32 * nb) * kStageD * 2 : (size_t)2 * (32 * nb) * kLdsStride) +
                       (gauss ? (size_t)256 * kGaussCopies * 2 : 0);
    dim3 grid((unsigned)plan.grid), block(kWaves * 64);
    if (lds > (size_t)kProjectMaxLds) return QLESS_ERR_DEVICE;
    const qless_status ready = device_ready();     // more than 64 KB of dynamic LDS has to be allowed per kernel
    if (ready != QLESS_OK) return ready;
#define QLESS_LAUNCH_NB(F32, AL, GA, DI, NBLK) do { \
        QLESS_LDS_KERNEL((project_kernel<F32, AL, GA, DI, NBLK>), kProjectMaxLds); \
        hipLaunchKernelGGL((project_kernel<F32, AL, GA, DI, NBLK>), grid, block, lds, st, a, gt); } while (0)
#define QLESS_LAUNCH(F32, AL, GA, DI) do { \
        if (nb == 4) QLESS_LAUNCH_NB(F32, AL, GA, DI, 4); else QLESS_LAUNCH_NB(F32, AL, GA, DI, 2); } while (0)
    if (dt == QLESS_F32) {
        if (aligned) { if (gauss) QLESS_LAUNCH(true, true, true, false); else QLESS_LAUNCH(true, true, false, false); }
        else         { if (gauss) QLESS_LAUNCH(true, false, true, false); else QLESS_LAUNCH(true, false, false, false); }
    } else if (direct) {
        if (gauss) QLESS_LAUNCH(false, true, true, true); else QLESS_LAUNCH(false, true, false, true);
    } else {
        if (aligned) { if (gauss) QLESS_LAUNCH(false, true, true, false); else QLESS_LAUNCH(false, true, false, false); }
        else         { if (gauss) QLESS_LAUNCH(false, false, true, false); else QLESS_LAUNCH(false, false, false, false); }
    }
#undef QLESS_LAUNCH
#undef QLESS_LAUNCH_NB
    if (launch_status() != QLESS_OK) return QLESS_ERR_DEVICE;
    *nsplit_out = (int)plan.nsplit;
    return QLESS_OK;
}

extern "C" qless_status qless_project(const void *G, qless_dtype dt, int64_t n, int64_t d_len,
                                      int64_t ldG, int64_t d_offset, int32_t k, qless_proj kind,
                                      uint64_t seed, int accumulate, float *P, int64_t ldP,
                                      void *ws, size_t ws_bytes, void *stream) {
    if (ldP < k || (n > 0 && !P)) return QLESS_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    int nsplit = 0;
    const qless_status rc = project_partials(G, dt, n, d_len, ldG, d_offset, k, kind, seed, ws, ws_bytes,
                                             st, &nsplit);
    if (rc != QLESS_OK || n == 0) return rc;
    if (nsplit == 0 && accumulate) return QLESS_OK;       // nothing to add
    const int64_t total = n * (int64_t)k;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(project_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                       (const float *)ws, nsplit, n, k, accumulate, P, ldP);
    return launch_status();
}

extern "C" qless_status qless_project_quantize(const void *G, qless_dtype dt, int64_t n, int64_t d_len,
                                               int64_t ldG, int64_t d_offset, int32_t k, qless_proj kind,
                                               uint64_t seed, int bits, void *codes, float *S, float *rnorm,
                                               float *P, int64_t ldP, void *ws, size_t ws_bytes,
                                               void *stream) {
    if (d_len <= 0 || (P && ldP < k)) return QLESS_ERR_INVALID_ARG;
    if (n > 0 && (!codes || !S || !rnorm)) return QLESS_ERR_INVALID_ARG;
    if ((uintptr_t)codes % 4) return QLESS_ERR_INVALID_ARG;
    if (!valid_bits(bits)) return QLESS_ERR_UNSUPPORTED;
    if (ws && (uintptr_t)ws % 16 != 0) return QLESS_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    int nsplit = 0;
    const qless_status rc = project_partials(G, dt, n, d_len, ldG, d_offset, k, kind, seed, ws, ws_bytes,
                                             st, &nsplit);
    if (rc != QLESS_OK || n == 0) return rc;
    return quantize_rows((const float *)ws, k, nsplit, (size_t)n * (size_t)k, P, ldP, n, k, bits, codes, S,
                         rnorm, st);
}

// P = (accumulate ? P : 0) + other, element by element (joins two accumulators when the last slice is
// too long-rowed for the fused path)
__global__ void __launch_bounds__(256)
add_rows_kernel(float *P, int64_t ldP, const float *other, int64_t ldO, int64_t n, int32_t k) {
    const int64_t total = n * (int64_t)k;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = i / k, m = i - row * k;
        P[row * ldP + m] = P[row * ldP + m] + other[row * ldO + m];
    }
}

extern "C" qless_status qless_project_quantize_slice(const void *G, qless_dtype dt, int64_t n, int64_t d_len,
                                                     int64_t ldG, int64_t d_offset, int32_t k, qless_proj kind,
                                                     uint64_t seed, int first, int last, float *P, int64_t ldP,
                                                     const float *P_other, int64_t ldO, int bits, void *codes,
                                                     float *S, float *rnorm, void *ws, size_t ws_bytes,
                                                     void *stream) {
    if (ldP < k || (n > 0 && !P) || (P_other && ldO < k)) return QLESS_ERR_INVALID_ARG;
    if (P_other && !last) return QLESS_ERR_INVALID_ARG;
    if (last) {
        if (n > 0 && (!codes || !S || !rnorm)) return QLESS_ERR_INVALID_ARG;
        if ((uintptr_t)codes % 4) return QLESS_ERR_INVALID_ARG;
        if (!valid_bits(bits)) return QLESS_ERR_UNSUPPORTED;
    }
    hipStream_t st = (hipStream_t)stream;
    int nsplit = 0;
    const qless_status rc = project_partials(G, dt, n, d_len, ldG, d_offset, k, kind, seed, ws, ws_bytes,
                                             st, &nsplit);
    if (rc != QLESS_OK || n == 0) return rc;
    const int64_t total = n * (int64_t)k;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    // the last slice of rows that fit in registers: its partial sums, the accumulator and the second
    // accumulator are added by the quantiser itself, in the order of the separate kernels
    const bool fused = last && nsplit > 0 && k <= 16384;
    if (!fused) {
        if (nsplit > 0 || first)
            hipLaunchKernelGGL(project_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                               (const float *)ws, nsplit, n, k, first ? 0 : 1, P, ldP);
        if (!last) return launch_status();
        if (P_other)
            hipLaunchKernelGGL(add_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, st, P, ldP, P_other, ldO, n, k);
        return quantize_rows(P, ldP, 1, 0, nullptr, 0, n, k, bits, codes, S, rnorm, st);
    }
    return quantize_rows((const float *)ws, k, nsplit, (size_t)n * (size_t)k, P, ldP, n, k, bits, codes, S,
                         rnorm, st, first ? nullptr : P, ldP, P_other, ldO);
}

extern "C" qless_status qless_generator_words(uint64_t seed, uint32_t m0, int32_t nrows,
                                              uint32_t w0, int32_t nwords, uint32_t salt,
                                              uint32_t *out, void *stream) {
    if (nrows < 0 || nwords < 0 || (!out && nrows > 0 && nwords > 0)) return QLESS_ERR_INVALID_ARG;
    const int64_t total = (int64_t)nrows * nwords;
    if (total == 0) return QLESS_OK;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(generator_words_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       (hipStream_t)stream, seed_keys(seed), m0, nrows, w0, nwords, salt, out);
    return launch_status();
}
