// qless_score: influence of every train example on every validation example from the packed
// datastore (paper Eq.(6),(7), Sec. 3.2), summed over checkpoints with learning-rate weights and
// reduced by max over validation examples.
//
// Integer dot products are exact; how they are formed depends on the code width:
//   8-/4-bit: int8 x int8 -> int32 MFMA (v_mfma_i32_32x32x32_i8) on codes unpacked in registers
//   2-/1-bit: the codes {-1, 0, +1} are exactly representable as FP4 (E2M1) values; the scaled FP4
//           matrix-core instructions multiply them and sum in fp32, which is exact for these integers
//           (|D| <= k <= 65536 < 2^24): v_mfma_scale_f32_32x32x64_f8f6f4 in score_mfma_kernel, and for at
//           most 16 val vectors v_mfma_scale_f32_16x16x128_f8f6f4 in score_stream_mfma_kernel, which
//           streams the train codes once at the speed of HBM
//   2-/1-bit with k not a multiple of 128 (or val codes too large for LDS): popcounts,
//           1-bit D = k - 2 popcount(a ^ b),
//           2-bit D = popcount(nz_a & nz_b) - 2 popcount(nz_a & nz_b & (sg_a ^ sg_b))
// The fp32 epilogue is a fixed sequence of single operations (compiled without contraction):
//   acc += ((float)D * rnorm_train) * (eta * rnorm_val), checkpoints in order, starting from +0.
//
// The popcount kernels give a workgroup a block of train rows and walk it over all validation
// tiles with the running row maximum in registers; the MFMA kernel gives every (train tile, val
// tile) pair its own workgroup and combines the row maxima with an exact integer atomicMax.
#include "common.h"
#include <atomic>

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

constexpr int kStreamVal = 8;                  // bit-plane codes against at most this many val vectors never take the tile kernel (no workspace)

// ------------------------------------------------------------------------------------------
// Matrix-core kernel for all four code widths.
//
// A small pre-pass expands the validation codes of every checkpoint to int8 rows (8-/4-bit) or
// FP4 rows (2-/1-bit), padded to the tile size and in the K order in which the train operand is
// unpacked, together with w'[c][z'] = eta_c * rnorm'_c(z').  The main kernel runs one workgroup
// per (256 or 128 train rows) x (32 / 64 / 128 val rows) tile.  Train operands are unpacked in
// registers on their way from LDS to the MFMA:
//   8-bit  bytes as stored                                              v_mfma_i32_32x32x32_i8
//   4-bit  (w<<4)&0xF0F0F0F0 and w&0xF0F0F0F0: bytes 16 q (even / odd elements); acc = 16 D
//   1-bit  a lane's 32 signs w become four dwords of FP4 codes,         v_mfma_scale_f32_32x32x64_f8f6f4
//          dword j = ((w << j) & 0x88888888) | 0x22222222: 0x2 = +1.0, 0xA = -1.0 (nibble n <- bit 4n+3-j)
//   2-bit  likewise from the two planes: ((sg << j) & 0x88888888) | ((nz shifted by j-2) & 0x22222222):
//          0xA = -1.0, 0x0 = 0, 0x2 = +1.0
// (for 1-bit codes and at most 64 validation vectors the packed validation rows are staged as they are
// and expanded in registers as well).
// Operand stages travel global -> LDS asynchronously through a ring of 2-4 swizzled buffers.
// Workgroups of the same train tile get ids 8 apart, so they run on one XCD and share the train
// rows through its L2; the row maximum over val tiles is combined with an order-preserving
// integer atomicMax (exact, order independent) and decoded by a last small kernel.
// ------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(16))) int i32x16;

constexpr int kKE = 128;                       // code elements per pipeline stage (most shapes)
// ... of the shapes for few validation vectors (val tile 32 or 64 wide) and codes below 8 bits
constexpr int narrow_stage_elements(int bits, int vt) {
    return bits == 1 ? 512                               // sign codes: 64 bytes per train row and stage
         : bits == 2 ? 512                               // two planes of 64 bytes
                     : (bits == 8 ? kKE : 256);     // whole 128-byte lines of every train row per stage
}
constexpr int log2c(int x) { return x <= 1 ? 0 : 1 + log2c(x / 2); }

struct ScorePrep {                             // workspace views (device pointers)
    int8_t *vexp;                              // [C][Mp][kp]
    float *vw;                                 // [C][Mp]
    int32_t *vbias;                            // [C][Mp] sign codes on wide tiles: what the scaled validation codes leave to add to a dot product
    unsigned int *smax;                        // [N] order-preserving keys of the row maxima
    int32_t Mp, kp;                            // padded validation rows / elements per row
    int32_t vrow;                              // bytes per expanded validation row: kp, or kp / 2 for 1-bit (FP4 codes)
};

__device__ inline unsigned int f32_order_key(float f) {
    const unsigned int u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ inline float f32_from_order_key(unsigned int k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

// position p (0..kp) of an expanded val row -> element index of the code vector
template <int BITS>
__device__ inline int val_source_element(int p) {
    if (BITS == 8) return p;
    if (BITS == 4) {
        // inside a half K-step of 16: [0,2,4,6,1,3,5,7,8,10,12,14,9,11,13,15]
        const int i = p & 15, base = p & ~15;
        const int d = i >> 2, b = i & 3;               // dword d, byte b
        return base + 8 * (d >> 1) + 2 * b + (d & 1);
    }
    // FP4 codes (1- and 2-bit), stages of 512 elements = 16 words of 32 codes per row.  K step ks of a
    // stage (64 positions), half h: the train lane reads the 16-byte chunk 2 (ks / 4) + h and uses its
    // dword ks % 4, i.e. word 4 (2 (ks / 4) + h) + ks % 4 of the stage; FP4 dword j, nibble n of the
    // expansion is bit 4 n + 3 - j of that word.
    const int g = p >> 6, h = (p >> 5) & 1, j = (p >> 3) & 3, n = p & 7;
    const int stage = g >> 3, ks = g & 7;
    const int word = 16 * stage + 4 * (2 * (ks >> 2) + h) + (ks & 3);
    return 32 * word + 4 * n + 3 - j;
}

template <int BITS, bool F16 = false>        // F16: rows are bfloat16 bytes, no code norms (see score_mfma_kernel)
__global__ void __launch_bounds__(256)
score_prepare_kernel(ScoreArgs a, ScorePrep w) {
    const int row = blockIdx.x, ci = blockIdx.y;        // row < Mp
    int8_t *dst = w.vexp + ((size_t)ci * w.Mp + row) * (size_t)w.vrow;
    const bool live = row < a.M;
    const unsigned char *src = a.vc[ci] + (int64_t)(live ? row : 0) * ((int64_t)a.k * BITS / 8);
    if (BITS <= 2) {
        // two FP4 codes per byte: 0x2 = +1.0, 0xA = -1.0, 0x0 = 0 (2-bit zeros, and past the end of the
        // vector).  1-bit with few validation vectors (vrow == 0): the main kernel stages the packed codes itself.
        // 1-bit on wide tiles: the train side feeds FP4 dword jd of a word as the word's bits 4 n + 3 - jd
        // left in place (no shift), i.e. as 2 s, s, s / 2 for jd = 1, 2, 3 with s = 1 for a negative code
        // a = 1 - 2 s; the validation code b of such a position is stored as -b, -2 b, -4 b, so that every
        // product is -2 s b = a b - b, and the sum of b over these positions is added back after the
        // dot product (vbias).  jd = 0 keeps +-1 on both sides.
        int bias = 0;
        for (int bi = threadIdx.x; bi < w.vrow; bi += 256) {
            unsigned byte = 0;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int p = 2 * bi + e;
                const int m = val_source_element<BITS>(p);               // source elements past k: code 0
                if (live && m < a.k) {
                    unsigned nz = 1u, neg;
                    if (BITS == 2) {
                        nz = (src[m >> 3] >> (m & 7)) & 1u;
                        neg = (src[a.k / 8 + (m >> 3)] >> (m & 7)) & 1u;
                        // the train side leaves its "non-zero" bit of dwords 1, 2, 3 in place (FP4 2, 1, 1/2):
                        // the validation magnitudes are 1/2, 1, 2 there, so that every product is a b
                        const int jd = (p >> 3) & 3;
                        const unsigned mag = jd == 1 ? 0x1u : (jd == 3 ? 0x4u : 0x2u);
                        byte |= (nz ? (mag | (neg << 3)) : 0u) << (4 * e);
                    } else {
                        neg = (src[m >> 3] >> (m & 7)) & 1u;
                        const int jd = (p >> 3) & 3;
                        const unsigned mag = jd == 3 ? 0x6u : (jd == 2 ? 0x4u : 0x2u);     // 4.0, 2.0, 1.0
                        const unsigned sgn = jd == 0 ? neg : neg ^ 1u;
                        byte |= (mag | (sgn << 3)) << (4 * e);
                        if (jd != 0) bias += neg ? -1 : 1;
                    }
                }
            }
            dst[bi] = (int8_t)byte;
        }
        if (BITS == 1 && w.vrow > 0) {
            __shared__ int sh_bias;
            if (threadIdx.x == 0) sh_bias = 0;
            __syncthreads();
            if (bias) atomicAdd(&sh_bias, bias);
            __syncthreads();
            if (threadIdx.x == 0) w.vbias[ci * w.Mp + row] = sh_bias;
        }
    } else {
        for (int p = threadIdx.x; p < w.kp; p += 256) {
            int q = 0;
            if (live && p < a.k) {
                const int m = val_source_element<BITS>(p);
                if (BITS == 8) q = (int8_t)src[m];
                else { q = (src[m >> 1] >> (4 * (m & 1))) & 0xF; if (q & 8) q -= 16; }
            }
            dst[p] = (int8_t)q;
        }
    }
    if (threadIdx.x == 0)
        w.vw[ci * w.Mp + row] = live ? (F16 ? a.eta[ci] : __fmul_rn(a.eta[ci], a.vr[ci][row])) : 0.0f;
    // the row-maximum keys start below every finite score
    if (ci == 0) {
        const int64_t per = (a.N + gridDim.x - 1) / gridDim.x;
        const int64_t lo = (int64_t)row * per;
        for (int64_t i = lo + threadIdx.x; i < lo + per && i < a.N; i += 256) w.smax[i] = 0u;
    }
}

// also leaves the keys cleared, so that a later launch on the same workspace needs no pre-pass
__global__ void score_finish_kernel(unsigned int *smax, int64_t N, float *score) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N;
         i += (int64_t)gridDim.x * blockDim.x) {
        score[i] = f32_from_order_key(smax[i]);
        smax[i] = 0u;
    }
}

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
template <bool F16> struct AccType { typedef i32x16 type; };
template <> struct AccType<true> { typedef f32x16 type; };
template <bool F16>
__device__ inline typename AccType<F16>::type mfma_step(i32x4 a, i32x4 b, typename AccType<F16>::type c);
template <>
__device__ inline i32x16 mfma_step<false>(i32x4 a, i32x4 b, i32x16 c) {
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
}
typedef __attribute__((ext_vector_type(8))) int i32x8;
// (x & 0x88888888) | y in one instruction.  The fused and-or takes a single literal, so callers
// keep a constant y (0x22222222: eight FP4 codes of +1.0) in a vector register.
__device__ inline uint32_t sign_bits_or(uint32_t x, uint32_t y) {
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "s"(0x88888888u), "v"(y));
    return r;
}
__device__ inline uint32_t fp4_ones() {
    uint32_t one = 0x22222222u;
    asm volatile("" : "+v"(one));                // held in a vector register
    return one;
}
// 64 FP4 (E2M1) products per lane pair, both scales 2^0: the sign codes' dot products, exact in fp32
__device__ inline f32x16 mfma_fp4(i32x8 a, i32x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 4, 4, 0, 127, 0, 127);
}
template <>
__device__ inline f32x16 mfma_step<true>(i32x4 a, i32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// ------------------------------------------------------------------------------------------
// 1-bit / 2-bit codes against at most 16 validation vectors on the matrix cores: streaming kernel,
// bound by HBM.
//
// No barrier after the start: every wavefront streams its own contiguous row range through a
// private LDS ring of 4 KB slots filled by asynchronous 16-byte copies; the validation codes and
// weights of all checkpoints stay in LDS for the whole kernel.  The dot products are formed by
// v_mfma_scale_f32_16x16x128_f8f6f4 on FP4 operands expanded in registers (7 vector ALU operations
// per 32 one-bit codes of a train row, whatever the number of validation vectors; popcounts would
// need 2 per validation vector):
//   * a wavefront takes passes of up to 160 rows = 10 panels of 16 rows.  For every (checkpoint,
//     128-byte slice) it expands the validation fragments of that slice once (A operand: val row
//     lane % 16; lane group lane / 16 takes 16-byte chunks 4 c + lane / 16, c = 0, 1, of the slice)
//     and multiplies them with all panels of the pass (B operand: train row lane % 16, same chunks),
//     8 instructions per panel and slice.  Both operands use the same chunk -> K position map, so
//     the order of the K elements inside an instruction does not matter.
//   * a ring slot holds one slice of 32 / BITS rows (PPS = 2 / BITS panels): 1 KB copies of 8 rows
//     x 128 bytes (whole cache lines).  Copy lane (row rr = lane / 8, position lane % 8) fetches
//     chunk (lane % 8) ^ rr, so the 8 rows of a copy that are read together come from 8 different
//     bank groups.  The ring has as many slots as LDS allows, normally 3.
//   * accumulator register v of lane (row lane % 16, group lane / 16) belongs to validation vector
//     4 (lane / 16) + v; after the last slice of a checkpoint it goes through the fp32 epilogue.
// Chunks past the end of a plane (k / 8 not a multiple of 128 bytes) are zeroed on the validation
// side (FP4 code 0), so whatever the train copy fetched there contributes nothing.
// ------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) float f32x4;
constexpr int kStreamMfmaVal = 16;             // validation vectors the kernel handles
constexpr int kStreamPassRows = 160;           // train rows of one pass of a wavefront

// 32 codes (bit c of `sg`: negative; bit c of `nz`: non-zero, 2-bit codes only) -> four dwords of FP4
// codes; nibble n of dword j holds code 4 n + 3 - j (0x2 = +1.0, 0xA = -1.0, 0x0 = 0); ones = fp4_ones()
template <int BITS>
__device__ inline i32x8 fp4_codes(uint32_t sg, uint32_t nz, uint32_t ones) {
    i32x8 r = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t mag = BITS == 1 ? ones : ((j >= 2 ? nz << (j - 2) : nz >> (2 - j)) & 0x22222222u);
        r[j] = (int)sign_bits_or(sg << j, mag);
    }
    return r;
}

// The ternary codes of the streaming kernel: the train side leaves the "non-zero" bit of dwords 1 .. 3 where
// it is (FP4 magnitudes 2, 1, 1/2; 12 operations per 32 codes instead of 14), the validation side takes
// the magnitudes 1/2, 1, 2 there, so that every product is the product of the codes.
__device__ inline i32x8 fp4_codes2_train(uint32_t sg, uint32_t nz) {
    i32x8 r = {0, 0, 0, 0, 0, 0, 0, 0};
    r[0] = (int)sign_bits_or(sg, (nz >> 2) & 0x22222222u);
    r[1] = (int)sign_bits_or(sg << 1, nz & 0x44444444u);
    r[2] = (int)sign_bits_or(sg << 2, nz & 0x22222222u);
    r[3] = (int)sign_bits_or(sg << 3, nz & 0x11111111u);
    return r;
}
__device__ inline i32x8 fp4_codes2_val(uint32_t sg, uint32_t nz) {
    i32x8 r = {0, 0, 0, 0, 0, 0, 0, 0};
    r[0] = (int)sign_bits_or(sg, (nz >> 2) & 0x22222222u);
    r[1] = (int)sign_bits_or(sg << 1, (nz >> 2) & 0x11111111u);
    r[2] = (int)sign_bits_or(sg << 2, nz & 0x22222222u);
    r[3] = (int)sign_bits_or(sg << 3, (nz << 2) & 0x44444444u);
    return r;
}

// blocks until at most n (wave-uniform, even, <= 14) vector memory operations are outstanding
__device__ inline void wait_vmcnt_even(int n) {
    switch (n) {
    case 0: wait_vmcnt<0>(); break;
    case 2: wait_vmcnt<2>(); break;
    case 4: wait_vmcnt<4>(); break;
    case 6: wait_vmcnt<6>(); break;
    case 8: wait_vmcnt<8>(); break;
    case 10: wait_vmcnt<10>(); break;
    case 12: wait_vmcnt<12>(); break;
    case 14: wait_vmcnt<14>(); break;
    default: wait_vmcnt<0>(); break;
    }
}

// MV = 8 or 16 validation rows held in LDS (M <= MV); NW wavefronts per workgroup, one workgroup per compute unit.
// A launch covers the checkpoints c0 .. c1 - 1 (all of them when their validation rows fit in LDS next
// to the rings; else groups of cg, one launch each): a launch that does not start at checkpoint 0
// continues from the fp32 sums the launch before left in `partial` ([N][16]), one that does not end
// at the last checkpoint leaves its sums there, so the order of the additions is that of one launch.
template <int BITS, int MV, int NW, int PPS>
__global__ void __launch_bounds__(64 * NW, NW / 4)
score_stream_mfma_kernel(ScoreArgs a, int64_t rb_each, int64_t rb_extra, int nb, unsigned ring_off,
                         int c0, int c1, int cg, float *partial) {
    constexpr int NPL = BITS;                   // bit planes per row
    constexpr int L = 2 * NPL * PPS;            // 1 KB copies per ring slot (PPS panels, one slice)
    constexpr int SLOT = L * 1024;
    constexpr int PASS = kStreamPassRows * 8 / NW;   // rows of a pass: fewer with more wavefronts (registers)
    constexpr int NP = PASS / 16;               // panels per pass
    static_assert(NP % PPS == 0, "whole ring slots per pass");
    // LDS: [C][MV] validation rows of cb + 16 bytes | [C][MV] weights | per wave a ring of nb slots
    extern __shared__ __attribute__((aligned(16))) unsigned char vlds[];
    const int lane = threadIdx.x & 63;
    const int cgp = lane & 7, crr = lane >> 3; // copy role: position and row inside a 1 KB copy
    const int l16 = lane & 15, kg = lane >> 4; // matrix role: row of the panel and chunk group
    const int wv_id = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // The train rows are dealt out evenly, to the row: wavefront w takes rb_each rows, the first rb_extra
    // wavefronts one more; w counts across workgroups first, so every compute unit gets its share
    // of the longer ranges
    const int64_t wave = (int64_t)wv_id * gridDim.x + blockIdx.x;
    const int64_t rb0 = wave * rb_each + (wave < rb_extra ? wave : rb_extra);
    const int64_t rb1 = rb0 + rb_each + (wave < rb_extra ? 1 : 0);
    const int cb = a.k * BITS / 8;              // bytes per row
    const int plane = a.k / 8;                  // bytes per bit plane, a multiple of 16 here
    const int nsl = (plane + 127) / 128;        // 128-byte slices per plane
    const int vstride = cb + 16;                // rows 4 banks apart: 8 rows read together do not collide
    const float *wlds = (const float *)(vlds + (size_t)cg * MV * vstride);
    unsigned char *ring = vlds + ring_off + (size_t)wv_id * nb * SLOT;
    const unsigned ring_lds = (unsigned)(uintptr_t)((__attribute__((address_space(3))) unsigned char *)ring);

    // validation codes and weights eta * rnorm' of every checkpoint -> LDS (rows past M repeat the
    // last one; they are masked at the output)
    {
        // four loads in flight per thread and round (the rounds are few: a round trip to L2 each)
        const int per_row = cb / 16, total = (c1 - c0) * MV * per_row;
        constexpr int kU = 4, kStep = 64 * NW;
        for (int i0 = threadIdx.x; i0 < total; i0 += kU * kStep) {
            uint4 val[kU];
            int dst[kU];
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                const int i = i0 + u * kStep < total ? i0 + u * kStep : total - 1;
                const int c16 = i % per_row, rowi = i / per_row, j = rowi % MV, ci = c0 + rowi / MV;
                const int jc = j < a.M ? j : a.M - 1;
                val[u] = *(const uint4 *)(a.vc[ci] + (int64_t)jc * cb + c16 * 16);
                dst[u] = rowi * vstride + c16 * 16;
            }
#pragma unroll
            for (int u = 0; u < kU; ++u)
                if (i0 + u * kStep < total) *(uint4 *)(vlds + dst[u]) = val[u];
        }
        float *wdst = (float *)(vlds + (size_t)cg * MV * vstride);
        for (int i = threadIdx.x; i < (c1 - c0) * MV; i += 64 * NW) {
            const int j = i % MV, ci = c0 + i / MV;
            wdst[i] = __fmul_rn(a.eta[ci], a.vr[ci][j < a.M ? j : a.M - 1]);
        }
        __syncthreads();
    }
    const int64_t r_end = rb1;
    const uint32_t ones = fp4_ones();

    for (int64_t rp = rb0; rp < r_end; rp += PASS) {              // wave-uniform loops
        const int rows = r_end - rp < PASS ? (int)(r_end - rp) : PASS;
        const int np = (rows + 15) / 16;
        const int ns = (np + PPS - 1) / PPS;     // ring slots per slice
        const int T = (c1 - c0) * nsl * ns;      // ring slots the pass consumes
        const int last = rows - 1;
        // producer state: the next slot to request is (f_ci, f_sl, f_p) into ring position f_pos
        int f_ci = c0, f_sl = 0, f_p = 0, f_pos = 0, f_it = 0;
        auto fetch = [&]() {
            int off = f_sl * 128 + ((cgp ^ crr) << 4);
            if (off >= plane) off = plane - 16;                              // zeroed on the validation side
            const unsigned char *base = a.tc[f_ci] + rp * cb;               // wave-uniform
            const unsigned slot = ring_lds + (unsigned)f_pos * (unsigned)SLOT;
#pragma unroll
            for (int b = 0; b < 2 * PPS; ++b) {
                int rl = f_p * (16 * PPS) + b * 8 + crr;
                if (rl > last) rl = last;                                    // clamped; masked at the output
#pragma unroll
                for (int q = 0; q < NPL; ++q)
                    global_to_lds16(base, (unsigned)(rl * cb + q * plane + off), slot + (unsigned)(b * NPL + q) * 1024u);
            }
            ++f_it;
            if (++f_pos == nb) f_pos = 0;
            if (++f_p == ns) { f_p = 0; if (++f_sl == nsl) { f_sl = 0; ++f_ci; } }
        };
        f32x4 acc[NP];
        float facc[NP][4];
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int v = 0; v < 4; ++v) { acc[p][v] = 0.0f; facc[p][v] = 0.0f; }
        if (c0 > 0) {                            // continue from the sums of the checkpoints before
#pragma unroll
            for (int p = 0; p < NP; ++p)
                if (p < np && p * 16 + l16 < rows) {
                    const float4 pv = *(const float4 *)(partial + (rp + p * 16 + l16) * 16 + 4 * kg);
                    facc[p][0] = pv.x; facc[p][1] = pv.y; facc[p][2] = pv.z; facc[p][3] = pv.w;
                }
            // the loads are awaited here, before the first ring copies: a wait for them later would drain the ring
#pragma unroll
            for (int p = 0; p < NP; ++p) asm volatile("" : "+v"(facc[p][0]), "+v"(facc[p][1]), "+v"(facc[p][2]), "+v"(facc[p][3]));
        }

        for (int i = 0; i < nb - 1 && i < T; ++i) fetch();
        int it = 0, pos = 0;
        for (int ci = c0; ci < c1; ++ci) {
            for (int sl = 0; sl < nsl; ++sl) {
                // validation fragments of this slice: 8 K steps (2 chunks x 4 dwords) of 4 FP4 dwords
                i32x8 vf[8];
                {
                    const unsigned char *vrow = vlds + (size_t)((ci - c0) * MV + (l16 & (MV - 1))) * vstride;
#pragma unroll
                    for (int c2 = 0; c2 < 2; ++c2) {
                        const int off = sl * 128 + (4 * c2 + kg) * 16;
                        const bool inside = off < plane;
                        const int offc = inside ? off : 0;
                        const uint4 sg = *(const uint4 *)(vrow + (NPL - 1) * plane + offc);
                        const uint4 nz = BITS == 2 ? *(const uint4 *)(vrow + offc) : sg;
                        vf[4 * c2 + 0] = BITS == 2 ? fp4_codes2_val(sg.x, nz.x) : fp4_codes<BITS>(sg.x, nz.x, ones);
                        vf[4 * c2 + 1] = BITS == 2 ? fp4_codes2_val(sg.y, nz.y) : fp4_codes<BITS>(sg.y, nz.y, ones);
                        vf[4 * c2 + 2] = BITS == 2 ? fp4_codes2_val(sg.z, nz.z) : fp4_codes<BITS>(sg.z, nz.z, ones);
                        vf[4 * c2 + 3] = BITS == 2 ? fp4_codes2_val(sg.w, nz.w) : fp4_codes<BITS>(sg.w, nz.w, ones);
                        if (sl * 128 + 128 > plane) {                        // wave-uniform: last, partial slice
                            const int keep = inside ? -1 : 0;
#pragma unroll
                            for (int e = 0; e < 4; ++e)
#pragma unroll
                                for (int j = 0; j < 4; ++j) vf[4 * c2 + e][j] &= keep;
                        }
                    }
                }
#pragma unroll
                for (int g = 0; g < NP / PPS; ++g) {
                    if (g < ns) {
                        // copies issued after this slot's: nb - 2 more slots, fewer at the end of the pass
                        const int younger = T - 1 - it < nb - 2 ? T - 1 - it : nb - 2;
                        wait_vmcnt_even(L * younger);
                        // the slot of step it - 1 is free: this wave's reads of it were consumed there
                        if (f_it < T) fetch();
                        const int rr = l16 & 7;
                        const unsigned char *rowp = ring + (size_t)pos * SLOT + (size_t)((l16 >> 3) * NPL) * 1024 + rr * 128;
                        uint4 sgv[PPS][2], nzv[PPS][2];
#pragma unroll
                        for (int h = 0; h < PPS; ++h)
#pragma unroll
                            for (int c2 = 0; c2 < 2; ++c2) {
                                const int chunk = ((4 * c2 + kg) ^ rr) << 4;
                                sgv[h][c2] = *(const uint4 *)(rowp + (2 * h * NPL + NPL - 1) * 1024 + chunk);
                                nzv[h][c2] = BITS == 2 ? *(const uint4 *)(rowp + 2 * h * NPL * 1024 + chunk) : sgv[h][c2];
                            }
#pragma unroll
                        for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                            for (int e = 0; e < 4; ++e)
#pragma unroll
                                for (int h = 0; h < PPS; ++h) {
                                    const uint4 sg = sgv[h][c2], nz = nzv[h][c2];
                                    const uint32_t sw = e == 0 ? sg.x : e == 1 ? sg.y : e == 2 ? sg.z : sg.w;
                                    const uint32_t nw = e == 0 ? nz.x : e == 1 ? nz.y : e == 2 ? nz.z : nz.w;
                                    acc[g * PPS + h] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                                        vf[4 * c2 + e], BITS == 2 ? fp4_codes2_train(sw, nw) : fp4_codes<BITS>(sw, nw, ones),
                                        acc[g * PPS + h], 4, 4, 0, 127, 0, 127);
                                }
                        ++it;
                        if (++pos == nb) pos = 0;
                    }
                }
            }
            // checkpoint epilogue
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                if (p < np) {
                    const float rt = a.tr[ci][rp + (p * 16 + l16 < rows ? p * 16 + l16 : last)];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float wv = wlds[(ci - c0) * MV + ((4 * kg + v) & (MV - 1))];
                        const float t = __fmul_rn(__fmul_rn(acc[p][v], rt), wv);      // acc holds the integer D exactly
                        facc[p][v] = __fadd_rn(facc[p][v], t);
                        acc[p][v] = 0.0f;
                    }
                }
            }
        }
        // outputs: lane (row, group kg) holds validation vectors 4 kg .. 4 kg + 3
        if (c1 < a.C) {                          // more checkpoints follow: leave the sums for the next launch
#pragma unroll
            for (int p = 0; p < NP; ++p)
                if (p < np && p * 16 + l16 < rows)
                    *(float4 *)(partial + (rp + p * 16 + l16) * 16 + 4 * kg) = float4{facc[p][0], facc[p][1], facc[p][2], facc[p][3]};
            continue;
        }
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            if (p < np) {
                const bool live = p * 16 + l16 < rows;
                const int64_t r = rp + p * 16 + l16;
                float m = neg_inf();
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int j = 4 * kg + v;
                    if (j < a.M) {
                        m = fmaxf(m, facc[p][v]);
                        if (a.full && live) a.full[r * a.M + j] = facc[p][v];
                    }
                }
                m = fmaxf(m, __shfl_xor(m, 16));
                m = fmaxf(m, __shfl_xor(m, 32));
                if (a.score && live && kg == 0) a.score[r] = m;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// 1-bit codes against a chunk of up to 64 validation vectors: the train rows are streamed as above,
// the products are 32 x 32 x 64 FP4 instructions.
//
// A wavefront works on tiles of 64 train rows (two panels of 32) x 64 validation vectors (two blocks
// of 32): per 64-element K step it expands one word of each panel and block (2 x 6 + 2 x 4 vector ALU
// operations, the bits of both operands left in place: see fp4_train_in_place) for 4 matrix-core instructions.
// The per-checkpoint sums of the tile stay in registers, so a wavefront walks its rows in passes
// of up to 64; the wavefronts of a workgroup have equally many passes.
//   * Train rows: a private ring per wavefront; a slot is a 64-byte slice of the 64 rows (four 1 KB
//     copies of 16 rows x 64 bytes, chunk (lane % 4) ^ ((row / 2) % 4) at position lane % 4, so that 8
//     rows read together use all banks).  The ring runs through all passes without a break.
//   * Validation rows (for the sign codes the pre-pass's copy with bits 0 and 2 of every nibble
//     swapped): all of them do not fit in LDS next to the rings, so the workgroup keeps a
//     window of WB bytes of every row of one checkpoint, double buffered.  The windows follow each
//     other in "phases" (pass, checkpoint, window).  The window of phase g + 1 is copied
//     asynchronously during phase g, each wavefront its share; before the one barrier per phase a
//     wavefront waits for its own share only (vector memory operations complete in order, so it
//     waits until at most the ring copies it issued later are outstanding: nothing is drained).
//     Rows are WB bytes apart, chunk c of row r at position c ^ (r % 8).
//   * Lane (row l, half h) takes chunks 2 c + h, c = 0, 1, of a slice on both operands; dword j of
//     a chunk is K step 4 c + j.
// More than 64 validation vectors are handled by one launch per chunk of 64 (the train codes are
// streamed again), later launches combining their row maxima with the score already there.
// ------------------------------------------------------------------------------------------
constexpr int kStream32Val = 64;               // validation vectors per launch
constexpr int kStream32Waves = 8;

__device__ inline void wait_vmcnt_upto(int n) {    // n wave-uniform, 0 <= n; waits for less when n > 24
    switch (n) {
    case 0: wait_vmcnt<0>(); break;   case 1: wait_vmcnt<1>(); break;   case 2: wait_vmcnt<2>(); break;
    case 3: wait_vmcnt<3>(); break;   case 4: wait_vmcnt<4>(); break;   case 5: wait_vmcnt<5>(); break;
    case 6: wait_vmcnt<6>(); break;   case 7: wait_vmcnt<7>(); break;   case 8: wait_vmcnt<8>(); break;
    case 9: wait_vmcnt<9>(); break;   case 10: wait_vmcnt<10>(); break; case 11: wait_vmcnt<11>(); break;
    case 12: wait_vmcnt<12>(); break; case 13: wait_vmcnt<13>(); break; case 14: wait_vmcnt<14>(); break;
    case 15: wait_vmcnt<15>(); break; case 16: wait_vmcnt<16>(); break; case 17: wait_vmcnt<17>(); break;
    case 18: wait_vmcnt<18>(); break; case 19: wait_vmcnt<19>(); break; case 20: wait_vmcnt<20>(); break;
    case 21: wait_vmcnt<21>(); break; case 22: wait_vmcnt<22>(); break; case 23: wait_vmcnt<23>(); break;
    default: wait_vmcnt<24>(); break;
    }
}

// Sign codes with the bits of both operands left where they are (no shifts).  A word's bit 4 n + 3 - jd
// feeds dword jd, nibble n of the FP4 operand; as FP4 codes the four nibble bits weigh -, 2, 1, 1/2, so
//   train word w:                 (w & 0x88888888) | 0x11111111 = +-1/2,   w & 0x44444444 = 2 s,   w & 0x22222222 = s,   w & 0x11111111 = s / 2
//   validation word w'' (a copy   (w'' & 0x88888888) | 0x11111111 = +-1/2, w'' & 0x11111111 = s'/2, w'' & 0x22222222 = s', w'' & 0x44444444 = 2 s'
//   with bits 0 and 2 of every nibble swapped by the pre-pass, so that dword jd holds the same codes):
// with s = 1 for a negative code a = 1 - 2 s.  Dword 0 multiplies to a b / 4, the others to s s', and
//   D = sum a b = 4 acc + 3 k / 4 - 2 St - 2 Sv,   St, Sv = the number of negative codes of a row outside dword 0
// (a b = 1 - 2 s - 2 s' + 4 s s').  All partial sums are multiples of 1/4 below k: exact in fp32.  St is
// counted here (two operations per word), Sv by the pre-pass: ten vector-ALU operations per pair of
// words instead of fourteen.
__device__ inline i32x8 fp4_train_in_place(uint32_t w, uint32_t halves) {
    i32x8 r = {0, 0, 0, 0, 0, 0, 0, 0};
    r[0] = (int)sign_bits_or(w, halves);
    r[1] = (int)(w & 0x44444444u); r[2] = (int)(w & 0x22222222u); r[3] = (int)(w & 0x11111111u);
    return r;
}
__device__ inline i32x8 fp4_val_in_place(uint32_t w, uint32_t halves) {
    i32x8 r = {0, 0, 0, 0, 0, 0, 0, 0};
    r[0] = (int)sign_bits_or(w, halves);
    r[1] = (int)(w & 0x11111111u); r[2] = (int)(w & 0x22222222u); r[3] = (int)(w & 0x44444444u);
    return r;
}
__device__ inline uint32_t fp4_halves() {
    uint32_t h = 0x11111111u;                    // eight FP4 codes of +0.5
    asm volatile("" : "+v"(h));                  // held in a vector register
    return h;
}

// One ring slot (64-byte slice of NPAN panels of 32 train rows) against VB blocks of 32 validation
// rows: 8 K steps.  sb: the slot; vwin: the validation window (bit-permuted copy); vcol: chunk index of
// the slice's first chunk inside the window; wb: bytes per window row; cnt: per panel, this lane's count
// of negative train codes outside dword 0.
template <int VB, int NPAN, int NPMAX>
__device__ inline void stream32_slice(const unsigned char *sb, const unsigned char *vwin, int vcol, int wb,
                                      int l32, int half, uint32_t halves, f32x16 (&acc)[NPMAX][VB], uint32_t (&cnt)[NPMAX]) {
    // K step ks = 4 c + j uses dword j of chunk 2 c + half.  The operands of step ks + 1 are expanded
    // between the matrix-core instructions of step ks (one instruction, then one operand's vector
    // ALU operations; scheduling barriers keep that order), so the matrix pipe is not left waiting
    // for a burst of expansions and the vector ALU is not blocked behind queued matrix instructions.
    uint4 tw[2][NPAN], vw[2][VB];
    auto load_words = [&](int c) {
        const int chunk = 2 * c + half;
#pragma unroll
        for (int p = 0; p < NPAN; ++p) {
            const int r = 32 * p + l32, rr = r & 15;
            tw[c][p] = *(const uint4 *)(sb + (r >> 4) * 1024 + rr * 64 + ((chunk ^ ((rr >> 1) & 3)) << 4));
        }
#pragma unroll
        for (int vb = 0; vb < VB; ++vb)
            vw[c][vb] = *(const uint4 *)(vwin + (size_t)(32 * vb + l32) * wb + (((vcol + chunk) ^ (l32 & 7)) << 4));
    };
    auto word = [](const uint4 &w, int j) { return j == 0 ? w.x : j == 1 ? w.y : j == 2 ? w.z : w.w; };
    auto train = [&](int c, int p, int j) {
        const uint32_t w = word(tw[c][p], j);
        cnt[p] += (uint32_t)__popc(w & 0x77777777u);
        return fp4_train_in_place(w, halves);
    };
    load_words(0);
    i32x8 tv[NPAN], vv[VB];
#pragma unroll
    for (int vb = 0; vb < VB; ++vb) vv[vb] = fp4_val_in_place(word(vw[0][vb], 0), halves);
#pragma unroll
    for (int p = 0; p < NPAN; ++p) tv[p] = train(0, p, 0);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        if (ks == 1) load_words(1);
        const int cn = (ks + 1) >> 2, jn = (ks + 1) & 3;       // next step's chunk and dword
        i32x8 tvn[NPAN], vvn[VB];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int p = 0; p < NPAN; ++p)
#pragma unroll
            for (int vb = 0; vb < VB; ++vb) {
                acc[p][vb] = mfma_fp4(vv[vb], tv[p], acc[p][vb]);
                const int slot = p * VB + vb;                   // this instruction's share of the expansions
                if (ks < 7) {
                    if (slot < VB) vvn[slot] = fp4_val_in_place(word(vw[cn][slot], jn), halves);
                    else if (slot < VB + NPAN) tvn[slot - VB] = train(cn, slot - VB, jn);
                    if (NPAN * VB < NPAN + VB && slot == NPAN * VB - 1) {   // fewer instructions than operands
#pragma unroll
                        for (int e = NPAN * VB; e < NPAN + VB; ++e) {
                            if (e < VB) vvn[e] = fp4_val_in_place(word(vw[cn][e], jn), halves);
                            else tvn[e - VB] = train(cn, e - VB, jn);
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        if (ks < 7) {
#pragma unroll
            for (int vb = 0; vb < VB; ++vb) vv[vb] = vvn[vb];
#pragma unroll
            for (int p = 0; p < NPAN; ++p) tv[p] = tvn[p];
        }
    }
}

// The same slot for 4- or 8-bit codes on the int8 matrix cores (v_mfma_i32_32x32x32_i8, 32 codes per
// instruction).  8 bits: a lane's 16-byte chunk 2 c + half is one K step of both operands.  4 bits:
// the chunk holds 32 train codes = two K steps; dwords 2 j, 2 j + 1 are unpacked as 16 q (bytes
// (w << 4) & 0xF0.. and w & 0xF0..: the even, then the odd nibbles), and the validation rows come
// int8-expanded in that order from the pre-pass (16 bytes per K step), so the accumulator holds 16 D.
template <int BITS, int VB, int VR, int NPAN, int NPMAX>
__device__ inline void stream32_slice_i8(const unsigned char *sb, const unsigned char *vwin, int slice, int wbv,
                                         int l32, int half, i32x16 (&acc)[NPMAX][VB]) {
    const int lv = VR < 32 ? (l32 & (VR - 1)) : l32;       // staged validation row of this lane (block 0)
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int chunk = 2 * c + half;
        i32x4 tw[NPAN];
#pragma unroll
        for (int p = 0; p < NPAN; ++p) {
            // the third panel has 16 staged rows: its lanes 16..31 re-read them (masked results)
            const int r = p == 2 ? 64 + (l32 & 15) : 32 * p + l32, rr = r & 15;
            tw[p] = *(const i32x4 *)(sb + (r >> 4) * 1024 + rr * 64 + ((chunk ^ ((rr >> 1) & 3)) << 4));
        }
        constexpr int STEPS = BITS == 4 ? 2 : 1;            // K steps per chunk
#pragma unroll
        for (int j = 0; j < STEPS; ++j) {
            const int vchunk = (BITS == 4 ? 8 * slice + 2 * chunk + j : 4 * slice + chunk);
            i32x4 vv[VB];
#pragma unroll
            for (int vb = 0; vb < VB; ++vb)
                vv[vb] = *(const i32x4 *)(vwin + (size_t)(32 * vb + lv) * wbv + ((vchunk ^ (lv & 7)) << 4));
#pragma unroll
            for (int p = 0; p < NPAN; ++p) {
                i32x4 tv;
                if (BITS == 8) {
                    tv = tw[p];
                } else {
                    const unsigned int px = (unsigned int)tw[p][2 * j], py = (unsigned int)tw[p][2 * j + 1];
                    tv[0] = (int)((px << 4) & 0xF0F0F0F0u); tv[1] = (int)(px & 0xF0F0F0F0u);
                    tv[2] = (int)((py << 4) & 0xF0F0F0F0u); tv[3] = (int)(py & 0xF0F0F0F0u);
                }
#pragma unroll
                for (int vb = 0; vb < VB; ++vb) acc[p][vb] = mfma_step<false>(vv[vb], tv, acc[p][vb]);
            }
        }
    }
}

// BITS = 1 (FP4 products), 4 or 8 (int8 products).  VB = 1 or 2 validation blocks of 32 (chunk of
// mc <= 32 VB vectors starting at m0); VR validation rows are staged (8, 16 or 32 VB: lanes past VR
// re-read the staged rows, their results are masked).  wb: train bytes per window, a power of two
// >= 128 that divides the row; the validation window of the same codes is wbv bytes per row (twice
// wb for the int8-expanded rows `vexp` of the 4-bit codes, else wb bytes of the codes themselves).
// npass: passes of the longest row range (workgroup-uniform)
template <int BITS, int VB, int VR>
__global__ void __launch_bounds__(64 * kStream32Waves, 2)
score_stream_mfma32_kernel(ScoreArgs a, const int8_t *vexp, const int32_t *vsum, int32_t Mp, int32_t vrow, int32_t m0, int32_t mc,
                           int64_t rb_each, int64_t rb_extra, int unit, int npass, int wb, int nb, unsigned ring_off) {
    static_assert(VR == 32 * VB || (VB == 1 && (VR == 8 || VR == 16)), "staged validation rows");
    constexpr int NW = kStream32Waves;
    // Rows of a pass: two panels of 32; the int8 shapes with one validation block have registers for
    // a third panel of 16 rows, which saves a whole pass over K when a wavefront's range is a little
    // more than two tiles (136 rows of 270 000 on 2048 wavefronts).
    // (the sign codes with one validation block take three full panels: 132 rows are then two passes, not three)
    constexpr int NPMAX = VB == 1 ? 3 : 2;
    constexpr int PASS = NPMAX == 3 ? (BITS == 1 ? 96 : 80) : 64;
    constexpr int NQ = PASS / 16;               // 1 KB copies per slot
    constexpr int SLOT = NQ * 1024;             // PASS rows x 64 bytes
    // LDS: 2 x [VR][wbv] validation windows | [C][32 VB] weights | rings
    extern __shared__ __attribute__((aligned(16))) unsigned char vlds[];
    const int lane = threadIdx.x & 63;
    const int cpos = lane & 3, crow = lane >> 2;   // copy role: position and row inside a 1 KB copy
    const int l32 = lane & 31, half = lane >> 5;   // matrix role
    const int wv_id = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t wave = (int64_t)wv_id * gridDim.x + blockIdx.x;
    const int64_t rb0 = wave * rb_each + (wave < rb_extra ? wave : rb_extra);
    const int64_t rb1 = rb0 + rb_each + (wave < rb_extra ? 1 : 0);
    const int cb = a.k * BITS / 8;              // bytes per row, a multiple of 64 here
    const int nsl = cb / 64;                    // 64-byte slices per row
    const int nwin = cb / wb, spw = wb / 64;    // windows per row, slices per window
    const int wbv = BITS == 4 ? 2 * wb : wb;    // validation bytes per window row
    const int wbytes = VR * wbv;                // one window buffer
    float *wlds = (float *)(vlds + (size_t)2 * wbytes);
    int *blds = (int *)(wlds + a.C * 32 * VB);  // sign codes: 3 k / 4 - 2 Sv per validation column and checkpoint
    unsigned char *ring = vlds + ring_off + (size_t)wv_id * nb * SLOT;
    const unsigned ring_lds = (unsigned)(uintptr_t)((__attribute__((address_space(3))) unsigned char *)ring);
    const unsigned vlds_lds = (unsigned)(uintptr_t)((__attribute__((address_space(3))) unsigned char *)vlds);
    const uint32_t halves = fp4_halves();

    for (int i = threadIdx.x; i < a.C * 32 * VB; i += 64 * NW) {
        const int j = i % (32 * VB), ci = i / (32 * VB);
        wlds[i] = __fmul_rn(a.eta[ci], a.vr[ci][m0 + (j < mc ? j : mc - 1)]);
        if (BITS == 1) blds[i] = 3 * (a.k / 4) - 2 * vsum[ci * a.M + m0 + (j < mc ? j : mc - 1)];
    }
    int64_t r_end = rb1 * unit;                 // blocks of `unit` rows are dealt out
    if (r_end > a.N) r_end = a.N;
    const int64_t r_begin = rb0 * unit;
    const int64_t my_rows = r_end > r_begin ? r_end - r_begin : 0;
    const int my_pass = (int)((my_rows + PASS - 1) / PASS);  // passes in which this wavefront has rows
    const int T = a.C * nsl;                                 // ring slots of a pass
    const int S = my_pass * T;                               // ring slots of this wavefront

    // ---- train ring: slot s is (pass s / T, checkpoint (s % T) / nsl, slice s % nsl)
    int f_ps = 0, f_ci = 0, f_sl = 0, f_pos = 0, f_it = 0;
    auto fetch = [&]() {
        const int64_t rp = r_begin + (int64_t)f_ps * PASS;
        const int lastr = (int)(r_end - rp < PASS ? r_end - rp : PASS) - 1;
        const int off = f_sl * 64 + ((cpos ^ ((crow >> 1) & 3)) << 4);
        const unsigned char *base = a.tc[f_ci] + rp * cb;                   // wave-uniform
        const unsigned slot = ring_lds + (unsigned)f_pos * (unsigned)SLOT;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            int rl = q * 16 + crow;
            if (rl > lastr) rl = lastr;                                      // clamped; masked at the output
            global_to_lds16(base, (unsigned)(rl * cb + off), slot + (unsigned)q * 1024u);
        }
        ++f_it;
        if (++f_pos == nb) f_pos = 0;
        if (++f_sl == nsl) { f_sl = 0; if (++f_ci == a.C) { f_ci = 0; ++f_ps; } }
    };
    // ---- validation windows: phase g is (pass g / (C nwin), checkpoint, window); buffer g % 2.
    // A window buffer is 32 VB wb / 1024 copies of 1 KB = 1024 / wb rows each; copy q belongs to
    // wavefront q % NW.  Rows past the chunk repeat its last one.
    const int nph = a.C * nwin, G = npass * nph;
    const int ncopy = wbytes / 1024, lpr = wbv / 16;         // copies per window; 16-byte chunks per row
    int v_cnt = 0;                                           // copies of the last request of this wavefront
    int v_at = 0;                                            // ring slots issued before that request
    auto fetch_window = [&](int g) {
        const int ph = g % nph, ci = ph / nwin, win = ph - ci * nwin;
        const unsigned buf = vlds_lds + (unsigned)((g & 1) * wbytes);
        v_cnt = 0;
        for (int q = wv_id; q < ncopy; q += NW) {
            const int g = q * 64 + lane, row = g / lpr, pos = g % lpr;      // chunk `pos` of staged row `row`
            const unsigned char *src;
            if (BITS == 4) {        // expanded rows, zero past M
                src = (const unsigned char *)vexp + ((size_t)ci * Mp + m0 + row) * (size_t)vrow + (size_t)win * wbv;
            } else {
                const int jc = m0 + (row < mc ? row : mc - 1);
                // sign codes: the pre-pass's copy of the validation rows with bits 0 and 2 of every nibble swapped
                src = (BITS == 1 ? (const unsigned char *)vexp + ((size_t)ci * a.M + jc) * (size_t)cb : a.vc[ci] + (int64_t)jc * cb) +
                      (int64_t)win * wb;
            }
            global_to_lds16(src + ((pos ^ (row & 7)) << 4), buf + (unsigned)q * 1024u);
            ++v_cnt;
        }
        v_at = f_it;
    };

    fetch_window(0);
    for (int i = 0; i < nb - 1 && i < S; ++i) fetch();
    int it = 0, pos = 0;
    for (int ps = 0; ps < npass; ++ps) {                                     // workgroup-uniform counts
        const int64_t rp = r_begin + (int64_t)ps * PASS;
        const int rows = ps < my_pass ? (r_end - rp < PASS ? (int)(r_end - rp) : PASS) : 0;   // wave-uniform
        const int last = rows - 1;
        typename AccType<BITS == 1>::type acc[NPMAX][VB];
        uint32_t cnt[NPMAX] = {};                // sign codes: negative train codes outside dword 0, this lane's half of K
        float facc[NPMAX][VB][16];
#pragma unroll
        for (int p = 0; p < NPMAX; ++p)
#pragma unroll
            for (int vb = 0; vb < VB; ++vb)
#pragma unroll
                for (int v = 0; v < 16; ++v) { acc[p][vb][v] = 0; facc[p][vb][v] = 0.0f; }
        for (int ci = 0; ci < a.C; ++ci) {
            for (int win = 0; win < nwin; ++win) {
                const int g = (ps * a.C + ci) * nwin + win;
                // this wavefront's share of window g has landed once at most the ring copies issued
                // after it are outstanding; the barrier makes every share visible and tells that
                // all wavefronts are done with window g - 1, whose buffer the next request reuses
                wait_vmcnt_upto(NQ * (f_it - v_at));
                __syncthreads();
                if (g + 1 < G) fetch_window(g + 1);
                if (rows > 0) {
                    const unsigned char *vwin = vlds + (size_t)(g & 1) * wbytes;
                    for (int s4 = 0; s4 < spw; ++s4) {
                        // operations issued after this slot's copies: the younger slots and, if it
                        // came later, the last window request
                        wait_vmcnt_upto(NQ * (f_it - 1 - it) + (it < v_at ? v_cnt : 0));
                        if (f_it < S) fetch();
                        const unsigned char *sb = ring + (size_t)pos * SLOT;
                        if constexpr (BITS == 1) {
                            if (NPMAX == 3 && rows > 64) stream32_slice<VB, NPMAX, NPMAX>(sb, vwin, 4 * s4, wb, l32, half, halves, acc, cnt);
                            else if (rows > 32) stream32_slice<VB, 2, NPMAX>(sb, vwin, 4 * s4, wb, l32, half, halves, acc, cnt);
                            else stream32_slice<VB, 1, NPMAX>(sb, vwin, 4 * s4, wb, l32, half, halves, acc, cnt);
                        } else {
                            if (NPMAX == 3 && rows > 64) stream32_slice_i8<BITS, VB, VR, NPMAX, NPMAX>(sb, vwin, s4, wbv, l32, half, acc);
                            else if (rows > 32) stream32_slice_i8<BITS, VB, VR, 2, NPMAX>(sb, vwin, s4, wbv, l32, half, acc);
                            else stream32_slice_i8<BITS, VB, VR, 1, NPMAX>(sb, vwin, s4, wbv, l32, half, acc);
                        }
                        ++it;
                        if (++pos == nb) pos = 0;
                    }
                }
            }
            if (rows > 0) {
                // checkpoint epilogue: accumulator v of lane (train row l32, half) is validation row
                // 8 (v / 4) + 4 half + v % 4 of its block
#pragma unroll
                for (int p = 0; p < NPMAX; ++p) {
                    if (32 * p >= rows) continue;                            // wave-uniform
                    const float rt = a.tr[ci][rp + (32 * p + l32 < rows ? 32 * p + l32 : last)];
                    // sign codes: St of train row l32 = the counts of the two lanes that share the row
                    int st2 = 0;
                    if (BITS == 1) { const uint32_t c = cnt[p]; st2 = 2 * (int)(c + (uint32_t)__shfl_xor((int)c, 32)); }
#pragma unroll
                    for (int vb = 0; vb < VB; ++vb)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int col = 32 * vb + 8 * (v >> 2) + 4 * half + (v & 3);
                            const float wv = wlds[ci * 32 * VB + col];
                            // 1-bit: 4 acc + 3 k / 4 - 2 Sv - 2 St (acc is a multiple of 1/4, exact); 4-bit: acc = 16 D (train codes scaled)
                            const float D = BITS == 1 ? (float)((int)((float)acc[p][vb][v] * 4.0f) + blds[ci * 32 * VB + col] - st2)
                                          : (float)(BITS == 4 ? ((int)acc[p][vb][v] >> 4) : (int)acc[p][vb][v]);
                            const float t = __fmul_rn(__fmul_rn(D, rt), wv);
                            facc[p][vb][v] = __fadd_rn(facc[p][vb][v], t);
                            acc[p][vb][v] = 0;
                        }
                }
#pragma unroll
                for (int p = 0; p < NPMAX; ++p) cnt[p] = 0u;
            }
        }
        if (rows > 0) {
#pragma unroll
            for (int p = 0; p < NPMAX; ++p) {
                if (32 * p >= rows) continue;
                const bool live = 32 * p + l32 < rows;
                const int64_t r = rp + 32 * p + l32;
                float m = neg_inf();
#pragma unroll
                for (int vb = 0; vb < VB; ++vb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int j = 32 * vb + 8 * (v >> 2) + 4 * half + (v & 3);
                        if (j < mc) {
                            m = fmaxf(m, facc[p][vb][v]);
                            if (a.full && live) a.full[r * a.M + m0 + j] = facc[p][vb][v];
                        }
                    }
                m = fmaxf(m, __shfl_xor(m, 32));
                if (a.score && live && half == 0) a.score[r] = m0 > 0 ? fmaxf(a.score[r], m) : m;
            }
        }
    }
}

// Shape of the NW waves of a workgroup: WX waves across the val tile, NW / WX down the train
// rows; each wave owns WR x WC accumulators of 32 x 32.  Train tile height MT = 32 WR NW / WX, val
// tile width VT = 32 WC WX:
//   M > 64: <2, 2, 2, 8> (64 x 64 per wave, 256 x 128 per workgroup), or for sign codes <2, 3, 1, 8>
//   (64 x 96 per wave, 512 x 96 per workgroup) when that pads M less;  M <= 64: <1, 2, 1, 8> (256 x 64);
//   M <= 32: <1, 1, 1, 8> (256 x 32) or <1, 1, 1, 4> (128 x 32), whichever fills the chip more evenly.
template <int BITS, int WR, int WC, int WX, int NW, bool VH = false>
struct MfmaShape {
    static constexpr int WY = NW / WX;
    static constexpr int MT = 32 * WR * WY;
    static constexpr int VT = 32 * WC * WX;
    // VH (one 32-wide val block, at most 16 validation vectors): only 16 validation rows are staged
    // (lanes 16..31 of the val operand re-read them; their results are masked), which leaves room for
    // one more workgroup per compute unit
    static constexpr int VROWS = VH ? 16 : VT;
    static_assert(!VH || (WC == 1 && WX == 1), "half val tiles exist for the 32-wide shape only");
    // Code elements per stage: a stage should bring 128 bytes of every train row (whole cache lines
    // when the codes are streamed from HBM) as far as the expanded validation rows leave room in LDS:
    // the shapes for few validation vectors take 256 elements (4- and 2-bit) or 512 (1-bit).
    static constexpr bool NARROW = WR == 1;              // the shapes for at most 64 validation vectors
    static constexpr int KE = narrow_stage_elements(BITS, 32 * WC * WX);
    static constexpr bool FP4 = BITS <= 2;               // sign / ternary codes go to the matrix core as FP4 +-1.0, 0
    static constexpr int TB = KE * BITS / 8;             // train bytes per row per stage
    static constexpr int TCPR = TB / 16;                 // 16-byte chunks per train row
    // val bytes per row per stage: int8-expanded; for the sign codes FP4-expanded by the pre-pass (wide
    // tiles, where the VALU has no room to expand both operands), or the packed signs themselves
    static constexpr bool VPACKED = BITS == 1 && NARROW;
    static constexpr int VROWB = VPACKED ? KE / 8 : (FP4 ? KE / 2 : KE);
    static constexpr int VCPR = VROWB / 16;              // 16-byte chunks per expanded val row
    // rows whose chunks share a bank group are 16 / CPR apart: the swizzle key is (row >> SH) % CPR
    static constexpr int TSH = log2c(16 / TCPR), VSH = log2c(16 / VCPR);
    static constexpr int TRAIN_BYTES = MT * TB, VAL_BYTES = VROWS * VROWB;
    static constexpr int TCH = MT * TCPR, VCH = VROWS * VCPR;
    static constexpr int NINST = (TCH + VCH) / 64;       // wavefront-wide copies per stage
    static constexpr int LPW = (NINST + NW - 1) / NW;    // per wave
    static constexpr int BUF = TRAIN_BYTES + VAL_BYTES + 1024;   // + 1 KB landing zone for padding copies
    // LDS ring depth.  The narrow shapes serve few validation vectors, where scoring streams the
    // train codes from HBM: two stages per workgroup and several workgroups per compute unit,
    // whose barriers and epilogues then overlap each other's copies.
    static constexpr int NBUF = NARROW ? 2 : ((158 * 1024) / BUF >= 4 ? 4 : (158 * 1024) / BUF);
    static constexpr int PLANES = BITS == 2 ? 2 : 1;     // separately stored bit planes of a train row
    static constexpr int PCH = TCPR / PLANES;            // chunks per plane and stage
    static constexpr int TSTEP = TB / PLANES;            // bytes a plane's source advances per stage
    static_assert(WY * WX == NW && TCH % 64 == 0 && (TCH + VCH) % 64 == 0, "whole wavefront copies");
    static_assert(NBUF >= 2 && NBUF * BUF <= 158 * 1024, "a ring of at least two stages fits in LDS");
};

// F16 (with BITS = 8 and k counted in bytes): the rows are bfloat16 vectors, the 16 bytes a lane feeds
// to the matrix core are eight bfloat16 values for v_mfma_f32_32x32x16_bf16 (same bytes, same
// addresses as the int8 operands), the accumulator is fp32 and the epilogue is acc += eta * D:
// the 16-bit LESS comparator (Eq.(2),(3)) on pre-normalised rows.
// AGG: instead of score / full the kernel writes, per train row, the maximum or the left-to-right fp32
// mean of acc over each group of consecutive validation columns (gout[N][T]).  One workgroup then takes a
// train tile through all validation tiles in order; after each tile the sums go through LDS (the stage
// ring is idle then) to one thread per train row, which walks the tile's columns in order and carries
// the running value of the open group in a register.
struct AggArgs { GroupEnds ge; int T, mean; float *gout; };

template <int BITS, int WR, int WC, int WX, int NW, bool F16 = false, bool VH = false, bool AGG = false>
__global__ void __launch_bounds__(64 * NW, (WR == 1 ? 4 : 2))
score_mfma_kernel(ScoreArgs a, ScorePrep w, int ttiles, int vtiles, AggArgs ag) {
    static_assert(!F16 || BITS == 8, "bfloat16 rows use the byte geometry of the 8-bit codes");
    using Sh = MfmaShape<BITS, WR, WC, WX, NW, VH>;
    constexpr int kMT = Sh::MT;
    constexpr int KE = Sh::KE, TB = Sh::TB, TCPR = Sh::TCPR, VCPR = Sh::VCPR, TSH = Sh::TSH, VSH = Sh::VSH, VT = Sh::VT;
    constexpr int TRAIN_BYTES = Sh::TRAIN_BYTES, VAL_BYTES = Sh::VAL_BYTES, TCH = Sh::TCH;
    constexpr int NINST = Sh::NINST, LPW = Sh::LPW, BUF = Sh::BUF, NBUF = Sh::NBUF;
    constexpr int TSTEP = Sh::TSTEP, PCH = Sh::PCH;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ unsigned int s_rowmax[kMT];

    // XCD-aware decode: the vtiles workgroups of one train tile get ids 8 apart
    const int64_t id = blockIdx.x;
    const int xcd = (int)(id & 7);
    const int64_t j = id >> 3;
    const int vt_first = AGG ? 0 : (int)(j % vtiles);
    const int vt_end = AGG ? vtiles : vt_first + 1;
    const int64_t tt = AGG ? id : (j / vtiles) * 8 + xcd;
    if (tt >= ttiles) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int wy = wave / WX, wx = wave % WX;
    const int trow = wy * 32 * WR, vcol = wx * 32 * WC;   // this wave's corner inside the tile
    const int64_t row0 = tt * kMT;
    int v0 = vt_first * VT;                             // advanced per validation tile (AGG)
    const int64_t cb = (int64_t)a.k * BITS / 8;
    const int nstages = (a.k + KE - 1) / KE;            // <= kp / KE: the expanded val rows cover every stage
    if (tid < kMT) s_rowmax[tid] = 0u;
    const unsigned lds0 = (unsigned)(uintptr_t)((__attribute__((address_space(3))) unsigned char *)smem);

    // ---- copy roles of this lane: LPW wavefront copies per stage -------------------------------
    // Copy q covers LDS chunks 64 q .. 64 q + 63 of the stage buffer, laid out [train rows][val rows]
    // without padding; inside a row the 16-byte chunks are XOR-swizzled so that the MFMA operand
    // reads (consecutive rows, same chunk) spread over the banks.  2-bit train rows hold the
    // "non-zero" chunks then the "negative" chunks of the stage (the planes are k/8 bytes apart).
    unsigned voff[LPW];         // lane offset from the stage's (uniform) train or val base
    unsigned vcolb[LPW];        // byte offset of the lane's chunk inside its plane's share of the stage (train copies)
    bool is_train[LPW];         // wave-uniform: a copy is all train chunks or all val chunks
    unsigned dst_off[LPW];      // wave-uniform LDS offset inside the buffer
#pragma unroll
    for (int u = 0; u < LPW; ++u) {
        const int q = wave * LPW + u;
        const int qq = q < NINST ? q : 0;
        const int t = qq * 64 + lane;
        dst_off[u] = q < NINST ? (unsigned)q * 1024u : (unsigned)(TRAIN_BYTES + VAL_BYTES);
        is_train[u] = qq * 64 < TCH;
        if (t < TCH) {
            const int r = t / TCPR, pos = t % TCPR;
            const int c = pos ^ ((r >> TSH) & (TCPR - 1));
            int64_t grow = row0 + r;
            if (grow > a.N - 1) grow = a.N - 1;          // rows past N re-read the last row (masked later)
            voff[u] = (unsigned)((grow - row0) * cb) + (unsigned)((c / PCH) * (a.k / 8) + (c % PCH) * 16);
            vcolb[u] = (c % PCH) * 16;
        } else {
            const int tv = t - TCH;
            const int r = tv / VCPR, pos = tv % VCPR;
            const int c = pos ^ ((r >> VSH) & (VCPR - 1));
            if (Sh::VPACKED) {
                // 1-bit, few validation vectors: the packed validation rows are staged as they are (rows past M re-read the last one)
                const int rc = v0 + r < a.M ? r : a.M - 1 - v0;
                voff[u] = (unsigned)rc * (unsigned)cb + c * 16;
                vcolb[u] = c * 16;
            } else {
                voff[u] = (unsigned)r * (unsigned)w.vrow + c * 16;
                vcolb[u] = 0;
            }
        }
    }
    const bool ragged = (a.k % KE) != 0;               // the last stage reaches past the end of the train rows / planes
    const int64_t plane_bytes = cb / Sh::PLANES;

    // ---- operand read addresses (swizzle folded into the lane's base, K-step applied by XOR) ---
    unsigned a_base[WR], b_base[WC];
#pragma unroll
    for (int b = 0; b < WR; ++b) {
        const int R = trow + 32 * b + l32;
        const int sw = (l32 >> TSH) & (TCPR - 1);       // trow + 32 b is a multiple of 32: the key is l32's
        if (BITS == 8) a_base[b] = R * TB + (sw >> 1) * 32 + ((half ^ (sw & 1)) * 16);
        else if (BITS == 4) a_base[b] = R * TB + sw * 16 + half * 8;
        else if (Sh::VPACKED) a_base[b] = R * TB + sw * 16 + half * 4;   // 4-byte reads, chunk chosen by XOR below
        else a_base[b] = R * TB + ((sw ^ half) << 4);   // bit planes: 16-byte reads of chunk 2 q + half, q by XOR below
    }
#pragma unroll
    for (int c = 0; c < WC; ++c) {
        const int lv = VH ? (l32 & 15) : l32;           // row of the staged val tile this lane reads
        const int Rv = vcol + 32 * c + lv;
        const int sw = (lv >> VSH) & (VCPR - 1);
        if (Sh::VPACKED) b_base[c] = TRAIN_BYTES + Rv * Sh::VROWB + sw * 16 + half * 4;  // 4-byte reads, chunk chosen by XOR
        else b_base[c] = TRAIN_BYTES + Rv * Sh::VROWB + (sw >> 1) * 32 + ((half ^ (sw & 1)) * 16);
    }

    // AGG: thread t < kMT owns train row t of the tile: index and running value of its open group
    int ag_group = 0;
    float ag_run = 0.0f;
    static_assert(!AGG || (!Sh::VPACKED && !VH), "group aggregation runs on the wide tiles");

  for (int vt = vt_first; vt < vt_end; ++vt) {
    v0 = vt * VT;
    float facc[WR][WC][16];
#pragma unroll
    for (int b = 0; b < WR; ++b)
#pragma unroll
        for (int c = 0; c < WC; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) facc[b][c][v] = 0.0f;

    const int total = a.C * nstages;                 // stages over all checkpoints, one pipeline
    auto issue = [&](int g) {                        // start the copies of global stage g
        const int ci = g / nstages, s = g - ci * nstages;
        const unsigned char *tbase = a.tc[ci] + row0 * cb + (int64_t)s * TSTEP;
        const unsigned char *vbase = Sh::VPACKED ? a.vc[ci] + (int64_t)v0 * cb + (int64_t)s * Sh::VROWB
                                             : (const unsigned char *)w.vexp + ((size_t)ci * w.Mp + v0) * (size_t)w.vrow + (size_t)s * Sh::VROWB;
        const unsigned buf = lds0 + (unsigned)(g % NBUF) * BUF;
        const bool tail = ragged && s == nstages - 1;
#pragma unroll
        for (int u = 0; u < LPW; ++u) {
            unsigned off = voff[u];
            if (tail && (is_train[u] || Sh::VPACKED)) {
                // chunks past the row end re-read its last 16 bytes (the matching val bytes are zero, or,
                // for the packed sign codes, the K steps past the end are not computed)
                const int64_t over = (int64_t)s * (is_train[u] ? TSTEP : Sh::VROWB) + vcolb[u] - (plane_bytes - 16);
                if (over > 0) off -= (unsigned)over;
            }
            global_to_lds16(is_train[u] ? tbase : vbase, off, buf + dst_off[u]);
        }
    };

    // prologue: NBUF-1 stages in flight
#pragma unroll
    for (int g = 0; g < NBUF - 1; ++g)
        if (g < total) issue(g);

    int g = 0;
    const uint32_t ones = fp4_ones();
    for (int ci = 0; ci < a.C; ++ci) {
        typename AccType<F16 || BITS <= 2>::type acc[WR][WC];
#pragma unroll
        for (int b = 0; b < WR; ++b)
#pragma unroll
            for (int c = 0; c < WC; ++c)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[b][c][v] = 0;

        for (int s = 0; s < nstages; ++s, ++g) {
            // the copies of stage g are the oldest outstanding ones; NBUF-2 younger stages may stay in
            // flight (near the end fewer are outstanding, so waiting for everything is exact there)
            if (g + NBUF - 2 < total) wait_vmcnt<(NBUF - 2) * LPW>(); else wait_vmcnt<0>();
            __syncthreads();                         // stage g visible to all; buffer of stage g-1 free
            if (g + NBUF - 1 < total) issue(g + NBUF - 1);
            const unsigned char *sb = smem + (g % NBUF) * BUF;
            if constexpr (BITS == 1 && !Sh::VPACKED) {
                // sign codes as FP4: one 64-element K step per matrix-core instruction.  A lane reads 16
                // bytes of its row (chunk 2 q + half: four words of 32 signs) per four K steps; word j
                // becomes four dwords of FP4 codes, dword jd = bits 3 - jd of every nibble, left where they
                // are: (w & 0x88888888) | 0x22222222 = +-1.0, then w & 0x44444444, w & 0x22222222,
                // w & 0x11111111 = 2 s, s, s / 2 (four operations per word; the pre-pass scaled the
                // validation codes of those positions to match, see score_prepare_kernel).  The pre-expanded
                // validation rows follow the same order and are zero past the end of the vectors.
                // The validation fragments of K step ks + 1 and the train words of the next four steps are
                // requested before the matrix instructions of step ks (scheduling barriers keep that
                // order), so a wave waits for LDS once per stage instead of once per step; the train
                // fragments of step ks + 1 are expanded between the matrix instructions of step ks, each
                // instruction followed by its share of the expansions (scheduling groups).
                i32x4 wq[KE / 256][WR], bq[WC], bn[WC];
#pragma unroll
                for (int b = 0; b < WR; ++b) wq[0][b] = *(const i32x4 *)(sb + a_base[b]);
#pragma unroll
                for (int c = 0; c < WC; ++c) bq[c] = *(const i32x4 *)(sb + b_base[c]);
                auto expand = [&](unsigned int wd) {
                    i32x8 r = {0, 0, 0, 0, 0, 0, 0, 0};
                    r[0] = (int)sign_bits_or(wd, ones); r[1] = (int)(wd & 0x44444444u);
                    r[2] = (int)(wd & 0x22222222u); r[3] = (int)(wd & 0x11111111u);
                    return r;
                };
                i32x8 afc[WR], afn[WR];
#pragma unroll
                for (int b = 0; b < WR; ++b) afc[b] = expand((unsigned int)wq[0][b][0]);
#pragma unroll
                for (int ks = 0; ks < KE / 64; ++ks) {
                    const int q = ks >> 2, j = ks & 3;
                    if (ks + 1 < KE / 64) {
#pragma unroll
                        for (int c = 0; c < WC; ++c) bn[c] = *(const i32x4 *)(sb + (b_base[c] ^ ((ks + 1) << 5)));
                    }
                    if (j == 1 && q + 1 < KE / 256) {
#pragma unroll
                        for (int b = 0; b < WR; ++b) wq[q + 1][b] = *(const i32x4 *)(sb + (a_base[b] ^ ((q + 1) << 5)));
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    i32x8 bf[WC];
#pragma unroll
                    for (int c = 0; c < WC; ++c) bf[c] = i32x8{bq[c][0], bq[c][1], bq[c][2], bq[c][3], 0, 0, 0, 0};
#pragma unroll
                    for (int b = 0; b < WR; ++b)
#pragma unroll
                        for (int c = 0; c < WC; ++c) acc[b][c] = mfma_fp4(afc[b], bf[c], acc[b][c]);
                    if (ks + 1 < KE / 64) {
#pragma unroll
                        for (int b = 0; b < WR; ++b) afn[b] = expand((unsigned int)wq[(ks + 1) >> 2][b][(ks + 1) & 3]);
                    }
#pragma unroll
                    for (int i = 0; i < WR * WC; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one matrix instruction
                        __builtin_amdgcn_sched_group_barrier(0x002, 4 / WC > 0 ? 4 / WC : 1, 0);   // its share of the 4 WR expansion operations
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int c = 0; c < WC; ++c) bq[c] = bn[c];
#pragma unroll
                    for (int b = 0; b < WR; ++b) afc[b] = afn[b];
                }
            } else if constexpr (BITS == 1) {
                // few validation vectors: both operands are packed rows, read as 4-byte words (K step ks:
                // word 2 ks + half) and expanded in registers.  K steps of the last stage that start past
                // the end of the vectors are skipped (k % 64 == 0).
                const int ksteps = (a.k - s * KE) / 64 < KE / 64 ? (a.k - s * KE) / 64 : KE / 64;
#pragma unroll
                for (int ks = 0; ks < KE / 64; ++ks) {
                    if (ks >= ksteps) break;
                    i32x8 af[WR], bf[WC];
#pragma unroll
                    for (int b = 0; b < WR; ++b) {
                        const unsigned int wd = *(const unsigned int *)(sb + (a_base[b] ^ ((ks >> 1) << 4)) + 8 * (ks & 1));
#pragma unroll
                        for (int jd = 0; jd < 4; ++jd) af[b][jd] = (int)sign_bits_or(wd << jd, ones);
#pragma unroll
                        for (int jd = 4; jd < 8; ++jd) af[b][jd] = 0;
                    }
#pragma unroll
                    for (int c = 0; c < WC; ++c) {
                        const unsigned int wd = *(const unsigned int *)(sb + (b_base[c] ^ ((ks >> 1) << 4)) + 8 * (ks & 1));
#pragma unroll
                        for (int jd = 0; jd < 4; ++jd) bf[c][jd] = (int)sign_bits_or(wd << jd, ones);
#pragma unroll
                        for (int jd = 4; jd < 8; ++jd) bf[c][jd] = 0;
                    }
#pragma unroll
                    for (int b = 0; b < WR; ++b)
#pragma unroll
                        for (int c = 0; c < WC; ++c)
                            acc[b][c] = mfma_fp4(af[b], bf[c], acc[b][c]);
                }
            } else if constexpr (BITS == 2) {
                // ternary codes as FP4 {-1.0, 0, +1.0}: nibble bit 3 <- "negative" plane, bit 1 <- "non-zero"
                // plane; 16-byte reads of both planes per four K steps, dword jd of the
                // expansion takes bits 4 n + 3 - jd of the two plane words
#pragma unroll
                for (int q = 0; q < KE / 256; ++q) {
                    i32x4 wnq[WR], wgq[WR];
#pragma unroll
                    for (int b = 0; b < WR; ++b) {
                        wnq[b] = *(const i32x4 *)(sb + (a_base[b] ^ (q << 5)));
                        wgq[b] = *(const i32x4 *)(sb + (a_base[b] ^ (q << 5) ^ (PCH << 4)));
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int ks = 4 * q + j;
                        i32x8 af[WR], bf[WC];
#pragma unroll
                        for (int b = 0; b < WR; ++b) {
                            const unsigned int wn = (unsigned int)wnq[b][j], wg = (unsigned int)wgq[b][j];
                            // dword 0: magnitude 1.0 from the shifted plane; dwords 1 .. 3: the plane bit where it
                            // is (2, 1, 1/2; the pre-pass scaled the validation codes to match): 12 operations
                            af[b][0] = (int)sign_bits_or(wg, (wn >> 2) & 0x22222222u);
                            af[b][1] = (int)sign_bits_or(wg << 1, wn & 0x44444444u);
                            af[b][2] = (int)sign_bits_or(wg << 2, wn & 0x22222222u);
                            af[b][3] = (int)sign_bits_or(wg << 3, wn & 0x11111111u);
#pragma unroll
                            for (int jd = 4; jd < 8; ++jd) af[b][jd] = 0;
                        }
#pragma unroll
                        for (int c = 0; c < WC; ++c) {
                            const i32x4 lo = *(const i32x4 *)(sb + (b_base[c] ^ (ks << 5)));
                            bf[c] = i32x8{lo[0], lo[1], lo[2], lo[3], 0, 0, 0, 0};
                        }
#pragma unroll
                        for (int b = 0; b < WR; ++b)
#pragma unroll
                            for (int c = 0; c < WC; ++c)
                                acc[b][c] = mfma_fp4(af[b], bf[c], acc[b][c]);
                    }
                }
            } else if constexpr (!Sh::NARROW) {
                // int8 (or bfloat16) operands, wide tiles: the fragments of K step ks + 1 are requested before the
                // matrix instructions of step ks (scheduling barriers keep that order)
                i32x4 aq[WR], bq[WC], an[WR], bn[WC];
                auto load_step = [&](int ks, i32x4 (&fa)[WR], i32x4 (&fb)[WC]) {
#pragma unroll
                    for (int b = 0; b < WR; ++b) {
                        if (BITS == 8) {
                            fa[b] = *(const i32x4 *)(sb + (a_base[b] ^ (ks << 5)));
                        } else {
                            const uint2 pa = *(const uint2 *)(sb + (a_base[b] ^ (ks << 4)));
                            fa[b] = i32x4{(int)pa.x, (int)pa.y, 0, 0};
                        }
                    }
#pragma unroll
                    for (int c = 0; c < WC; ++c) fb[c] = *(const i32x4 *)(sb + (b_base[c] ^ (ks << 5)));
                };
                load_step(0, aq, bq);
#pragma unroll
                for (int ks = 0; ks < KE / 32; ++ks) {
                    if (ks + 1 < KE / 32) load_step(ks + 1, an, bn);
                    __builtin_amdgcn_sched_barrier(0);
                    i32x4 af[WR];
#pragma unroll
                    for (int b = 0; b < WR; ++b) {
                        if (BITS == 8) {
                            af[b] = aq[b];
                        } else {
                            const unsigned int px = (unsigned int)aq[b][0], py = (unsigned int)aq[b][1];
                            af[b][0] = (int)((px << 4) & 0xF0F0F0F0u); af[b][1] = (int)(px & 0xF0F0F0F0u);
                            af[b][2] = (int)((py << 4) & 0xF0F0F0F0u); af[b][3] = (int)(py & 0xF0F0F0F0u);
                        }
                    }
#pragma unroll
                    for (int b = 0; b < WR; ++b)
#pragma unroll
                        for (int c = 0; c < WC; ++c)
                            acc[b][c] = mfma_step<F16>(af[b], bq[c], acc[b][c]);
                    __builtin_amdgcn_sched_barrier(0);
                    if (ks + 1 < KE / 32) {
#pragma unroll
                        for (int b = 0; b < WR; ++b) aq[b] = an[b];
#pragma unroll
                        for (int c = 0; c < WC; ++c) bq[c] = bn[c];
                    }
                }
            } else {
#pragma unroll
                for (int ks = 0; ks < KE / 32; ++ks) {
                    i32x4 af[WR], bf[WC];
#pragma unroll
                    for (int b = 0; b < WR; ++b) {
                        if (BITS == 8) {
                            af[b] = *(const i32x4 *)(sb + (a_base[b] ^ (ks << 5)));
                        } else {
                            const uint2 pa = *(const uint2 *)(sb + (a_base[b] ^ (ks << 4)));
                            af[b][0] = (int)((pa.x << 4) & 0xF0F0F0F0u); af[b][1] = (int)(pa.x & 0xF0F0F0F0u);
                            af[b][2] = (int)((pa.y << 4) & 0xF0F0F0F0u); af[b][3] = (int)(pa.y & 0xF0F0F0F0u);
                        }
                    }
#pragma unroll
                    for (int c = 0; c < WC; ++c) bf[c] = *(const i32x4 *)(sb + (b_base[c] ^ (ks << 5)));
#pragma unroll
                    for (int b = 0; b < WR; ++b)
#pragma unroll
                        for (int c = 0; c < WC; ++c)
                            acc[b][c] = mfma_step<F16>(af[b], bf[c], acc[b][c]);
                }
            }
        }
        // checkpoint epilogue.  acc[b][c][v]: train row 32b + 8(v/4) + 4 half + v%4, val col 32c + l32.
        // Lane L < 32 WR of the wave holds rnorm of train row (trow + L); rows are fetched by shuffle.
        int64_t myrow = row0 + trow + (lane & (32 * WR - 1));
        if (myrow > a.N - 1) myrow = a.N - 1;
        // bfloat16 rows: no train factor (the 16-bit comparator's rows are unit vectors) unless the caller
        // gives one (mixed precision: rows of integer codes with their 1 / ||q||)
        const float rt_lane = (F16 && !a.tr[ci]) ? 1.0f : a.tr[ci][myrow];
        float wv[WC];
        int vbias[WC];
#pragma unroll
        for (int c = 0; c < WC; ++c) {
            const int col = v0 + vcol + 32 * c + l32;               // < Mp (padded)
            wv[c] = w.vw[ci * w.Mp + col];
            vbias[c] = (BITS == 1 && !Sh::VPACKED) ? w.vbias[ci * w.Mp + col] : 0;
        }
#pragma unroll
        for (int b = 0; b < WR; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float rt = __shfl(rt_lane, 32 * b + 8 * (v >> 2) + 4 * half + (v & 3), 64);
#pragma unroll
                for (int c = 0; c < WC; ++c) {
                    float t;
                    if (F16) {
                        t = __fmul_rn(__fmul_rn((float)acc[b][c][v], rt), wv[c]);     // rt = 1: the product is acc itself
                    } else {
                        int D = BITS == 4 ? ((int)acc[b][c][v] >> 4) : (int)acc[b][c][v];   // 1-/2-bit: an exact integer in fp32
                        if (BITS == 1 && !Sh::VPACKED) D += vbias[c];
                        t = __fmul_rn(__fmul_rn((float)D, rt), wv[c]);
                    }
                    facc[b][c][v] = __fadd_rn(facc[b][c][v], t);
                }
            }
    }
    if constexpr (AGG) {
        // the tile's sums go to LDS as [kMT][VT + 1] floats (odd stride: a wavefront's rows fall in different
        // banks); every copy of the tile has landed and every wavefront has read its last stage by now
        constexpr int LD = VT + 1;
        float *tile = (float *)smem;
        __syncthreads();
#pragma unroll
        for (int b = 0; b < WR; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int rloc = trow + 32 * b + 8 * (v >> 2) + 4 * half + (v & 3);
#pragma unroll
                for (int c = 0; c < WC; ++c) tile[rloc * LD + vcol + 32 * c + l32] = facc[b][c][v];
            }
        __syncthreads();
        if (tid < kMT && row0 + tid < a.N) {
            const float *trowp = tile + tid * LD;
            const int ncol = a.M - v0 < VT ? a.M - v0 : VT;
            for (int jc = 0; jc < ncol; ++jc) {
                const int col = v0 + jc;
                const int g0 = ag_group ? ag.ge.end[ag_group - 1] : 0, g1 = ag.ge.end[ag_group];
                const float x = trowp[jc];
                if (ag.mean) ag_run = __fadd_rn(col == g0 ? 0.0f : ag_run, x);
                else ag_run = (col == g0 || x > ag_run) ? x : ag_run;
                if (col == g1 - 1) {
                    ag.gout[(row0 + tid) * ag.T + ag_group] = ag.mean ? __fdiv_rn(ag_run, (float)(g1 - g0)) : ag_run;
                    ++ag_group;
                }
            }
        }
        __syncthreads();                             // the next tile's copies overwrite the buffer
        continue;
    }
    // tile epilogue: optional full matrix, row maxima over this val tile
#pragma unroll
    for (int b = 0; b < WR; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int rloc = trow + 32 * b + 8 * (v >> 2) + 4 * half + (v & 3);
            const int64_t r = row0 + rloc;
            float m = neg_inf();
#pragma unroll
            for (int c = 0; c < WC; ++c) {
                const int col = v0 + vcol + 32 * c + l32;
                if (col < a.M) {
                    m = fmaxf(m, facc[b][c][v]);
                    if (a.full && r < a.N) a.full[r * a.M + col] = facc[b][c][v];
                }
            }
            if (a.score) {
#pragma unroll
                for (int o = 16; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
                if (l32 == 0 && m > neg_inf()) atomicMax(&s_rowmax[rloc], f32_order_key(m));
            }
        }
    if (a.score) {
        __syncthreads();
        if (tid < kMT && row0 + tid < a.N && s_rowmax[tid] != 0u) atomicMax(&w.smax[row0 + tid], s_rowmax[tid]);
    }
  }
}

constexpr size_t kLdsPerCU = 160 * 1024;       // LDS of one compute unit
constexpr size_t kStaticLds = 1024;            // s_rowmax
// Compute units of the current device (256 on MI355X).
static int compute_units() {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        cus = 256;
    return cus;
}

struct MfmaPlan { int32_t vt, Mp, kp; size_t off_vw, off_vbias, off_smax, total; };
static MfmaPlan mfma_plan(int64_t N, int32_t M, int32_t k, int bits, int C, bool wide128 = false) {
    MfmaPlan p{};
    p.vt = (M > 64 || wide128) ? 128 : (M > 32 ? 64 : 32);
    // sign codes: 512 x 96 tiles (64 x 96 per wave) where 96-wide tiles pad the validation set less than
    // 128-wide ones (M = 285: 288 instead of 384 columns)
    if (!wide128 && bits == 1 && M > 64 && (M + 95) / 96 * 96 < (M + 127) / 128 * 128) p.vt = 96;
    p.Mp = (M + p.vt - 1) / p.vt * p.vt;
    const int ke = narrow_stage_elements(bits, p.vt);                 // MfmaShape::KE of the shape used
    p.kp = (k + ke - 1) / ke * ke;
    size_t o = (size_t)C * p.Mp * (size_t)p.kp;
    o = (o + 255) & ~(size_t)255;
    p.off_vw = o;   o += (size_t)C * p.Mp * 4;
    o = (o + 255) & ~(size_t)255;
    p.off_vbias = o; o += (size_t)C * p.Mp * 4;
    o = (o + 255) & ~(size_t)255;
    p.off_smax = o; o += (size_t)(N > 0 ? N : 1) * 4;
    p.total = o;
    return p;
}
// The bit planes are copied in 16-byte chunks: k must be a multiple of 128 for the 1-/2-bit codes.
// With at most 8 validation vectors those codes never take this path (and never need its
// workspace): the streaming kernel serves them, or the popcount kernel if their validation codes
// do not fit in LDS.
static bool use_mfma_path(int bits, int32_t M, int32_t k) { return bits >= 4 || (k % 128 == 0 && M > kStreamVal); }

// per_cu > 0 asks for exactly that many workgroups per compute unit (by padding the LDS request).
template <int BITS, int WR, int WC, int WX, int NW, bool F16 = false, bool VH = false>
static qless_status launch_mfma_shape(const ScoreArgs &a, const ScorePrep &w, int per_cu, hipStream_t st) {
    using Sh = MfmaShape<BITS, WR, WC, WX, NW, VH>;
    size_t lds = (size_t)Sh::NBUF * Sh::BUF;
    if (per_cu > 0) {
        const size_t share = ((size_t)kLdsPerCU / per_cu - kStaticLds) & ~(size_t)511;
        if (share > lds) lds = share;
    }
    // the kernel's static LDS (row maxima: 4 bytes per train row of the tile) counts against the same 160 KB
    constexpr int kMaxDynamic = (int)kLdsPerCU - 4 * Sh::MT;
    QLESS_LDS_KERNEL((score_mfma_kernel<BITS, WR, WC, WX, NW, F16, VH>), kMaxDynamic);
    if (lds > (size_t)kMaxDynamic) return QLESS_ERR_DEVICE;
    const int64_t ttiles = (a.N + Sh::MT - 1) / Sh::MT;
    // the shape that stages the packed validation rows itself addresses them relative to its first row, which
    // must exist: no tile may start past the last validation vector (the padded rows of the pre-pass do not
    // exist for it)
    const int vtiles = Sh::VPACKED ? (a.M + Sh::VT - 1) / Sh::VT : w.Mp / Sh::VT;
    if ((int64_t)vtiles * Sh::VT > w.Mp) return QLESS_ERR_DEVICE;      // weights are read up to the padded width
    const int64_t grid = 8 * (int64_t)vtiles * ((ttiles + 7) / 8);
    if (grid > 0x7FFFFFFF) return QLESS_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((score_mfma_kernel<BITS, WR, WC, WX, NW, F16, VH>), dim3((unsigned)grid), dim3(64 * NW), lds, st, a, w,
                       (int)ttiles, vtiles, AggArgs{});
    return QLESS_OK;
}

// Wide tiles with the group aggregation in the epilogue: one workgroup per train tile.
template <int BITS>
static qless_status launch_mfma_groups(const ScoreArgs &a, void *ws, const AggArgs &ag, hipStream_t st) {
    using Sh = MfmaShape<BITS, 2, 2, 2, 8, false>;
    const MfmaPlan p = mfma_plan(a.N, a.M, a.k, BITS, a.C, true);               // 128-wide validation tiles
    ScorePrep w{};
    unsigned char *base = (unsigned char *)ws;
    w.vexp = (int8_t *)base; w.vw = (float *)(base + p.off_vw); w.vbias = (int32_t *)(base + p.off_vbias);
    w.smax = (unsigned int *)(base + p.off_smax); w.Mp = p.Mp; w.kp = p.kp;
    w.vrow = BITS <= 2 ? p.kp / 2 : p.kp;
    hipLaunchKernelGGL((score_prepare_kernel<BITS, false>), dim3((unsigned)p.Mp, (unsigned)a.C), dim3(256), 0, st, a, w);
    constexpr int kMaxDynamic = (int)kLdsPerCU - 4 * Sh::MT;
    QLESS_LDS_KERNEL((score_mfma_kernel<BITS, 2, 2, 2, 8, false, false, true>), kMaxDynamic);
    size_t lds = (size_t)Sh::NBUF * Sh::BUF;
    const size_t tile = (size_t)Sh::MT * (Sh::VT + 1) * sizeof(float);
    if (tile > lds) lds = tile;
    if (lds > (size_t)kMaxDynamic) return QLESS_ERR_DEVICE;
    const int64_t ttiles = (a.N + Sh::MT - 1) / Sh::MT;
    hipLaunchKernelGGL((score_mfma_kernel<BITS, 2, 2, 2, 8, false, false, true>), dim3((unsigned)ttiles), dim3(64 * 8), lds, st,
                       a, w, (int)ttiles, p.Mp / Sh::VT, ag);
    return launch_status();
}

// Few validation vectors: every workgroup streams its train rows at the same pace, so the launch
// takes ceil(tiles / slots) rounds of equal length.  Pick the tile height (256 or 128 rows) and the
// number of workgroups per compute unit whose last round is fullest.
struct NarrowChoice { int nw, per_cu; };
template <int BITS, int WC, bool VH = false>
static NarrowChoice choose_narrow(int64_t N) {
    const int cus = compute_units();
    NarrowChoice best{8, 2};
    double best_eff = -1.0;
    for (int nw = 8; nw >= 4; nw -= 4) {
        const size_t need = nw == 8 ? (size_t)MfmaShape<BITS, 1, WC, 1, 8, VH>::NBUF * MfmaShape<BITS, 1, WC, 1, 8, VH>::BUF
                                    : (size_t)MfmaShape<BITS, 1, WC, 1, 4, VH>::NBUF * MfmaShape<BITS, 1, WC, 1, 4, VH>::BUF;
        const int64_t tiles = (N + 32 * nw - 1) / (32 * nw);
        int cap = (int)(kLdsPerCU / (need + kStaticLds));
        if (cap > 16 / nw) cap = 16 / nw;                 // at most 16 wavefronts per compute unit
        for (int pc = cap; pc >= 1; --pc) {
            if (pc * nw < 8) break;                       // keep at least 8 wavefronts per compute unit
            const int64_t slots = (int64_t)cus * pc;
            const int64_t rounds = (tiles + slots - 1) / slots;
            const double eff = (double)tiles / (double)(rounds * slots);
            if (eff > best_eff + 1e-9) { best_eff = eff; best = NarrowChoice{nw, pc}; }
        }
    }
    return best;
}

// prepare = false: the workspace still holds the pre-pass of an earlier launch with the same validation
// side and at least as many train rows (the finish kernel leaves the row maxima cleared)
template <int BITS, bool F16 = false>
static qless_status launch_mfma(const ScoreArgs &a, void *ws, hipStream_t st, bool prepare = true, int64_t plan_rows = 0) {
    const MfmaPlan p = mfma_plan(plan_rows > 0 ? plan_rows : a.N, a.M, a.k, BITS, a.C);
    ScorePrep w{};
    unsigned char *base = (unsigned char *)ws;
    w.vexp = (int8_t *)base; w.vw = (float *)(base + p.off_vw); w.vbias = (int32_t *)(base + p.off_vbias);
    w.smax = (unsigned int *)(base + p.off_smax); w.Mp = p.Mp; w.kp = p.kp;
    // a small datastore leaves most compute units without a 256 x 128 tile: 128 x 64 tiles fill four times as
    // many (the expanded validation rows are the same for both shapes; the sign codes' narrow shape stages the
    // packed validation rows itself)
    const bool small = !F16 && p.vt == 128 && ((a.N + 255) / 256) * (p.Mp / 128) * 2 <= compute_units();
    w.vrow = BITS == 1 ? (p.vt > 64 && !small ? p.kp / 2 : 0) : (BITS == 2 ? p.kp / 2 : p.kp);
    if (prepare)
        hipLaunchKernelGGL((score_prepare_kernel<BITS, F16>), dim3((unsigned)p.Mp, (unsigned)a.C), dim3(256), 0, st, a, w);
    qless_status rc;
    if (p.vt == 96) {
        if constexpr (BITS == 1) rc = launch_mfma_shape<BITS, 2, 3, 1, 8, F16>(a, w, 0, st);
        else rc = QLESS_ERR_UNSUPPORTED;
    } else if (p.vt == 128) {
        if (small) rc = launch_mfma_shape<BITS, 1, 2, 1, 4, F16>(a, w, 0, st);
        else rc = launch_mfma_shape<BITS, 2, 2, 2, 8, F16>(a, w, 0, st);
    }
    else if (p.vt == 64) {
        const NarrowChoice c = choose_narrow<BITS, 2>(a.N);
        if (c.nw == 8) rc = launch_mfma_shape<BITS, 1, 2, 1, 8, F16>(a, w, c.per_cu, st);
        else rc = launch_mfma_shape<BITS, 1, 2, 1, 4, F16>(a, w, c.per_cu, st);
    } else if ((BITS == 2 || BITS == 4) && a.M <= 16) {
        // the expanded validation rows of these widths are large next to the train rows of a stage
        const NarrowChoice c = choose_narrow<BITS, 1, true>(a.N);
        if (c.nw == 8) rc = launch_mfma_shape<BITS, 1, 1, 1, 8, F16, true>(a, w, c.per_cu, st);
        else rc = launch_mfma_shape<BITS, 1, 1, 1, 4, F16, true>(a, w, c.per_cu, st);
    } else {
        const NarrowChoice c = choose_narrow<BITS, 1>(a.N);
        if (c.nw == 8) rc = launch_mfma_shape<BITS, 1, 1, 1, 8, F16>(a, w, c.per_cu, st);
        else rc = launch_mfma_shape<BITS, 1, 1, 1, 4, F16>(a, w, c.per_cu, st);
    }
    if (rc != QLESS_OK) return rc;
    if (a.score) {
        int64_t blocks = (a.N + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(score_finish_kernel, dim3((unsigned)blocks), dim3(256), 0, st, w.smax, a.N, a.score);
    }
    return launch_status();
}

// LDS plan of score_stream_mfma_kernel: validation rows and weights, then 8 rings of nb slots
// (nb = 0: does not fit)
constexpr int kStreamWaves = 8;                                      // wavefronts per workgroup of the kernel
// cg: checkpoints per launch, the most whose validation rows leave room for rings of two slots (fewer
// than C: the launches hand their fp32 sums on through a workspace of N x 16 floats)
struct StreamMfmaPlan { int mv, nb, cg; size_t val_bytes, lds; };
static StreamMfmaPlan stream_mfma_plan(int32_t M, int32_t k, int bits, int C) {
    StreamMfmaPlan p{};
    p.mv = M <= 8 ? 8 : 16;
    const size_t slot = 4096;                                        // 32 / bits rows of one 128-byte slice
    for (p.cg = C; p.cg >= 1; --p.cg) {
        p.val_bytes = (((size_t)p.cg * p.mv * ((size_t)k * bits / 8 + 16 + 4)) + 1023) & ~(size_t)1023;
        const size_t room = 158 * 1024 > p.val_bytes ? (158 * 1024 - p.val_bytes) / (kStreamWaves * slot) : 0;
        p.nb = room < 2 ? 0 : (room > 5 ? 5 : (int)room);            // waits: 4 copies per slot x (nb - 2) <= 14
        if (p.nb >= 2) break;
    }
    if (p.cg < 1) { p.cg = 0; p.nb = 0; }
    p.lds = p.val_bytes + (size_t)kStreamWaves * p.nb * slot;
    return p;
}
static size_t stream_mfma_partial_bytes(const StreamMfmaPlan &p, int64_t N, int C) {
    return p.nb >= 2 && p.cg < C ? (size_t)N * 16 * sizeof(float) : 0;
}
static qless_status launch_stream_mfma(const ScoreArgs &a, int bits, const StreamMfmaPlan &sp, float *partial, hipStream_t st) {
    constexpr int NW = kStreamWaves;
    QLESS_LDS_KERNEL((score_stream_mfma_kernel<1, 8, NW, 2>), 158 * 1024);
    QLESS_LDS_KERNEL((score_stream_mfma_kernel<1, 16, NW, 2>), 158 * 1024);
    QLESS_LDS_KERNEL((score_stream_mfma_kernel<2, 8, NW, 1>), 158 * 1024);
    QLESS_LDS_KERNEL((score_stream_mfma_kernel<2, 16, NW, 1>), 158 * 1024);
    // at most one workgroup per compute unit; the rows are dealt out evenly over all wavefronts (a wavefront
    // with work gets about 8 rows or more, what one of its copies covers)
    const int64_t total_rb = (a.N + 7) / 8;
    int64_t groups = compute_units();
    if (groups * NW > total_rb) groups = (total_rb + NW - 1) / NW;
    const int64_t waves = groups * NW;
    const int64_t each = a.N / waves, extra = a.N % waves;
    const dim3 grid((unsigned)groups), block(64 * NW);
    const unsigned ro = (unsigned)sp.val_bytes;
    for (int c0 = 0; c0 < a.C; c0 += sp.cg) {
        const int c1 = c0 + sp.cg < a.C ? c0 + sp.cg : a.C;
        if (bits == 1 && sp.mv == 8) hipLaunchKernelGGL((score_stream_mfma_kernel<1, 8, NW, 2>), grid, block, sp.lds, st, a, each, extra, sp.nb, ro, c0, c1, sp.cg, partial);
        else if (bits == 1) hipLaunchKernelGGL((score_stream_mfma_kernel<1, 16, NW, 2>), grid, block, sp.lds, st, a, each, extra, sp.nb, ro, c0, c1, sp.cg, partial);
        else if (sp.mv == 8) hipLaunchKernelGGL((score_stream_mfma_kernel<2, 8, NW, 1>), grid, block, sp.lds, st, a, each, extra, sp.nb, ro, c0, c1, sp.cg, partial);
        else hipLaunchKernelGGL((score_stream_mfma_kernel<2, 16, NW, 1>), grid, block, sp.lds, st, a, each, extra, sp.nb, ro, c0, c1, sp.cg, partial);
    }
    return launch_status();
}

// LDS plan of score_stream_mfma32_kernel: two validation windows (vr rows of wbv bytes), weights,
// 8 rings of nb slots (nb = 0: does not fit).  Narrower windows cost more barriers, deeper rings
// hide more memory latency: the widest window that leaves room for three slots, else for two.
#ifndef QLESS_STREAM32_MAX_M
#define QLESS_STREAM32_MAX_M 192
#endif
constexpr int kStream32MaxVal = QLESS_STREAM32_MAX_M;                // 1-bit: beyond this the tile kernel takes over
struct Stream32Plan { int wb, nb; size_t val_bytes, lds; };
static Stream32Plan stream_mfma32_plan(int bits, int vb, int vr, int32_t k, int C) {
    Stream32Plan best{};
    const int cb = k * bits / 8;
    const size_t slot = vb == 1 ? (bits == 1 ? 6144 : 5120) : 4096;  // 96, 80 or 64 rows x 64 bytes
    // (the sign codes with one validation block, whose slots are 96 rows, do better with a ring of two and
    // windows four times as wide: fewer barriers; measured 0.246 -> 0.236 ms at M = 32)
    for (int want = (bits == 1 && vb == 1) ? 2 : 3; want >= 2 && best.nb == 0; --want)
        for (int wb = 2048; wb >= 128; wb >>= 1) {
            if (cb % wb) continue;
            const int wbv = bits == 4 ? 2 * wb : wb;
            const size_t val = (((size_t)2 * vr * wbv + (size_t)C * 32 * vb * (bits == 1 ? 8 : 4)) + 1023) & ~(size_t)1023;
            if (val + (size_t)kStream32Waves * want * slot > kLdsPerCU) continue;
            best.wb = wb; best.nb = want; best.val_bytes = val;
            best.lds = val + (size_t)kStream32Waves * want * slot;
            break;
        }
    return best;
}
static int stream32_rows(int32_t mc) { return mc <= 8 ? 8 : (mc <= 16 ? 16 : (mc <= 32 ? 32 : (mc <= 64 ? 64 : 96))); }

template <int BITS, int VB, int VR>
static qless_status launch_stream32_shape(const ScoreArgs &a, const ScorePrep &w, int32_t m0, int32_t mc, hipStream_t st) {
    constexpr int NW = kStream32Waves;
    QLESS_LDS_KERNEL((score_stream_mfma32_kernel<BITS, VB, VR>), (int)kLdsPerCU);
    // at most one workgroup per compute unit; blocks of rows are dealt out evenly over all wavefronts: 8-row
    // blocks, or, where a wavefront gets more than a pass of two 32-row panels, whole panels -- the rows
    // beyond full passes then make one more panel for a few wavefronts (one per compute unit first)
    // instead of a nearly empty extra pass for half of them
    constexpr int kPass = VB == 1 ? (BITS == 1 ? 96 : 80) : 64;      // rows of a pass, as in the kernel
    int64_t groups = compute_units();
    if (groups * NW > (a.N + 7) / 8) groups = ((a.N + 7) / 8 + NW - 1) / NW;
    const int64_t waves = groups * NW;
    const int unit = (kPass != 80 && a.N >= waves * 64) ? 32 : 8;
    const int64_t total_rb = (a.N + unit - 1) / unit;
    const int64_t each = total_rb / waves, extra = total_rb % waves;
    const int npass = (int)(((each + (extra > 0 ? 1 : 0)) * unit + kPass - 1) / kPass);
    const Stream32Plan sp = stream_mfma32_plan(BITS, VB, VR, a.k, a.C);
    hipLaunchKernelGGL((score_stream_mfma32_kernel<BITS, VB, VR>), dim3((unsigned)groups), dim3(64 * NW), sp.lds, st, a,
                       (const int8_t *)w.vexp, (const int32_t *)w.vbias, w.Mp, w.vrow, m0, mc, each, extra, unit, npass, sp.wb, sp.nb,
                       (unsigned)sp.val_bytes);
    return QLESS_OK;
}

// Pre-pass of the sign codes' streaming path: a copy of the validation rows with bits 0 and 2 of every
// nibble swapped, and per row the number of negative codes outside bit 3 of the nibbles (Sv).  One
// workgroup per (validation row, checkpoint); k is a multiple of 512 here.
__global__ void __launch_bounds__(256)
score_permute_kernel(ScoreArgs a, uint32_t *vperm, int32_t *vsum) {
    __shared__ int total;
    const int row = blockIdx.x, ci = blockIdx.y, words = a.k / 32;
    const uint32_t *src = (const uint32_t *)(a.vc[ci] + (int64_t)row * (a.k / 8));
    uint32_t *dst = vperm + ((size_t)ci * a.M + row) * (size_t)words;
    if (threadIdx.x == 0) total = 0;
    __syncthreads();
    int mine = 0;
    for (int t = threadIdx.x; t < words; t += 256) {
        const uint32_t w = src[t];
        dst[t] = (w & 0xAAAAAAAAu) | ((w & 0x11111111u) << 2) | ((w & 0x44444444u) >> 2);
        mine += __popc(w & 0x77777777u);
    }
    if (mine) atomicAdd(&total, mine);
    __syncthreads();
    if (threadIdx.x == 0) vsum[ci * a.M + row] = total;
}
struct PermPlan { size_t off_sum, total; };
static PermPlan perm_plan(int32_t M, int32_t k, int C) {
    PermPlan p{};
    p.off_sum = ((size_t)C * M * (size_t)(k / 8) + 255) & ~(size_t)255;
    p.total = p.off_sum + (((size_t)C * M * 4 + 255) & ~(size_t)255);
    return p;
}

// 1-bit codes: the pre-pass, then one launch per chunk of 64 validation vectors
static qless_status launch_stream_mfma32(const ScoreArgs &a, void *ws, hipStream_t st) {
    const PermPlan pp = perm_plan(a.M, a.k, a.C);
    ScorePrep w{};
    w.vexp = (int8_t *)ws; w.vbias = (int32_t *)((unsigned char *)ws + pp.off_sum);
    hipLaunchKernelGGL(score_permute_kernel, dim3((unsigned)a.M, (unsigned)a.C), dim3(256), 0, st, a, (uint32_t *)w.vexp, w.vbias);
    for (int32_t m0 = 0; m0 < a.M; m0 += kStream32Val) {
        const int32_t mc = a.M - m0 < kStream32Val ? a.M - m0 : kStream32Val;
        const qless_status rc = mc > 32 ? launch_stream32_shape<1, 2, 64>(a, w, m0, mc, st)
                                        : launch_stream32_shape<1, 1, 32>(a, w, m0, mc, st);
        if (rc != QLESS_OK) return rc;
    }
    return launch_status();
}

// 4- and 8-bit codes against at most 96 / 32 validation vectors: one launch; the 4-bit validation rows are
// int8-expanded by the pre-pass into the workspace first
static bool use_stream_i8(int bits, int32_t M, int32_t k, int C) {
    // measured against the tile kernel at N = 270 000: ahead up to 96 validation vectors at 4 bits (one pass of three
    // 32-wide blocks: 1.33 against 1.45 ms at M = 81), up to 32 at 8 bits (M = 40: 1.77 against 1.65 ms; M = 81: equal)
    if (bits < 4 || M > (bits == 4 ? 96 : 32) || (k * bits / 8) % 128 != 0) return false;
    const int vr = stream32_rows(M);
    return stream_mfma32_plan(bits, vr > 32 ? vr / 32 : 1, vr, k, C).nb >= 2;
}
template <int BITS>
static qless_status launch_stream_i8(const ScoreArgs &a, void *ws, hipStream_t st) {
    ScorePrep w{};
    if (BITS == 4) {
        const MfmaPlan p = mfma_plan(a.N, a.M, a.k, BITS, a.C);
        unsigned char *base = (unsigned char *)ws;
        w.vexp = (int8_t *)base; w.vw = (float *)(base + p.off_vw); w.vbias = (int32_t *)(base + p.off_vbias);
        w.smax = (unsigned int *)(base + p.off_smax); w.Mp = p.Mp; w.kp = p.kp; w.vrow = p.kp;
        hipLaunchKernelGGL((score_prepare_kernel<BITS, false>), dim3((unsigned)p.Mp, (unsigned)a.C), dim3(256), 0, st, a, w);
    }
    const int vr = stream32_rows(a.M);
    qless_status rc;
    if (vr == 8) rc = launch_stream32_shape<BITS, 1, 8>(a, w, 0, a.M, st);
    else if (vr == 16) rc = launch_stream32_shape<BITS, 1, 16>(a, w, 0, a.M, st);
    else if (vr == 32) rc = launch_stream32_shape<BITS, 1, 32>(a, w, 0, a.M, st);
    else if (vr == 64) rc = launch_stream32_shape<BITS, 2, 64>(a, w, 0, a.M, st);
    else rc = launch_stream32_shape<BITS, 3, 96>(a, w, 0, a.M, st);
    return rc != QLESS_OK ? rc : launch_status();
}

template <int BITS, int RT, int CT, int TY, int TX>
static void launch_popcount(const ScoreArgs &a, hipStream_t st) {
    constexpr int TN = RT * TY, TM = CT * TX, SW = BITS * 16 + 4, RSTEP = 256 / (8 * BITS);
    constexpr int TMP = ((TM + RSTEP - 1) / RSTEP) * RSTEP;
    const size_t lds = 2 * (size_t)(TN + TMP) * SW * 4;
    const unsigned grid = (unsigned)((a.N + TN - 1) / TN);
    hipLaunchKernelGGL((score_popcount_kernel<BITS, RT, CT, TY, TX>), dim3(grid), dim3(256), lds, st, a);
}

// ------------------------------------------------------------------------------------------
// Mixed precision: b-bit train codes against bfloat16 validation rows.  The train codes of a block
// of rows are written out as bfloat16 values (small integers: exact) and the block is scored by the
// bfloat16 matrix-core kernel of the 16-bit comparator with the code norms as train factors.
// ------------------------------------------------------------------------------------------
constexpr int64_t kMixedRows = 8192;           // train rows per block

struct ExpandArgs {
    const unsigned char *tc[QLESS_MAX_CHECKPOINTS];
    uint16_t *out;                             // [C][rows][k] bfloat16
    int64_t r0, rows;
    int32_t k;
    int C;
};

__device__ inline uint32_t bf16_pair(int lo, int hi) {                // exact for |values| < 256
    return (__float_as_uint((float)lo) >> 16) | (__float_as_uint((float)hi) & 0xFFFF0000u);
}

// one thread per 8 consecutive codes of a row
template <int BITS>
__global__ void __launch_bounds__(256)
mixed_expand_kernel(ExpandArgs e) {
    const int per_row = e.k / 8;
    const int64_t total = (int64_t)e.C * e.rows * per_row;
    const int64_t cb = (int64_t)e.k * BITS / 8;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int g = (int)(i % per_row);
        const int64_t rr = i / per_row;
        const int64_t r = rr % e.rows;
        const int ci = (int)(rr / e.rows);
        const unsigned char *src = e.tc[ci] + (e.r0 + r) * cb;
        int q[8];
        if (BITS == 8) {
            const uint2 w = *(const uint2 *)(src + 8 * g);
#pragma unroll
            for (int t = 0; t < 4; ++t) { q[t] = (int)(int8_t)(w.x >> (8 * t)); q[4 + t] = (int)(int8_t)(w.y >> (8 * t)); }
        } else if (BITS == 4) {
            const uint32_t w = *(const uint32_t *)(src + 4 * g);
#pragma unroll
            for (int t = 0; t < 8; ++t) q[t] = ((int)(w << (28 - 4 * t))) >> 28;       // sign-extended nibble t
        } else {
            const unsigned sg = src[(BITS == 2 ? e.k / 8 : 0) + g];
            const unsigned nz = BITS == 2 ? src[g] : 0xFFu;
#pragma unroll
            for (int t = 0; t < 8; ++t) q[t] = ((nz >> t) & 1u) ? (((sg >> t) & 1u) ? -1 : 1) : 0;
        }
        uint4 o;
        o.x = bf16_pair(q[0], q[1]); o.y = bf16_pair(q[2], q[3]); o.z = bf16_pair(q[4], q[5]); o.w = bf16_pair(q[6], q[7]);
        *(uint4 *)(e.out + ((size_t)ci * e.rows + r) * (size_t)e.k + 8 * g) = o;
    }
}

struct MixedPlan { int64_t rows; size_t off_tiles, total; };
static MixedPlan mixed_plan(int64_t N, int32_t M, int32_t k, int C) {
    MixedPlan p{};
    p.rows = N < kMixedRows ? (N > 0 ? N : 1) : kMixedRows;
    size_t o = (size_t)C * (size_t)p.rows * (size_t)k * 2;
    o = (o + 255) & ~(size_t)255;
    p.off_tiles = o;
    p.total = o + mfma_plan(p.rows, M, 2 * k, 8, C).total;
    return p;
}

}  // namespace qless

using namespace qless;

extern "C" size_t qless_score_mixed_workspace(int64_t N, int32_t M, int32_t k, int bits, int C) {
    if (N < 0 || M < 1 || k <= 0 || k > 32768 || C < 1 || !valid_bits(bits)) return 0;
    return mixed_plan(N, M, k, C).total;
}

extern "C" qless_status qless_score_mixed(const void *const *train_codes, const float *const *train_rnorm,
                                          const void *const *val16, const float *eta, int C, int64_t N, int32_t M,
                                          int32_t k, int bits, float *score, float *full, void *ws, size_t ws_bytes,
                                          void *stream) {
    if (!train_codes || !train_rnorm || !val16 || !eta) return QLESS_ERR_INVALID_ARG;
    if (C < 1 || N < 0 || M < 1 || k <= 0) return QLESS_ERR_INVALID_ARG;
    if (!score && !full) return QLESS_ERR_INVALID_ARG;
    if (C > QLESS_MAX_CHECKPOINTS || !valid_bits(bits) || k % 64 != 0 || k > 32768) return QLESS_ERR_UNSUPPORTED;
    if (N > (int64_t)0x7FFFFFFF) return QLESS_ERR_UNSUPPORTED;
    for (int i = 0; i < C; ++i) {
        if (!val16[i] || (N > 0 && (!train_codes[i] || !train_rnorm[i]))) return QLESS_ERR_INVALID_ARG;
        if ((uintptr_t)val16[i] % 16 || (uintptr_t)train_codes[i] % 16) return QLESS_ERR_INVALID_ARG;
    }
    if (N == 0) return QLESS_OK;
    const MixedPlan mp = mixed_plan(N, M, k, C);
    if (!ws || ws_bytes < mp.total || (uintptr_t)ws % 16) return QLESS_ERR_WORKSPACE;
    const qless_status ready = device_ready();
    if (ready != QLESS_OK) return ready;
    hipStream_t st = (hipStream_t)stream;
    ExpandArgs e{};
    e.out = (uint16_t *)ws; e.k = k; e.C = C;
    for (int i = 0; i < C; ++i) e.tc[i] = (const unsigned char *)train_codes[i];
    for (int64_t r0 = 0; r0 < N; r0 += mp.rows) {
        const int64_t rows = N - r0 < mp.rows ? N - r0 : mp.rows;
        e.r0 = r0; e.rows = rows;
        int64_t blocks = ((int64_t)C * rows * (k / 8) + 255) / 256;
        if (blocks > 16384) blocks = 16384;
        switch (bits) {
            case 8: hipLaunchKernelGGL(mixed_expand_kernel<8>, dim3((unsigned)blocks), dim3(256), 0, st, e); break;
            case 4: hipLaunchKernelGGL(mixed_expand_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, st, e); break;
            case 2: hipLaunchKernelGGL(mixed_expand_kernel<2>, dim3((unsigned)blocks), dim3(256), 0, st, e); break;
            default: hipLaunchKernelGGL(mixed_expand_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, st, e); break;
        }
        ScoreArgs a{};
        for (int i = 0; i < C; ++i) {
            a.tc[i] = (const unsigned char *)(e.out + (size_t)i * rows * (size_t)k);
            a.vc[i] = (const unsigned char *)val16[i];
            a.tr[i] = train_rnorm[i] + r0; a.vr[i] = nullptr; a.eta[i] = eta[i];
        }
        a.C = C; a.N = rows; a.M = M; a.k = 2 * k;                    // k in bytes from here on
        a.score = score ? score + r0 : nullptr;
        a.full = full ? full + r0 * (int64_t)M : nullptr;
        const qless_status rc = launch_mfma<8, true>(a, (unsigned char *)ws + mp.off_tiles, st, r0 == 0, mp.rows);
        if (rc != QLESS_OK) return rc;
    }
    return launch_status();
}

extern "C" size_t qless_score_workspace(int64_t N, int32_t M, int32_t k, int bits, int C) {
    if (N < 0 || M < 1 || k <= 0 || C < 1 || !valid_bits(bits)) return 0;
    size_t need = 0;
    if (bits <= 2 && M <= kStreamMfmaVal && k % 128 == 0)      // checkpoint groups hand their sums on through the workspace
        need = stream_mfma_partial_bytes(stream_mfma_plan(M, k, bits, C), N, C);
    if (bits == 1 && M <= kStream32MaxVal && k % 512 == 0 && stream_mfma32_plan(1, 2, 64, k, C).nb >= 2) {
        const size_t perm = perm_plan(M, k, C).total;           // the streaming path's copy of the validation rows
        if (perm > need) need = perm;
    }
    if (!use_mfma_path(bits, M, k)) return need;
    const size_t tiles = mfma_plan(N, M, k, bits, C).total;
    return tiles > need ? tiles : need;
}

extern "C" qless_status qless_score(const void *const *train_codes, const float *const *train_rnorm,
                                    const void *const *val_codes, const float *const *val_rnorm,
                                    const float *eta, int C, int64_t N, int32_t M, int32_t k, int bits,
                                    float *score, float *full, void *ws, size_t ws_bytes, void *stream) {
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
    const qless_status ready = device_ready();            // LDS limits of the kernels, once per device
    if (ready != QLESS_OK) return ready;
    if (bits <= 2 && M <= kStreamMfmaVal && k % 128 == 0) {
        const StreamMfmaPlan sp = stream_mfma_plan(M, k, bits, C);
        if (sp.nb >= 2) {
            const size_t need = stream_mfma_partial_bytes(sp, N, C);
            if (need && (!ws || ws_bytes < need)) return QLESS_ERR_WORKSPACE;
            if (need && (uintptr_t)ws % 16) return QLESS_ERR_WORKSPACE;
            return launch_stream_mfma(a, bits, sp, (float *)ws, st);
        }
    }
    if (bits == 1 && M <= kStream32MaxVal && k % 512 == 0 && stream_mfma32_plan(1, 2, 64, k, C).nb >= 2) {
        if (!ws || ws_bytes < perm_plan(M, k, C).total || (uintptr_t)ws % 16) return QLESS_ERR_WORKSPACE;
        return launch_stream_mfma32(a, ws, st);
    }
    if (use_mfma_path(bits, M, k)) {
        const size_t need = mfma_plan(N, M, k, bits, C).total;
        if (!ws || ws_bytes < need) return QLESS_ERR_WORKSPACE;
        if ((uintptr_t)ws % 16) return QLESS_ERR_WORKSPACE;
        if (N > (int64_t)0x7FFFFFFF) return QLESS_ERR_UNSUPPORTED;
        if (use_stream_i8(bits, M, k, C)) return bits == 8 ? launch_stream_i8<8>(a, ws, st) : launch_stream_i8<4>(a, ws, st);
        if (bits == 8) return launch_mfma<8>(a, ws, st);
        if (bits == 4) return launch_mfma<4>(a, ws, st);
        if (bits == 2) return launch_mfma<2>(a, ws, st);
        return launch_mfma<1>(a, ws, st);
    }
    // bit-plane codes with rows that are not multiples of 16 bytes, or a handful of val vectors whose
    // codes do not fit in LDS: popcount kernels
    if (bits == 1) {
        if (M > 32) launch_popcount<1, 8, 4, 16, 16>(a, st);
        else if (M > 8) launch_popcount<1, 8, 4, 32, 8>(a, st);
        else launch_popcount<1, 8, 1, 32, 8>(a, st);
    } else if (bits == 2) {
        if (M > 32) launch_popcount<2, 4, 4, 16, 16>(a, st);
        else if (M > 8) launch_popcount<2, 4, 4, 32, 8>(a, st);
        else launch_popcount<2, 8, 1, 32, 8>(a, st);
    }
    return launch_status();
}

// Influence aggregated over groups of validation columns without the N x M matrix in memory.
static bool groups_fused(int32_t M, int32_t k, int bits) { return M > 64 && (bits >= 4 || k % 128 == 0); }

extern "C" size_t qless_score_groups_workspace(int64_t N, int32_t M, int32_t k, int bits, int C) {
    if (N < 0 || M < 1 || k <= 0 || C < 1 || !valid_bits(bits)) return 0;
    if (groups_fused(M, k, bits)) return mfma_plan(N, M, k, bits, C, true).total;
    // few validation vectors (or bit planes that are not whole 16-byte chunks): the matrix is small; it is
    // written to the workspace by the ordinary paths and aggregated from there
    size_t full = ((size_t)N * (size_t)M * sizeof(float) + 255) & ~(size_t)255;
    return full + qless_score_workspace(N, M, k, bits, C) + 16;
}

extern "C" qless_status qless_score_groups(const void *const *train_codes, const float *const *train_rnorm,
                                           const void *const *val_codes, const float *const *val_rnorm,
                                           const float *eta, int C, int64_t N, int32_t M, int32_t k, int bits,
                                           const int32_t *group_end, int T, qless_agg mode, float *out,
                                           void *ws, size_t ws_bytes, void *stream) {
    if (!train_codes || !train_rnorm || !val_codes || !val_rnorm || !eta || !group_end) return QLESS_ERR_INVALID_ARG;
    if (C < 1 || N < 0 || M < 1 || k <= 0 || T < 1) return QLESS_ERR_INVALID_ARG;
    if (mode != QLESS_AGG_MAX && mode != QLESS_AGG_MEAN) return QLESS_ERR_UNSUPPORTED;
    if (T > QLESS_MAX_GROUPS) return QLESS_ERR_UNSUPPORTED;
    if (C > QLESS_MAX_CHECKPOINTS || !valid_bits(bits) || k % 64 != 0 || k > 65536) return QLESS_ERR_UNSUPPORTED;
    if (N > (int64_t)0x7FFFFFFF) return QLESS_ERR_UNSUPPORTED;
    AggArgs ag{};
    for (int t = 0; t < T; ++t) {
        const int32_t g0 = t ? group_end[t - 1] : 0;
        if (group_end[t] <= g0 || group_end[t] > M) return QLESS_ERR_INVALID_ARG;
        ag.ge.end[t] = group_end[t];
    }
    if (group_end[T - 1] != M) return QLESS_ERR_INVALID_ARG;
    if (N == 0) return QLESS_OK;
    if (!out) return QLESS_ERR_INVALID_ARG;
    const size_t need = qless_score_groups_workspace(N, M, k, bits, C);
    if (!ws || ws_bytes < need || (uintptr_t)ws % 16) return QLESS_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    ag.T = T; ag.mean = mode == QLESS_AGG_MEAN ? 1 : 0; ag.gout = out;
    if (!groups_fused(M, k, bits)) {
        float *full = (float *)ws;
        const size_t full_bytes = ((size_t)N * (size_t)M * sizeof(float) + 255) & ~(size_t)255;
        const qless_status rc = qless_score(train_codes, train_rnorm, val_codes, val_rnorm, eta, C, N, M, k, bits,
                                            nullptr, full, (unsigned char *)ws + full_bytes, ws_bytes - full_bytes, stream);
        if (rc != QLESS_OK) return rc;
        return aggregate_rows(full, N, M, ag.ge, T, ag.mean, out, st);
    }
    ScoreArgs a{};
    for (int i = 0; i < C; ++i) {
        if (!val_codes[i] || !val_rnorm[i] || !train_codes[i] || !train_rnorm[i]) return QLESS_ERR_INVALID_ARG;
        if ((uintptr_t)val_codes[i] % 16 || (uintptr_t)train_codes[i] % 16) return QLESS_ERR_INVALID_ARG;
        a.tc[i] = (const unsigned char *)train_codes[i]; a.vc[i] = (const unsigned char *)val_codes[i];
        a.tr[i] = train_rnorm[i]; a.vr[i] = val_rnorm[i]; a.eta[i] = eta[i];
    }
    a.C = C; a.N = N; a.M = M; a.k = k; a.score = nullptr; a.full = nullptr;
    const qless_status ready = device_ready();
    if (ready != QLESS_OK) return ready;
    switch (bits) {
        case 8: return launch_mfma_groups<8>(a, ws, ag, st);
        case 4: return launch_mfma_groups<4>(a, ws, ag, st);
        case 2: return launch_mfma_groups<2>(a, ws, ag, st);
        default: return launch_mfma_groups<1>(a, ws, ag, st);
    }
}

// 16-bit LESS comparator: bfloat16 rows scored by the 8-bit kernel geometry on 2k bytes per row.
extern "C" size_t qless_score16_workspace(int64_t N, int32_t M, int32_t k, int C) {
    if (N < 0 || M < 1 || k <= 0 || k > 32768 || C < 1) return 0;
    return mfma_plan(N, M, 2 * k, 8, C).total;
}

extern "C" qless_status qless_score16(const void *const *train16, const void *const *val16, const float *eta,
                                      int C, int64_t N, int32_t M, int32_t k, float *score, float *full,
                                      void *ws, size_t ws_bytes, void *stream) {
    if (!train16 || !val16 || !eta) return QLESS_ERR_INVALID_ARG;
    if (C < 1 || N < 0 || M < 1 || k <= 0) return QLESS_ERR_INVALID_ARG;
    if (!score && !full) return QLESS_ERR_INVALID_ARG;
    if (C > QLESS_MAX_CHECKPOINTS || k % 64 != 0 || k > 32768) return QLESS_ERR_UNSUPPORTED;
    if (N > (int64_t)0x7FFFFFFF) return QLESS_ERR_UNSUPPORTED;
    ScoreArgs a{};
    for (int i = 0; i < C; ++i) {
        if (!val16[i] || (N > 0 && !train16[i])) return QLESS_ERR_INVALID_ARG;
        if ((uintptr_t)val16[i] % 16 || (uintptr_t)train16[i] % 16) return QLESS_ERR_INVALID_ARG;
        a.tc[i] = (const unsigned char *)train16[i]; a.vc[i] = (const unsigned char *)val16[i];
        a.tr[i] = nullptr; a.vr[i] = nullptr; a.eta[i] = eta[i];
    }
    a.C = C; a.N = N; a.M = M; a.k = 2 * k; a.score = score; a.full = full;     // k in bytes from here on
    if (N == 0) return QLESS_OK;
    const size_t need = mfma_plan(N, M, a.k, 8, C).total;
    if (!ws || ws_bytes < need) return QLESS_ERR_WORKSPACE;
    if ((uintptr_t)ws % 16) return QLESS_ERR_WORKSPACE;
    const qless_status ready = device_ready();
    if (ready != QLESS_OK) return ready;
    return launch_mfma<8, true>(a, ws, (hipStream_t)stream);
}
