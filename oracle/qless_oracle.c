/*
 * QLESS oracle: a plain, slow, obviously-correct CPU statement of what the gradient-datastore and
 * influence path computes.  TEST INFRASTRUCTURE ONLY: nothing in the product path may call, link
 * or import this file; only the test-suite, the smoke check and the benchmark's CPU-baseline leg do.
 * It shares no code, header, table or constant generator with the HIP library.
 *
 * What each function follows (QLESS paper, arXiv 2502.01703):
 *   oracle_project      Eq.(1), Sec. 2.2 / Sec. 2.4 / Sec. 3.1:  g = R x,  R in R^{k x d} random,
 *                       Rademacher or Gaussian-like; R is a pure function of (seed, m, j).
 *   oracle_quantize     Eq.(4),(5), Sec. 2.3 / Sec. 3.1: S = max|g|, alpha = 2^(b-1)-1,
 *                       q = round(alpha g / S); b = 1 is the sign code of Table 3 / Sec. 5.
 *   oracle_quantize_absmean  Sec. 5 / Table 3 variant; formula is this build's reading (see there).
 *   oracle_score        Eq.(6),(7), Sec. 3.2: cosine of the quantised vectors, learning-rate
 *                       weighted sum over checkpoints; then max over validation vectors.
 *   oracle_topk         Sec. 4.1 ("select the top 5 %"): largest scores, ties by smaller index.
 *   oracle_aggregate    maximum / mean of the pairwise influences over groups of validation examples
 *                       (no formula in the paper: parity unpinned)
 *   oracle_less_cosine  Eq.(2),(3), Sec. 2.2: the un-quantised LESS influence (comparator only).
 *   oracle_less16_*     the same comparator from a stored 16-bit (bfloat16) datastore (Table 1 baseline).
 *   oracle_score_mixed  Eq.(7) with b-bit train codes against 16-bit validation rows (this build's variant).
 *
 * Arithmetic: projection sums in fp64 in index order and rounds once to fp32; integer dot
 * products in int64; the score epilogue is a fixed sequence of single fp32 operations (this file
 * must be compiled with -ffp-contract=off).  Parallelism: OpenMP over independent outputs only.
 *
 * Pins: tests/test_oracle_*.py (brute force, closed forms, invariants, paper's storage column).
 * Unpinned: nothing in this file depends on the paper's accuracy tables (they need the paper's
 * models and datasets) -- those are "parity unpinned" and not reproduced.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_BAD_ARG 1

/* ------------------------------------------------------------------------------------------
 * Random matrix R(seed, m, j).  The paper only says "randomly initialised", "Gaussian or
 * Rademacher" (Sec. 2.2, 2.4); the generator below is this build's reading, written from its
 * prose specification:
 *
 *   mix(x):  x ^= x>>16; x *= 0x85EBCA6B; x ^= x>>13; x *= 0xC2B2AE35; x ^= x>>16   (mod 2^32)
 *   s0 = mix(seed_lo + 0x9E3779B9),  s1 = mix(seed_hi ^ s0 ^ 0x7F4A7C15)
 *   keyA(m) = mix(s1 + m*0x9E3779B1),  keyB(m) = mix(keyA(m) ^ s0 ^ 0x5BD1E995)
 *   word(m, w, salt):  x = keyA(m) + (w*0x9E3779B1) + salt*0x68E31DA4
 *                      x ^= x>>16; x *= 0x85EBCA6B; x ^= keyB(m);
 *                      x ^= x>>13; x *= 0xC2B2AE35; x ^= x>>16
 *   Rademacher:  R[m][j] = -1 if bit beta(j mod 32) of word(m, floor(j/32), 0) is set, else +1,
 *                beta(c) = 4*(c mod 8) + 3 - floor(c/8).
 *   Gaussian-like: see oracle_gauss_value().
 * ------------------------------------------------------------------------------------------ */
static uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= 0x85EBCA6Bu; x ^= x >> 13; x *= 0xC2B2AE35u; x ^= x >> 16;
    return x;
}
typedef struct { uint32_t a, b; } rowkey_t;

static rowkey_t row_key(uint64_t seed, uint32_t m) {
    uint32_t lo = (uint32_t)(seed & 0xFFFFFFFFu), hi = (uint32_t)(seed >> 32);
    uint32_t s0 = mix32(lo + 0x9E3779B9u);
    uint32_t s1 = mix32(hi ^ s0 ^ 0x7F4A7C15u);
    rowkey_t r;
    r.a = mix32(s1 + m * 0x9E3779B1u);
    r.b = mix32(r.a ^ s0 ^ 0x5BD1E995u);
    return r;
}
static uint32_t key_word(rowkey_t key, uint32_t w, uint32_t salt) {
    uint32_t x = key.a + w * 0x9E3779B1u + salt * 0x68E31DA4u;
    x ^= x >> 16; x *= 0x85EBCA6Bu; x ^= key.b;
    x ^= x >> 13; x *= 0xC2B2AE35u; x ^= x >> 16;
    return x;
}
uint32_t oracle_word(uint64_t seed, uint32_t m, uint32_t w, uint32_t salt) {
    return key_word(row_key(seed, m), w, salt);
}
static int beta_bit(int c) { return 4 * (c & 7) + 3 - (c >> 3); }

/* Gaussian-like entries: a 256-entry table of standard-normal quantiles, each rounded to the
 * nearest bfloat16 (so the entry is exactly representable in the GPU's operand type):
 *   T[i] = bf16_rne( Phi^{-1}((i + 1/2) / 256) ),  i = 0..255
 * R[m][j] = T[ byte (j mod 4) of word(m, floor(j/4), 1) ]   (byte 0 = least significant).
 * Phi^{-1} is found by bisection on Phi(x) = erfc(-x/sqrt 2)/2 in fp64. */
static double g_table[256];
static int g_table_ready = 0;
static double bf16_round(double v) {
    float f = (float)v; uint32_t u; memcpy(&u, &f, 4);
    uint32_t lsb = (u >> 16) & 1u; u += 0x7FFFu + lsb; u &= 0xFFFF0000u;
    memcpy(&f, &u, 4); return (double)f;
}
static void build_gauss_table(void) {
    for (int i = 0; i < 256; ++i) {
        double p = (i + 0.5) / 256.0, lo = -10.0, hi = 10.0;
        for (int it = 0; it < 200; ++it) {
            double mid = 0.5 * (lo + hi);
            double c = 0.5 * erfc(-mid / sqrt(2.0));
            if (c < p) lo = mid; else hi = mid;
        }
        g_table[i] = bf16_round(0.5 * (lo + hi));
    }
    g_table_ready = 1;
}
void oracle_gauss_table(double *out256) {
    if (!g_table_ready) build_gauss_table();
    memcpy(out256, g_table, sizeof(g_table));
}

/* R[m][j] as a double, straight from the definition (slow; used by tests and the row sampler). */
double oracle_r_entry(uint64_t seed, int kind, uint32_t m, uint64_t j) {
    rowkey_t key = row_key(seed, m);
    if (kind == 0) {
        uint32_t h = key_word(key, (uint32_t)(j >> 5), 0u);
        return ((h >> beta_bit((int)(j & 31))) & 1u) ? -1.0 : 1.0;
    }
    if (!g_table_ready) build_gauss_table();
    uint32_t h = key_word(key, (uint32_t)(j >> 2), 1u);
    return g_table[(h >> (8 * (int)(j & 3))) & 0xFFu];
}

static double load_g(const void *G, int dtype, int64_t idx) {
    if (dtype == 0) return (double)((const float *)G)[idx];
    uint32_t u = ((uint32_t)((const uint16_t *)G)[idx]) << 16;   /* bfloat16 -> fp32, exact */
    float f; memcpy(&f, &u, 4); return (double)f;
}

/* Eq.(1): out[i][r] = sum_{j<d_len} R[rows[r]][d_offset + j] * G[i][j], fp64, index order.
 * rows == NULL means rows 0..nrows-1.  out is n x nrows, row-major, fp64. */
int oracle_project_rows(const void *G, int dtype, int64_t n, int64_t d_len, int64_t ldG,
                        int64_t d_offset, int kind, uint64_t seed,
                        const int32_t *rows, int32_t nrows, double *out) {
    if (!G || !out || n < 0 || d_len < 0 || nrows < 0 || (dtype != 0 && dtype != 1) ||
        (kind != 0 && kind != 1) || d_offset < 0 || ldG < d_len) return ORACLE_BAD_ARG;
    /* the word counter has 32 bits: 32 columns per Rademacher word, 4 per Gaussian word; past these
     * limits columns would repeat, so such a column range is outside the definition of R */
    if (d_offset + d_len > (kind == 0 ? ((int64_t)1 << 37) : ((int64_t)1 << 34))) return ORACLE_BAD_ARG;
    if (kind == 1 && !g_table_ready) build_gauss_table();
    int64_t r;
    #pragma omp parallel for schedule(dynamic, 1)
    for (r = 0; r < nrows; ++r) {
        uint32_t m = rows ? (uint32_t)rows[r] : (uint32_t)r;
        rowkey_t key = row_key(seed, m);
        double *rrow = (double *)malloc(sizeof(double) * 4096);
        double *acc = (double *)calloc((size_t)(n > 0 ? n : 1), sizeof(double));
        /* walk j in index order, 4096 entries of R at a time (R is materialised, never G) */
        for (int64_t j0 = 0; j0 < d_len; j0 += 4096) {
            int64_t len = d_len - j0 < 4096 ? d_len - j0 : 4096;
            for (int64_t t = 0; t < len; ++t) {
                uint64_t j = (uint64_t)(d_offset + j0 + t);
                if (kind == 0) {
                    uint32_t h = key_word(key, (uint32_t)(j >> 5), 0u);
                    rrow[t] = ((h >> beta_bit((int)(j & 31))) & 1u) ? -1.0 : 1.0;
                } else {
                    uint32_t h = key_word(key, (uint32_t)(j >> 2), 1u);
                    rrow[t] = g_table[(h >> (8 * (int)(j & 3))) & 0xFFu];
                }
            }
            for (int64_t i = 0; i < n; ++i) {
                double a = acc[i];
                for (int64_t t = 0; t < len; ++t)
                    a += rrow[t] * load_g(G, dtype, i * ldG + j0 + t);
                acc[i] = a;
            }
        }
        for (int64_t i = 0; i < n; ++i) out[i * (int64_t)nrows + r] = acc[i];
        free(acc); free(rrow);
    }
    return ORACLE_OK;
}

/* Eq.(1), all k rows; P (n x k, leading dimension ldP) receives fl32(sum) or, when accumulate
 * is non-zero, fl32((double)P_old + sum). */
int oracle_project(const void *G, int dtype, int64_t n, int64_t d_len, int64_t ldG,
                   int64_t d_offset, int32_t k, int kind, uint64_t seed, int accumulate,
                   float *P, int64_t ldP) {
    if (!P || k <= 0 || ldP < k) return ORACLE_BAD_ARG;
    double *tmp = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1) * (size_t)k);
    if (!tmp) return ORACLE_BAD_ARG;
    int rc = oracle_project_rows(G, dtype, n, d_len, ldG, d_offset, kind, seed, NULL, k, tmp);
    if (rc == ORACLE_OK)
        for (int64_t i = 0; i < n; ++i)
            for (int32_t m = 0; m < k; ++m) {
                double v = tmp[i * (int64_t)k + m];
                if (accumulate) v += (double)P[i * ldP + m];
                P[i * ldP + m] = (float)v;
            }
    free(tmp);
    return rc;
}

/* ------------------------------------------------------------------------------------------
 * Quantiser, Eq.(4),(5).  Canonical arithmetic (what the datastore holds):
 *   S = max_m |P_m| (exact),  scale = fl32(alpha / S),  q = clamp(rne(fl32(P * scale)), +-alpha)
 *   b = 1: q = -1 if P < 0 else +1 (the sign code; Eq.(5) degenerates at alpha = 0)
 *   S == 0: q = 0 (b >= 2), all +1 (b = 1)
 *   n2 = sum q^2 (int64);  rnorm = fl32(1 / sqrt((double) n2)),  0 when n2 == 0.
 * Packed layout (little-endian element order, k a multiple of 64):
 *   8-bit: int8 at byte m.   4-bit: two's-complement nibbles, element 2t low, 2t+1 high.
 *   2-bit: two bit-planes, k/8 bytes "non-zero" then k/8 bytes "negative", element m at bit
 *          m%8 of byte m/8.   1-bit: the "negative" plane only.
 * ------------------------------------------------------------------------------------------ */
static int alpha_of(int bits) { return (1 << (bits - 1)) - 1; }
int64_t oracle_code_bytes(int32_t k, int bits) { return (int64_t)k * bits / 8; }

static void pack_row(const int8_t *q, int32_t k, int bits, uint8_t *dst) {
    memset(dst, 0, (size_t)((int64_t)k * bits / 8));
    for (int32_t m = 0; m < k; ++m) {
        int v = q[m];
        if (bits == 8) dst[m] = (uint8_t)(int8_t)v;
        else if (bits == 4) dst[m >> 1] |= (uint8_t)((v & 0xF) << (4 * (m & 1)));
        else if (bits == 2) {
            if (v != 0) dst[m >> 3] |= (uint8_t)(1u << (m & 7));
            if (v < 0) dst[k / 8 + (m >> 3)] |= (uint8_t)(1u << (m & 7));
        } else { if (v < 0) dst[m >> 3] |= (uint8_t)(1u << (m & 7)); }
    }
}
static void unpack_row(const uint8_t *src, int32_t k, int bits, int8_t *q) {
    for (int32_t m = 0; m < k; ++m) {
        int v;
        if (bits == 8) v = (int8_t)src[m];
        else if (bits == 4) { v = (src[m >> 1] >> (4 * (m & 1))) & 0xF; if (v & 8) v -= 16; }
        else if (bits == 2) {
            int nz = (src[m >> 3] >> (m & 7)) & 1, sg = (src[k / 8 + (m >> 3)] >> (m & 7)) & 1;
            v = nz ? (sg ? -1 : 1) : 0;
        } else v = ((src[m >> 3] >> (m & 7)) & 1) ? -1 : 1;
        q[m] = (int8_t)v;
    }
}
int oracle_unpack(const uint8_t *codes, int64_t n, int32_t k, int bits, int8_t *q) {
    if (!codes || !q || k <= 0 || k % 64 || (bits != 1 && bits != 2 && bits != 4 && bits != 8))
        return ORACLE_BAD_ARG;
    int64_t cb = oracle_code_bytes(k, bits);
    for (int64_t i = 0; i < n; ++i) unpack_row(codes + i * cb, k, bits, q + i * (int64_t)k);
    return ORACLE_OK;
}
int oracle_pack(const int8_t *q, int64_t n, int32_t k, int bits, uint8_t *codes) {
    if (!codes || !q || k <= 0 || k % 64 || (bits != 1 && bits != 2 && bits != 4 && bits != 8))
        return ORACLE_BAD_ARG;
    int64_t cb = oracle_code_bytes(k, bits);
    for (int64_t i = 0; i < n; ++i) pack_row(q + i * (int64_t)k, k, bits, codes + i * cb);
    return ORACLE_OK;
}

/* literal != 0 selects the paper-literal real-number formula evaluated in fp64,
 * q = rne(alpha * (double)P / (double)S), instead of the canonical fp32 sequence. */
static void quantize_row(const float *p, int32_t k, int bits, int literal, int8_t *q, float *S_out) {
    float S = 0.0f;
    for (int32_t m = 0; m < k; ++m) { float a = fabsf(p[m]); if (a > S) S = a; }
    *S_out = S;
    if (bits == 1) { for (int32_t m = 0; m < k; ++m) q[m] = (p[m] < 0.0f) ? -1 : 1; return; }
    int alpha = alpha_of(bits);
    if (S == 0.0f) { memset(q, 0, (size_t)k); return; }
    if (literal) {
        for (int32_t m = 0; m < k; ++m) {
            double r = nearbyint((double)alpha * (double)p[m] / (double)S);
            if (r > alpha) r = alpha; if (r < -alpha) r = -alpha;
            q[m] = (int8_t)r;
        }
    } else {
        volatile float scale = (float)alpha / S;
        for (int32_t m = 0; m < k; ++m) {
            volatile float t = p[m] * scale;
            float r = nearbyintf(t);
            if (r > (float)alpha) r = (float)alpha; if (r < -(float)alpha) r = -(float)alpha;
            q[m] = (int8_t)r;
        }
    }
}
/* ------------------------------------------------------------------------------------------
 * Absmean variant (Sec. 5, Table 3: the scale follows the mean absolute value instead of the
 * maximum, which empties the zero bin at low widths).  The paper prints no formula; this build's
 * reading (parity unpinned against the paper) is the BitNet-style rule
 *     S = mean_m |g_m|,   q = clamp(rne(g / S), -alpha, alpha),   b = 1: the sign code.
 * So that S does not depend on the order of a floating-point summation, the mean is defined in
 * fixed point: with A = max|g| = f * 2^E, f in [0.5, 1),
 *     u_m = trunc(|g_m| * 2^(32-E))   (an integer below 2^32),   U = sum_m u_m   (exact),
 *     S = fl32( fl64(U) / k * 2^(E-32) ),   scale = fl32(1 / S),   q = clamp(rne(fl32(g * scale))).
 * A zero vector gives S = 0 and zero codes (all +1 for b = 1).
 * ------------------------------------------------------------------------------------------ */
static void quantize_row_absmean(const float *p, int32_t k, int bits, int8_t *q, float *S_out) {
    float A = 0.0f;
    for (int32_t m = 0; m < k; ++m) { float a = fabsf(p[m]); if (a > A) A = a; }
    if (bits == 1) for (int32_t m = 0; m < k; ++m) q[m] = (p[m] < 0.0f) ? -1 : 1;
    else memset(q, 0, (size_t)k);
    *S_out = 0.0f;
    if (A == 0.0f) return;
    int E;
    (void)frexpf(A, &E);
    uint64_t U = 0;
    for (int32_t m = 0; m < k; ++m) U += (uint64_t)ldexpf(fabsf(p[m]), 32 - E);
    double mean = ldexp((double)U / (double)k, E - 32);
    float S = (float)mean;
    *S_out = S;
    if (bits == 1 || S == 0.0f) return;
    int alpha = alpha_of(bits);
    volatile float scale = 1.0f / S;
    for (int32_t m = 0; m < k; ++m) {
        volatile float t = p[m] * scale;
        float r = nearbyintf(t);
        if (r > (float)alpha) r = (float)alpha; if (r < -(float)alpha) r = -(float)alpha;
        q[m] = (int8_t)r;
    }
}
int oracle_quantize_absmean(const float *P, int64_t ldP, int64_t n, int32_t k, int bits,
                            uint8_t *codes, int8_t *q_out, float *S, float *rnorm) {
    if (!P || !S || !rnorm || k <= 0 || k % 64 || ldP < k ||
        (bits != 1 && bits != 2 && bits != 4 && bits != 8)) return ORACLE_BAD_ARG;
    int64_t cb = oracle_code_bytes(k, bits);
    int64_t i;
    #pragma omp parallel for
    for (i = 0; i < n; ++i) {
        int8_t *q = (int8_t *)malloc((size_t)k);
        quantize_row_absmean(P + i * ldP, k, bits, q, S + i);
        int64_t n2 = 0;
        for (int32_t m = 0; m < k; ++m) n2 += (int64_t)q[m] * q[m];
        rnorm[i] = n2 ? (float)(1.0 / sqrt((double)n2)) : 0.0f;
        if (codes) pack_row(q, k, bits, codes + i * cb);
        if (q_out) memcpy(q_out + i * (int64_t)k, q, (size_t)k);
        free(q);
    }
    return ORACLE_OK;
}

int oracle_quantize_unpacked(const float *P, int64_t ldP, int64_t n, int32_t k, int bits,
                             int literal, int8_t *q, float *S) {
    if (!P || !q || !S || k <= 0 || ldP < k || (bits != 1 && bits != 2 && bits != 4 && bits != 8))
        return ORACLE_BAD_ARG;
    int64_t i;
    #pragma omp parallel for
    for (i = 0; i < n; ++i) quantize_row(P + i * ldP, k, bits, literal, q + i * (int64_t)k, S + i);
    return ORACLE_OK;
}
int oracle_quantize(const float *P, int64_t ldP, int64_t n, int32_t k, int bits,
                    uint8_t *codes, float *S, float *rnorm) {
    if (!P || !codes || !S || !rnorm || k <= 0 || k % 64 || ldP < k ||
        (bits != 1 && bits != 2 && bits != 4 && bits != 8)) return ORACLE_BAD_ARG;
    int64_t cb = oracle_code_bytes(k, bits);
    int64_t i;
    #pragma omp parallel for
    for (i = 0; i < n; ++i) {
        int8_t *q = (int8_t *)malloc((size_t)k);
        quantize_row(P + i * ldP, k, bits, 0, q, S + i);
        int64_t n2 = 0;
        for (int32_t m = 0; m < k; ++m) n2 += (int64_t)q[m] * q[m];
        rnorm[i] = n2 ? (float)(1.0 / sqrt((double)n2)) : 0.0f;
        pack_row(q, k, bits, codes + i * cb);
        free(q);
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------
 * Influence, Eq.(6),(7) + max over validation vectors.
 *   D_i(z,z') = sum_m q_{z,i,m} q_{z',i,m}            exact integer, from unpacked codes
 *   w'_i(z')  = eta_i (*) rnorm'_i(z')
 *   t_i       = ((float)D_i (*) rnorm_i(z)) (*) w'_i(z')
 *   acc       = ((0 (+) t_0) (+) t_1) (+) ...         single fp32 operations, this order
 *   score[z]  = max_{z'} acc(z,z')
 * full (N x M) is optional and receives acc.
 * ------------------------------------------------------------------------------------------ */
int oracle_score(const uint8_t *const *train_codes, const float *const *train_rnorm,
                 const uint8_t *const *val_codes, const float *const *val_rnorm,
                 const float *eta, int C, int64_t N, int32_t M, int32_t k, int bits,
                 float *score, float *full) {
    if (!train_codes || !train_rnorm || !val_codes || !val_rnorm || !eta || C <= 0 || N < 0 ||
        M <= 0 || k <= 0 || k % 64 || (bits != 1 && bits != 2 && bits != 4 && bits != 8) ||
        (!score && !full)) return ORACLE_BAD_ARG;
    int64_t cb = oracle_code_bytes(k, bits);
    int8_t *vq = (int8_t *)malloc((size_t)C * (size_t)M * (size_t)k);
    if (!vq) return ORACLE_BAD_ARG;
    for (int i = 0; i < C; ++i)
        for (int32_t v = 0; v < M; ++v)
            unpack_row(val_codes[i] + (int64_t)v * cb, k, bits, vq + ((int64_t)i * M + v) * k);
    int64_t z;
    #pragma omp parallel for schedule(static)
    for (z = 0; z < N; ++z) {
        int8_t *tq = (int8_t *)malloc((size_t)C * (size_t)k);
        for (int i = 0; i < C; ++i) unpack_row(train_codes[i] + z * cb, k, bits, tq + (int64_t)i * k);
        float best = 0.0f;
        for (int32_t v = 0; v < M; ++v) {
            volatile float acc = 0.0f;
            for (int i = 0; i < C; ++i) {
                const int8_t *a = tq + (int64_t)i * k, *b = vq + ((int64_t)i * M + v) * k;
                int64_t D = 0;
                for (int32_t m = 0; m < k; ++m) D += (int64_t)a[m] * (int64_t)b[m];
                volatile float w = eta[i] * val_rnorm[i][v];
                volatile float t = (float)D * train_rnorm[i][z];
                volatile float t2 = t * w;
                acc = acc + t2;
            }
            float a = acc;
            if (full) full[z * (int64_t)M + v] = a;
            if (v == 0 || a > best) best = a;
        }
        if (score) score[z] = best;
        free(tq);
    }
    free(vq);
    return ORACLE_OK;
}

/* Top-k: the k_sel largest scores, ordered by (score descending, index ascending). */
typedef struct { float s; int64_t i; } sc_t;
static int cmp_sc(const void *pa, const void *pb) {
    const sc_t *a = (const sc_t *)pa, *b = (const sc_t *)pb;
    if (a->s > b->s) return -1; if (a->s < b->s) return 1;
    return (a->i < b->i) ? -1 : (a->i > b->i);
}
int oracle_topk(const float *score, int64_t N, int64_t k_sel, int64_t *idx, float *val) {
    if (!score || !idx || N < 0 || k_sel < 0 || k_sel > N) return ORACLE_BAD_ARG;
    sc_t *a = (sc_t *)malloc(sizeof(sc_t) * (size_t)(N > 0 ? N : 1));
    for (int64_t i = 0; i < N; ++i) { a[i].s = score[i]; a[i].i = i; }
    qsort(a, (size_t)N, sizeof(sc_t), cmp_sc);   /* total order on (s, i): result is unique */
    for (int64_t t = 0; t < k_sel; ++t) { idx[t] = a[t].i; if (val) val[t] = a[t].s; }
    free(a);
    return ORACLE_OK;
}

/* Aggregation of the pairwise influences over groups of validation examples (Sec. 4.1 ranks by
 * the influence summed over checkpoints and its benchmarks have sub-tasks, but the paper gives no formula:
 * parity unpinned against the paper; the benchmark spec fixes the maximum over all validation examples).
 * Group t is the columns [group_end[t-1], group_end[t]) of full (group_end[-1] = 0).
 *   mode 0: out[z][t] = the maximum of the group's entries (the first of equal ones, compared with >)
 *   mode 1: out[z][t] = fl32(s / n), s the fp32 sum of the entries in column order from +0, n their number */
int oracle_aggregate(const float *full, int64_t N, int32_t M, const int32_t *group_end, int T, int mode,
                     float *out) {
    if (!full || !group_end || !out || N < 0 || M < 1 || T < 1 || (mode != 0 && mode != 1)) return ORACLE_BAD_ARG;
    for (int t = 0; t < T; ++t) {
        const int32_t g0 = t ? group_end[t - 1] : 0;
        if (group_end[t] <= g0 || group_end[t] > M) return ORACLE_BAD_ARG;
    }
    if (group_end[T - 1] != M) return ORACLE_BAD_ARG;
    for (int64_t z = 0; z < N; ++z)
        for (int t = 0; t < T; ++t) {
            const int32_t g0 = t ? group_end[t - 1] : 0, g1 = group_end[t];
            const float *row = full + z * (int64_t)M;
            if (mode == 0) {
                float m = row[g0];
                for (int32_t j = g0 + 1; j < g1; ++j) if (row[j] > m) m = row[j];
                out[z * (int64_t)T + t] = m;
            } else {
                volatile float s = 0.0f;               /* one fp32 rounding per addition */
                for (int32_t j = g0; j < g1; ++j) s = s + row[j];
                const volatile float n = (float)(g1 - g0);
                out[z * (int64_t)T + t] = s / n;
            }
        }
    return ORACLE_OK;
}

/* LESS comparator, Eq.(2),(3): sum_i eta_i <g'/|g'|, g/|g|> on un-quantised fp32 projections,
 * in fp64.  out is N x M. */
int oracle_less_cosine(const float *const *train_P, const float *const *val_P, const float *eta,
                       int C, int64_t N, int32_t M, int32_t k, double *out) {
    if (!train_P || !val_P || !eta || !out || C <= 0 || k <= 0) return ORACLE_BAD_ARG;
    int64_t z;
    #pragma omp parallel for
    for (z = 0; z < N; ++z)
        for (int32_t v = 0; v < M; ++v) {
            double acc = 0.0;
            for (int i = 0; i < C; ++i) {
                const float *a = train_P[i] + z * (int64_t)k, *b = val_P[i] + (int64_t)v * k;
                double ab = 0, aa = 0, bb = 0;
                for (int32_t m = 0; m < k; ++m) {
                    ab += (double)a[m] * b[m]; aa += (double)a[m] * a[m]; bb += (double)b[m] * b[m];
                }
                if (aa > 0 && bb > 0) acc += (double)eta[i] * ab / (sqrt(aa) * sqrt(bb));
            }
            out[z * (int64_t)M + v] = acc;
        }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------
 * LESS comparator in its stored 16-bit form (Sec. 2.2 / Table 1: the baseline keeps the normalised
 * projected gradients at 16 bits).  This build's reading of "16-bit" is bfloat16:
 *   store:  y = bf16_rne( fl32( x * fl32(1 / sqrt(sum_m x_m^2)) ) ),  the sum in fp64, index order;
 *           a zero vector is stored as zeros.  Output: bfloat16 bit patterns.
 *   score:  acc(z,z') = sum_i eta_i * <y_{z,i}, y_{z',i}>   in fp64 from the stored values (Eq.(2),(3)
 *           with the cosine's denominators already folded into the store);  score = max_z' acc.
 * ------------------------------------------------------------------------------------------ */
static uint16_t bf16_bits_rne(float f) {
    uint32_t u; memcpy(&u, &f, 4);
    uint32_t r = u + 0x7FFFu + ((u >> 16) & 1u);      /* finite inputs only */
    return (uint16_t)(r >> 16);
}
static double bf16_value(uint16_t b) {
    uint32_t u = (uint32_t)b << 16; float f; memcpy(&f, &u, 4);
    return (double)f;
}
int oracle_less16_store(const float *P, int64_t ldP, int64_t n, int32_t k, uint16_t *out) {
    if (!P || !out || k <= 0 || ldP < k) return ORACLE_BAD_ARG;
    int64_t i;
    #pragma omp parallel for
    for (i = 0; i < n; ++i) {
        const float *x = P + i * ldP;
        double ss = 0.0;
        for (int32_t m = 0; m < k; ++m) ss += (double)x[m] * (double)x[m];
        volatile float inv = ss > 0.0 ? (float)(1.0 / sqrt(ss)) : 0.0f;
        for (int32_t m = 0; m < k; ++m) {
            volatile float y = x[m] * inv;
            out[i * (int64_t)k + m] = bf16_bits_rne(y);
        }
    }
    return ORACLE_OK;
}
int oracle_less16_score(const uint16_t *const *train, const uint16_t *const *val, const float *eta,
                        int C, int64_t N, int32_t M, int32_t k, double *score, double *full) {
    if (!train || !val || !eta || C <= 0 || N < 0 || M <= 0 || k <= 0 || (!score && !full)) return ORACLE_BAD_ARG;
    int64_t z;
    #pragma omp parallel for
    for (z = 0; z < N; ++z) {
        double best = 0.0;
        for (int32_t v = 0; v < M; ++v) {
            double acc = 0.0;
            for (int i = 0; i < C; ++i) {
                const uint16_t *a = train[i] + z * (int64_t)k, *b = val[i] + (int64_t)v * k;
                double d = 0.0;
                for (int32_t m = 0; m < k; ++m) d += bf16_value(a[m]) * bf16_value(b[m]);
                acc += (double)eta[i] * d;
            }
            if (full) full[z * (int64_t)M + v] = acc;
            if (v == 0 || acc > best) best = acc;
        }
        if (score) score[z] = best;
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------
 * Mixed-precision influence: the train datastore keeps its b-bit codes (Sec. 3.1) while the few
 * validation gradients stay at 16 bits as in LESS (Sec. 2.2: stored unit-normalised; read as
 * bfloat16 like oracle_less16_store).  Eq.(7) with the validation factor of Eq.(6) replaced by
 * the stored unit vector y' of Eq.(2):
 *   acc(z,z') = sum_i eta_i * rnorm_i(z) * sum_m q_{z,i,m} * y'_{z',i,m},   score[z] = max_z' acc(z,z')
 * everything in fp64 from the stored values (codes as integers, rnorm as the stored fp32, y' as
 * the stored bfloat16).  The paper quantises both sides alike (Sec. 3.2); this variant is this
 * build's reading of "validation gradients kept at higher precision" and is pinned by brute
 * force and by the cases in which it must coincide with oracle_score / oracle_less16_score.
 * ------------------------------------------------------------------------------------------ */
int oracle_score_mixed(const uint8_t *const *train_codes, const float *const *train_rnorm,
                       const uint16_t *const *val16, const float *eta, int C, int64_t N, int32_t M,
                       int32_t k, int bits, double *score, double *full) {
    if (!train_codes || !train_rnorm || !val16 || !eta || C <= 0 || N < 0 || M <= 0 || k <= 0 || k % 64 ||
        (bits != 1 && bits != 2 && bits != 4 && bits != 8) || (!score && !full)) return ORACLE_BAD_ARG;
    int64_t cb = oracle_code_bytes(k, bits);
    int64_t z;
    #pragma omp parallel for schedule(static)
    for (z = 0; z < N; ++z) {
        int8_t *tq = (int8_t *)malloc((size_t)C * (size_t)k);
        for (int i = 0; i < C; ++i) unpack_row(train_codes[i] + z * cb, k, bits, tq + (int64_t)i * k);
        double best = 0.0;
        for (int32_t v = 0; v < M; ++v) {
            double acc = 0.0;
            for (int i = 0; i < C; ++i) {
                const int8_t *a = tq + (int64_t)i * k;
                const uint16_t *b = val16[i] + (int64_t)v * k;
                double d = 0.0;
                for (int32_t m = 0; m < k; ++m) d += (double)a[m] * bf16_value(b[m]);
                acc += (double)eta[i] * (double)train_rnorm[i][z] * d;
            }
            if (full) full[z * (int64_t)M + v] = acc;
            if (v == 0 || acc > best) best = acc;
        }
        if (score) score[z] = best;
        free(tq);
    }
    return ORACLE_OK;
}

int oracle_num_threads(void) {
    int n = 1;
    #pragma omp parallel
    {
        #pragma omp master
        n =
#ifdef _OPENMP
            omp_get_num_threads();
#else
            1;
#endif
    }
    return n;
}
