/*
 * qless.h -- C ABI of the MI355X (gfx950) QLESS gradient-datastore and influence engine.
 *
 * The calls follow the pipeline of the QLESS paper (arXiv 2502.01703):
 *   qless_project   Eq.(1)        random projection of per-example gradients, d -> k
 *   qless_quantize  Eq.(4),(5)    absmax b-bit quantisation into the packed gradient datastore
 *   qless_project_quantize        both of the above in one call
 *   qless_score     Eq.(6),(7)    normalised quantised cosine, learning-rate weighted over
 *                                 checkpoints, reduced by max over validation examples
 *   qless_topk      Sec. 4.1      selection of the highest-scoring training examples
 *   qless_aggregate Sec. 4.1      maximum / mean of the influences over groups of validation examples
 *
 * Conventions common to every call
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are ordinary
 *     host memory read before the call returns.  The library allocates and frees nothing on
 *     the device.  Its only state is set up once per device (see qless_init): the dynamic-LDS
 *     limits of its kernels and the address of one fixed device array; no result depends on it.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream);
 *     no call synchronises.  Outputs are valid once the caller has synchronised the stream.
 *   - Every call returns a qless_status.  Arguments are validated on the host before anything
 *     is launched; on any status other than QLESS_OK no output has been touched.
 *   - Workspace sizes come from the matching *_workspace() query with the same shape
 *     arguments; a workspace may be reused by later calls on the same stream.  A workspace that is
 *     missing, too small or not aligned as its call states gives QLESS_ERR_WORKSPACE.
 *   - HIP graph capture: every entry point only enqueues kernels (no allocation, no memset, no copy,
 *     no synchronisation) and may be captured, provided qless_init() has run on that device before
 *     the capture begins (without it the first launching call on a device does the set-up, which
 *     is host-side work that must not fall inside a capture).
 *   - Inputs must be finite (no NaN/Inf); this is not checked.
 */
#ifndef QLESS_H
#define QLESS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QLESS_OK = 0,
    QLESS_ERR_INVALID_ARG = 1,   /* null pointer, negative size, leading dimension too small */
    QLESS_ERR_UNSUPPORTED = 2,   /* bits not in {1,2,4,8}, k not a multiple of 64, ... */
    QLESS_ERR_WORKSPACE = 3,     /* workspace missing, smaller than the query's answer, or misaligned */
    QLESS_ERR_DEVICE = 4         /* the HIP runtime reported an error at launch */
} qless_status;

typedef enum { QLESS_F32 = 0, QLESS_BF16 = 1 } qless_dtype;
typedef enum { QLESS_RADEMACHER = 0, QLESS_GAUSSIAN = 1 } qless_proj;

#define QLESS_MAX_CHECKPOINTS 16

const char *qless_status_string(qless_status s);

/* One-time set-up for the current device (hipSetDevice): allows the library's kernels their dynamic
 * LDS (up to 160 KB per workgroup) and looks up the device address of the array behind
 * qless_topk_noalloc.  Host-side only: nothing is launched, allocated or synchronised.  Optional:
 * every entry point that launches such a kernel does the same on its first call on a device; call
 * it explicitly before capturing entry points into a HIP graph.  Thread-safe; later calls return at
 * once.  QLESS_ERR_DEVICE if there is no usable device. */
qless_status qless_init(void);

/* ---------------------------------------------------------------------------------------------
 * Projection, Eq.(1) (Sec. 2.2; matrix families of Sec. 2.4):  P[i][m] = sum_j R[m][d_offset+j] G[i][j]
 *
 * R is k x (any number of columns), never stored: entry (m, j) is a pure function of
 * (seed, m, j).  QLESS_RADEMACHER: entries +-1 (unscaled).  QLESS_GAUSSIAN: entries from a
 * 256-level table of standard-normal quantiles rounded to bfloat16.
 *
 *   G          device, n x d_len, row-major with leading dimension ldG (elements), dtype dt
 *   d_offset   column of R that G's column 0 multiplies; lets a caller feed a long gradient in
 *              slices (per layer).  Must be a multiple of 32; d_offset + d_len <= 2^36 for
 *              QLESS_RADEMACHER and <= 2^34 for QLESS_GAUSSIAN (its generator numbers words of
 *              four columns with 32 bits; beyond that columns would repeat): QLESS_ERR_UNSUPPORTED.
 *   k          projected dimension, a positive multiple of 64
 *   accumulate 0: P = R G      non-zero: P = P + R G   (slices are summed in call order)
 *   P          device, n x k fp32, leading dimension ldP >= k
 *   ws         device workspace, 16-byte aligned, of at least qless_project_workspace(n, d_len, k) bytes
 * Arithmetic: gradient values enter as bfloat16 (fp32 input is rounded to nearest-even),
 * products are exact, sums are fp32 in a fixed order (results are run-to-run identical).
 * n == 0 or d_len == 0 is valid (P is zero-filled unless accumulating).
 * ------------------------------------------------------------------------------------------- */
size_t qless_project_workspace(int64_t n, int64_t d_len, int32_t k);
qless_status qless_project(const void *G, qless_dtype dt, int64_t n, int64_t d_len, int64_t ldG,
                           int64_t d_offset, int32_t k, qless_proj kind, uint64_t seed,
                           int accumulate, float *P, int64_t ldP,
                           void *ws, size_t ws_bytes, void *stream);

/* Diagnostic: the generator's raw 32-bit words, out[r * nwords + t] = word(seed, m0 + r, w0 + t,
 * salt) for r < nrows, t < nwords (device, uint32).  Rademacher signs are read from salt 0
 * (32 columns per word), Gaussian table indices from salt 1 (4 columns per word). */
qless_status qless_generator_words(uint64_t seed, uint32_t m0, int32_t nrows, uint32_t w0,
                                   int32_t nwords, uint32_t salt, uint32_t *out, void *stream);
/* Diagnostic: the 256 Gaussian table values as fp32 (host output). */
qless_status qless_gaussian_table(float *host_out256);

/* ---------------------------------------------------------------------------------------------
 * Quantisation, Eq.(4),(5) (Sec. 2.3, 3.1); bits = 1 is the sign code (Table 3, Sec. 5).
 * Per row:  S = max_m |P[m]|;  bits >= 2: q = clamp(rne(P * fl32(alpha / S)), -alpha, alpha) with
 * alpha = 2^(bits-1) - 1;  bits == 1: q = -1 if P < 0 else +1.  A zero row gives q = 0
 * (bits >= 2) or all +1 (bits == 1) and S = 0.
 *
 *   P      device, n x k fp32, leading dimension ldP >= k;  k a positive multiple of 64
 *   codes  device, 4-byte aligned (QLESS_ERR_INVALID_ARG otherwise), n rows of k*bits/8 bytes, packed:
 *            8: int8 at byte m        4: two's-complement nibbles, element 2t low, 2t+1 high
 *            2: k/8 bytes "non-zero" plane then k/8 bytes "negative" plane, element m at bit
 *               m%8 of byte m/8       1: the "negative" plane only
 *   S      device, n fp32: the stored scale of Sec. 3.1
 *   rnorm  device, n fp32: 1 / ||q||_2  (0 for an all-zero code), the factor of Eq.(6)
 * ------------------------------------------------------------------------------------------- */
qless_status qless_quantize(const float *P, int64_t ldP, int64_t n, int32_t k, int bits,
                            void *codes, float *S, float *rnorm, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Absmean variant of the quantiser (Sec. 5 and Table 3 compare it with absmax; the paper gives no
 * formula, the rule below is this library's reading):
 *   S = mean_m |P[m]|;  bits >= 2: q = clamp(rne(P * fl32(1 / S)), -alpha, alpha);  bits == 1: the sign code.
 * The mean is evaluated in fixed point (32 fractional bits below the binary exponent of max|P|, each
 * term truncated, the integer sum divided by k in fp64 and rounded to fp32), so S does not depend on
 * the order of the additions.  Arguments, packed layout and rnorm as for qless_quantize; S receives
 * the mean.  Codes of either variant are scored by qless_score unchanged.
 * ------------------------------------------------------------------------------------------- */
qless_status qless_quantize_absmean(const float *P, int64_t ldP, int64_t n, int32_t k, int bits,
                                    void *codes, float *S, float *rnorm, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Datastore build in one call (Sec. 3.1: project, then quantise and store): Eq.(1) followed by
 * Eq.(4),(5) on the same rows without a round trip of P through memory.  Arguments as in
 * qless_project (no accumulate: the call covers a whole gradient or one stand-alone slice; d_len >= 1)
 * and qless_quantize.  codes, S, rnorm are bit-identical to qless_project followed by
 * qless_quantize with the same arguments.
 *   P     device, n x k fp32 with leading dimension ldP >= k receiving the projection, or NULL
 *   ws    device workspace, 16-byte aligned, of at least qless_project_workspace(n, d_len, k) bytes
 * ------------------------------------------------------------------------------------------- */
qless_status qless_project_quantize(const void *G, qless_dtype dt, int64_t n, int64_t d_len, int64_t ldG,
                                    int64_t d_offset, int32_t k, qless_proj kind, uint64_t seed,
                                    int bits, void *codes, float *S, float *rnorm,
                                    float *P, int64_t ldP, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * The same datastore build for gradients that arrive in slices (Sec. 3.1 projects and stores each
 * gradient as it is extracted; per-example gradients come layer by layer).  One call per slice, in any
 * fixed order of the caller's choosing:
 *   P = (first ? 0 : P) + R[:, d_offset : d_offset + d_len] G        (fp32, the slice's own partial sums
 *                                                                     added first, then the running P)
 * and on the slice with last != 0, after that addition, P = P + P_other (if given) and then
 * Eq.(4),(5) on the rows of P into codes, S, rnorm.  The result is the same bits as qless_project with
 * accumulate over the same slices in the same order followed by qless_quantize; on the last slice the
 * additions and the quantiser run in one kernel (k <= 16384), so that slice's partial sums and the
 * final P are not read back from memory.
 *   P        device, n x k fp32 accumulator with leading dimension ldP >= k; holds the projection afterwards
 *   P_other  device, n x k fp32 with leading dimension ldO, or NULL; only with last != 0.  It lets a caller
 *            run alternate slices on two streams, each stream with its own accumulator and workspace
 *            (so that one slice's tail overlaps the next one's start), and join the two sums in a fixed
 *            order; the caller orders the last call after the other stream's work (an event).
 *   codes, S, rnorm, bits   as for qless_quantize; read only when last != 0
 *   ws       as for qless_project (16-byte aligned, qless_project_workspace(n, d_len, k) bytes)
 * d_len == 0 is valid (the slice adds nothing).
 * ------------------------------------------------------------------------------------------- */
qless_status qless_project_quantize_slice(const void *G, qless_dtype dt, int64_t n, int64_t d_len, int64_t ldG,
                                          int64_t d_offset, int32_t k, qless_proj kind, uint64_t seed,
                                          int first, int last, float *P, int64_t ldP,
                                          const float *P_other, int64_t ldO, int bits, void *codes,
                                          float *S, float *rnorm, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Influence scores, Eq.(6),(7) (Sec. 3.2) and the max over validation examples:
 *   acc(z, z') = sum_{i<C} eta[i] * <q_{z,i}, q_{z',i}> * rnorm_i(z) * rnorm'_i(z')
 *   score[z]   = max_{z' < M} acc(z, z')
 * The integer dot product is exact; the fp32 epilogue is
 *   ((float)D * rnorm_i(z)) * (eta[i] * rnorm'_i(z')),  added over i = 0..C-1 starting from +0,
 * each operation rounded once (no fused multiply-add).
 *
 *   train_codes, val_codes   host arrays of C device pointers to N (resp. M) packed rows, each
 *                            pointer 16-byte aligned
 *   train_rnorm, val_rnorm   host arrays of C device pointers to N (resp. M) fp32
 *   eta        host, C learning-rate weights;  1 <= C <= QLESS_MAX_CHECKPOINTS
 *   k          a multiple of 64, at most 65536 (integer dot products stay inside int32)
 *   score      device, N fp32, or NULL
 *   full       device, N x M fp32 row-major receiving acc, or NULL (at least one of the two)
 *   ws         device workspace, 16-byte aligned, of at least qless_score_workspace(N, M, k, bits, C)
 *              bytes (0 for the configurations that need none).  It holds the validation codes
 *              expanded for the tiled matrix-core path and the running row maxima; for sign codes
 *              against 17 .. 192 validation vectors a bit-permuted copy of the validation codes and
 *              their per-row counts; the path that streams bit-plane codes against at most 16
 *              validation vectors leaves it untouched, unless the checkpoints are scored in groups of
 *              launches (their validation rows do not all fit in LDS): then it carries N x 16 fp32
 *              sums from one launch to the next.
 * N == 0 is valid; M >= 1.  Whichever kernels a shape selects, the results are the same bits.  With
 * more than 64 validation vectors a call may consist of several launches that update score in
 * place: score and full are complete once the stream has run the whole call.
 * ------------------------------------------------------------------------------------------- */
size_t qless_score_workspace(int64_t N, int32_t M, int32_t k, int bits, int C);
qless_status qless_score(const void *const *train_codes, const float *const *train_rnorm,
                         const void *const *val_codes, const float *const *val_rnorm,
                         const float *eta, int C, int64_t N, int32_t M, int32_t k, int bits,
                         float *score, float *full, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * The 16-bit LESS comparator (Sec. 2.2, Eq.(2),(3); the "16-bit" row of Table 1), for measuring the
 * un-quantised baseline on the same machine.  "16-bit" is read as bfloat16.
 *
 * qless_normalize16:  out[i][m] = bf16_rne( fl32( P[i][m] * fl32(1 / ||P_i||_2) ) ), the squared norm
 *   summed in fp64; a zero row is stored as zeros.
 *     P    device, n x k fp32, leading dimension ldP >= k;  k a positive multiple of 64
 *     out  device, n x k bfloat16 (dense rows)
 * qless_score16:  acc(z, z') = sum_{i<C} eta[i] * <y_{z,i}, y_{z',i}> over the stored rows, products exact,
 *   sums in fp32 on the matrix cores (order unspecified: results agree with an fp64 evaluation to
 *   about 1e-5, not bit for bit);  score[z] = max_{z'} acc(z, z').
 *     train16, val16  host arrays of C device pointers to N (resp. M) bfloat16 rows of k, 16-byte aligned
 *     eta             host, C weights;  k a multiple of 64, at most 32768
 *     score, full, ws, ws_bytes, stream   as for qless_score; workspace from qless_score16_workspace
 * ------------------------------------------------------------------------------------------- */
qless_status qless_normalize16(const float *P, int64_t ldP, int64_t n, int32_t k, void *out, void *stream);
size_t qless_score16_workspace(int64_t N, int32_t M, int32_t k, int C);
qless_status qless_score16(const void *const *train16, const void *const *val16, const float *eta,
                           int C, int64_t N, int32_t M, int32_t k, float *score, float *full,
                           void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Mixed-precision influence: the train datastore keeps its b-bit codes (Sec. 3.1, Eq.(4),(5)), the
 * validation gradients stay at 16 bits as stored by qless_normalize16 (Sec. 2.2, Eq.(2)); Eq.(7) with
 * the unit vector y' in place of the normalised validation code:
 *   acc(z, z') = sum_{i<C} eta[i] * rnorm_i(z) * <q_{z,i}, y'_{z',i}>,    score[z] = max_{z'} acc(z, z')
 * (the paper quantises both sides alike; this variant is the library's own).  Products are exact, sums
 * are fp32 on the matrix cores in an unspecified order, the epilogue is (D * rnorm_i(z)) * eta[i] added
 * over i in order: results agree with an fp64 evaluation to sum|eta| * (k/16 + 24) * 2^-24, not bit for bit.
 *   train_codes, train_rnorm   as for qless_score (host arrays of C device pointers; codes 16-byte aligned)
 *   val16      host array of C device pointers to M bfloat16 rows of k, 16-byte aligned
 *   k          a multiple of 64, at most 32768;  bits in {1, 2, 4, 8};  1 <= C <= QLESS_MAX_CHECKPOINTS
 *   score, full, stream   as for qless_score
 *   ws         device workspace, 16-byte aligned, of at least qless_score_mixed_workspace(N, M, k, bits, C)
 *              bytes: blocks of 8192 train rows are written out as bfloat16 values there and scored in turn
 * ------------------------------------------------------------------------------------------- */
size_t qless_score_mixed_workspace(int64_t N, int32_t M, int32_t k, int bits, int C);
qless_status qless_score_mixed(const void *const *train_codes, const float *const *train_rnorm,
                               const void *const *val16, const float *eta, int C, int64_t N, int32_t M,
                               int32_t k, int bits, float *score, float *full,
                               void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Selection (Sec. 4.1: the top 5 % by score): indices of the k_sel largest scores ordered by
 * (score descending, index ascending); +0 and -0 compare equal.
 *
 *   score  device, N fp32 (N < 2^32)     idx  device, k_sel int64
 *   val    device, k_sel fp32 receiving score[idx[t]], or NULL
 *   ws     device workspace, 8-byte aligned, of at least qless_topk_workspace(N, k_sel) bytes
 * 0 <= k_sel <= N.  Errors: QLESS_ERR_INVALID_ARG (sizes, null pointers), QLESS_ERR_WORKSPACE
 * (ws missing, too small or misaligned), QLESS_ERR_UNSUPPORTED (N >= 2^32); nothing is launched then.
 * ------------------------------------------------------------------------------------------- */
size_t qless_topk_workspace(int64_t N, int64_t k_sel);
qless_status qless_topk(const float *score, int64_t N, int64_t k_sel, int64_t *idx, float *val,
                        void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * qless_topk for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, same
 * results and same errors as qless_topk, without ws: the workspace is a fixed array inside the
 * library's device image (about 0.8 MB on every GPU the library runs on, held until the process
 * ends).  Limits: N <= QLESS_TOPK_NOALLOC_MAX_N and k_sel <= QLESS_TOPK_NOALLOC_MAX_SEL, beyond
 * them QLESS_ERR_UNSUPPORTED and nothing is launched.  The call allocates and frees nothing.  All
 * calls on one GPU share that GPU's array: two calls that overlap on one GPU (different streams
 * without ordering between them) race; calls on one stream, or ordered by events, are safe, and a
 * call needs nothing of what the call before left in the array.  The array's address is looked up
 * on the first call on each device (no allocation, no device work).
 * ------------------------------------------------------------------------------------------- */
#define QLESS_TOPK_NOALLOC_MAX_N 4194304
#define QLESS_TOPK_NOALLOC_MAX_SEL 65536
qless_status qless_topk_noalloc(const float *score, int64_t N, int64_t k_sel, int64_t *idx, float *val,
                                void *stream);

/* ---------------------------------------------------------------------------------------------
 * Aggregation of pairwise influences over groups of validation examples (Sec. 4.1 ranks the training
 * examples by their influence summed over checkpoints and evaluates on benchmarks with sub-tasks,
 * without a formula for combining validation examples; qless_score reduces by the maximum over all
 * of them).  From the
 * full matrix of qless_score / qless_score16:
 *   QLESS_AGG_MAX   out[z][t] = max of full[z][j] over group t (the first of equal values)
 *   QLESS_AGG_MEAN  out[z][t] = fl32(s / n), s = the fp32 sum of the group's entries in column order
 *                   starting from +0 (one rounding per addition), n = their number
 * Group t is the columns [group_end[t-1], group_end[t]) with group_end[-1] = 0.
 *
 *   full       device, N x M fp32 row-major          out   device, N x T fp32 row-major
 *   group_end  host, T strictly increasing column ends, group_end[T-1] == M;  1 <= T <= QLESS_MAX_GROUPS
 * ------------------------------------------------------------------------------------------- */
#define QLESS_MAX_GROUPS 64
typedef enum { QLESS_AGG_MAX = 0, QLESS_AGG_MEAN = 1 } qless_agg;
qless_status qless_aggregate(const float *full, int64_t N, int32_t M, const int32_t *group_end, int T,
                             qless_agg mode, float *out, void *stream);

/* ---------------------------------------------------------------------------------------------
 * qless_score and qless_aggregate in one call: out[z][t] = maximum or mean, as defined for
 * qless_aggregate, of acc(z, z') of qless_score over the validation columns of group t -- the same bits
 * as the two calls, without the N x M matrix in memory (with more than 64 validation vectors the
 * aggregation is the epilogue of the scoring kernel; below that the matrix is small and passes through
 * the workspace).  Arguments as for qless_score and qless_aggregate;
 *   out   device, N x T fp32 row-major
 *   ws    device workspace, 16-byte aligned, of at least qless_score_groups_workspace(N, M, k, bits, C) bytes
 * ------------------------------------------------------------------------------------------- */
size_t qless_score_groups_workspace(int64_t N, int32_t M, int32_t k, int bits, int C);
qless_status qless_score_groups(const void *const *train_codes, const float *const *train_rnorm,
                                const void *const *val_codes, const float *const *val_rnorm,
                                const float *eta, int C, int64_t N, int32_t M, int32_t k, int bits,
                                const int32_t *group_end, int T, qless_agg mode, float *out,
                                void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QLESS_H */
