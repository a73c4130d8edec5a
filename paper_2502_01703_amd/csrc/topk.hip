// qless_topk: indices of the k_sel largest scores, ordered by (score descending, index ascending)
// (paper Sec. 4.1: the top 5 % of the training examples by influence score).
//
// Every example gets a 64-bit key  (order-preserving image of the fp32 score) << 32 | (2^32-1 - index);
// keys are distinct and "larger key" is exactly "selected earlier".  Steps:
//   1. radix-select the k_sel-th largest key in passes of 8 bits (keys are formed on the fly from
//   the scores); the passes stop as soon as the bucket that holds the k_sel-th key is selected as a
//   whole.  Up to 32768 scores one workgroup does all (up to 8) passes in a single launch (a launch
//   costs more than such a pass; beyond that size the ~50 instructions per key and pass are too
//   many for one compute unit).  Above that, one histogram launch for each of the four digits of
//   the score, whose workgroups each first pick the digit of the pass before from its finished
//   histogram (a 256-bin scan, cheaper than a launch of its own); if the threshold score T is then
//   shared by more examples than are still to be taken, the r with the smallest indices are the
//   first r in array order: a count of the examples with score T per 1024 examples and an exclusive
//   scan of these counts give every such example its position among them;
//   2. compact all selected keys (exactly k_sel of them; one atomic per workgroup and 1024 examples);
//   3. order them, descending: up to 16384 selected keys by rank (every key counts the larger ones
//   among all of them, k_sel^2 comparisons spread over the whole chip, and is written to the slot of
//   its rank: two short launches); above that, a bitonic network (LDS spans of 4096 keys with global
//   steps in between), then  4. decode indices and gather the scores.
#include "common.h"
#include <atomic>
#include <mutex>

namespace qless {

constexpr int kSortBlock = 4096;   // keys sorted per workgroup in LDS (32 KB)
constexpr int kSortOne = 16384;    // most (padded) selected keys that are ordered by rank instead of sorted
constexpr int kPasses = 4;         // 8-bit digits of the score half of the keys (histogram launches)
constexpr int64_t kSelectSmallMax = 32768;   // scores one workgroup selects from in a single launch

struct TopkPlan {
    int64_t padded;                // power of two >= k_sel (>= kSortBlock)
    size_t off_sel, off_hist, off_state, off_rank, off_ties, total;
    int64_t chunks;                // groups of 1024 examples
};

static TopkPlan topk_plan(int64_t N, int64_t k_sel) {
    TopkPlan p{};
    int64_t pad = kSortBlock;
    while (pad < k_sel) pad <<= 1;
    p.padded = pad;
    size_t o = 0;
    p.off_sel = o;   o += (size_t)pad * 8;
    p.off_hist = o;  o += kPasses * 256 * 4;        // one histogram per pass
    p.off_state = o; o += (kPasses + 1) * 32 + 32;  // state before each pass and after the last; compaction cursor
    p.off_rank = o;  o += (size_t)pad * 4;          // ranks of the selected keys
    p.chunks = (N + 1023) / 1024;
    p.off_ties = o;  o += (size_t)(p.chunks + 1) * 4;   // examples at the threshold score per 1024 examples
    p.total = o;
    return p;
}

struct SelectState {
    unsigned long long prefix;     // high digits of the threshold found so far
    unsigned long long remaining;  // rank still to locate inside the current prefix bucket
    unsigned int count;            // compaction cursor (of the last state only)
    unsigned int done;             // the threshold is final: later passes return at once
    unsigned long long pad_;       // 32 bytes per state
};

__device__ inline uint32_t order_key(float f) {
    if (f == 0.0f) f = 0.0f;                       // -0 and +0 compare equal
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ inline unsigned long long make_key(float sc, int64_t i) {
    return ((unsigned long long)order_key(sc) << 32) | (0xFFFFFFFFull - (unsigned long long)i);
}

// state[0] = nothing chosen yet; all histograms and the compaction cursor (state[kPasses].count) cleared
__global__ void __launch_bounds__(256) topk_init_kernel(unsigned int *hist, SelectState *state, unsigned long long k_sel) {
    if (threadIdx.x == 0) {
        state[0].prefix = 0; state[0].remaining = k_sel; state[0].count = 0; state[0].done = 0;
        state[kPasses].count = 0;
    }
    for (int p = 0; p < kPasses; ++p) hist[p * 256 + threadIdx.x] = 0;
}

// Suffix sums over 256 bins and the digit that holds the remaining rank `rem` (walking from the top):
// thread d < 256 passes its bin count; the thread of the chosen digit returns true, with the rank
// left inside that bin in `left`.  `above` is LDS scratch of 257 entries.  All threads of the
// workgroup call it (barriers inside).
__device__ inline bool pick_digit(unsigned long long *above, unsigned int mine, unsigned long long rem,
                                  unsigned long long &left) {
    const int d = (int)threadIdx.x;
    if (d < 256) above[d] = mine;
    if (d == 0) above[256] = 0;
    __syncthreads();
    for (int step = 1; step < 256; step <<= 1) {    // Hillis-Steele
        const unsigned long long add = (d < 256 && d + step < 256) ? above[d + step] : 0ull;
        __syncthreads();
        if (d < 256) above[d] += add;
        __syncthreads();
    }
    // the digit is the largest d with above[d] >= rem; if no bin reaches the rank it is 0
    bool here = false;
    if (d < 256) {
        here = (above[d] >= rem && above[d + 1] < rem) || (d == 0 && above[0] < rem);
        if (here) left = rem - above[d + 1];
    }
    return here;
}

// All passes of the selection in one workgroup (small N).  A wavefront adds the digit of its first
// matching lane once for all lanes that share it (the leading digits of scores are few), the other
// lanes add their own.
__global__ void __launch_bounds__(1024)
topk_select_small_kernel(const float *score, int64_t N, unsigned long long k_sel, SelectState *state) {
    __shared__ unsigned int h[256];
    __shared__ unsigned long long above[257];
    __shared__ unsigned long long sh_prefix, sh_rem;
    __shared__ int sh_done;
    const int lane = threadIdx.x & 63;
    unsigned long long prefix = 0, rem = k_sel;
    constexpr int kU = 8;
    const int64_t n_up = (N + 1024 * kU - 1) / (1024 * kU) * (1024 * kU);
    for (int pass = 0; pass < 8; ++pass) {              // all eight digits of the 64-bit keys
        if (threadIdx.x < 256) h[threadIdx.x] = 0;
        if (threadIdx.x == 0) sh_done = 0;
        __syncthreads();
        const int shift = 56 - 8 * pass;
        const unsigned long long himask = pass == 0 ? 0ull : (~0ull << (shift + 8));
        for (int64_t base = 0; base < n_up; base += 1024 * kU) {  // same trip count for all lanes
            float v[kU];
#pragma unroll
            for (int u = 0; u < kU; ++u) {                         // kU loads in flight per thread
                const int64_t i = base + u * 1024 + threadIdx.x;
                v[u] = i < N ? score[i] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                const int64_t i = base + u * 1024 + threadIdx.x;
                bool match = false;
                unsigned int d = 0;
                if (i < N) {
                    const unsigned long long key = make_key(v[u], i);
                    match = ((key ^ prefix) & himask) == 0;
                    d = (unsigned int)(key >> shift) & 0xFFu;
                }
                const unsigned long long act = __ballot(match);
                if (act) {
                    const int leader = __ffsll((long long)act) - 1;
                    const unsigned int d0 = (unsigned int)__builtin_amdgcn_readlane((int)d, leader);
                    const unsigned long long same = __ballot(match && d == d0);
                    if (lane == leader) atomicAdd(&h[d0], (unsigned int)__popcll(same));
                    if (match && d != d0) atomicAdd(&h[d], 1u);
                }
            }
        }
        __syncthreads();
        const unsigned int mine = threadIdx.x < 256 ? h[threadIdx.x] : 0u;
        unsigned long long left = 0;
        if (pick_digit(above, mine, rem, left)) {
            sh_prefix = prefix | ((unsigned long long)threadIdx.x << shift);
            sh_rem = left;
            sh_done = left == (unsigned long long)mine;             // the whole bucket is selected
        }
        __syncthreads();
        prefix = sh_prefix; rem = sh_rem;
        const int done = sh_done;
        __syncthreads();
        if (done) break;
    }
    if (threadIdx.x == 0) {
        state[kPasses].prefix = prefix; state[kPasses].remaining = rem; state[kPasses].count = 0; state[kPasses].done = 1;
    }
}

// The state after the digit pick of pass `pass` (from the state before it and the pass's finished
// histogram), computed by every thread of a 256-thread workgroup alike; workgroup 0 also records
// it in state[pass + 1].  `above` and `sh` are LDS scratch.
__device__ inline SelectState next_state(int pass, SelectState *state, const unsigned int *hist,
                                         unsigned long long *above, SelectState *sh) {
    const SelectState before = state[pass];
    if (before.done) {                              // uniform
        if (blockIdx.x == 0 && threadIdx.x == 0) { state[pass + 1].prefix = before.prefix; state[pass + 1].remaining = before.remaining; state[pass + 1].done = 1; }
        return before;
    }
    const unsigned int mine = hist[pass * 256 + threadIdx.x];
    unsigned long long left = 0;
    if (pick_digit(above, mine, before.remaining, left)) {
        sh->prefix = before.prefix | ((unsigned long long)threadIdx.x << (56 - 8 * pass));
        sh->remaining = left;
        sh->done = left == (unsigned long long)mine;    // the whole bucket is selected: the prefix with zeros below is the threshold
    }
    __syncthreads();
    SelectState after = *sh;
    after.count = 0;
    __syncthreads();
    if (blockIdx.x == 0 && threadIdx.x == 0) { state[pass + 1].prefix = after.prefix; state[pass + 1].remaining = after.remaining; state[pass + 1].done = after.done; }
    return after;
}

constexpr int kHistPer = 8;                         // examples per thread and round of the histogram
// histogram of digit `pass` (0 = most significant byte) over keys whose higher digits equal the prefix
// chosen so far; the pick of the pass before is done here first, by every workgroup for itself
__global__ void __launch_bounds__(256)
topk_hist_kernel(const float *score, int64_t N, int pass, SelectState *state, unsigned int *hist) {
    __shared__ unsigned int h[256];
    __shared__ unsigned long long above[257];
    __shared__ SelectState sh;
    const SelectState cur = pass == 0 ? state[0] : next_state(pass - 1, state, hist, above, &sh);
    if (cur.done) return;                           // uniform
    h[threadIdx.x] = 0;
    __syncthreads();
    const unsigned long long prefix = cur.prefix;
    const int shift = 56 - 8 * pass;
    // bits above the current digit: pass 0 has none (mask 0), later passes compare them all
    const unsigned long long himask = pass == 0 ? 0ull : (~0ull << (shift + 8));
    // a workgroup takes kHistPer * 256 consecutive examples at a time (few workgroups: every one of them ends
    // with up to 256 atomics on the same global bins), kHistPer loads in flight per thread
    for (int64_t c0 = (int64_t)blockIdx.x * (256 * kHistPer); c0 < N; c0 += (int64_t)gridDim.x * (256 * kHistPer)) {   // uniform
        float v[kHistPer];
#pragma unroll
        for (int u = 0; u < kHistPer; ++u) {
            const int64_t i = c0 + u * 256 + threadIdx.x;
            v[u] = i < N ? score[i] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < kHistPer; ++u) {
            const int64_t i = c0 + u * 256 + threadIdx.x;
            const unsigned long long key = make_key(v[u], i);
            const bool match = i < N && ((key ^ prefix) & himask) == 0;
            const unsigned int d = (unsigned int)(key >> shift) & 0xFFu;
            // the leading digits of scores are few: the lanes that share the digit of the first matching
            // lane are added at once, the others one by one
            const unsigned long long act = __ballot(match);
            if (act) {
                const int leader = __ffsll((long long)act) - 1;
                const unsigned int d0 = (unsigned int)__builtin_amdgcn_readlane((int)d, leader);
                const unsigned long long same = __ballot(match && d == d0);
                if ((int)(threadIdx.x & 63) == leader) atomicAdd(&h[d0], (unsigned int)__popcll(same));
                if (match && d != d0) atomicAdd(&h[d], 1u);
            }
        }
    }
    __syncthreads();
    if (h[threadIdx.x]) atomicAdd(&hist[pass * 256 + threadIdx.x], h[threadIdx.x]);
}

constexpr int kCompactPer = 4;                      // examples per thread and round
constexpr int kChunk = 256 * kCompactPer;           // examples per round of a workgroup

// After the last histogram: picks its digit; unless the threshold bucket is taken whole, counts the
// examples whose score is the threshold score in every group of kChunk examples.
__global__ void __launch_bounds__(256)
topk_tie_count_kernel(const float *score, int64_t N, SelectState *state, const unsigned int *hist,
                      unsigned int *ties) {
    __shared__ unsigned long long above[257];
    __shared__ SelectState sh;
    __shared__ unsigned int cnt;
    const SelectState fin = next_state(kPasses - 1, state, hist, above, &sh);
    if (fin.done) return;                           // uniform
    const uint32_t T = (uint32_t)(fin.prefix >> 32);
    for (int64_t c0 = (int64_t)blockIdx.x * kChunk; c0 < N; c0 += (int64_t)gridDim.x * kChunk) {
        if (threadIdx.x == 0) cnt = 0;
        __syncthreads();
        unsigned int mine = 0;
#pragma unroll
        for (int u = 0; u < kCompactPer; ++u) {
            const int64_t i = c0 + u * 256 + threadIdx.x;
            const bool tie = i < N && order_key(score[i]) == T;
            mine += (unsigned int)__popcll(__ballot(tie));
        }
        if ((threadIdx.x & 63) == 0 && mine) atomicAdd(&cnt, mine);
        __syncthreads();
        if (threadIdx.x == 0) ties[c0 / kChunk] = cnt;
        __syncthreads();
    }
}

// One workgroup: exclusive scan, in place, of the per-group counts.
__global__ void __launch_bounds__(1024)
topk_tie_scan_kernel(const SelectState *state, unsigned int *ties, int64_t chunks) {
    __shared__ unsigned int part[1024];
    __shared__ unsigned int carry;
    if (state[kPasses].done) return;                // written by the launch before
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int64_t b = 0; b < chunks; b += 1024) {
        const int64_t c = b + threadIdx.x;
        const unsigned int v = c < chunks ? ties[c] : 0u;
        part[threadIdx.x] = v;
        __syncthreads();
        for (int step = 1; step < 1024; step <<= 1) {   // Hillis-Steele, inclusive
            const unsigned int add = (int)threadIdx.x >= step ? part[threadIdx.x - step] : 0u;
            __syncthreads();
            part[threadIdx.x] += add;
            __syncthreads();
        }
        const unsigned int base = carry;
        if (c < chunks) ties[c] = base + part[threadIdx.x] - v;
        __syncthreads();
        if (threadIdx.x == 1023) carry = base + part[1023];
        __syncthreads();
    }
}

// The selected keys (exactly k_sel of them) are gathered in any order; the slots from k_sel to
// padded and the ranks are cleared.  A workgroup takes kChunk consecutive examples at a time and one
// atomic for all it selects among them.  Selected: key >= threshold key when the selection ended
// with a whole bucket; otherwise score above the threshold score T, or equal to it and among the
// first `remaining` such examples in array order (`ties` holds how many precede each group).
__global__ void __launch_bounds__(256)
topk_compact_kernel(const float *score, int64_t N, SelectState *state, const unsigned int *ties,
                    unsigned long long *sel, unsigned int *rank, int64_t k_sel, int64_t padded) {
    __shared__ unsigned int offs[4 * kCompactPer + 1];
    __shared__ unsigned int toffs[4 * kCompactPer];
    const SelectState fin = state[kPasses];
    const bool by_position = !fin.done;             // uniform
    const unsigned long long thr = by_position ? (fin.prefix | 0xFFFFFFFFull) + 1ull : fin.prefix;   // T + 1 in the score half
    const bool none_above = by_position && thr == 0ull;     // T is the largest score key: nothing lies above it
    const uint32_t T = (uint32_t)(fin.prefix >> 32);
    unsigned int *cursor = &state[kPasses].count;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t span = N > padded ? N : padded;
    for (int64_t c0 = (int64_t)blockIdx.x * kChunk; c0 < span; c0 += (int64_t)gridDim.x * kChunk) {   // uniform per workgroup
        unsigned long long key[kCompactPer], mask[kCompactPer], tmask[kCompactPer];
        bool take[kCompactPer], tie[kCompactPer];
#pragma unroll
        for (int u = 0; u < kCompactPer; ++u) {
            const int64_t i = c0 + u * 256 + threadIdx.x;
            if (i >= k_sel && i < padded) sel[i] = 0;   // padding sorts last (real keys are > 0)
            if (i < padded) rank[i] = 0;
            key[u] = 0; take[u] = false; tie[u] = false;
            if (i < N) {
                key[u] = make_key(score[i], i);
                take[u] = !none_above && key[u] >= thr;
                tie[u] = by_position && (uint32_t)(key[u] >> 32) == T;
            }
        }
        if (by_position) {
            // position of every example with the threshold score among all of them, in array order
            // (element u * 256 + 64 * wave + lane of the group: order by u, then wave, then lane)
#pragma unroll
            for (int u = 0; u < kCompactPer; ++u) {
                tmask[u] = __ballot(tie[u]);
                if (lane == 0) toffs[u * 4 + wave] = (unsigned int)__popcll(tmask[u]);
            }
            __syncthreads();
            if (threadIdx.x == 0) {
                unsigned int run = c0 < N ? ties[c0 / kChunk] : 0u;
                for (int q = 0; q < 4 * kCompactPer; ++q) { const unsigned int v = toffs[q]; toffs[q] = run; run += v; }
            }
            __syncthreads();
#pragma unroll
            for (int u = 0; u < kCompactPer; ++u) {
                const unsigned long long pos = (unsigned long long)toffs[u * 4 + wave] +
                                               (unsigned long long)__popcll(tmask[u] & ((1ull << lane) - 1ull));
                if (tie[u] && pos < fin.remaining) take[u] = true;
            }
        }
#pragma unroll
        for (int u = 0; u < kCompactPer; ++u) {
            mask[u] = __ballot(take[u]);
            if (lane == 0) offs[wave * kCompactPer + u] = (unsigned int)__popcll(mask[u]);
        }
        __syncthreads();
        if (threadIdx.x == 0) {                      // exclusive prefix over the 16 counts, then one atomic
            unsigned int run = 0;
            for (int q = 0; q < 4 * kCompactPer; ++q) { const unsigned int v = offs[q]; offs[q] = run; run += v; }
            offs[4 * kCompactPer] = run ? atomicAdd(cursor, run) : 0u;
        }
        __syncthreads();
        const unsigned int wgbase = offs[4 * kCompactPer];
#pragma unroll
        for (int u = 0; u < kCompactPer; ++u) {
            const unsigned int pos = wgbase + offs[wave * kCompactPer + u] +
                                     (unsigned int)__popcll(mask[u] & ((1ull << lane) - 1ull));
            if (take[u] && (int64_t)pos < k_sel) sel[pos] = key[u];
        }
        __syncthreads();                             // offs and toffs are reused by the next round
    }
}

// Rank of every selected key = how many selected keys are larger (keys are distinct): workgroup
// (x, y) counts, for its 256 * kRankPer keys, the larger ones among keys [y * seg, (y + 1) * seg),
// staged in LDS 1024 at a time and read by all lanes at once (a broadcast).  k_sel^2 comparisons: for
// k_sel <= kSortOne only.
constexpr int kRankPer = 1;                         // keys per thread (two measured no faster)
__global__ void __launch_bounds__(256)
topk_rank_kernel(const unsigned long long *sel, int64_t k_sel, int64_t seg, unsigned int *rank) {
    __shared__ __attribute__((aligned(16))) unsigned long long tile[1024];
    unsigned long long mine[kRankPer];
    unsigned int cnt[kRankPer];
#pragma unroll
    for (int e = 0; e < kRankPer; ++e) {
        const int64_t i = ((int64_t)blockIdx.x * kRankPer + e) * 256 + threadIdx.x;
        mine[e] = i < k_sel ? sel[i] : ~0ull;
        cnt[e] = 0;
    }
    const int64_t j0 = (int64_t)blockIdx.y * seg;
    const int64_t j1 = j0 + seg < k_sel ? j0 + seg : k_sel;
    for (int64_t jb = j0; jb < j1; jb += 1024) {
        __syncthreads();
        for (int t = threadIdx.x; t < 1024; t += 256) tile[t] = jb + t < j1 ? sel[jb + t] : 0ull;   // 0 is below every key
        __syncthreads();
#pragma unroll 8
        for (int t = 0; t < 1024; t += 2) {
            const ulonglong2 pr = *(const ulonglong2 *)&tile[t];
#pragma unroll
            for (int e = 0; e < kRankPer; ++e) cnt[e] += (pr.x > mine[e]) + (pr.y > mine[e]);
        }
    }
#pragma unroll
    for (int e = 0; e < kRankPer; ++e) {
        const int64_t i = ((int64_t)blockIdx.x * kRankPer + e) * 256 + threadIdx.x;
        if (i < k_sel && cnt[e]) atomicAdd(&rank[i], cnt[e]);
    }
}

// idx / val in rank order
__global__ void __launch_bounds__(256)
topk_scatter_kernel(const unsigned long long *sel, const unsigned int *rank, int64_t k_sel, const float *score,
                    int64_t N, int64_t *idx, float *val) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= k_sel) return;
    const int64_t i = (int64_t)(0xFFFFFFFFull - (sel[t] & 0xFFFFFFFFull));
    const unsigned int r = rank[t];
    if ((int64_t)r >= k_sel) return;                 // cannot happen with distinct keys
    idx[r] = i;
    if (val) val[r] = score[i < N ? i : N - 1];
}

// Bitonic network, descending.  Stage size kk (sub-sequence length), step jj (partner distance).
__device__ inline void cmpswap_desc(unsigned long long &x, unsigned long long &y, bool desc) {
    if ((x < y) == desc) { const unsigned long long t = x; x = y; y = t; }
}

// all steps with jj < kSortBlock for stages kk_from..kk_to inside LDS.  Thread t handles the pairs t
// and t + 1024 of a step; for a partner distance jj <= 64 both pairs of every thread of a wavefront lie
// inside two 128-element segments that only this wavefront touches, so consecutive steps with
// jj <= 64 need no workgroup barrier (LDS operations of a wavefront complete in order).
__global__ void __launch_bounds__(1024)
topk_bitonic_local_kernel(unsigned long long *data, int64_t kk_from, int64_t kk_to) {
    __shared__ unsigned long long s[kSortBlock];
    const int64_t base = (int64_t)blockIdx.x * kSortBlock;
    for (int t = threadIdx.x; t < kSortBlock; t += 1024) s[t] = data[base + t];
    __syncthreads();
    bool wide_before = true;                           // the previous step crossed wavefront segments
    for (int64_t kk = kk_from; kk <= kk_to; kk <<= 1) {
        int64_t j0 = kk >> 1;
        if (j0 >= kSortBlock) j0 = kSortBlock >> 1;
        for (int lj = 63 - __builtin_clzll((unsigned long long)j0); lj >= 0; --lj) {   // partner distance 2^lj
            const int jj = 1 << lj;
            const bool wide = jj > 64;
            if (wide || wide_before) __syncthreads();
            else { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); __builtin_amdgcn_wave_barrier(); }
            wide_before = wide;
            for (int t = threadIdx.x; t < kSortBlock / 2; t += 1024) {
                const int lo = ((t >> lj) << (lj + 1)) | (t & (jj - 1));
                const int hi = lo + jj;
                const bool desc = (((base + lo) & kk) == 0);
                unsigned long long x = s[lo], y = s[hi];
                cmpswap_desc(x, y, desc);
                s[lo] = x; s[hi] = y;
            }
        }
    }
    __syncthreads();
    for (int t = threadIdx.x; t < kSortBlock; t += 1024) data[base + t] = s[t];
}

__global__ void topk_bitonic_global_kernel(unsigned long long *data, int64_t n, int64_t kk, int64_t jj) {
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < n / 2;
         t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t lo = (t / jj) * 2 * jj + (t % jj), hi = lo + jj;
        const bool desc = ((lo & kk) == 0);
        unsigned long long x = data[lo], y = data[hi];
        if ((x < y) == desc) { data[lo] = y; data[hi] = x; }
    }
}

__global__ void topk_emit_kernel(const unsigned long long *sel, int64_t k_sel, const float *score,
                                 int64_t N, int64_t *idx, float *val) {
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < k_sel;
         t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t i = (int64_t)(0xFFFFFFFFull - (sel[t] & 0xFFFFFFFFull));
        idx[t] = i;
        if (val) val[t] = score[i < N ? i : N - 1];
    }
}

}  // namespace qless

using namespace qless;

extern "C" size_t qless_topk_workspace(int64_t N, int64_t k_sel) {
    if (N < 0 || k_sel < 0) return 0;
    return topk_plan(N, k_sel).total;
}

// Enqueues the whole selection on `st`; `ws` holds at least topk_plan(N, k_sel).total bytes, 8-byte
// aligned; 1 <= k_sel <= N < 2^32, all pointers checked by the caller.
static qless_status topk_run(const float *score, int64_t N, int64_t k_sel, int64_t *idx, float *val,
                             void *ws, hipStream_t st) {
    const TopkPlan p = topk_plan(N, k_sel);
    unsigned char *w = (unsigned char *)ws;
    unsigned long long *sel = (unsigned long long *)(w + p.off_sel);
    unsigned int *hist = (unsigned int *)(w + p.off_hist);
    SelectState *state = (SelectState *)(w + p.off_state);
    unsigned int *rank = (unsigned int *)(w + p.off_rank);
    unsigned int *ties = (unsigned int *)(w + p.off_ties);

    auto blocks_for = [](int64_t n) { int64_t b = (n + 255) / 256; if (b < 1) b = 1; if (b > 2048) b = 2048; return (unsigned)b; };
    const bool small = N <= kSelectSmallMax;
    if (small) {
        hipLaunchKernelGGL(topk_select_small_kernel, dim3(1), dim3(1024), 0, st, score, N, (unsigned long long)k_sel, state);
    } else {
        hipLaunchKernelGGL(topk_init_kernel, dim3(1), dim3(256), 0, st, hist, state, (unsigned long long)k_sel);
        int64_t hblocks = (N + 256 * kHistPer - 1) / (256 * kHistPer);
        if (hblocks > 2048) hblocks = 2048;
        for (int pass = 0; pass < kPasses; ++pass)
            hipLaunchKernelGGL(topk_hist_kernel, dim3((unsigned)hblocks), dim3(256), 0, st, score, N, pass, state, hist);
    }
    const int64_t span = N > p.padded ? N : p.padded;
    int64_t cblocks = (span + kChunk - 1) / kChunk;
    if (cblocks > 2048) cblocks = 2048;
    if (!small) {
        int64_t tblocks = (N + kChunk - 1) / kChunk;
        if (tblocks > 2048) tblocks = 2048;
        hipLaunchKernelGGL(topk_tie_count_kernel, dim3((unsigned)tblocks), dim3(256), 0, st, score, N, state,
                           (const unsigned int *)hist, ties);
        hipLaunchKernelGGL(topk_tie_scan_kernel, dim3(1), dim3(1024), 0, st, (const SelectState *)state, ties, p.chunks);
    }
    hipLaunchKernelGGL(topk_compact_kernel, dim3((unsigned)cblocks), dim3(256), 0, st, score, N, state,
                       (const unsigned int *)ties, sel, rank, k_sel, p.padded);
    if (p.padded <= kSortOne) {
        // few selected keys: rank every key among all of them, then write in rank order
        const unsigned kb = (unsigned)((k_sel + 255) / 256);
        const int64_t seg = 1024;
        const unsigned rb = (unsigned)((k_sel + 256 * kRankPer - 1) / (256 * kRankPer));
        hipLaunchKernelGGL(topk_rank_kernel, dim3(rb, (unsigned)((k_sel + seg - 1) / seg)), dim3(256), 0, st,
                           (const unsigned long long *)sel, k_sel, seg, rank);
        hipLaunchKernelGGL(topk_scatter_kernel, dim3(kb), dim3(256), 0, st, (const unsigned long long *)sel,
                           (const unsigned int *)rank, k_sel, score, N, idx, val);
        return launch_status();
    }
    // many selected keys: sort them, descending, with a bitonic network
    const unsigned nblk = (unsigned)(p.padded / kSortBlock);
    hipLaunchKernelGGL(topk_bitonic_local_kernel, dim3(nblk), dim3(1024), 0, st, sel, (int64_t)2, (int64_t)kSortBlock);
    for (int64_t kk = 2 * kSortBlock; kk <= p.padded; kk <<= 1) {
        for (int64_t jj = kk >> 1; jj >= kSortBlock; jj >>= 1)
            hipLaunchKernelGGL(topk_bitonic_global_kernel, dim3(blocks_for(p.padded / 2)), dim3(256), 0, st, sel, p.padded, kk, jj);
        hipLaunchKernelGGL(topk_bitonic_local_kernel, dim3(nblk), dim3(1024), 0, st, sel, kk, kk);
    }
    hipLaunchKernelGGL(topk_emit_kernel, dim3(blocks_for(k_sel)), dim3(256), 0, st, sel, k_sel, score, N, idx, val);
    return launch_status();
}

static qless_status topk_check(const float *score, int64_t N, int64_t k_sel, const int64_t *idx) {
    if (N < 0 || k_sel < 0 || k_sel > N) return QLESS_ERR_INVALID_ARG;
    if (N > 0 && !score) return QLESS_ERR_INVALID_ARG;
    if (k_sel > 0 && !idx) return QLESS_ERR_INVALID_ARG;
    if (N >= ((int64_t)1 << 32)) return QLESS_ERR_UNSUPPORTED;
    return QLESS_OK;
}

extern "C" qless_status qless_topk(const float *score, int64_t N, int64_t k_sel, int64_t *idx,
                                   float *val, void *ws, size_t ws_bytes, void *stream) {
    const qless_status rc = topk_check(score, N, k_sel, idx);
    if (rc != QLESS_OK || k_sel == 0) return rc;
    if (!ws || ws_bytes < topk_plan(N, k_sel).total) return QLESS_ERR_WORKSPACE;
    if ((uintptr_t)ws % 8) return QLESS_ERR_WORKSPACE;
    return topk_run(score, N, k_sel, idx, val, ws, (hipStream_t)stream);
}

// ------------------------------------------------------------------------------------------
// The same selection for callers that cannot allocate: its workspace is a file-scope device
// array, one copy per GPU.  On the host the array's name only stands for the symbol; the
// address the kernels receive is the one hipGetSymbolAddress returns on each device.
// ------------------------------------------------------------------------------------------
constexpr int64_t kNoAllocMaxN = QLESS_TOPK_NOALLOC_MAX_N;
constexpr int64_t kNoAllocMaxSel = QLESS_TOPK_NOALLOC_MAX_SEL;
// topk_plan(kNoAllocMaxN, kNoAllocMaxSel).total, rounded up (checked at set-up)
constexpr size_t kScratchBytes = (size_t)kNoAllocMaxSel * 12 + 4096 + 256 + (size_t)(kNoAllocMaxN / 1024 + 2) * 4 + 256;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex scratch_mutex;
static std::atomic<void *> scratch_ptr[kMaxDevices];

// device address of this GPU's copy of `scratch` (resolved once per device, with that device current)
qless_status qless::topk_scratch_address(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return QLESS_ERR_DEVICE;
    void *p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lock(scratch_mutex);
        p = scratch_ptr[dev].load(std::memory_order_relaxed);
        if (!p) {
            if (topk_plan(kNoAllocMaxN, kNoAllocMaxSel).total > kScratchBytes) return QLESS_ERR_WORKSPACE;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return QLESS_ERR_DEVICE;
            scratch_ptr[dev].store(p, std::memory_order_release);
        }
    }
    *out = p;
    return QLESS_OK;
}

extern "C" qless_status qless_topk_noalloc(const float *score, int64_t N, int64_t k_sel, int64_t *idx,
                                           float *val, void *stream) {
    const qless_status rc = topk_check(score, N, k_sel, idx);
    if (rc != QLESS_OK) return rc;
    if (N > kNoAllocMaxN || k_sel > kNoAllocMaxSel) return QLESS_ERR_UNSUPPORTED;
    if (k_sel == 0) return QLESS_OK;
    void *ws = nullptr;
    const qless_status rs = topk_scratch_address(&ws);
    if (rs != QLESS_OK) return rs;
    // every word of the workspace that a launch reads is written earlier in the same call (init /
    // select kernels clear histograms, states and the cursor; the compaction clears padding and ranks;
    // the tie counts are written before they are scanned), so nothing of the call before survives
    return topk_run(score, N, k_sel, idx, val, ws, (hipStream_t)stream);
}
