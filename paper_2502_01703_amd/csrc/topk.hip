// qless_topk: indices of the k_sel largest scores, ordered by (score descending, index ascending)
// (paper Sec. 4.1: the top 5 % of the training examples by influence score).
//
// Every example gets a 64-bit key  (order-preserving image of the fp32 score) << 32 | (2^32-1 - index);
// keys are distinct and "larger key" is exactly "selected earlier".  Steps:
//   1. radix-select the k_sel-th largest key, up to 8 passes of 8 bits (keys are formed on the fly
//   from the scores); the passes stop as soon as the bucket that holds the k_sel-th key is selected
//   as a whole (without ties at the threshold that is after the four digits of the score).  Up to
//   32768 scores one workgroup does all passes in a single launch (a launch costs more than such a
//   pass; beyond that size the ~50 instructions per key and pass are too many for one compute
//   unit); above that, a histogram launch and a one-workgroup digit pick per pass;  2. compact all keys >= threshold (exactly k_sel of them; one atomic per
//   wavefront);
//   3. sort them descending with a bitonic network (LDS for spans up to 4096, global steps
//   above);  4. decode indices and gather the scores.
#include "common.h"

namespace qless {

constexpr int kSortBlock = 4096;   // keys sorted per workgroup in LDS (32 KB)
constexpr int64_t kSelectSmallMax = 32768;   // scores one workgroup selects from in a single launch

struct TopkPlan {
    int64_t padded;                // power of two >= k_sel (>= kSortBlock)
    size_t off_sel, off_hist, off_state, total;
};

static TopkPlan topk_plan(int64_t N, int64_t k_sel) {
    TopkPlan p{};
    int64_t pad = kSortBlock;
    while (pad < k_sel) pad <<= 1;
    p.padded = pad;
    size_t o = 0;
    p.off_sel = o;   o += (size_t)pad * 8;
    p.off_hist = o;  o += 256 * 4;
    p.off_state = o; o += 64;
    p.total = o;
    return p;
}

struct SelectState {
    unsigned long long prefix;     // high digits of the threshold found so far
    unsigned long long remaining;  // rank still to locate inside the current prefix bucket
    unsigned int count;            // compaction cursor
    unsigned int done;             // the threshold is final: later passes return at once
};

__device__ inline uint32_t order_key(float f) {
    if (f == 0.0f) f = 0.0f;                       // -0 and +0 compare equal
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ inline unsigned long long make_key(float sc, int64_t i) {
    return ((unsigned long long)order_key(sc) << 32) | (0xFFFFFFFFull - (unsigned long long)i);
}

__global__ void __launch_bounds__(256) topk_init_kernel(unsigned int *hist, SelectState *state, unsigned long long k_sel) {
    if (threadIdx.x == 0) { state->prefix = 0; state->remaining = k_sel; state->count = 0; state->done = 0; }
    hist[threadIdx.x] = 0;
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
    for (int pass = 0; pass < 8; ++pass) {
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
    if (threadIdx.x == 0) { state->prefix = prefix; state->remaining = rem; state->count = 0; state->done = 1; }
}

// histogram of digit `pass` (0 = most significant byte) over keys whose higher digits equal prefix
__global__ void __launch_bounds__(256)
topk_hist_kernel(const float *score, int64_t N, int pass, const SelectState *state,
                 unsigned int *hist) {
    __shared__ unsigned int h[256];
    if (state->done) return;                        // uniform: written by an earlier launch
    h[threadIdx.x] = 0;
    __syncthreads();
    const unsigned long long prefix = state->prefix;
    const int shift = 56 - 8 * pass;
    // bits above the current digit: pass 0 has none (mask 0), later passes compare them all
    const unsigned long long himask = pass == 0 ? 0ull : (~0ull << (shift + 8));
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N;
         i += (int64_t)gridDim.x * blockDim.x) {
        const unsigned long long key = make_key(score[i], i);
        const bool match = ((key ^ prefix) & himask) == 0;
        if (match) atomicAdd(&h[(key >> shift) & 0xFF], 1u);
    }
    __syncthreads();
    if (h[threadIdx.x]) atomicAdd(&hist[threadIdx.x], h[threadIdx.x]);
}

// one workgroup: the digit that holds the remaining rank, walking the 256 bins from the top
__global__ void __launch_bounds__(256)
topk_pick_kernel(int pass, SelectState *state, unsigned int *hist) {
    __shared__ unsigned long long above[257];      // above[d] = counted keys with digit >= d
    if (state->done) return;
    const unsigned int mine = hist[threadIdx.x];
    hist[threadIdx.x] = 0;                          // ready for the next pass
    unsigned long long left = 0;
    if (pick_digit(above, mine, state->remaining, left)) {
        state->prefix |= (unsigned long long)threadIdx.x << (56 - 8 * pass);
        state->remaining = left;
        // the whole bucket is selected: the prefix with zeros below is the threshold
        if (left == (unsigned long long)mine) state->done = 1;
    }
}

// Keys >= threshold (exactly k_sel of them) are gathered in any order; the slots from k_sel to
// padded are cleared.  One atomic per wavefront: its selected lanes take consecutive positions.
__global__ void topk_compact_kernel(const float *score, int64_t N, SelectState *state,
                                    unsigned long long *sel, int64_t k_sel, int64_t padded) {
    const unsigned long long thr = state->prefix;
    const int lane = threadIdx.x & 63;
    const int64_t span = N > padded ? N : padded;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < span;
         i += (int64_t)gridDim.x * blockDim.x) {
        if (i >= k_sel && i < padded) sel[i] = 0;   // padding sorts last (real keys are > 0)
        unsigned long long key = 0;
        bool take = false;
        if (i < N) { key = make_key(score[i], i); take = key >= thr; }
        const unsigned long long mask = __ballot(take);
        if (mask) {
            const int leader = __ffsll((long long)mask) - 1;
            unsigned int base = 0;
            if (lane == leader) base = atomicAdd(&state->count, (unsigned int)__popcll(mask));
            base = __shfl(base, leader);
            const unsigned int pos = base + (unsigned int)__popcll(mask & ((1ull << lane) - 1ull));
            if (take && (int64_t)pos < k_sel) sel[pos] = key;
        }
    }
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
        int64_t jj = kk >> 1;
        if (jj >= kSortBlock) jj = kSortBlock >> 1;
        for (; jj > 0; jj >>= 1) {
            const bool wide = jj > 64;
            if (wide || wide_before) __syncthreads();
            else { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); __builtin_amdgcn_wave_barrier(); }
            wide_before = wide;
            for (int t = threadIdx.x; t < kSortBlock / 2; t += 1024) {
                const int lo = (int)(((int64_t)t / jj) * 2 * jj + ((int64_t)t % jj));
                const int hi = lo + (int)jj;
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

extern "C" qless_status qless_topk(const float *score, int64_t N, int64_t k_sel, int64_t *idx,
                                   float *val, void *ws, size_t ws_bytes, void *stream) {
    if (N < 0 || k_sel < 0 || k_sel > N) return QLESS_ERR_INVALID_ARG;
    if (N > 0 && !score) return QLESS_ERR_INVALID_ARG;
    if (k_sel > 0 && !idx) return QLESS_ERR_INVALID_ARG;
    if (N >= ((int64_t)1 << 32)) return QLESS_ERR_UNSUPPORTED;
    if (k_sel == 0) return QLESS_OK;
    const TopkPlan p = topk_plan(N, k_sel);
    if (!ws || ws_bytes < p.total) return QLESS_ERR_WORKSPACE;
    if ((uintptr_t)ws % 8) return QLESS_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    unsigned char *w = (unsigned char *)ws;
    unsigned long long *sel = (unsigned long long *)(w + p.off_sel);
    unsigned int *hist = (unsigned int *)(w + p.off_hist);
    SelectState *state = (SelectState *)(w + p.off_state);

    auto blocks_for = [](int64_t n) { int64_t b = (n + 255) / 256; if (b < 1) b = 1; if (b > 2048) b = 2048; return (unsigned)b; };
    if (N <= kSelectSmallMax) {
        hipLaunchKernelGGL(topk_select_small_kernel, dim3(1), dim3(1024), 0, st, score, N, (unsigned long long)k_sel, state);
    } else {
        hipLaunchKernelGGL(topk_init_kernel, dim3(1), dim3(256), 0, st, hist, state, (unsigned long long)k_sel);
        for (int pass = 0; pass < 8; ++pass) {
            hipLaunchKernelGGL(topk_hist_kernel, dim3(blocks_for(N)), dim3(256), 0, st, score, N, pass, state, hist);
            hipLaunchKernelGGL(topk_pick_kernel, dim3(1), dim3(256), 0, st, pass, state, hist);
        }
    }
    const int64_t span = N > p.padded ? N : p.padded;
    hipLaunchKernelGGL(topk_compact_kernel, dim3(blocks_for(span)), dim3(256), 0, st, score, N, state, sel, k_sel, p.padded);
    // sort the selected keys, descending
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
