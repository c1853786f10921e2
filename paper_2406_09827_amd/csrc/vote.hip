// Vote over the index sets of an ensemble of masks (paper appendix "Ensemble Hierarchical Top-k
// Approximation"): per query block, a key block's votes are the number of the n_e sets that hold it; blocks
// with at least theta_vote votes are kept (1 = union, n_e = intersection); with tau = 1 at most kb of them,
// more votes first, the lower position among equal votes.
//
// One wave per (sequence, head, query block); four per workgroup, no workgroup barrier.  Every set arrives
// sorted (ascending positions, then padding), so nothing is sorted here either: an entry finds its votes by
// a binary search in each of the other sets, the first set that holds a position owns it, and the place of a
// kept position in the output is the number of kept positions below it, summed over the sets from prefix
// counts of a bit array (one bit per entry, one 64-bit word per wave-wide ballot).
#include "common.h"
#include "launch.h"

namespace hipattn {

constexpr int kVoteMaxEntries = 4096;  // n_e * kb
constexpr int kVoteMaxSets = 16;

// first index in the ascending run a[0 .. n) whose value is >= v
__device__ __forceinline__ int lower_bound(const int *a, int n, int v)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid] < v) lo = mid + 1; else hi = mid;
    }
    return lo;
}

template <int MAXE>
__global__ __launch_bounds__(kThreads) void vote_kernel(const int32_t *__restrict__ samples, int32_t *__restrict__ out,
                                                        int64_t n_units, int n_e, int kb, int theta, int tau)
{
    constexpr int W = MAXE / 64;  // bit-array words
    __shared__ int vals_s[4][MAXE];
    __shared__ uint64_t bits_s[4][W];
    __shared__ int wpre_s[4][W + 1];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t u = (int64_t)blockIdx.x * 4 + wave;
    if (u >= n_units) return;
    int *vals = vals_s[wave];
    uint64_t *bits = bits_s[wave];
    int *wpre = wpre_s[wave];
    const int M = n_e * kb, iters = (M + 63) >> 6;
    const int width = tau ? kb : M;
    int32_t *row = out + u * width;

    for (int i = lane; i < M; i += 64) {
        const int e = i / kb, j = i - e * kb;
        const int v = samples[((int64_t)e * n_units + u) * kb + j];
        vals[i] = v < 0 ? kSentinel : v;   // "no block" entries sort last
    }
    wave_lds_sync();

    // prefix counts of the bit array: wpre[w] = bits set in words 0 .. w-1
    auto publish = [&](int it, bool flag) __attribute__((always_inline)) {
        const uint64_t m = __ballot(flag);
        if (lane == 0) bits[it] = m;
    };
    auto scan_words = [&]() __attribute__((always_inline)) {
        wave_lds_sync();
        int c = lane < iters ? __popcll(bits[lane]) : 0;   // iters <= 64
        int incl = c;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int t = __shfl_up(incl, d, 64);
            if (lane >= d) incl += t;
        }
        if (lane < iters) wpre[lane + 1] = incl;
        if (lane == 0) wpre[0] = 0;
        wave_lds_sync();
    };
    auto prefix = [&](int g) __attribute__((always_inline)) {   // bits set among entries 0 .. g-1
        const int w = g >> 6, r = g & 63;
        return wpre[w] + (r ? __popcll(bits[w] & ((1ull << r) - 1)) : 0);
    };
    // flagged entries with a position below v, over all sets
    auto below = [&](int v) __attribute__((always_inline)) {
        int n = 0;
        for (int e = 0; e < n_e; ++e) n += prefix(e * kb + lower_bound(vals + e * kb, kb, v)) - prefix(e * kb);
        return n;
    };

    // pass 1: votes of every entry; an entry stands for its position if no earlier set holds it
    constexpr int IT = MAXE / 64;
    uint8_t votes[IT];   // 0: not a candidate
    int level_cnt[kVoteMaxSets + 1];
#pragma unroll
    for (int c = 0; c <= kVoteMaxSets; ++c) level_cnt[c] = 0;
#pragma unroll
    for (int it = 0; it < IT; ++it) {
        votes[it] = 0;
        if (it < iters) {
            const int i = it * 64 + lane;
            int n = 0;
            bool owner = false;
            if (i < M && vals[i] != kSentinel) {
                const int v = vals[i], e = i / kb;
                owner = true;
                for (int e2 = 0; e2 < n_e; ++e2) {
                    const int pos = lower_bound(vals + e2 * kb, kb, v);
                    const bool hit = pos < kb && vals[e2 * kb + pos] == v;
                    n += hit;
                    if (hit && e2 < e) owner = false;
                }
            }
            if (owner && n >= theta) votes[it] = (uint8_t)n;
            if (tau) {
#pragma unroll
                for (int c = 1; c <= kVoteMaxSets; ++c)
                    if (c <= n_e) level_cnt[c] += __popcll(__ballot(votes[it] == c));
            }
        }
    }
    // truncation to kb: positions with more than `level` votes stay, of those with exactly `level` votes the
    // `need` lowest positions
    int level = 0, need = 0;
    if (tau) {
        int total = 0;
#pragma unroll
        for (int c = 1; c <= kVoteMaxSets; ++c) total += level_cnt[c];   // (levels above n_e stay 0)
        if (total > kb) {
            int acc = 0;
#pragma unroll
            for (int c = kVoteMaxSets; c >= 1; --c) {
                if (level == 0 && acc + level_cnt[c] >= kb) { level = c; need = kb - acc; }
                acc += level_cnt[c];
            }
        }
    }
    if (level > 0) {
#pragma unroll
        for (int it = 0; it < IT; ++it)
            if (it < iters) publish(it, votes[it] == level);
        scan_words();
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            if (it < iters) {
                const int i = it * 64 + lane;
                if (votes[it] != 0 && (votes[it] < level || (votes[it] == level && below(vals[min(i, M - 1)]) >= need))) votes[it] = 0;
            }
        }
        wave_lds_sync();   // every lane is done with the level bits before they are overwritten
    }
    // pass 3: kept positions in ascending order
#pragma unroll
    for (int it = 0; it < IT; ++it)
        if (it < iters) publish(it, votes[it] != 0);
    scan_words();
    const int n_kept = wpre[iters];
#pragma unroll
    for (int it = 0; it < IT; ++it) {
        if (it < iters) {
            const int i = it * 64 + lane;
            if (votes[it] != 0) row[below(vals[i])] = vals[i];
        }
    }
    for (int j = n_kept + lane; j < width; j += 64) row[j] = kSentinel;
}

bool vote_supported(int n_e, int kb) { return n_e >= 1 && n_e <= kVoteMaxSets && kb >= 1 && (int64_t)n_e * kb <= kVoteMaxEntries; }

hipError_t launch_vote(const int32_t *samples, int32_t *out, int64_t n_units, int n_e, int kb, int theta, int tau, hipStream_t st)
{
    if (n_units == 0) return hipSuccess;
    const int64_t blocks = (n_units + 3) / 4;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    dim3 grid((unsigned)blocks), block(kThreads);
    const int M = n_e * kb;
    if (M <= 1024) hipLaunchKernelGGL((vote_kernel<1024>), grid, block, 0, st, samples, out, n_units, n_e, kb, theta, tau);
    else hipLaunchKernelGGL((vote_kernel<4096>), grid, block, 0, st, samples, out, n_units, n_e, kb, theta, tau);
    return hipGetLastError();
}

}  // namespace hipattn
