// Algorithm 2 "Pruned Attention", the line  I = argtop_k(S[j], B / block size),
// plus the local and diagonal blocks that are always kept.
//
// One wavefront per (batch, head, segment) row.  The row lives in registers (lane l owns blocks
// l, l+64, ...).  Scores are mapped to order-preserving unsigned keys; the k-th largest key is found
// by an MSB-first radix search (one wave-wide count per bit: a compare per key, the lane masks counted on the
// scalar unit) that stops at the first bit whose count is exactly k; everything above it is taken, ties at
// the threshold go to the smallest indices, and the result is compacted in index order, so the
// list comes out ascending.  Long rows are first thinned to the few keys that can be among the k largest.
#include "kernels.h"

namespace cp {
namespace {

struct SelectArgs {
    const float* scores; int32_t* idx; int32_t* cnt;
    long long rows;            // B*H*n1 lists (H = query heads, or KV heads when the lists are shared)
    int n1, n2, r, budget, local, list_len;
    int group;                 // shared lists: query heads per KV head, whose scores are merged by max
};


__device__ __forceinline__ uint32_t ordered_key(float x) {
    uint32_t u = __float_as_uint(x);
    if (u == 0x80000000u) u = 0;                       // -0 ranks with +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// key of block i for list row `row`: the row's own score, or (SHARED) the largest score of the block among the
// query heads of the row's KV head (scores [B, Hq, n1, n2], query head = KV head * group + member)
template <bool SHARED>
__device__ __forceinline__ uint32_t row_key(const SelectArgs& a, long long row, int j, int i) {
    if (!SHARED) return ordered_key(a.scores[row * a.n2 + i]);
    const long long bh = row / a.n1;
    uint32_t kx = 0;
    for (int g2 = 0; g2 < a.group; ++g2)
        kx = max(kx, ordered_key(a.scores[((bh * a.group + g2) * a.n1 + j) * a.n2 + i]));
    return kx;
}

__device__ __forceinline__ int wave_sum(int v) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// The k-th largest of the wave's 64 * N keys (padding keys are 0 and never counted): MSB-first radix search, one
// wave-wide count per bit (a compare per key, the lane masks counted on the scalar unit).  It stops at the first
// bit whose count is exactly k: the keys at or above that trial value are then the k largest (the k-th and the
// (k+1)-th differ), and the value returned separates them just as well as the k-th key itself.
// Always: count(key >= result) >= k, provided k keys are non-zero.
template <int N>
__device__ __forceinline__ uint32_t kth_largest(const uint32_t (&key)[N], int k) {
    uint32_t thr = 0;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t trial = thr | (1u << bit);
        int c = 0;
#pragma unroll
        for (int m = 0; m < N; ++m) c += (int)__popcll(__ballot(key[m] >= trial));
        if (c >= k) thr = trial;
        if (c == k) break;
    }
    return thr;
}

// Writes, in slot order (slot m, then lane), the index of every key above thr and of the first keys equal to thr
// until k are taken; returns how many were written.  index(m) = the block index of the lane's key m.
template <int N, typename Index>
__device__ __forceinline__ int take_largest(const uint32_t (&key)[N], uint32_t thr, int k, int n_slots, int lane,
                                            int32_t* out, Index index) {
    int above = 0;
#pragma unroll
    for (int m = 0; m < N; ++m) above += (int)__popcll(__ballot(key[m] > thr));
    int ties_left = k - above;                         // the keys equal to thr that still fit (0 if none is)
    int written = 0;
#pragma unroll
    for (int m = 0; m < N; ++m) {
        if (m >= n_slots) break;                        // wave-uniform
        const bool valid = key[m] != 0u;                // padding keys are 0, the key of a score never is
        const bool tie = valid && key[m] == thr;
        const unsigned long long tie_mask = __ballot(tie);
        const int tie_rank = __popcll(tie_mask & ((1ull << lane) - 1ull));
        const bool take = valid && (key[m] > thr || (tie && tie_rank < ties_left));
        const unsigned long long take_mask = __ballot(take);
        if (take) out[written + __popcll(take_mask & ((1ull << lane) - 1ull))] = index(m);
        written += __popcll(take_mask);
        ties_left -= min(ties_left, (int)__popcll(tie_mask));
        __builtin_amdgcn_sched_barrier(0);              // keeps the ballot masks of one step from piling up in SGPRs
    }
    return written;
}

constexpr int kCandPerLane = 4;                         // the prefilter keeps at most 64 * 4 candidates per row
constexpr int kPrefilterMaxK = 128;                     // and is used for k up to half that many buckets

// The search over one row with PER_LANE keys per lane (64 * PER_LANE >= the row's candidates).
// Long rows are thinned first: the lane's keys fall into four buckets (slot mod 4), so the wave has 256 bucket
// maxima; the k-th largest of them, T, has at least k keys at or above it, so the k largest keys of the row are
// among the keys >= T (about k..1.4 k of them when large scores are spread over the lanes).  Those are compacted
// in index order into the wave's LDS region (at most 4 per lane) and the exact search runs on them: the same list,
// ties included, with a fraction of the compares.  A row with more than 256 keys >= T (many equal scores) is
// searched in full.
template <int PER_LANE, bool SHARED>
__device__ __forceinline__ int select_row(const SelectArgs& a, long long row, int j, int n_cand, int kj, int lane,
                                          int32_t* out, uint2* cand) {
    uint32_t key[PER_LANE];
#pragma unroll
    for (int m = 0; m < PER_LANE; ++m) {
        const int i = m * 64 + lane;
        const uint32_t kx = row_key<SHARED>(a, row, j, min(i, a.n2 - 1));   // unconditional load: no per-element exec masks to keep
        key[m] = (i < n_cand) ? kx : 0u;                   // 0 is below every trial threshold: never counted
    }
    if (PER_LANE > kCandPerLane && kj <= kPrefilterMaxK) {
        uint32_t top[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int m = 0; m < PER_LANE; ++m) top[m & 3] = max(top[m & 3], key[m]);
        const uint32_t T = kth_largest<4>(top, kj);        // > 0: the row has kj <= 128 valid keys in distinct buckets
        int total = 0;
#pragma unroll
        for (int m = 0; m < PER_LANE; ++m) total += (int)__popcll(__ballot(key[m] >= T));
        if (T != 0u && total <= 64 * kCandPerLane) {        // wave-uniform
            int base = 0;
#pragma unroll
            for (int m = 0; m < PER_LANE; ++m) {
                const bool in = key[m] >= T;
                const unsigned long long mask = __ballot(in);
                if (in) cand[base + __popcll(mask & ((1ull << lane) - 1ull))] = make_uint2(key[m], (unsigned)(m * 64 + lane));
                base += (int)__popcll(mask);
                __builtin_amdgcn_sched_barrier(0);
            }
            // the wave reads back what its own lanes wrote: LDS operations of a wave complete in order
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            uint32_t ck[kCandPerLane]; int ci[kCandPerLane];
#pragma unroll
            for (int c = 0; c < kCandPerLane; ++c) {
                const int pos = c * 64 + lane;
                const uint2 e = cand[min(pos, 64 * kCandPerLane - 1)];
                ck[c] = pos < total ? e.x : 0u; ci[c] = (int)e.y;
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // before the region is written for the wave's next row
            const uint32_t thr = kth_largest<kCandPerLane>(ck, kj);
            return take_largest<kCandPerLane>(ck, thr, kj, (total + 63) / 64, lane, out, [&](int c) { return ci[c]; });
        }
    }
    const uint32_t thr = kth_largest<PER_LANE>(key, kj);
    return take_largest<PER_LANE>(key, thr, kj, (n_cand + 63) / 64, lane, out, [&](int m) { return m * 64 + lane; });
}

// MAX_PER_LANE: 64 * MAX_PER_LANE >= n2, a multiple of 8.  A row early in the sequence has few candidates: the
// search is compiled for eight row lengths (eighths of the maximum) and a wave takes the shortest that holds its row.
template <int MAX_PER_LANE, bool SHARED>
__global__ __launch_bounds__(256) void select_kernel(SelectArgs a) {
    const int lane = threadIdx.x & 63;
    const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.rows) return;
    const int j = (int)(row % a.n1);
    const int diag_lo = j * a.r;
    const int diag_hi = min(a.n2, diag_lo + a.r);
    const int n_local = min(a.local, diag_lo);
    const int n_cand = diag_lo - n_local;
    const int kj = min(a.budget, n_cand);
    int32_t* out = a.idx + row * a.list_len;
    __shared__ uint2 cand_all[4][64 * kCandPerLane];
    uint2* cand = cand_all[threadIdx.x >> 6];

    int written = 0;
    if (kj > 0) {
        constexpr int E = MAX_PER_LANE / 8;
        const int eighths = (n_cand + 64 * E - 1) / (64 * E);          // wave-uniform, 1 .. 8
        switch (eighths) {
            case 1: written = select_row<1 * E, SHARED>(a, row, j, n_cand, kj, lane, out, cand); break;
            case 2: written = select_row<2 * E, SHARED>(a, row, j, n_cand, kj, lane, out, cand); break;
            case 3: written = select_row<3 * E, SHARED>(a, row, j, n_cand, kj, lane, out, cand); break;
            case 4: written = select_row<4 * E, SHARED>(a, row, j, n_cand, kj, lane, out, cand); break;
            case 5: written = select_row<5 * E, SHARED>(a, row, j, n_cand, kj, lane, out, cand); break;
            case 6: written = select_row<6 * E, SHARED>(a, row, j, n_cand, kj, lane, out, cand); break;
            case 7: written = select_row<7 * E, SHARED>(a, row, j, n_cand, kj, lane, out, cand); break;
            default: written = select_row<8 * E, SHARED>(a, row, j, n_cand, kj, lane, out, cand); break;
        }
    }
    // local blocks then the segment's own blocks
    const int fixed = diag_hi - n_cand;
    for (int x = lane; x < fixed; x += 64) out[written + x] = n_cand + x;
    const int total = written + fixed;
    for (int x = total + lane; x < a.list_len; x += 64) out[x] = -1;
    if (lane == 0) a.cnt[row] = total;
}


// Rows longer than 4096 blocks: one 256-thread workgroup per row, thread t owns blocks t, t+256, ...; the same
// radix search with the wave counts added up through LDS, and a compaction whose prefix runs over the four waves.
constexpr int kWideThreads = 256, kWidePerThread = 32;       // 8192 blocks
template <bool SHARED>
__global__ __launch_bounds__(kWideThreads) void select_wide_kernel(SelectArgs a) {
    __shared__ int part[2][4];                             // double-buffered per-wave partial counts
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long row = blockIdx.x;
    const int j = (int)(row % a.n1);
    const int diag_lo = j * a.r;
    const int diag_hi = min(a.n2, diag_lo + a.r);
    const int n_local = min(a.local, diag_lo);
    const int n_cand = diag_lo - n_local;
    const int kj = min(a.budget, n_cand);
    int32_t* out = a.idx + row * a.list_len;

    uint32_t key[kWidePerThread];
#pragma unroll
    for (int m = 0; m < kWidePerThread; ++m) {
        const int i = m * kWideThreads + tid;
        const uint32_t kx = row_key<SHARED>(a, row, j, min(i, a.n2 - 1));
        key[m] = (i < n_cand) ? kx : 0u;                   // 0 is below every trial threshold: never counted
    }
    int step = 0;
    auto block_sum = [&](int v) {                          // same value in every thread; one barrier per call
        v = wave_sum(v);
        if (lane == 0) part[step & 1][wave] = v;
        __syncthreads();
        const int t = part[step & 1][0] + part[step & 1][1] + part[step & 1][2] + part[step & 1][3];
        ++step;
        return t;
    };
    int written = 0;
    if (kj > 0) {                                          // uniform over the workgroup
        uint32_t thr = 0;
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t trial = thr | (1u << bit);
            int c = 0;
#pragma unroll
            for (int m = 0; m < kWidePerThread; ++m) c += (key[m] >= trial) ? 1 : 0;
            const int t = block_sum(c);
            if (t >= kj) thr = trial;
            if (t == kj) break;                            // uniform: exactly the list, see select_row
        }
        int above = 0;
#pragma unroll
        for (int m = 0; m < kWidePerThread; ++m) above += (key[m] > thr) ? 1 : 0;
        int ties_left = kj - block_sum(above);             // >= 1 by construction of thr
#pragma unroll
        for (int m = 0; m < kWidePerThread; ++m) {
            if (m * kWideThreads >= n_cand) break;          // uniform
            const int i = m * kWideThreads + tid;
            const bool valid = key[m] != 0u;
            const bool tie = valid && key[m] == thr;
            // ties before this thread in index order: earlier waves of this step, then earlier lanes
            const unsigned long long tie_mask = __ballot(tie);
            const int tie_w = (int)__popcll(tie_mask);
            if (lane == 0) part[step & 1][wave] = tie_w;
            __syncthreads();
            int tie_before = 0, tie_all = 0;
            for (int w = 0; w < 4; ++w) { const int x = part[step & 1][w]; tie_all += x; if (w < wave) tie_before += x; }
            ++step;
            const int tie_rank = tie_before + (int)__popcll(tie_mask & ((1ull << lane) - 1ull));
            const bool take = valid && (key[m] > thr || (tie && tie_rank < ties_left));
            const unsigned long long take_mask = __ballot(take);
            if (lane == 0) part[step & 1][wave] = (int)__popcll(take_mask);
            __syncthreads();
            int take_before = 0, take_all = 0;
            for (int w = 0; w < 4; ++w) { const int x = part[step & 1][w]; take_all += x; if (w < wave) take_before += x; }
            ++step;
            if (take) out[written + take_before + (int)__popcll(take_mask & ((1ull << lane) - 1ull))] = i;
            written += take_all;
            ties_left -= min(ties_left, tie_all);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    const int fixed = diag_hi - n_cand;
    for (int x = tid; x < fixed; x += kWideThreads) out[written + x] = n_cand + x;
    const int total = written + fixed;
    for (int x = total + tid; x < a.list_len; x += kWideThreads) out[x] = -1;
    if (tid == 0) a.cnt[row] = total;
}

}  // namespace

template <bool SHARED>
hipError_t launch_select_impl(const Shape& sh, const float* scores, int32_t* idx, int32_t* cnt, hipStream_t st) {
    SelectArgs a;
    a.scores = scores; a.idx = idx; a.cnt = cnt;
    a.rows = (long long)sh.batch * (SHARED ? sh.hkv : sh.hq) * sh.n1;
    a.group = sh.hq / sh.hkv;
    a.n1 = sh.n1; a.n2 = sh.n2; a.r = sh.r; a.budget = sh.budget; a.local = sh.local; a.list_len = sh.list_len;
    const unsigned grid = (unsigned)((a.rows + 3) / 4);
    if (sh.n2 <= 64 * 8) hipLaunchKernelGGL((select_kernel<8, SHARED>), dim3(grid), dim3(256), 0, st, a);
    else if (sh.n2 <= 64 * 32) hipLaunchKernelGGL((select_kernel<32, SHARED>), dim3(grid), dim3(256), 0, st, a);
    else if (sh.n2 <= 64 * 64) hipLaunchKernelGGL((select_kernel<64, SHARED>), dim3(grid), dim3(256), 0, st, a);
    else {
        if (a.rows > 0x7fffffffLL || sh.n2 > kWideThreads * kWidePerThread) return hipErrorInvalidValue;
        hipLaunchKernelGGL(select_wide_kernel<SHARED>, dim3((unsigned)a.rows), dim3(kWideThreads), 0, st, a);
    }
    return hipGetLastError();
}

hipError_t launch_select(const Shape& sh, const float* scores, int32_t* idx, int32_t* cnt, bool shared, hipStream_t st) {
    return shared ? launch_select_impl<true>(sh, scores, idx, cnt, st) : launch_select_impl<false>(sh, scores, idx, cnt, st);
}

}  // namespace cp
