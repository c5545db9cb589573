// Algorithm 2 "Pruned Attention", the line  I = argtop_k(S[j], B / block size),
// plus the local and diagonal blocks that are always kept.
//
// One wavefront per (batch, head, segment) row.  The row lives in registers (lane l owns blocks
// l, l+64, ...).  Scores are mapped to order-preserving unsigned keys; the k-th largest key is found
// by an MSB-first radix search (one wave-wide count per bit: a compare per key, the lane masks counted on the
// scalar unit); everything above it is taken, ties at
// the threshold go to the smallest indices, and the result is compacted in index order, so the
// list comes out ascending.
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

template <int PER_LANE, bool SHARED>
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

    uint32_t key[PER_LANE];
#pragma unroll
    for (int m = 0; m < PER_LANE; ++m) {
        const int i = m * 64 + lane;
        const uint32_t kx = row_key<SHARED>(a, row, j, min(i, a.n2 - 1));   // unconditional load: no per-element exec masks to keep
        key[m] = (i < n_cand) ? kx : 0u;                   // 0 is below every trial threshold: never counted
    }
    int written = 0;
    if (kj > 0) {
        uint32_t thr = 0;
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t trial = thr | (1u << bit);
            int c = 0;                                  // wave-wide count on the scalar unit: one compare per key
#pragma unroll
            for (int m = 0; m < PER_LANE; ++m) c += (int)__popcll(__ballot(key[m] >= trial));   // trial >= 1: padding keys stay out
            if (c >= kj) thr = trial;
        }
        int above = 0;
#pragma unroll
        for (int m = 0; m < PER_LANE; ++m) above += (int)__popcll(__ballot(key[m] > thr));
        int ties_left = kj - above;                    // >= 1 by construction of thr
#pragma unroll
        for (int m = 0; m < PER_LANE; ++m) {
            if (m * 64 >= n_cand) break;                // wave-uniform
            const int i = m * 64 + lane;
            const bool valid = key[m] != 0u;            // padding keys are 0, the key of a score never is
            const bool tie = valid && key[m] == thr;
            const unsigned long long tie_mask = __ballot(tie);
            const int tie_rank = __popcll(tie_mask & ((1ull << lane) - 1ull));
            const bool take = valid && (key[m] > thr || (tie && tie_rank < ties_left));
            const unsigned long long take_mask = __ballot(take);
            if (take) out[written + __popcll(take_mask & ((1ull << lane) - 1ull))] = i;
            written += __popcll(take_mask);
            ties_left -= min(ties_left, (int)__popcll(tie_mask));
            __builtin_amdgcn_sched_barrier(0);          // keeps the ballot masks of one step from piling up in SGPRs
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
            if (block_sum(c) >= kj) thr = trial;
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
