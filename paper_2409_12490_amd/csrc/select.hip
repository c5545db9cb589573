// Algorithm 2 "Pruned Attention", the line  I = argtop_k(S[j], B / block size),
// plus the local and diagonal blocks that are always kept.
//
// One wavefront per (batch, head, segment) row.  The row lives in registers (lane l owns blocks
// l, l+64, ...).  Scores are mapped to order-preserving unsigned keys; the k-th largest key is found
// by an MSB-first radix search (one wave-wide count per bit); everything above it is taken, ties at
// the threshold go to the smallest indices, and the result is compacted in index order, so the
// list comes out ascending.
#include "kernels.h"

namespace cp {
namespace {

struct SelectArgs {
    const float* scores; int32_t* idx; int32_t* cnt;
    long long rows;            // B*H*n1
    int n1, n2, r, budget, local, list_len;
};

__device__ __forceinline__ uint32_t ordered_key(float x) {
    uint32_t u = __float_as_uint(x);
    if (u == 0x80000000u) u = 0;                       // -0 ranks with +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int wave_sum(int v) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

template <int PER_LANE>
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
    const float* s = a.scores + row * a.n2;
    int32_t* out = a.idx + row * a.list_len;

    uint32_t key[PER_LANE];
#pragma unroll
    for (int m = 0; m < PER_LANE; ++m) {
        const int i = m * 64 + lane;
        key[m] = (i < n_cand) ? ordered_key(s[i]) : 0u;   // only compared where i < n_cand
    }
    int written = 0;
    if (kj > 0) {
        uint32_t thr = 0;
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t trial = thr | (1u << bit);
            int c = 0;
#pragma unroll
            for (int m = 0; m < PER_LANE; ++m) c += (m * 64 + lane < n_cand && key[m] >= trial) ? 1 : 0;
            if (wave_sum(c) >= kj) thr = trial;
        }
        int above = 0;
#pragma unroll
        for (int m = 0; m < PER_LANE; ++m) above += (m * 64 + lane < n_cand && key[m] > thr) ? 1 : 0;
        int ties_left = kj - wave_sum(above);          // >= 1 by construction of thr
#pragma unroll
        for (int m = 0; m < PER_LANE; ++m) {
            if (m * 64 >= n_cand) break;                // wave-uniform
            const int i = m * 64 + lane;
            const bool valid = i < n_cand;
            const bool tie = valid && key[m] == thr;
            const unsigned long long tie_mask = __ballot(tie);
            const int tie_rank = __popcll(tie_mask & ((1ull << lane) - 1ull));
            const bool take = valid && (key[m] > thr || (tie && tie_rank < ties_left));
            const unsigned long long take_mask = __ballot(take);
            if (take) out[written + __popcll(take_mask & ((1ull << lane) - 1ull))] = i;
            written += __popcll(take_mask);
            ties_left -= min(ties_left, (int)__popcll(tie_mask));
        }
    }
    // local blocks then the segment's own blocks
    const int fixed = diag_hi - n_cand;
    for (int x = lane; x < fixed; x += 64) out[written + x] = n_cand + x;
    const int total = written + fixed;
    for (int x = total + lane; x < a.list_len; x += 64) out[x] = -1;
    if (lane == 0) a.cnt[row] = total;
}

}  // namespace

hipError_t launch_select(const Shape& sh, const float* scores, int32_t* idx, int32_t* cnt, hipStream_t st) {
    SelectArgs a;
    a.scores = scores; a.idx = idx; a.cnt = cnt;
    a.rows = (long long)sh.batch * sh.hq * sh.n1;
    a.n1 = sh.n1; a.n2 = sh.n2; a.r = sh.r; a.budget = sh.budget; a.local = sh.local; a.list_len = sh.list_len;
    const unsigned grid = (unsigned)((a.rows + 3) / 4);
    if (sh.n2 <= 64 * 8) hipLaunchKernelGGL(select_kernel<8>, dim3(grid), dim3(256), 0, st, a);
    else if (sh.n2 <= 64 * 32) hipLaunchKernelGGL(select_kernel<32>, dim3(grid), dim3(256), 0, st, a);
    else hipLaunchKernelGGL(select_kernel<128>, dim3(grid), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace cp
