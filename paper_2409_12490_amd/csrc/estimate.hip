// Algorithm 1 "Estimation of Query Criticality in One Layer" on gfx950.
//
//   pool_kernel   element-wise max/min representatives of every query segment and key block
//                 (the reshape + max/min lines).  Streams Q and K once: HBM-bound.
//   score_kernel  four representative products, row softmax over blocks, (S1+S3)/2 vs (S2+S4)/2,
//                 element-wise max, block causal mask, layer fusion.
#include "kernels.h"

namespace cp {
namespace {

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
// both inputs hold exact bf16 values, so taking the upper halves loses nothing
__device__ __forceinline__ uint32_t pack_bf16_exact(float lo, float hi) {
    return (__float_as_uint(lo) >> 16) | (__float_as_uint(hi) & 0xffff0000u);
}

struct PoolArgs {
    const void* q; const void* k; void* qrep; void* krep;
    int n, s, b, n1, n2, hq, hkv;
    long long q_groups, k_groups;          // B*Hq*n1, B*Hkv*n2
    long long qs0, qs1, qs2, ks0, ks1, ks2;
};

// One wavefront per group (a segment of Q or a block of K).  bf16: a lane owns 8 channels (16 B),
// 16 lanes cover one 256 B token row, the wave covers 4 rows per load.
__global__ __launch_bounds__(256) void pool_bf16_kernel(PoolArgs a) {
    const int lane = threadIdx.x & 63;
    const long long gid = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (gid >= a.q_groups + a.k_groups) return;
    const uint16_t* src; uint16_t* dst; long long tok_stride; int t0, t1;
    if (gid < a.q_groups) {
        const int j = (int)(gid % a.n1); const long long bh = gid / a.n1;
        const int h = (int)(bh % a.hq); const int bb = (int)(bh / a.hq);
        src = (const uint16_t*)a.q + bb * a.qs0 + h * a.qs1; tok_stride = a.qs2;
        t0 = j * a.s; t1 = min(a.n, t0 + a.s);
        dst = (uint16_t*)a.qrep + gid * 2 * kHeadDim;
    } else {
        const long long g = gid - a.q_groups;
        const int i = (int)(g % a.n2); const long long bh = g / a.n2;
        const int h = (int)(bh % a.hkv); const int bb = (int)(bh / a.hkv);
        src = (const uint16_t*)a.k + bb * a.ks0 + h * a.ks1; tok_stride = a.ks2;
        t0 = i * a.b; t1 = min(a.n, t0 + a.b);
        dst = (uint16_t*)a.krep + g * 2 * kHeadDim;
    }
    const int chunk = lane & 15, rsub = lane >> 4;
    float hi[8], lo[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { hi[e] = -INFINITY; lo[e] = INFINITY; }
    const uint16_t* p = src + (long long)(t0 + rsub) * tok_stride + chunk * 8;
    int t = t0 + rsub;
    for (; t + 12 < t1; t += 16) {           // four independent 16 B loads in flight
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = *(const uint4*)(p + (long long)(4 * u) * tok_stride);
        p += 16 * tok_stride;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float x0 = bf16_lo(w[e]), x1 = bf16_hi(w[e]);
                hi[2 * e] = fmaxf(hi[2 * e], x0); lo[2 * e] = fminf(lo[2 * e], x0);
                hi[2 * e + 1] = fmaxf(hi[2 * e + 1], x1); lo[2 * e + 1] = fminf(lo[2 * e + 1], x1);
            }
        }
    }
    for (; t < t1; t += 4) {
        const uint4 v = *(const uint4*)p; p += 4 * tok_stride;
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float x0 = bf16_lo(w[e]), x1 = bf16_hi(w[e]);
            hi[2 * e] = fmaxf(hi[2 * e], x0); lo[2 * e] = fminf(lo[2 * e], x0);
            hi[2 * e + 1] = fmaxf(hi[2 * e + 1], x1); lo[2 * e + 1] = fminf(lo[2 * e + 1], x1);
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        hi[e] = fmaxf(hi[e], __shfl_xor(hi[e], 16)); hi[e] = fmaxf(hi[e], __shfl_xor(hi[e], 32));
        lo[e] = fminf(lo[e], __shfl_xor(lo[e], 16)); lo[e] = fminf(lo[e], __shfl_xor(lo[e], 32));
    }
    if (rsub == 0) {
        uint4 o;
        o.x = pack_bf16_exact(hi[0], hi[1]); o.y = pack_bf16_exact(hi[2], hi[3]);
        o.z = pack_bf16_exact(hi[4], hi[5]); o.w = pack_bf16_exact(hi[6], hi[7]);
        *(uint4*)(dst + chunk * 8) = o;
        o.x = pack_bf16_exact(lo[0], lo[1]); o.y = pack_bf16_exact(lo[2], lo[3]);
        o.z = pack_bf16_exact(lo[4], lo[5]); o.w = pack_bf16_exact(lo[6], lo[7]);
        *(uint4*)(dst + kHeadDim + chunk * 8) = o;
    }
}

// fp32: a lane owns 4 channels (16 B), 32 lanes cover one 512 B row, the wave covers 2 rows per load.
__global__ __launch_bounds__(256) void pool_fp32_kernel(PoolArgs a) {
    const int lane = threadIdx.x & 63;
    const long long gid = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (gid >= a.q_groups + a.k_groups) return;
    const float* src; float* dst; long long tok_stride; int t0, t1;
    if (gid < a.q_groups) {
        const int j = (int)(gid % a.n1); const long long bh = gid / a.n1;
        const int h = (int)(bh % a.hq); const int bb = (int)(bh / a.hq);
        src = (const float*)a.q + bb * a.qs0 + h * a.qs1; tok_stride = a.qs2;
        t0 = j * a.s; t1 = min(a.n, t0 + a.s);
        dst = (float*)a.qrep + gid * 2 * kHeadDim;
    } else {
        const long long g = gid - a.q_groups;
        const int i = (int)(g % a.n2); const long long bh = g / a.n2;
        const int h = (int)(bh % a.hkv); const int bb = (int)(bh / a.hkv);
        src = (const float*)a.k + bb * a.ks0 + h * a.ks1; tok_stride = a.ks2;
        t0 = i * a.b; t1 = min(a.n, t0 + a.b);
        dst = (float*)a.krep + g * 2 * kHeadDim;
    }
    const int chunk = lane & 31, rsub = lane >> 5;
    float hi[4], lo[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) { hi[e] = -INFINITY; lo[e] = INFINITY; }
    for (int t = t0 + rsub; t < t1; t += 2) {
        const float4 v = *(const float4*)(src + (long long)t * tok_stride + chunk * 4);
        const float x[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) { hi[e] = fmaxf(hi[e], x[e]); lo[e] = fminf(lo[e], x[e]); }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        hi[e] = fmaxf(hi[e], __shfl_xor(hi[e], 32));
        lo[e] = fminf(lo[e], __shfl_xor(lo[e], 32));
    }
    if (rsub == 0) {
        *(float4*)(dst + chunk * 4) = make_float4(hi[0], hi[1], hi[2], hi[3]);
        *(float4*)(dst + kHeadDim + chunk * 4) = make_float4(lo[0], lo[1], lo[2], lo[3]);
    }
}

// ---------------------------------------------------------------------------------------------
// score: one workgroup per (batch, head, segment) row of S.
// ---------------------------------------------------------------------------------------------
struct ScoreArgs {
    const void* qrep; const void* krep; const float* prev; float* scores;
    int hq, hkv, n1, n2, r, domain;
    float scale, alpha;
};

__device__ __forceinline__ float block_reduce_max(float v, float* red) {
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}
__device__ __forceinline__ float block_reduce_sum(float v, float* red) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

template <bool BF16>
__global__ __launch_bounds__(256) void score_valu_kernel(ScoreArgs a) {
    extern __shared__ float smem[];
    float* qr = smem;                 // [2][128]
    float* red = smem + 2 * kHeadDim; // [4]
    float* z = red + 4;               // [4][n2]
    const int j = blockIdx.x, h = blockIdx.y, bb = blockIdx.z;
    const int tid = threadIdx.x;
    const long long qrow = ((long long)bb * a.hq + h) * a.n1 + j;
    const int g = h / (a.hq / a.hkv);
    const long long kbase = ((long long)bb * a.hkv + g) * a.n2;
    if (BF16) {
        const uint16_t* src = (const uint16_t*)a.qrep + qrow * 2 * kHeadDim;
        qr[tid] = __uint_as_float((uint32_t)src[tid] << 16);
    } else {
        qr[tid] = ((const float*)a.qrep)[qrow * 2 * kHeadDim + tid];
    }
    __syncthreads();
    const int vis = min(a.n2, (j + 1) * a.r);               // first block wholly after the segment
    const int dom = a.domain == 0 ? a.n2 : vis;
    for (int i = tid; i < a.n2; i += 256) {
        float zz[4] = {0.f, 0.f, 0.f, 0.f};
        if (BF16) {
            const uint4* km = (const uint4*)((const uint16_t*)a.krep + (kbase + i) * 2 * kHeadDim);
#pragma unroll 4
            for (int c = 0; c < 16; ++c) {
                const uint4 hi4 = km[c], lo4 = km[16 + c];
                const uint32_t wh[4] = {hi4.x, hi4.y, hi4.z, hi4.w}, wl[4] = {lo4.x, lo4.y, lo4.z, lo4.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int ch = c * 8 + 2 * e;
                    const float kh0 = bf16_lo(wh[e]), kh1 = bf16_hi(wh[e]);
                    const float kl0 = bf16_lo(wl[e]), kl1 = bf16_hi(wl[e]);
                    const float qh0 = qr[ch], qh1 = qr[ch + 1], ql0 = qr[kHeadDim + ch], ql1 = qr[kHeadDim + ch + 1];
                    zz[0] = fmaf(qh0, kh0, zz[0]); zz[0] = fmaf(qh1, kh1, zz[0]);
                    zz[1] = fmaf(qh0, kl0, zz[1]); zz[1] = fmaf(qh1, kl1, zz[1]);
                    zz[2] = fmaf(ql0, kh0, zz[2]); zz[2] = fmaf(ql1, kh1, zz[2]);
                    zz[3] = fmaf(ql0, kl0, zz[3]); zz[3] = fmaf(ql1, kl1, zz[3]);
                }
            }
        } else {
            const float4* km = (const float4*)((const float*)a.krep + (kbase + i) * 2 * kHeadDim);
#pragma unroll 4
            for (int c = 0; c < 32; ++c) {
                const float4 hi4 = km[c], lo4 = km[32 + c];
                const float kh[4] = {hi4.x, hi4.y, hi4.z, hi4.w}, kl[4] = {lo4.x, lo4.y, lo4.z, lo4.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float qh = qr[c * 4 + e], ql = qr[kHeadDim + c * 4 + e];
                    zz[0] = fmaf(qh, kh[e], zz[0]); zz[1] = fmaf(qh, kl[e], zz[1]);
                    zz[2] = fmaf(ql, kh[e], zz[2]); zz[3] = fmaf(ql, kl[e], zz[3]);
                }
            }
        }
        const bool in_dom = i < dom;
#pragma unroll
        for (int w = 0; w < 4; ++w) z[w * a.n2 + i] = in_dom ? zz[w] * a.scale : -INFINITY;
    }
    __syncthreads();
    float mx[4], inv[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        float m = -INFINITY;
        for (int i = tid; i < a.n2; i += 256) m = fmaxf(m, z[w * a.n2 + i]);
        mx[w] = block_reduce_max(m, red);
    }
    constexpr float kLog2e = 1.4426950408889634f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        float sum = 0.f;
        for (int i = tid; i < a.n2; i += 256) {
            const float e = exp2f((z[w * a.n2 + i] - mx[w]) * kLog2e);
            z[w * a.n2 + i] = e;
            sum += e;
        }
        inv[w] = 1.0f / block_reduce_sum(sum, red);
    }
    float* out = a.scores + qrow * a.n2;
    const float* prev = a.prev ? a.prev + qrow * a.n2 : nullptr;
    for (int i = tid; i < a.n2; i += 256) {
        const float s1 = z[i] * inv[0], s2 = z[a.n2 + i] * inv[1];
        const float s3 = z[2 * a.n2 + i] * inv[2], s4 = z[3 * a.n2 + i] * inv[3];
        float s = fmaxf((s1 + s3) * 0.5f, (s2 + s4) * 0.5f);
        if (i >= vis) s = 0.f;
        if (prev) s = a.alpha * s + (1.0f - a.alpha) * prev[i];
        if (fabsf(s) < 1.17549435e-38f) s = 0.f;
        out[i] = s;
    }
}


// ---------------------------------------------------------------------------------------------
// score, bf16: the four representative products as one bf16 MFMA GEMM (representatives are exact
// bf16 values, so every product is exact and only the fp32 accumulation rounds).
//
// Workgroup = 4 waves = 16 segments of one (batch, head).  A operand (32 rows) = [Q_max of the 16
// segments ; Q_min of the 16 segments], kept in registers.  B operand = 32 blocks of K_max, then the same
// 32 blocks of K_min, read straight from global memory (1 MiB per KV head, L2 resident).  In the 32x32
// result a lane holds, for its block column, both query representatives of 8 segments; with the two
// MFMA results that is all of S1..S4 for 8 (segment, block) pairs in one lane.  Wave w takes the block
// tiles w, w+4, ...  Pass 1 finds every row's max and sum of exponentials (online, per lane, then
// reduced over lanes and waves); pass 2 recomputes the products and writes the combined score.
// ---------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) {
    union { uint4 u; bf16x8 b; } c; c.u = v; return c.b;
}

constexpr int kSegPerWg = 16;

__global__ __launch_bounds__(256) void score_mfma_kernel(ScoreArgs a) {
    __shared__ float red_m[4][2][2][kSegPerWg];   // [wave][a][bb][segment]
    __shared__ float red_l[4][2][2][kSegPerWg];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;
    const int j0 = blockIdx.x * kSegPerWg, h = blockIdx.y, bb_ = blockIdx.z;
    const int g = h / (a.hq / a.hkv);
    const long long qrow0 = ((long long)bb_ * a.hq + h) * a.n1;
    const long long kbase = ((long long)bb_ * a.hkv + g) * a.n2;
    constexpr float kLog2e = 1.4426950408889634f;
    const float c = a.scale * kLog2e;                        // logits in log2 units

    // A fragments: row m = l32 -> representative (m >> 4) of segment j0 + (m & 15)
    bf16x8 qf[8];
    {
        const int jq = min(j0 + (l32 & 15), a.n1 - 1);
        const uint16_t* src = (const uint16_t*)a.qrep + ((qrow0 + jq) * 2 + (l32 >> 4)) * kHeadDim + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[ks] = as_bf16x8(*(const uint4*)(src + 16 * ks));
    }
    // the lane's 8 segments: register r of an accumulator is row 8*(r>>2) + 4*hh + (r&3)
    //   representative = r >> 3, segment slot x = ((r >> 2) & 1) * 4 + (r & 3) -> segment j0 + 8*((r>>2)&1) + 4*hh + (r&3)
    int vis[8];                                             // first block wholly after the segment
#pragma unroll
    for (int x = 0; x < 8; ++x) {
        const int j = j0 + 8 * (x >> 2) + 4 * hh + (x & 3);
        vis[x] = min(a.n2, (j + 1) * a.r);
    }
    const int ntile = (a.n2 + 31) / 32;

    // Z for one 32-block tile: z[bb][r]
    auto tile_z = [&](int nt, f32x16 (&z)[2]) {
        const int i = min(nt * 32 + l32, a.n2 - 1);
        const uint16_t* src = (const uint16_t*)a.krep + (kbase + i) * 2 * kHeadDim + 8 * hh;
#pragma unroll
        for (int b2 = 0; b2 < 2; ++b2) {
#pragma unroll
            for (int r = 0; r < 16; ++r) z[b2][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 kf = as_bf16x8(*(const uint4*)(src + b2 * kHeadDim + 16 * ks));
                z[b2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[ks], kf, z[b2], 0, 0, 0);
            }
        }
    };

    // ---- pass 1: per lane online max / sum of 2^(c z) over its block columns -------------------
    float m[2][16], l[2][16];
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
        for (int r = 0; r < 16; ++r) { m[b2][r] = -INFINITY; l[b2][r] = 0.f; }
    for (int nt = wave; nt < ntile; nt += 4) {
        f32x16 z[2];
        tile_z(nt, z);
        const int i = nt * 32 + l32;
#pragma unroll
        for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int x = ((r >> 2) & 1) * 4 + (r & 3);
                const bool in_dom = i < (a.domain == 0 ? a.n2 : vis[x]);
                const float v = in_dom ? z[b2][r] * c : -INFINITY;
                const float mn = fmaxf(m[b2][r], v);
                const float ms = (mn == -INFINITY) ? 0.f : mn;
                l[b2][r] = l[b2][r] * exp2f(m[b2][r] - ms) + exp2f(v - ms);
                m[b2][r] = mn;
            }
    }
    // reduce over the 32 lanes of a half (block columns), then over the waves
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float mm = m[b2][r], ll = l[b2][r];
#pragma unroll
            for (int o = 16; o > 0; o >>= 1) {
                const float m2 = __shfl_xor(mm, o), l2 = __shfl_xor(ll, o);
                const float mn = fmaxf(mm, m2);
                const float ms = (mn == -INFINITY) ? 0.f : mn;
                ll = ll * exp2f(mm - ms) + l2 * exp2f(m2 - ms);
                mm = mn;
            }
            if (l32 == 0) {
                const int seg = 8 * ((r >> 2) & 1) + 4 * hh + (r & 3);
                red_m[wave][r >> 3][b2][seg] = mm;
                red_l[wave][r >> 3][b2][seg] = ll;
            }
        }
    __syncthreads();
    float inv[2][16];                                       // 1 / sum, and m becomes the final max
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int seg = 8 * ((r >> 2) & 1) + 4 * hh + (r & 3);
            float mm = -INFINITY;
#pragma unroll
            for (int w = 0; w < 4; ++w) mm = fmaxf(mm, red_m[w][r >> 3][b2][seg]);
            const float ms = (mm == -INFINITY) ? 0.f : mm;
            float ll = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) ll += red_l[w][r >> 3][b2][seg] * exp2f(red_m[w][r >> 3][b2][seg] - ms);
            m[b2][r] = ms;
            inv[b2][r] = ll > 0.f ? 1.0f / ll : 0.f;
        }

    // ---- pass 2: recompute, normalise, combine, mask, fuse, store -------------------------------
    for (int nt = wave; nt < ntile; nt += 4) {
        f32x16 z[2];
        tile_z(nt, z);
        const int i = nt * 32 + l32;
        if (i >= a.n2) continue;
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const int j = j0 + 8 * (x >> 2) + 4 * hh + (x & 3);
            if (j >= a.n1) continue;
            const int r0 = 4 * (x >> 2) + (x & 3), r1 = r0 + 8;   // Q_max row and Q_min row of the segment
            const bool in_dom = i < (a.domain == 0 ? a.n2 : vis[x]);
            float p[2][2];
#pragma unroll
            for (int b2 = 0; b2 < 2; ++b2) {
                p[0][b2] = in_dom ? exp2f(z[b2][r0] * c - m[b2][r0]) * inv[b2][r0] : 0.f;
                p[1][b2] = in_dom ? exp2f(z[b2][r1] * c - m[b2][r1]) * inv[b2][r1] : 0.f;
            }
            // S1 = (max,max), S2 = (max,min), S3 = (min,max), S4 = (min,min)
            float sc = fmaxf((p[0][0] + p[1][0]) * 0.5f, (p[0][1] + p[1][1]) * 0.5f);
            if (i >= vis[x]) sc = 0.f;
            const long long off = (qrow0 + j) * a.n2 + i;
            if (a.prev) sc = a.alpha * sc + (1.0f - a.alpha) * a.prev[off];
            if (fabsf(sc) < 1.17549435e-38f) sc = 0.f;
            a.scores[off] = sc;
        }
    }
}

}  // namespace

hipError_t launch_pool(const Shape& sh, const void* q, const void* k, void* qrep, void* krep, hipStream_t st) {
    PoolArgs a;
    a.q = q; a.k = k; a.qrep = qrep; a.krep = krep;
    a.n = sh.n; a.s = sh.s; a.b = sh.b; a.n1 = sh.n1; a.n2 = sh.n2; a.hq = sh.hq; a.hkv = sh.hkv;
    a.q_groups = (long long)sh.batch * sh.hq * sh.n1;
    a.k_groups = (long long)sh.batch * sh.hkv * sh.n2;
    a.qs0 = sh.qs[0]; a.qs1 = sh.qs[1]; a.qs2 = sh.qs[2];
    a.ks0 = sh.kvs[0]; a.ks1 = sh.kvs[1]; a.ks2 = sh.kvs[2];
    const long long groups = a.q_groups + a.k_groups;
    const unsigned grid = (unsigned)((groups + 3) / 4);
    if (sh.dtype == 1) hipLaunchKernelGGL(pool_bf16_kernel, dim3(grid), dim3(256), 0, st, a);
    else hipLaunchKernelGGL(pool_fp32_kernel, dim3(grid), dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_score(const Shape& sh, const void* qrep, const void* krep, const float* prev, float* scores,
                        hipStream_t st) {
    ScoreArgs a;
    a.qrep = qrep; a.krep = krep; a.prev = prev; a.scores = scores;
    a.hq = sh.hq; a.hkv = sh.hkv; a.n1 = sh.n1; a.n2 = sh.n2; a.r = sh.r; a.domain = sh.softmax_domain;
    a.scale = sh.score_scale; a.alpha = sh.alpha;
    if (sh.dtype == 1) {
        dim3 grid_m((sh.n1 + kSegPerWg - 1) / kSegPerWg, sh.hq, sh.batch);
        hipLaunchKernelGGL(score_mfma_kernel, grid_m, dim3(256), 0, st, a);
        return hipGetLastError();
    }
    const size_t smem = (2 * kHeadDim + 4 + 4 * (size_t)sh.n2) * sizeof(float);
    dim3 grid(sh.n1, sh.hq, sh.batch);
    const void* fn = sh.dtype == 1 ? (const void*)score_valu_kernel<true> : (const void*)score_valu_kernel<false>;
    if (smem > 48 * 1024) {
        const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    if (sh.dtype == 1) hipLaunchKernelGGL(score_valu_kernel<true>, grid, dim3(256), smem, st, a);
    else hipLaunchKernelGGL(score_valu_kernel<false>, grid, dim3(256), smem, st, a);
    return hipGetLastError();
}

}  // namespace cp
