// Algorithm 1 "Estimation of Query Criticality in One Layer" on gfx950.
//
//   pool_kernel   element-wise max/min representatives of every query segment and key block
//                 (the reshape + max/min lines).  Streams Q and K once: HBM-bound.
//   score_kernel  four representative products, row softmax over blocks, (S1+S3)/2 vs (S2+S4)/2,
//                 element-wise max, block causal mask, layer fusion.
#include "kernels.h"

namespace cp {
namespace {

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
// both inputs hold exact bf16 values, so taking the upper halves loses nothing
__device__ __forceinline__ uint32_t pack_bf16_exact(float lo, float hi) {
    return (__float_as_uint(lo) >> 16) | (__float_as_uint(hi) & 0xffff0000u);
}

// 16 bytes that are read once: streamed past the caches (measured: 6.2 instead of 5.4 TB/s for the pooling pass)
typedef __attribute__((ext_vector_type(4))) unsigned pool_u32x4;
__device__ __forceinline__ uint4 load_once(const void* p) {
    const pool_u32x4 x = __builtin_nontemporal_load((const pool_u32x4*)p);
    return make_uint4(x[0], x[1], x[2], x[3]);
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
    for (; t + 28 < t1; t += 32) {           // eight independent 16 B loads in flight
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = load_once(p + (long long)(4 * u) * tok_stride);
        p += 32 * tok_stride;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float x0 = bf16_lo(w[e]), x1 = bf16_hi(w[e]);
                hi[2 * e] = fmaxf(hi[2 * e], x0); lo[2 * e] = fminf(lo[2 * e], x0);
                hi[2 * e + 1] = fmaxf(hi[2 * e + 1], x1); lo[2 * e + 1] = fminf(lo[2 * e + 1], x1);
            }
        }
    }
    for (; t + 12 < t1; t += 16) {           // four independent 16 B loads in flight
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = load_once(p + (long long)(4 * u) * tok_stride);
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
        const uint4 v = load_once(p); p += 4 * tok_stride;
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
// score, fp32 (correctness configuration): one workgroup per (batch, head, segment) row of S, plain fp32 FMA.
// ---------------------------------------------------------------------------------------------
struct ScoreArgs {
    const void* qrep; const void* krep; const float* prev; float* scores;
    float* stats;                          // bf16 path: per-chunk softmax statistics (see score_stats_kernel)
    int hq, hkv, n1, n2, r, domain;
    int nchunk, n1_pad;
    int parts;                             // bf16 path: waves that share 16 segments and split the tiles of a chunk (1, 2, 4, 8)
    float scale, alpha;
};
constexpr int kScoreWaves = 8;             // waves per workgroup of the bf16 score kernels, 16 segments each
constexpr int kScoreSegPerWg = 16 * kScoreWaves;
constexpr int kScoreChunk = 256;           // blocks per workgroup
constexpr int kScorePiece = 64;            // blocks per LDS buffer (32 KiB of representatives), two buffers

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
    qr[tid] = ((const float*)a.qrep)[qrow * 2 * kHeadDim + tid];
    __syncthreads();
    const int vis = min(a.n2, (j + 1) * a.r);               // first block wholly after the segment
    const int dom = a.domain == 0 ? a.n2 : vis;
    for (int i = tid; i < a.n2; i += 256) {
        float zz[4] = {0.f, 0.f, 0.f, 0.f};
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
// score, bf16: the four representative products as bf16 MFMA GEMMs (representatives are exact bf16
// values, so every product is exact and only the fp32 accumulation rounds).
//
// The blocks of a (batch, head) are cut into chunks of 256; a workgroup = 8 waves takes one chunk and 128
// segments, wave w the segments 16w .. 16w+15.  Z^T = K_rep . Q_rep^T: the A operand is a tile of 32 blocks
// of K_max (then K_min); the chunk's representatives go global -> LDS once for all eight waves in four
// pieces of 64 blocks (global_load_lds, no register staging, two 32 KiB buffers: the next piece lands while
// the current one is used; two workgroups per compute unit); the B operand, column n = (segment n >> 1, representative n & 1), stays in
// registers.  A lane then holds, for its column, 16 blocks of the tile in registers: the softmax
// statistics over blocks are in-lane reductions plus one exchange between the wave halves, and the two
// query representatives of a segment sit in neighbouring lanes (one DPP exchange per score).
//
//   score_stats_kernel   per chunk and column: max and sum of 2^(c z - max) of the two products  -> stats
//   score_write_kernel   merges the chunk statistics, recomputes the products of its chunk, normalises,
//                        combines (S1+S3)/2 vs (S2+S4)/2, masks, fuses, stores.  Chunks that lie wholly
//                        after every segment of the workgroup are written without any product.
// ---------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
#define SCORE_LDS(T, off) ((__attribute__((address_space(3))) T*)(uintptr_t)(off))

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) {
    union { uint4 u; bf16x8 b; } c; c.u = v; return c.b;
}
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) {
    union { u32x4 u; bf16x8 b; } c; c.u = v; return c.b;
}
__device__ __forceinline__ float halves_max(float x) {     // max over lanes l and l ^ 32
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float halves_sum(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float neighbour(float x) {      // the value of lane l ^ 1
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xF, 0xF, true));
}

struct ScoreTile {
    static constexpr int kTileBlocks = 32;                  // blocks per MFMA tile
    static constexpr int kTileBytes = kTileBlocks * 2 * kHeadDim * 2;   // max row + min row per block, bf16
};

// The part both kernels share: the workgroup's coordinates, the B operand, the staged A tiles.
struct ScoreCtx {
    int lane, wave, l32, hh;
    int part;                                               // tiles nt = part (mod parts) of the chunk are this wave's
    int chunk, j0, seg, rep, h, bb_;
    int i_begin, i_end, ntile;                              // blocks of the chunk, tiles of 32
    long long qrow0;                                        // row of segment 0 of this (batch, head) in scores
    const uint16_t* ksrc;                                   // K representatives of block 0 of this KV head
    int vis;                                                // first block wholly after the lane's segment
    int vis_wg;                                             // ... after the last segment of the workgroup
    int vis_wave, vis_wave_max;                             // ... after the first / last segment of the wave
    bf16x8 qf[8];
    unsigned lds0;
};

__device__ __forceinline__ void score_setup(const ScoreArgs& a, ScoreCtx& c, unsigned lds0) {
    const int tid = threadIdx.x;
    c.lane = tid & 63; c.wave = tid >> 6; c.l32 = c.lane & 31; c.hh = c.lane >> 5;
    c.chunk = blockIdx.x;
    // a short sequence has fewer than 8 x 16 segments: waves then share their 16 segments and split the tiles
    const int seg_waves = kScoreWaves / a.parts;
    c.part = c.wave / seg_waves;
    c.j0 = blockIdx.y * kScoreSegPerWg + 16 * (c.wave % seg_waves);
    c.h = blockIdx.z % a.hq; c.bb_ = blockIdx.z / a.hq;
    c.seg = c.j0 + (c.l32 >> 1); c.rep = c.l32 & 1;
    c.i_begin = c.chunk * kScoreChunk; c.i_end = min(a.n2, c.i_begin + kScoreChunk);
    c.ntile = (c.i_end - c.i_begin + ScoreTile::kTileBlocks - 1) / ScoreTile::kTileBlocks;
    c.qrow0 = ((long long)c.bb_ * a.hq + c.h) * a.n1;
    const int g = c.h / (a.hq / a.hkv);
    c.ksrc = (const uint16_t*)a.krep + ((long long)c.bb_ * a.hkv + g) * a.n2 * 2 * kHeadDim;
    c.vis = min(a.n2, (min(c.seg, a.n1 - 1) + 1) * a.r);
    c.vis_wg = min(a.n2, min(a.n1, (int)(blockIdx.y + 1) * kScoreSegPerWg) * a.r);
    c.vis_wave = min(a.n2, (min(c.j0, a.n1 - 1) + 1) * a.r);
    c.vis_wave_max = min(a.n2, min(a.n1, c.j0 + 16) * a.r);
    c.lds0 = lds0;
    const uint16_t* src = (const uint16_t*)a.qrep + ((c.qrow0 + min(c.seg, a.n1 - 1)) * 2 + c.rep) * kHeadDim + 8 * c.hh;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) c.qf[ks] = as_bf16x8(*(const uint4*)(src + 16 * ks));
}
// Piece p of the chunk, global -> LDS buffer p & 1: instruction x of wave w (X instructions each) writes the
// 1 KiB at 1024 * (X w + x) = rows 4 (X w + x) .. +3 of the piece (row = 2 * block + representative, 256 B); a
// lane's 16 bytes land at lane * 16 inside that KiB, so the XOR swizzle of the 16-byte chunks by the block
// index (which spreads the 32 row reads of a fragment over all banks) is applied to the global address.
// Blocks past the last one repeat it.
__device__ __forceinline__ void score_load_piece(const ScoreArgs& a, const ScoreCtx& c, int p) {
    const unsigned long long pv = (unsigned long long)c.ksrc;
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)pv);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(pv >> 32));
    const void* sbase = (const void*)(((unsigned long long)hi << 32) | lo);
    constexpr int kPerWave = kScorePiece / 2 / kScoreWaves;  // 1 KiB instructions per wave
    constexpr unsigned kPieceBytes = kScorePiece * 2 * kHeadDim * 2;
#pragma unroll
    for (int x = 0; x < kPerWave; ++x) {
        const int row = 4 * (kPerWave * c.wave + x) + (c.lane >> 4);
        const int blk = min(c.i_begin + p * kScorePiece + (row >> 1), a.n2 - 1);
        const int lc = (c.lane & 15) ^ ((row >> 1) & 15);
        const unsigned voff = (unsigned)(((blk * 2 + (row & 1)) * kHeadDim + lc * 8) * 2);
        const unsigned dst =
            __builtin_amdgcn_readfirstlane(c.lds0 + (p & 1) * kPieceBytes + 1024u * (kPerWave * c.wave + x));
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(voff), "s"(sbase)
                     : "memory");   // m0: reserved for the compiler, which sets it anew before each use of its own
    }
}
// every load of this wave has landed, every wave has arrived (and is done with the buffer that is filled next)
__device__ __forceinline__ void score_chunk_ready() {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
}
// z[b2][r] = K_rep(b2)[block 8*(r>>2) + 4*hh + (r&3) of the tile] . Q_rep[column]
__device__ __forceinline__ void score_tile(const ScoreCtx& c, int nt, f32x16 (&z)[2]) {   // tile nt of the chunk
    const unsigned base = c.lds0 + (nt & 3) * ScoreTile::kTileBytes + c.l32 * 512;
    const int sw = c.l32 & 15;
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2) {
#pragma unroll
        for (int r = 0; r < 16; ++r) z[b2][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 kf = as_bf16x8(*SCORE_LDS(const u32x4, base + b2 * 256 + (((2 * ks + c.hh) ^ sw) << 4)));
            z[b2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, c.qf[ks], z[b2], 0, 0, 0);
        }
    }
}
// statistics of chunk part cc (= chunk * parts + part), product b2, column col:
// stats[(((bh * nchunk * parts + cc) * 2 + b2) * 2 + which) * cols + col]
__device__ __forceinline__ long long stats_index(const ScoreArgs& a, const ScoreCtx& c, int cc, int b2, int which) {
    const long long cols = 2LL * a.n1_pad;
    return ((((long long)blockIdx.z * (a.nchunk * a.parts) + cc) * 2 + b2) * 2 + which) * cols + 2 * c.seg + c.rep;
}

__global__ __launch_bounds__(64 * kScoreWaves, 4) void score_stats_kernel(ScoreArgs a) {
    __shared__ __attribute__((aligned(1024))) unsigned char tiles[2 * kScorePiece * 2 * kHeadDim * 2];
    ScoreCtx c;
    score_setup(a, c, (unsigned)(uintptr_t)tiles);
    if (a.domain == 1 && c.i_begin >= c.vis_wg) return;     // uniform: no visible block for any segment here
    constexpr float kLog2e = 1.4426950408889634f;
    const float cs = a.scale * kLog2e;                      // logits in log2 units
    const int dom = a.domain == 0 ? a.n2 : c.vis;
    const int dom_wave = a.domain == 0 ? a.n2 : c.vis_wave; // blocks below it count for every column of the wave
    float m[2] = {-INFINITY, -INFINITY}, l[2] = {0.f, 0.f};
    score_load_piece(a, c, 0);
    for (int nt = 0; nt < c.ntile; ++nt) {
        if ((nt & 1) == 0) {                                // a new piece: wait for it, start the next one
            score_chunk_ready();
            if (nt + 2 < c.ntile) score_load_piece(a, c, (nt >> 1) + 1);
        }
        if ((nt & (a.parts - 1)) != c.part) continue;       // another wave's tile
        f32x16 z[2];
        score_tile(c, nt, z);
        const int i0 = c.i_begin + nt * ScoreTile::kTileBlocks + 4 * c.hh;
        if (cs > 0.f && c.i_begin + (nt + 1) * ScoreTile::kTileBlocks <= dom_wave) {
            // every block of the tile counts for every column of the wave: no masks, the scale folded into one fma
#pragma unroll
            for (int b2 = 0; b2 < 2; ++b2) {
                float mt = fmaxf(z[b2][0], z[b2][1]);
#pragma unroll
                for (int r = 2; r < 16; r += 2) mt = fmaxf(fmaxf(z[b2][r], z[b2][r + 1]), mt);
                mt = halves_max(mt) * cs;
                const float mn = fmaxf(m[b2], mt);
                float sum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(fmaf(z[b2][r], cs, -mn));
                l[b2] = l[b2] * __builtin_amdgcn_exp2f(m[b2] - mn) + sum;
                m[b2] = mn;
            }
            continue;
        }
#pragma unroll
        for (int b2 = 0; b2 < 2; ++b2) {
            float v[16];
            float mt = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                v[r] = (i0 + 8 * (r >> 2) + (r & 3) < dom) ? z[b2][r] * cs : -INFINITY;
                mt = fmaxf(mt, v[r]);
            }
            mt = halves_max(mt);
            const float mn = fmaxf(m[b2], mt);
            const float ms = (mn == -INFINITY) ? 0.f : mn;
            float sum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) sum += exp2f(v[r] - ms);
            l[b2] = l[b2] * exp2f(m[b2] - ms) + sum;        // per-half partial sums under a common max
            m[b2] = mn;
        }
    }
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2) {
        const float lt = halves_sum(l[b2]);
        if (c.hh == 0) {
            a.stats[stats_index(a, c, c.chunk * a.parts + c.part, b2, 0)] = m[b2];
            a.stats[stats_index(a, c, c.chunk * a.parts + c.part, b2, 1)] = lt;
        }
    }
}

__global__ __launch_bounds__(64 * kScoreWaves, 4) void score_write_kernel(ScoreArgs a) {
    __shared__ __attribute__((aligned(1024))) unsigned char tiles[2 * kScorePiece * 2 * kHeadDim * 2];
    ScoreCtx c;
    score_setup(a, c, (unsigned)(uintptr_t)tiles);
    const bool vec = (a.n2 & 3) == 0;                       // rows of scores are 16-byte aligned
    auto finish = [&](float sc, long long off) {            // fusion and the subnormal flush
        if (a.prev) sc = a.alpha * sc + (1.0f - a.alpha) * a.prev[off];
        if (fabsf(sc) < 1.17549435e-38f) sc = 0.f;
        return sc;
    };
    if (c.i_begin >= c.vis_wg) {                            // uniform: nothing of this chunk is visible
        const int width = c.i_end - c.i_begin;
        for (int x = threadIdx.x; x < kScoreSegPerWg * width; x += 64 * kScoreWaves) {
            const int j = blockIdx.y * kScoreSegPerWg + x / width;
            if (j >= a.n1) break;
            const long long off = (c.qrow0 + j) * a.n2 + c.i_begin + x % width;
            a.scores[off] = finish(0.f, off);
        }
        return;
    }
    constexpr float kLog2e = 1.4426950408889634f;
    const float cs = a.scale * kLog2e;
    const int dom = a.domain == 0 ? a.n2 : c.vis;
    score_load_piece(a, c, 0);                              // the merge below runs while the piece lands
    // merge the chunk statistics of the lane's column: the lane does the product b2 = hh, the same column's
    // lane in the other wave half does the other one (domain 1: chunks past the workgroup's last visible
    // block were never written)
    const int ncc = (a.domain == 0 ? a.nchunk : (c.vis_wg + kScoreChunk - 1) / kScoreChunk) * a.parts;
    float mx[2], inv[2];
    {
        float M = -INFINITY, L = 0.f;
        const long long step = stats_index(a, c, 1, 0, 0) - stats_index(a, c, 0, 0, 0);
        const float* sm_ = a.stats + stats_index(a, c, 0, c.hh, 0);
        const float* sl_ = a.stats + stats_index(a, c, 0, c.hh, 1);
#pragma unroll 4
        for (int cc = 0; cc < ncc; ++cc) {
            const float mc = sm_[cc * step], lc = sl_[cc * step];
            const float mn = fmaxf(M, mc);
            const float ms = (mn == -INFINITY) ? 0.f : mn;
            L = L * exp2f(M - ms) + lc * exp2f(mc - ms);
            M = mn;
        }
        const float own_m = (M == -INFINITY) ? 0.f : M;
        const float own_i = L > 0.f ? 1.0f / L : 0.f;
        const auto rm = __builtin_amdgcn_permlane32_swap(__float_as_uint(own_m), __float_as_uint(own_m), false, false);
        const auto ri = __builtin_amdgcn_permlane32_swap(__float_as_uint(own_i), __float_as_uint(own_i), false, false);
        const float oth_m = __uint_as_float(c.hh ? rm[0] : rm[1]);   // the value of lane l ^ 32
        const float oth_i = __uint_as_float(c.hh ? ri[0] : ri[1]);
        mx[0] = c.hh ? oth_m : own_m; mx[1] = c.hh ? own_m : oth_m;
        inv[0] = c.hh ? oth_i : own_i; inv[1] = c.hh ? own_i : oth_i;
    }
    // 2^(c z + fold) = 2^(c z - max) / sum / 2; usable when every column of the wave has a positive sum
    float fold[2];
    fold[0] = -mx[0] + __log2f(inv[0]) - 1.0f; fold[1] = -mx[1] + __log2f(inv[1]) - 1.0f;
    const bool l_pos = __builtin_amdgcn_ballot_w64(inv[0] > 0.f && inv[1] > 0.f) == ~0ull;
    for (int nt = 0; nt < c.ntile; ++nt) {
        if ((nt & 1) == 0) {                                // a new piece: wait for it, start the next one
            score_chunk_ready();
            if (nt + 2 < c.ntile) score_load_piece(a, c, (nt >> 1) + 1);
        }
        if ((nt & (a.parts - 1)) != c.part) continue;       // another wave's tile
        f32x16 z[2];
        const bool unseen = c.i_begin + nt * ScoreTile::kTileBlocks >= c.vis_wave_max;   // by every segment of the wave
        if (!unseen) score_tile(c, nt, z);
        const int i0 = c.i_begin + nt * ScoreTile::kTileBlocks + 4 * c.hh;
        // S1 = (max,max), S2 = (max,min), S3 = (min,max), S4 = (min,min): the lane has the products of its
        // query representative with K_max (b2 = 0) and K_min (b2 = 1), its neighbour those of the other one
        float sc[16];
        const int tile_end = c.i_begin + (nt + 1) * ScoreTile::kTileBlocks;
        if (unseen) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sc[r] = 0.f;
        } else if (cs > 0.f && tile_end <= c.vis_wave && l_pos) {
            // every block of the tile is visible to every segment of the wave: 1/sum and the 1/2 of the average
            // are folded into the exponent
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p0 = __builtin_amdgcn_exp2f(fmaf(z[0][r], cs, fold[0]));
                const float p1 = __builtin_amdgcn_exp2f(fmaf(z[1][r], cs, fold[1]));
                sc[r] = fmaxf(p0 + neighbour(p0), p1 + neighbour(p1));
            }
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = i0 + 8 * (r >> 2) + (r & 3);
                const bool in_dom = i < dom;
                const float p0 = in_dom ? exp2f(z[0][r] * cs - mx[0]) * inv[0] : 0.f;
                const float p1 = in_dom ? exp2f(z[1][r] * cs - mx[1]) * inv[1] : 0.f;
                const float t0 = p0 + neighbour(p0), t1 = p1 + neighbour(p1);
                sc[r] = (i < c.vis) ? fmaxf(t0, t1) * 0.5f : 0.f;
            }
        }
        // both lanes of a pair hold the segment's 16 scores: representative 0 stores blocks 0-7 and 16-23 of
        // the lane half's 16, representative 1 the rest, four consecutive blocks at a time
        if (c.seg < a.n1) {
#pragma unroll
            for (int g2 = 0; g2 < 2; ++g2) {
                const int g = 2 * g2 + c.rep;               // wave-varying but only two values: both compiled
                const int i = i0 + 8 * g;
                const long long off = (c.qrow0 + c.seg) * a.n2 + i;
                float w[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = c.rep ? sc[4 * (2 * g2 + 1) + e] : sc[4 * (2 * g2) + e];
                if (vec) {
                    if (i < a.n2) {
                        float4 o;
                        if (a.prev) {
                            const float4 pv = *(const float4*)(a.prev + off);
                            o.x = a.alpha * w[0] + (1.0f - a.alpha) * pv.x; o.y = a.alpha * w[1] + (1.0f - a.alpha) * pv.y;
                            o.z = a.alpha * w[2] + (1.0f - a.alpha) * pv.z; o.w = a.alpha * w[3] + (1.0f - a.alpha) * pv.w;
                        } else { o.x = w[0]; o.y = w[1]; o.z = w[2]; o.w = w[3]; }
                        if (fabsf(o.x) < 1.17549435e-38f) o.x = 0.f;
                        if (fabsf(o.y) < 1.17549435e-38f) o.y = 0.f;
                        if (fabsf(o.z) < 1.17549435e-38f) o.z = 0.f;
                        if (fabsf(o.w) < 1.17549435e-38f) o.w = 0.f;
                        *(float4*)(a.scores + off) = o;
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (i + e < a.n2) a.scores[off + e] = finish(w[e], off + e);
                }
            }
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

// waves of a score workgroup that share their segments: all eight take different segments unless the sequence
// has too few of them
static int score_parts(int n1) { return n1 <= 16 ? 8 : n1 <= 32 ? 4 : n1 <= 64 ? 2 : 1; }

size_t score_stats_bytes(const Shape& sh) {
    if (sh.dtype != 1) return 0;
    const size_t nchunk = (size_t)((sh.n2 + kScoreChunk - 1) / kScoreChunk) * score_parts(sh.n1);
    const size_t n1_pad = (size_t)((sh.n1 + kScoreSegPerWg - 1) / kScoreSegPerWg) * kScoreSegPerWg;
    return (size_t)sh.batch * sh.hq * nchunk * 2 * 2 * (2 * n1_pad) * sizeof(float);
}

hipError_t launch_score(const Shape& sh, const void* qrep, const void* krep, const float* prev, float* scores,
                        float* stats, hipStream_t st) {
    ScoreArgs a;
    a.qrep = qrep; a.krep = krep; a.prev = prev; a.scores = scores; a.stats = stats;
    a.hq = sh.hq; a.hkv = sh.hkv; a.n1 = sh.n1; a.n2 = sh.n2; a.r = sh.r; a.domain = sh.softmax_domain;
    a.scale = sh.score_scale; a.alpha = sh.alpha;
    a.nchunk = (sh.n2 + kScoreChunk - 1) / kScoreChunk;
    a.n1_pad = (sh.n1 + kScoreSegPerWg - 1) / kScoreSegPerWg * kScoreSegPerWg;
    a.parts = score_parts(sh.n1);
    if (sh.dtype == 1) {
        if ((long long)sh.batch * sh.hq > 65535) return hipErrorInvalidValue;
        dim3 grid_m(a.nchunk, a.n1_pad / kScoreSegPerWg, sh.batch * sh.hq);
        hipLaunchKernelGGL(score_stats_kernel, grid_m, dim3(64 * kScoreWaves), 0, st, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(score_write_kernel, grid_m, dim3(64 * kScoreWaves), 0, st, a);
        return hipGetLastError();
    }
    const size_t smem = (2 * kHeadDim + 4 + 4 * (size_t)sh.n2) * sizeof(float);
    dim3 grid(sh.n1, sh.hq, sh.batch);
    const void* fn = (const void*)score_valu_kernel;
    if (smem > 48 * 1024) {
        const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(score_valu_kernel, grid, dim3(256), smem, st, a);
    return hipGetLastError();
}

}  // namespace cp
