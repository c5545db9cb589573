// bf16 MFMA flash attention for gfx950: Algorithm 2's per-segment loop over a block list
// (block-sparse, gathered K/V tiles) and Eq. 2 dense causal attention (no list) from one kernel body.
//
// Workgroup = 4 wave64 = 256 query rows of one segment (sparse) or of the sequence (dense); a wave owns
// 64 rows as two 32-row MFMA sub-tiles.  The key loop walks 64-token tiles of the "virtual" token list
// (the listed blocks laid end to end).  Per tile and wave:
//
//   S^T[key][q] = K_tile . Q^T      32x32x16 bf16 MFMA, A = K rows from LDS (ds_read_b128), B = Q
//                                   fragments that stay in registers for the whole kernel.
//   online softmax                  S^T puts one query per lane column, so row max / row sum are
//                                   in-lane reductions plus one v_permlane32_swap between wave halves.
//   O^T[ch][q] += V^T . P^T         A = V read from LDS through the transposing ds_read_b64_tr_b16,
//                                   B = P^T taken straight from the S^T accumulators (the key order
//                                   inside a 16-key MFMA step is chosen so no shuffle is needed).
//
// The two sub-tiles are software-pipelined against each other so that the softmax VALU work of one
// overlaps the MFMA work of the other:  A: QK(0) | B: QK(1) + softmax(0) | C: PV(0) + softmax(1) | D: PV(1).
//
// K/V tiles go global -> LDS directly (global_load_lds_dwordx4, no register staging) into a ring of three
// buffers: tile t+2 is in flight while tile t is consumed, one barrier per tile.  The block list of the
// segment is copied to LDS once, so the key loop itself issues no other global loads and the only
// vmcnt waits in it are the hand-placed ones that pace the ring.  Rows are 256 B with the 16-byte chunks XOR-swizzled by the row index instead
// of padded (the DMA writes 1 KiB contiguous per wave instruction), which keeps both the 16 B row
// reads of K and the transposed 8 B reads of V free of bank conflicts.
#include "kernels.h"

#include <type_traits>

namespace cp {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 v4bf16_lds;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
#define LDS_PTR(T, off) ((__attribute__((address_space(3))) T*)(uintptr_t)(off))

constexpr int TQ = 256;               // query rows per workgroup
constexpr int TK = 64;                // key tokens per tile
constexpr int NBUF = 3;               // K/V tile ring in LDS
constexpr int kTileBytes = TK * 256;  // one K or V tile in LDS
constexpr int kTokOff = 0;                         // [NBUF][TK] token position of every tile row
constexpr int kVOff = 1024;                        // [NBUF] V tiles
constexpr int kKOff = kVOff + NBUF * kTileBytes;   // [NBUF] K tiles
constexpr int kListOff = kKOff + NBUF * kTileBytes;   // the segment's block list (sparse only)
constexpr int kMaxListLds = 14336;                 // entries; longer lists are rejected by the API

struct ArgsB {
    const uint16_t* q; const uint16_t* k; const uint16_t* v; const int32_t* idx; const int32_t* cnt;
    uint16_t* out; float* lse;
    int batch, hq, hkv, n, s, b, n1, list_len, qtiles;
    float scale_log2e, scale;
    long long qs0, qs1, qs2, ks0, ks1, ks2, os0, os1, os2;
};

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) {
    union { uint4 u; bf16x8 b; } c; c.u = v; return c.b;
}
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) {
    union { u32x4 u; bf16x8 b; } c; c.u = v; return c.b;
}
// Keep a value live (and computed) at this point of the program: stops the compiler from sinking the
// producer below a later branch or from leaving a load pending into the loop.
__device__ __forceinline__ void pin(const bf16x8& v) { asm volatile("" ::"v"(v)); }
__device__ __forceinline__ void pin_acc(const bf16x8& v) { asm volatile("" ::"a"(v)); }

// 16 bytes per lane from global memory straight into LDS at (lds_base + lane * 16); lds_base is
// wave-uniform.  Issued through inline asm so the compiler does not serialise later LDS reads of the
// OTHER buffer behind it; the matching s_waitcnt vmcnt(0) is issued by hand before the tile barrier.
__device__ __forceinline__ void dma16(const void* sbase, unsigned voff, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(sbase)
                 : "memory");
}

__device__ __forceinline__ const uint16_t* uniform_ptr(const uint16_t* p) {   // into SGPRs
    const unsigned long long v = (unsigned long long)p;
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return (const uint16_t*)(((unsigned long long)hi << 32) | lo);
}

__device__ __forceinline__ float half_max(float x) {      // max over lanes l and l^32
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <bool DENSE>
__global__ __launch_bounds__(256, 1) void attn_bf16_kernel(ArgsB a) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hh = lane >> 5;

    // ---- which (batch, head, segment, query tile) this workgroup owns --------------------------
    int bb, h, j = 0, qt;
    const int G = a.hq / a.hkv;
    if (DENSE) {
        // heaviest query tiles first; consecutive workgroups walk the KV heads so that the query
        // heads sharing one KV head land on the same XCD (workgroup id mod 8) at the same time.
        const int bh_count = a.batch * a.hq, bkv = a.batch * a.hkv;
        const int x = blockIdx.x % bh_count;
        qt = a.qtiles - 1 - blockIdx.x / bh_count;
        const int bkvh = x % bkv, gq = x / bkv;
        bb = bkvh / a.hkv; h = (bkvh % a.hkv) * G + gq;
    } else {
        // (batch, KV head) groups run one after another; inside a group every XCD gets a contiguous
        // range of segments, with the query tiles and query heads of one segment adjacent.
        const int per_group = G * a.n1 * a.qtiles;
        const int grp = blockIdx.x / per_group;
        int lid = blockIdx.x % per_group;
        if ((per_group & 7) == 0) lid = (lid & 7) * (per_group >> 3) + (lid >> 3);
        qt = lid % a.qtiles; lid /= a.qtiles;
        const int gq = lid % G; j = lid / G;
        bb = grp / a.hkv; h = (grp % a.hkv) * G + gq;
    }
    const int g = h / G;
    const int q_lo = DENSE ? qt * TQ : j * a.s + qt * TQ;
    const int q_end = DENSE ? a.n : min(a.n, (j + 1) * a.s);
    if (q_lo >= q_end) return;                                   // uniform: tile past a short segment
    const int q_last = min(q_end, q_lo + TQ) - 1;
    const int wq_lo = q_lo + 64 * wave;
    const int wq_last = min(q_end, wq_lo + 64) - 1;              // < wq_lo when the wave has no rows

    const uint16_t* qp = a.q + bb * a.qs0 + h * a.qs1;
    const uint16_t* kp = uniform_ptr(a.k + bb * a.ks0 + g * a.ks1);
    const uint16_t* vp = uniform_ptr(a.v + bb * a.ks0 + g * a.ks1);

    // ---- Q fragments (B operand: column = query l32, 8 channels at 16*ks + 8*hh) ---------------
    int qpos[2];
    bf16x8 qf[2][8];
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
        qpos[t2] = wq_lo + 32 * t2 + l32;
        const bool ok = qpos[t2] < q_end;
        const uint16_t* src = qp + (long long)(ok ? qpos[t2] : q_lo) * a.qs2 + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            uint4 v = *(const uint4*)(src + 16 * ks);
            if (!ok) v = make_uint4(0, 0, 0, 0);
            qf[t2][ks] = as_bf16x8(v);
        }
    }

#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) pin_acc(qf[t2][ks]);     // Q has arrived before the key loop starts

    // ---- the virtual token list --------------------------------------------------------------
    int count = 0;
    if (!DENSE) {
        const long long lrow = ((long long)bb * a.hq + h) * a.n1 + j;
        const int32_t* list = a.idx + lrow * a.list_len;
        count = a.cnt[lrow];
        for (int x = tid; x < count; x += 256) *LDS_PTR(int, lds0 + kListOff + x * 4) = list[x];
        __syncthreads();
    }
    // positions 0 .. total-1 of the listed blocks laid end to end (host checks count * b < 2^31)
    const unsigned total = DENSE ? (unsigned)q_last + 1u : (unsigned)count * (unsigned)a.b;
    const unsigned ub = (unsigned)a.b;
    int ntiles = (int)((total + TK - 1) / TK);
    if (!DENSE) {   // drop trailing tiles that start after the last query row (lists are ascending)
        while (ntiles > 0) {
            const unsigned p = (unsigned)(ntiles - 1) * TK;
            const unsigned e = p / ub;
            const int tok = *LDS_PTR(const int, lds0 + kListOff + e * 4) * a.b + (int)(p - e * ub);
            if (tok <= q_last) break;
            --ntiles;
        }
    }

    // ---- tile loader: wave w, instruction i fills rows 16*i + 4*w .. +3; lane -> (row, 16 B chunk) --
    const int lrow = 4 * wave + (lane >> 4);                 // row within a 16-row group (= row & 15)
    const int pch = lane & 15;                               // physical chunk the lane's 16 bytes land in
    const int kch = pch ^ lrow;                              // K: chunk swizzle = row & 15
    const int vch = pch ^ (2 * (lrow & 7));                  // V: chunk swizzle = 2 * (row & 7)
    // The list is walked incrementally: for each of the lane's 4 rows, (e, off) = (entry, offset inside
    // the block) of the next tile to fetch; one tile further on they advance by (64 / b, 64 % b).
    const unsigned step_e = TK / ub, step_off = TK % ub;
    unsigned we[4], woff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { we[i] = (16 * i + lrow) / ub; woff[i] = (16 * i + lrow) % ub; }
    int ent[4], eoff[4];       // block index (-1: past the list) and in-block offset of the lane's rows, fetched tile
    int dense_tile = 0;        // dense: the tile the next tile_offsets() call describes
    auto fetch_entries = [&]() {                             // call once per tile, in tile order
        if (DENSE) return;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int v = *LDS_PTR(const int, lds0 + kListOff + min(we[i], (unsigned)max(count - 1, 0)) * 4);
            ent[i] = (we[i] < (unsigned)count) ? v : -1;
            eoff[i] = (int)woff[i];
            we[i] += step_e; woff[i] += step_off;
            if (woff[i] >= ub) { woff[i] -= ub; we[i] += 1; }
        }
    };
    // byte offsets (from kp / vp) of the lane's 4 K and 4 V chunks of the next tile, and the rows' tokens
    const unsigned tok_bytes = (unsigned)a.ks2 * 2u;         // host checks n * tok_bytes < 2^32, both < 2^24
    unsigned koff[4], voff[4]; int tokv[4];
    auto tile_offsets = [&]() {                              // call once per tile, in tile order, before fetch_entries
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int tok; bool valid;
            if (DENSE) { tok = dense_tile * TK + 16 * i + lrow; valid = (unsigned)tok < total; }
            else { tok = ent[i] * a.b + eoff[i]; valid = ent[i] >= 0 && tok < a.n; }
            const unsigned base = __umul24(valid ? (unsigned)tok : 0u, tok_bytes);  // invalid rows read token 0, masked later
            koff[i] = base + kch * 16;
            voff[i] = base + vch * 16;
            tokv[i] = valid ? tok : 0x7fffffff;
        }
        ++dense_tile;
    };
    auto dma_k = [&](int i, int buf) { dma16(kp, koff[i], lds0 + kKOff + buf * kTileBytes + (16 * i + 4 * wave) * 256); };
    auto dma_v = [&](int i, int buf) { dma16(vp, voff[i], lds0 + kVOff + buf * kTileBytes + (16 * i + 4 * wave) * 256); };
    auto put_tok = [&](int buf) {
        if (pch == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) *LDS_PTR(int, lds0 + kTokOff + buf * TK * 4 + (16 * i + lrow) * 4) = tokv[i];
        }
    };

    // ---- per-lane LDS read addresses (bytes, buffer 0) -----------------------------------------
    // K: row 32*kt + l32, logical chunk 2*ks + hh  ->  physical chunk (2*ks) ^ ((l32 & 15) ^ hh)
    unsigned k_addr[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
        k_addr[ks] = lds0 + kKOff + l32 * 256 + (((unsigned)ks << 5) ^ (unsigned)(((l32 & 15) ^ hh) << 4));
    // V (transposed read, 16-lane groups): lane supplies row 4*hh + (i16 >> 2) (+16*t4, +8), 8-byte unit
    // 2*(32*dt + 16*((lane>>4)&1))/8 + (i16 & 3)
    const int i16 = lane & 15;
    const int v_m = 4 * hh + (i16 >> 2);
    const unsigned v_z = (unsigned)((2 * ((lane >> 4) & 1) + ((i16 & 3) >> 1)) ^ (2 * v_m));
    unsigned v_addr[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
        v_addr[dt] = lds0 + kVOff + v_m * 256 + ((((unsigned)dt << 2) ^ v_z) << 4) + (i16 & 1) * 8;

    f32x16 o[4][2];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[dt][t2][r] = 0.f;
    float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};
    const float c = a.scale_log2e;

    auto mask = [&](f32x16 (&s)[2], int t2, unsigned tok_base) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int gg = 0; gg < 4; ++gg) {
                const i32x4 t4 = *LDS_PTR(const i32x4, tok_base + (32 * kt + 8 * gg + 4 * hh) * 4);
                const int tv[4] = {t4[0], t4[1], t4[2], t4[3]};
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (tv[i] > qpos[t2]) s[kt][4 * gg + i] = -INFINITY;
            }
    };
    auto rescale = [&](int t2, float alpha) {
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[dt][t2][r] *= alpha;
        }
    };
    // pieces of the online softmax of one 64-key x 32-query sub-tile, issued between MFMAs
    auto row_max16 = [&](const f32x16& v) {
        float mx = fmaxf(v[0], v[1]);
#pragma unroll
        for (int r = 2; r < 16; ++r) mx = fmaxf(mx, v[r]);
        return mx;
    };
    // new running max -> rescale factor alpha and the scaled offset ms; updates m_run
    auto new_max = [&](int t2, float mx, float& alpha, float& ms) {
        mx = half_max(mx);
        const float m_new = fmaxf(m_run[t2], mx);
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        alpha = __builtin_amdgcn_exp2f((m_run[t2] - m_safe) * c);
        ms = m_safe * c;
        m_run[t2] = m_new;
    };

    bf16x8 kf[2][8];                                         // K fragments of the tile about to be consumed
    auto read_k = [&](int buf) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
                kf[kt][ks] = as_bf16x8(*LDS_PTR(const u32x4, k_addr[ks] + buf * kTileBytes + kt * 32 * 256));
    };

    // One tile.  On entry: tile t sits in ring slot BUF with its K fragments already in kf, tile t+1 is
    // in flight into slot BUF+1, the DMA offsets of tile t+2 are in koff/voff (its row tokens already in
    // LDS) and the list entries of tile t+3 are in ent/eoff.
    auto body = [&](auto bufc, int t) {
        constexpr int BUF = decltype(bufc)::value;
        constexpr int BUF1 = (BUF + 1) % NBUF, BUF2 = (BUF + 2) % NBUF;
        const unsigned tok_base = lds0 + kTokOff + BUF * TK * 4;
        const int first_tok = *LDS_PTR(const int, tok_base);
        const int last_tok = *LDS_PTR(const int, tok_base + (TK - 1) * 4);
        const bool active = first_tok <= wq_last;                    // wave-uniform
        f32x16 s1[2];
        bf16x8 vf[4][4], pf1[4];
        if (active) {
            // ---- phase A: S^T(0) = K Q0^T, the loads of tile t+2 ride along ------------------
            f32x16 s0[2];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) { s0[kt][r] = 0.f; s1[kt][r] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
                    s0[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kt][ks], qf[0][ks], s0[kt], 0, 0, 0);
                if (ks < 4) dma_k(ks, BUF2); else dma_v(ks - 4, BUF2);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (last_tok > wq_lo) mask(s0, 0, tok_base);

            auto read_v = [&](int t4) {
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) {
                    const unsigned ad = v_addr[dt] + BUF * kTileBytes + t4 * 16 * 256;
                    const v4bf16_lds lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(v4bf16_lds, ad));
                    const v4bf16_lds hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(v4bf16_lds, ad + 8 * 256));
#pragma unroll
                    for (int e = 0; e < 4; ++e) { vf[t4][dt][e] = lo[e]; vf[t4][dt][4 + e] = hi[e]; }
                }
            };
            // exp of values [lo, hi) of a sub-tile (value v lives in s[v >> 4][v & 15]), partial row sums
            auto exp_range = [&](f32x16 (&s)[2], int lo, int hi, float ms, float& rs0, float& rs1) {
#pragma unroll
                for (int v = lo; v < hi; ++v) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(s[v >> 4][v & 15], c, -ms));
                    s[v >> 4][v & 15] = p;
                    if (v & 1) rs1 += p; else rs0 += p;
                }
            };
            auto to_pf = [&](const f32x16 (&s)[2], bf16x8 (&pf)[4]) {
#pragma unroll
                for (int t4 = 0; t4 < 4; ++t4)
#pragma unroll
                    for (int e = 0; e < 8; ++e) pf[t4][e] = (__bf16)s[t4 >> 1][8 * (t4 & 1) + e];
            };
            constexpr int kLo[6] = {0, 6, 11, 16, 22, 27}, kHi[6] = {6, 11, 16, 22, 27, 32};

            // ---- phase B: S^T(1) = K Q1^T (two MFMAs per step)  ||  softmax(0) ------------------
            float alpha0, alpha1, ms, mxa, rs0 = 0.f, rs1 = 0.f;
            bf16x8 pf0[4];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
                    s1[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kt][ks], qf[1][ks], s1[kt], 0, 0, 0);
                if (ks == 0) mxa = row_max16(s0[0]);
                else if (ks == 1) new_max(0, fmaxf(mxa, row_max16(s0[1])), alpha0, ms);
                else exp_range(s0, kLo[ks - 2], kHi[ks - 2], ms, rs0, rs1);
                if (ks == 6) read_v(0);
                if (ks == 7) read_v(1);
                __builtin_amdgcn_sched_barrier(0);
            }
            l_run[0] = l_run[0] * alpha0 + (rs0 + rs1);      // per-half partial sums, merged at the end
            to_pf(s0, pf0);
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) pin(pf0[t4]);
            if (last_tok > wq_lo + 32) mask(s1, 1, tok_base);
            rescale(0, alpha0);
            // ---- phase C: O^T(0) += V^T P0^T (two MFMAs per step)  ||  softmax(1) -------------
            rs0 = 0.f; rs1 = 0.f;
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                if (x == 0) read_v(2);
                if (x == 1) read_v(3);
#pragma unroll
                for (int y = 0; y < 2; ++y) {
                    const int t4 = x >> 1, dt = 2 * (x & 1) + y;
                    o[dt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t4][dt], pf0[t4], o[dt][0], 0, 0, 0);
                }
                if (x == 0) mxa = row_max16(s1[0]);
                else if (x == 1) new_max(1, fmaxf(mxa, row_max16(s1[1])), alpha1, ms);
                else exp_range(s1, kLo[x - 2], kHi[x - 2], ms, rs0, rs1);
                __builtin_amdgcn_sched_barrier(0);
            }
            l_run[1] = l_run[1] * alpha1 + (rs0 + rs1);
            to_pf(s1, pf1);
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) pin(pf1[t4]);
            rescale(1, alpha1);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) { dma_k(i, BUF2); dma_v(i, BUF2); }
        }
        // tile t+1 has landed (this wave's rows): at most the 8 loads of tile t+2 may still be in flight.
        // After the barrier nobody reads slot BUF any more and everybody's rows of tile t+1 are in LDS.
        asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        __syncthreads();
        if (active) {
            // ---- phase D: O^T(1) += V^T P1^T  ||  K fragments of tile t+1, loader state of tile t+3 ----
            read_k(BUF1);
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
                    o[dt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t4][dt], pf1[t4], o[dt][1], 0, 0, 0);
                if (t4 == 0) { tile_offsets(); put_tok(BUF); }
                if (t4 == 1) fetch_entries();
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            tile_offsets(); put_tok(BUF); fetch_entries();
        }
    };

    // ---- prologue: tiles 0 and 1 in flight, loader state primed for tile 2 and entries of tile 3 ----
    if (ntiles > 0) {
        fetch_entries();
        tile_offsets(); fetch_entries(); put_tok(0);
#pragma unroll
        for (int i = 0; i < 4; ++i) { dma_k(i, 0); dma_v(i, 0); }
        tile_offsets(); fetch_entries(); put_tok(1);
#pragma unroll
        for (int i = 0; i < 4; ++i) { dma_k(i, 1); dma_v(i, 1); }
        tile_offsets(); fetch_entries(); put_tok(2);
        asm volatile("s_waitcnt vmcnt(8)" ::: "memory");             // tile 0 has landed
    }
    __syncthreads();
    if (ntiles > 0) read_k(0);
    for (int t = 0; t < ntiles; t += 3) {
        body(std::integral_constant<int, 0>{}, t);
        if (t + 1 < ntiles) body(std::integral_constant<int, 1>{}, t + 1);
        if (t + 2 < ntiles) body(std::integral_constant<int, 2>{}, t + 2);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                 // no DMA may outlive the workgroup

    // ---- epilogue: O^T[ch][q] / l  ->  out[q][ch] ------------------------------------------------
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
        const float l_tot = half_sum(l_run[t2]);
        const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
        if (qpos[t2] < q_end) {
            uint16_t* op = a.out + bb * a.os0 + h * a.os1 + (long long)qpos[t2] * a.os2;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int gg = 0; gg < 4; ++gg) {
                    bf16x4 w;
#pragma unroll
                    for (int i = 0; i < 4; ++i) w[i] = (__bf16)(o[dt][t2][4 * gg + i] * inv);
                    *(bf16x4*)(op + 32 * dt + 8 * gg + 4 * hh) = w;
                }
            if (a.lse && hh == 0)
                a.lse[((long long)bb * a.hq + h) * a.n + qpos[t2]] =
                    l_tot > 0.f ? m_run[t2] * a.scale + __logf(l_tot) : -INFINITY;
        }
    }
}

}  // namespace

hipError_t launch_attn_bf16(const Shape& sh, const void* q, const void* k, const void* v, const int32_t* idx,
                            const int32_t* cnt, void* out, float* lse, hipStream_t st) {
    ArgsB a;
    a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v; a.idx = idx; a.cnt = cnt;
    a.out = (uint16_t*)out; a.lse = lse;
    a.batch = sh.batch; a.hq = sh.hq; a.hkv = sh.hkv; a.n = sh.n; a.s = sh.s; a.b = sh.b; a.n1 = sh.n1;
    a.list_len = sh.list_len;
    a.scale = sh.attn_scale;
    a.scale_log2e = sh.attn_scale * 1.4426950408889634f;
    a.qs0 = sh.qs[0]; a.qs1 = sh.qs[1]; a.qs2 = sh.qs[2];
    a.ks0 = sh.kvs[0]; a.ks1 = sh.kvs[1]; a.ks2 = sh.kvs[2];
    a.os0 = sh.os[0]; a.os1 = sh.os[1]; a.os2 = sh.os[2];
    hipError_t e;
    if (idx) {
        a.qtiles = (sh.s + TQ - 1) / TQ;
        const long long grid = (long long)sh.batch * sh.hq * sh.n1 * a.qtiles;
        if (sh.list_len > kMaxListLds) return hipErrorInvalidValue;
        const int smem = kListOff + ((sh.list_len * 4 + 1023) & ~1023);
        e = hipFuncSetAttribute((const void*)attn_bf16_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(attn_bf16_kernel<false>, dim3((unsigned)grid), dim3(256), smem, st, a);
    } else {
        a.qtiles = (sh.n + TQ - 1) / TQ;
        const long long grid = (long long)sh.batch * sh.hq * a.qtiles;
        e = hipFuncSetAttribute((const void*)attn_bf16_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                kListOff);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(attn_bf16_kernel<true>, dim3((unsigned)grid), dim3(256), kListOff, st, a);
    }
    return hipGetLastError();
}

}  // namespace cp
