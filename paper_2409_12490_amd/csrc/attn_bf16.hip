// bf16 MFMA flash attention for gfx950: Algorithm 2's per-segment loop over a block list
// (block-sparse, gathered K/V tiles) and Eq. 2 dense causal attention (no list) from one kernel body.
//
// Workgroup = 8 wave64 = 256 query rows of one segment (sparse) or of the sequence (dense); a wave owns
// 32 rows (one MFMA tile).  The key loop walks 64-token tiles of the "virtual" token list (the listed
// blocks laid end to end).  Per tile and wave:
//
//   QK   S^T[key][q] = K_tile . Q^T   32x32x16 bf16 MFMA, A = K rows from LDS (ds_read_b128), B = Q
//                                     fragments that stay in registers for the whole kernel.
//   SM   online softmax               S^T puts one query per lane column, so row max / row sum are
//                                     in-lane reductions plus one v_permlane32_swap between wave halves.
//   PV   O^T[ch][q] += V^T . P^T      A = V read from LDS through the transposing ds_read_b64_tr_b16,
//                                     B = P^T taken straight from the S^T accumulators (the key order
//                                     inside a 16-key MFMA step is chosen so no shuffle is needed).
//
// One wave cannot overlap its own MFMA and VALU work to any useful degree on this hardware, two waves
// on one SIMD can.  So every SIMD holds two waves (w and w+4).  A wave alternates between a matrix phase
// MM(t) = PV(t-1) interleaved with QK(t) (32 independent-enough MFMAs that keep the matrix pipe full) and the
// softmax phase SM(t); the two waves of a SIMD run half a period apart:
//     waves 0-3:  MM(t)  SM(t)                   waves 4-7:  SM(t)  MM(t+1)
// which puts the softmax VALU work of one wave under the MFMA work of the other.
//
// K/V tiles go global -> LDS directly (global_load_lds_dwordx4, no register staging) into rings of four
// slots each: K of tile t+3 and V of tile t+2 are issued while tile t is consumed (K of tile t+1 and V of
// tile t-1 are still being read then), one barrier per tile.  Rows are 256 B with the 16-byte chunks XOR-swizzled by the row index instead of
// padded (the DMA writes 1 KiB contiguous per wave instruction), which keeps both the 16 B row reads of K
// and the transposed 8 B reads of V free of bank conflicts.  The block list of the segment is copied to
// LDS once, so the key loop itself issues no other global loads and the only vmcnt waits in it are the
// hand-placed ones that pace the ring.
#include "kernels.h"

namespace cp {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 v4bf16_lds;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(2))) int i32x2;
#define LDS_PTR(T, off) ((__attribute__((address_space(3))) T*)(uintptr_t)(off))

constexpr int TQ = 256;               // query rows per workgroup
constexpr int WQ = 32;                // query rows per wave
constexpr int TK = 64;                // key tokens per tile
constexpr int NBUF = 4;               // K/V tile ring in LDS
constexpr int kTileBytes = TK * 256;  // one K or V tile in LDS
constexpr int kTokOff = 0;                            // [NBUF][TK] token position of every tile row
constexpr int kVOff = 1024;                           // [NBUF] V tiles
constexpr int kKOff = kVOff + NBUF * kTileBytes;      // [NBUF] K tiles
constexpr int kListOff = kKOff + NBUF * kTileBytes;   // the segment's block list (sparse only)
constexpr float kLazyLog2 = 8.0f;        // see the softmax phase: how far a row's max may outgrow its reference point
constexpr int kOutPitch = 272;                        // epilogue staging: one output row + 16 B, in bytes
static_assert(kListOff + kMaxListBf16 * 4 <= 160 * 1024, "LDS budget");
static_assert(8 * WQ * kOutPitch <= 2 * NBUF * kTileBytes, "epilogue staging reuses the tile rings");

struct ArgsB {
    const uint16_t* q; const uint16_t* k; const uint16_t* v; const int32_t* idx; const int32_t* cnt;
    uint16_t* out; float* lse;
    int batch, hq, hkv, n, s, b, n1, list_len, qtiles;
    int shared_lists;                     // lists are per (batch, KV head, segment) instead of per query head
    float scale_log2e, scale;
    long long qs0, qs1, qs2, ks0, ks1, ks2, os0, os1, os2;
};

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) {
    union { uint4 u; bf16x8 b; } c; c.u = v; return c.b;
}
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) {
    union { u32x4 u; bf16x8 b; } c; c.u = v; return c.b;
}
// Keep a value computed at this point of the program (stops a load from staying pending into the loop).
__device__ __forceinline__ void pin(const bf16x8& v) { asm volatile("" ::"v"(v)); }

// 16 bytes per lane from global memory (uniform base + per-lane byte offset) straight into LDS at
// (lds_base + lane * 16); lds_base is wave-uniform.  Issued through inline asm so the compiler does not
// serialise later LDS reads of OTHER ring slots behind it; the matching s_waitcnt vmcnt is placed by hand
// before the tile barrier.  m0 is written here and not named as a clobber: it is a reserved register for the
// compiler, which keeps no value in it across statements and sets it anew before each use of its own (naming it
// only draws "clobber list contains reserved registers").
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

// MODE 0: sparse, any block size (row tokens of every tile kept in LDS); MODE 1: sparse, block size a
// multiple of 64 (every tile is 64 consecutive tokens, described by its first token alone); MODE 2: dense;
// MODE 3: sparse, block size a multiple of 32 but not of 64 (the paper's own setting is 32): a tile is two runs
// of 32 consecutive tokens, described by their two first tokens.
constexpr int kFragLook = 3;               // depth of the LDS fragment ring, see the matrix phase
template <int MODE, int KLOOK = kFragLook>
__global__ __launch_bounds__(512, 1) void attn_bf16_kernel(ArgsB a) {
    constexpr bool DENSE = MODE == 2, FAST = MODE != 0, HALF = MODE == 3;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hh = lane >> 5;
    const bool rotated = wave >= 4;                              // shares its SIMD with wave - 4

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
        // (batch, KV head) groups run one after another.  Workgroups reach the compute units round-robin and in
        // order: workgroup x + 256 follows workgroup x on the same unit and starts only after every workgroup
        // before it has started, so a round of 256 workgroups lasts as long as its slowest member.  The first
        // query tile of a segment sees fewer keys than the last (the plain order, both tiles in every round, left
        // the units with the short tiles idle 6 us per item; measured with per-wave time stamps), so a round
        // takes 256 (query head, segment) pairs at ONE query tile and the next round the same pairs at the next
        // tile.  Inside a round every XCD (workgroup id mod 8) gets 32 consecutive pairs: the query heads of a
        // few neighbouring segments.
        constexpr int kRound = 256;
        const int pairs = G * a.n1;
        const int per_group = pairs * a.qtiles;
        const int grp = blockIdx.x / per_group;
        const int x = blockIdx.x % per_group;
        const int full = pairs / kRound * kRound;                // pairs that fill whole rounds
        int u;
        if (x < full * a.qtiles) {
            const int y = x % (kRound * a.qtiles), pos = y % kRound;
            qt = y / kRound;
            u = x / (kRound * a.qtiles) * kRound + (pos & 7) * (kRound / 8) + (pos >> 3);
        } else {
            const int rest = pairs - full, y = x - full * a.qtiles;
            qt = y / rest;
            u = full + y % rest;
        }
        const int gq = u % G; j = u / G;
        bb = grp / a.hkv; h = (grp % a.hkv) * G + gq;
    }
    const int g = h / G;
    const int q_lo = DENSE ? qt * TQ : j * a.s + qt * TQ;
    const int q_end = DENSE ? a.n : min(a.n, (j + 1) * a.s);
    if (q_lo >= q_end) return;                                   // uniform: tile past a short segment
    const int q_last = min(q_end, q_lo + TQ) - 1;
    const int wq_lo = q_lo + WQ * wave;
    const int wq_last = min(q_end, wq_lo + WQ) - 1;              // < wq_lo when the wave has no rows

    const uint16_t* qp = a.q + bb * a.qs0 + h * a.qs1;
    const uint16_t* kp = uniform_ptr(a.k + bb * a.ks0 + g * a.ks1);
    const uint16_t* vp = uniform_ptr(a.v + bb * a.ks0 + g * a.ks1);

    // ---- the virtual token list --------------------------------------------------------------
    // Its loads are issued before those of Q (the scheduling barrier keeps the compiler from hoisting Q's loads
    // above them): loads return in order, the list row comes from L2 / Infinity Cache (the selection has just
    // written it) and the first K/V tiles cannot be asked for before it is here, while Q comes from HBM and is
    // not needed before those tiles have landed.
    int count = 0, list_first = -1;
    const int32_t* list = nullptr;
    if (!DENSE) {
        const long long lrow = a.shared_lists ? ((long long)bb * a.hkv + g) * a.n1 + j : ((long long)bb * a.hq + h) * a.n1 + j;
        list = a.idx + lrow * a.list_len;
        // the whole row (its pitch is list_len) is copied, so that its loads do not wait for the count
        if (tid < a.list_len) list_first = list[tid];
        count = min(max(a.cnt[lrow], 0), a.list_len);             // a bad count must not run past the list's LDS region
        __builtin_amdgcn_sched_barrier(0);
    }
    // ---- Q fragments (B operand: column = query l32, 8 channels at 16*ks + 8*hh) ---------------
    const int qpos = wq_lo + l32;
    bf16x8 qf[8];
    {
        const bool ok = qpos < q_end;
        const uint16_t* src = qp + (long long)(ok ? qpos : q_lo) * a.qs2 + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            uint4 v = *(const uint4*)(src + 16 * ks);
            if (!ok) v = make_uint4(0, 0, 0, 0);
            qf[ks] = as_bf16x8(v);
        }
    }

    if (!DENSE) {
        if (tid < a.list_len) *LDS_PTR(int, lds0 + kListOff + tid * 4) = list_first;
        for (int x = tid + 512; x < a.list_len; x += 512) *LDS_PTR(int, lds0 + kListOff + x * 4) = list[x];
    }
    __syncthreads();
    // positions 0 .. total-1 of the listed blocks laid end to end (host checks count * b < 2^31)
    const unsigned total = DENSE ? (unsigned)q_last + 1u : (unsigned)count * (unsigned)a.b;
    const unsigned ub = (unsigned)a.b;
    int ntiles = (int)((total + TK - 1) / TK);
    // MODE 3: the first tokens of the two halves of every tile, worked out once by all threads and kept in LDS
    // behind the list (8 bytes per tile), so that the key loop reads a tile's description instead of walking the list
    const unsigned tab0 = lds0 + kListOff + (((unsigned)a.list_len * 4u + 1023u) & ~1023u);
    if (HALF) {
        for (int x = tid; x < ntiles; x += 512) {
            const unsigned p0 = (unsigned)x * TK, e0 = p0 / ub, p1 = p0 + 32, e1 = p1 / ub;
            const int lo = *LDS_PTR(const int, lds0 + kListOff + e0 * 4) * a.b + (int)(p0 - e0 * ub);
            const int hi = e1 < (unsigned)count ? *LDS_PTR(const int, lds0 + kListOff + e1 * 4) * a.b + (int)(p1 - e1 * ub) : -1;
            i32x2 d; d[0] = lo; d[1] = hi;
            *LDS_PTR(i32x2, tab0 + x * 8) = d;
        }
        __syncthreads();
    }
    if (!DENSE) {   // drop trailing tiles that start after the last query row (lists are ascending)
        while (ntiles > 0) {
            int tok;
            if (HALF) tok = *LDS_PTR(const int, tab0 + (ntiles - 1) * 8);
            else {
                const unsigned p = (unsigned)(ntiles - 1) * TK;
                const unsigned e = p / ub;
                tok = *LDS_PTR(const int, lds0 + kListOff + e * 4) * a.b + (int)(p - e * ub);
            }
            if (tok <= q_last) break;
            --ntiles;
        }
    }

    // ---- tile loader: wave w fills rows 4*w .. 4*w+3 and 32 + 4*w .. +3 of K and of V (4 instructions) ----
    const int r4 = lane >> 4;                                // row inside the wave's 4-row group
    const int pch = lane & 15;                               // physical chunk the lane's 16 bytes land in
    const int kch = pch ^ ((4 * wave + r4) & 15);            // K: logical chunk, swizzle = row & 15
    const int vch = pch ^ (4 * r4);                          // V: logical chunk, swizzle = 4 * (row & 3)
    const unsigned tok_bytes = (unsigned)a.ks2 * 2u;         // host checks n * tok_bytes < 2^32, both < 2^24
    // byte offsets (from kp / vp) of the lane's chunks: koff/voff = the tile described last; V is issued one
    // step later than K, so its offsets wait in voff_issue.  Both wave roles issue their loads right after their
    // matrix phase.
    unsigned koff[2], voff[2], voff_issue[2];
    auto issue_k = [&](int slot) {
#pragma unroll
        for (int i = 0; i < 2; ++i) dma16(kp, koff[i], lds0 + kKOff + slot * kTileBytes + (32 * i + 4 * wave) * 256);
    };
    auto issue_v = [&](int slot, bool first) {               // first: straight from voff (prologue), else from voff_issue
#pragma unroll
        for (int i = 0; i < 2; ++i)
            dma16(vp, first ? voff[i] : voff_issue[i], lds0 + kVOff + slot * kTileBytes + (32 * i + 4 * wave) * 256);
    };
    // all loads but those issued in this step have landed (the last steps of a workgroup issue two or none: there
    // is no tile left to fetch)
    auto dma_wait = [&](int issued) {
        if (issued == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else if (issued == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    };

    // MODE 0 state: the list is walked incrementally per lane row: (e, off) = (entry, offset inside the
    // block) of the next tile to fetch; one tile further on they advance by (64 / b, 64 % b).
    const unsigned step_e = TK / ub, step_off = TK % ub;
    unsigned we[2], woff[2];
    int ent[2], eoff[2], tokv[2];
    // MODE 1/2 state: first token of tiles t .. t+3 (-1: no such tile) and the walk over the list.
    int nb[4] = {-1, -1, -1, -1};
    int nb2[4] = {-1, -1, -1, -1};                           // MODE 3: first token of the second half of tiles t .. t+3
    int walk_e = 0, walk_off = 0, dense_tile = 0;
    unsigned lane_k[2], lane_v[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const unsigned row = 32 * i + 4 * wave + r4;
        we[i] = row / ub; woff[i] = row % ub;
        lane_k[i] = row * tok_bytes + kch * 16;
        lane_v[i] = row * tok_bytes + vch * 16;
    }
    auto fetch_entries = [&]() {                             // MODE 0: call once per tile, in tile order
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int v = *LDS_PTR(const int, lds0 + kListOff + min(we[i], (unsigned)max(count - 1, 0)) * 4);
            ent[i] = (we[i] < (unsigned)count) ? v : -1;
            eoff[i] = (int)woff[i];
            we[i] += step_e; woff[i] += step_off;
            if (woff[i] >= ub) { woff[i] -= ub; we[i] += 1; }
        }
    };
    auto tile_offsets = [&]() {                              // MODE 0: offsets + row tokens of the fetched tile
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int tok = ent[i] * a.b + eoff[i];
            const bool valid = ent[i] >= 0 && (unsigned)tok < (unsigned)a.n;   // also rejects entries whose token index wrapped
            const unsigned base = __umul24(valid ? (unsigned)tok : 0u, tok_bytes);  // invalid rows read token 0, masked later
            koff[i] = base + kch * 16;
            voff[i] = base + vch * 16;
            tokv[i] = valid ? tok : 0x7fffffff;
        }
    };
    auto put_tok = [&](int slot) {
        if (pch == 0) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
                *LDS_PTR(int, lds0 + kTokOff + slot * TK * 4 + (32 * i + 4 * wave + r4) * 4) = tokv[i];
        }
    };
    int pre_ent = 0; bool early = false;                   // the list entry of the next walk step, fetched at the start of the tile step
    i32x2 pre_tile = {-1, -1};                     // MODE 3: the description of the next tile to queue
    int walk_t = 0;                                        // MODE 3: that tile's index
    auto prefetch_entry = [&]() {
        if (HALF) { pre_tile = *LDS_PTR(const i32x2, tab0 + min(walk_t, max(ntiles - 1, 0)) * 8); early = true; }
        else if (FAST && !DENSE) { pre_ent = *LDS_PTR(const int, lds0 + kListOff + min(walk_e, max(count - 1, 0)) * 4); early = true; }
    };
    auto next_base = [&]() -> int {                          // MODE 1/2: first token of the next tile in order, -1 past the end
        int base = -1;
        if (DENSE) {
            if (dense_tile < ntiles) base = dense_tile * TK;
            ++dense_tile;
        } else {
            if (walk_e < count)
                base = __builtin_amdgcn_readfirstlane(early ? pre_ent : *LDS_PTR(const int, lds0 + kListOff + walk_e * 4)) * a.b + walk_off;
            walk_off += TK;
            if (walk_off >= a.b) { walk_off = 0; ++walk_e; }
        }
        return base;
    };
    auto next_halves = [&](int& lo, int& hi) {               // MODE 3: the next tile in order, (-1, -1) past the end
        i32x2 d = pre_tile;
        if (!early) d = *LDS_PTR(const i32x2, tab0 + min(walk_t, max(ntiles - 1, 0)) * 8);
        const bool ok = walk_t < ntiles;
        lo = ok ? __builtin_amdgcn_readfirstlane(d[0]) : -1;
        hi = ok ? __builtin_amdgcn_readfirstlane(d[1]) : -1;
        ++walk_t;
    };
    auto half_offsets = [&](int lo, int hi) {                // MODE 3: offsets of the tile whose halves start at lo / hi
        if (lo >= 0 && hi >= 0 && lo <= a.n - 32 && hi <= a.n - 32) {   // uniform: both halves exist in full
            const unsigned s0 = (unsigned)lo * tok_bytes, s1 = (unsigned)(hi - 32) * tok_bytes;   // lane_k[1] holds row 32 + ...
            koff[0] = s0 + lane_k[0]; voff[0] = s0 + lane_v[0];
            koff[1] = s1 + lane_k[1]; voff[1] = s1 + lane_v[1];
        } else {                                             // ragged or missing half: rows without a token read token 0
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int base = i ? hi : lo;
                const int tok = base + 4 * wave + r4;
                const bool valid = base >= 0 && (unsigned)tok < (unsigned)a.n;
                const unsigned sb = __umul24(valid ? (unsigned)tok : 0u, tok_bytes);
                koff[i] = sb + kch * 16; voff[i] = sb + vch * 16;
            }
        }
    };
    auto base_offsets = [&](int base) {                      // MODE 1/2: offsets of the tile that starts at token base
        if (base >= 0 && base <= a.n - TK) {                 // uniform: the whole tile exists
            const unsigned sb = (unsigned)base * tok_bytes;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                koff[i] = sb + lane_k[i]; voff[i] = sb + lane_v[i];
            }
        } else {                                             // ragged last tile or no tile: invalid rows read token 0
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int tok = base + 32 * i + 4 * wave + r4;
                const bool valid = base >= 0 && (unsigned)tok < (unsigned)a.n;
                const unsigned sb = __umul24(valid ? (unsigned)tok : 0u, tok_bytes);
                koff[i] = sb + kch * 16; voff[i] = sb + vch * 16;
            }
        }
    };
    // describe the next tile in order (its DMA offsets go to koff/voff); MODE 0 also publishes its row tokens
    auto describe_next = [&](int slot) {
        voff_issue[0] = voff[0]; voff_issue[1] = voff[1];
        if (HALF) {
            nb[0] = nb[1]; nb[1] = nb[2]; nb[2] = nb[3];
            nb2[0] = nb2[1]; nb2[1] = nb2[2]; nb2[2] = nb2[3];
            next_halves(nb[3], nb2[3]);
            half_offsets(nb[3], nb2[3]);
        } else if (FAST) {
            nb[0] = nb[1]; nb[1] = nb[2]; nb[2] = nb[3]; nb[3] = next_base();
            base_offsets(nb[3]);
        } else {
            tile_offsets(); put_tok(slot); fetch_entries();
        }
    };

    // ---- per-lane LDS read addresses (bytes, ring slot 0) ----------------------------------------
    // K: row 32*kt + l32, logical chunk 2*ks + hh  ->  physical chunk (2*ks) ^ ((l32 & 15) ^ hh)
    // = k_base ^ (ks << 5): the row part has its low 8 bits clear (the LDS base is 1 KiB aligned)
    const unsigned k_base = (lds0 + kKOff + l32 * 256) | (unsigned)(((l32 & 15) ^ hh) << 4);
    // V (transposed read, 16-lane groups): lane supplies row 4*hh + (i16 >> 2) (+16*t4, +8) and the 8-byte
    // unit of channels 32*dt + 16*gbit + 4*(i16 & 3); physical chunk = logical chunk ^ 4*(row & 3)
    const int i16 = lane & 15, gbit = (lane >> 4) & 1;
    unsigned v_addr[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
        v_addr[dt] = lds0 + kVOff + (4 * hh + (i16 >> 2)) * 256 +
                     ((((unsigned)(dt ^ (i16 >> 2)) << 2) + 2 * gbit + ((i16 & 3) >> 1)) << 4) + (i16 & 1) * 8;

    f32x16 o[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float c = a.scale_log2e;
    const float lazy_raw = kLazyLog2 / c;                        // the same margin in units of the raw logits

    // ---- the three phases ---------------------------------------------------------------------
    // LDS fragments reach the MFMAs through a small ring of registers: the read of fragment j + kLook is issued
    // before the MFMA that consumes fragment j, so every MFMA has its operand kLook MFMAs (32 cycles each) after
    // the read was issued, with (kLook + 1) x 4 registers in all.  The first kLook fragments of a matrix phase are
    // read before the softmax phase that precedes it.  (Measured: depth 3 and 4 are equal within 1 %, deeper rings
    // are slower; reading in groups of four into two alternating register groups costs 12 more registers and is
    // 0.5 % (sparse) to 2.4 % (dense) slower.)
    // The read addresses carry the ring slot they point into (ka: the K slot, va: the V slot) and are moved on by
    // one slot per tile step, so that a fragment read needs no address arithmetic, only an immediate offset.
    unsigned ka[8], va[4];
    int ka_slot = 0, va_slot = 0;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) ka[ks] = k_base ^ (ks << 5);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) va[dt] = v_addr[dt];
    auto next_k_slot = [&]() {
        const unsigned d = ka_slot == NBUF - 1 ? (unsigned)(-(NBUF - 1) * kTileBytes) : (unsigned)kTileBytes;
        ka_slot = (ka_slot + 1) & (NBUF - 1);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) ka[ks] += d;
    };
    auto next_v_slot = [&]() {
        const unsigned d = va_slot == NBUF - 1 ? (unsigned)(-(NBUF - 1) * kTileBytes) : (unsigned)kTileBytes;
        va_slot = (va_slot + 1) & (NBUF - 1);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) va[dt] += d;
    };
    constexpr int kLook = KLOOK;
    bf16x8 ring[kLook + 1];
    auto read_k = [&](int ks, int kt, bf16x8& f) {           // K: channel step ks, key half kt
        f = as_bf16x8(*LDS_PTR(const u32x4, ka[ks] + kt * 32 * 256));
    };
    auto read_v = [&](int t4, int dt, bf16x8& f) {           // V: 16 keys t4, channel tile dt
        const unsigned ad = va[dt] + t4 * 16 * 256;
        const v4bf16_lds lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(v4bf16_lds, ad));
        const v4bf16_lds hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(v4bf16_lds, ad + 8 * 256));
#pragma unroll
        for (int e = 0; e < 4; ++e) { f[e] = lo[e]; f[4 + e] = hi[e]; }
    };
    // fragment j of a matrix phase.  kind 0: QK alone (16: ks = j / 2, kt = j % 2); kind 1: PV alone (16: t4 = j / 4,
    // dt = j % 4); kind 2: PV of one tile interleaved with QK of the next in groups of four (32)
    auto frag_read = [&](int kind, int j, bf16x8& f) __attribute__((always_inline)) {
        if (kind == 0) read_k(j >> 1, j & 1, f);
        else if (kind == 1) read_v(j >> 2, j & 3, f);
        else if ((j & 7) < 4) read_v(j >> 3, j & 3, f);
        else read_k(2 * (j >> 3) + (((j & 7) - 4) >> 1), j & 1, f);
    };
    auto frag_mfma = [&](int kind, int j, const bf16x8& f, f32x16 (&s)[2], const bf16x8 (&pf)[4]) __attribute__((always_inline)) {
        const bool is_v = kind == 1 || (kind == 2 && (j & 7) < 4);
        if (is_v) {
            const int t4 = kind == 1 ? (j >> 2) : (j >> 3), dt = j & 3;
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, pf[t4], o[dt], 0, 0, 0);
        } else {
            const int ks = kind == 0 ? (j >> 1) : 2 * (j >> 3) + (((j & 7) - 4) >> 1), kt = j & 1;
            s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, qf[ks], s[kt], 0, 0, 0);
        }
    };
    auto read_kg = [&](int, int) __attribute__((always_inline)) {    // first fragments of a phase that starts with QK
#pragma unroll
        for (int j = 0; j < kLook; ++j) frag_read(0, j, ring[j]);
    };
    auto read_vg = [&](int, int) __attribute__((always_inline)) {    // ... that starts with PV
#pragma unroll
        for (int j = 0; j < kLook; ++j) frag_read(1, j, ring[j]);
    };
    auto zero_s = [&](f32x16 (&s)[2]) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kt][r] = 0.f;
    };
    auto run_frags = [&](int kind, f32x16 (&s)[2], const bf16x8 (&pf)[4]) __attribute__((always_inline)) {
        const int n = kind == 2 ? 32 : 16;
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            if (j < n) {
                if (j + kLook < n) frag_read(kind, j + kLook, ring[(j + kLook) % (kLook + 1)]);
                frag_mfma(kind, j, ring[j % (kLook + 1)], s, pf);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    bf16x8 no_p[4];
    auto qk = [&](f32x16 (&s)[2]) __attribute__((always_inline)) { zero_s(s); run_frags(0, s, no_p); };
    auto pv = [&](const bf16x8 (&pf)[4]) __attribute__((always_inline)) { f32x16 no_s[2]; run_frags(1, no_s, pf); };
    auto mm_both = [&](f32x16 (&s)[2], const bf16x8 (&pf)[4]) __attribute__((always_inline)) { zero_s(s); run_frags(2, s, pf); };
    auto mask = [&](f32x16 (&s)[2], int slot) {
        const unsigned tok_base = lds0 + kTokOff + slot * TK * 4;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int gg = 0; gg < 4; ++gg) {
                const i32x4 t4 = *LDS_PTR(const i32x4, tok_base + (32 * kt + 8 * gg + 4 * hh) * 4);
                const int tv[4] = {t4[0], t4[1], t4[2], t4[3]};
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (tv[i] > qpos) s[kt][4 * gg + i] = -INFINITY;
            }
    };
    // MODE 1/2: the tile holds tokens base .. base+63; key row kr is visible iff base + kr <= min(qpos, n-1)
    auto mask_base = [&](f32x16 (&s)[2], int base) {
        const int lim = min(qpos, a.n - 1) - base - 4 * hh;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int gg = 0; gg < 4; ++gg)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (32 * kt + 8 * gg + i > lim) s[kt][4 * gg + i] = -INFINITY;
    };
    // MODE 3: key row 32*kt + kr of the tile is token (kt ? hi : lo) + kr; a missing half (-1) is masked whole
    auto mask_halves = [&](f32x16 (&s)[2], int lo, int hi) {
        const int top = min(qpos, a.n - 1) - 4 * hh;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            const int base = kt ? hi : lo;
            const int lim = base < 0 ? -1 : top - base;
#pragma unroll
            for (int gg = 0; gg < 4; ++gg)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (8 * gg + i > lim) s[kt][4 * gg + i] = -INFINITY;
        }
    };
    // S^T tile -> P^T fragments; running max / sum; O rescaled when any row's max moved
    auto sm = [&](f32x16 (&s)[2], bf16x8 (&pf)[4]) {
        float mx = fmaxf(s[0][0], s[0][1]), my = fmaxf(s[1][0], s[1][1]);   // two chains of v_max3
#pragma unroll
        for (int r = 2; r < 16; r += 2) {
            mx = fmaxf(fmaxf(s[0][r], s[0][r + 1]), mx);
            my = fmaxf(fmaxf(s[1][r], s[1][r + 1]), my);
        }
        mx = half_max(fmaxf(mx, my));
        // The reference point of a row moves only when the row's max has outgrown it by more than 2^kLazyLog2 in the
        // exponent: until then P is computed against the old reference (P <= 2^kLazyLog2, exact in fp32 and well inside
        // bf16's range; O, l and the final O / l all carry the same factor), and O needs no rescaling.
        const float m_new = (mx > m_run + lazy_raw) ? mx : m_run;
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_safe) * c);
        const float ms = m_safe * c;
        m_run = m_new;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kt][r] = __builtin_amdgcn_exp2f(fmaf(s[kt][r], c, -ms));
        // P^T as B operand: 16-key step t4 = 2*kt + gp takes accumulator registers 8*gp .. 8*gp+7.  The row
        // sum adds up the bf16-rounded values that the PV contraction actually uses, two per instruction.
        bf16x2 one2; one2[0] = (__bf16)1.0f; one2[1] = (__bf16)1.0f;
        float rs0 = 0.f, rs1 = 0.f;
#pragma unroll
        for (int t4 = 0; t4 < 4; ++t4) {
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[t4][e] = (__bf16)s[t4 >> 1][8 * (t4 & 1) + e];
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                bf16x2 pr; pr[0] = pf[t4][e]; pr[1] = pf[t4][e + 1];
                if (e & 2) rs1 = __builtin_amdgcn_fdot2_f32_bf16(pr, one2, rs1, false);
                else rs0 = __builtin_amdgcn_fdot2_f32_bf16(pr, one2, rs0, false);
            }
        }
        l_run = l_run * alpha + (rs0 + rs1);                 // per-half partial sums, merged at the end
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
        }
    };
    auto first_tok = [&](int slot) { return *LDS_PTR(const int, lds0 + kTokOff + slot * TK * 4); };
    auto last_tok = [&](int slot) { return *LDS_PTR(const int, lds0 + kTokOff + slot * TK * 4 + (TK - 1) * 4); };
    // tile t (ring slot) as seen by this wave: does any of its rows see the tile, does the tile need a mask
    auto tile_active = [&](int slot, int base) {
        return FAST ? (base >= 0 && base <= wq_last) : (first_tok(slot) <= wq_last);
    };
    auto mask_if_needed = [&](f32x16 (&s)[2], int slot, int base) {
        if (HALF) {                                          // slot: position in the nb / nb2 queue (0 = this tile)
            const int hi = nb2[0], top = max(base, hi);
            if (hi < 0 || top + 31 > wq_lo || top + 32 > a.n) mask_halves(s, base, hi);
        }
        else if (FAST) { if (base + TK - 1 > wq_lo || base + TK > a.n) mask_base(s, base); }
        else { if (last_tok(slot) > wq_lo) mask(s, slot); }
    };
    // end of a tile step: tile t+2 has landed (this wave's rows; at most the 4 loads of tile t+3 are still in
    // flight), then everybody is past its reads of tile t; afterwards the loader moves on to tile t+4 (its
    // row tokens, in MODE 0, go into the slot tile t just vacated).
    auto step_end = [&](int slot, int issued) {
        if (FAST) describe_next(slot);                       // registers only
        dma_wait(issued);
        __syncthreads();
        if (!FAST) describe_next(slot);                      // writes the row tokens into the vacated slot
    };

    // ---- prologue: K of tiles 0-2 and V of tiles 0-1 in flight; tiles up to 3 described -------------
    if (ntiles > 0) {
        if (!FAST) fetch_entries();
#pragma unroll
        for (int s3 = 0; s3 < 4; ++s3) {
            if (HALF) { next_halves(nb[s3], nb2[s3]); half_offsets(nb[s3], nb2[s3]); }
            else if (FAST) { nb[s3] = next_base(); base_offsets(nb[s3]); }
            else { tile_offsets(); fetch_entries(); put_tok(s3); }
            if (s3 == 0) { issue_k(0); issue_v(0, true); }
            if (s3 == 1) { issue_k(1); }                     // K0 V0 K1 first: they are needed at once
            if (s3 == 1 || s3 == 2) {
                if (s3 == 2) { issue_v(1, false); issue_k(2); }
                voff_issue[0] = voff[0]; voff_issue[1] = voff[1];
            }
        }
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) pin(qf[ks]);                      // Q has arrived: no wait for it is left in the key loop
    if (ntiles > 0) dma_wait(4);                                     // K0, V0, K1 have landed
    __syncthreads();
    // from here on: koff = K offsets of tile 3, voff_issue = V offsets of tile 2, voff = V offsets of tile 3

    f32x16 s[2]; bf16x8 pf[4];
    if (!rotated) {
        // step t: ka points into the slot of K(t), va into the slot of V(t-1)
        bool have_p = false;                                         // P^T of tile t-1 waits for its PV
        bool act = ntiles > 0 && tile_active(0, nb[0]);              // wave-uniform; once false it stays false
        va_slot = NBUF - 1;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) va[dt] += (NBUF - 1) * kTileBytes;
        if (act) read_kg(0, 0);
        for (int t = 0; t < ntiles; ++t) {
            const int slot = t & 3, nslot = (t + 1) & 3;
            prefetch_entry();
            __builtin_amdgcn_s_setprio(3);                               // matrix phase: its MFMAs go ahead of the partner's VALU work
            if (have_p && act) mm_both(s, pf);
            else if (act) qk(s);
            else if (have_p) pv(pf);
            __builtin_amdgcn_s_setprio(0);
            const int issued = t + 3 < ntiles ? 4 : (t + 2 < ntiles ? 2 : 0);
            if (issued >= 2) issue_v((t + 2) & 3, false);                // after the matrix phase, which starts with the step
            if (issued == 4) issue_k((t + 3) & 3);
            next_k_slot(); next_v_slot();                                // K(t+1), V(t)
            const bool act_next = act && (t + 1 < ntiles) && tile_active(nslot, nb[1]);
            if (act) {
                read_vg(0, 0);                                       // first group of the next matrix phase
                mask_if_needed(s, slot, nb[0]);
                sm(s, pf);
            }
            have_p = act; act = act_next;
            step_end(slot, issued);
        }
        if (have_p) pv(pf);
    } else {
        // step t: va points into the slot of V(t), ka into the slot of K(t+1)
        bool have_s = ntiles > 0 && tile_active(0, nb[0]);
        if (have_s) { read_kg(0, 0); qk(s); }
        next_k_slot();
        for (int t = 0; t < ntiles; ++t) {
            const int slot = t & 3, nslot = (t + 1) & 3;
            prefetch_entry();
            const bool act_next = have_s && (t + 1 < ntiles) && tile_active(nslot, nb[1]);
            if (have_s) {
                read_vg(0, 0);                                       // first group of the matrix phase below
                mask_if_needed(s, slot, nb[0]);
                sm(s, pf);
                __builtin_amdgcn_s_setprio(3);
                if (act_next) mm_both(s, pf);
                else pv(pf);
                __builtin_amdgcn_s_setprio(0);
            }
            const int issued = t + 3 < ntiles ? 4 : (t + 2 < ntiles ? 2 : 0);
            if (issued >= 2) issue_v((t + 2) & 3, false);                // after the matrix phase, like waves 0-3
            if (issued == 4) issue_k((t + 3) & 3);
            next_k_slot(); next_v_slot();
            have_s = act_next;
            step_end(slot, issued);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                 // no DMA may outlive the workgroup

    // ---- epilogue: O^T[ch][q] / l -> out[q][ch], transposed through LDS so that global stores are whole rows ----
    {
        const float l_tot = half_sum(l_run);
        const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
        __syncthreads();                                             // every wave is past its last tile reads
        const unsigned stage = lds0 + kVOff + wave * (WQ * kOutPitch);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int gg = 0; gg < 4; ++gg) {
                bf16x4 w;
#pragma unroll
                for (int i = 0; i < 4; ++i) w[i] = (__bf16)(o[dt][4 * gg + i] * inv);
                *LDS_PTR(bf16x4, stage + l32 * kOutPitch + (32 * dt + 8 * gg + 4 * hh) * 2) = w;
            }
        // the wave reads back only what it wrote itself: 4 rows of 256 B per instruction
        uint16_t* ob = a.out + bb * a.os0 + h * a.os1;
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const int row = 4 * x + r4;
            const u32x4 val = *LDS_PTR(const u32x4, stage + row * kOutPitch + pch * 16);
            if (wq_lo + row < q_end) *(u32x4*)(ob + (long long)(wq_lo + row) * a.os2 + pch * 8) = val;
        }
        if (a.lse && hh == 0 && qpos < q_end)
            a.lse[((long long)bb * a.hq + h) * a.n + qpos] = l_tot > 0.f ? m_run * a.scale + __logf(l_tot) : -INFINITY;
    }
}

}  // namespace

hipError_t launch_attn_bf16(const Shape& sh, const void* q, const void* k, const void* v, const int32_t* idx,
                            const int32_t* cnt, bool shared_lists, void* out, float* lse, hipStream_t st) {
    ArgsB a;
    a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v; a.idx = idx; a.cnt = cnt;
    a.out = (uint16_t*)out; a.lse = lse;
    a.batch = sh.batch; a.hq = sh.hq; a.hkv = sh.hkv; a.n = sh.n; a.s = sh.s; a.b = sh.b; a.n1 = sh.n1;
    a.list_len = sh.list_len; a.shared_lists = shared_lists ? 1 : 0;
    a.scale = sh.attn_scale;
    a.scale_log2e = sh.attn_scale * 1.4426950408889634f;
    a.qs0 = sh.qs[0]; a.qs1 = sh.qs[1]; a.qs2 = sh.qs[2];
    a.ks0 = sh.kvs[0]; a.ks1 = sh.kvs[1]; a.ks2 = sh.kvs[2];
    a.os0 = sh.os[0]; a.os1 = sh.os[1]; a.os2 = sh.os[2];
    hipError_t e;
    if (idx) {
        if (sh.list_len > kMaxListBf16) return hipErrorInvalidValue;
        a.qtiles = (sh.s + TQ - 1) / TQ;
        const long long grid = (long long)sh.batch * sh.hq * sh.n1 * a.qtiles;
        const int smem = kListOff + ((sh.list_len * 4 + 1023) & ~1023);
        const int tab_bytes = (int)(((long long)sh.list_len * sh.b + TK - 1) / TK) * 8;     // MODE 3: tile descriptions
        if (sh.b % TK == 0) {
            e = hipFuncSetAttribute((const void*)attn_bf16_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(attn_bf16_kernel<1>, dim3((unsigned)grid), dim3(512), smem, st, a);
        } else if (sh.b % 32 == 0 && smem + tab_bytes <= 160 * 1024) {
            e = hipFuncSetAttribute((const void*)attn_bf16_kernel<3>, hipFuncAttributeMaxDynamicSharedMemorySize, smem + tab_bytes);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(attn_bf16_kernel<3>, dim3((unsigned)grid), dim3(512), smem + tab_bytes, st, a);
        } else {
            e = hipFuncSetAttribute((const void*)attn_bf16_kernel<0>, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(attn_bf16_kernel<0>, dim3((unsigned)grid), dim3(512), smem, st, a);
        }
    } else {
        a.qtiles = (sh.n + TQ - 1) / TQ;
        const long long grid = (long long)sh.batch * sh.hq * a.qtiles;
        e = hipFuncSetAttribute((const void*)attn_bf16_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                kListOff);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(attn_bf16_kernel<2>, dim3((unsigned)grid), dim3(512), kListOff, st, a);
    }
    return hipGetLastError();
}

}  // namespace cp
