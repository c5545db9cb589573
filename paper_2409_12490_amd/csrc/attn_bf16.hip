// bf16 MFMA flash attention for gfx950: Algorithm 2's per-segment loop over a block list
// (block-sparse, gathered K/V tiles) and Eq. 2 dense causal attention (no list) from one kernel body.
//
// Workgroup = 4 wave64 = 256 query rows of one segment (sparse) or of the sequence (dense); a wave owns
// 64 rows as two 32-row MFMA tiles.  The key loop walks 64-token tiles of the "virtual" token list
// (the listed blocks laid end to end).  Per tile and wave:
//
//   S^T[key][q] = K_tile . Q^T      32x32x16 bf16 MFMA, A = K rows from LDS (ds_read_b128), B = Q
//                                   fragments that stay in registers for the whole kernel.
//   online softmax                  S^T puts one query per lane column, so row max / row sum are
//                                   in-lane reductions plus one exchange between the wave halves.
//   O^T[ch][q] += V^T . P^T         A = V read from LDS through the transposing ds_read_b64_tr_b16,
//                                   B = P^T taken straight from the S^T accumulators (the key order
//                                   inside a 16-key MFMA step is chosen so no shuffle is needed).
//
// K/V tiles are staged global -> registers -> LDS, double buffered, one barrier per tile.
#include "kernels.h"

namespace cp {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 v4bf16_lds;

constexpr int TQ = 256;     // query rows per workgroup
constexpr int TK = 64;      // key tokens per tile
constexpr int KP = 136;     // K row pitch in LDS, bf16 elements (272 B: conflict-free 16 B row reads)
constexpr int VP = 144;     // V row pitch in LDS (288 B: conflict-free transposed 8 B reads)
constexpr int kSmemBytes = 2 * TK * KP * 2 + 2 * TK * VP * 2 + 2 * TK * 4;

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

template <bool DENSE>
__global__ __launch_bounds__(256, 1) void attn_bf16_kernel(ArgsB a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint16_t* Ks = (uint16_t*)smem;                 // [2][TK*KP]
    uint16_t* Vs = Ks + 2 * TK * KP;                // [2][TK*VP]
    int* Tok = (int*)(Vs + 2 * TK * VP);            // [2][TK] token position of every tile row

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
    const uint16_t* kp = a.k + bb * a.ks0 + g * a.ks1;
    const uint16_t* vp = a.v + bb * a.ks0 + g * a.ks1;

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

    // ---- the virtual token list --------------------------------------------------------------
    const int32_t* list = nullptr; int count = 0;
    if (!DENSE) {
        const long long lrow = ((long long)bb * a.hq + h) * a.n1 + j;
        list = a.idx + lrow * a.list_len;
        count = a.cnt[lrow];
    }
    // positions 0 .. total-1 of the listed blocks laid end to end (host checks count * b < 2^31)
    const unsigned total = DENSE ? (unsigned)q_last + 1u : (unsigned)count * (unsigned)a.b;
    const unsigned ub = (unsigned)a.b;
    int ntiles = (int)((total + TK - 1) / TK);
    if (!DENSE) {   // drop trailing tiles that start after the last query row (lists are ascending)
        while (ntiles > 0) {
            const unsigned p = (unsigned)(ntiles - 1) * TK;
            const unsigned e = p / ub;
            const int tok = list[e] * a.b + (int)(p - e * ub);
            if (tok <= q_last) break;
            --ntiles;
        }
    }

    // ---- staging: thread -> (rows r0 + 16*i, 16-byte chunk c16) of the 64 x 128 tile --------------
    const int c16 = tid & 15, r0 = tid >> 4;
    uint4 kr[4], vr[4]; int tk[4];
    auto fetch = [&](int t) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = r0 + 16 * i;
            const unsigned p = (unsigned)t * TK + row;
            int tok; bool valid;
            if (DENSE) { tok = (int)p; valid = p < total; }
            else {
                const unsigned e = p / ub;
                valid = e < (unsigned)count;
                tok = valid ? list[e] * a.b + (int)(p - e * ub) : 0;
                valid = valid && tok < a.n;
            }
            kr[i] = make_uint4(0, 0, 0, 0); vr[i] = kr[i];
            if (valid) {
                kr[i] = *(const uint4*)(kp + (long long)tok * a.ks2 + c16 * 8);
                vr[i] = *(const uint4*)(vp + (long long)tok * a.ks2 + c16 * 8);
            }
            tk[i] = valid ? tok : 0x7fffffff;
        }
    };
    auto stash = [&](int buf) {
        uint16_t* kd = Ks + buf * TK * KP; uint16_t* vd = Vs + buf * TK * VP; int* td = Tok + buf * TK;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = r0 + 16 * i;
            *(uint4*)(kd + row * KP + c16 * 8) = kr[i];
            *(uint4*)(vd + row * VP + c16 * 8) = vr[i];
            if (c16 == 0) td[row] = tk[i];
        }
    };

    f32x16 o[4][2];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[dt][t2][r] = 0.f;
    float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};
    const float c = a.scale_log2e;

    if (ntiles > 0) { fetch(0); stash(0); }
    __syncthreads();

    for (int t = 0; t < ntiles; ++t) {
        const int cur = t & 1;
        const bool more = t + 1 < ntiles;
        if (more) fetch(t + 1);

        const uint16_t* Kc = Ks + cur * TK * KP;
        const uint16_t* Vc = Vs + cur * TK * VP;
        const int* Tc = Tok + cur * TK;
        const int first_tok = Tc[0], last_tok = Tc[TK - 1];
        if (first_tok <= wq_last) {                                  // wave-uniform
            // ---- S^T = K Q^T ----------------------------------------------------------------
            f32x16 sacc[2][2];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                    for (int r = 0; r < 16; ++r) sacc[kt][t2][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
                for (int kt = 0; kt < 2; ++kt) {
                    const bf16x8 kf = as_bf16x8(*(const uint4*)(Kc + (32 * kt + l32) * KP + 16 * ks + 8 * hh));
#pragma unroll
                    for (int t2 = 0; t2 < 2; ++t2)
                        sacc[kt][t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t2][ks], sacc[kt][t2], 0, 0, 0);
                }
            }
            // ---- causal / validity mask: only tiles that reach past the wave's first row ------
            if (last_tok > wq_lo) {
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int gg = 0; gg < 4; ++gg) {
                        const int4 t4 = *(const int4*)(Tc + 32 * kt + 8 * gg + 4 * hh);
                        const int tv[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
                        for (int i = 0; i < 4; ++i)
#pragma unroll
                            for (int t2 = 0; t2 < 2; ++t2)
                                if (tv[i] > qpos[t2]) sacc[kt][t2][4 * gg + i] = -INFINITY;
                    }
            }
            // ---- online softmax, one query per lane column ----------------------------------
            bf16x8 pf[2][4];
            float alpha[2];
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2) {
                float mx = sacc[0][t2][0];
#pragma unroll
                for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sacc[0][t2][r]);
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[1][t2][r]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_run[t2], mx);
                const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
                alpha[t2] = __builtin_amdgcn_exp2f((m_run[t2] - m_safe) * c);
                const float ms = m_safe * c;
                float rs = 0.f;
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kt][t2][r], c, -ms));
                        sacc[kt][t2][r] = p;
                        rs += p;
                    }
                l_run[t2] = l_run[t2] * alpha[t2] + rs;          // per-half partial sums, merged at the end
                m_run[t2] = m_new;
                // P^T as B operand: 16-key step t4 = 2*kt + gp takes register groups 2*gp and 2*gp+1
#pragma unroll
                for (int t4 = 0; t4 < 4; ++t4) {
                    const int kt = t4 >> 1, base = 8 * (t4 & 1);
#pragma unroll
                    for (int e = 0; e < 8; ++e) pf[t2][t4][e] = (__bf16)sacc[kt][t2][base + e];
                }
            }
            if (__builtin_amdgcn_ballot_w64(alpha[0] != 1.0f || alpha[1] != 1.0f) != 0) {
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                    for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                        for (int r = 0; r < 16; ++r) o[dt][t2][r] *= alpha[t2];
            }
            // ---- O^T += V^T P^T ---------------------------------------------------------------
            const int i16 = lane & 15;
            const uint16_t* vbase = Vc + (4 * hh + (i16 >> 2)) * VP + 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) {
                    const uint16_t* p0 = vbase + (16 * t4) * VP + 32 * dt;
                    const v4bf16_lds lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                        (__attribute__((address_space(3))) v4bf16_lds*)(p0));
                    const v4bf16_lds hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                        (__attribute__((address_space(3))) v4bf16_lds*)(p0 + 8 * VP));
                    bf16x8 vf;
#pragma unroll
                    for (int e = 0; e < 4; ++e) { vf[e] = lo[e]; vf[4 + e] = hi[e]; }
#pragma unroll
                    for (int t2 = 0; t2 < 2; ++t2)
                        o[dt][t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[t2][t4], o[dt][t2], 0, 0, 0);
                }
            }
        }
        if (more) stash(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue: O^T[ch][q] / l  ->  out[q][ch] ------------------------------------------------
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
        const float l_tot = l_run[t2] + __shfl_xor(l_run[t2], 32);
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
        e = hipFuncSetAttribute((const void*)attn_bf16_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                kSmemBytes);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(attn_bf16_kernel<false>, dim3((unsigned)grid), dim3(256), kSmemBytes, st, a);
    } else {
        a.qtiles = (sh.n + TQ - 1) / TQ;
        const long long grid = (long long)sh.batch * sh.hq * a.qtiles;
        e = hipFuncSetAttribute((const void*)attn_bf16_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                kSmemBytes);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(attn_bf16_kernel<true>, dim3((unsigned)grid), dim3(256), kSmemBytes, st, a);
    }
    return hipGetLastError();
}

}  // namespace cp
