// fp32 attention (correctness configuration): Algorithm 2's per-segment loop over a block list,
// or Eq. 2 dense causal attention when no list is given.  Plain fp32 FMA flash loop, no reduced
// precision anywhere: 32 query rows x 32 gathered key tokens per step.
#include "kernels.h"

namespace cp {
namespace {

constexpr int TQ = 32, TK = 32, PITCH = kHeadDim + 4;   // floats; 528 B rows keep float4 alignment

struct Args32 {
    const float* q; const float* k; const float* v; const int32_t* idx; const int32_t* cnt;
    float* out; float* lse;
    int hq, hkv, n, s, b, n1, list_len, qtiles;   // qtiles: per segment (sparse) or per sequence (dense)
    int shared_lists;                             // lists are per (batch, KV head, segment) instead of per query head
    float scale;
    long long qs0, qs1, qs2, ks0, ks1, ks2, os0, os1, os2;
};

template <bool DENSE>
__global__ __launch_bounds__(256) void attn_fp32_kernel(Args32 a) {
    __shared__ __attribute__((aligned(16))) float Qs[TQ * PITCH];
    __shared__ __attribute__((aligned(16))) float Ks[TK * PITCH];
    __shared__ __attribute__((aligned(16))) float Vs[TK * PITCH];
    __shared__ float Ps[TQ * (TK + 1)];
    __shared__ int Tok[TK];

    const int tid = threadIdx.x;
    long long w = blockIdx.x;
    const int qt = (int)(w % a.qtiles); w /= a.qtiles;
    int j = 0;
    if (!DENSE) { j = (int)(w % a.n1); w /= a.n1; }
    const int h = (int)(w % a.hq); const int bb = (int)(w / a.hq);
    const int g = h / (a.hq / a.hkv);

    const int q_lo = DENSE ? qt * TQ : j * a.s + qt * TQ;
    const int q_end = DENSE ? a.n : min(a.n, (j + 1) * a.s);       // rows >= q_end do not exist
    if (q_lo >= q_end) return;                                     // uniform: tile past a short segment
    const int q_last = min(q_end, q_lo + TQ) - 1;
    const float* qp = a.q + bb * a.qs0 + h * a.qs1;
    const float* kp = a.k + bb * a.ks0 + g * a.ks1;
    const float* vp = a.v + bb * a.ks0 + g * a.ks1;

    for (int x = tid; x < TQ * 32; x += 256) {
        const int row = x >> 5, c4 = x & 31;
        float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
        if (q_lo + row < q_end) val = *(const float4*)(qp + (long long)(q_lo + row) * a.qs2 + c4 * 4);
        *(float4*)(Qs + row * PITCH + c4 * 4) = val;
    }

    const int32_t* list = nullptr; int count = 0;
    if (!DENSE) {
        const long long lrow = a.shared_lists ? ((long long)bb * a.hkv + g) * a.n1 + j : ((long long)bb * a.hq + h) * a.n1 + j;
        list = a.idx + lrow * a.list_len;
        count = min(max(a.cnt[lrow], 0), a.list_len);
    }
    const long long total = DENSE ? (long long)q_last + 1 : (long long)count * a.b;   // virtual key positions
    const int ntiles = (int)((total + TK - 1) / TK);

    const int qr = tid >> 3, sub = tid & 7;
    const int qpos = q_lo + qr;
    float m = -INFINITY, l = 0.f;
    float o[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) o[e] = 0.f;
    constexpr float kLog2e = 1.4426950408889634f;

    for (int t = 0; t < ntiles; ++t) {
        __syncthreads();                                   // previous tile fully consumed
        for (int x = tid; x < TK * 32; x += 256) {
            const int row = x >> 5, c4 = x & 31;
            const long long p = (long long)t * TK + row;
            int tok; bool valid;
            if (DENSE) { tok = (int)p; valid = p < total; }
            else {
                const int e = (int)(p / a.b);
                valid = e < count;
                const long long blk = valid ? list[e] : 0;
                const long long tk = blk * a.b + (p - (long long)e * a.b);
                valid = valid && blk >= 0 && tk < a.n;             // entries outside the sequence are masked rows
                tok = valid ? (int)tk : 0;
            }
            float4 kv = make_float4(0.f, 0.f, 0.f, 0.f), vv = kv;
            if (valid) {
                kv = *(const float4*)(kp + (long long)tok * a.ks2 + c4 * 4);
                vv = *(const float4*)(vp + (long long)tok * a.ks2 + c4 * 4);
            }
            *(float4*)(Ks + row * PITCH + c4 * 4) = kv;
            *(float4*)(Vs + row * PITCH + c4 * 4) = vv;
            if (c4 == 0) Tok[row] = valid ? tok : 0x7fffffff;
        }
        __syncthreads();
        if (Tok[0] > q_last) break;                        // ascending lists: nothing visible from here on
        // ---- S = scale * Q K^T : thread (qr, sub) owns keys sub, sub+8, sub+16, sub+24
        float sc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
        for (int c = 0; c < kHeadDim; c += 4) {
            const float4 qv = *(const float4*)(Qs + qr * PITCH + c);
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const float4 kv = *(const float4*)(Ks + (sub + 8 * x) * PITCH + c);
                sc[x] = fmaf(qv.x, kv.x, sc[x]); sc[x] = fmaf(qv.y, kv.y, sc[x]);
                sc[x] = fmaf(qv.z, kv.z, sc[x]); sc[x] = fmaf(qv.w, kv.w, sc[x]);
            }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            sc[x] = (Tok[sub + 8 * x] <= qpos) ? sc[x] * a.scale : -INFINITY;
            mx = fmaxf(mx, sc[x]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 1)); mx = fmaxf(mx, __shfl_xor(mx, 2)); mx = fmaxf(mx, __shfl_xor(mx, 4));
        const float m_new = fmaxf(m, mx);
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = exp2f((m - m_safe) * kLog2e);
        float rs = 0.f;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const float p = exp2f((sc[x] - m_safe) * kLog2e);
            Ps[qr * (TK + 1) + sub + 8 * x] = p;
            rs += p;
        }
        rs += __shfl_xor(rs, 1); rs += __shfl_xor(rs, 2); rs += __shfl_xor(rs, 4);
        l = l * alpha + rs;
        m = m_new;
#pragma unroll
        for (int e = 0; e < 16; ++e) o[e] *= alpha;
        __syncthreads();
        // ---- O += P V : thread (qr, sub) owns channels 4*sub + 32*x .. +3, x = 0..3
#pragma unroll 4
        for (int key = 0; key < TK; ++key) {
            const float p = Ps[qr * (TK + 1) + key];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const float4 vv = *(const float4*)(Vs + key * PITCH + 4 * sub + 32 * x);
                o[4 * x + 0] = fmaf(p, vv.x, o[4 * x + 0]); o[4 * x + 1] = fmaf(p, vv.y, o[4 * x + 1]);
                o[4 * x + 2] = fmaf(p, vv.z, o[4 * x + 2]); o[4 * x + 3] = fmaf(p, vv.w, o[4 * x + 3]);
            }
        }
    }
    if (qpos < q_end) {
        const float inv = l > 0.f ? 1.0f / l : 0.f;
        float* op = a.out + bb * a.os0 + h * a.os1 + (long long)qpos * a.os2;
#pragma unroll
        for (int x = 0; x < 4; ++x)
            *(float4*)(op + 4 * sub + 32 * x) =
                make_float4(o[4 * x] * inv, o[4 * x + 1] * inv, o[4 * x + 2] * inv, o[4 * x + 3] * inv);
        if (a.lse && sub == 0)
            a.lse[((long long)bb * a.hq + h) * a.n + qpos] = l > 0.f ? m + logf(l) : -INFINITY;
    }
}

}  // namespace

hipError_t launch_attn_fp32(const Shape& sh, const void* q, const void* k, const void* v, const int32_t* idx,
                            const int32_t* cnt, bool shared_lists, void* out, float* lse, hipStream_t st) {
    Args32 a;
    a.q = (const float*)q; a.k = (const float*)k; a.v = (const float*)v; a.idx = idx; a.cnt = cnt;
    a.out = (float*)out; a.lse = lse;
    a.hq = sh.hq; a.hkv = sh.hkv; a.n = sh.n; a.s = sh.s; a.b = sh.b; a.n1 = sh.n1; a.list_len = sh.list_len;
    a.shared_lists = shared_lists ? 1 : 0;
    a.scale = sh.attn_scale;
    a.qs0 = sh.qs[0]; a.qs1 = sh.qs[1]; a.qs2 = sh.qs[2];
    a.ks0 = sh.kvs[0]; a.ks1 = sh.kvs[1]; a.ks2 = sh.kvs[2];
    a.os0 = sh.os[0]; a.os1 = sh.os[1]; a.os2 = sh.os[2];
    if (idx) {
        a.qtiles = (sh.s + TQ - 1) / TQ;
        const long long grid = (long long)sh.batch * sh.hq * sh.n1 * a.qtiles;
        hipLaunchKernelGGL(attn_fp32_kernel<false>, dim3((unsigned)grid), dim3(256), 0, st, a);
    } else {
        a.qtiles = (sh.n + TQ - 1) / TQ;
        const long long grid = (long long)sh.batch * sh.hq * a.qtiles;
        hipLaunchKernelGGL(attn_fp32_kernel<true>, dim3((unsigned)grid), dim3(256), 0, st, a);
    }
    return hipGetLastError();
}

}  // namespace cp
