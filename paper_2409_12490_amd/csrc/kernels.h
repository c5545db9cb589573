// Internal launch interface between the C ABI (api.hip) and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cp {

constexpr int kHeadDim = 128;
constexpr int kMaxListBf16 = 6144;    // block-list entries the bf16 attention kernel keeps in LDS

struct Shape {
    int batch, hq, hkv, n, s, b, r, n1, n2;   // r = s / b
    int budget, local, list_len;
    int dtype;                                // 0 fp32, 1 bf16
    float attn_scale, score_scale, alpha;
    int softmax_domain;
    int64_t qs[3], kvs[3], os[3];             // element strides: batch, head, token
};

// Algorithm 1, max/min lines: representatives in the storage dtype.
// qrep [B,Hq,n1,2,128], krep [B,Hkv,n2,2,128]; index 0 = max, 1 = min.
hipError_t launch_pool(const Shape& sh, const void* q, const void* k, void* qrep, void* krep, hipStream_t st);

// Algorithm 1, score lines (four products, softmax, combine, mask, fusion).
// stats: score_stats_bytes() of scratch (bf16: per-chunk softmax statistics; fp32: unused, 0 bytes).
size_t score_stats_bytes(const Shape& sh);
hipError_t launch_score(const Shape& sh, const void* qrep, const void* krep, const float* prev, float* scores,
                        float* stats, hipStream_t st);

// Algorithm 2, top-k line.  shared: one list per (batch, KV head, segment) from the max of the scores of the
// KV head's query heads (idx [B,Hkv,n1,list_len], cnt [B,Hkv,n1]) instead of one per query head.
hipError_t launch_select(const Shape& sh, const float* scores, int32_t* idx, int32_t* cnt, bool shared, hipStream_t st);

// Algorithm 2 attention loop (idx != nullptr) or Eq. 2 dense causal attention (idx == nullptr).
// shared_lists: idx/cnt hold one list per KV head (see launch_select) instead of one per query head.
hipError_t launch_attn_bf16(const Shape& sh, const void* q, const void* k, const void* v, const int32_t* idx,
                            const int32_t* cnt, bool shared_lists, void* out, float* lse, hipStream_t st);
hipError_t launch_attn_fp32(const Shape& sh, const void* q, const void* k, const void* v, const int32_t* idx,
                            const int32_t* cnt, bool shared_lists, void* out, float* lse, hipStream_t st);

}  // namespace cp
