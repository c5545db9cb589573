// C ABI of the library: argument checks, then kernel launches on the caller's stream.
#include "../../include/critiprefill.h"
#include "kernels.h"

#include <cmath>
#include <mutex>

// Scratch of critiprefill_estimate_static: the representatives and score statistics that critiprefill_estimate
// keeps in the caller's workspace.  One copy per GPU the library runs on, held until the process ends.  In host
// code this name is only a handle for hipGetSymbolAddress; kernels and copies get the resolved device address.
static __device__ __align__(256) unsigned char scratch[CRITIPREFILL_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];    // device address of `scratch` on each device, resolved on first use

// Device address of this device's copy of `scratch` (nullptr on failure).
void* static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

constexpr int kMaxBlocks = 8192;     // score kernel keeps four logit rows in LDS; select keeps a row in registers

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int make_shape(const critiprefill_params* p, cp::Shape* sh) {
    if (!p) return CP_ERR_NULL;
    if (p->batch <= 0 || p->n_q_heads <= 0 || p->n_kv_heads <= 0 || p->seq_len <= 0 || p->segment_size <= 0 ||
        p->block_size <= 0 || p->budget_blocks < 0 || p->local_blocks < 0)
        return CP_ERR_SHAPE;
    if (p->n_q_heads % p->n_kv_heads != 0 || p->segment_size % p->block_size != 0) return CP_ERR_SHAPE;
    if (!(p->attn_scale >= 0.f) || !(p->score_scale >= 0.f)) return CP_ERR_SHAPE;
    if (p->head_dim != cp::kHeadDim) return CP_ERR_UNSUPPORTED;
    if (p->dtype != CP_DTYPE_FP32 && p->dtype != CP_DTYPE_BF16) return CP_ERR_UNSUPPORTED;
    if (p->softmax_domain != 0 && p->softmax_domain != 1) return CP_ERR_UNSUPPORTED;
    sh->batch = p->batch; sh->hq = p->n_q_heads; sh->hkv = p->n_kv_heads; sh->n = p->seq_len;
    sh->s = p->segment_size; sh->b = p->block_size; sh->r = sh->s / sh->b;
    sh->n1 = (sh->n + sh->s - 1) / sh->s; sh->n2 = (sh->n + sh->b - 1) / sh->b;
    sh->budget = p->budget_blocks; sh->local = p->local_blocks;
    const long long ll = (long long)sh->budget + sh->local + sh->r;
    if (ll * sh->b >= (1ll << 31) || ll > (1 << 24)) return CP_ERR_UNSUPPORTED;
    if ((long long)sh->batch * sh->hq * sh->n1 * ((sh->s + 31) / 32) >= (1ll << 31)) return CP_ERR_UNSUPPORTED;
    sh->list_len = (int)ll;
    sh->dtype = p->dtype;
    const float dflt = 1.0f / std::sqrt((float)p->head_dim);
    sh->attn_scale = p->attn_scale > 0.f ? p->attn_scale : dflt;
    sh->score_scale = p->score_scale > 0.f ? p->score_scale : dflt;
    sh->alpha = p->alpha;
    sh->softmax_domain = p->softmax_domain;
    for (int i = 0; i < 3; ++i) {
        sh->qs[i] = p->q_stride[i]; sh->kvs[i] = p->kv_stride[i]; sh->os[i] = p->o_stride[i];
    }
    return CP_OK;
}

int check_strides(const int64_t* s, int n_tokens_min_stride) {
    for (int i = 0; i < 3; ++i)
        if (s[i] < 0 || (s[i] & 7)) return CP_ERR_ALIGN;
    if (s[2] < n_tokens_min_stride) return CP_ERR_SHAPE;
    return CP_OK;
}

int check_attn(const cp::Shape& sh, const void* q, const void* k, const void* v, const void* out, const float* lse) {
    if (!q || !k || !v || !out) return CP_ERR_NULL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || (lse && !aligned16(lse)))
        return CP_ERR_ALIGN;
    int e;
    if ((e = check_strides(sh.qs, cp::kHeadDim)) != CP_OK) return e;
    if ((e = check_strides(sh.kvs, cp::kHeadDim)) != CP_OK) return e;
    if ((e = check_strides(sh.os, cp::kHeadDim)) != CP_OK) return e;
    if (sh.dtype == CP_DTYPE_BF16) {
        // the bf16 kernel addresses K/V rows with 32-bit byte offsets from the (batch, head) base
        const long long tok_bytes = (long long)sh.kvs[2] * 2;
        if (tok_bytes >= (1 << 24) || sh.n >= (1 << 24) || (long long)sh.n * tok_bytes >= (1ll << 32))
            return CP_ERR_UNSUPPORTED;
    }
    return CP_OK;
}

// workspace of critiprefill_estimate: [Q representatives | K representatives | score statistics]
size_t workspace_layout(const cp::Shape& sh, size_t* krep_offset, size_t* stats_offset) {
    const size_t esz = sh.dtype == CP_DTYPE_BF16 ? 2 : 4;
    size_t qb = (size_t)sh.batch * sh.hq * sh.n1 * 2 * cp::kHeadDim * esz;
    qb = (qb + 255) & ~(size_t)255;
    size_t kb = (size_t)sh.batch * sh.hkv * sh.n2 * 2 * cp::kHeadDim * esz;
    kb = (kb + 255) & ~(size_t)255;
    if (krep_offset) *krep_offset = qb;
    if (stats_offset) *stats_offset = qb + kb;
    return qb + kb + cp::score_stats_bytes(sh);
}

}  // namespace

extern "C" {

int32_t critiprefill_list_len(const critiprefill_params* p) {
    cp::Shape sh;
    const int e = make_shape(p, &sh);
    return e == CP_OK ? sh.list_len : e;
}

size_t critiprefill_workspace_bytes(const critiprefill_params* p) {
    cp::Shape sh;
    if (make_shape(p, &sh) != CP_OK) return 0;
    return workspace_layout(sh, nullptr, nullptr);
}

namespace {
// use_static: the workspace is this device's static scratch (limited to CRITIPREFILL_STATIC_SCRATCH_BYTES)
int estimate_common(const critiprefill_params* p, const void* q, const void* k, const float* prev_scores,
                    float* scores, void* workspace, size_t workspace_bytes, bool use_static, void* hip_stream) {
    cp::Shape sh;
    int e = make_shape(p, &sh);
    if (e != CP_OK) return e;
    if (!q || !k || !scores || (!use_static && !workspace)) return CP_ERR_NULL;
    if (sh.n2 > kMaxBlocks) return CP_ERR_UNSUPPORTED;
    if (sh.dtype == CP_DTYPE_BF16 && (long long)sh.batch * sh.hq > 65535) return CP_ERR_UNSUPPORTED;   // grid.z of the score kernels
    if (!aligned16(q) || !aligned16(k) || !aligned16(scores) || (!use_static && !aligned16(workspace)) ||
        (prev_scores && !aligned16(prev_scores)))
        return CP_ERR_ALIGN;
    if ((e = check_strides(sh.qs, cp::kHeadDim)) != CP_OK) return e;
    if ((e = check_strides(sh.kvs, cp::kHeadDim)) != CP_OK) return e;
    size_t koff = 0, soff = 0;
    const size_t need = workspace_layout(sh, &koff, &soff);
    if (use_static) {
        if (need > (size_t)CRITIPREFILL_STATIC_SCRATCH_BYTES) return CP_ERR_WORKSPACE;
        workspace = static_scratch();
        if (!workspace) return CP_ERR_LAUNCH;
    } else if (workspace_bytes < need) {
        return CP_ERR_WORKSPACE;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    void* qrep = workspace;
    void* krep = (char*)workspace + koff;
    if (cp::launch_pool(sh, q, k, qrep, krep, st) != hipSuccess) return CP_ERR_LAUNCH;
    float* stats = (float*)((char*)workspace + soff);
    if (cp::launch_score(sh, qrep, krep, prev_scores, scores, stats, st) != hipSuccess) return CP_ERR_LAUNCH;
    return CP_OK;
}
}  // namespace

int critiprefill_estimate(const critiprefill_params* p, const void* q, const void* k, const float* prev_scores,
                          float* scores, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return estimate_common(p, q, k, prev_scores, scores, workspace, workspace_bytes, false, hip_stream);
}

int critiprefill_estimate_static(const critiprefill_params* p, const void* q, const void* k,
                                 const float* prev_scores, float* scores, void* hip_stream) {
    return estimate_common(p, q, k, prev_scores, scores, nullptr, 0, true, hip_stream);
}

namespace {
int select_common(const critiprefill_params* p, const float* scores, int32_t* block_idx, int32_t* block_cnt,
                  bool shared, void* hip_stream) {
    cp::Shape sh;
    const int e = make_shape(p, &sh);
    if (e != CP_OK) return e;
    if (!scores || !block_idx || !block_cnt) return CP_ERR_NULL;
    if (sh.n2 > kMaxBlocks) return CP_ERR_UNSUPPORTED;
    if (!aligned16(scores) || !aligned16(block_idx) || !aligned16(block_cnt)) return CP_ERR_ALIGN;
    if (cp::launch_select(sh, scores, block_idx, block_cnt, shared, (hipStream_t)hip_stream) != hipSuccess)
        return CP_ERR_LAUNCH;
    return CP_OK;
}

int sparse_common(const critiprefill_params* p, const void* q, const void* k, const void* v, const int32_t* block_idx,
                  const int32_t* block_cnt, bool shared, void* out, float* lse, void* hip_stream) {
    cp::Shape sh;
    int e = make_shape(p, &sh);
    if (e != CP_OK) return e;
    if (!block_idx || !block_cnt) return CP_ERR_NULL;
    if ((e = check_attn(sh, q, k, v, out, lse)) != CP_OK) return e;
    if (!aligned16(block_idx) || !aligned16(block_cnt)) return CP_ERR_ALIGN;
    if (sh.dtype == CP_DTYPE_BF16 && sh.list_len > cp::kMaxListBf16) return CP_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)hip_stream;
    const hipError_t he = sh.dtype == CP_DTYPE_BF16
                              ? cp::launch_attn_bf16(sh, q, k, v, block_idx, block_cnt, shared, out, lse, st)
                              : cp::launch_attn_fp32(sh, q, k, v, block_idx, block_cnt, shared, out, lse, st);
    return he == hipSuccess ? CP_OK : CP_ERR_LAUNCH;
}
}  // namespace

int critiprefill_select(const critiprefill_params* p, const float* scores, int32_t* block_idx, int32_t* block_cnt,
                        void* hip_stream) {
    return select_common(p, scores, block_idx, block_cnt, false, hip_stream);
}

int critiprefill_select_shared(const critiprefill_params* p, const float* scores, int32_t* block_idx,
                               int32_t* block_cnt, void* hip_stream) {
    return select_common(p, scores, block_idx, block_cnt, true, hip_stream);
}

int critiprefill_sparse_attn(const critiprefill_params* p, const void* q, const void* k, const void* v,
                             const int32_t* block_idx, const int32_t* block_cnt, void* out, float* lse,
                             void* hip_stream) {
    return sparse_common(p, q, k, v, block_idx, block_cnt, false, out, lse, hip_stream);
}

int critiprefill_sparse_attn_shared(const critiprefill_params* p, const void* q, const void* k, const void* v,
                                    const int32_t* block_idx, const int32_t* block_cnt, void* out, float* lse,
                                    void* hip_stream) {
    return sparse_common(p, q, k, v, block_idx, block_cnt, true, out, lse, hip_stream);
}

int critiprefill_dense_causal_attn(const critiprefill_params* p, const void* q, const void* k, const void* v,
                                   void* out, float* lse, void* hip_stream) {
    cp::Shape sh;
    int e = make_shape(p, &sh);
    if (e != CP_OK) return e;
    if ((e = check_attn(sh, q, k, v, out, lse)) != CP_OK) return e;
    hipStream_t st = (hipStream_t)hip_stream;
    const hipError_t he = sh.dtype == CP_DTYPE_BF16
                              ? cp::launch_attn_bf16(sh, q, k, v, nullptr, nullptr, false, out, lse, st)
                              : cp::launch_attn_fp32(sh, q, k, v, nullptr, nullptr, false, out, lse, st);
    return he == hipSuccess ? CP_OK : CP_ERR_LAUNCH;
}

const char* critiprefill_strerror(int status) {
    switch (status) {
        case CP_OK: return "ok";
        case CP_ERR_NULL: return "a required pointer is NULL";
        case CP_ERR_SHAPE: return "invalid shape parameters";
        case CP_ERR_UNSUPPORTED: return "unsupported configuration";
        case CP_ERR_ALIGN: return "pointer or stride alignment";
        case CP_ERR_WORKSPACE: return "workspace too small";
        case CP_ERR_LAUNCH: return "kernel launch failed";
        default: return "unknown status";
    }
}

int critiprefill_version(void) { return 200; }

}  // extern "C"
