/*
 * critiprefill.h - C ABI of the MI355X (gfx950) prefill-attention library.
 *
 * The library runs the CritiPrefill prefill-attention path on one GPU:
 *
 *   critiprefill_estimate          Algorithm 1 "Estimation of Query Criticality in One Layer"
 *   critiprefill_select            Algorithm 2 "Pruned Attention", the argtop_k(S[j], B/block size) step
 *   critiprefill_sparse_attn       Algorithm 2, the per-segment attention loop
 *   critiprefill_select_shared / critiprefill_sparse_attn_shared   the same two steps with one list per KV head
 *   critiprefill_dense_causal_attn Eq. 2 (O = softmax(Q K^T / sqrt(d)) V) with the prefill causal mask
 *
 * Conventions common to all entry points
 * --------------------------------------
 * Pointers: every data pointer is DEVICE memory owned by the caller, 16-byte aligned.  Inputs are
 *   only read; outputs are fully overwritten.  The library allocates and frees nothing.
 * Stream:   `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *   enqueue work on that stream and never synchronise; results are ready when the stream reaches
 *   that point.
 * Layouts:  Q and O are [batch, n_q_heads, seq_len, head_dim], K and V are
 *   [batch, n_kv_heads, seq_len, head_dim]; the strides of the first three axes are given in
 *   ELEMENTS in the parameter block, the channel stride is 1.  Query head h reads K/V head
 *   h / (n_q_heads / n_kv_heads) (the single-head description of the paper extended head by head).
 *   n1 = ceil(seq_len / segment_size) query segments, n2 = ceil(seq_len / block_size) KV blocks,
 *   r = segment_size / block_size blocks under one segment.
 * Errors:   the return value is 0 on success or a negative CP_ERR_* code.  All checks happen before
 *   any kernel is launched; on error no output is touched.  Nothing is printed and nothing throws.
 */
#ifndef CRITIPREFILL_H
#define CRITIPREFILL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    CP_OK = 0,
    CP_ERR_NULL = -1,        /* a required pointer is NULL */
    CP_ERR_SHAPE = -2,       /* non-positive size, n_q_heads % n_kv_heads != 0, block_size does not divide segment_size */
    CP_ERR_UNSUPPORTED = -3, /* head_dim != 128, unknown dtype or softmax_domain, n2 > 8192, list longer than the API allows,
                                bf16 estimate with batch * n_q_heads > 65535 */
    CP_ERR_ALIGN = -4,       /* a pointer is not 16-byte aligned or a stride is not a multiple of 8 elements */
    CP_ERR_WORKSPACE = -5,   /* workspace smaller than critiprefill_workspace_bytes() */
    CP_ERR_LAUNCH = -6       /* the HIP runtime refused a launch */
};

enum { CP_DTYPE_FP32 = 0, CP_DTYPE_BF16 = 1 };

typedef struct critiprefill_params {
    int32_t batch, n_q_heads, n_kv_heads, head_dim; /* head_dim must be 128 */
    int32_t seq_len;                                /* n: queries and keys share positions 0..n-1 (prefill) */
    int32_t segment_size, block_size;               /* s, b; b divides s */
    int32_t budget_blocks;                          /* k = budget tokens / block size (Algorithm 2) */
    int32_t local_blocks;                           /* L blocks just before the segment that are always kept */
    int32_t dtype;                                  /* CP_DTYPE_*: element type of Q, K, V, O */
    float attn_scale;                               /* logit scale of attention; 0 -> 1/sqrt(head_dim) (Eq. 2) */
    float score_scale;                              /* logit scale inside the estimation softmax; 0 -> 1/sqrt(head_dim) */
    float alpha;                                    /* layer fusion S = alpha*S + (1-alpha)*S' (Algorithm 1); used only with prev_scores */
    int32_t softmax_domain;                         /* 0: softmax over all n2 blocks, mask afterwards (listing order); 1: over visible blocks */
    int64_t q_stride[3], kv_stride[3], o_stride[3]; /* elements: batch, head, token */
} critiprefill_params;

/* Length of one block list: budget_blocks + local_blocks + r. */
int32_t critiprefill_list_len(const critiprefill_params *p);

/* Bytes of scratch critiprefill_estimate needs (the max/min representatives of Algorithm 1 and, for bf16,
 * the per-chunk softmax statistics of the score step). */
size_t critiprefill_workspace_bytes(const critiprefill_params *p);

/*
 * Algorithm 1.  Writes scores[batch, n_q_heads, n1, n2] (fp32, contiguous): for every query head the
 * element-wise max/min representatives of each segment and block, the four representative products
 * scaled by score_scale with a row softmax over blocks, S = max((S1+S3)/2, (S2+S4)/2), blocks that
 * lie wholly after the segment set to 0, and, when prev_scores is not NULL, the layer fusion
 * alpha*S + (1-alpha)*prev_scores (prev_scores has the shape of scores; it may alias scores).
 * Values below the smallest normal fp32 are written as 0.
 * q, k: device, dtype per params.  workspace: device, >= critiprefill_workspace_bytes().
 */
int critiprefill_estimate(const critiprefill_params *p, const void *q, const void *k,
                          const float *prev_scores, float *scores,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * critiprefill_estimate for callers that cannot allocate device memory and have no workspace to hand in
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels and
 * the same result, bit for bit, with the scratch in a fixed array inside the library's device image
 * instead of a caller workspace.  Calls no allocating routine.
 * Limit: critiprefill_workspace_bytes(p) must not exceed CRITIPREFILL_STATIC_SCRATCH_BYTES (32 MiB; the five
 * benchmark configurations need 1 to 28 MiB), otherwise CP_ERR_WORKSPACE and nothing is launched.
 * Every GPU the library runs on holds its own copy of the array until the process ends; the device that is
 * current at the call is used (it must be the device of hip_stream).  All calls on one GPU share the array:
 * two calls whose kernels may overlap (different streams, or threads) race; calls on one stream are ordered.
 * Nothing in the array has to start at zero (every value read by a call was written by that call).
 * CP_ERR_LAUNCH if the array's device address cannot be resolved.
 */
#define CRITIPREFILL_STATIC_SCRATCH_BYTES (32u << 20)
int critiprefill_estimate_static(const critiprefill_params *p, const void *q, const void *k,
                                 const float *prev_scores, float *scores, void *hip_stream);

/*
 * Algorithm 2, the top-k line.  For every row (batch, head, segment j) of scores: the candidates are
 * blocks 0 .. j*r - L_j - 1 with L_j = min(local_blocks, j*r); the min(budget_blocks, #candidates)
 * largest scores are kept (ties to the smaller index); the list written to
 * block_idx[batch, n_q_heads, n1, list_len] (int32) is those indices ascending, then the L_j local
 * blocks, then the segment's own blocks; the unused tail is -1 and block_cnt[batch, n_q_heads, n1]
 * (int32) holds the list length.
 */
int critiprefill_select(const critiprefill_params *p, const float *scores,
                        int32_t *block_idx, int32_t *block_cnt, void *hip_stream);

/*
 * Algorithm 2, the attention loop, all segments in one launch.  Query t of segment j attends to the
 * tokens u <= t of the blocks listed in block_idx[batch, head, j, 0..block_cnt-1] (any strictly
 * ascending list of block indices < n2 is accepted; row pitch critiprefill_list_len()).
 * out has the dtype and strides (o_stride) of the parameter block.  lse (nullable) receives
 * log(sum exp(scaled logits)) per query, fp32 [batch, n_q_heads, seq_len]; a query with no visible
 * key gets output 0 and lse -inf.
 */
int critiprefill_sparse_attn(const critiprefill_params *p, const void *q, const void *k, const void *v,
                             const int32_t *block_idx, const int32_t *block_cnt,
                             void *out, float *lse, void *hip_stream);

/*
 * Extension of the paper's single-head description (it gives no rule for sharing a list between heads):
 * ONE list per (batch, KV head, segment) for all query heads of that KV head, taken from the element-wise
 * maximum of their scores.  critiprefill_select_shared reads scores[batch, n_q_heads, n1, n2] and writes
 * block_idx[batch, n_kv_heads, n1, list_len] / block_cnt[batch, n_kv_heads, n1] by the same rule as
 * critiprefill_select applied to max over the group's heads; critiprefill_sparse_attn_shared is
 * critiprefill_sparse_attn reading those lists (query head h uses the list of KV head
 * h / (n_q_heads / n_kv_heads)).  Same argument checks and errors as the per-head entry points.
 */
int critiprefill_select_shared(const critiprefill_params *p, const float *scores,
                               int32_t *block_idx, int32_t *block_cnt, void *hip_stream);
int critiprefill_sparse_attn_shared(const critiprefill_params *p, const void *q, const void *k, const void *v,
                                    const int32_t *block_idx, const int32_t *block_cnt,
                                    void *out, float *lse, void *hip_stream);

/* Eq. 2 with the causal mask u <= t: the dense baseline.  Same tensors as sparse_attn, no lists. */
int critiprefill_dense_causal_attn(const critiprefill_params *p, const void *q, const void *k, const void *v,
                                   void *out, float *lse, void *hip_stream);

const char *critiprefill_strerror(int status);
int critiprefill_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CRITIPREFILL_H */
