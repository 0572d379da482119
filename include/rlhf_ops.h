/*
 * rlhf_ops.h -- kernel-level entry points of the same library, for per-kernel parity tests
 * and roofline measurements.  The stage API in rlhf.h is built from exactly these kernels.
 *
 * All pointers are DEVICE pointers owned by the caller; `stream` is a hipStream_t (NULL =
 * the default stream).  Calls enqueue work and return without waiting.  Return values are
 * rlhf_status codes (0 = OK, RLHF_EINVAL for unsupported shapes, RLHF_EDEVICE for a failed
 * launch).  dtype is an rlhf_dtype: the storage type of the weights.
 */
#ifndef RLHF_OPS_H
#define RLHF_OPS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Linear projection y = W x of a decoder block (the matrix work of both the memory-bound
 * decoding phase, Section 4.2, and the prefill-like inference forward, Section 2.1):
 * C[s][m][n] = sum over the s-th K range of A[m][k] * W[n][k].  W [N,K] row-major in dtype;
 * A [M,K] in dtype, or (act_half != 0, bf16 weights only) in IEEE half, the activation type
 * of prefill / scoring passes; C float32 [nsplit][M][N]; the caller sums the nsplit partial
 * planes.  K must be a multiple of 8 (bf16) or 4 (fp32).  variant 0 takes the tiling the
 * stage uses for M rows; a positive value forces one of the library's tilings (benchmarks;
 * RLHF_EINVAL if it does not exist or cannot split K).  rlhf_op_gemm_nsplit returns the split
 * the stage itself would choose for this shape, at most max_split. */
int rlhf_op_gemm_nsplit(int dtype, int M, int N, int K, int max_split);
int rlhf_op_gemm(int dtype, int act_half, const void* A, const void* W, float* C, int M, int N, int K,
                 int nsplit, int variant, void* stream);

/* Gate||up projection of the SwiGLU MLP with the activation fused into the epilogue, as the
 * stage runs it in prefill / scoring passes: act[m][c] = silu(<A[m], W[c]>) * <A[m], W[ffn + c]>.
 * W_gate_up bf16 [2*ffn, K] (gate rows, then up rows); A and act IEEE half (act_half != 0) or
 * bf16, [M, K] and [M, ffn].  Needs M >= 512, ffn and K multiples of 8 (else RLHF_EINVAL). */
int rlhf_op_gemm_swiglu(int act_half, const void* A, const void* W_gate_up, void* act, int M, int ffn, int K,
                        void* stream);

/* QKV projection of a prefill / scoring pass with the rotary embedding fused into the epilogue,
 * as the stage runs it for bf16 models (Section 2.1, the attention input of a decoder block):
 * row m of A [M, K] (IEEE half if act_half != 0, else bf16) times W_qkv bf16
 * [(n_q_heads + 2*n_kv_heads)*head_dim, K] (query rows, key rows, value rows); query and key
 * heads are rotated by position pos[m] (pair (i, i + head_dim/2), cosine and sine taken from
 * table, float32 [max position][head_dim/2][cos, sin]); results are rounded to A's type and
 * written to q [M, n_q_heads*head_dim] and, where non-NULL, to k, v [M, n_kv_heads*head_dim] and
 * to the paged pool (layout as in rlhf_op_paged_decode_attention) at token slot kv_dst[m] =
 * page*16 + offset.  Needs M >= 512, K a multiple of 64, head_dim 64 or 128 (else RLHF_EINVAL). */
int rlhf_op_gemm_rope(int act_half, const void* A, const void* W_qkv, const int32_t* pos, const int32_t* kv_dst,
                      const float* table, void* q, void* k, void* v, void* pool, int M, int K, int layer,
                      int n_layers, int n_q_heads, int n_kv_heads, int head_dim, void* stream);

/* Decode attention of one step (Section 2.1, decoding phase): row r holds one query
 * [n_q_heads * head_dim] and attends to the ctx_len[r] cached tokens of the sample whose
 * page-table row is row_sample[r].  pool layout: [page][layer][K|V][kv_head][16][head_dim].
 * Here dtype is the element type of q, pool and out: RLHF_FP32, RLHF_BF16, or 2 = IEEE half
 * (what the stage uses for bf16 models).
 * part_acc / part_ml are float32 scratch of rows*n_q_heads*nsplit*head_dim and
 * rows*n_q_heads*nsplit*2 entries (unused when nsplit == 1). */
int rlhf_op_paged_decode_attention(int dtype, const void* q, const void* pool, const int32_t* page_table,
                                   int pt_stride, const int32_t* row_sample, const int32_t* ctx_len,
                                   void* out, float* part_acc, float* part_ml, int rows, int layer,
                                   int nsplit, int n_layers, int n_q_heads, int n_kv_heads, int head_dim,
                                   void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same decode attention with the split-KV partials
 * kept in a scratch array built into the library instead of caller-supplied part_acc / part_ml.
 * The call allocates nothing.  Limits: rows * n_q_heads * nsplit <= 16384 and head_dim <= 128
 * (the scratch is 16384 * 130 floats = 8.1 MiB per GPU, held until the process ends); beyond them
 * RLHF_EINVAL, with the reason available from rlhf_last_error(NULL).  All calls on one GPU share
 * that scratch: two such calls whose work overlaps in time on one GPU (different streams or
 * threads) race; calls ordered on one stream are safe.  Same kernels, same results as
 * rlhf_op_paged_decode_attention for the same nsplit. */
int rlhf_op_paged_decode_attention_noalloc(int dtype, const void* q, const void* pool, const int32_t* page_table,
                                           int pt_stride, const int32_t* row_sample, const int32_t* ctx_len,
                                           void* out, int rows, int layer, int nsplit, int n_layers,
                                           int n_q_heads, int n_kv_heads, int head_dim, void* stream);

/* Packed variable-length causal attention of the prefill / inference forward (Section 2.1):
 * float32 q [T, n_q_heads*head_dim], k, v [T, n_kv_heads*head_dim]; row r belongs to the
 * sequence that starts at row row_start[r] and is its row_pos[r]-th token.  out is IEEE half
 * (out_half != 0) or float32. */
int rlhf_op_varlen_attention(int out_half, const float* q, const float* k, const float* v,
                             const int32_t* row_start, const int32_t* row_pos, void* out, int rows,
                             int n_q_heads, int n_kv_heads, int head_dim, void* stream);

/* The same attention on the matrix units, as used for bf16 models: q, k, v, out IEEE half.
 * Queries are cut into tiles of 128 rows that do not straddle sequences: tile i covers rows
 * tile_start[i] + tile_q0[i] .. (at most 128, up to the end) of the sequence that starts at
 * row tile_start[i] and has tile_len[i] rows.  rows = rows of the packed buffers.
 * head_dim must be 64 or 128. */
int rlhf_op_flash_attention(const void* q, const void* k, const void* v, const int32_t* tile_start,
                            const int32_t* tile_q0, const int32_t* tile_len, void* out, int n_tiles,
                            int rows, int n_q_heads, int n_kv_heads, int head_dim, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RLHF_OPS_H */
