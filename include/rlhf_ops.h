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
/* Half copies of the weights: rlhf_op_bf16_to_half converts n (even) bf16 elements to IEEE half the
 * way the kernels do on the fly (exact for magnitudes >= 2^-14, toward zero on half's subnormal
 * grid below).  With such a copy as W, rlhf_op_gemm takes dtype = 2 (A must be half, K a multiple
 * of 64; the 256 x 256 tiling with both operands loaded global -> LDS directly, any nsplit whose
 * ranges are non-empty; A and W each smaller than 4 GiB, since the loads address them with 32-bit
 * byte offsets, else RLHF_EINVAL), and rlhf_op_gemm_swiglu / rlhf_op_gemm_rope /
 * rlhf_op_lm_head_logprob take act_half = 2 under the same conditions.  This is what the stage runs in prefill / scoring passes when the engine option
 * half_weight_copies is set; results are bit-identical to the bf16-weight path. */
int rlhf_op_bf16_to_half(const void* src, void* dst, int64_t n, void* stream);
int rlhf_op_gemm_nsplit(int dtype, int M, int N, int K, int max_split);
int rlhf_op_gemm(int dtype, int act_half, const void* A, const void* W, float* C, int M, int N, int K,
                 int nsplit, int variant, void* stream);

/* Host-side copy of the workgroup -> tile mapping of the compute-bound (256 x 256) launches, for
 * tests of that mapping: rlhf_op_gemm_tall_grid is the number of workgroups launched for a grid of
 * tiles_m x tiles_n tiles; rlhf_op_gemm_tall_tile returns 1 and the tile (*tm, *tn) workgroup bid
 * computes, 0 if it has none, RLHF_EINVAL on bad arguments.  The 8 XCDs (bid modulo 8) walk the same
 * panel of 8 tile rows at the same time, each over a contiguous group of tile columns of its own. */
int rlhf_op_gemm_tall_grid(int tiles_m, int tiles_n);
int rlhf_op_gemm_tall_tile(int bid, int tiles_m, int tiles_n, int* tm, int* tn);

/* Gate||up projection of the SwiGLU MLP with the activation fused into the epilogue, as the
 * stage runs it in prefill / scoring passes: act[m][c] = silu(<A[m], W[c]>) * <A[m], W[ffn + c]>.
 * W_gate_up bf16 [2*ffn, K] (gate rows, then up rows); A and act IEEE half (act_half != 0) or
 * bf16, [M, K] and [M, ffn].  Needs M >= 512, ffn and K multiples of 8 (else RLHF_EINVAL); or
 * 1 <= M <= 16 and K a multiple of 256: the few-row kernel of decode steps, whose workgroups walk
 * the whole K range (no split) so that SwiGLU can ride in the epilogue there too. */
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
 * page*16 + offset.  Needs M >= 512, K a multiple of 64, head_dim 64 or 128 (else RLHF_EINVAL); or
 * 1 <= M <= 16 and K a multiple of 256: the few-row kernel of decode steps (no K split, rotary and
 * the KV-cache append in its epilogue). */
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

/* ---- row-wise kernels of the decoder block and of the heads.  act_dtype is the element type of
 * the 16-bit (or float) activations a kernel writes or reads: RLHF_FP32, RLHF_BF16, or 2 = IEEE
 * half.  "nsplit / sstride": a float input given as nsplit partial planes, plane s at x + s *
 * sstride elements (the split-K output of rlhf_op_gemm, summed in plane order by the consumer). */

/* RMSNorm of a decoder block (the reading of "LLaMA", Section 7: y = x * rsqrt(mean(x^2) + eps) * g,
 * statistics in float), fused with the residual add: v = h[src] + sum of the partial planes at
 * row src; xn[r] = norm(v) * g.  row_idx == NULL: src = r and v is written back to h (the residual
 * stream); otherwise src = row_idx[r] and h is left alone.  d a multiple of 8, at most 8192;
 * nsplit in [0, 16] (0: no planes). */
int rlhf_op_rmsnorm(int act_dtype, float* h, const float* part, int nsplit, int64_t sstride,
                    const int32_t* row_idx, const float* g, void* xn, int rows, int d, float eps, void* stream);

/* Rotary embedding and KV-cache append of decode steps and short passes: qkv [rows, (Hq + 2 Hkv)
 * * hd] float planes; query and key heads are rotated by pos[r] (pair (i, i + hd/2); table float32
 * [max position][hd/2][cos, sin]); q [rows, Hq*hd] and, if non-NULL, k, v [rows, Hkv*hd] are
 * written in act_dtype, and k, v also to token slot kv_dst[r] = page*16 + offset of `layer` in
 * the paged pool when pool != NULL (layout as in rlhf_op_paged_decode_attention). */
int rlhf_op_rope_kv(int act_dtype, const float* qkv, int nsplit, int64_t sstride, const int32_t* pos,
                    const int32_t* kv_dst, const float* table, void* q, void* k, void* v, void* pool,
                    int layer, int rows, int n_layers, int n_q_heads, int n_kv_heads, int head_dim,
                    void* stream);

/* SwiGLU of decode steps: gu [rows, 2*ffn] float planes (gate columns, then up columns);
 * act[r][c] = silu(gate) * up in act_dtype.  ffn a multiple of 8. */
int rlhf_op_swiglu(int act_dtype, const float* gu, int nsplit, int64_t sstride, void* act, int rows, int ffn,
                   void* stream);

/* Greedy choice of the generation stage (Section 2.1; lowest id on ties) over float logit planes
 * [rows, vocab]: token y = argmax (or forced[r] if forced != NULL and forced[r] >= 0) is written to
 * tokens[tok_dst[r]] (and picked[r] if non-NULL) and log_softmax(logits[r])[y] to lp[lp_dst[r]].
 * scratch: rlhf_op_pick_scratch_floats(rows) floats. */
int64_t rlhf_op_pick_scratch_floats(int rows);
int rlhf_op_pick(const float* logits, int nsplit, int64_t sstride, int rows, int vocab, const int32_t* forced,
                 int32_t* tokens, const int32_t* tok_dst, float* lp, const int32_t* lp_dst, int32_t* picked,
                 float* scratch, void* stream);

/* Log-prob of given tokens (inference stage, Section 2.1): out[out_dst[r]] =
 * log_softmax(logits[r])[tokens[target_idx[r]]]. */
int rlhf_op_gather_lp(const float* logits, int nsplit, int64_t sstride, int rows, int vocab,
                      const int32_t* tokens, const int32_t* target_idx, float* out, const int32_t* out_dst,
                      void* stream);

/* LM head of the inference stage fused with the log-softmax gather (Section 2.1: the Reference
 * and Actor log-probabilities of the generated tokens), as the stage runs it for bf16 models: for
 * row m of A [M, K] (IEEE half if act_half != 0, else bf16) and W_head bf16 [vocab, K],
 *   out[out_dst[m]] = log_softmax(W_head A[m])[tokens[target_idx[m]]]
 * without the [M, vocab] logits ever being written: the GEMM's epilogue keeps, per row and per 128
 * vocabulary columns, the maximum and the sum of exponentials, and a merge kernel finishes.
 * scratch: rlhf_op_lm_head_logprob_scratch_floats(M, vocab) floats.  K a multiple of 64. */
int64_t rlhf_op_lm_head_logprob_scratch_floats(int M, int vocab);
int rlhf_op_lm_head_logprob(int act_half, const void* A, const void* W_head, const int32_t* tokens,
                            const int32_t* target_idx, float* out, const int32_t* out_dst, float* scratch, int M,
                            int vocab, int K, void* stream);

/* Value / reward head (Section 2.1: the Critic evaluates each action, the Reward model scores the
 * sample): out[out_dst[r]] = <xn[r], w>, xn [rows, d] in act_dtype, w [d] in w_dtype (RLHF_FP32 or
 * RLHF_BF16).  Supported pairs: (fp32, fp32), (fp32, bf16), (half, bf16), (bf16, bf16). */
int rlhf_op_head_dot(int act_dtype, int w_dtype, const void* xn, const void* w, int rows, int d, float* out,
                     const int32_t* out_dst, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RLHF_OPS_H */
