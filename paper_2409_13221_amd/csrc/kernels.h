// Host-callable launchers of the HIP kernels.  Every launcher validates nothing: the engine
// checks shapes and bounds on the host before it launches (see engine.cpp).  All pointers are
// device pointers.  "nsplit / sstride": a float input that is the sum of nsplit partial
// buffers, partial s at x + s * sstride (split-K GEMM output consumed without a reduce pass).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace rlhf {

// Storage types.  Weights are kF32 or kBF16.  With bf16 weights every activation fed to the
// matrix units and the KV pool are kF16: IEEE half keeps 11 significant bits against bf16's 8,
// and the bf16 weights convert to half exactly on their way into LDS.  (The kernels also accept
// bf16 activations and a bf16 pool; the engine does not use them.)
enum DType { kF32 = 0, kBF16 = 1, kF16 = 2 };

struct Dims {
    int n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    int page_tokens;
};

// ---- GEMM: C[s][m][n] = sum over k in split s of A[m][k] * W[n][k];  C float, split stride M*N
// (wdt, adt) in {(kF32,kF32), (kBF16,kBF16), (kBF16,kF16)}
int gemm_choose_nsplit(int wdt, int M, int N, int K, int max_split);
// wdt == kF16 (with adt == kF16, K a multiple of 64): W is a half copy of a bf16 matrix, made with
// launch_bf16_to_half; the 256 x 256 tiling then loads both operands global -> LDS directly.  The
// fused-epilogue launchers below accept it too.  gemm_is_tall: the shapes launch_gemm runs with that tiling.
bool gemm_is_tall(int M, int N, int K, int nsplit);
int gemm_tall_grid(int tiles_m, int tiles_n);                                  // workgroups launched for a tile grid
bool gemm_tall_tile(int bid, int tiles_m, int tiles_n, int* tm, int* tn);      // false: the workgroup has no tile
hipError_t launch_bf16_to_half(hipStream_t st, const void* src, void* dst, size_t n_elements);
// variant 0 = the tiling chosen from M; > 0 forces one (tuning / benchmarks).
hipError_t launch_gemm(hipStream_t st, int wdt, int adt, const void* A, const void* W, float* C,
                       int M, int N, int K, int nsplit, int variant = 0);

// Gate||up projection with SwiGLU fused into the epilogue (tall passes of bf16 models):
// act[m][c] = silu(<A[m], W[c]>) * <A[m], W[ffn + c]>, written as adt [M, ffn].
bool gemm_swiglu_supported(int wdt, int adt, int M, int ffn, int K);
hipError_t launch_gemm_swiglu(hipStream_t st, int wdt, int adt, const void* A, const void* W_gate_up,
                              void* act, int M, int ffn, int K);

// QKV projection of a tall pass with rotary embedding, type conversion and the scatter to q / k / v
// (and to the paged pool, if given) in the epilogue: replaces launch_gemm + launch_rope_kv there.
// Element type of q, k, v, pool = adt.  k, v may be NULL (nothing but the pool wants them).
struct RopeOut {
    const int* pos = nullptr;       // [M] rotary position of each row
    const int* kv_dst = nullptr;    // [M] page * page_tokens + offset (needed with pool)
    const float* table = nullptr;   // [max_pos][head_dim/2][cos, sin]
    void* q = nullptr;              // [M, Hq*hd]
    void* k = nullptr;              // [M, Hkv*hd] or NULL
    void* v = nullptr;
    void* pool = nullptr;           // paged KV pool or NULL
    int layer = 0, n_layers = 0, n_q_heads = 0, n_kv_heads = 0, head_dim = 0, page_tokens = 16;
};
bool gemm_rope_supported(int wdt, int adt, int M, int K, const Dims& dm);
hipError_t launch_gemm_rope(hipStream_t st, int wdt, int adt, const void* A, const void* Wqkv, int M, int K,
                            const RopeOut& ro);

// Few rows (1..16), bf16 weights: a kernel whose workgroups walk the whole K range (no split), so that
// the step that consumes the projection rides in its epilogue and needs no launch of its own.
// mode 0: C float [M, N]; mode 1: gate||up with SwiGLU, act [M, ffn] of type adt (N = 2 ffn);
// mode 2: QKV with rotary embedding and the q / k / v / paged-pool scatter (ep.ro as in launch_gemm_rope).
// K must be a multiple of 256.  Mode 0 may also split K (nsplit float planes, (K / 64) a multiple of
// 4 * nsplit).
struct RowsEpi {
    void* act = nullptr;       // mode 1
    int ffn = 0;
    RopeOut ro;                // mode 2
};
bool gemm_rows16_supported(int wdt, int adt, int M, int K);
hipError_t launch_gemm_rows16(hipStream_t st, int wdt, int adt, int mode, const void* A, const void* W, float* C,
                              int M, int N, int K, const RowsEpi& ep, int nsplit = 1);

// LM head of a scoring pass fused with the log-softmax gather: the logits stay in registers.  Per
// row m the GEMM leaves n_part = gemm_lse_partials(N) pairs (max, sum of exp(z - max)), one per 128
// columns (a pair whose columns all lie beyond N is (-inf, 0)), and the logit of the row's target
// token tokens[target_idx[m]] in tgt[m]; launch_lse_merge finishes
// out[out_dst[m]] = tgt[m] - log sum_n exp(z[m][n]).
struct LseOut {
    const int* tokens = nullptr;       // token buffer
    const int* target_idx = nullptr;   // [M] index into tokens of each row's target
    float* part_max = nullptr;         // [M, n_part]
    float* part_sum = nullptr;         // [M, n_part]
    float* tgt = nullptr;              // [M]
    int n_part = 0;
};
bool gemm_lse_supported(int wdt, int adt, int K);
int gemm_lse_partials(int N);
hipError_t launch_gemm_lse(hipStream_t st, int wdt, int adt, const void* A, const void* W_head, int M, int N, int K,
                           const LseOut& lo);
hipError_t launch_lse_merge(hipStream_t st, const float* part_max, const float* part_sum, const float* tgt,
                            int n_part, int rows, float* out, const int* out_dst, int* nonfinite = nullptr);

// ---- elementwise / row kernels
hipError_t launch_embed(hipStream_t st, int dtype, const int* tokens, const int* tok_idx,
                        const void* table, float* h, int rows, int d, int vocab);
// v = h[src] + sum partials[src];  (row_idx == NULL: src = r and h[src] = v is written back)
// xn[r] = v * rsqrt(mean(v^2) + eps) * g
hipError_t launch_rmsnorm(hipStream_t st, int adt, float* h, const float* part, int nsplit,
                          size_t sstride, const int* row_idx, const float* g, void* xn, int rows,
                          int d, float eps);
// Rotary on Q and K heads of qkv rows.  q_out [rows, Hq*hd] and, if non-NULL, k_out/v_out
// [rows, Hkv*hd] have type qdt; if pool != NULL and kv_dst[r] >= 0, K/V of row r also go (as
// type pdt) to token slot kv_dst[r] (= page * page_tokens + offset) of `layer` in the paged pool.
// (qdt, pdt) in {(kF32,kF32), (kBF16,kBF16), (kF16,kF16)}.
hipError_t launch_rope_kv(hipStream_t st, int qdt, int pdt, const float* qkv, int nsplit, size_t sstride,
                          const int* pos, const int* kv_dst, const float* rope_table,
                          void* q_out, void* k_out, void* v_out, void* pool, int layer,
                          int rows, const Dims& dm);
hipError_t launch_swiglu(hipStream_t st, int adt, const float* gu, int nsplit, size_t sstride,
                         void* act, int rows, int ffn);
// Greedy choice per logit row (lowest id on ties), optional imposed token forced[r] >= 0;
// writes the emitted token to tokens[tok_dst[r]] and picked[r], its log-prob to lp[lp_dst[r]].
// nonfinite (here and below, may be NULL): *nonfinite is set to 1 when a written result is not finite.
// scratch: pick_scratch_floats(rows) floats.
hipError_t launch_pick(hipStream_t st, const float* logits, int nsplit, size_t sstride, int rows,
                       int vocab, const int* forced, int* tokens, const int* tok_dst, float* lp,
                       const int* lp_dst, int* picked, float* scratch, int* nonfinite = nullptr);
size_t pick_scratch_floats(int rows);
// lp[out_dst[r]] = log_softmax(logits[r])[tokens[target_idx[r]]]
hipError_t launch_gather_lp(hipStream_t st, const float* logits, int nsplit, size_t sstride,
                            int rows, int vocab, const int* tokens, const int* target_idx,
                            float* out, const int* out_dst, int* nonfinite = nullptr);
// out[out_dst[r]] = <xn[r], w>;  xn of type adt (or float), w of type wdt
hipError_t launch_head_dot(hipStream_t st, int adt, int wdt, const void* xn, const void* w, int rows,
                           int d, float* out, const int* out_dst, int* nonfinite = nullptr);
hipError_t launch_noop(hipStream_t st);   // empty kernel (calibrates event brackets)
// page_table[upd_idx[i]] = upd_val[i]
hipError_t launch_scatter_int(hipStream_t st, int* dst, const int* idx, const int* val, int n);

// ---- GAE as one matrix multiply: D = delta (zero-padded [n, Lp]), U[t][s] = (gamma lam)^(s-t)
hipError_t launch_gae_delta(hipStream_t st, const float* lp_actor, const float* lp_ref, const float* values,
                            const float* reward, const int* gen_len, int stride, float gamma, float kl_coef,
                            float* D, int n, int Lp);
hipError_t launch_gae_matrix(hipStream_t st, float* U, int Lp, double gamma_lam);
hipError_t launch_gae_returns(hipStream_t st, const float* A, const float* values, const int* gen_len,
                              int stride, float* R, int n, int Lp);

// ---- attention
// Decode: one query row per active sample against its paged K/V.  q [rows, Hq*hd]; out the same.
// row_sample[r] selects the page-table row; ctx_len[r] keys are visible.  part_* hold split
// partials when nsplit > 1 (sizes rows*Hq*nsplit*(hd or 1)).
hipError_t launch_decode_attn(hipStream_t st, int dtype, const void* q, const void* pool,
                              const int* page_table, int pt_stride, const int* row_sample,
                              const int* ctx_len, void* out, float* part_acc, float* part_ml,
                              int rows, int layer, int nsplit, const Dims& dm);
// Prefill / scoring: packed varlen causal attention over contiguous float q [T,Hq*hd], k, v
// [T,Hkv*hd]; out has type odt; row r belongs to the sequence starting at row_start[r] and sits at position
// row_pos[r] in it (sees keys row_start[r] .. row_start[r] + row_pos[r]).
hipError_t launch_prefill_attn(hipStream_t st, int odt, const float* q, const float* k,
                               const float* v, const int* row_start, const int* row_pos,
                               void* out, int rows, const Dims& dm);

// The same on the matrix units for bf16 models: q, k, v, out IEEE half.  The queries are cut
// into tiles of kFlashTile rows that never straddle a sequence: tile i covers rows
// tile_start[i] + tile_q0[i] .. of the sequence that starts at row tile_start[i] and has
// tile_len[i] rows.  T_total = rows of the packed buffers (loads are clamped to it).
constexpr int kFlashTile = 128;
hipError_t launch_flash_attn(hipStream_t st, const void* q, const void* k, const void* v,
                             const int* tile_start, const int* tile_q0, const int* tile_len, void* out,
                             int n_tiles, int T_total, const Dims& dm);

size_t pool_page_elems(const Dims& dm);  // elements of one page over all layers

// Error text of a call without a context; rlhf_last_error(NULL) returns it (per thread).
void set_global_error(const char* msg);

}  // namespace rlhf
