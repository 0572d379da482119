// Kernel-level C entry points (include/rlhf_ops.h): thin argument checks around the launchers.
#include "../../include/rlhf_ops.h"

#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/rlhf.h"
#include "kernels.h"

using namespace rlhf;

// Split-KV partials of rlhf_op_paged_decode_attention_noalloc: per (row, query head, split) one
// float accumulator of up to 128 dims, then the (max, sum) pairs.  One copy per GPU, held until
// the process ends; its device address is looked up once per device.
constexpr size_t kNoAllocSlots = 16384;
constexpr size_t kNoAllocMaxHd = 128;
static __device__ __align__(256) float scratch[kNoAllocSlots * (kNoAllocMaxHd + 2)];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
float* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (the array's name is only a host-side
// handle; every GPU has its own copy at its own address).
int scratch_of_current_device(float** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        set_global_error("rlhf_op_paged_decode_attention_noalloc: cannot identify the current device");
        return RLHF_EDEVICE;
    }
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            set_global_error("rlhf_op_paged_decode_attention_noalloc: hipGetSymbolAddress failed");
            return RLHF_EDEVICE;
        }
        g_scratch_ptr[dev] = (float*)p;
    }
    *out = g_scratch_ptr[dev];
    return RLHF_OK;
}
}  // namespace

static int status_of(hipError_t e) {
    if (e == hipSuccess) return RLHF_OK;
    return e == hipErrorInvalidValue ? RLHF_EINVAL : RLHF_EDEVICE;
}

extern "C" int rlhf_op_gemm_nsplit(int dtype, int M, int N, int K, int max_split) {
    if (M <= 0 || N <= 0 || K <= 0 || max_split < 1) return 1;
    return gemm_choose_nsplit(dtype == RLHF_BF16 ? kBF16 : kF32, M, N, K, max_split);
}

extern "C" int rlhf_op_gemm(int dtype, int act_half, const void* A, const void* W, float* C, int M, int N,
                            int K, int nsplit, int variant, void* stream) {
    if (!A || !W || !C || M < 0 || N < 0 || K <= 0 || nsplit < 1) return RLHF_EINVAL;
    if (dtype == 2) {        // W is a half copy of a bf16 matrix (rlhf_op_bf16_to_half), A is half
        if (!act_half) return RLHF_EINVAL;
        return status_of(launch_gemm((hipStream_t)stream, kF16, kF16, A, W, C, M, N, K, nsplit, variant));
    }
    if (dtype != RLHF_BF16 && dtype != RLHF_FP32) return RLHF_EINVAL;
    if (act_half && dtype != RLHF_BF16) return RLHF_EINVAL;
    const int wdt = dtype == RLHF_BF16 ? kBF16 : kF32;
    return status_of(launch_gemm((hipStream_t)stream, wdt, act_half ? kF16 : wdt, A, W, C, M, N, K, nsplit, variant));
}

extern "C" int rlhf_op_paged_decode_attention(int dtype, const void* q, const void* pool,
                                              const int32_t* page_table, int pt_stride,
                                              const int32_t* row_sample, const int32_t* ctx_len, void* out,
                                              float* part_acc, float* part_ml, int rows, int layer, int nsplit,
                                              int n_layers, int n_q_heads, int n_kv_heads, int head_dim,
                                              void* stream) {
    if (!q || !pool || !page_table || !row_sample || !ctx_len || !out || rows < 0 || nsplit < 1 ||
        layer < 0 || layer >= n_layers || n_kv_heads <= 0 || n_q_heads % n_kv_heads)
        return RLHF_EINVAL;
    if (nsplit > 1 && (!part_acc || !part_ml)) return RLHF_EINVAL;
    Dims dm{n_layers, n_q_heads * head_dim, n_q_heads, n_kv_heads, head_dim, 0, 0, 16};
    const int dt = dtype == 2 ? kF16 : dtype == RLHF_BF16 ? kBF16 : kF32;
    return status_of(launch_decode_attn((hipStream_t)stream, dt, q, pool,
                                        page_table, pt_stride, row_sample, ctx_len, out, part_acc, part_ml,
                                        rows, layer, nsplit, dm));
}

extern "C" int rlhf_op_paged_decode_attention_noalloc(int dtype, const void* q, const void* pool,
                                                      const int32_t* page_table, int pt_stride,
                                                      const int32_t* row_sample, const int32_t* ctx_len,
                                                      void* out, int rows, int layer, int nsplit, int n_layers,
                                                      int n_q_heads, int n_kv_heads, int head_dim, void* stream) {
    if (!q || !pool || !page_table || !row_sample || !ctx_len || !out || rows < 0 || nsplit < 1 ||
        layer < 0 || layer >= n_layers || n_kv_heads <= 0 || n_q_heads <= 0 || n_q_heads % n_kv_heads) {
        set_global_error("rlhf_op_paged_decode_attention_noalloc: bad argument");
        return RLHF_EINVAL;
    }
    const size_t slots = (size_t)rows * n_q_heads * nsplit;
    if (head_dim <= 0 || (size_t)head_dim > kNoAllocMaxHd || slots > kNoAllocSlots) {
        set_global_error("rlhf_op_paged_decode_attention_noalloc: rows * n_q_heads * nsplit must not exceed 16384 "
                         "and head_dim must not exceed 128 (the size of the built-in scratch)");
        return RLHF_EINVAL;
    }
    float* sc = nullptr;
    const int rc = scratch_of_current_device(&sc);
    if (rc != RLHF_OK) return rc;
    float* part_acc = sc;                                   // [slots][head_dim]
    float* part_ml = sc + kNoAllocSlots * kNoAllocMaxHd;    // [slots][2]
    Dims dm{n_layers, n_q_heads * head_dim, n_q_heads, n_kv_heads, head_dim, 0, 0, 16};
    const int dt = dtype == 2 ? kF16 : dtype == RLHF_BF16 ? kBF16 : kF32;
    const hipError_t e = launch_decode_attn((hipStream_t)stream, dt, q, pool, page_table, pt_stride, row_sample,
                                            ctx_len, out, part_acc, part_ml, rows, layer, nsplit, dm);
    if (e != hipSuccess) set_global_error("rlhf_op_paged_decode_attention_noalloc: unsupported shape or launch failure");
    return status_of(e);
}

extern "C" int rlhf_op_varlen_attention(int out_half, const float* q, const float* k, const float* v,
                                        const int32_t* row_start, const int32_t* row_pos, void* out,
                                        int rows, int n_q_heads, int n_kv_heads, int head_dim, void* stream) {
    if (!q || !k || !v || !row_start || !row_pos || !out || rows < 0 || n_kv_heads <= 0 ||
        n_q_heads % n_kv_heads)
        return RLHF_EINVAL;
    Dims dm{1, n_q_heads * head_dim, n_q_heads, n_kv_heads, head_dim, 0, 0, 16};
    return status_of(launch_prefill_attn((hipStream_t)stream, out_half ? kF16 : kF32, q, k, v, row_start,
                                         row_pos, out, rows, dm));
}

extern "C" int rlhf_op_flash_attention(const void* q, const void* k, const void* v, const int32_t* tile_start,
                                       const int32_t* tile_q0, const int32_t* tile_len, void* out, int n_tiles,
                                       int rows, int n_q_heads, int n_kv_heads, int head_dim, void* stream) {
    if (!q || !k || !v || !tile_start || !tile_q0 || !tile_len || !out || n_tiles < 0 || rows <= 0 ||
        n_kv_heads <= 0 || n_q_heads % n_kv_heads)
        return RLHF_EINVAL;
    Dims dm{1, n_q_heads * head_dim, n_q_heads, n_kv_heads, head_dim, 0, 0, 16};
    return status_of(launch_flash_attn((hipStream_t)stream, q, k, v, tile_start, tile_q0, tile_len, out, n_tiles,
                                       rows, dm));
}

extern "C" int rlhf_op_gemm_swiglu(int act_half, const void* A, const void* W_gate_up, void* act, int M, int ffn,
                                   int K, void* stream) {
    if (!A || !W_gate_up || !act) return RLHF_EINVAL;
    const int adt = act_half ? kF16 : kBF16, wdt = act_half == 2 ? kF16 : kBF16;
    if (M >= 1 && M <= 16) {            // the few-row kernel of decode steps (no K split, SwiGLU in its epilogue)
        if (!gemm_rows16_supported(wdt, adt, M, K) || ffn <= 0 || ffn % 8) return RLHF_EINVAL;
        RowsEpi ep;
        ep.act = act;
        ep.ffn = ffn;
        return status_of(launch_gemm_rows16((hipStream_t)stream, wdt, adt, 1, A, W_gate_up, nullptr, M, 2 * ffn, K, ep));
    }
    if (!gemm_swiglu_supported(wdt, adt, M, ffn, K)) return RLHF_EINVAL;
    return status_of(launch_gemm_swiglu((hipStream_t)stream, wdt, adt, A, W_gate_up, act, M, ffn, K));
}

extern "C" int rlhf_op_gemm_rope(int act_half, const void* A, const void* W_qkv, const int32_t* pos,
                                 const int32_t* kv_dst, const float* table, void* q, void* k, void* v, void* pool,
                                 int M, int K, int layer, int n_layers, int n_q_heads, int n_kv_heads, int head_dim,
                                 void* stream) {
    if (!A || !W_qkv || !pos || !table || !q || (pool && !kv_dst) || n_q_heads <= 0 || n_kv_heads <= 0 ||
        n_q_heads % n_kv_heads || layer < 0 || layer >= n_layers)
        return RLHF_EINVAL;
    const int adt = act_half ? kF16 : kBF16, wdt = act_half == 2 ? kF16 : kBF16;
    Dims dm{n_layers, K, n_q_heads, n_kv_heads, head_dim, 0, 0, 16};
    RopeOut ro;
    ro.pos = pos; ro.kv_dst = kv_dst; ro.table = table;
    ro.q = q; ro.k = k; ro.v = v; ro.pool = pool;
    ro.layer = layer; ro.n_layers = n_layers;
    ro.n_q_heads = n_q_heads; ro.n_kv_heads = n_kv_heads; ro.head_dim = head_dim;
    if (M >= 1 && M <= 16) {            // the few-row kernel of decode steps (no K split, rotary in its epilogue)
        if (!gemm_rows16_supported(wdt, adt, M, K) || (head_dim != 64 && head_dim != 128)) return RLHF_EINVAL;
        RowsEpi ep;
        ep.ro = ro;
        return status_of(launch_gemm_rows16((hipStream_t)stream, wdt, adt, 2, A, W_qkv, nullptr, M,
                                            (n_q_heads + 2 * n_kv_heads) * head_dim, K, ep));
    }
    if (!gemm_rope_supported(wdt, adt, M, K, dm)) return RLHF_EINVAL;
    return status_of(launch_gemm_rope((hipStream_t)stream, wdt, adt, A, W_qkv, M, K, ro));
}

// ---- row-wise kernels

static int act_of(int act_dtype) { return act_dtype == 2 ? kF16 : act_dtype == RLHF_BF16 ? kBF16 : act_dtype == RLHF_FP32 ? kF32 : -1; }

extern "C" int rlhf_op_rmsnorm(int act_dtype, float* h, const float* part, int nsplit, int64_t sstride,
                               const int32_t* row_idx, const float* g, void* xn, int rows, int d, float eps,
                               void* stream) {
    const int adt = act_of(act_dtype);
    if (adt < 0 || !h || !g || !xn || rows < 0 || d <= 0 || nsplit < 0 || (nsplit > 0 && (!part || sstride < 0)))
        return RLHF_EINVAL;
    return status_of(launch_rmsnorm((hipStream_t)stream, adt, h, part, nsplit, (size_t)sstride, row_idx, g, xn, rows,
                                    d, eps));
}

extern "C" int rlhf_op_rope_kv(int act_dtype, const float* qkv, int nsplit, int64_t sstride, const int32_t* pos,
                               const int32_t* kv_dst, const float* table, void* q, void* k, void* v, void* pool,
                               int layer, int rows, int n_layers, int n_q_heads, int n_kv_heads, int head_dim,
                               void* stream) {
    const int adt = act_of(act_dtype);
    if (adt < 0 || !qkv || !pos || !table || !q || nsplit < 1 || sstride < 0 || rows < 0 || (pool && !kv_dst) ||
        n_q_heads <= 0 || n_kv_heads <= 0 || head_dim <= 0 || head_dim % 2 || layer < 0 || layer >= n_layers)
        return RLHF_EINVAL;
    Dims dm{n_layers, n_q_heads * head_dim, n_q_heads, n_kv_heads, head_dim, 0, 0, 16};
    return status_of(launch_rope_kv((hipStream_t)stream, adt, adt, qkv, nsplit, (size_t)sstride, pos, kv_dst, table,
                                    q, k, v, pool, layer, rows, dm));
}

extern "C" int rlhf_op_swiglu(int act_dtype, const float* gu, int nsplit, int64_t sstride, void* act, int rows,
                              int ffn, void* stream) {
    const int adt = act_of(act_dtype);
    if (adt < 0 || !gu || !act || nsplit < 1 || sstride < 0 || rows < 0 || ffn <= 0) return RLHF_EINVAL;
    return status_of(launch_swiglu((hipStream_t)stream, adt, gu, nsplit, (size_t)sstride, act, rows, ffn));
}

extern "C" int64_t rlhf_op_pick_scratch_floats(int rows) { return rows > 0 ? (int64_t)pick_scratch_floats(rows) : 0; }

extern "C" int rlhf_op_pick(const float* logits, int nsplit, int64_t sstride, int rows, int vocab,
                            const int32_t* forced, int32_t* tokens, const int32_t* tok_dst, float* lp,
                            const int32_t* lp_dst, int32_t* picked, float* scratch, void* stream) {
    if (!logits || !tokens || !tok_dst || !lp || !lp_dst || !scratch || nsplit < 1 || sstride < 0 || rows < 0 ||
        vocab < 1)
        return RLHF_EINVAL;
    return status_of(launch_pick((hipStream_t)stream, logits, nsplit, (size_t)sstride, rows, vocab, forced, tokens,
                                 tok_dst, lp, lp_dst, picked, scratch));
}

extern "C" int rlhf_op_gather_lp(const float* logits, int nsplit, int64_t sstride, int rows, int vocab,
                                 const int32_t* tokens, const int32_t* target_idx, float* out,
                                 const int32_t* out_dst, void* stream) {
    if (!logits || !tokens || !target_idx || !out || !out_dst || nsplit < 1 || sstride < 0 || rows < 0 || vocab < 1)
        return RLHF_EINVAL;
    return status_of(launch_gather_lp((hipStream_t)stream, logits, nsplit, (size_t)sstride, rows, vocab, tokens,
                                      target_idx, out, out_dst));
}

extern "C" int rlhf_op_head_dot(int act_dtype, int w_dtype, const void* xn, const void* w, int rows, int d,
                                float* out, const int32_t* out_dst, void* stream) {
    const int adt = act_of(act_dtype);
    if (adt < 0 || (w_dtype != RLHF_FP32 && w_dtype != RLHF_BF16) || !xn || !w || !out || !out_dst || rows < 0 ||
        d <= 0 || d % 8)
        return RLHF_EINVAL;
    return status_of(launch_head_dot((hipStream_t)stream, adt, w_dtype == RLHF_BF16 ? kBF16 : kF32, xn, w, rows, d,
                                     out, out_dst));
}

extern "C" int64_t rlhf_op_lm_head_logprob_scratch_floats(int M, int vocab) {
    if (M <= 0 || vocab <= 0) return 0;
    return (int64_t)M * (2 * gemm_lse_partials(vocab) + 1);
}

extern "C" int rlhf_op_lm_head_logprob(int act_half, const void* A, const void* W_head, const int32_t* tokens,
                                       const int32_t* target_idx, float* out, const int32_t* out_dst,
                                       float* scratch, int M, int vocab, int K, void* stream) {
    if (!A || !W_head || !tokens || !target_idx || !out || !out_dst || !scratch || M < 0 || vocab < 1 || K <= 0)
        return RLHF_EINVAL;
    const int adt = act_half ? kF16 : kBF16, wdt = act_half == 2 ? kF16 : kBF16;
    if (!gemm_lse_supported(wdt, adt, K)) return RLHF_EINVAL;
    LseOut lo;
    lo.n_part = gemm_lse_partials(vocab);
    lo.tokens = tokens;
    lo.target_idx = target_idx;
    lo.part_max = scratch;
    lo.part_sum = scratch + (size_t)M * lo.n_part;
    lo.tgt = scratch + (size_t)2 * M * lo.n_part;
    hipError_t e = launch_gemm_lse((hipStream_t)stream, wdt, adt, A, W_head, M, vocab, K, lo);
    if (e == hipSuccess)
        e = launch_lse_merge((hipStream_t)stream, lo.part_max, lo.part_sum, lo.tgt, lo.n_part, M, out, out_dst);
    return status_of(e);
}

extern "C" int rlhf_op_bf16_to_half(const void* src, void* dst, int64_t n, void* stream) {
    if (!src || !dst || n < 0 || n % 2) return RLHF_EINVAL;
    return status_of(launch_bf16_to_half((hipStream_t)stream, src, dst, (size_t)n));
}

extern "C" int rlhf_op_gemm_tall_grid(int tiles_m, int tiles_n) {
    return tiles_m > 0 && tiles_n > 0 ? gemm_tall_grid(tiles_m, tiles_n) : 0;
}

extern "C" int rlhf_op_gemm_tall_tile(int bid, int tiles_m, int tiles_n, int* tm, int* tn) {
    if (bid < 0 || tiles_m <= 0 || tiles_n <= 0 || !tm || !tn) return RLHF_EINVAL;
    return gemm_tall_tile(bid, tiles_m, tiles_n, tm, tn) ? 1 : 0;
}
