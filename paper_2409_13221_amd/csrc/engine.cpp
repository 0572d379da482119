// Host side of the fused generation + inference stage: the C ABI of include/rlhf.h, the
// continuous-batching bookkeeping (admission against the KV budget, page tables, retirement,
// scoring-batch formation) and the launch sequences of the decode step and of the prefill /
// scoring forward.  All arithmetic of the method runs in the HIP kernels declared in
// kernels.h; this file only decides what to launch, on which stream, over which rows.
#include "../../include/rlhf.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <deque>
#include <string>
#include <vector>

#include "kernels.h"

using namespace rlhf;

namespace {

thread_local char g_create_error[512] = "";

struct RoleWeights {
    bool bound = false;
    rlhf_weights w{};
    // IEEE-half copies of the bf16 matrices for the tall (prefill / scoring) passes, owned by the
    // library (engine option half_weight_copies); NULL members: no copy, the bf16 tensor is used
    rlhf_weights h16{};
    std::vector<void*> owned;
};

// Pinned host staging + one device arena for small per-pass integer metadata.  The host runs
// ahead of the device, so host slots form a ring guarded by events; the device arena is
// rewritten by a stream-ordered copy, after the kernels of the previous pass on that stream.
struct MetaRing {
    static constexpr int kSlots = 8;
    int* host[kSlots] = {};
    hipEvent_t ev[kSlots] = {};
    bool used[kSlots] = {};
    int* dev = nullptr;
    size_t cap = 0;
    int next = 0;

    hipError_t init(size_t cap_ints) {
        cap = cap_ints;
        hipError_t e = hipMalloc((void**)&dev, cap * sizeof(int));
        if (e != hipSuccess) return e;
        for (int i = 0; i < kSlots; ++i) {
            e = hipHostMalloc((void**)&host[i], cap * sizeof(int), hipHostMallocDefault);
            if (e != hipSuccess) return e;
            e = hipEventCreateWithFlags(&ev[i], hipEventDisableTiming);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    void destroy() {
        for (int i = 0; i < kSlots; ++i) {
            if (host[i]) (void)hipHostFree(host[i]);
            if (ev[i]) (void)hipEventDestroy(ev[i]);
        }
        if (dev) (void)hipFree(dev);
    }
    hipError_t begin(int** out) {
        if (used[next]) {
            hipError_t e = hipEventSynchronize(ev[next]);
            if (e != hipSuccess) return e;
        }
        *out = host[next];
        return hipSuccess;
    }
    hipError_t commit(hipStream_t st, size_t n_ints) {
        hipError_t e = hipMemcpyAsync(dev, host[next], n_ints * sizeof(int), hipMemcpyHostToDevice, st);
        if (e != hipSuccess) return e;
        e = hipEventRecord(ev[next], st);
        used[next] = true;
        next = (next + 1) % kSlots;
        return e;
    }
};

struct Workspace {
    int rows_cap = 0;
    float* h = nullptr;       // [rows, d] residual stream (float)
    void* xn = nullptr;       // [rows, d] normed activations (storage type)
    float* part = nullptr;    // split-K partial outputs of the GEMM in flight
    size_t part_cap = 0;      // floats
    void* q = nullptr;        // [rows, Hq*hd]
    void* k = nullptr;        // [rows, Hkv*hd] (batch passes)
    void* v = nullptr;
    void* attn = nullptr;     // [rows, Hq*hd]
    void* act = nullptr;      // [rows, ffn]
    void* xsel = nullptr;     // [rows, d] final-norm rows selected for the head (storage type; float for d -> 1 heads)
    float* logits = nullptr;  // [logit_rows, vocab] (batch passes; decode uses `part`)
    int logit_rows = 0;
    float* pick_scratch = nullptr;  // per-chunk partial results of the greedy pick
    float* attn_acc = nullptr;  // decode split-KV partials
    float* attn_ml = nullptr;
    size_t attn_slots = 0;
    std::vector<void*> owned;
};

// Optional per-kernel-class timing: every `every`-th launch of a class is bracketed by two
// events on its stream; algorithmic bytes / flops of the sampled launches are summed beside.
enum KClass { kGemmDecode = 0, kGemmBatch = 1, kAttnDecode = 2, kAttnBatch = 3, kClassCount = 4 };

struct Profiler {
    bool on = false;
    int every = 1;
    // Event pairs in flight.  rlhf_run_stage folds them into the sums below once the stage has
    // drained, so the cap bounds the samples of ONE stage; launches beyond it go untimed and are
    // counted in `dropped` (a caller who sees dropped > 0 should raise sample_every).
    static constexpr size_t kMaxSamples = 1 << 16;
    struct Rec { hipEvent_t a, b; int cls; double bytes, flops; };
    std::vector<Rec> recs;                 // recs[0..n_used) are live; events are reused across runs
    size_t n_used = 0;
    int64_t launches[kClassCount] = {};
    double tot_bytes[kClassCount] = {}, tot_flops[kClassCount] = {};
    int64_t sampled[kClassCount] = {}, dropped[kClassCount] = {};
    double bracket_overhead_ms = 0;        // cost of an event bracket beyond its kernels, measured at begin
    double s_ms[kClassCount] = {}, s_bytes[kClassCount] = {}, s_flops[kClassCount] = {};
};

struct Sample {
    int P = 0, max_new = 0, target = 0, reserve = 0;
    int ctx = 0, gen_len = 0, admit_step = -1;
    bool has_forced_len = false, finished = false, retired = false;
    std::vector<int> pages;
};

}  // namespace

struct rlhf_ctx {
    rlhf_model_cfg mc{};
    rlhf_engine_cfg ec{};
    Dims dm{};
    int dtype = 0, esz = 2;
    int max_pages = 0, pool_pages = 0;
    char err[512] = "";

    hipStream_t sd = nullptr, ss = nullptr;            // the streams decode / scoring work goes to NOW
    hipStream_t sd_full = nullptr, ss_full = nullptr;  // whole chip
    hipStream_t sd_part = nullptr, ss_part = nullptr;  // disjoint CU masks for co-running (optional)
    bool own_sd = false, own_ss = false;
    hipEvent_t ev_sw_d = nullptr, ev_sw_s = nullptr, ev_score_last = nullptr;
    hipEvent_t ev_dep = nullptr;                       // decode -> score dependency
    hipEvent_t ev_d0 = nullptr, ev_d1 = nullptr, ev_s0 = nullptr, ev_s1 = nullptr;
    std::vector<hipEvent_t> step_events;

    RoleWeights roles[4];

    void* pool = nullptr;
    int* d_page_table = nullptr;   // [max_samples, max_pages]
    int* d_tokens = nullptr;       // [max_samples, max_ctx]   prompt + response
    float* d_lp_actor = nullptr;   // [max_samples, max_ctx]   indexed by output index j-1
    float* d_lp_rescored = nullptr;
    float* d_lp_ref = nullptr;
    float* d_values = nullptr;
    float* d_reward = nullptr;     // [max_samples]
    float* d_rope = nullptr;       // [max_ctx, hd/2, 2]
    int* d_nonfinite = nullptr;    // set by the kernels that write results when one is not finite
    int* d_picked = nullptr;       // [max_active] tokens of the last pick (stop_on_eos)
    int* h_picked = nullptr;       // pinned

    Workspace ws_dec, ws_pre, ws_score;
    MetaRing meta_dec, meta_pre, meta_score;
    Profiler prof;

    // ---- stage state (host integers)
    int N = 0;
    std::vector<Sample> smp;
    std::vector<int> h_prompt;            // packed prompts
    std::vector<int64_t> h_prompt_off;
    std::vector<int> h_forced;            // [N * max_ctx] imposed token per output index, -1 = free
    std::deque<int> waiting;
    std::vector<int> active;
    std::vector<int> free_list;
    int reserved = 0;
    std::vector<int> retired;
    size_t n_scored = 0;
    std::vector<int> batch_offsets{0};
    std::vector<int> batch_step;
    int step = 0;
    bool score_used = false;
    int64_t acc_weight_bytes = 0, acc_kv_bytes = 0, acc_prefill_tokens = 0;

    int fail(int code, const char* fmt, ...) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(err, sizeof err, fmt, ap);
        va_end(ap);
        return code;
    }
};

#define HIPCK(ctx, call)                                                                       \
    do {                                                                                       \
        hipError_t e_ = (call);                                                                \
        if (e_ != hipSuccess)                                                                  \
            return (ctx)->fail(RLHF_EDEVICE, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), \
                               __FILE__, __LINE__);                                            \
    } while (0)

namespace {

int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Run `launch` (a callable returning hipError_t), timing it if this launch is sampled.
template <typename F>
hipError_t profiled(rlhf_ctx* c, hipStream_t st, int cls, double bytes, double flops, F&& launch) {
    Profiler& p = c->prof;
    if (!p.on) return launch();
    const int64_t k = p.launches[cls]++;
    p.tot_bytes[cls] += bytes;
    p.tot_flops[cls] += flops;
    if (k % p.every != 0) return launch();
    if (p.n_used >= Profiler::kMaxSamples) { p.dropped[cls] += 1; return launch(); }
    if (p.n_used == p.recs.size()) {
        Profiler::Rec r{};
        hipError_t e = hipEventCreate(&r.a);
        if (e != hipSuccess) return e;
        e = hipEventCreate(&r.b);
        if (e != hipSuccess) return e;
        p.recs.push_back(r);
    }
    Profiler::Rec& r = p.recs[p.n_used++];
    r.cls = cls;
    r.bytes = bytes;
    r.flops = flops;
    hipError_t e = hipEventRecord(r.a, st);
    if (e != hipSuccess) return e;
    e = launch();
    if (e != hipSuccess) return e;
    return hipEventRecord(r.b, st);
}

// Fold the finished event pairs into the per-class sums (both streams must have drained).
hipError_t profiler_fold(Profiler& p) {
    for (size_t i = 0; i < p.n_used; ++i) {
        float ms = 0.f;
        hipError_t e = hipEventElapsedTime(&ms, p.recs[i].a, p.recs[i].b);
        if (e != hipSuccess) return e;
        const int k = p.recs[i].cls;
        p.sampled[k] += 1;
        p.s_ms[k] += ms;
        p.s_bytes[k] += p.recs[i].bytes;
        p.s_flops[k] += p.recs[i].flops;
    }
    p.n_used = 0;
    return hipSuccess;
}

// Activation and KV-pool type: float for a float model, IEEE half for a bf16 model.
int act_type(const rlhf_ctx* c, bool /*batch*/) { return c->dtype == kBF16 ? kF16 : kF32; }

hipError_t gemm_profiled(rlhf_ctx* c, hipStream_t st, int cls, int adt, const void* A, const void* W, float* C,
                         int M, int N, int K, int nsplit, bool w_is_half_copy = false) {
    const double bytes = ((double)N * K + (double)M * K) * c->esz + (double)M * N * 4;
    return profiled(c, st, cls, bytes, 2.0 * M * N * K,
                    [&] { return launch_gemm(st, w_is_half_copy ? kF16 : c->dtype, adt, A, W, C, M, N, K, nsplit); });
}

template <typename T>
hipError_t dev_alloc(Workspace* ws, T** p, size_t n_bytes) {
    void* q = nullptr;
    hipError_t e = hipMalloc(&q, n_bytes ? n_bytes : 256);
    if (e == hipSuccess) {
        *p = (T*)q;
        if (ws) ws->owned.push_back(q);
    }
    return e;
}

int alloc_workspace(rlhf_ctx* c, Workspace& ws, int rows, bool decode) {
    const rlhf_model_cfg& m = c->mc;
    const size_t d = m.d_model, qd = (size_t)m.n_q_heads * m.head_dim, kvd = (size_t)m.n_kv_heads * m.head_dim;
    const size_t qkv_w = qd + 2 * kvd, f = m.ffn, V = m.vocab, es = c->esz;
    ws.rows_cap = rows;
    const size_t widest = std::max({qkv_w, 2 * f, d});
    if (decode) {
        // room for split-K partials of few-row GEMMs and for [rows, vocab] logits
        ws.part_cap = std::max((size_t)rows * std::max(widest, V) * 2, (size_t)16 * 16 * std::max(widest, V));
        ws.attn_slots = std::max((size_t)rows * m.n_q_heads, (size_t)16384);
    } else {
        ws.part_cap = (size_t)rows * widest;
        ws.logit_rows = std::min(rows, 2048);
    }
    HIPCK(c, dev_alloc(&ws, &ws.h, rows * d * 4));
    HIPCK(c, dev_alloc(&ws, (char**)&ws.xn, rows * d * es));
    HIPCK(c, dev_alloc(&ws, &ws.part, ws.part_cap * 4));
    HIPCK(c, dev_alloc(&ws, (char**)&ws.q, rows * qd * es));
    HIPCK(c, dev_alloc(&ws, (char**)&ws.attn, rows * qd * es));
    HIPCK(c, dev_alloc(&ws, (char**)&ws.act, rows * f * es));
    HIPCK(c, dev_alloc(&ws, (char**)&ws.xsel, rows * d * 4));    // float rows for the value / reward head
    HIPCK(c, dev_alloc(&ws, &ws.pick_scratch, pick_scratch_floats(rows) * 4));
    if (decode) {
        HIPCK(c, dev_alloc(&ws, &ws.attn_acc, ws.attn_slots * m.head_dim * 4));
        HIPCK(c, dev_alloc(&ws, &ws.attn_ml, ws.attn_slots * 2 * 4));
    } else {
        HIPCK(c, dev_alloc(&ws, (char**)&ws.k, rows * kvd * es));
        HIPCK(c, dev_alloc(&ws, (char**)&ws.v, rows * kvd * es));
        HIPCK(c, dev_alloc(&ws, &ws.logits, (size_t)ws.logit_rows * V * 4));
    }
    return RLHF_OK;
}

void free_workspace(Workspace& ws) {
    for (void* p : ws.owned) (void)hipFree(p);
    ws.owned.clear();
}

const char* layer_ptr(const void* base, int layer, size_t rows, size_t cols, int esz) {
    return (const char*)base + (size_t)layer * rows * cols * esz;
}

int nsplit_for(const rlhf_ctx* c, const Workspace& ws, int M, int N, int K) {
    const size_t per = (size_t)M * N;
    int cap = (int)std::min<size_t>(16, per ? ws.part_cap / per : 1);
    if (cap < 1) cap = 1;
    return gemm_choose_nsplit(c->dtype, M, N, K, cap);
}

enum AttnMode { kModeDecode, kModeBatch };

struct PassMeta {         // device pointers into a MetaRing arena
    const int* tok_idx = nullptr;
    const int* pos = nullptr;
    const int* kv_dst = nullptr;       // NULL: no pool writes
    const int* row_sample = nullptr;   // decode
    const int* ctx_len = nullptr;      // decode
    const int* row_start = nullptr;    // batch (float models)
    const int* tile_start = nullptr;   // batch (bf16 models): query tiles of the MFMA attention
    const int* tile_q0 = nullptr;
    const int* tile_len = nullptr;
    int n_tiles = 0;
    double attn_bytes = 0, attn_flops = 0;   // algorithmic, per layer (for the profiler)
};

// Embedding and all decoder layers over `rows` rows.  On return ws.h holds the residual
// stream except for the last down-projection, whose split-K partials are still in ws.part:
// (*pend_ns, *pend_stride) describe them for the final norm.
int forward_layers(rlhf_ctx* c, hipStream_t st, Workspace& ws, const RoleWeights& rw, int rows,
                   const PassMeta& pm, AttnMode mode, int attn_nsplit, int* pend_ns,
                   size_t* pend_stride) {
    const rlhf_weights& w = rw.w;
    const rlhf_weights& wh = rw.h16;              // half copies (members may be NULL)
    const rlhf_model_cfg& m = c->mc;
    const int d = m.d_model, qd = m.n_q_heads * m.head_dim, kvd = m.n_kv_heads * m.head_dim;
    const int qkv_w = qd + 2 * kvd, f = m.ffn, es = c->esz, dt = c->dtype;
    const int gcls = mode == kModeDecode ? kGemmDecode : kGemmBatch;
    const int adt = act_type(c, mode == kModeBatch);
    const int qdt = adt;               // q/k/v of a pass share the activation type
    HIPCK(c, launch_embed(st, dt, c->d_tokens, pm.tok_idx, w.embed, ws.h, rows, d, m.vocab));
    int pns = 0;
    size_t pstride = 0;
    for (int l = 0; l < m.n_layers; ++l) {
        HIPCK(c, launch_rmsnorm(st, adt, ws.h, ws.part, pns, pstride, nullptr, w.g_attn + (size_t)l * d,
                                ws.xn, rows, d, m.rms_eps));
        int ns = 0;
        const bool few = gemm_rows16_supported(dt, adt, rows, d) && (m.head_dim == 64 || m.head_dim == 128);
        if (few) {
            // up to 16 rows: the projection walks the whole K range, rotary + KV append ride in its epilogue
            RowsEpi ep;
            ep.ro.pos = pm.pos;
            ep.ro.kv_dst = pm.kv_dst;
            ep.ro.table = c->d_rope;
            ep.ro.q = ws.q;
            ep.ro.k = mode == kModeBatch ? ws.k : nullptr;
            ep.ro.v = mode == kModeBatch ? ws.v : nullptr;
            ep.ro.pool = pm.kv_dst ? c->pool : nullptr;
            ep.ro.layer = l; ep.ro.n_layers = m.n_layers;
            ep.ro.n_q_heads = m.n_q_heads; ep.ro.n_kv_heads = m.n_kv_heads; ep.ro.head_dim = m.head_dim;
            ep.ro.page_tokens = c->ec.page_tokens;
            const double bytes = ((double)qkv_w * d + (double)rows * d) * es + (double)rows * qkv_w * es;
            const void* wq = layer_ptr(w.wqkv, l, qkv_w, d, es);
            HIPCK(c, profiled(c, st, gcls, bytes, 2.0 * rows * qkv_w * d, [&] {
                return launch_gemm_rows16(st, dt, adt, 2, ws.xn, wq, nullptr, rows, qkv_w, d, ep);
            }));
        } else if (mode == kModeBatch && gemm_rope_supported(dt, adt, rows, d, c->dm)) {
            // tall pass: rotary, rounding and the q / k / v / pool scatter ride in the GEMM's epilogue
            RopeOut ro;
            ro.pos = pm.pos;
            ro.kv_dst = pm.kv_dst;
            ro.table = c->d_rope;
            ro.q = ws.q; ro.k = ws.k; ro.v = ws.v;
            ro.pool = pm.kv_dst ? c->pool : nullptr;
            ro.layer = l; ro.n_layers = m.n_layers;
            ro.n_q_heads = m.n_q_heads; ro.n_kv_heads = m.n_kv_heads; ro.head_dim = m.head_dim;
            ro.page_tokens = c->ec.page_tokens;
            const double bytes = ((double)qkv_w * d + (double)rows * d) * es + (double)rows * qkv_w * es;
            const bool hw = wh.wqkv && adt == kF16;
            const void* wq = layer_ptr(hw ? wh.wqkv : w.wqkv, l, qkv_w, d, es);
            HIPCK(c, profiled(c, st, gcls, bytes, 2.0 * rows * qkv_w * d,
                              [&] { return launch_gemm_rope(st, hw ? kF16 : dt, adt, ws.xn, wq, rows, d, ro); }));
        } else {
            ns = nsplit_for(c, ws, rows, qkv_w, d);
            HIPCK(c, gemm_profiled(c, st, gcls, adt, ws.xn, layer_ptr(w.wqkv, l, qkv_w, d, es), ws.part, rows, qkv_w, d, ns));
            HIPCK(c, launch_rope_kv(st, qdt, adt, ws.part, ns, (size_t)rows * qkv_w, pm.pos, pm.kv_dst, c->d_rope,
                                    ws.q, mode == kModeBatch ? ws.k : nullptr,
                                    mode == kModeBatch ? ws.v : nullptr, pm.kv_dst ? c->pool : nullptr, l,
                                    rows, c->dm));
        }
        if (mode == kModeDecode) {
            HIPCK(c, profiled(c, st, kAttnDecode, pm.attn_bytes, pm.attn_flops, [&] {
                return launch_decode_attn(st, adt, ws.q, c->pool, c->d_page_table, c->max_pages, pm.row_sample,
                                          pm.ctx_len, ws.attn, ws.attn_acc, ws.attn_ml, rows, l, attn_nsplit,
                                          c->dm);
            }));
        } else {
            HIPCK(c, profiled(c, st, kAttnBatch, pm.attn_bytes, pm.attn_flops, [&] {
                if (adt == kF16)
                    return launch_flash_attn(st, ws.q, ws.k, ws.v, pm.tile_start, pm.tile_q0, pm.tile_len, ws.attn,
                                             pm.n_tiles, rows, c->dm);
                return launch_prefill_attn(st, adt, (const float*)ws.q, (const float*)ws.k, (const float*)ws.v,
                                           pm.row_start, pm.pos, ws.attn, rows, c->dm);
            }));
        }
        ns = nsplit_for(c, ws, rows, d, qd);
        {
            const bool hw = wh.wo && adt == kF16 && mode == kModeBatch && gemm_is_tall(rows, d, qd, ns);
            HIPCK(c, gemm_profiled(c, st, gcls, adt, ws.attn, layer_ptr(hw ? wh.wo : w.wo, l, d, qd, es), ws.part, rows,
                                   d, qd, ns, hw));
        }
        HIPCK(c, launch_rmsnorm(st, adt, ws.h, ws.part, ns, (size_t)rows * d, nullptr,
                                w.g_mlp + (size_t)l * d, ws.xn, rows, d, m.rms_eps));
        if (few && f % 8 == 0) {
            RowsEpi ep;
            ep.act = ws.act;
            ep.ffn = f;
            const void* wgu = layer_ptr(w.w_gate_up, l, 2 * (size_t)f, d, es);
            const double bytes = (2.0 * f * d + (double)rows * d) * es + (double)rows * f * es;
            HIPCK(c, profiled(c, st, gcls, bytes, 4.0 * rows * f * d, [&] {
                return launch_gemm_rows16(st, dt, adt, 1, ws.xn, wgu, nullptr, rows, 2 * f, d, ep);
            }));
        } else if (gemm_swiglu_supported(dt, adt, rows, f, d)) {
            const bool hw = wh.w_gate_up && adt == kF16 && d % 64 == 0;
            const void* wgu = layer_ptr(hw ? wh.w_gate_up : w.w_gate_up, l, 2 * (size_t)f, d, es);
            const double bytes = (2.0 * f * d + (double)rows * d) * es + (double)rows * f * es;
            HIPCK(c, profiled(c, st, gcls, bytes, 4.0 * rows * f * d,
                              [&] { return launch_gemm_swiglu(st, hw ? kF16 : dt, adt, ws.xn, wgu, ws.act, rows, f, d); }));
        } else {
            ns = nsplit_for(c, ws, rows, 2 * f, d);
            HIPCK(c, gemm_profiled(c, st, gcls, adt, ws.xn, layer_ptr(w.w_gate_up, l, 2 * (size_t)f, d, es), ws.part,
                                   rows, 2 * f, d, ns));
            HIPCK(c, launch_swiglu(st, adt, ws.part, ns, (size_t)rows * 2 * f, ws.act, rows, f));
        }
        pns = nsplit_for(c, ws, rows, d, f);
        pstride = (size_t)rows * d;
        {
            const bool hw = wh.w_down && adt == kF16 && mode == kModeBatch && gemm_is_tall(rows, d, f, pns);
            HIPCK(c, gemm_profiled(c, st, gcls, adt, ws.act, layer_ptr(hw ? wh.w_down : w.w_down, l, d, f, es), ws.part,
                                   rows, d, f, pns, hw));
        }
    }
    *pend_ns = pns;
    *pend_stride = pstride;
    return RLHF_OK;
}

}  // namespace

// =========================================================================== create/destroy

extern "C" const char* rlhf_last_error(const rlhf_ctx* ctx) { return ctx ? ctx->err : g_create_error; }

// Message of a failed call that has no context (rlhf_create, the kernel-level entry points);
// read back with rlhf_last_error(NULL) on the same thread.
void rlhf::set_global_error(const char* msg) { snprintf(g_create_error, sizeof g_create_error, "%s", msg); }

extern "C" void rlhf_destroy(rlhf_ctx* c) {
    if (!c) return;
    for (hipStream_t st : {c->sd_full, c->ss_full, c->sd_part, c->ss_part})
        if (st) (void)hipStreamSynchronize(st);
    free_workspace(c->ws_dec);
    free_workspace(c->ws_pre);
    free_workspace(c->ws_score);
    for (RoleWeights& r : c->roles) {
        for (void* p : r.owned) (void)hipFree(p);
        r.owned.clear();
    }
    c->meta_dec.destroy();
    c->meta_pre.destroy();
    c->meta_score.destroy();
    void* bufs[] = {c->pool, c->d_page_table, c->d_tokens, c->d_lp_actor, c->d_lp_rescored, c->d_lp_ref,
                    c->d_values, c->d_reward, c->d_rope, c->d_picked, c->d_nonfinite};
    for (void* p : bufs)
        if (p) (void)hipFree(p);
    if (c->h_picked) (void)hipHostFree(c->h_picked);
    hipEvent_t evs[] = {c->ev_dep, c->ev_d0, c->ev_d1, c->ev_s0, c->ev_s1, c->ev_sw_d, c->ev_sw_s, c->ev_score_last};
    for (hipEvent_t e : evs)
        if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->step_events) (void)hipEventDestroy(e);
    for (auto& r : c->prof.recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    if (c->own_sd && c->sd_full) (void)hipStreamDestroy(c->sd_full);
    if (c->own_ss && c->ss_full) (void)hipStreamDestroy(c->ss_full);
    if (c->sd_part) (void)hipStreamDestroy(c->sd_part);
    if (c->ss_part) (void)hipStreamDestroy(c->ss_part);
    delete c;
}

static int create_impl(rlhf_ctx* c) {
    const rlhf_model_cfg& m = c->mc;
    const rlhf_engine_cfg& e = c->ec;
    if (m.n_layers < 0 || m.d_model <= 0 || m.n_q_heads <= 0 || m.n_kv_heads <= 0 || m.ffn <= 0 || m.vocab <= 1)
        return c->fail(RLHF_EINVAL, "model dimensions must be positive");
    if (m.dtype != RLHF_FP32 && m.dtype != RLHF_BF16) return c->fail(RLHF_EINVAL, "dtype must be FP32 or BF16");
    if (m.d_model % 8 || m.ffn % 8 || m.d_model > 8192)
        return c->fail(RLHF_EINVAL, "d_model and ffn must be multiples of 8, d_model <= 8192");
    if (m.n_q_heads % m.n_kv_heads) return c->fail(RLHF_EINVAL, "n_q_heads must be a multiple of n_kv_heads");
    const int G = m.n_q_heads / m.n_kv_heads;
    const bool attn_ok = (m.head_dim == 128 && (G == 1 || (G == 8 && m.dtype == RLHF_BF16))) ||
                         (m.head_dim == 64 && G == 1);
    if (!attn_ok)
        return c->fail(RLHF_EINVAL, "unsupported attention shape: head_dim %d, group %d (have 128x{1,8}, 64x1)",
                       m.head_dim, G);
    if (e.page_tokens != 16) return c->fail(RLHF_EINVAL, "page_tokens must be 16");
    if (e.max_samples <= 0 || e.max_ctx <= 1 || e.max_active <= 0 || e.max_batch_tokens < e.max_ctx)
        return c->fail(RLHF_EINVAL, "engine limits: need max_samples, max_active > 0, max_batch_tokens >= max_ctx > 1");
    if (e.eos_id < 0 || e.eos_id >= m.vocab) return c->fail(RLHF_EINVAL, "eos_id out of range");
    if (!(m.rms_eps >= 0.f) || !(m.rope_base > 1.f)) return c->fail(RLHF_EINVAL, "rms_eps / rope_base");

    c->dtype = m.dtype == RLHF_BF16 ? kBF16 : kF32;
    c->esz = m.dtype == RLHF_BF16 ? 2 : 4;
    c->dm = Dims{m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn, m.vocab, e.page_tokens};
    c->max_pages = ceil_div(e.max_ctx, e.page_tokens);
    const size_t page_bytes = std::max<size_t>(pool_page_elems(c->dm) * c->esz, 1);
    const int64_t pages = e.kv_pool_bytes / (int64_t)page_bytes;
    if (pages < 1 || pages > (int64_t)1 << 27)
        return c->fail(RLHF_ENOMEM, "kv_pool_bytes %lld holds %lld pages of %zu bytes",
                       (long long)e.kv_pool_bytes, (long long)pages, page_bytes);
    c->pool_pages = (int)pages;

    int n_cus = 0;
    {
        int dev = 0;
        HIPCK(c, hipGetDevice(&dev));
        HIPCK(c, hipDeviceGetAttribute(&n_cus, hipDeviceAttributeMultiprocessorCount, dev));
    }
    if (e.half_weight_copies != 0 && e.half_weight_copies != 1)
        return c->fail(RLHF_EINVAL, "half_weight_copies must be 0 or 1");
    if (e.corun_decode_cus < 0 || e.corun_decode_cus >= n_cus || e.corun_decode_cus % 32 || (e.optimistic_admission != 0 && e.optimistic_admission != 1))
        return c->fail(RLHF_EINVAL, "corun_decode_cus must be a multiple of 32 in [0, %d) and optimistic_admission 0 or 1", n_cus);
    auto make_masked = [&](hipStream_t* st, int lo, int hi) -> hipError_t {   // CU-mask bits [lo, hi)
        std::vector<uint32_t> mask((n_cus + 31) / 32, 0u);
        for (int bit = lo; bit < hi; ++bit) mask[bit >> 5] |= 1u << (bit & 31);
        return hipExtStreamCreateWithCUMask(st, (uint32_t)mask.size(), mask.data());
    };
    if (e.decode_stream) c->sd_full = (hipStream_t)e.decode_stream;
    else { HIPCK(c, hipStreamCreateWithFlags(&c->sd_full, hipStreamNonBlocking)); c->own_sd = true; }
    if (e.score_stream) c->ss_full = (hipStream_t)e.score_stream;
    else { HIPCK(c, hipStreamCreateWithFlags(&c->ss_full, hipStreamNonBlocking)); c->own_ss = true; }
    if (e.corun_decode_cus > 0) {
        HIPCK(c, make_masked(&c->sd_part, 0, e.corun_decode_cus));
        HIPCK(c, make_masked(&c->ss_part, e.corun_decode_cus, n_cus));
    }
    c->sd = c->sd_full;
    c->ss = c->ss_full;
    HIPCK(c, hipEventCreateWithFlags(&c->ev_sw_d, hipEventDisableTiming));
    HIPCK(c, hipEventCreateWithFlags(&c->ev_sw_s, hipEventDisableTiming));
    HIPCK(c, hipEventCreateWithFlags(&c->ev_score_last, hipEventDisableTiming));
    HIPCK(c, hipEventCreateWithFlags(&c->ev_dep, hipEventDisableTiming));
    HIPCK(c, hipEventCreate(&c->ev_d0));
    HIPCK(c, hipEventCreate(&c->ev_d1));
    HIPCK(c, hipEventCreate(&c->ev_s0));
    HIPCK(c, hipEventCreate(&c->ev_s1));

    const size_t ns = e.max_samples, mc = e.max_ctx;
    HIPCK(c, hipMalloc(&c->pool, (size_t)c->pool_pages * page_bytes));
    HIPCK(c, hipMalloc((void**)&c->d_page_table, ns * c->max_pages * sizeof(int)));
    HIPCK(c, hipMalloc((void**)&c->d_tokens, ns * mc * sizeof(int)));
    HIPCK(c, hipMalloc((void**)&c->d_lp_actor, ns * mc * 4));
    HIPCK(c, hipMalloc((void**)&c->d_lp_rescored, ns * mc * 4));
    HIPCK(c, hipMalloc((void**)&c->d_lp_ref, ns * mc * 4));
    HIPCK(c, hipMalloc((void**)&c->d_values, ns * mc * 4));
    HIPCK(c, hipMalloc((void**)&c->d_reward, ns * 4));
    HIPCK(c, hipMalloc((void**)&c->d_picked, (size_t)e.max_active * sizeof(int)));
    HIPCK(c, hipMalloc((void**)&c->d_nonfinite, sizeof(int)));
    HIPCK(c, hipMemset(c->d_nonfinite, 0, sizeof(int)));
    HIPCK(c, hipHostMalloc((void**)&c->h_picked, (size_t)e.max_active * sizeof(int), hipHostMallocDefault));
    HIPCK(c, hipMemset(c->d_page_table, 0, ns * c->max_pages * sizeof(int)));

    {   // rotary table in double, stored as float (cos, sin) per (position, pair)
        const int half = m.head_dim / 2;
        std::vector<float> tab((size_t)e.max_ctx * m.head_dim);
        for (int p = 0; p < e.max_ctx; ++p)
            for (int k = 0; k < half; ++k) {
                const double ang = (double)p * std::pow((double)m.rope_base, -2.0 * k / m.head_dim);
                tab[((size_t)p * half + k) * 2] = (float)std::cos(ang);
                tab[((size_t)p * half + k) * 2 + 1] = (float)std::sin(ang);
            }
        HIPCK(c, hipMalloc((void**)&c->d_rope, tab.size() * 4));
        HIPCK(c, hipMemcpy(c->d_rope, tab.data(), tab.size() * 4, hipMemcpyHostToDevice));
    }

    int rc;
    if ((rc = alloc_workspace(c, c->ws_dec, e.max_active, true))) return rc;
    if ((rc = alloc_workspace(c, c->ws_pre, e.max_batch_tokens, false))) return rc;
    if ((rc = alloc_workspace(c, c->ws_score, e.max_batch_tokens, false))) return rc;
    HIPCK(c, c->meta_dec.init((size_t)e.max_active * 10 + (size_t)e.max_active * 2 + 64));
    // prefill metadata also carries the page-table updates of the admitted prompts
    HIPCK(c, c->meta_pre.init((size_t)e.max_batch_tokens * 9 + (size_t)e.max_samples * 12 +
                              2 * ((size_t)e.max_batch_tokens / e.page_tokens + e.max_samples) + 64));
    HIPCK(c, c->meta_score.init((size_t)e.max_batch_tokens * 9 + (size_t)e.max_samples * 8 + 64));
    return RLHF_OK;
}

extern "C" int rlhf_create(const rlhf_model_cfg* model, const rlhf_engine_cfg* engine, rlhf_ctx** out) {
    if (out) *out = nullptr;
    if (!model || !engine || !out) {
        snprintf(g_create_error, sizeof g_create_error, "rlhf_create: NULL argument");
        return RLHF_EINVAL;
    }
    rlhf_ctx* c = new rlhf_ctx();
    c->mc = *model;
    c->ec = *engine;
    const int rc = create_impl(c);
    if (rc != RLHF_OK) {
        snprintf(g_create_error, sizeof g_create_error, "%s", c->err);
        rlhf_destroy(c);
        return rc;
    }
    *out = c;
    return RLHF_OK;
}

extern "C" int rlhf_load_weights(rlhf_ctx* c, int role, const rlhf_weights* w) {
    if (!c) return RLHF_EINVAL;
    if (role < 0 || role > 3 || !w) return c->fail(RLHF_EINVAL, "rlhf_load_weights: bad role or NULL weights");
    if (!w->embed || !w->g_final || !w->head ||
        (c->mc.n_layers > 0 && (!w->wqkv || !w->wo || !w->w_gate_up || !w->w_down || !w->g_attn || !w->g_mlp)))
        return c->fail(RLHF_EINVAL, "rlhf_load_weights: NULL tensor");
    const void* ptrs[] = {w->embed, w->wqkv, w->wo, w->w_gate_up, w->w_down, w->g_attn, w->g_mlp, w->g_final, w->head};
    for (const void* p : ptrs)
        if (p && ((uintptr_t)p & 15)) return c->fail(RLHF_EINVAL, "rlhf_load_weights: tensors must be 16-byte aligned");
    RoleWeights& rw = c->roles[role];
    int rc = rlhf_sync(c);                       // nothing in flight may still read copies about to be freed
    if (rc) return rc;
    for (void* p : rw.owned) (void)hipFree(p);
    rw.owned.clear();
    rw.h16 = rlhf_weights{};
    rw.w = *w;
    rw.bound = true;
    if (c->ec.half_weight_copies && c->dtype == kBF16) {
        const rlhf_model_cfg& m = c->mc;
        const size_t d = m.d_model, qd = (size_t)m.n_q_heads * m.head_dim, kvd = (size_t)m.n_kv_heads * m.head_dim;
        const size_t L = m.n_layers, f = m.ffn;
        struct Item { const void* src; const void** dst; size_t n, per_matrix; };
        const Item items[] = {
            {w->wqkv, &rw.h16.wqkv, L * (qd + 2 * kvd) * d, (qd + 2 * kvd) * d},
            {w->wo, &rw.h16.wo, L * d * qd, d * qd},
            {w->w_gate_up, &rw.h16.w_gate_up, L * 2 * f * d, 2 * f * d},
            {w->w_down, &rw.h16.w_down, L * d * f, d * f},
            {w->head, &rw.h16.head, (role == RLHF_ACTOR || role == RLHF_REF) ? (size_t)m.vocab * d : 0, (size_t)m.vocab * d},
        };
        // the kernels that take the copies address an operand with 32-bit byte offsets: a matrix, or a pass's
        // activations, of 4 GiB or more stays on the bf16-weight path
        const size_t lim = (size_t)1 << 32;
        const bool acts_fit = (size_t)c->ec.max_batch_tokens * std::max(d, f) * 2 < lim;
        for (const Item& it : items) {
            if (it.n == 0 || !it.src || !acts_fit || it.per_matrix * 2 >= lim) continue;
            void* p = nullptr;
            if (hipMalloc(&p, it.n * 2) != hipSuccess) {
                (void)hipGetLastError();
                for (void* q : rw.owned) (void)hipFree(q);
                rw.owned.clear();
                rw.h16 = rlhf_weights{};
                rw.bound = false;
                return c->fail(RLHF_ENOMEM, "rlhf_load_weights: no device memory for the half copies of role %d "
                                            "(%zu bytes); leave room beside kv_pool_bytes or turn half_weight_copies off",
                               role, it.n * 2);
            }
            rw.owned.push_back(p);
            HIPCK(c, launch_bf16_to_half(c->sd_full, it.src, p, it.n));
            *it.dst = p;
        }
        HIPCK(c, hipStreamSynchronize(c->sd_full));
    }
    return RLHF_OK;
}

extern "C" int rlhf_sync(rlhf_ctx* c) {
    if (!c) return RLHF_EINVAL;
    for (hipStream_t st : {c->sd_full, c->ss_full, c->sd_part, c->ss_part})
        if (st) HIPCK(c, hipStreamSynchronize(st));
    return RLHF_OK;
}

namespace {
// Continue a logical stream (decode or scoring) on another HIP stream: the new one first waits
// for everything issued on the old one.
int switch_stream(rlhf_ctx* c, hipStream_t* cur, hipStream_t next, hipEvent_t ev) {
    if (*cur == next || !next) return RLHF_OK;
    HIPCK(c, hipEventRecord(ev, *cur));
    HIPCK(c, hipStreamWaitEvent(next, ev, 0));
    *cur = next;
    return RLHF_OK;
}
}  // namespace

// =================================================================================== submit

extern "C" int rlhf_submit(rlhf_ctx* c, int32_t n, const int32_t* prompt_tokens,
                           const int64_t* prompt_offsets, const int32_t* max_new,
                           const int32_t* forced_len, const int32_t* forced_tokens,
                           const int64_t* forced_offsets) {
    if (!c) return RLHF_EINVAL;
    if (n < 0 || n > c->ec.max_samples) return c->fail(RLHF_EINVAL, "rlhf_submit: n = %d outside [0, %d]", n, c->ec.max_samples);
    if (n > 0 && (!prompt_tokens || !prompt_offsets || !max_new)) return c->fail(RLHF_EINVAL, "rlhf_submit: NULL array");
    if (forced_tokens && !forced_offsets) return c->fail(RLHF_EINVAL, "rlhf_submit: forced_tokens without forced_offsets");
    const int mc = c->ec.max_ctx, pt = c->ec.page_tokens;
    std::vector<Sample> smp(n);
    for (int i = 0; i < n; ++i) {
        const int64_t P = prompt_offsets[i + 1] - prompt_offsets[i];
        if (P < 1 || max_new[i] < 1 || P + max_new[i] > mc)
            return c->fail(RLHF_EINVAL, "rlhf_submit: sample %d has prompt %lld, max_new %d (need >= 1, sum <= max_ctx %d)",
                           i, (long long)P, max_new[i], mc);
        Sample& s = smp[i];
        s.P = (int)P;
        s.max_new = max_new[i];
        s.target = max_new[i];
        if (forced_len) {
            if (forced_len[i] < 1 || forced_len[i] > max_new[i])
                return c->fail(RLHF_EINVAL, "rlhf_submit: forced_len[%d] = %d outside [1, max_new]", i, forced_len[i]);
            s.target = forced_len[i];
            s.has_forced_len = true;
        }
        s.reserve = ceil_div(s.P + s.max_new, pt);
        if (s.reserve > c->pool_pages)
            return c->fail(RLHF_ENOMEM, "rlhf_submit: sample %d reserves %d pages, the pool has %d", i, s.reserve, c->pool_pages);
        for (int64_t k = prompt_offsets[i]; k < prompt_offsets[i + 1]; ++k)
            if (prompt_tokens[k] < 0 || prompt_tokens[k] >= c->mc.vocab)
                return c->fail(RLHF_EINVAL, "rlhf_submit: token %d of sample %d out of range", prompt_tokens[k], i);
        if (forced_tokens) {
            const int64_t fl = forced_offsets[i + 1] - forced_offsets[i];
            if (fl < 0 || fl > s.max_new) return c->fail(RLHF_EINVAL, "rlhf_submit: forced_offsets of sample %d", i);
            for (int64_t k = forced_offsets[i]; k < forced_offsets[i + 1]; ++k)
                if (forced_tokens[k] >= c->mc.vocab) return c->fail(RLHF_EINVAL, "rlhf_submit: forced token out of range");
        }
    }
    int rc = rlhf_sync(c);
    if (rc) return rc;

    c->N = n;
    c->smp.swap(smp);
    c->h_prompt.assign(prompt_tokens, prompt_tokens + (n ? prompt_offsets[n] : 0));
    c->h_prompt_off.assign(prompt_offsets, prompt_offsets + (n ? n + 1 : 0));
    c->h_forced.assign((size_t)n * mc, -1);
    std::vector<int> tok((size_t)n * mc, 0);
    for (int i = 0; i < n; ++i) {
        Sample& s = c->smp[i];
        std::copy(prompt_tokens + prompt_offsets[i], prompt_tokens + prompt_offsets[i + 1], tok.begin() + (size_t)i * mc);
        if (forced_tokens)
            for (int64_t k = forced_offsets[i]; k < forced_offsets[i + 1]; ++k)
                c->h_forced[(size_t)i * mc + (k - forced_offsets[i])] = forced_tokens[k] < 0 ? -1 : forced_tokens[k];
        if (s.has_forced_len) c->h_forced[(size_t)i * mc + s.target - 1] = c->ec.eos_id;
    }
    if (n) HIPCK(c, hipMemcpy(c->d_tokens, tok.data(), tok.size() * sizeof(int), hipMemcpyHostToDevice));
    // results of roles that are never scored read back as NaN (all-ones bit pattern), not as
    // leftovers of an earlier stage
    for (float* r : {c->d_lp_actor, c->d_lp_rescored, c->d_lp_ref, c->d_values})
        HIPCK(c, hipMemset(r, 0xFF, (size_t)c->ec.max_samples * mc * 4));
    HIPCK(c, hipMemset(c->d_reward, 0xFF, (size_t)c->ec.max_samples * 4));
    HIPCK(c, hipMemset(c->d_nonfinite, 0, sizeof(int)));
    c->waiting.clear();
    for (int i = 0; i < n; ++i) c->waiting.push_back(i);
    c->active.clear();
    c->free_list.resize(c->pool_pages);
    for (int p = 0; p < c->pool_pages; ++p) c->free_list[p] = c->pool_pages - 1 - p;   // pop_back issues 0, 1, 2, ...
    c->reserved = 0;
    c->retired.clear();
    c->n_scored = 0;
    c->batch_offsets.assign(1, 0);
    c->batch_step.clear();
    c->step = 0;
    c->score_used = false;
    c->acc_weight_bytes = c->acc_kv_bytes = c->acc_prefill_tokens = 0;
    return RLHF_OK;
}

// ============================================================================ generate step

namespace {

int take_page(rlhf_ctx* c, Sample& s) {
    const int pg = c->free_list.back();
    c->free_list.pop_back();
    s.pages.push_back(pg);
    return pg;
}

// Imposed token at output index j (1-based) of sample i, or -1.
int forced_at(const rlhf_ctx* c, int i, int j) { return c->h_forced[(size_t)i * c->ec.max_ctx + (j - 1)]; }

// Head over selected rows of a batch pass: logits in row chunks, then pick / gather.
struct HeadPlan {
    int n_sel = 0;
    const int* sel_rows = nullptr;     // device: rows of the pass whose hidden state feeds the head
    // pick (prefill): per selected row
    const int* forced = nullptr;
    const int* tok_dst = nullptr;
    const int* lp_dst = nullptr;
    // gather (scoring log-probs): per selected row
    const int* target_idx = nullptr;
    const int* out_dst = nullptr;
    float* out = nullptr;
};

int lm_head_chunks(rlhf_ctx* c, hipStream_t st, Workspace& ws, const rlhf_weights& w, const HeadPlan& hp,
                   bool pick) {
    const rlhf_model_cfg& m = c->mc;
    const int d = m.d_model, V = m.vocab;
    for (int r0 = 0; r0 < hp.n_sel; r0 += ws.logit_rows) {
        const int nr = std::min(ws.logit_rows, hp.n_sel - r0);
        const char* x = (const char*)ws.xsel + (size_t)r0 * d * c->esz;
        HIPCK(c, gemm_profiled(c, st, kGemmBatch, act_type(c, true), x, w.head, ws.logits, nr, V, d, 1));
        if (pick)
            HIPCK(c, launch_pick(st, ws.logits, 1, 0, nr, V, hp.forced + r0, c->d_tokens, hp.tok_dst + r0,
                                 c->d_lp_actor, hp.lp_dst + r0, nullptr, ws.pick_scratch, c->d_nonfinite));
        else
            HIPCK(c, launch_gather_lp(st, ws.logits, 1, 0, nr, V, c->d_tokens, hp.target_idx + r0, hp.out,
                                      hp.out_dst + r0, c->d_nonfinite));
    }
    return RLHF_OK;
}

// LM head of a scoring pass with the log-softmax gather fused into the GEMM's epilogue: the
// [rows, vocab] logits never reach memory, only 2 * ceil(vocab / 256) (max, sum exp) pairs and the
// target logit per row, which a merge kernel turns into log-probs.  The partials live in the
// workspace's logits buffer.
int lm_head_logprob_fused(rlhf_ctx* c, hipStream_t st, Workspace& ws, const RoleWeights& rw, const HeadPlan& hp) {
    const bool hw = rw.h16.head != nullptr && act_type(c, true) == kF16;
    const void* head = hw ? rw.h16.head : rw.w.head;
    const int wdt = hw ? kF16 : c->dtype;
    const rlhf_model_cfg& m = c->mc;
    const int d = m.d_model, V = m.vocab, adt = act_type(c, true);
    const int n_part = gemm_lse_partials(V);
    const size_t per_row = (size_t)2 * n_part + 1;
    const size_t cap_rows = (size_t)ws.logit_rows * V / per_row;
    if (cap_rows < 1) return c->fail(RLHF_EINVAL, "internal: no room for the LM head's partials");
    for (int r0 = 0; r0 < hp.n_sel; r0 += (int)std::min<size_t>(cap_rows, 1 << 30)) {
        const int nr = (int)std::min<size_t>(cap_rows, (size_t)(hp.n_sel - r0));
        LseOut lo;
        lo.tokens = c->d_tokens;
        lo.target_idx = hp.target_idx + r0;
        lo.part_max = ws.logits;
        lo.part_sum = ws.logits + (size_t)nr * n_part;
        lo.tgt = ws.logits + (size_t)2 * nr * n_part;
        lo.n_part = n_part;
        const char* x = (const char*)ws.xsel + (size_t)r0 * d * c->esz;
        const double bytes = ((double)V * d + (double)nr * d) * c->esz + (double)nr * per_row * 4;
        HIPCK(c, profiled(c, st, kGemmBatch, bytes, 2.0 * nr * V * d,
                          [&] { return launch_gemm_lse(st, wdt, adt, x, head, nr, V, d, lo); }));
        HIPCK(c, launch_lse_merge(st, lo.part_max, lo.part_sum, lo.tgt, n_part, nr, hp.out, hp.out_dst + r0,
                                  c->d_nonfinite));
    }
    return RLHF_OK;
}

// Query tiles of the MFMA attention for sequences of the given lengths packed back to back:
// writes tile_start / tile_q0 / tile_len (n each) at dst, dst + n, dst + 2n; returns n.
int count_tiles(const std::vector<int>& lens) {
    int n = 0;
    for (int L : lens) n += ceil_div(L, kFlashTile);
    return n;
}
void fill_tiles(const std::vector<int>& lens, int* dst) {
    const int n = count_tiles(lens);
    int t = 0, start = 0;
    for (int L : lens) {
        for (int q0 = 0; q0 < L; q0 += kFlashTile, ++t) {
            dst[t] = start;
            dst[n + t] = q0;
            dst[2 * n + t] = L;
        }
        start += L;
    }
}

// Algorithmic cost of one layer's packed causal attention over sequences of the given lengths.
void batch_attn_cost(const rlhf_ctx* c, const std::vector<int>& lens, int T, PassMeta* pm) {
    const double qd = (double)c->mc.n_q_heads * c->mc.head_dim, kvd = (double)c->mc.n_kv_heads * c->mc.head_dim;
    double pairs = 0;
    for (int L : lens) {
        const double t = L;
        pairs += t * (t + 1) / 2;
    }
    pm->attn_flops = 4.0 * qd * pairs;
    pm->attn_bytes = (double)T * (2 * qd + 2 * kvd) * c->esz;
}

// Rows a sample needs when it is (re-)admitted: its prompt, plus, after a migration (Section
// 4.2, "Migration mechanism", second choice: only the tokens travel and the KV cache is
// regenerated by rerunning the prefill), every generated token but the newest, which the same
// step's decode feeds.
int prefill_rows(const Sample& s) { return s.P + std::max(s.gen_len - 1, 0); }

// Prefill of newly admitted samples [group], whose rows total `T` <= max_batch_tokens.  A
// first-time sample gets its first output token from the last prompt row; a migrated one emits
// nothing.
int prefill_group(rlhf_ctx* c, const std::vector<int>& group, int T) {
    const int mc = c->ec.max_ctx, pt = c->ec.page_tokens, n = (int)group.size();
    int* hm;
    HIPCK(c, c->meta_pre.begin(&hm));
    // layout: tok_idx[T] pos[T] row_start[T] kv_dst[T] | sel[n] forced[n] tok_dst[n] lp_dst[n] | upd_idx[U] upd_val[U]
    int* tok_idx = hm;
    int* pos = hm + T;
    int* row_start = hm + 2 * T;
    int* kv_dst = hm + 3 * T;
    int* sel = hm + 4 * T;
    int* forced = sel + n;
    int* tok_dst = forced + n;
    int* lp_dst = tok_dst + n;
    int* upd = lp_dst + n;
    std::vector<int> upd_idx, upd_val, lens;
    int row = 0, n_sel = 0;
    for (int gi = 0; gi < n; ++gi) {
        const int i = group[gi];
        Sample& s = c->smp[i];
        const int start = row, rows_i = prefill_rows(s);
        lens.push_back(rows_i);
        for (int p = 0; p < rows_i; ++p, ++row) {
            if (p % pt == 0) {
                const int pg = take_page(c, s);
                upd_idx.push_back(i * c->max_pages + p / pt);
                upd_val.push_back(pg);
            }
            tok_idx[row] = i * mc + p;
            pos[row] = p;
            row_start[row] = start;
            kv_dst[row] = s.pages[p / pt] * pt + p % pt;
        }
        s.ctx = rows_i;
        s.admit_step = c->step;
        if (s.gen_len == 0) {
            s.gen_len = 1;
            sel[n_sel] = row - 1;
            forced[n_sel] = forced_at(c, i, 1);
            tok_dst[n_sel] = i * mc + s.P;
            lp_dst[n_sel] = i * mc + 0;
            ++n_sel;
        }
    }
    const int U = (int)upd_idx.size();
    std::copy(upd_idx.begin(), upd_idx.end(), upd);
    std::copy(upd_val.begin(), upd_val.end(), upd + U);
    const int n_tiles = count_tiles(lens);
    const size_t tiles_off = (size_t)4 * T + 4 * n + 2 * U;
    const size_t n_ints = tiles_off + 3 * (size_t)n_tiles;
    if (n_ints > c->meta_pre.cap) return c->fail(RLHF_EINVAL, "internal: prefill metadata overflow");
    fill_tiles(lens, hm + tiles_off);
    HIPCK(c, c->meta_pre.commit(c->sd, n_ints));
    const int* dm_ = c->meta_pre.dev;
    HIPCK(c, launch_scatter_int(c->sd, c->d_page_table, dm_ + 4 * T + 4 * n, dm_ + 4 * T + 4 * n + U, U));

    PassMeta pm;
    pm.tok_idx = dm_;
    pm.pos = dm_ + T;
    pm.row_start = dm_ + 2 * T;
    pm.kv_dst = dm_ + 3 * T;
    pm.tile_start = dm_ + tiles_off;
    pm.tile_q0 = dm_ + tiles_off + n_tiles;
    pm.tile_len = dm_ + tiles_off + 2 * n_tiles;
    pm.n_tiles = n_tiles;
    batch_attn_cost(c, lens, T, &pm);
    const rlhf_weights& w = c->roles[RLHF_ACTOR].w;
    Workspace& ws = c->ws_pre;
    int pns;
    size_t pstride;
    int rc = forward_layers(c, c->sd, ws, c->roles[RLHF_ACTOR], T, pm, kModeBatch, 1, &pns, &pstride);
    if (rc) return rc;
    if (n_sel > 0) {
        HIPCK(c, launch_rmsnorm(c->sd, act_type(c, true), ws.h, ws.part, pns, pstride, dm_ + 4 * T, w.g_final, ws.xsel,
                                n_sel, c->mc.d_model, c->mc.rms_eps));
        HeadPlan hp;
        hp.n_sel = n_sel;
        hp.forced = dm_ + 4 * T + n;
        hp.tok_dst = dm_ + 4 * T + 2 * n;
        hp.lp_dst = dm_ + 4 * T + 3 * n;
        rc = lm_head_chunks(c, c->sd, ws, w, hp, true);
        if (rc) return rc;
    }
    c->acc_prefill_tokens += T;
    return RLHF_OK;
}

int decode_rows(rlhf_ctx* c, const std::vector<int>& rows_ids) {
    const int R = (int)rows_ids.size();
    const int mc = c->ec.max_ctx, pt = c->ec.page_tokens;
    int* hm;
    HIPCK(c, c->meta_dec.begin(&hm));
    // layout: tok_idx pos kv_dst row_sample ctx_len tok_dst lp_dst forced (R each) | upd_idx[U] upd_val[U]
    int* a[8];
    for (int k = 0; k < 8; ++k) a[k] = hm + k * R;
    int* upd = hm + 8 * R;
    int U = 0;
    int64_t kv_tokens = 0;
    int max_ctx_len = 0;
    for (int r = 0; r < R; ++r) {
        const int i = rows_ids[r];
        Sample& s = c->smp[i];
        const int p = s.ctx;                 // position being written
        if (p % pt == 0) {
            const int pg = take_page(c, s);
            upd[U] = i * c->max_pages + p / pt;
            upd[R + U] = pg;                 // provisional slot; compacted below
            ++U;
        }
        a[0][r] = i * mc + p;
        a[1][r] = p;
        a[2][r] = s.pages[p / pt] * pt + p % pt;
        a[3][r] = i;
        a[4][r] = p + 1;
        a[5][r] = i * mc + p + 1;
        a[6][r] = i * mc + (p + 1 - s.P);
        a[7][r] = forced_at(c, i, p + 2 - s.P);
        s.ctx = p + 1;
        s.gen_len += 1;
        kv_tokens += p + 2;                  // p+1 keys read, one written
        max_ctx_len = std::max(max_ctx_len, p + 1);
    }
    for (int u = 0; u < U; ++u) upd[U + u] = upd[R + u];
    HIPCK(c, c->meta_dec.commit(c->sd, (size_t)8 * R + 2 * U));
    const int* dmeta = c->meta_dec.dev;
    HIPCK(c, launch_scatter_int(c->sd, c->d_page_table, dmeta + 8 * R, dmeta + 8 * R + U, U));

    PassMeta pm;
    pm.tok_idx = dmeta;
    pm.pos = dmeta + R;
    pm.kv_dst = dmeta + 2 * R;
    pm.row_sample = dmeta + 3 * R;
    pm.ctx_len = dmeta + 4 * R;
    {
        const double kvd_ = (double)c->mc.n_kv_heads * c->mc.head_dim, qd_ = (double)c->mc.n_q_heads * c->mc.head_dim;
        const double keys = (double)(kv_tokens - R);           // sum of visible keys over rows
        pm.attn_bytes = (keys * 2 * kvd_ + 2.0 * R * qd_) * c->esz;
        pm.attn_flops = 4.0 * keys * qd_;
    }
    // split long contexts so that a handful of samples still fills the chip
    Workspace& ws = c->ws_dec;
    const int blocks = R * c->mc.n_kv_heads;
    int asplit = std::max(1, 1024 / std::max(blocks, 1));
    asplit = std::min(asplit, std::max(1, ceil_div(max_ctx_len, pt) / 8));
    asplit = std::min<int>(asplit, 32);
    asplit = (int)std::min<size_t>(asplit, ws.attn_slots / ((size_t)R * c->mc.n_q_heads));
    if (asplit < 1) asplit = 1;

    const rlhf_weights& w = c->roles[RLHF_ACTOR].w;
    int pns;
    size_t pstride;
    int rc = forward_layers(c, c->sd, ws, c->roles[RLHF_ACTOR], R, pm, kModeDecode, asplit, &pns, &pstride);
    if (rc) return rc;
    const int d = c->mc.d_model, V = c->mc.vocab;
    HIPCK(c, launch_rmsnorm(c->sd, act_type(c, false), ws.h, ws.part, pns, pstride, nullptr, w.g_final, ws.xsel, R, d,
                            c->mc.rms_eps));
    const int ns = nsplit_for(c, ws, R, V, d);
    HIPCK(c, gemm_profiled(c, c->sd, kGemmDecode, act_type(c, false), ws.xsel, w.head, ws.part, R, V, d, ns));
    HIPCK(c, launch_pick(c->sd, ws.part, ns, (size_t)R * V, R, V, dmeta + 7 * R, c->d_tokens, dmeta + 5 * R,
                         c->d_lp_actor, dmeta + 6 * R, c->d_picked, ws.pick_scratch, c->d_nonfinite));
    // algorithmic bytes of this step
    const rlhf_model_cfg& m = c->mc;
    const int64_t qd = (int64_t)m.n_q_heads * m.head_dim, kvd = (int64_t)m.n_kv_heads * m.head_dim;
    const int64_t per_layer = (qd + 2 * kvd) * m.d_model + m.d_model * qd + 3LL * m.d_model * m.ffn;
    c->acc_weight_bytes += (m.n_layers * per_layer + (int64_t)m.vocab * m.d_model) * c->esz;
    c->acc_kv_bytes += kv_tokens * 2 * m.n_layers * kvd * c->esz;
    return RLHF_OK;
}

// stop_on_eos: fetch the tokens just picked for `ids` (pick order) and mark finished samples.
int check_eos(rlhf_ctx* c, const std::vector<int>& ids, const int* d_src) {
    if (!c->ec.stop_on_eos || ids.empty()) return RLHF_OK;
    HIPCK(c, hipMemcpyAsync(c->h_picked, d_src, ids.size() * sizeof(int), hipMemcpyDeviceToHost, c->sd));
    HIPCK(c, hipStreamSynchronize(c->sd));
    for (size_t r = 0; r < ids.size(); ++r)
        if (c->h_picked[r] == c->ec.eos_id) c->smp[ids[r]].finished = true;
    return RLHF_OK;
}

bool sample_done(const Sample& s) { return s.finished || s.gen_len >= s.target; }

// The listed active samples give their pages back (each in reverse page-table order), release
// their reservation and leave the active array; the caller puts them back into the queue.
void release_samples(rlhf_ctx* c, const int* ids, int n) {
    std::vector<char> listed(c->smp.size(), 0);
    for (int k = 0; k < n; ++k) {
        Sample& s = c->smp[ids[k]];
        listed[ids[k]] = 1;
        for (auto it = s.pages.rbegin(); it != s.pages.rend(); ++it) c->free_list.push_back(*it);
        s.pages.clear();
        s.ctx = 0;
        c->reserved -= s.reserve;
    }
    std::vector<int> keep;
    for (int i : c->active)
        if (!listed[i]) keep.push_back(i);
    c->active.swap(keep);
}

}  // namespace

extern "C" int rlhf_generate_step(rlhf_ctx* c, rlhf_step_info* out) {
    if (!c) return RLHF_EINVAL;
    if (!c->roles[RLHF_ACTOR].bound) return c->fail(RLHF_ESTATE, "rlhf_generate_step: Actor weights not loaded");
    if (c->waiting.empty() && c->active.empty()) return c->fail(RLHF_ESTATE, "rlhf_generate_step: nothing to generate");
    // admission: FIFO, first misfit blocks the queue.  The test is the reservation at the cap, or,
    // under optimistic admission, the pages needed now plus one spare page per running sample.
    std::vector<int> newcomers;
    int free_now = (int)c->free_list.size();
    while (!c->waiting.empty() && (int)(c->active.size() + newcomers.size()) < c->ec.max_active) {
        const int i = c->waiting.front();
        if (c->ec.optimistic_admission) {
            const int need = ceil_div(prefill_rows(c->smp[i]) + 1, c->ec.page_tokens);
            const int running = (int)(c->active.size() + newcomers.size());
            if (need > free_now || (running > 0 && free_now - need < running)) break;
            free_now -= need;
        } else if (c->reserved + c->smp[i].reserve > c->pool_pages) {
            break;
        }
        c->waiting.pop_front();
        c->reserved += c->smp[i].reserve;
        newcomers.push_back(i);
    }
    int n_prefill = 0;
    // prefill in groups that fit one batch pass
    size_t g0 = 0;
    while (g0 < newcomers.size()) {
        std::vector<int> group;
        int T = 0;
        size_t g1 = g0;
        std::vector<int> fresh;
        while (g1 < newcomers.size() && T + prefill_rows(c->smp[newcomers[g1]]) <= c->ec.max_batch_tokens) {
            T += prefill_rows(c->smp[newcomers[g1]]);
            group.push_back(newcomers[g1]);
            if (c->smp[newcomers[g1]].gen_len == 0) fresh.push_back(newcomers[g1]);
            ++g1;
        }
        int rc = prefill_group(c, group, T);
        if (rc) return rc;
        if (c->ec.stop_on_eos) {
            // picked tokens of a prefill are not in d_picked; read them from the token buffer
            for (int i : fresh) {
                int y;
                HIPCK(c, hipMemcpyAsync(&y, c->d_tokens + (size_t)i * c->ec.max_ctx + c->smp[i].P, sizeof(int),
                                        hipMemcpyDeviceToHost, c->sd));
                HIPCK(c, hipStreamSynchronize(c->sd));
                if (y == c->ec.eos_id) c->smp[i].finished = true;
            }
        }
        n_prefill += T;
        g0 = g1;
    }
    for (int i : newcomers) c->active.push_back(i);
    int n_preempted = 0;
    if (c->ec.optimistic_admission) {
        // the decode below takes a page for every sample that sits on a page boundary: if they are
        // not all there, the most recently admitted unfinished samples give theirs back
        std::vector<int> victims;
        for (;;) {
            int need = 0, last = -1;
            for (int i : c->active)
                if (!sample_done(c->smp[i])) {
                    need += c->smp[i].ctx % c->ec.page_tokens == 0;
                    last = i;
                }
            if (need <= (int)c->free_list.size()) break;
            release_samples(c, &last, 1);
            victims.push_back(last);
        }
        for (int v : victims) c->waiting.push_front(v);   // earliest admitted victim ends up first
        n_preempted = (int)victims.size();
    }
    std::vector<int> rows;
    for (int i : c->active)
        if (!sample_done(c->smp[i])) rows.push_back(i);
    if (!rows.empty()) {
        int rc = decode_rows(c, rows);
        if (rc) return rc;
        rc = check_eos(c, rows, c->d_picked);
        if (rc) return rc;
    }
    if (out) {
        out->step = c->step;
        out->n_admitted = (int)newcomers.size();
        out->n_prefill_tokens = n_prefill;
        out->n_decoded = (int)rows.size();
        out->n_active = (int)c->active.size();
        out->n_preempted = n_preempted;
    }
    c->step += 1;
    return RLHF_OK;
}

extern "C" int rlhf_retire(rlhf_ctx* c, int32_t* retired_ids, int32_t* n_retired) {
    if (!c) return RLHF_EINVAL;
    int n = 0;
    std::vector<int> keep;
    keep.reserve(c->active.size());
    for (int i : c->active) {
        Sample& s = c->smp[i];
        if (sample_done(s)) {
            for (auto it = s.pages.rbegin(); it != s.pages.rend(); ++it) c->free_list.push_back(*it);
            s.pages.clear();
            c->reserved -= s.reserve;
            s.retired = true;
            c->retired.push_back(i);
            if (retired_ids) retired_ids[n] = i;
            ++n;
        } else {
            keep.push_back(i);
        }
    }
    c->active.swap(keep);
    if (n_retired) *n_retired = n;
    return RLHF_OK;
}

extern "C" int rlhf_migrate(rlhf_ctx* c, const int32_t* ids, int32_t n, int32_t to_back) {
    if (!c || n < 0 || (n > 0 && !ids)) return RLHF_EINVAL;
    std::vector<char> listed(c->smp.size(), 0);
    for (int k = 0; k < n; ++k) {
        const int i = ids[k];
        if (i < 0 || i >= (int)c->smp.size()) return c->fail(RLHF_EINVAL, "rlhf_migrate: id %d out of range", i);
        if (listed[i]) return c->fail(RLHF_EINVAL, "rlhf_migrate: id %d listed twice", i);
        listed[i] = 1;
        const bool is_active = std::find(c->active.begin(), c->active.end(), i) != c->active.end();
        if (!is_active || sample_done(c->smp[i]))
            return c->fail(RLHF_EINVAL, "rlhf_migrate: sample %d is not an unfinished active sample", i);
    }
    // work already enqueued on the decode stream that reads these pages runs before whatever is
    // enqueued later and writes them again: stream order is the only ordering needed
    release_samples(c, ids, n);
    if (to_back)
        for (int k = 0; k < n; ++k) c->waiting.push_back(ids[k]);
    else
        for (int k = n - 1; k >= 0; --k) c->waiting.push_front(ids[k]);
    return RLHF_OK;
}

// ================================================================================== scoring

namespace {

// One packed pass over samples ids[lo, hi) (total T rows) for one role.
int score_pass(rlhf_ctx* c, hipStream_t st, MetaRing& meta, Workspace& ws, const int* ids, int n, int T, int role) {
    const int mc = c->ec.max_ctx;
    int* hm;
    HIPCK(c, meta.begin(&hm));
    int n_sel = 0;
    for (int k = 0; k < n; ++k) n_sel += role == RLHF_REWARD ? 1 : c->smp[ids[k]].gen_len;
    // layout: tok_idx[T] pos[T] row_start[T] | sel[n_sel] target_idx[n_sel] out_dst[n_sel]
    int* tok_idx = hm;
    int* pos = hm + T;
    int* row_start = hm + 2 * T;
    int* sel = hm + 3 * T;
    int* target = sel + n_sel;
    int* out_dst = target + n_sel;
    std::vector<int> lens;
    for (int k = 0; k < n; ++k) lens.push_back(c->smp[ids[k]].P + c->smp[ids[k]].gen_len);
    const int n_tiles = count_tiles(lens);
    const size_t tiles_off = (size_t)3 * T + 3 * n_sel;
    if (tiles_off + 3 * (size_t)n_tiles > meta.cap) return c->fail(RLHF_EINVAL, "internal: scoring metadata overflow");
    fill_tiles(lens, hm + tiles_off);
    int row = 0, si = 0;
    for (int k = 0; k < n; ++k) {
        const int i = ids[k];
        const Sample& s = c->smp[i];
        const int Ti = s.P + s.gen_len, start = row;
        for (int p = 0; p < Ti; ++p, ++row) {
            tok_idx[row] = i * mc + p;
            pos[row] = p;
            row_start[row] = start;
        }
        if (role == RLHF_REWARD) {
            sel[si] = start + Ti - 1;
            target[si] = 0;
            out_dst[si] = i;
            ++si;
        } else {
            for (int j = 1; j <= s.gen_len; ++j, ++si) {
                sel[si] = start + s.P + j - 2;          // the position that predicts y_j (0-based)
                target[si] = i * mc + s.P + j - 1;      // y_j itself sits one position later
                out_dst[si] = i * mc + j - 1;
            }
        }
    }
    HIPCK(c, meta.commit(st, tiles_off + 3 * (size_t)n_tiles));
    const int* dmeta = meta.dev;
    PassMeta pm;
    pm.tok_idx = dmeta;
    pm.pos = dmeta + T;
    pm.row_start = dmeta + 2 * T;
    pm.tile_start = dmeta + tiles_off;
    pm.tile_q0 = dmeta + tiles_off + n_tiles;
    pm.tile_len = dmeta + tiles_off + 2 * n_tiles;
    pm.n_tiles = n_tiles;
    batch_attn_cost(c, lens, T, &pm);
    const rlhf_weights& w = c->roles[role].w;
    int pns;
    size_t pstride;
    int rc = forward_layers(c, st, ws, c->roles[role], T, pm, kModeBatch, 1, &pns, &pstride);
    if (rc) return rc;
    const int d = c->mc.d_model;
    // selected rows may exceed the workspace rows only if n_sel > T, which cannot happen
    // The d -> 1 heads read the final-norm row in float (no rounding to the 16-bit activation type
    // in front of a single dot product); the LM head's GEMM takes the activation type.
    const bool scalar_head = role == RLHF_CRITIC || role == RLHF_REWARD;
    const int adt = scalar_head ? kF32 : act_type(c, true);
    HIPCK(c, launch_rmsnorm(st, adt, ws.h, ws.part, pns, pstride, dmeta + 3 * T, w.g_final, ws.xsel, n_sel, d,
                            c->mc.rms_eps));
    if (role == RLHF_CRITIC)
        HIPCK(c, launch_head_dot(st, adt, c->dtype, ws.xsel, w.head, n_sel, d, c->d_values, dmeta + 3 * T + 2 * n_sel,
                                 c->d_nonfinite));
    else if (role == RLHF_REWARD)
        HIPCK(c, launch_head_dot(st, adt, c->dtype, ws.xsel, w.head, n_sel, d, c->d_reward, dmeta + 3 * T + 2 * n_sel,
                                 c->d_nonfinite));
    else {
        HeadPlan hp;
        hp.n_sel = n_sel;
        hp.target_idx = dmeta + 3 * T + n_sel;
        hp.out_dst = dmeta + 3 * T + 2 * n_sel;
        hp.out = role == RLHF_REF ? c->d_lp_ref : c->d_lp_rescored;
        rc = gemm_lse_supported(c->dtype, adt, d) ? lm_head_logprob_fused(c, st, ws, c->roles[role], hp)
                                                  : lm_head_chunks(c, st, ws, w, hp, false);
        if (rc) return rc;
    }
    return RLHF_OK;
}

int score_ids(rlhf_ctx* c, const int* ids, int n, uint32_t role_mask, bool on_score_stream) {
    if (n <= 0) return RLHF_OK;
    for (int role = 0; role < 4; ++role)
        if ((role_mask & RLHF_ROLE_BIT(role)) && !c->roles[role].bound)
            return c->fail(RLHF_ESTATE, "rlhf_score: role %d has no weights", role);
    for (int k = 0; k < n; ++k) {
        if (ids[k] < 0 || ids[k] >= c->N) return c->fail(RLHF_EINVAL, "rlhf_score: sample id %d out of range", ids[k]);
        if (!sample_done(c->smp[ids[k]]) || c->smp[ids[k]].gen_len < 1)
            return c->fail(RLHF_ESTATE, "rlhf_score: sample %d is still generating", ids[k]);
    }
    if (on_score_stream && c->ss_part) {
        // generation still running: keep to the scoring share of the chip; otherwise take it all
        const bool generating = !c->waiting.empty() || !c->active.empty();
        int rc = switch_stream(c, &c->ss, generating ? c->ss_part : c->ss_full, c->ev_sw_s);
        if (rc) return rc;
    }
    hipStream_t st = on_score_stream ? c->ss : c->sd;
    Workspace& ws = on_score_stream ? c->ws_score : c->ws_pre;
    MetaRing& meta = on_score_stream ? c->meta_score : c->meta_pre;
    if (on_score_stream) {
        // the tokens being scored were written by work already enqueued on the decode stream
        HIPCK(c, hipEventRecord(c->ev_dep, c->sd));
        HIPCK(c, hipStreamWaitEvent(c->ss, c->ev_dep, 0));
        if (!c->score_used) {
            HIPCK(c, hipEventRecord(c->ev_s0, c->ss));
            c->score_used = true;
        }
    }
    // sub-passes bounded by the workspace rows; a sample is never split
    int lo = 0;
    while (lo < n) {
        int hi = lo, T = 0;
        while (hi < n && T + c->smp[ids[hi]].P + c->smp[ids[hi]].gen_len <= c->ec.max_batch_tokens) {
            T += c->smp[ids[hi]].P + c->smp[ids[hi]].gen_len;
            ++hi;
        }
        for (int role = 0; role < 4; ++role)
            if (role_mask & RLHF_ROLE_BIT(role)) {
                int rc = score_pass(c, st, meta, ws, ids + lo, hi - lo, T, role);
                if (rc) return rc;
            }
        lo = hi;
    }
    if (on_score_stream) HIPCK(c, hipEventRecord(c->ev_score_last, c->ss));
    return RLHF_OK;
}

// Cut the un-scored part of the retired FIFO into batches of <= chunk tokens (at least one sample
// each): a batch closes once the next retired sample would not fit.  Flush the rest when
// generation is over.  Returns the number of batches closed.
int form_batches(rlhf_ctx* c, int chunk_tokens) {
    const long chunk = std::max(1, chunk_tokens);
    const bool done = c->waiting.empty() && c->active.empty();
    int closed = 0;
    for (;;) {
        size_t k = c->n_scored;
        long tok = 0;
        while (k < c->retired.size()) {
            const Sample& s = c->smp[c->retired[k]];
            const long t = s.P + s.gen_len;
            if (k > c->n_scored && tok + t > chunk) break;
            tok += t;
            ++k;
        }
        const bool full = k < c->retired.size();      // the next sample is there and does not fit
        if (k > c->n_scored && (full || done)) {
            c->n_scored = k;
            c->batch_offsets.push_back((int)k);
            c->batch_step.push_back(c->step - 1);
            ++closed;
        } else {
            break;
        }
    }
    return closed;
}

}  // namespace

extern "C" int rlhf_score(rlhf_ctx* c, int32_t n, const int32_t* sample_ids, uint32_t role_mask,
                          int32_t on_score_stream) {
    if (!c) return RLHF_EINVAL;
    if (n < 0 || (n > 0 && !sample_ids)) return c->fail(RLHF_EINVAL, "rlhf_score: bad arguments");
    if (role_mask & ~0xFu) return c->fail(RLHF_EINVAL, "rlhf_score: unknown role bits");
    return score_ids(c, sample_ids, n, role_mask, on_score_stream != 0);
}

// ================================================================================ run stage

namespace {
// A decode step is launch-bound when its chain of dependent kernels (about ten per layer, each
// at least ~5 us however small) takes longer than streaming the step's weights at ~5 TB/s.  Then
// a second stream has no idle bandwidth or matrix time to fill and only adds event traffic: the
// serial plan is the faster one (measured: 0.81x and 0.93x for the fused plan on the two small
// shapes, 1.03-1.05x on the three large ones).
bool decode_is_launch_bound(const rlhf_ctx* c) {
    const rlhf_model_cfg& m = c->mc;
    const double qd = (double)m.n_q_heads * m.head_dim, kvd = (double)m.n_kv_heads * m.head_dim;
    const double per_layer = (qd + 2 * kvd) * m.d_model + m.d_model * qd + 3.0 * m.d_model * m.ffn;
    const double stream_us = (m.n_layers * per_layer + (double)m.vocab * m.d_model) * c->esz / 5.0e6;
    const double launch_us = (10.0 * m.n_layers + 4) * 5.0;
    return stream_us < launch_us;
}
}  // namespace

extern "C" int rlhf_run_stage(rlhf_ctx* c, const rlhf_stage_opts* opts, rlhf_stage_stats* out) {
    if (!c) return RLHF_EINVAL;
    if (!opts) return c->fail(RLHF_EINVAL, "rlhf_run_stage: NULL options");
    if (opts->fused < 0 || opts->fused > 2) return c->fail(RLHF_EINVAL, "rlhf_run_stage: fused must be 0, 1 or 2");
    rlhf_stage_opts resolved = *opts;
    if (resolved.fused == 2) resolved.fused = decode_is_launch_bound(c) ? 0 : 1;
    const rlhf_stage_opts* o = &resolved;
    if (c->step != 0 || !c->retired.empty()) return c->fail(RLHF_ESTATE, "rlhf_run_stage: call rlhf_submit first");
    if (o->role_mask & ~0xFu) return c->fail(RLHF_EINVAL, "rlhf_run_stage: unknown role bits");
    const bool timing = o->trace_step_ms && o->trace_cap > 0;
    int rc = rlhf_sync(c);
    if (rc) return rc;
    const auto t0 = std::chrono::steady_clock::now();
    HIPCK(c, hipEventRecord(c->ev_d0, c->sd));
    const size_t first_batch = c->batch_step.size();
    int n_steps = 0;
    auto run_new_batches = [&](int closed) -> int {
        const size_t nb = c->batch_step.size();
        for (size_t b = nb - closed; b < nb; ++b) {
            const int lo = c->batch_offsets[b], hi = c->batch_offsets[b + 1];
            int r = score_ids(c, c->retired.data() + lo, hi - lo, o->role_mask, o->fused != 0);
            if (r) return r;
        }
        return RLHF_OK;
    };
    while (!c->waiting.empty() || !c->active.empty()) {
        if (c->sd_part) {
            // share the chip only while scoring work is actually in flight
            const bool scoring = c->score_used && hipEventQuery(c->ev_score_last) == hipErrorNotReady;
            rc = switch_stream(c, &c->sd, scoring ? c->sd_part : c->sd_full, c->ev_sw_d);
            if (rc) return rc;
        }
        if (timing && n_steps < o->trace_cap) {
            while ((int)c->step_events.size() < 2 * (n_steps + 1)) {
                hipEvent_t e;
                HIPCK(c, hipEventCreate(&e));
                c->step_events.push_back(e);
            }
            HIPCK(c, hipEventRecord(c->step_events[2 * n_steps], c->sd));
        }
        rlhf_step_info info;
        const int64_t bytes_before = c->acc_weight_bytes + c->acc_kv_bytes;
        rc = rlhf_generate_step(c, &info);
        if (rc) return rc;
        if (timing && n_steps < o->trace_cap) HIPCK(c, hipEventRecord(c->step_events[2 * n_steps + 1], c->sd));
        int nret;
        rc = rlhf_retire(c, nullptr, &nret);
        if (rc) return rc;
        if (n_steps < o->trace_cap) {
            if (o->trace_active) o->trace_active[n_steps] = (int)c->active.size();
            if (o->trace_decoded) o->trace_decoded[n_steps] = info.n_decoded;
            if (o->trace_prefill_tokens) o->trace_prefill_tokens[n_steps] = info.n_prefill_tokens;
            if (o->trace_step_bytes)
                o->trace_step_bytes[n_steps] = c->acc_weight_bytes + c->acc_kv_bytes - bytes_before;
        }
        ++n_steps;
        const int remaining = (int)(c->waiting.size() + c->active.size());
        if (o->fused && remaining > 0 && remaining < o->R_t) {
            rc = run_new_batches(form_batches(c, o->score_chunk_tokens));
            if (rc) return rc;
        }
    }
    HIPCK(c, hipEventRecord(c->ev_d1, c->sd));
    if ((rc = switch_stream(c, &c->sd, c->sd_full, c->ev_sw_d))) return rc;
    rc = run_new_batches(form_batches(c, o->score_chunk_tokens));   // generation is over: flush
    if (rc) return rc;
    if (c->score_used) HIPCK(c, hipEventRecord(c->ev_s1, c->ss));
    else HIPCK(c, hipEventRecord(c->ev_d1, c->sd));                  // serial scoring ran on the decode stream
    if ((rc = switch_stream(c, &c->ss, c->ss_full, c->ev_sw_s))) return rc;
    rc = rlhf_sync(c);
    if (rc) return rc;
    const auto t1 = std::chrono::steady_clock::now();
    if (c->prof.on) HIPCK(c, profiler_fold(c->prof));
    if (timing)
        for (int s = 0; s < std::min(n_steps, o->trace_cap); ++s)
            HIPCK(c, hipEventElapsedTime(&o->trace_step_ms[s], c->step_events[2 * s], c->step_events[2 * s + 1]));
    if (out) {
        memset(out, 0, sizeof *out);
        out->n_steps = n_steps;
        out->n_batches = (int)(c->batch_step.size() - first_batch);
        for (const Sample& s : c->smp) {
            out->generated_tokens += s.gen_len;
            out->scored_tokens += s.P + s.gen_len;
        }
        out->prefill_tokens = c->acc_prefill_tokens;
        out->wall_ms = std::chrono::duration<double, std::milli>(t1 - t0).count();
        float ms = 0.f;
        HIPCK(c, hipEventElapsedTime(&ms, c->ev_d0, c->ev_d1));
        out->decode_stream_ms = ms;
        if (c->score_used) {
            HIPCK(c, hipEventElapsedTime(&ms, c->ev_s0, c->ev_s1));
            out->score_stream_ms = ms;
        }
        out->decode_weight_bytes = c->acc_weight_bytes;
        out->decode_kv_bytes = c->acc_kv_bytes;
        out->fused_used = o->fused;
    }
    return RLHF_OK;
}

// ======================================================================== results / snapshot

extern "C" int rlhf_get_results(rlhf_ctx* c, rlhf_results* out) {
    if (!c) return RLHF_EINVAL;
    if (!out) return c->fail(RLHF_EINVAL, "rlhf_get_results: NULL");
    int rc = rlhf_sync(c);
    if (rc) return rc;
    const int n = c->N, mc = c->ec.max_ctx;
    int64_t total = 0;
    for (int i = 0; i < n; ++i) total += c->smp[i].gen_len;
    const bool packed = out->tokens || out->lp_actor || out->lp_actor_rescored || out->lp_ref || out->values;
    if (packed && out->packed_capacity < total)
        return c->fail(RLHF_EINVAL, "rlhf_get_results: packed_capacity %lld < %lld", (long long)out->packed_capacity, (long long)total);
    if (out->gen_len)
        for (int i = 0; i < n; ++i) out->gen_len[i] = c->smp[i].gen_len;
    if (out->resp_offsets) {
        out->resp_offsets[0] = 0;
        for (int i = 0; i < n; ++i) out->resp_offsets[i + 1] = out->resp_offsets[i] + c->smp[i].gen_len;
    }
    std::vector<float> buf;
    auto fetch_packed = [&](const float* dsrc, float* dst) -> int {
        if (!dst || n == 0) return RLHF_OK;
        buf.resize((size_t)n * mc);
        HIPCK(c, hipMemcpy(buf.data(), dsrc, buf.size() * 4, hipMemcpyDeviceToHost));
        int64_t o = 0;
        for (int i = 0; i < n; ++i) {
            std::copy(buf.begin() + (size_t)i * mc, buf.begin() + (size_t)i * mc + c->smp[i].gen_len, dst + o);
            o += c->smp[i].gen_len;
        }
        return RLHF_OK;
    };
    if ((rc = fetch_packed(c->d_lp_actor, out->lp_actor))) return rc;
    if ((rc = fetch_packed(c->d_lp_rescored, out->lp_actor_rescored))) return rc;
    if ((rc = fetch_packed(c->d_lp_ref, out->lp_ref))) return rc;
    if ((rc = fetch_packed(c->d_values, out->values))) return rc;
    if (out->tokens && n) {
        std::vector<int> tb((size_t)n * mc);
        HIPCK(c, hipMemcpy(tb.data(), c->d_tokens, tb.size() * sizeof(int), hipMemcpyDeviceToHost));
        int64_t o = 0;
        for (int i = 0; i < n; ++i) {
            const Sample& s = c->smp[i];
            std::copy(tb.begin() + (size_t)i * mc + s.P, tb.begin() + (size_t)i * mc + s.P + s.gen_len, out->tokens + o);
            o += s.gen_len;
        }
    }
    if (out->reward && n) HIPCK(c, hipMemcpy(out->reward, c->d_reward, (size_t)n * 4, hipMemcpyDeviceToHost));
    // The 16-bit activation path has no scaling: a model whose activations leave IEEE half's range
    // (|x| > 65504) produces infinities and then NaNs.  Every kernel that writes a result raises
    // this flag when the value is not finite; the outputs above are still delivered.
    int bad = 0;
    HIPCK(c, hipMemcpy(&bad, c->d_nonfinite, sizeof(int), hipMemcpyDeviceToHost));
    if (bad)
        return c->fail(RLHF_ENONFINITE, "rlhf_get_results: a log-prob, value or reward of this stage is not finite "
                                        "(activations outside the range of the 16-bit path?)");
    return RLHF_OK;
}

extern "C" int rlhf_debug_snapshot(rlhf_ctx* c, rlhf_snapshot* o) {
    if (!c) return RLHF_EINVAL;
    if (!o) return c->fail(RLHF_EINVAL, "rlhf_debug_snapshot: NULL");
    const int n = c->N;
    o->step = c->step;
    o->n_samples = n;
    o->n_waiting = (int)c->waiting.size();
    o->n_active = (int)c->active.size();
    o->n_retired = (int)c->retired.size();
    o->n_batches = (int)c->batch_step.size();
    o->n_free = (int)c->free_list.size();
    o->reserved_pages = c->reserved;
    o->pool_pages = c->pool_pages;
    o->max_pages = c->max_pages;
    if (o->cap_samples < n || o->cap_max_pages < c->max_pages ||
        (o->free_list && o->cap_pool_pages < c->pool_pages))
        return c->fail(RLHF_EINVAL, "rlhf_debug_snapshot: capacities too small (need %d samples, %d pages/sample, %d pool pages)",
                       n, c->max_pages, c->pool_pages);
    if (o->active) std::copy(c->active.begin(), c->active.end(), o->active);
    for (int i = 0; i < n; ++i) {
        const Sample& s = c->smp[i];
        if (o->ctx) o->ctx[i] = s.ctx;
        if (o->gen_len) o->gen_len[i] = s.gen_len;
        if (o->n_pages) o->n_pages[i] = (int)s.pages.size();
        if (o->page_table) {
            int* row = o->page_table + (size_t)i * o->cap_max_pages;
            std::fill(row, row + o->cap_max_pages, -1);
            std::copy(s.pages.begin(), s.pages.end(), row);
        }
    }
    if (o->free_list) std::copy(c->free_list.begin(), c->free_list.end(), o->free_list);
    if (o->retired) std::copy(c->retired.begin(), c->retired.end(), o->retired);
    if (o->batch_offsets) std::copy(c->batch_offsets.begin(), c->batch_offsets.end(), o->batch_offsets);
    if (o->batch_step) std::copy(c->batch_step.begin(), c->batch_step.end(), o->batch_step);
    return RLHF_OK;
}

// ====================================================================================== GAE

extern "C" int rlhf_compute_gae(rlhf_ctx* c, float gamma, float lam, float kl_coef, float* advantages,
                                float* returns, int64_t packed_capacity) {
    if (!c) return RLHF_EINVAL;
    if (!(gamma >= 0.f && gamma <= 1.f) || !(lam >= 0.f && lam <= 1.f))
        return c->fail(RLHF_EINVAL, "rlhf_compute_gae: gamma and lam must be in [0, 1]");
    int rc = rlhf_sync(c);
    if (rc) return rc;
    const int n = c->N, mc = c->ec.max_ctx;
    int64_t total = 0;
    int Lmax = 0;
    std::vector<int> gl(n);
    for (int i = 0; i < n; ++i) {
        const Sample& s = c->smp[i];
        if (!sample_done(s) || s.gen_len < 1) return c->fail(RLHF_ESTATE, "rlhf_compute_gae: sample %d is not finished", i);
        gl[i] = s.gen_len;
        total += s.gen_len;
        Lmax = std::max(Lmax, s.gen_len);
    }
    if ((advantages || returns) && packed_capacity < total)
        return c->fail(RLHF_EINVAL, "rlhf_compute_gae: packed_capacity %lld < %lld", (long long)packed_capacity, (long long)total);
    if (n == 0) return RLHF_OK;
    const int Lp = (Lmax + 15) / 16 * 16;
    float *D = nullptr, *U = nullptr, *A = nullptr, *R = nullptr;
    int* d_gl = nullptr;
    auto cleanup = [&] { for (void* p : {(void*)D, (void*)U, (void*)A, (void*)R, (void*)d_gl}) if (p) (void)hipFree(p); };
#define GAECK(call)                                                                              \
    do {                                                                                         \
        hipError_t e_ = (call);                                                                  \
        if (e_ != hipSuccess) { cleanup(); return c->fail(RLHF_EDEVICE, "%s failed: %s", #call, hipGetErrorString(e_)); } \
    } while (0)
    GAECK(hipMalloc((void**)&D, (size_t)n * Lp * 4));
    GAECK(hipMalloc((void**)&A, (size_t)n * Lp * 4));
    GAECK(hipMalloc((void**)&R, (size_t)n * Lp * 4));
    GAECK(hipMalloc((void**)&U, (size_t)Lp * Lp * 4));
    GAECK(hipMalloc((void**)&d_gl, (size_t)n * sizeof(int)));
    GAECK(hipMemcpyAsync(d_gl, gl.data(), (size_t)n * sizeof(int), hipMemcpyHostToDevice, c->sd));
    GAECK(launch_gae_delta(c->sd, c->d_lp_actor, c->d_lp_ref, c->d_values, c->d_reward, d_gl, mc, gamma, kl_coef, D, n, Lp));
    GAECK(launch_gae_matrix(c->sd, U, Lp, (double)gamma * (double)lam));
    GAECK(launch_gemm(c->sd, kF32, kF32, D, U, A, n, Lp, Lp, 1));          // A = D U^T, one matrix multiply
    GAECK(launch_gae_returns(c->sd, A, c->d_values, d_gl, mc, R, n, Lp));
    std::vector<float> ha((size_t)n * Lp), hr((size_t)n * Lp);
    GAECK(hipMemcpyAsync(ha.data(), A, ha.size() * 4, hipMemcpyDeviceToHost, c->sd));
    GAECK(hipMemcpyAsync(hr.data(), R, hr.size() * 4, hipMemcpyDeviceToHost, c->sd));
    GAECK(hipStreamSynchronize(c->sd));
#undef GAECK
    cleanup();
    int64_t o = 0;
    for (int i = 0; i < n; ++i) {
        if (advantages) std::copy(ha.begin() + (size_t)i * Lp, ha.begin() + (size_t)i * Lp + gl[i], advantages + o);
        if (returns) std::copy(hr.begin() + (size_t)i * Lp, hr.begin() + (size_t)i * Lp + gl[i], returns + o);
        o += gl[i];
    }
    return RLHF_OK;
}

// ================================================================================ profiling

extern "C" int rlhf_profile_begin(rlhf_ctx* c, int32_t sample_every) {
    if (!c) return RLHF_EINVAL;
    if (sample_every < 1) return c->fail(RLHF_EINVAL, "rlhf_profile_begin: sample_every must be >= 1");
    int rc = rlhf_sync(c);
    if (rc) return rc;
    Profiler& p = c->prof;
    p.on = true;
    p.every = sample_every;
    p.n_used = 0;
    for (int k = 0; k < kClassCount; ++k) {
        p.launches[k] = p.sampled[k] = p.dropped[k] = 0;
        p.tot_bytes[k] = p.tot_flops[k] = p.s_ms[k] = p.s_bytes[k] = p.s_flops[k] = 0;
    }
    {   // What a bracket costs beyond the kernels inside it.  A bracket around one empty kernel takes
        // overhead + d, around two of them overhead + 2 d (d = an empty kernel with its dispatch gap), so
        // overhead = 2 t1 - t2, from the medians of 33 brackets of each kind, taken alternately.
        constexpr int kCal = 33;
        hipEvent_t ev[4 * kCal];
        for (hipEvent_t& e : ev) HIPCK(c, hipEventCreate(&e));
        for (int i = 0; i < 2 * kCal; ++i) {
            HIPCK(c, hipEventRecord(ev[2 * i], c->sd));
            HIPCK(c, launch_noop(c->sd));
            if (i & 1) HIPCK(c, launch_noop(c->sd));
            HIPCK(c, hipEventRecord(ev[2 * i + 1], c->sd));
        }
        HIPCK(c, hipStreamSynchronize(c->sd));
        float one[kCal], two[kCal];
        for (int i = 0; i < 2 * kCal; ++i)
            HIPCK(c, hipEventElapsedTime((i & 1) ? &two[i / 2] : &one[i / 2], ev[2 * i], ev[2 * i + 1]));
        std::sort(one, one + kCal);
        std::sort(two, two + kCal);
        p.bracket_overhead_ms = std::max(0.0, 2.0 * one[kCal / 2] - two[kCal / 2]);
        for (hipEvent_t e : ev) (void)hipEventDestroy(e);
    }
    return RLHF_OK;
}

extern "C" int rlhf_profile_end(rlhf_ctx* c, rlhf_kernel_profile* out) {
    if (!c) return RLHF_EINVAL;
    if (!out) return c->fail(RLHF_EINVAL, "rlhf_profile_end: NULL");
    int rc = rlhf_sync(c);
    if (rc) return rc;
    Profiler& p = c->prof;
    p.on = false;
    HIPCK(c, profiler_fold(p));
    for (int k = 0; k < kClassCount; ++k) {
        memset(&out[k], 0, sizeof out[k]);
        out[k].launches = p.launches[k];
        out[k].total_bytes = p.tot_bytes[k];
        out[k].total_flops = p.tot_flops[k];
        out[k].sampled = p.sampled[k];
        out[k].sampled_ms = p.s_ms[k];
        out[k].sampled_bytes = p.s_bytes[k];
        out[k].sampled_flops = p.s_flops[k];
        out[k].dropped = p.dropped[k];
        out[k].bracket_overhead_ms = p.bracket_overhead_ms;
    }
    return RLHF_OK;
}
