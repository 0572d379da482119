// Attention kernels.
//
// Decode (the memory-bound phase of Section 2.2 / 4.2): one query per active sample against
// that sample's paged K/V.  A workgroup owns (sample, KV head, split); its four waves take the
// pages of the split round-robin.  A page's K tile ([page_tokens][hd], contiguous) is read
// with 16-byte loads, consecutive lanes on consecutive chunks; a lane holds 8 dims of one
// token, the q.k dot product is finished with xor-shuffles inside the hd/8-lane group, and
// the softmax runs online in float.  Each lane accumulates p*V for its own tokens; lanes are
// merged by shuffles at the end, waves through LDS, splits by a small merge kernel (LSE
// merge), so that a few long samples still spread over the whole chip.
//
// With eight query heads per KV head (half precision) the decode kernel is an MFMA one, see
// k_decode_attn_gqa.
//
// Prefill / scoring of float models uses the same inner loop over 16-token tiles of contiguous
// K/V (one workgroup per query row and KV head); bf16 models use the MFMA kernel at the end of
// this file.
#include "common.h"
#include "kernels.h"

namespace rlhf {

constexpr int kPT = 16;  // tokens per page / tile

template <typename T> struct Chunk;           // 8 elements of T held raw
template <> struct Chunk<bf16_t> { uint4 r; };
template <> struct Chunk<f16_t> { uint4 r; };
template <> struct Chunk<float> { float4 a, b; };

// A decode step reads every cached K and V once: the loads are non-temporal (evict first), so that
// the KV stream does not push out of the L2 what a GEMM on the other stream keeps there.
typedef uint32_t u32x4_nt_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld_stream16(const void* p) {
    const u32x4_nt_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt_t*>(p));
    return make_uint4(v[0], v[1], v[2], v[3]);
}
template <typename T> __device__ __forceinline__ Chunk<T> ld_chunk(const T* p);
template <> __device__ __forceinline__ Chunk<bf16_t> ld_chunk<bf16_t>(const bf16_t* p) {
    Chunk<bf16_t> c; c.r = ld_stream16(p); return c;
}
template <> __device__ __forceinline__ Chunk<f16_t> ld_chunk<f16_t>(const f16_t* p) {
    Chunk<f16_t> c; c.r = ld_stream16(p); return c;
}
template <> __device__ __forceinline__ Chunk<float> ld_chunk<float>(const float* p) {
    Chunk<float> c;
    c.a = *reinterpret_cast<const float4*>(p);
    c.b = *reinterpret_cast<const float4*>(p + 4);
    return c;
}
template <typename T> __device__ __forceinline__ void unpack(const Chunk<T>& c, float (&o)[8]);
template <> __device__ __forceinline__ void unpack<bf16_t>(const Chunk<bf16_t>& c, float (&o)[8]) {
    o[0] = __uint_as_float(c.r.x << 16); o[1] = __uint_as_float(c.r.x & 0xFFFF0000u);
    o[2] = __uint_as_float(c.r.y << 16); o[3] = __uint_as_float(c.r.y & 0xFFFF0000u);
    o[4] = __uint_as_float(c.r.z << 16); o[5] = __uint_as_float(c.r.z & 0xFFFF0000u);
    o[6] = __uint_as_float(c.r.w << 16); o[7] = __uint_as_float(c.r.w & 0xFFFF0000u);
}
template <> __device__ __forceinline__ void unpack<f16_t>(const Chunk<f16_t>& c, float (&o)[8]) {
    const f16x8_t h = *reinterpret_cast<const f16x8_t*>(&c.r);
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (float)h[e];
}
template <> __device__ __forceinline__ void unpack<float>(const Chunk<float>& c, float (&o)[8]) {
    o[0] = c.a.x; o[1] = c.a.y; o[2] = c.a.z; o[3] = c.a.w;
    o[4] = c.b.x; o[5] = c.b.y; o[6] = c.b.z; o[7] = c.b.w;
}

// Per-lane running softmax state for one query head.
struct HeadState {
    float m, l;
    float acc[8];
};

// Process one tile of up to 16 tokens for G query heads.  HD/8 lanes share a token (each 8
// dims); TPP tokens per pass; PASSES passes cover the tile.
//   kt, vt : tile bases (token 0, dim 0) with token stride `tstride` elements
//   n_valid: tokens of this tile that exist (1..16)
template <typename T, int HD> struct TileRegs {      // one tile's K and V chunks of a lane
    static constexpr int PASSES = kPT / (64 / (HD / 8));
    Chunk<T> kc[PASSES], vc[PASSES];
};

template <typename T, int HD>
__device__ __forceinline__ void load_tile(const T* __restrict__ kt, const T* __restrict__ vt, size_t tstride,
                                          int n_valid, int lane, TileRegs<T, HD>& tr) {
    constexpr int CPT = HD / 8, TPP = 64 / CPT, PASSES = kPT / TPP;
    const int dc = lane % CPT, tsub = lane / CPT;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int tok = p * TPP + tsub;
        const int tk = tok < n_valid ? tok : 0;   // clamp: keep the load in bounds, mask below
        tr.kc[p] = ld_chunk<T>(kt + (size_t)tk * tstride + dc * 8);
        tr.vc[p] = ld_chunk<T>(vt + (size_t)tk * tstride + dc * 8);
    }
}

template <typename T, int HD, int G>
__device__ __forceinline__ void consume_tile(const TileRegs<T, HD>& tr, int n_valid, const float (&q)[G][8],
                                             HeadState (&st)[G], int lane) {
    constexpr int CPT = HD / 8, TPP = 64 / CPT, PASSES = kPT / TPP;
    const int tsub = lane / CPT;
    const Chunk<T>(&kc)[PASSES] = tr.kc;
    const Chunk<T>(&vc)[PASSES] = tr.vc;
    float s[G][PASSES];
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        float kf[8];
        unpack<T>(kc[p], kf);
        const bool valid = (p * TPP + tsub) < n_valid;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) d += q[g][e] * kf[e];
#pragma unroll
            for (int o = 1; o < CPT; o <<= 1) d += __shfl_xor(d, o, kWave);
            s[g][p] = valid ? d : -INFINITY;
        }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float mx = s[g][0];
#pragma unroll
        for (int p = 1; p < PASSES; ++p) mx = fmaxf(mx, s[g][p]);
#pragma unroll
        for (int o = CPT; o < 64; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o, kWave));
        const float m_new = fmaxf(st[g].m, mx);            // finite: token 0 of a tile is valid
        const float alpha = __expf(st[g].m - m_new);       // exp(-inf) = 0 on the first tile
        st[g].m = m_new;
        st[g].l *= alpha;
#pragma unroll
        for (int e = 0; e < 8; ++e) st[g].acc[e] *= alpha;
#pragma unroll
        for (int p = 0; p < PASSES; ++p) s[g][p] = __expf(s[g][p] - m_new);
    }
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        float vf[8];
        unpack<T>(vc[p], vf);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            st[g].l += s[g][p];
#pragma unroll
            for (int e = 0; e < 8; ++e) st[g].acc[e] += s[g][p] * vf[e];
        }
    }
}

template <typename T, int HD, int G>
__device__ __forceinline__ void attend_tile(const T* __restrict__ kt, const T* __restrict__ vt,
                                            size_t tstride, int n_valid, const float (&q)[G][8],
                                            HeadState (&st)[G], int lane) {
    TileRegs<T, HD> tr;
    load_tile<T, HD>(kt, vt, tstride, n_valid, lane, tr);
    consume_tile<T, HD, G>(tr, n_valid, q, st, lane);
}

// Merge lanes (token sub-groups) of a wave, then the four waves through LDS.  On return,
// threads with (wave 0 .. ) hold nothing special: results are in sm/sl/sacc for all G heads:
//   sm[g], sl[g], sacc[g][HD] = block-wide max, sum, un-normalised accumulator.
template <int HD, int G>
__device__ __forceinline__ void block_merge(HeadState (&st)[G], int lane, int wave, float* s_m,
                                            float* s_l, float* s_acc /*[4][G][HD]*/) {
    constexpr int CPT = HD / 8;
    const int dc = lane % CPT;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        // every lane of the wave already shares m; l and acc are per token sub-group
        float l = st[g].l;
#pragma unroll
        for (int o = CPT; o < 64; o <<= 1) l += __shfl_xor(l, o, kWave);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float a = st[g].acc[e];
#pragma unroll
            for (int o = CPT; o < 64; o <<= 1) a += __shfl_xor(a, o, kWave);
            if (lane < CPT) s_acc[(wave * G + g) * HD + dc * 8 + e] = a;
        }
        if (lane == 0) { s_m[wave * G + g] = st[g].m; s_l[wave * G + g] = l; }
    }
    __syncthreads();
}

// After the waves' (max, sum, accumulator) sit in LDS: merge them and write either the output
// row or this split's partial.
template <typename T, int HD, int G>
__device__ __forceinline__ void decode_block_finish(const float* s_m, const float* s_l, const float* s_acc,
                                                    int r, int kh, int split, int nsplit, int Hq,
                                                    T* __restrict__ out, float* __restrict__ part_acc,
                                                    float* __restrict__ part_ml) {
    for (int i = threadIdx.x; i < G * HD; i += 256) {
        const int g = i / HD, e = i - g * HD;
        float mt = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) mt = fmaxf(mt, s_m[w * G + g]);
        float lt = 0.f, at = 0.f;
        if (mt > -INFINITY) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float f = __expf(s_m[w * G + g] - mt);
                lt += s_l[w * G + g] * f;
                at += s_acc[(w * G + g) * HD + e] * f;
            }
        }
        const int h = kh * G + g;
        if (nsplit == 1) {
            out[((size_t)r * Hq + h) * HD + e] = from_f32<T>(at / lt);
        } else {
            const size_t slot = ((size_t)r * Hq + h) * nsplit + split;
            part_acc[slot * HD + e] = at;
            if (e == 0) { part_ml[slot * 2] = mt; part_ml[slot * 2 + 1] = lt; }
        }
    }
}

template <typename T, int HD, int G>
__global__ __launch_bounds__(256) void k_decode_attn(const T* __restrict__ q,
                                                     const T* __restrict__ pool,
                                                     const int* __restrict__ page_table,
                                                     int pt_stride,
                                                     const int* __restrict__ row_sample,
                                                     const int* __restrict__ ctx_len,
                                                     T* __restrict__ out, float* __restrict__ part_acc,
                                                     float* __restrict__ part_ml, int layer,
                                                     int nsplit, int n_layers, int Hkv) {
    __shared__ float s_m[4 * G], s_l[4 * G];
    __shared__ float s_acc[4 * G * HD];
    const int r = blockIdx.x, kh = blockIdx.y, split = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int Hq = Hkv * G;
    const int ctx = ctx_len[r];
    const int n_pages = (ctx + kPT - 1) / kPT;
    const int pps = (n_pages + nsplit - 1) / nsplit;
    const int pb = split * pps, pe = min(n_pages, pb + pps);
    const int* pt = page_table + (size_t)row_sample[r] * pt_stride;
    constexpr int CPT = HD / 8;
    const int dc = lane % CPT;
    const float scale = rsqrtf((float)HD);

    float qf[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        load8<T>(q + ((size_t)r * Hq + kh * G + g) * HD + dc * 8, qf[g]);
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[g][e] *= scale;
    }
    HeadState st[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        st[g].m = -INFINITY; st[g].l = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) st[g].acc[e] = 0.f;
    }
    const size_t page_elems = (size_t)n_layers * 2 * Hkv * kPT * HD;
    const size_t head_off = ((size_t)layer * 2 * Hkv + kh) * kPT * HD;
    const size_t v_off = (size_t)Hkv * kPT * HD;
    // A wave walks pages pb + wave, + 4, ...  The page index of the next tile is fetched before
    // this tile's K and V, so that a tile costs one memory round trip instead of two dependent
    // ones.  (Fetching K and V a tile ahead as well was measured: 120 registers instead of 73, the
    // kernel no longer fits beside a scoring workgroup on a compute unit, and the stage is slower.)
    int pi = pb + wave;
    int page = pi < pe ? pt[pi] : 0;
    for (; pi < pe; pi += 4) {
        const int page_next = pi + 4 < pe ? pt[pi + 4] : 0;
        const T* kt = pool + (size_t)page * page_elems + head_off;
        attend_tile<T, HD, G>(kt, kt + v_off, (size_t)HD, min(kPT, ctx - pi * kPT), qf, st, lane);
        page = page_next;
    }
    block_merge<HD, G>(st, lane, wave, s_m, s_l, s_acc);
    decode_block_finish<T, HD, G>(s_m, s_l, s_acc, r, kh, split, nsplit, Hq, out, part_acc, part_ml);
}

// ------------------------------------------------- decode attention for grouped KV heads, MFMA
// With G query heads per KV head the VALU kernel above spends its time in the per-head dot
// products and their shuffles.  Here a wave handles a 16-token page with matrix instructions:
//   S^T[token][head] = K[token][:] . Q[head][:]      4 x mfma 16x16x32 (heads padded to 16)
//   O^T[dim][head]  += V^T[dim][token] P^T[token][head]      8 x mfma 16x16x16, one per 16 dims
// The first product leaves a lane with four consecutive tokens of ONE head (head = lane % 16),
// which is both what the online softmax needs (a head's state lives in its own lanes; the row
// maximum and sum cross the four token groups with two xor-shuffles) and, rounded to half, the
// second product's right operand.  Its left operand wants four tokens of one dim per lane while
// memory holds eight dims of one token per 16 bytes, so the V page is staged in LDS by rows
// (row pitch 264 bytes: the four token groups of a read fall into different banks) and read back
// transposed.  The second product leaves a lane with dims of its own head again, so rescaling by
// the softmax correction needs no exchange.  Waves take pages round-robin and are merged, like the
// splits, by (max, sum, accumulator).
typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));

template <int HD, int G>
__global__ __launch_bounds__(256) void k_decode_attn_gqa(const f16_t* __restrict__ q,
                                                         const f16_t* __restrict__ pool,
                                                         const int* __restrict__ page_table, int pt_stride,
                                                         const int* __restrict__ row_sample,
                                                         const int* __restrict__ ctx_len,
                                                         f16_t* __restrict__ out, float* __restrict__ part_acc,
                                                         float* __restrict__ part_ml, int layer, int nsplit,
                                                         int n_layers, int Hkv) {
    static_assert(HD == 128 && G <= 16, "one 16-wide head block, eight 16-dim blocks");
    constexpr int VROW = HD + 4;                       // halves per staged V row (264 bytes)
    constexpr int kStage = 16 * VROW / 2;              // floats per wave of staging
    constexpr int kBuf = 4 * G * HD > 4 * kStage ? 4 * G * HD : 4 * kStage;
    __shared__ float s_m[4 * G], s_l[4 * G];
    __shared__ __attribute__((aligned(16))) float s_buf[kBuf];   // V staging, then the waves' accumulators
    const int r = blockIdx.x, kh = blockIdx.y, split = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int head = lane & 15, tg = lane >> 4;        // the lane's head (or token, or dim) and token group
    const int Hq = Hkv * G;
    const int ctx = ctx_len[r];
    const int n_pages = (ctx + kPT - 1) / kPT;
    const int pps = (n_pages + nsplit - 1) / nsplit;
    const int pb = split * pps, pe = min(n_pages, pb + pps);
    const int* pt = page_table + (size_t)row_sample[r] * pt_stride;
    const float scale = rsqrtf((float)HD);
    const size_t page_elems = (size_t)n_layers * 2 * Hkv * kPT * HD;
    const size_t head_off = ((size_t)layer * 2 * Hkv + kh) * kPT * HD;
    const size_t v_off = (size_t)Hkv * kPT * HD;

    f16x8_t qb[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        qb[ks] = f16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
        if (head < G)
            qb[ks] = *reinterpret_cast<const f16x8_t*>(q + ((size_t)r * Hq + kh * G + head) * HD + ks * 32 + tg * 8);
    }
    float m = -INFINITY, l = 0.f;
    f32x4_t o[8];
#pragma unroll
    for (int b = 0; b < 8; ++b) o[b] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    f16_t* vs = reinterpret_cast<f16_t*>(s_buf) + wave * 16 * VROW;

    int page = pb + wave < pe ? pt[pb + wave] : 0;      // page indices are fetched one tile ahead
    for (int pi = pb + wave; pi < pe; pi += 4) {
        const f16_t* kt = pool + (size_t)page * page_elems + head_off;
        const f16_t* vt = kt + v_off;
        page = pi + 4 < pe ? pt[pi + 4] : 0;
        const int n_valid = min(kPT, ctx - pi * kPT);
        // tokens past the context are read from token 0 (finite data) and masked below
        const int tk = head < n_valid ? head : 0;
        f16x8_t ka[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            ka[ks] = __builtin_nontemporal_load(reinterpret_cast<const f16x8_t*>(kt + (size_t)tk * HD + ks * 32 + tg * 8));
        uint2 vr[4][2];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int tok = i * 4 + tg;
            const uint4 x = ld_stream16(vt + (size_t)(tok < n_valid ? tok : 0) * HD + head * 8);
            vr[i][0] = make_uint2(x.x, x.y);
            vr[i][1] = make_uint2(x.z, x.w);
        }
        f32x4_t st = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) st = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka[ks], qb[ks], st, 0, 0, 0);
        float sc[4], mx = -INFINITY;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            sc[e] = tg * 4 + e < n_valid ? st[e] * scale : -INFINITY;
            mx = fmaxf(mx, sc[e]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
        mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
        const float m_new = fmaxf(m, mx);               // finite: token 0 of a page is valid
        const float alpha = __expf(m - m_new);          // exp(-inf) = 0 on the first page
        float ls = 0.f;
        f16x4_t pa;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float p = __expf(sc[e] - m_new);
            ls += p;
            pa[e] = (f16_t)p;
        }
        ls += __shfl_xor(ls, 16, kWave);
        ls += __shfl_xor(ls, 32, kWave);
        l = l * alpha + ls;
        m = m_new;
#pragma unroll
        for (int b = 0; b < 8; ++b)
#pragma unroll
            for (int e = 0; e < 4; ++e) o[b][e] *= alpha;
        // stage the page's V rows, then read them back with tokens along the lane's four values
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f16_t* dst = vs + (i * 4 + tg) * VROW + head * 8;
            *reinterpret_cast<uint2*>(dst) = vr[i][0];
            *reinterpret_cast<uint2*>(dst + 4) = vr[i][1];
        }
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            f16x4_t va;
#pragma unroll
            for (int e = 0; e < 4; ++e) va[e] = vs[(tg * 4 + e) * VROW + b * 16 + head];
            o[b] = __builtin_amdgcn_mfma_f32_16x16x16f16(va, pa, o[b], 0, 0, 0);
        }
    }
    __syncthreads();                                    // every wave is done with its staging rows
    float* s_acc = s_buf;
    if (head < G) {
        if (tg == 0) { s_m[wave * G + head] = m; s_l[wave * G + head] = l; }
#pragma unroll
        for (int b = 0; b < 8; ++b)
#pragma unroll
            for (int e = 0; e < 4; ++e) s_acc[(wave * G + head) * HD + b * 16 + tg * 4 + e] = o[b][e];
    }
    __syncthreads();
    decode_block_finish<f16_t, HD, G>(s_m, s_l, s_acc, r, kh, split, nsplit, Hq, out, part_acc, part_ml);
}

// LSE merge of the split partials: one block per (row, head), HD threads.
template <typename T>
__global__ void k_attn_merge(const float* __restrict__ part_acc, const float* __restrict__ part_ml,
                             T* __restrict__ out, int nsplit, int HD) {
    const size_t rh = blockIdx.x;
    const int e = threadIdx.x;
    float mt = -INFINITY;
    for (int s = 0; s < nsplit; ++s) mt = fmaxf(mt, part_ml[(rh * nsplit + s) * 2]);
    float lt = 0.f, at = 0.f;
    for (int s = 0; s < nsplit; ++s) {
        const float m = part_ml[(rh * nsplit + s) * 2];
        if (m == -INFINITY) continue;
        const float f = __expf(m - mt);
        lt += part_ml[(rh * nsplit + s) * 2 + 1] * f;
        at += part_acc[(rh * nsplit + s) * HD + e] * f;
    }
    out[rh * HD + e] = from_f32<T>(at / lt);
}

template <typename T, int HD, int G>
static hipError_t decode_launch(hipStream_t st, const void* q, const void* pool,
                                const int* page_table, int pt_stride, const int* row_sample,
                                const int* ctx_len, void* out, float* part_acc, float* part_ml,
                                int rows, int layer, int nsplit, const Dims& dm) {
    dim3 grid(rows, dm.n_kv_heads, nsplit);
    k_decode_attn<T, HD, G><<<grid, 256, 0, st>>>((const T*)q, (const T*)pool, page_table, pt_stride,
                                                  row_sample, ctx_len, (T*)out, part_acc, part_ml,
                                                  layer, nsplit, dm.n_layers, dm.n_kv_heads);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || nsplit == 1) return e;
    k_attn_merge<T><<<rows * dm.n_q_heads, HD, 0, st>>>(part_acc, part_ml, (T*)out, nsplit, HD);
    return hipGetLastError();
}

hipError_t launch_decode_attn(hipStream_t st, int dtype, const void* q, const void* pool,
                              const int* page_table, int pt_stride, const int* row_sample,
                              const int* ctx_len, void* out, float* part_acc, float* part_ml,
                              int rows, int layer, int nsplit, const Dims& dm) {
    if (rows <= 0) return hipSuccess;
    if (dm.page_tokens != kPT || nsplit < 1) return hipErrorInvalidValue;
    const int G = dm.n_q_heads / dm.n_kv_heads, hd = dm.head_dim;
#define RLHF_DEC(TT, HD_, G_)                                                                     \
    return decode_launch<TT, HD_, G_>(st, q, pool, page_table, pt_stride, row_sample, ctx_len, out, \
                                      part_acc, part_ml, rows, layer, nsplit, dm)
    if (dtype == kBF16) {
        if (hd == 128 && G == 1) RLHF_DEC(bf16_t, 128, 1);
        if (hd == 128 && G == 8) RLHF_DEC(bf16_t, 128, 8);
        if (hd == 64 && G == 1) RLHF_DEC(bf16_t, 64, 1);
    } else if (dtype == kF16) {
        if (hd == 128 && G == 1) RLHF_DEC(f16_t, 128, 1);
        if (hd == 128 && G == 8) {
            dim3 grid(rows, dm.n_kv_heads, nsplit);
            k_decode_attn_gqa<128, 8><<<grid, 256, 0, st>>>((const f16_t*)q, (const f16_t*)pool, page_table, pt_stride,
                                                            row_sample, ctx_len, (f16_t*)out, part_acc, part_ml, layer,
                                                            nsplit, dm.n_layers, dm.n_kv_heads);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess || nsplit == 1) return e;
            k_attn_merge<f16_t><<<rows * dm.n_q_heads, 128, 0, st>>>(part_acc, part_ml, (f16_t*)out, nsplit, 128);
            return hipGetLastError();
        }
        if (hd == 64 && G == 1) RLHF_DEC(f16_t, 64, 1);
    } else {
        if (hd == 128 && G == 1) RLHF_DEC(float, 128, 1);
        if (hd == 64 && G == 1) RLHF_DEC(float, 64, 1);
    }
#undef RLHF_DEC
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------- prefill / scoring (v1)
template <typename TO, int HD, int G>
__global__ __launch_bounds__(256) void k_prefill_attn(const float* __restrict__ q,
                                                      const float* __restrict__ k,
                                                      const float* __restrict__ v,
                                                      const int* __restrict__ row_start,
                                                      const int* __restrict__ row_pos,
                                                      TO* __restrict__ out, int Hkv) {
    typedef float T;
    __shared__ float s_m[4 * G], s_l[4 * G];
    __shared__ float s_acc[4 * G * HD];
    const int r = blockIdx.x, kh = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int Hq = Hkv * G;
    const int ctx = row_pos[r] + 1;
    const size_t start = row_start[r];
    constexpr int CPT = HD / 8;
    const int dc = lane % CPT;
    const float scale = rsqrtf((float)HD);
    float qf[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        load8<T>(q + ((size_t)r * Hq + kh * G + g) * HD + dc * 8, qf[g]);
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[g][e] *= scale;
    }
    HeadState st[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        st[g].m = -INFINITY; st[g].l = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) st[g].acc[e] = 0.f;
    }
    const size_t tstride = (size_t)Hkv * HD;
    const int n_tiles = (ctx + kPT - 1) / kPT;
    for (int ti = wave; ti < n_tiles; ti += 4) {
        const size_t base = (start + (size_t)ti * kPT) * tstride + (size_t)kh * HD;
        attend_tile<T, HD, G>(k + base, v + base, tstride, min(kPT, ctx - ti * kPT), qf, st, lane);
    }
    block_merge<HD, G>(st, lane, wave, s_m, s_l, s_acc);
    for (int i = threadIdx.x; i < G * HD; i += 256) {
        const int g = i / HD, e = i - g * HD;
        float mt = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) mt = fmaxf(mt, s_m[w * G + g]);
        float lt = 0.f, at = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float f = __expf(s_m[w * G + g] - mt);
            lt += s_l[w * G + g] * f;
            at += s_acc[(w * G + g) * HD + e] * f;
        }
        out[((size_t)r * Hq + kh * G + g) * HD + e] = from_f32<TO>(at / lt);
    }
}

hipError_t launch_prefill_attn(hipStream_t st, int odt, const float* q, const float* k,
                               const float* v, const int* row_start, const int* row_pos, void* out,
                               int rows, const Dims& dm) {
    if (rows <= 0) return hipSuccess;
    const int G = dm.n_q_heads / dm.n_kv_heads, hd = dm.head_dim;
    dim3 grid(rows, dm.n_kv_heads);
#define RLHF_PRE(TT, HD_, G_)                                                                      \
    do {                                                                                           \
        k_prefill_attn<TT, HD_, G_><<<grid, 256, 0, st>>>(q, k, v, row_start, row_pos, (TT*)out,   \
                                                          dm.n_kv_heads);                          \
        return hipGetLastError();                                                                  \
    } while (0)
    if (odt == kF32) {
        if (hd == 128 && G == 1) RLHF_PRE(float, 128, 1);
        if (hd == 64 && G == 1) RLHF_PRE(float, 64, 1);
    }
#undef RLHF_PRE
    return hipErrorInvalidValue;
}

// ------------------------------------------------------ prefill / scoring, half precision
// Packed varlen causal attention on the matrix units (bf16 models).  q, k, v, out are IEEE half
// [T, heads*HD].  A workgroup owns one tile of 128 consecutive queries of one sequence and one
// query head; each of its four waves owns 32 queries.  Keys are walked in tiles of 64: the K
// tile sits in LDS row-major (16-byte chunks XOR-swizzled), the V tile transposed ([d][key]) so
// that the second product can read runs of keys.  Per key tile and wave:
//   S^T[key][q] = K Q^T     (v_mfma_f32_16x16x32_f16, K rows as the A operand)
//   online softmax along keys: a lane holds 16 keys of one query, lane groups are merged by
//   two xor-shuffles; the running sum stays per lane until the end
//   O^T[d][q] += V^T P^T    (P re-used from the lane's own registers as the B operand)
// Masking covers causality and the sequence end; rows past the sequence end are not stored.
constexpr int kFaBM = 128, kFaBN = 64, kFaVStride = kFaBN + 8;

template <int HD>
__global__ __launch_bounds__(256, 2) void k_flash_attn(const f16_t* __restrict__ q,
                                                    const f16_t* __restrict__ k,
                                                    const f16_t* __restrict__ v,
                                                    const int* __restrict__ tile_start,
                                                    const int* __restrict__ tile_q0,
                                                    const int* __restrict__ tile_len,
                                                    f16_t* __restrict__ out, int Hq, int Hkv,
                                                    int T_total) {
    constexpr int KS = HD / 32;        // MFMA steps along d for Q K^T
    constexpr int DF = HD / 16;        // 16-wide d fragments of the output
    constexpr int CH = HD / 8;         // 16-byte chunks per K/V row
    constexpr int LD_IT = kFaBN * CH / 256;
    __shared__ __attribute__((aligned(16))) f16_t sK[kFaBN * HD];
    __shared__ __attribute__((aligned(16))) f16_t sVt[HD * kFaVStride];

    const int tile = blockIdx.x, h = blockIdx.y;
    const int kh = h / (Hq / Hkv);
    const int s0 = tile_start[tile], q0 = tile_q0[tile], L = tile_len[tile];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int fr = lane & 15, g = lane >> 4;
    const size_t qstride = (size_t)Hq * HD, kstride = (size_t)Hkv * HD;
    const float sl2e = rsqrtf((float)HD) * 1.44269504088896f;     // log2(e) / sqrt(HD)

    // Q fragments (B operand): query fr of each 16-row fragment, 8 dims at (s*32 + g*8)
    f16x8_t qf[2][KS];
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const int row = min(q0 + wave * 32 + m * 16 + fr, L - 1);
        const f16_t* src = q + (size_t)(s0 + row) * qstride + (size_t)h * HD + g * 8;
#pragma unroll
        for (int s = 0; s < KS; ++s) qf[m][s] = *reinterpret_cast<const f16x8_t*>(src + s * 32);
    }
    f32x4_t oacc[DF][2];
#pragma unroll
    for (int d = 0; d < DF; ++d)
#pragma unroll
        for (int m = 0; m < 2; ++m) oacc[d][m] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    float m_run[2] = {-1e30f, -1e30f}, l_run[2] = {0.f, 0.f};

    const int q_last = min(q0 + kFaBM, L) - 1;
    const int n_kt = q_last / kFaBN + 1;

    // K: a thread takes 16-byte chunks of consecutive rows' pieces (coalesced), stored row-major.
    // V: a thread takes the same chunk of two neighbouring keys, so that the transposed store
    // writes whole 32-bit words [d][key pair]; the 32 pairs of a half wave land in 32 different
    // banks and the other half wave (next chunk: 8 d rows = 288 words further) in the other 32.
    static_assert(LD_IT % 2 == 0 && kFaVStride % 2 == 0, "V is stored in key pairs");
    static_assert(LD_IT == 2 || LD_IT == 4, "64 keys x 64 or 128 dims over 256 threads");
    uint4 rk0, rk1, rk2 = make_uint4(0, 0, 0, 0), rk3 = rk2, rva0, rvb0, rva1 = rk2, rvb1 = rk2;
    auto k_src = [&](int kt, int i) {
        const int idx = t + i * 256;
        const size_t grow = (size_t)min(s0 + kt * kFaBN + idx / CH, T_total - 1);
        return reinterpret_cast<const uint4*>(k + grow * kstride + (size_t)kh * HD + (idx % CH) * 8);
    };
    auto v_src = [&](int kt, int i, int u) {
        const int item = t + i * 256;
        const size_t grow = (size_t)min(s0 + kt * kFaBN + 2 * (item & 31) + u, T_total - 1);
        return reinterpret_cast<const uint4*>(v + grow * kstride + (size_t)kh * HD + (item >> 5) * 8);
    };
    auto k_dst = [&](int i) {
        const int idx = t + i * 256;
        const int row = idx / CH, c = idx % CH;
        const int pc = (CH == 16) ? (c ^ (row & 15)) : (c ^ ((row >> 1) & 7));
        return reinterpret_cast<uint4*>(&sK[row * HD + pc * 8]);
    };
    auto v_store = [&](int i, const uint4& va, const uint4& vb) {
        uint32_t* sVt32 = reinterpret_cast<uint32_t*>(sVt);
        const int item = t + i * 256;
        const int pr = item & 31, c = item >> 5;
        uint32_t* d0 = sVt32 + (c * 8) * (kFaVStride / 2) + pr;
        d0[0 * (kFaVStride / 2)] = (va.x & 0xFFFFu) | (vb.x << 16);
        d0[1 * (kFaVStride / 2)] = (va.x >> 16) | (vb.x & 0xFFFF0000u);
        d0[2 * (kFaVStride / 2)] = (va.y & 0xFFFFu) | (vb.y << 16);
        d0[3 * (kFaVStride / 2)] = (va.y >> 16) | (vb.y & 0xFFFF0000u);
        d0[4 * (kFaVStride / 2)] = (va.z & 0xFFFFu) | (vb.z << 16);
        d0[5 * (kFaVStride / 2)] = (va.z >> 16) | (vb.z & 0xFFFF0000u);
        d0[6 * (kFaVStride / 2)] = (va.w & 0xFFFFu) | (vb.w << 16);
        d0[7 * (kFaVStride / 2)] = (va.w >> 16) | (vb.w & 0xFFFF0000u);
    };
#define RLHF_FA_GLOAD(kt_)                                                       \
    do {                                                                         \
        rk0 = *k_src(kt_, 0); rk1 = *k_src(kt_, 1);                              \
        if (LD_IT == 4) { rk2 = *k_src(kt_, 2); rk3 = *k_src(kt_, 3); }          \
        rva0 = *v_src(kt_, 0, 0); rvb0 = *v_src(kt_, 0, 1);                      \
        if (LD_IT == 4) { rva1 = *v_src(kt_, 1, 0); rvb1 = *v_src(kt_, 1, 1); }  \
    } while (0)
#define RLHF_FA_SSTORE()                                                         \
    do {                                                                         \
        *k_dst(0) = rk0; *k_dst(1) = rk1;                                        \
        if (LD_IT == 4) { *k_dst(2) = rk2; *k_dst(3) = rk3; }                    \
        v_store(0, rva0, rvb0);                                                  \
        if (LD_IT == 4) v_store(1, rva1, rvb1);                                  \
    } while (0)

    RLHF_FA_GLOAD(0);
    for (int kt = 0; kt < n_kt; ++kt) {
        __syncthreads();                       // the previous tile has been consumed
        RLHF_FA_SSTORE();
        __syncthreads();
        if (kt + 1 < n_kt) RLHF_FA_GLOAD(kt + 1);

        // ---- S^T = K Q^T
        f32x4_t sacc[4][2];
#pragma unroll
        for (int f = 0; f < 4; ++f)
#pragma unroll
            for (int m = 0; m < 2; ++m) sacc[f][m] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s) {
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                const int row = f * 16 + fr, c = s * 4 + g;
                const int pc = (CH == 16) ? (c ^ (row & 15)) : (c ^ ((row >> 1) & 7));
                const f16x8_t kf = *reinterpret_cast<const f16x8_t*>(&sK[row * HD + pc * 8]);
#pragma unroll
                for (int m = 0; m < 2; ++m)
                    sacc[f][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf, qf[m][s], sacc[f][m], 0, 0, 0);
            }
        }
        // ---- mask, online softmax (per query = per lane column).  Running maxima are kept on the
        // raw scores; 1/sqrt(HD) and log2(e) are folded into one multiply-add in front of exp2.
        // Only tiles that reach past this wave's first query need the causal mask (a valid query
        // never sees keys past the end of its sequence: key <= query < L).
        const bool diag = kt * kFaBN + kFaBN - 1 > q0 + wave * 32;
        f16x8_t pb[2][2];
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const int qrow = q0 + wave * 32 + m * 16 + fr;
            if (diag) {
#pragma unroll
                for (int f = 0; f < 4; ++f)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (kt * kFaBN + f * 16 + g * 4 + r > qrow) sacc[f][m][r] = -INFINITY;
            }
            float mx = fmaxf(fmaxf(sacc[0][m][0], sacc[0][m][1]), fmaxf(sacc[0][m][2], sacc[0][m][3]));
#pragma unroll
            for (int f = 1; f < 4; ++f)
                mx = fmaxf(mx, fmaxf(fmaxf(sacc[f][m][0], sacc[f][m][1]), fmaxf(sacc[f][m][2], sacc[f][m][3])));
            mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
            mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
            const float m_new = fmaxf(m_run[m], mx);
            const float alpha = __builtin_amdgcn_exp2f((m_run[m] - m_new) * sl2e);
            m_run[m] = m_new;
            const float mc = m_new * sl2e;
            float ls = 0.f;
#pragma unroll
            for (int f = 0; f < 4; ++f)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(sacc[f][m][r], sl2e, -mc));
                    ls += p;
                    pb[m][f >> 1][(f & 1) * 4 + r] = (f16_t)p;
                }
            l_run[m] = l_run[m] * alpha + ls;
#pragma unroll
            for (int d = 0; d < DF; ++d) oacc[d][m] *= alpha;
        }
        // ---- O^T += V^T P^T
#pragma unroll
        for (int d = 0; d < DF; ++d) {
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const f16_t* vr = &sVt[(d * 16 + fr) * kFaVStride + s2 * 32 + g * 4];
                const uint2 lo = *reinterpret_cast<const uint2*>(vr);
                const uint2 hi = *reinterpret_cast<const uint2*>(vr + 16);
                const uint4 packed = make_uint4(lo.x, lo.y, hi.x, hi.y);
                const f16x8_t vf = *reinterpret_cast<const f16x8_t*>(&packed);
#pragma unroll
                for (int m = 0; m < 2; ++m)
                    oacc[d][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vf, pb[m][s2], oacc[d][m], 0, 0, 0);
            }
        }
    }
    // ---- normalise and store: a lane holds d = 16*df + 4g + r of query fr
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        float l = l_run[m];
        l += __shfl_xor(l, 16, kWave);
        l += __shfl_xor(l, 32, kWave);
        const int qrow = q0 + wave * 32 + m * 16 + fr;
        if (qrow >= L) continue;
        const float inv = 1.f / l;
        f16_t* dst = out + (size_t)(s0 + qrow) * qstride + (size_t)h * HD + g * 4;
#pragma unroll
        for (int d = 0; d < DF; ++d) {
            typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
            f16x4_t o;
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = (f16_t)(oacc[d][m][r] * inv);
            *reinterpret_cast<f16x4_t*>(dst + d * 16) = o;
        }
    }
}

#undef RLHF_FA_GLOAD
#undef RLHF_FA_SSTORE

hipError_t launch_flash_attn(hipStream_t st, const void* q, const void* k, const void* v,
                             const int* tile_start, const int* tile_q0, const int* tile_len, void* out,
                             int n_tiles, int T_total, const Dims& dm) {
    if (n_tiles <= 0) return hipSuccess;
    dim3 grid(n_tiles, dm.n_q_heads);
    if (dm.head_dim == 128)
        k_flash_attn<128><<<grid, 256, 0, st>>>((const f16_t*)q, (const f16_t*)k, (const f16_t*)v, tile_start,
                                                tile_q0, tile_len, (f16_t*)out, dm.n_q_heads, dm.n_kv_heads,
                                                T_total);
    else if (dm.head_dim == 64)
        k_flash_attn<64><<<grid, 256, 0, st>>>((const f16_t*)q, (const f16_t*)k, (const f16_t*)v, tile_start,
                                               tile_q0, tile_len, (f16_t*)out, dm.n_q_heads, dm.n_kv_heads,
                                               T_total);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace rlhf
