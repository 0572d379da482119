// C[m][n] = sum_k A[m][k] * W[n][k]   (activations times a row-major weight matrix, y = W x)
//
// bf16 weights: LDS-tiled MFMA kernel (v_mfma_f32_16x16x32_{bf16,f16}, float accumulate).
// Activations are half (what the stage uses for bf16 models) or bf16; for half the bf16 weight
// chunks are converted to half, exactly, between the global load and the LDS store.  One
// template serves the decode regime (few rows: the weight matrix streams from HBM once, split
// along K so that enough workgroups are in flight to saturate bandwidth) and the prefill /
// scoring regime (thousands of rows: compute-bound 256x256 tiles).  Global loads are 16 bytes per lane,
// consecutive lanes along K; tiles sit in LDS with an XOR swizzle of the 16-byte chunk index
// so that the MFMA-fragment reads (16 rows x one chunk per quarter wave) spread over the banks.
// Split-K partials are written to separate buffers and summed by the consumer kernel, which
// keeps the result deterministic (no float atomics).
//
// fp32: a plain LDS-tiled kernel for the float configuration (small model; not tuned).
#include "common.h"
#include "kernels.h"
#include <type_traits>

namespace rlhf {

// 16-byte chunk swizzle inside an LDS tile row: the fragment read of a quarter wave takes one
// chunk column of 16 consecutive rows; XOR-ing the chunk index with row bits spreads those 16
// reads over all banks (rows of 128 bytes: two rows per 256-byte bank sweep; rows of 64 bytes:
// four).
template <int TK> __device__ __forceinline__ int swz(int row, int chunk) {
    return TK == 64 ? (chunk ^ ((row >> 1) & 7)) : (chunk ^ ((row >> 2) & 3));
}

template <bool AF16> struct Mfma;
template <> struct Mfma<false> {
    typedef bf16x8_t frag;
    static __device__ __forceinline__ f32x4_t run(frag a, frag b, f32x4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};
template <> struct Mfma<true> {
    typedef f16x8_t frag;
    static __device__ __forceinline__ f32x4_t run(frag a, frag b, f32x4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
};

// Tile index of a workgroup.  Few-row launches (XCD == false) walk the N tiles in order, the
// row tiles of a column tile next to each other so that its weights are fetched once.
// Compute-bound launches (XCD == true): the tile grid is cut into panels of kGroupM tile rows.
// Inside a panel the tile columns are dealt to the 8 XCDs (workgroup id modulo 8, the order in
// which the dispatcher deals workgroups to XCDs) in contiguous groups, and an XCD walks its
// group column by column.  Two things follow.  The workgroups resident on one XCD at a time
// cover a compact block of kGroupM x 4 tiles, so its L2 re-serves the A rows and W rows they
// share.  And all XCDs work on the SAME panel of A rows at the same time, each on W columns of
// its own: an A panel is requested by the eight L2s within a short time of each other (one
// fetch from HBM, the others from the memory-side cache even while a decode stream sweeps its
// weights through that cache) and every W column is fetched by one XCD only, once per panel.
// (Before, each XCD walked its own contiguous eighth of the panel-ordered tile list; the
// eight of them then sat on up to four different A panels and up to eight W ranges, and with the
// memory-side cache swept by the decode stream the scoring GEMMs pulled several times their
// operands from HBM.)
constexpr int kGroupM = 8;
__host__ __device__ inline int xcd_cols(int tiles_n) { return (tiles_n + 7) >> 3; }   // tile columns per XCD
inline int xcd_grid(int tiles_m, int tiles_n) { return 8 * tiles_m * xcd_cols(tiles_n); }
template <bool XCD>
__host__ __device__ __forceinline__ bool tile_of(int bid, int tiles_m, int tiles_n, int& tm, int& tn) {
    if (!XCD) {           // the (at most two) row tiles of one column tile run side by side
        tn = bid / tiles_m;
        tm = bid - tn * tiles_m;
        return true;
    }
    const int xcd = bid & 7, slot = bid >> 3;
    const int cx = xcd_cols(tiles_n);
    const int c_lo = xcd * cx;
    const int c_n = min(tiles_n, c_lo + cx) - c_lo;          // this XCD's columns (may be <= 0 at the end)
    if (c_n <= 0) return false;
    const int per_panel = kGroupM * c_n;
    const int full = tiles_m / kGroupM;
    int panel = slot / per_panel, r = slot - panel * per_panel, rows = kGroupM;
    if (panel >= full) {                                     // the last, shorter panel
        panel = full;
        r = slot - full * per_panel;
        rows = tiles_m - full * kGroupM;
        if (rows <= 0 || r >= rows * c_n) return false;
    }
    tm = panel * kGroupM + r % rows;
    tn = c_lo + r / rows;
    return true;
}

// A: 16-bit activations (bf16 if !AF16, half if AF16); W: bf16.
// TM x TN output tile per workgroup of WM x WN waves; each wave owns (TM/WM) x (TN/WN), built
// from 16x16 MFMA fragments; K advances in LDS tiles of TK (32 or 64) elements, double-buffered.
//
// SWIGLU: W is a gate||up matrix [2f, K] (gate rows, then up rows) and N = 2f.  The tile's
// columns alternate, in blocks of 16, between gate rows and the matching up rows, so that a
// lane ends up with gate and up of the same output column in neighbouring fragments; the
// epilogue writes act = silu(gate) * up as 16-bit [M, f] (of the activation type) to C and the
// float [M, 2f] intermediate never exists.
//
// ADMA: the activation tile, which never needs converting, goes from global memory straight
// into LDS (global_load_lds, 16 bytes per lane, 1 KB per wave and instruction: the lane picks
// the global chunk whose swizzled place it fills).  That frees its staging registers, which
// is what lets a decode workgroup sit beside one of these on a compute unit.  Needs whole K
// tiles (K a multiple of TK, no split); rows past M are clamped (computed, never stored).
//
// ROPE (= head_dim, 64 or 128; 0 = off): W is a layer's QKV matrix and the epilogue finishes the
// projection: query and key heads are rotated (pair (k, k + head_dim/2); a wave tile of 128
// columns holds whole heads, so both halves of a pair sit in one lane, in fragments head_dim/32
// apart), everything is rounded to the activation type and written where attention reads it:
// q, k, v row-major, and k, v also into the paged pool when the pass fills the cache.  The
// float [M, (Hq + 2 Hkv) head_dim] intermediate and the separate rotary kernel disappear.
//
// LSE: W is an LM head [vocab, K] and the logits never leave the registers: the epilogue reduces
// each wave's 128 columns of a row to (max, sum of exp(z - max)), writes that pair as one of the
// row's 2 * tiles_n partials, and the lane that holds the row's target column stores that logit.
// A small merge kernel turns the partials into log_softmax(z)[target] (k_lse_merge).
//
// BDMA: W is IEEE half in memory (a copy of the bf16 matrix made when the weights were bound) and
// goes global -> LDS directly like the activations: no staging registers, no conversion, no LDS
// stores in the loop.  Both operands then come in as buffer loads (buffer_load_dwordx4 ... lds):
// a lane's 32-bit byte offset is fixed for the whole K walk, which is the instruction's scalar
// offset, so issuing a load costs one scalar add for M0 and no vector work (operands < 4 GiB).
// Needs ADMA's conditions and half activations.
//
// RING (> 1, register-staged tiles only): that many K tiles are kept in flight in registers, so that a
// workgroup which streams its weights over the whole K range (no split) still has enough bytes on
// their way to keep HBM busy.
template <int TM, int TN, int TK, int WM, int WN, bool AF16, bool XCD, bool SWIGLU, bool ADMA = false, int ROPE = 0,
          bool LSE = false, bool BDMA = false, int RING = 1>
__global__ __launch_bounds__(WM * WN * 64) void k_gemm_bf16(const bf16_t* __restrict__ A,
                                                           const bf16_t* __restrict__ W,
                                                           float* __restrict__ C, int M, int N, int K,
                                                           int kchunk, int tiles_m, int tiles_n,
                                                           const RopeOut ro = RopeOut{},
                                                           const LseOut lo = LseOut{}) {
    constexpr int NT = WM * WN * 64;
    constexpr int FM = TM / WM / 16, FN = TN / WN / 16;
    constexpr int CH = TK / 8;                            // 16-byte chunks per tile row
    constexpr int A_CH = TM * CH, B_CH = TN * CH;
    constexpr int A_IT = (A_CH + NT - 1) / NT, B_IT = (B_CH + NT - 1) / NT;
    __shared__ __attribute__((aligned(16))) bf16_t sA[2][TM * TK];
    __shared__ __attribute__((aligned(16))) bf16_t sB[2][TN * TK];

    int tm, tn;
    if (!tile_of<XCD>(blockIdx.x, tiles_m, tiles_n, tm, tn)) return;
    const int m0 = tm * TM, n0 = tn * TN;
    const int split = blockIdx.y;
    const int kbeg = split * kchunk;
    const int kend = min(K, kbeg + kchunk);
    const int nk = (kend - kbeg + TK - 1) / TK;

    // the wave index as a scalar: the wave's tile origin and the LDS destinations of its direct loads
    // then live in scalar registers
    const int t = threadIdx.x, lane = t & 63, w = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = w / WN, wn = w - wm * WN;

    // direct path: wave w fills the 1 KB blocks w * D_IT .. of the A tile (1024 / (2 TK) rows each)
    constexpr int D_RPB = 512 / TK, D_IT = ADMA ? TM / D_RPB / (NT / 64) : 1;
    static_assert(!ADMA || (TM / D_RPB) % (NT / 64) == 0, "A tile blocks must divide among the waves");
    size_t da[D_IT];
    if (ADMA) {
#pragma unroll
        for (int i = 0; i < D_IT; ++i) {
            const int row = (w * D_IT + i) * D_RPB + lane / CH, p = lane % CH;
            // LDS chunk p of this row holds global chunk c with swz(row, c) == p; the swizzle is an XOR
            const int c = swz<TK>(row, p);
            da[i] = (size_t)min(m0 + row, M - 1) * K + c * 8;
        }
    }
    static_assert(!BDMA || (ADMA && AF16), "half weights go with half activations on the direct path");
    constexpr int DB_IT = BDMA ? TN / D_RPB / (NT / 64) : 1;
    static_assert(!BDMA || (TN / D_RPB) % (NT / 64) == 0, "W tile blocks must divide among the waves");
    size_t db[DB_IT];
    if (BDMA) {
#pragma unroll
        for (int i = 0; i < DB_IT; ++i) {
            const int row = (w * DB_IT + i) * D_RPB + lane / CH, p = lane % CH;
            const int c = swz<TK>(row, p);
            int gn = min(n0 + row, N - 1);        // rows past N are clamped (computed, never stored)
            if (SWIGLU) {
                const int oc = min((n0 >> 1) + (row >> 5) * 16 + (row & 15), (N >> 1) - 1);
                gn = ((row >> 4) & 1) * (N >> 1) + oc;
            }
            db[i] = (size_t)gn * K + c * 8;
        }
    }
    typedef __attribute__((address_space(3))) void* lds_ptr_t;
    typedef const __attribute__((address_space(1))) void* glb_ptr_t;
    // BDMA: both operands come in through buffer loads (buffer_load_dwordx4 ... lds): the lane's 32-bit byte
    // offset never changes, the walk along K is a scalar offset, so a direct load costs no vector ALU work
    // and half the address traffic of a 64-bit global load.
    uint32_t oa[D_IT], ob[DB_IT];
#if defined(__HIP_DEVICE_COMPILE__)          // the buffer resource type exists in the device pass only
    __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc((void*)A, 0, BDMA ? -1 : 0, 0x00020000);
    __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void*)W, 0, BDMA ? -1 : 0, 0x00020000);
#endif
    if (BDMA) {
#pragma unroll
        for (int i = 0; i < D_IT; ++i) oa[i] = (uint32_t)(da[i] * 2);
#pragma unroll
        for (int i = 0; i < DB_IT; ++i) ob[i] = (uint32_t)(db[i] * 2);
    }

    uint4 ra[ADMA ? 1 : A_IT], rb[BDMA ? 1 : B_IT];
    auto gload = [&](int kt, uint4* ra, uint4* rb) {
        const int k0 = kbeg + kt * TK;
        if (BDMA) {
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
            for (int i = 0; i < D_IT; ++i)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (lds_ptr_t)&sA[kt & 1][(w * D_IT + i) * 512], 16, oa[i],
                                                         k0 * 2, 0, 0);
#pragma unroll
            for (int i = 0; i < DB_IT; ++i)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_w, (lds_ptr_t)&sB[kt & 1][(w * DB_IT + i) * 512], 16, ob[i],
                                                         k0 * 2, 0, 0);
#endif
        } else if (ADMA) {
            // issued first: the wait the compiler places before the next LDS reads then covers
            // these and leaves the weight loads below in flight
#pragma unroll
            for (int i = 0; i < D_IT; ++i)
                __builtin_amdgcn_global_load_lds((glb_ptr_t)(A + da[i] + k0),
                                                 (lds_ptr_t)&sA[kt & 1][(w * D_IT + i) * 512], 16, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < (ADMA ? 0 : A_IT); ++i) {
            const int idx = t + i * NT;
            const int row = idx / CH, c = idx % CH;
            const int gm = m0 + row, gk = k0 + c * 8;
            ra[i] = make_uint4(0, 0, 0, 0);
            if (idx < A_CH && gm < M && gk < kend)
                ra[i] = *reinterpret_cast<const uint4*>(A + (size_t)gm * K + gk);
        }
#pragma unroll
        for (int i = 0; i < (BDMA ? 0 : B_IT); ++i) {
            const int idx = t + i * NT;
            const int row = idx / CH, c = idx % CH;
            int gn = n0 + row;
            bool ok = gn < N;
            if (SWIGLU) {      // tile column -> gate row (even 16-blocks) or up row (odd) of out col
                const int oc = (n0 >> 1) + (row >> 5) * 16 + (row & 15);
                ok = oc < (N >> 1);
                gn = ((row >> 4) & 1) * (N >> 1) + oc;
            }
            const int gk = k0 + c * 8;
            rb[i] = make_uint4(0, 0, 0, 0);
            if (idx < B_CH && ok && gk < kend) {
                if (XCD) {
                    rb[i] = *reinterpret_cast<const uint4*>(W + (size_t)gn * K + gk);
                } else {
                    // few-row launches read every weight once: stream them past the caches (evict first), so
                    // that a tall GEMM on the other stream keeps its tiles in the L2 they share
                    typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
                    const u32x4v v = __builtin_nontemporal_load(reinterpret_cast<const u32x4v*>(W + (size_t)gn * K + gk));
                    rb[i] = make_uint4(v[0], v[1], v[2], v[3]);
                }
            }
        }
    };
    auto sstore = [&](int buf, uint4* ra, uint4* rb) {
#pragma unroll
        for (int i = 0; i < (ADMA ? 0 : A_IT); ++i) {
            const int idx = t + i * NT;
            const int row = idx / CH, c = idx % CH;
            if (idx < A_CH)
                *reinterpret_cast<uint4*>(&sA[buf][row * TK + swz<TK>(row, c) * 8]) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < (BDMA ? 0 : B_IT); ++i) {
            const int idx = t + i * NT;
            const int row = idx / CH, c = idx % CH;
            if (AF16) {   // bf16 -> half once per element per workgroup (exact in half's normal range)
                rb[i].x = bf16x2_to_f16x2(rb[i].x); rb[i].y = bf16x2_to_f16x2(rb[i].y);
                rb[i].z = bf16x2_to_f16x2(rb[i].z); rb[i].w = bf16x2_to_f16x2(rb[i].w);
            }
            if (idx < B_CH)
                *reinterpret_cast<uint4*>(&sB[buf][row * TK + swz<TK>(row, c) * 8]) = rb[i];
        }
    };

    f32x4_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    const int fr = lane & 15, fq = lane >> 4;
    auto compute = [&](int buf) {
        if constexpr (ADMA) {
            // The fragment reads and their waits are written out by hand.  If the compiler saw LDS
            // reads here it would first wait for the global -> LDS loads of the NEXT tile issued just
            // above (it cannot tell the two buffers apart), and the prefetch would overlap nothing.
            // As it is, those loads are waited for where the loop needs them: by the weight tile's
            // LDS stores and by the fence of the barrier at the end of the step.
            static_assert(!ADMA || (FM == 4 && FN == 8 && TK == 64), "hand-placed reads are for the 64 x 128 wave tile");
            typedef typename Mfma<AF16>::frag frag;
            const uint32_t xr = (fr >> 1) & 7;       // row part of the swizzle: row bases are multiples of 16
            const uint32_t pa0 = (uint32_t)(size_t)(lds_ptr_t)&sA[buf][0] + (wm * (TM / WM) + fr) * (TK * 2);
            const uint32_t pb0 = (uint32_t)(size_t)(lds_ptr_t)&sB[buf][0] + (wn * (TN / WN) + fr) * (TK * 2);
#define RLHF_DS_READ(dst, addr, off) asm volatile("ds_read_b128 %0, %1 offset:" #off : "=v"(dst) : "v"(addr) : "memory")
#define RLHF_LGKM0(...) asm volatile("s_waitcnt lgkmcnt(0)" : __VA_ARGS__ : : "memory")
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                frag fa[4], fb[8];
                const uint32_t co = ((uint32_t)(s * 4 + fq) ^ xr) * 16;
                const uint32_t pa = pa0 + co, pb = pb0 + co;
                RLHF_DS_READ(fa[0], pa, 0); RLHF_DS_READ(fa[1], pa, 2048);
                RLHF_DS_READ(fa[2], pa, 4096); RLHF_DS_READ(fa[3], pa, 6144);
                RLHF_DS_READ(fb[0], pb, 0); RLHF_DS_READ(fb[1], pb, 2048);
                RLHF_DS_READ(fb[2], pb, 4096); RLHF_DS_READ(fb[3], pb, 6144);
                RLHF_LGKM0("+v"(fa[0]), "+v"(fa[1]), "+v"(fa[2]), "+v"(fa[3]), "+v"(fb[0]), "+v"(fb[1]), "+v"(fb[2]),
                           "+v"(fb[3]));
                RLHF_DS_READ(fb[4], pb, 8192); RLHF_DS_READ(fb[5], pb, 10240);
                RLHF_DS_READ(fb[6], pb, 12288); RLHF_DS_READ(fb[7], pb, 14336);
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = Mfma<AF16>::run(fb[j], fa[i], acc[i][j]);
                __builtin_amdgcn_sched_barrier(0);
                RLHF_LGKM0("+v"(fb[4]), "+v"(fb[5]), "+v"(fb[6]), "+v"(fb[7]));
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 4; j < 8; ++j) acc[i][j] = Mfma<AF16>::run(fb[j], fa[i], acc[i][j]);
                __builtin_amdgcn_sched_barrier(0);
            }
#undef RLHF_DS_READ
#undef RLHF_LGKM0
            return;
        }
#pragma unroll
        for (int s = 0; s < TK / 32; ++s) {
            typename Mfma<AF16>::frag fa[FM], fb[FN];
            const int c = s * 4 + fq;
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                const int row = wm * (TM / WM) + i * 16 + fr;
                fa[i] = *reinterpret_cast<const typename Mfma<AF16>::frag*>(&sA[buf][row * TK + swz<TK>(row, c) * 8]);
            }
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int row = wn * (TN / WN) + j * 16 + fr;
                fb[j] = *reinterpret_cast<const typename Mfma<AF16>::frag*>(&sB[buf][row * TK + swz<TK>(row, c) * 8]);
            }
            // weights are the MFMA "A" operand: D[i = n][j = m], so a lane ends up holding four
            // consecutive n of one row m and stores them as one float4.
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = Mfma<AF16>::run(fb[j], fa[i], acc[i][j]);
        }
    };
    if constexpr (RING > 1) {
        static_assert(RING == 1 || (!ADMA && !BDMA && RING % 2 == 0), "the register ring holds register-staged tiles");
        // ring slot j holds tile kt with kt % RING == j; the slot of the tile that has just gone to LDS
        // is refilled with the tile RING steps ahead (the waits for a slot's loads follow from its use)
        uint4 qa[RING][A_IT], qb[RING][B_IT];
#pragma unroll
        for (int j = 0; j < RING; ++j)
            if (j < nk) gload(j, qa[j], qb[j]);
        if (nk > 0) sstore(0, qa[0], qb[0]);
        __syncthreads();
        for (int kt0 = 0; kt0 < nk; kt0 += RING) {
#pragma unroll
            for (int j = 0; j < RING; ++j) {
                const int kt = kt0 + j;
                if (kt < nk) {
                    gload(kt + RING, qa[j], qb[j]);      // past the range every lane's guard is off: nothing is loaded
                    compute(j & 1);
                    if (kt + 1 < nk) sstore((j + 1) & 1, qa[(j + 1) % RING], qb[(j + 1) % RING]);
                    __syncthreads();
                }
            }
        }
    } else {
        if (nk > 0) {
            gload(0, ra, rb);
            sstore(0, ra, rb);
        }
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            const int buf = kt & 1;
            if (kt + 1 < nk) gload(kt + 1, ra, rb);
            compute(buf);
            if (kt + 1 < nk) sstore(buf ^ 1, ra, rb);
            __syncthreads();
        }
    }

    if (SWIGLU) {
        static_assert(!SWIGLU || (FN % 4 == 0), "gate and up fragments come in pairs, pairs are stored two at a time");
        const int f = N >> 1;
        uint16_t* act = reinterpret_cast<uint16_t*>(C);
        const bool odd = fq & 1;
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const int m = m0 + wm * (TM / WM) + i * 16 + fr;
            // silu(gate) * up of fragment pair (j, j + 1): four consecutive output columns in 8 bytes
            auto packed = [&](int j) {
                float o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float g = acc[i][j][e];
                    o[e] = g / (1.f + __expf(-g)) * acc[i][j + 1][e];
                }
                uint2 pk;
                if (AF16) {
                    fp16x2_t a = {(__fp16)o[0], (__fp16)o[1]}, b = {(__fp16)o[2], (__fp16)o[3]};
                    pk.x = *reinterpret_cast<uint32_t*>(&a);
                    pk.y = *reinterpret_cast<uint32_t*>(&b);
                } else {
                    pk.x = (uint32_t)f32_to_bf16(o[0]) | ((uint32_t)f32_to_bf16(o[1]) << 16);
                    pk.y = (uint32_t)f32_to_bf16(o[2]) | ((uint32_t)f32_to_bf16(o[3]) << 16);
                }
                return pk;
            };
            // Two fragment pairs cover 32 consecutive output columns; neighbouring quarter waves swap
            // one of them each, so that a lane stores eight consecutive columns (16 bytes).
#pragma unroll
            for (int j = 0; j < FN; j += 4) {
                const uint2 p0 = packed(j), p1 = packed(j + 2);
                const uint2 give = odd ? p0 : p1;
                uint2 got;
                got.x = (uint32_t)__shfl_xor((int)give.x, 16, kWave);
                got.y = (uint32_t)__shfl_xor((int)give.y, 16, kWave);
                const uint4 pk = odd ? make_uint4(got.x, got.y, p1.x, p1.y) : make_uint4(p0.x, p0.y, got.x, got.y);
                const int oc = (n0 >> 1) + ((wn * (TN / WN) + (odd ? j + 2 : j) * 16) >> 1) + (fq & 2) * 4;
                if (m >= M || oc >= f) continue;       // f is a multiple of 8: a group of 8 is in or out
                *reinterpret_cast<uint4*>(act + (size_t)m * f + oc) = pk;
            }
        }
        return;
    }
    if constexpr (ROPE > 0) {
        static_assert(ROPE == 0 || ((TN / WN) % ROPE == 0 && TN % ROPE == 0), "a wave tile holds whole heads");
        constexpr int HD = ROPE > 0 ? ROPE : 64, HALF = HD / 2, PF = HD / 32;   // PF: fragments between pair halves
        typedef typename std::conditional<AF16, f16_t, bf16_t>::type TO;
        TO* q_out = reinterpret_cast<TO*>(ro.q);
        TO* k_out = reinterpret_cast<TO*>(ro.k);
        TO* v_out = reinterpret_cast<TO*>(ro.v);
        TO* pool = reinterpret_cast<TO*>(ro.pool);
        const int Hq = ro.n_q_heads, Hkv = ro.n_kv_heads;
        static_assert(ROPE == 0 || FN % 2 == 0, "fragments are stored in pairs");
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const int m = m0 + wm * (TM / WM) + i * 16 + fr;
            const bool row_ok = m < M;
            const int mc = row_ok ? m : M - 1;
            const float* tab = ro.table + (size_t)ro.pos[mc] * HD;
            TO* prow = nullptr;                 // this token's K row of head 0 in the pool
            if (pool) {
                const int slot = ro.kv_dst[mc];
                prow = pool + ((size_t)(slot / ro.page_tokens) * ro.n_layers + ro.layer) * 2 * (size_t)Hkv * ro.page_tokens * HD +
                       (size_t)(slot % ro.page_tokens) * HD;
            }
            const size_t head_stride = (size_t)ro.page_tokens * HD;
            // rotated, rounded and packed fragment j of this row: four consecutive columns in 8 bytes
            auto packed = [&](int j) {
                const int c = (wn * (TN / WN) + j * 16 + fq * 4) % HD;
                const bool rot = n0 + wn * (TN / WN) + j * 16 < (Hq + Hkv) * HD;
                const bool first = ((j % (2 * PF)) < PF);
                float o[4];
                if (rot) {
                    const int jp = first ? j + PF : j - PF;
                    const int k = first ? c : c - HALF;
                    const float4 t0 = *reinterpret_cast<const float4*>(tab + 2 * k);
                    const float4 t1 = *reinterpret_cast<const float4*>(tab + 2 * k + 4);
                    const float cs[4] = {t0.x, t0.z, t1.x, t1.z}, sn[4] = {t0.y, t0.w, t1.y, t1.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float a = first ? acc[i][j][e] : acc[i][jp][e];
                        const float b = first ? acc[i][jp][e] : acc[i][j][e];
                        o[e] = first ? a * cs[e] - b * sn[e] : a * sn[e] + b * cs[e];
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = acc[i][j][e];
                }
                uint2 pk;
                if (AF16) {
                    fp16x2_t a = {(__fp16)o[0], (__fp16)o[1]}, b = {(__fp16)o[2], (__fp16)o[3]};
                    pk.x = *reinterpret_cast<uint32_t*>(&a);
                    pk.y = *reinterpret_cast<uint32_t*>(&b);
                } else {
                    pk.x = (uint32_t)f32_to_bf16(o[0]) | ((uint32_t)f32_to_bf16(o[1]) << 16);
                    pk.y = (uint32_t)f32_to_bf16(o[2]) | ((uint32_t)f32_to_bf16(o[3]) << 16);
                }
                return pk;
            };
            // Fragments j and j + 1 cover 32 consecutive columns, four at a time per quarter wave.
            // Neighbouring quarter waves swap one fragment each, after which a lane holds eight
            // consecutive columns (16 bytes) and a row's 64 bytes are written by four lanes.
            const bool odd = fq & 1;
#pragma unroll
            for (int j = 0; j < FN; j += 2) {
                const uint2 p0 = packed(j), p1 = packed(j + 1);
                const uint2 give = odd ? p0 : p1;
                uint2 got;
                got.x = (uint32_t)__shfl_xor((int)give.x, 16, kWave);
                got.y = (uint32_t)__shfl_xor((int)give.y, 16, kWave);
                const uint4 pk = odd ? make_uint4(got.x, got.y, p1.x, p1.y) : make_uint4(p0.x, p0.y, got.x, got.y);
                const int n = n0 + wn * (TN / WN) + (odd ? j + 1 : j) * 16 + (fq & 2) * 4;
                if (!row_ok || n >= N) continue;     // N is a multiple of head_dim: a group of 8 is in or out
                const int head = n / HD, c = n - head * HD;
                if (head < Hq) {
                    *reinterpret_cast<uint4*>(q_out + ((size_t)m * Hq + head) * HD + c) = pk;
                } else {
                    const bool is_k = head < Hq + Hkv;
                    const int kh = is_k ? head - Hq : head - Hq - Hkv;
                    TO* dst = is_k ? k_out : v_out;
                    if (dst) *reinterpret_cast<uint4*>(dst + ((size_t)m * Hkv + kh) * HD + c) = pk;
                    if (prow)
                        *reinterpret_cast<uint4*>(prow + (is_k ? 0 : (size_t)Hkv * head_stride) + kh * head_stride + c) = pk;
                }
            }
        }
        return;
    }
    if constexpr (LSE) {
        const int pcol = tn * WN + wn;                       // this wave's partial of the row
        const int ncol0 = n0 + wn * (TN / WN) + fq * 4;
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const int m = m0 + wm * (TM / WM) + i * 16 + fr;
            const bool row_ok = m < M;
            int t = -1;
            if (row_ok) t = min(max(lo.tokens[lo.target_idx[m]], 0), N - 1);
            float mx = -INFINITY;
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int n = ncol0 + j * 16 + e;
                    if (n < N) mx = fmaxf(mx, acc[i][j][e]);
                    if (n == t) lo.tgt[m] = acc[i][j][e];
                }
            mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
            mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
            float se = 0.f;
            if (mx > -INFINITY) {
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (ncol0 + j * 16 + e < N) se += __expf(acc[i][j][e] - mx);
            }
            se += __shfl_xor(se, 16, kWave);
            se += __shfl_xor(se, 32, kWave);
            if (row_ok && fq == 0) {
                lo.part_max[(size_t)m * lo.n_part + pcol] = mx;
                lo.part_sum[(size_t)m * lo.n_part + pcol] = se;
            }
        }
        return;
    }
    float* Cs = C + (size_t)split * M * N;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int m = m0 + wm * (TM / WM) + i * 16 + fr;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int n = n0 + wn * (TN / WN) + j * 16 + fq * 4;
            float* dst = Cs + (size_t)m * N + n;
            if (n + 3 < N && (N & 3) == 0) {
                *reinterpret_cast<float4*>(dst) =
                    make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (n + e < N) dst[e] = acc[i][j][e];
            }
        }
    }
}

// ------------------------------------------------------- few rows, whole K range per workgroup
// Up to 16 activation rows against 64 weight rows per workgroup, the workgroup walking the WHOLE K
// range (no split, so the result is final and an epilogue can finish the layer's next step).  With
// few workgroups per compute unit the bytes in flight have to come from depth instead: a ring of
// RING K tiles per thread in registers.  The loop is free of branches around the loads (rows past
// M or N are clamped and discarded at the store, K is a whole number of tiles), because the
// compiler otherwise waits for ALL outstanding loads at every tile and the ring is worth nothing.
// Tiles pass through LDS as in k_gemm_bf16 (same swizzle, weights converted to half on the way).
//   MODE 0: C[m][n] float, one plane.
//   MODE 1 (SwiGLU): W = gate||up [2f, K]; the workgroup's 64 rows are 32 gate rows and the matching
//           32 up rows; act[m][c] = silu(gate) * up, 16-bit, [M, f].
//   MODE 2 (rotary + KV append): W = QKV; the 64 rows are columns [c, c+32) and [c+half, c+half+32) of
//           one head (half = head_dim / 2), so both members of every rotary pair meet in the workgroup;
//           query heads go to q, key / value heads to the paged pool (and k / v if given).
// (Measured on the 7B shapes at 8 rows: QKV 21.6 us and gate||up 39.6 us with a ring of 8, against
// 20.2 and 34.3 us for the split-K kernel, whose consumers then cost a launch each; a ring of 16
// and two wave groups on alternate tiles were both slower; without the ring, 57 and 60 us.)
template <int RING, int MODE, bool AF16>
__global__ __launch_bounds__(256) void k_gemm_rows16(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W,
                                                     float* __restrict__ C, int M, int N, int K, const RowsEpi ep) {
    constexpr int TM = 16, TN = 64, TK = 64;
    __shared__ __attribute__((aligned(16))) bf16_t sA[2][TM * TK];
    __shared__ __attribute__((aligned(16))) bf16_t sB[2][TN * TK];
    __shared__ float sx[TM][TN + 1];                       // epilogue exchange (MODE 1, 2)
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int fr = lane & 15, fq = lane >> 4;
    const int nk = K / TK / (int)gridDim.y;                // mode 0 may split K over blockIdx.y (float planes)
    const int blk = blockIdx.x;
    A += (size_t)blockIdx.y * nk * TK;
    W += (size_t)blockIdx.y * nk * TK;
    C += (size_t)blockIdx.y * M * N;

    // weight row of tile row r
    auto wrow = [&](int r) -> int {
        if (MODE == 1) {                                   // rows 0..31: gate columns blk*32 + r; 32..63: the up rows
            const int c = min(blk * 32 + (r & 31), ep.ffn - 1);
            return (r >> 5) * ep.ffn + c;
        }
        if (MODE == 2) {
            const int hd = ep.ro.head_dim, half = hd >> 1, per_head = half / 32;
            const int head = blk / per_head, c = (blk - head * per_head) * 32;
            return head * hd + (r >> 5) * half + c + (r & 31);
        }
        return min(blk * TN + r, N - 1);
    };
    // loader: one 16-byte chunk of A for the first 128 threads, two of W for everybody
    const int ar = (t >> 3) & 15, ac = t & 7;              // A: row 0..15 (threads 128.. duplicate 0..127), chunk
    const bf16_t* pa = A + (size_t)min(ar, M - 1) * K + ac * 8;
    const bf16_t* pb[2];
    int br[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        br[i] = (t + i * 256) >> 3;
        pb[i] = W + (size_t)wrow(br[i]) * K + ac * 8;
    }
    const int a_dst = ar * TK + swz<TK>(ar, ac) * 8;
    int b_dst[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) b_dst[i] = br[i] * TK + swz<TK>(br[i], ac) * 8;

    // The ring lives in registers: every index below is a compile-time constant after unrolling
    // (macros, not lambdas taking an index: an array indexed through a lambda parameter is put in
    // scratch memory, whose reloads wait for every outstanding load).  Threads 128..255 carry a
    // duplicate of the activation chunk of thread t - 128 and store it to the same place.
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));   // a vector type, not a struct: stays in registers
    u32x4_t qa[RING], qb0[RING], qb1[RING];
#define RLHF_ROWS_GLOAD(KT, J)                                                            \
    do {                                                                                  \
        qa[J] = *reinterpret_cast<const u32x4_t*>(pa + (size_t)(KT) * TK);                \
        qb0[J] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(pb[0] + (size_t)(KT) * TK)); \
        qb1[J] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(pb[1] + (size_t)(KT) * TK)); \
    } while (0)
#define RLHF_ROWS_CVT(R)                                                                  \
    do {                                                                                  \
        if (AF16) {                                                                       \
            R[0] = bf16x2_to_f16x2(R[0]); R[1] = bf16x2_to_f16x2(R[1]);                   \
            R[2] = bf16x2_to_f16x2(R[2]); R[3] = bf16x2_to_f16x2(R[3]);                   \
        }                                                                                 \
    } while (0)
#define RLHF_ROWS_SSTORE(BUF, J)                                                          \
    do {                                                                                  \
        *reinterpret_cast<u32x4_t*>(&sA[BUF][a_dst]) = qa[J];                             \
        u32x4_t r0_ = qb0[J], r1_ = qb1[J];                                               \
        RLHF_ROWS_CVT(r0_);                                                               \
        RLHF_ROWS_CVT(r1_);                                                               \
        *reinterpret_cast<u32x4_t*>(&sB[BUF][b_dst[0]]) = r0_;                            \
        *reinterpret_cast<u32x4_t*>(&sB[BUF][b_dst[1]]) = r1_;                            \
    } while (0)
    f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const int rb_ = w * 16 + fr;
    const int fa_off0 = fr * TK + swz<TK>(fr, fq) * 8, fa_off1 = fr * TK + swz<TK>(fr, 4 + fq) * 8;
    const int fb_off0 = rb_ * TK + swz<TK>(rb_, fq) * 8, fb_off1 = rb_ * TK + swz<TK>(rb_, 4 + fq) * 8;
    typedef typename Mfma<AF16>::frag frag_t;
#define RLHF_ROWS_COMPUTE(BUF)                                                            \
    do {                                                                                  \
        const frag_t fa0_ = *reinterpret_cast<const frag_t*>(&sA[BUF][fa_off0]);          \
        const frag_t fb0_ = *reinterpret_cast<const frag_t*>(&sB[BUF][fb_off0]);          \
        const frag_t fa1_ = *reinterpret_cast<const frag_t*>(&sA[BUF][fa_off1]);          \
        const frag_t fb1_ = *reinterpret_cast<const frag_t*>(&sB[BUF][fb_off1]);          \
        acc = Mfma<AF16>::run(fb0_, fa0_, acc);                                           \
        acc = Mfma<AF16>::run(fb1_, fa1_, acc);                                           \
    } while (0)
#pragma unroll
    for (int j = 0; j < RING; ++j) RLHF_ROWS_GLOAD(j, j);  // nk >= RING (checked by the launcher)
    RLHF_ROWS_SSTORE(0, 0);
    __syncthreads();
    int kt0 = 0;
    for (; kt0 + RING < nk; kt0 += RING) {
#pragma unroll
        for (int j = 0; j < RING; ++j) {
            RLHF_ROWS_GLOAD(kt0 + j + RING, j);
            RLHF_ROWS_COMPUTE(j & 1);
            RLHF_ROWS_SSTORE((j + 1) & 1, (j + 1) % RING);
            __syncthreads();
        }
    }
#pragma unroll
    for (int j = 0; j < RING; ++j) {                       // the last RING tiles: nothing left to load
        RLHF_ROWS_COMPUTE(j & 1);
        if (j + 1 < RING) RLHF_ROWS_SSTORE((j + 1) & 1, j + 1);
        __syncthreads();
    }
#undef RLHF_ROWS_GLOAD
#undef RLHF_ROWS_CVT
#undef RLHF_ROWS_SSTORE
#undef RLHF_ROWS_COMPUTE
    // the lane holds row m = fr, tile columns w*16 + fq*4 + e
    if (MODE == 0) {
        const int n = blk * TN + w * 16 + fq * 4;
        if (fr < M && n + 3 < N)
            *reinterpret_cast<float4*>(C + (size_t)fr * N + n) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        else if (fr < M)
            for (int e = 0; e < 4; ++e)
                if (n + e < N) C[(size_t)fr * N + n + e] = acc[e];
        return;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) sx[fr][w * 16 + fq * 4 + e] = acc[e];
    __syncthreads();
    typedef typename std::conditional<AF16, f16_t, bf16_t>::type TO;
    if (MODE == 1) {
        TO* act = reinterpret_cast<TO*>(ep.act);
        for (int i = t; i < TM * 32; i += 256) {
            const int m = i >> 5, c = i & 31, oc = blk * 32 + c;
            if (m < M && oc < ep.ffn) {
                const float g = sx[m][c], u = sx[m][32 + c];
                act[(size_t)m * ep.ffn + oc] = from_f32<TO>(g / (1.f + __expf(-g)) * u);
            }
        }
        return;
    }
    if (MODE == 2) {
        const RopeOut& ro = ep.ro;
        const int hd = ro.head_dim, half = hd >> 1, per_head = half / 32;
        const int head = blk / per_head, c0 = (blk - head * per_head) * 32;
        const int Hq = ro.n_q_heads, Hkv = ro.n_kv_heads;
        TO* q_out = reinterpret_cast<TO*>(ro.q);
        TO* k_out = reinterpret_cast<TO*>(ro.k);
        TO* v_out = reinterpret_cast<TO*>(ro.v);
        TO* pool = reinterpret_cast<TO*>(ro.pool);
        for (int i = t; i < TM * 32; i += 256) {
            const int m = i >> 5, c = i & 31;
            if (m >= M) continue;
            float a = sx[m][c], b = sx[m][32 + c];           // dims c0 + c and c0 + c + half of the head
            if (head < Hq + Hkv) {
                const float* tab = ro.table + ((size_t)ro.pos[m] * half + c0 + c) * 2;
                const float cs = tab[0], sn = tab[1];
                const float fa_ = a * cs - b * sn, fb_ = a * sn + b * cs;
                a = fa_; b = fb_;
            }
            const int d0 = c0 + c, d1 = c0 + c + half;
            if (head < Hq) {
                TO* dst = q_out + ((size_t)m * Hq + head) * hd;
                dst[d0] = from_f32<TO>(a);
                dst[d1] = from_f32<TO>(b);
            } else {
                const bool is_k = head < Hq + Hkv;
                const int kh = is_k ? head - Hq : head - Hq - Hkv;
                TO* lin = is_k ? k_out : v_out;
                if (lin) {
                    lin[((size_t)m * Hkv + kh) * hd + d0] = from_f32<TO>(a);
                    lin[((size_t)m * Hkv + kh) * hd + d1] = from_f32<TO>(b);
                }
                if (pool) {
                    const int slot = ro.kv_dst[m], pt = ro.page_tokens;
                    TO* dst = pool + ((size_t)(slot / pt) * ro.n_layers + ro.layer) * 2 * (size_t)Hkv * pt * hd +
                              (size_t)(is_k ? 0 : Hkv) * pt * hd + (size_t)kh * pt * hd + (size_t)(slot % pt) * hd;
                    dst[d0] = from_f32<TO>(a);
                    dst[d1] = from_f32<TO>(b);
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------ fp32 path
// 64x64 tile, K step 16, 256 threads each computing a 4x4 block.
__global__ __launch_bounds__(256) void k_gemm_f32(const float* __restrict__ A,
                                                  const float* __restrict__ W,
                                                  float* __restrict__ C, int M, int N, int K,
                                                  int kchunk, int tiles_n) {
    __shared__ float sA[16][64 + 4];
    __shared__ float sB[16][64 + 4];
    const int tile = blockIdx.x;
    const int tm = tile / tiles_n, tn = tile - tm * tiles_n;
    const int m0 = tm * 64, n0 = tn * 64;
    const int split = blockIdx.y;
    const int kbeg = split * kchunk, kend = min(K, kbeg + kchunk);
    const int t = threadIdx.x;
    const int ty = t >> 4, tx = t & 15;        // 16 x 16 threads, 4 x 4 outputs each
    const int lr = t >> 2, lc = (t & 3) * 4;   // loader: row 0..63, k offset 0,4,8,12
    float acc[4][4] = {};
    for (int k0 = kbeg; k0 < kend; k0 += 16) {
        float4 va = make_float4(0, 0, 0, 0), vb = make_float4(0, 0, 0, 0);
        if (m0 + lr < M && k0 + lc < kend)
            va = *reinterpret_cast<const float4*>(A + (size_t)(m0 + lr) * K + k0 + lc);
        if (n0 + lr < N && k0 + lc < kend)
            vb = *reinterpret_cast<const float4*>(W + (size_t)(n0 + lr) * K + k0 + lc);
        __syncthreads();
        sA[lc + 0][lr] = va.x; sA[lc + 1][lr] = va.y; sA[lc + 2][lr] = va.z; sA[lc + 3][lr] = va.w;
        sB[lc + 0][lr] = vb.x; sB[lc + 1][lr] = vb.y; sB[lc + 2][lr] = vb.z; sB[lc + 3][lr] = vb.w;
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = sA[kk][ty * 4 + i]; b[i] = sB[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
        }
    }
    float* Cs = C + (size_t)split * M * N;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n < N) Cs[(size_t)m * N + n] = acc[i][j];
        }
    }
}

// ----------------------------------------------------------------------------- dispatch
namespace {
// Tilings.  Variants 1-4 stream the weights for few rows (split along K); 5-7 are the
// compute-bound tilings of prefill / scoring passes.  Measured at M = 8192 on the 7B layer
// shapes (half activations): 5: 650-820, 6: 800-900, 7: 950-1050 TFLOP/s.  Tried and dropped:
// 256x256 with four 128x128 wave tiles (750-830), global loads two tiles ahead (no change: L2
// latency is already hidden), fragment loads software-pipelined against the MFMAs (-5 %),
// 256x256 with 32-wide K tiles (half the LDS and fewer registers, so that a decode workgroup fits
// beside it on a compute unit: 740-890 alone, no net gain for the fused stage).  For up to 64
// rows, 64-column tiles (20-32 KB of LDS, 52-72 registers) stream as fast as or slightly faster
// than 128-column ones (36-48 KB, 68-108) and fit beside a 256x256 workgroup on a compute unit;
// 32-wide K tiles (64-byte row pieces) are slower.
struct TileCfg { int variant, tm, tn, tk; bool xcd; };
constexpr TileCfg kCfgs[] = {
    {0, 0, 0, 0, false},
    {1, 16, 64, 64, false}, {2, 32, 64, 64, false}, {3, 64, 64, 64, false}, {4, 128, 128, 64, false},
    {5, 128, 128, 64, true}, {6, 256, 128, 32, true}, {7, 256, 256, 64, true},
    {8, 16, 64, 64, false},      // k_gemm_rows16: up to 16 rows, whole K range per workgroup (no split)
};
constexpr int kNumCfgs = sizeof(kCfgs) / sizeof(kCfgs[0]);

// Few rows: the smallest row tile that holds them, weights streamed once, K split.  Many rows:
// the 256 x 256 tiling, unless its tiles would leave much of the chip idle (a prefill of a few
// hundred tokens, a narrow N): then 128 x 128 tiles with K split, which trades some efficiency
// per workgroup for having all compute units busy.
// 129..256 rows of a large matrix: one row of 256 x 256 tiles, K split so that the tiles times the
// splits come close to, and never exceed, one workgroup per compute unit (a second round of such
// workgroups costs more than it adds: at M = 256 the 7B-shape QKV takes 42.8 us with 4 splits = 192
// workgroups, 60 us with 6 = 288; gate||up 71 us with 2 = 172, 96 us with 3 = 258; against 54 and
// 97 us for 128 x 128 tiles).  Returns 0 when the tall tiling is not the better one.
int tall_split_for_mid_rows(int M, int N, int K, int max_split) {
    if (M <= 128 || M > 256 || K % 64 || (long)N * K < 40L * 1000 * 1000) return 0;
    const int tiles = (N + 255) / 256;
    int ns = 256 / tiles;
    if (ns > K / 256) ns = K / 256;          // at least four K tiles per split
    if (ns > 16) ns = 16;
    if (ns > max_split) ns = max_split;
    if (ns < 1 || tiles * ns < 160) return 0;
    while (ns > 1) {                          // every split gets a K range
        const int kchunk = ((K + ns - 1) / ns + 63) / 64 * 64;
        if ((long)(ns - 1) * kchunk < K) break;
        --ns;
    }
    return ns;
}

int pick_variant(int M, int N, int K = 0, int nsplit = 0) {
    if (M <= 16) return 1;
    if (M <= 32) return 2;
    if (M <= 64) return 3;
    if (M <= 256) return (K > 0 && nsplit > 0 && tall_split_for_mid_rows(M, N, K, nsplit) == nsplit) ? 7 : 4;
    const long tiles = (long)((M + 255) / 256) * ((N + 255) / 256);
    const long rounds = (tiles + 255) / 256;            // one 256 x 256 tile per compute unit at a time
    return tiles * 10 >= rounds * 256 * 6 ? 7 : 4;      // at least 60 % of the tile slots filled
}
constexpr int kTargetBlocks = 1024;      // about four workgroups per compute unit (tiles of up to 64 rows)
}  // namespace

// True when launch_gemm would run the 256 x 256 tiling for this shape and split (the shapes for
// which a half copy of the weights, if there is one, is the better operand).
// The tile a workgroup of a compute-bound launch takes (host copy of the device mapping, for tests).
int gemm_tall_grid(int tiles_m, int tiles_n) { return xcd_grid(tiles_m, tiles_n); }
bool gemm_tall_tile(int bid, int tiles_m, int tiles_n, int* tm, int* tn) {
    return tile_of<true>(bid, tiles_m, tiles_n, *tm, *tn);
}

bool gemm_is_tall(int M, int N, int K, int nsplit) { return K % 64 == 0 && kCfgs[pick_variant(M, N, K, nsplit)].xcd; }

// bf16 -> IEEE half, element by element (round toward zero; exact in half's normal range, values
// below 2^-14 land on half's subnormal grid): the same conversion the kernels apply on the fly.
__global__ void k_bf16_to_half(const uint32_t* __restrict__ src, uint32_t* __restrict__ dst, size_t n_pairs) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_pairs; i += (size_t)gridDim.x * 256)
        dst[i] = bf16x2_to_f16x2(src[i]);
}
hipError_t launch_bf16_to_half(hipStream_t st, const void* src, void* dst, size_t n) {
    if (n == 0) return hipSuccess;
    if (n % 2) return hipErrorInvalidValue;
    k_bf16_to_half<<<4096, 256, 0, st>>>((const uint32_t*)src, (uint32_t*)dst, n / 2);
    return hipGetLastError();
}

int gemm_choose_nsplit(int wdt, int M, int N, int K, int max_split) {
    int tm, tn, kgran;
    if (wdt == kBF16) {
        const int tall = tall_split_for_mid_rows(M, N, K, max_split);
        if (tall > 0) return tall;
        const TileCfg& c = kCfgs[pick_variant(M, N)];
        if (c.xcd) return 1;
        tm = c.tm; tn = c.tn; kgran = c.tk;
    } else { tm = 64; tn = 64; kgran = 16; }
    const long tiles = (long)((M + tm - 1) / tm) * ((N + tn - 1) / tn);
    const int kmax = K / (4 * kgran) > 0 ? K / (4 * kgran) : 1;   // keep >= 4 K tiles per split
    int ns;
    if (tm >= 128) {
        // 128-row tiles: every split writes a float plane of M x N that the consumer reads back,
        // which at these M is no longer small beside the weights.  Take the split that minimises
        // (weight bytes + plane bytes) / (share of the chip in use), 384 workgroups filling it.
        const double wbytes = 2.0 * N * K, plane = 8.0 * M * N;
        double best = 0;
        ns = 1;
        for (int c = 1; c <= kmax && c <= max_split; c *= 2) {
            const double fill = (double)(tiles * c) / 384.0;
            const double cost = (wbytes + plane * c) / (fill < 1.0 ? fill : 1.0);
            if (c == 1 || cost < best) { best = cost; ns = c; }
        }
    } else {
        ns = (int)((kTargetBlocks + tiles - 1) / tiles);
    }
    if (ns > kmax) ns = kmax;
    if (ns > max_split) ns = max_split;
    if (ns < 1) ns = 1;
    // a split that would get no K range is pointless: shrink until every split is non-empty
    while (ns > 1) {
        int kchunk = ((K + ns - 1) / ns + kgran - 1) / kgran * kgran;
        if ((long)(ns - 1) * kchunk < K) break;
        --ns;
    }
    return ns;
}

bool gemm_rows16_supported(int wdt, int adt, int M, int K) {
    return wdt == kBF16 && (adt == kF16 || adt == kBF16) && M >= 1 && M <= 16 && K % 64 == 0 && (K / 64) % 4 == 0;
}

// mode 0: plain (C float [M, N]); 1: SwiGLU (ep.act, ep.ffn; N = 2 * ffn); 2: rotary + KV append (ep.ro)
hipError_t launch_gemm_rows16(hipStream_t st, int wdt, int adt, int mode, const void* A, const void* W, float* C,
                              int M, int N, int K, const RowsEpi& ep, int nsplit) {
    if (!gemm_rows16_supported(wdt, adt, M, K) || mode < 0 || mode > 2 || nsplit < 1) return hipErrorInvalidValue;
    if (nsplit > 1 && (mode != 0 || (K / 64) % (4 * nsplit))) return hipErrorInvalidValue;
    int blocks = (N + 63) / 64;
    if (mode == 1) {
        if (!ep.act || ep.ffn <= 0 || N != 2 * ep.ffn) return hipErrorInvalidValue;
        blocks = (ep.ffn + 31) / 32;
    }
    if (mode == 2) {
        const RopeOut& ro = ep.ro;
        if ((ro.head_dim != 64 && ro.head_dim != 128) || !ro.pos || !ro.table || !ro.q || (ro.pool && !ro.kv_dst) ||
            N != (ro.n_q_heads + 2 * ro.n_kv_heads) * ro.head_dim)
            return hipErrorInvalidValue;
        blocks = N / 64;
    }
    const bf16_t* a = (const bf16_t*)A;
    const bf16_t* w = (const bf16_t*)W;
    const bool r8 = (K / 64 / nsplit) % 8 == 0;         // a split's K tiles must be a multiple of the ring depth
    const dim3 grid(blocks, nsplit);
#define RLHF_ROWS(MODE_, AF_)                                                                          \
    do {                                                                                               \
        if (r8) k_gemm_rows16<8, MODE_, AF_><<<grid, 256, 0, st>>>(a, w, C, M, N, K, ep);              \
        else k_gemm_rows16<4, MODE_, AF_><<<grid, 256, 0, st>>>(a, w, C, M, N, K, ep);                 \
    } while (0)
    if (adt == kF16) {
        if (mode == 0) RLHF_ROWS(0, true); else if (mode == 1) RLHF_ROWS(1, true); else RLHF_ROWS(2, true);
    } else {
        if (mode == 0) RLHF_ROWS(0, false); else if (mode == 1) RLHF_ROWS(1, false); else RLHF_ROWS(2, false);
    }
#undef RLHF_ROWS
    return hipGetLastError();
}

template <bool AF16>
static hipError_t launch_bf16(hipStream_t st, int variant, const bf16_t* a, const bf16_t* w, float* C, int M,
                              int N, int K, int nsplit) {
    const TileCfg& c = kCfgs[variant];
    const int tiles_m = (M + c.tm - 1) / c.tm, tiles_n = (N + c.tn - 1) / c.tn;
    const int kchunk = ((K + nsplit - 1) / nsplit + c.tk - 1) / c.tk * c.tk;
    int blocks = tiles_m * tiles_n;
    if (c.xcd) blocks = xcd_grid(tiles_m, tiles_n);
    dim3 grid(blocks, nsplit);
#define RLHF_GEMM(TM, TN, TK, WM, WN, XCD)                                                            \
    k_gemm_bf16<TM, TN, TK, WM, WN, AF16, XCD, false><<<grid, WM * WN * 64, 0, st>>>(a, w, C, M, N, K, kchunk, \
                                                                                     tiles_m, tiles_n)
    switch (variant) {
        case 1: RLHF_GEMM(16, 64, 64, 1, 4, false); break;
        case 2: RLHF_GEMM(32, 64, 64, 1, 4, false); break;
        case 3: RLHF_GEMM(64, 64, 64, 2, 2, false); break;
        case 4: RLHF_GEMM(128, 128, 64, 2, 2, false); break;
        case 8: {
            if (!gemm_rows16_supported(kBF16, AF16 ? kF16 : kBF16, M, K)) return hipErrorInvalidValue;
            return launch_gemm_rows16(st, kBF16, AF16 ? kF16 : kBF16, 0, a, w, C, M, N, K, RowsEpi{}, nsplit);
        }
        case 5: RLHF_GEMM(128, 128, 64, 2, 2, true); break;
        case 6: RLHF_GEMM(256, 128, 32, 2, 2, true); break;
        case 7:                                                  // eight waves, wave tile 64 x 128
            if (K % 64 == 0)
                k_gemm_bf16<256, 256, 64, 4, 2, AF16, true, false, true><<<grid, 512, 0, st>>>(a, w, C, M, N, K, kchunk,
                                                                                             tiles_m, tiles_n);
            else
                RLHF_GEMM(256, 256, 64, 4, 2, true);
            break;
        default: return hipErrorInvalidValue;
    }
#undef RLHF_GEMM
    return hipGetLastError();
}

// wdt == kF16: the matrix is a half copy of the bf16 weights and goes global -> LDS directly.
static bool half_weights_ok(int wdt, int adt, int K) { return wdt != kF16 || (adt == kF16 && K % 64 == 0); }
// the half-weight kernels address both operands with 32-bit byte offsets per lane
static bool half_offsets_ok(int wdt, long M, long N, long K) {
    return wdt != kF16 || ((M > N ? M : N) * K * 2 < (1L << 32));
}

bool gemm_swiglu_supported(int wdt, int adt, int M, int ffn, int K) {
    return (wdt == kBF16 || wdt == kF16) && half_weights_ok(wdt, adt, K) && (adt == kF16 || adt == kBF16) && M >= 512 &&
           ffn % 8 == 0 && K % 8 == 0;
}

hipError_t launch_gemm_swiglu(hipStream_t st, int wdt, int adt, const void* A, const void* W_gate_up,
                              void* act, int M, int ffn, int K) {
    if (!gemm_swiglu_supported(wdt, adt, M, ffn, K) || !half_offsets_ok(wdt, M, 2L * ffn, K)) return hipErrorInvalidValue;
    constexpr int TM = 256, TN = 256;
    const int N = 2 * ffn;
    const int tiles_m = (M + TM - 1) / TM, tiles_n = (N + TN - 1) / TN;
    dim3 grid(xcd_grid(tiles_m, tiles_n), 1);
    const int kchunk = (K + 63) / 64 * 64;
#define RLHF_SWIGLU(AF, DMA)                                               \
    k_gemm_bf16<TM, TN, 64, 4, 2, AF, true, true, DMA><<<grid, 512, 0, st>>>( \
        (const bf16_t*)A, (const bf16_t*)W_gate_up, (float*)act, M, N, K, kchunk, tiles_m, tiles_n)
    const bool dma = K % 64 == 0;
    if (wdt == kF16)
        k_gemm_bf16<TM, TN, 64, 4, 2, true, true, true, true, 0, false, true><<<grid, 512, 0, st>>>(
            (const bf16_t*)A, (const bf16_t*)W_gate_up, (float*)act, M, N, K, kchunk, tiles_m, tiles_n);
    else if (adt == kF16) { if (dma) RLHF_SWIGLU(true, true); else RLHF_SWIGLU(true, false); }
    else { if (dma) RLHF_SWIGLU(false, true); else RLHF_SWIGLU(false, false); }
#undef RLHF_SWIGLU
    return hipGetLastError();
}

bool gemm_rope_supported(int wdt, int adt, int M, int K, const Dims& dm) {
    return (wdt == kBF16 || wdt == kF16) && half_weights_ok(wdt, adt, K) && (adt == kF16 || adt == kBF16) && M >= 512 &&
           K % 64 == 0 && (dm.head_dim == 64 || dm.head_dim == 128);
}

hipError_t launch_gemm_rope(hipStream_t st, int wdt, int adt, const void* A, const void* Wqkv, int M, int K,
                            const RopeOut& ro) {
    Dims dm{};
    dm.head_dim = ro.head_dim;
    if (!gemm_rope_supported(wdt, adt, M, K, dm) || !ro.pos || !ro.table || !ro.q || (ro.pool && !ro.kv_dst))
        return hipErrorInvalidValue;
    constexpr int TM = 256, TN = 256;
    const int N = (ro.n_q_heads + 2 * ro.n_kv_heads) * ro.head_dim;
    if (!half_offsets_ok(wdt, M, N, K)) return hipErrorInvalidValue;
    const int tiles_m = (M + TM - 1) / TM, tiles_n = (N + TN - 1) / TN;
    dim3 grid(xcd_grid(tiles_m, tiles_n), 1);
    const bf16_t* a = (const bf16_t*)A;
    const bf16_t* w = (const bf16_t*)Wqkv;
#define RLHF_ROPE(AF, HD)                                                                             \
    k_gemm_bf16<TM, TN, 64, 4, 2, AF, true, false, true, HD><<<grid, 512, 0, st>>>(a, w, nullptr, M, N, K, K, \
                                                                                   tiles_m, tiles_n, ro)
#define RLHF_ROPE_HALF_W(HD)                                                                                    \
    k_gemm_bf16<TM, TN, 64, 4, 2, true, true, false, true, HD, false, true><<<grid, 512, 0, st>>>(a, w, nullptr, M, N, \
                                                                                                  K, K, tiles_m, tiles_n, ro)
    if (wdt == kF16) { if (ro.head_dim == 128) RLHF_ROPE_HALF_W(128); else RLHF_ROPE_HALF_W(64); }
    else if (adt == kF16) { if (ro.head_dim == 128) RLHF_ROPE(true, 128); else RLHF_ROPE(true, 64); }
    else { if (ro.head_dim == 128) RLHF_ROPE(false, 128); else RLHF_ROPE(false, 64); }
#undef RLHF_ROPE
#undef RLHF_ROPE_HALF_W
    return hipGetLastError();
}

bool gemm_lse_supported(int wdt, int adt, int K) {
    return (wdt == kBF16 || wdt == kF16) && half_weights_ok(wdt, adt, K) && (adt == kF16 || adt == kBF16) && K % 64 == 0;
}

int gemm_lse_partials(int N) { return (N + 255) / 256 * 2; }

hipError_t launch_gemm_lse(hipStream_t st, int wdt, int adt, const void* A, const void* W_head, int M, int N, int K,
                           const LseOut& lo) {
    if (M <= 0) return hipSuccess;
    if (!gemm_lse_supported(wdt, adt, K) || N <= 0 || !lo.tokens || !lo.target_idx || !lo.part_max || !lo.part_sum ||
        !lo.tgt || lo.n_part != gemm_lse_partials(N) || !half_offsets_ok(wdt, M, N, K))
        return hipErrorInvalidValue;
    constexpr int TM = 256, TN = 256;
    const int tiles_m = (M + TM - 1) / TM, tiles_n = (N + TN - 1) / TN;
    dim3 grid(xcd_grid(tiles_m, tiles_n), 1);
    const bf16_t* a = (const bf16_t*)A;
    const bf16_t* w = (const bf16_t*)W_head;
    if (wdt == kF16)
        k_gemm_bf16<TM, TN, 64, 4, 2, true, true, false, true, 0, true, true><<<grid, 512, 0, st>>>(
            a, w, nullptr, M, N, K, K, tiles_m, tiles_n, RopeOut{}, lo);
    else if (adt == kF16)
        k_gemm_bf16<TM, TN, 64, 4, 2, true, true, false, true, 0, true><<<grid, 512, 0, st>>>(
            a, w, nullptr, M, N, K, K, tiles_m, tiles_n, RopeOut{}, lo);
    else
        k_gemm_bf16<TM, TN, 64, 4, 2, false, true, false, true, 0, true><<<grid, 512, 0, st>>>(
            a, w, nullptr, M, N, K, K, tiles_m, tiles_n, RopeOut{}, lo);
    return hipGetLastError();
}

hipError_t launch_gemm(hipStream_t st, int wdt, int adt, const void* A, const void* W, float* C,
                       int M, int N, int K, int nsplit, int variant) {
    if (M <= 0 || N <= 0) return hipSuccess;
    if (nsplit < 1 || K <= 0) return hipErrorInvalidValue;
    if (wdt == kF16) {
        // half copy of a bf16 matrix: the tall tiling with both operands global -> LDS directly
        if (adt != kF16 || K % 64 || (variant != 0 && variant != 7) || !half_offsets_ok(wdt, M, N, K))
            return hipErrorInvalidValue;
        const int tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
        const int kchunk = ((K + nsplit - 1) / nsplit + 63) / 64 * 64;
        if ((long)(nsplit - 1) * kchunk >= K) return hipErrorInvalidValue;
        dim3 grid(xcd_grid(tiles_m, tiles_n), nsplit);
        k_gemm_bf16<256, 256, 64, 4, 2, true, true, false, true, 0, false, true><<<grid, 512, 0, st>>>(
            (const bf16_t*)A, (const bf16_t*)W, C, M, N, K, kchunk, tiles_m, tiles_n);
        return hipGetLastError();
    }
    if (wdt == kBF16) {
        if (adt != kBF16 && adt != kF16) return hipErrorInvalidValue;
        if (K % 8 || variant < 0 || variant >= kNumCfgs) return hipErrorInvalidValue;
        if (variant == 0) {
            variant = pick_variant(M, N, K, nsplit);
            if (kCfgs[variant].xcd && nsplit != 1 && M > 256) variant = 4;   // a caller-imposed split of a tall GEMM
        }
        const bf16_t* a = (const bf16_t*)A;
        const bf16_t* w = (const bf16_t*)W;
        return adt == kF16 ? launch_bf16<true>(st, variant, a, w, C, M, N, K, nsplit)
                           : launch_bf16<false>(st, variant, a, w, C, M, N, K, nsplit);
    }
    if (K % 4 || adt != kF32) return hipErrorInvalidValue;
    const int tiles_m = (M + 63) / 64, tiles_n = (N + 63) / 64;
    const int kchunk = ((K + nsplit - 1) / nsplit + 15) / 16 * 16;
    dim3 grid(tiles_m * tiles_n, nsplit);
    k_gemm_f32<<<grid, 256, 0, st>>>((const float*)A, (const float*)W, C, M, N, K, kchunk, tiles_n);
    return hipGetLastError();
}

}  // namespace rlhf
