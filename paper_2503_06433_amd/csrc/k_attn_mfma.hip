// bf16 MFMA attention for gfx950 against the paged cache: causal prefill and
// split-KV decode.  Both kernels compute the TRANSPOSED products
//     S^T = K * Q^T        (rows = cached tokens, columns = queries)
//     O^T = V^T * P^T      (rows = head dimension, columns = queries)
// so that the accumulator of the first product is already in the register
// layout the second product wants for its B operand (each lane owns one query
// column and a run of tokens): P never travels through LDS or across lanes.
// K pages are [head][16][D] and V pages are stored transposed, [head][D][16] (token order 0-3, 8-11, 4-7, 12-15),
// so both MFMA A operands are plain vector loads straight from the pages.
//
// The contraction order inside one MFMA is free as long as both operands agree:
// the token <-> k-slot assignment below is chosen to match what the S^T
// accumulator holds, and the V^T operand is gathered with the same assignment.
#include <type_traits>

#include "ss_device.h"
#include "ss_kernels.h"

namespace SS_NS {
using namespace ssk;

// 2^x on the hardware's exponential unit (v_exp_f32, about 1 ulp for normal results; results below the
// normal range flush to zero, which a softmax weight may).  The library exp2f wraps the same instruction
// in range scaling for denormal results: four more VALU operations per element in the innermost loop.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// max of a value with the one held by the lane 32 positions away (v_permlane32_swap: no LDS round trip)
__device__ __forceinline__ float max_with_other_half(float x) {
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

typedef half8_t bf16x8_t;       // MFMA operand: 8 elements of the 16-bit type
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef int i32x8_t __attribute__((ext_vector_type(8)));

struct __attribute__((aligned(8))) vec8 { uint32_t w[2]; };

union Frag {
    bf16x8_t v;
    vec16 q;
    vec8 h[2];
    uint32_t w[4];
};

// ======================================================================
// Prefill.  Block = 4 waves = 256 consecutive queries of one (sequence, q head);
// each wave owns QT = 2 tiles of 32 queries and walks the pages its queries can
// see, two pages (32 tokens) per step, with v_mfma_f32_32x32x16_bf16:
//   accumulator register v of lane l <-> token 8*(v/4) + 4*(l/32) + v%4, query l%32.
// Every K and V^T fragment loaded from the pages feeds both query tiles.
// ======================================================================
template <int D, int QT>
__global__ __launch_bounds__(256) void attn_prefill_mfma_kernel(const bf16_t* __restrict__ qkv,
                                                                bf16_t* __restrict__ out, int n_q, int n_kv,
                                                                BatchMeta bm, const bf16_t* __restrict__ k_pool,
                                                                const bf16_t* __restrict__ v_pool,
                                                                float scale_log2e) {
    constexpr int KS = D / 16;      // k-steps of the score product
    constexpr int DT = D / 32;      // 32-row tiles of O^T
    const int sq = blockIdx.z, a = blockIdx.y;
    const int q_begin = bm.cu_q[sq], q_len = bm.cu_q[sq + 1] - q_begin;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q0 = blockIdx.x * (128 * QT) + wave * (32 * QT);
    if (q0 >= q_len) return;
    const int before = bm.kv_before[sq];
    const int g = a / (n_q / n_kv);
    const int lq = lane & 31, g2 = lane >> 5;
    const int last_q = (q0 + 32 * QT - 1 < q_len) ? q0 + 32 * QT - 1 : q_len - 1;
    const int n_pages = (before + last_q) / 16 + 1;
    const size_t row_stride = (size_t)(n_q + 2 * n_kv) * D;

    Frag qf[QT][KS];
    int p[QT];
    bool valid[QT];
#pragma unroll
    for (int t = 0; t < QT; ++t) {
        const int qi = q0 + t * 32 + lq;
        valid[t] = qi < q_len;
        p[t] = before + (valid[t] ? qi : 0);
        const bf16_t* qp = qkv + (size_t)(q_begin + (valid[t] ? qi : 0)) * row_stride + (size_t)a * D + g2 * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[t][ks].q = *reinterpret_cast<const vec16*>(qp + ks * 16);
    }
    f32x16_t o[QT][DT];
    float m[QT], l[QT];
#pragma unroll
    for (int t = 0; t < QT; ++t) {
        m[t] = -INFINITY;
        l[t] = 0.f;
#pragma unroll
        for (int u = 0; u < DT; ++u)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[t][u][v] = 0.f;
    }

    const int32_t* pt = bm.page_tables + (size_t)sq * bm.pt_stride;
    const size_t page_elems = (size_t)n_kv * 16 * D;
    const size_t head_off = (size_t)g * 16 * D;
    const int tok = lq;                       // token row this lane loads of the 32-token step
    for (int pi = 0; pi < n_pages; pi += 2) {
        const int pA = pt[pi];
        const int pB = pt[(pi + 1 < n_pages) ? pi + 1 : pi];
        // ---- S^T = K Q^T for both query tiles
        const bf16_t* kp = k_pool + (size_t)(tok < 16 ? pA : pB) * page_elems + head_off + (size_t)(tok & 15) * D + g2 * 8;
        f32x16_t s[QT];
#pragma unroll
        for (int t = 0; t < QT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) s[t][v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            Frag kf;
            kf.q = *reinterpret_cast<const vec16*>(kp + ks * 16);
#pragma unroll
            for (int t = 0; t < QT; ++t) s[t] = SS_MFMA_32x32x16(kf.v, qf[t][ks].v, s[t], 0, 0, 0);
        }
        // ---- mask + streaming softmax (per query column = per lane pair l, l^32)
        const int t0 = pi * 16;
        Frag pfA[QT], pfB[QT];
#pragma unroll
        for (int t = 0; t < QT; ++t) {
            float mx = m[t];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int tpos = t0 + 8 * (v >> 2) + 4 * g2 + (v & 3);
                s[t][v] = (tpos <= p[t]) ? s[t][v] * scale_log2e : -INFINITY;
                mx = fmaxf(mx, s[t][v]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float alpha = fast_exp2(m[t] - mx);
            m[t] = mx;
            float rs = 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) { s[t][v] = fast_exp2(s[t][v] - mx); rs += s[t][v]; }
            l[t] = l[t] * alpha + rs;
#pragma unroll
            for (int u = 0; u < DT; ++u)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[t][u][v] *= alpha;
            // k-slots of step A: tokens {4*g2 + i, 8 + 4*g2 + i} of page A; step B: the same of page B
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                pfA[t].w[i] = pack_bf16x2(s[t][2 * i], s[t][2 * i + 1]);
                pfB[t].w[i] = pack_bf16x2(s[t][8 + 2 * i], s[t][8 + 2 * i + 1]);
            }
        }
        // ---- O^T += V^T P^T
        // the page keeps each row as [0-3, 8-11, 4-7, 12-15] (halves swapped in rows with bit 3 of the row index set,
        // see vpos): lane group g2's eight tokens are 16 contiguous bytes
        const int vhalf = g2 ^ ((lq >> 3) & 1);
        const bf16_t* vA = v_pool + (size_t)pA * page_elems + head_off + (size_t)lq * 16 + 8 * vhalf;
        const bf16_t* vB = v_pool + (size_t)pB * page_elems + head_off + (size_t)lq * 16 + 8 * vhalf;
#pragma unroll
        for (int u = 0; u < DT; ++u) {
            Frag va, vb;
            va.q = *reinterpret_cast<const vec16*>(vA + u * 32 * 16);
            vb.q = *reinterpret_cast<const vec16*>(vB + u * 32 * 16);
#pragma unroll
            for (int t = 0; t < QT; ++t) {
                o[t][u] = SS_MFMA_32x32x16(va.v, pfA[t].v, o[t][u], 0, 0, 0);
                o[t][u] = SS_MFMA_32x32x16(vb.v, pfB[t].v, o[t][u], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < QT; ++t) {
        l[t] += __shfl_xor(l[t], 32, 64);
        if (valid[t]) {
            const float inv = 1.0f / l[t];
            bf16_t* op = out + (size_t)(q_begin + q0 + t * 32 + lq) * ((size_t)n_q * D) + (size_t)a * D;
#pragma unroll
            for (int u = 0; u < DT; ++u)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    vec8 w;
                    w.w[0] = pack_bf16x2(o[t][u][4 * j] * inv, o[t][u][4 * j + 1] * inv);
                    w.w[1] = pack_bf16x2(o[t][u][4 * j + 2] * inv, o[t][u][4 * j + 3] * inv);
                    *reinterpret_cast<vec8*>(op + u * 32 + 8 * j + 4 * g2) = w;
                }
        }
    }
}

// ----------------------------------------------------------------------
// Prefill, LDS-staged.  A block of 8 waves works on one item at a time: 256 consecutive queries of one (sequence, q head).  The K
// and V^T chunks of 64 tokens (4 pages, 32 KB) are brought into a three-stage LDS ring (two tiles in flight) with direct
// global->LDS loads and shared by all eight waves, which cuts the L2 traffic of the attention by 8
// against every wave fetching its own operands.  K rows (256 bytes) are stored with the 16-byte
// chunk index XOR-ed with the row number, so the 16 rows one pass of a fragment read touches fall
// on different banks; V^T chunks are stored exactly as in the page (a fragment read is 1 KB
// contiguous).  A wave skips the MFMAs of tiles none of its queries can see, but takes part in every
// load and barrier.
// ----------------------------------------------------------------------
__device__ __forceinline__ void dma16a(const void* gptr, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_addr) : "memory");
}

template <int D>
__global__ __launch_bounds__(512) void attn_prefill_lds_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ out,
                                                               int n_q, int n_kv, BatchMeta bm,
                                                               const bf16_t* __restrict__ k_pool,
                                                               const bf16_t* __restrict__ v_pool, float scale_log2e) {
    static_assert(D == 128, "layout below assumes 256-byte K rows");
    constexpr int KS = D / 16, DT = D / 32, NS = 3;
    constexpr int KBYTES = 64 * D * 2, STAGE = 2 * KBYTES;     // 16 KB of K + 16 KB of V^T
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    // Persistent blocks, one per compute unit: block b walks its list of items (sequence, q head, block of
    // 256 queries) that the host has laid out (see BatchMeta::pf_items): launching a block of this size per
    // item costs 3-4 us of dispatch each, a sixth of the kernel's time on prompts of one or two thousand tokens.
    const int G = n_q / n_kv;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lq = lane & 31, g2 = lane >> 5;
    const size_t row_stride = (size_t)(n_q + 2 * n_kv) * D;
    const size_t page_elems = (size_t)n_kv * 16 * D;
    const uint32_t lds_base = (uint32_t)(uintptr_t)smem;
    for (int pj = 0;; ++pj) {
    // the item's record through the scalar cache: one load, a few hundred nanoseconds (as ordinary loads the
    // six values would be as many dependent round trips, the loop's memory clobbers keep them from being merged)
    const int32_t* item = bm.pf_items + ((size_t)blockIdx.x * bm.pf_stride + pj) * 8;
    i32x8_t rec;
    asm volatile("s_load_dwordx8 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(rec) : "s"(item) : "memory");
    const int sq = rec[0];
    if (sq < 0) break;                                         // end of the list: the whole block leaves
    const int a = rec[1], qb0 = rec[2], q_begin = rec[3], q_len = rec[4];
    const int g = a / G;
    // every wave is done with the LDS stages of the previous item before the first requests of this one
    __builtin_amdgcn_s_barrier();
    const int before = rec[5];
    const int q0 = qb0 + wave * 32;
    const int qi = q0 + lq;
    const bool valid = qi < q_len;
    const int p = before + (valid ? qi : 0);
    // last position any query of this wave / of the block can see
    const int wave_last = before + ((q0 + 31 < q_len) ? q0 + 31 : q_len - 1);
    const bool wave_active = q0 < q_len;
    const int blk_last = before + ((qb0 + 255 < q_len) ? qb0 + 255 : q_len - 1);
    const int n_pages = blk_last / 16 + 1;
    const int n_tiles = (n_pages + 3) / 4;
    const int32_t* pt = bm.page_tables + (size_t)sq * bm.pt_stride;
    const size_t head_off = (size_t)g * 16 * D;

    f32x16_t o[DT];
#pragma unroll
    for (int u = 0; u < DT; ++u)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[u][v] = 0.f;
    float m = -INFINITY, l = 0.f;

    // DMA assignment per stage: wave w brings K rows [8w, 8w+8) (two loads of 4 rows) and V^T pieces 2w, 2w+1
    // (piece i = page i/4 of the tile, d rows [32*(i%4), +32): 1 KB contiguous in the page).  All of a wave's
    // rows and pieces lie in page w/2 of the tile, so one page-table entry per wave and tile is needed.  Lane i
    // holds the entry for tile pages_base + i (refilled every 64 tiles) and the loop picks it with a lane
    // read: no memory access, and so no wait for one, sits between the barrier and the requests.
    int pages_vec;
    auto load_pages = [&](int base) {
        int pg = (base + lane) * 4 + (wave >> 1);
        pg = pg < n_pages ? pg : n_pages - 1;
        pages_vec = pt[pg];
    };
    load_pages(0);
    auto issue = [&](int tile) {
        const uint32_t st = lds_base + (uint32_t)(tile % NS) * STAGE;
        const int page = __builtin_amdgcn_readlane(pages_vec, tile & 63);
        const size_t page_off = (size_t)page * page_elems + head_off;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = wave * 8 + i * 4 + (lane >> 4);     // token row of the tile
            const int chunk = (lane & 15) ^ (row & 15);
            const bf16_t* src = k_pool + page_off + (size_t)(row & 15) * D + chunk * 8;
            dma16a(src, st + (wave * 8 + i * 4) * 256);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int piece = wave * 2 + i;
            const bf16_t* src = v_pool + page_off + (size_t)(piece & 3) * 512 + lane * 8;
            dma16a(src, st + KBYTES + piece * 1024);
        }
    };

    // One step of the streaming softmax (base 2, scale folded into the exponent) on the 32 tokens of a
    // score accumulator: updates m and l, leaves the weights packed as the B operands of the two P V
    // products and returns the factor the accumulated output has to be multiplied by.  The reference
    // maximum m follows the true running maximum only when that has grown by more than 8 (in the exponent's
    // units): until then weights may reach 2^8 instead of 1, which fp32 sums and the 16-bit weights hold
    // without loss, the result o / l is the same, and the 64 multiplications of the output accumulator
    // are skipped in all but the first steps of a row.
    auto softmax_step = [&](f32x16_t& sc, Frag& pfA, Frag& pfB) {
        float mr = fmaxf(fmaxf(sc[0], sc[1]), sc[2]);
#pragma unroll
        for (int v = 3; v < 15; v += 2) mr = fmaxf(fmaxf(mr, sc[v]), sc[v + 1]);
        mr = fmaxf(mr, sc[15]);
        mr = max_with_other_half(mr);
        const float mx = fmaxf(m, mr * scale_log2e);
        const bool moved = mx - m > 8.0f;               // also true for the first step (m = -inf)
        const float alpha = moved ? fast_exp2(m - mx) : 1.0f;
        m = moved ? mx : m;
        float rs = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) { sc[v] = fast_exp2(fmaf(sc[v], scale_log2e, -m)); rs += sc[v]; }
        l = l * alpha + rs;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            pfA.w[i] = pack_bf16x2(sc[2 * i], sc[2 * i + 1]);
            pfB.w[i] = pack_bf16x2(sc[8 + 2 * i], sc[8 + 2 * i + 1]);
        }
        // the weights are complete here, not wherever their first use is moved to
        asm volatile("" : "+v"(pfA.w[0]), "+v"(pfA.w[1]), "+v"(pfA.w[2]), "+v"(pfA.w[3]), "+v"(pfB.w[0]), "+v"(pfB.w[1]),
                          "+v"(pfB.w[2]), "+v"(pfB.w[3]));
        return alpha;
    };
    // causal mask of a score accumulator whose first token is t0
    auto mask_step = [&](f32x16_t& sc, int t0) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int tpos = t0 + 8 * (v >> 2) + 4 * g2 + (v & 3);
            sc[v] = (tpos <= p) ? sc[v] : -INFINITY;
        }
    };
    auto rescale = [&](float alpha) {
        if (__ballot(alpha != 1.0f) != 0ull) {          // the reference maximum moved for some query of the wave
#pragma unroll
            for (int u = 0; u < DT; ++u)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[u][v] *= alpha;
        }
    };

    // Start of a block: the page-table entries first (the tile requests need them), then the requests for
    // the first two tiles, then the query fragments, whose load latency the tile requests overlap.  The query
    // fragments are loads into registers, the tiles loads into LDS; the two kinds do not complete in issue
    // order with respect to each other, so the counter arithmetic of the loop (vmcnt <= 4: everything but
    // the newest tile has landed) holds only while nothing but tile loads is in flight: the loop is entered
    // with everything landed.  (The empty statements make the loaded registers inputs of something that
    // precedes, in program order, what must follow the load.)
    asm volatile("" : "+v"(pages_vec));
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_sched_barrier(0);
    issue(0);
    if (n_tiles > 1) issue(1);
    Frag qf[KS];
    {
        const bf16_t* qp = qkv + (size_t)(q_begin + (valid ? qi : 0)) * row_stride + (size_t)a * D + g2 * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks].q = *reinterpret_cast<const vec16*>(qp + ks * 16);
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qf[ks].w[0]), "+v"(qf[ks].w[1]), "+v"(qf[ks].w[2]), "+v"(qf[ks].w[3]));
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_sched_barrier(0);
    // No tile is requested past the last one (the block would only have to wait for it at the end), so the
    // last iteration waits for everything and the others for all but the newest tile.
    for (int it = 0; it < n_tiles; ++it) {
        if (it + 1 < n_tiles) __builtin_amdgcn_s_waitcnt(0x0F74);     // vmcnt <= 4: this wave's part of tile `it` has landed
        else __builtin_amdgcn_s_waitcnt(0x0F70);
        __builtin_amdgcn_s_barrier();                  // everyone's part landed; stage (it-1)%NS is free
        __builtin_amdgcn_sched_barrier(0);
        if (it + 2 < n_tiles) {
            if (((it + 2) & 63) == 0) {                // every 64 tiles; waited for here, so that no wait
                load_pages(it + 2);                    // is due where the entries are picked
                __builtin_amdgcn_s_waitcnt(0x0F70);
            }
            issue(it + 2);
        }
        if (!wave_active || it * 64 > wave_last) continue;     // nothing visible to this wave in the tile
        const uint8_t* st = smem + (it % NS) * STAGE;
        // The two halves of 32 tokens are software-pipelined so that the MFMA pipe and the vector ALU work at
        // the same time: the score product of the second half is issued next to the softmax of the first,
        // the P V product of the first half next to the softmax of the second, and every LDS fragment read
        // is issued a phase ahead of its use.  Only the last tile or two of a wave hold tokens that some of
        // its queries must not see (wave-uniform test); a half that is hidden altogether is computed and
        // masked like the rest (weights 0).
        const bool diag = it * 64 + 63 > before + q0;
        const uint8_t* kp = st + lq * 256;
        const int sw = lq & 15;                         // rows lq and 32 + lq share the swizzle
        Frag ka[KS], kb[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) ka[ks].v = *reinterpret_cast<const bf16x8_t*>(kp + (((ks * 2 + g2) ^ sw) << 4));
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kb[ks].v = *reinterpret_cast<const bf16x8_t*>(kp + 32 * 256 + (((ks * 2 + g2) ^ sw) << 4));
        f32x16_t s0, s1;
#pragma unroll
        for (int v = 0; v < 16; ++v) { s0[v] = 0.f; s1[v] = 0.f; }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) s0 = SS_MFMA_32x32x16(ka[ks].v, qf[ks].v, s0, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        const uint8_t* vp = st + KBYTES + lq * 32 + (g2 ^ ((lq >> 3) & 1)) * 16;      // halves swapped in rows 8-15 of 16 (vpos)
        Frag va[DT], vb[DT];
#pragma unroll
        for (int u = 0; u < DT; ++u) {
            va[u].v = *reinterpret_cast<const bf16x8_t*>(vp + u * 1024);
            vb[u].v = *reinterpret_cast<const bf16x8_t*>(vp + 4096 + u * 1024);
        }
        if (diag) mask_step(s0, it * 64);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) s1 = SS_MFMA_32x32x16(kb[ks].v, qf[ks].v, s1, 0, 0, 0);
        Frag pA, pB;
        float alpha = softmax_step(s0, pA, pB);
#pragma unroll
        for (int i = 0; i < KS; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);      // vector ALU work of the softmax
            __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);      // two exponentials
        }
        __builtin_amdgcn_sched_barrier(0);
        if (diag) mask_step(s1, it * 64 + 32);
        rescale(alpha);
        Frag vc[DT], vd[DT];
#pragma unroll
        for (int u = 0; u < DT; ++u) {
            vc[u].v = *reinterpret_cast<const bf16x8_t*>(vp + 8192 + u * 1024);
            vd[u].v = *reinterpret_cast<const bf16x8_t*>(vp + 12288 + u * 1024);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < DT; ++u) {
            o[u] = SS_MFMA_32x32x16(va[u].v, pA.v, o[u], 0, 0, 0);
            o[u] = SS_MFMA_32x32x16(vb[u].v, pB.v, o[u], 0, 0, 0);
        }
        Frag pC, pD;
        alpha = softmax_step(s1, pC, pD);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);          // the row maximum has to be there before
        __builtin_amdgcn_sched_group_barrier(0x002, 16, 0);         // the first exponential
#pragma unroll
        for (int i = 1; i < 2 * DT; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 7, 0);
            __builtin_amdgcn_sched_group_barrier(0x400, 3, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        rescale(alpha);
#pragma unroll
        for (int u = 0; u < DT; ++u) {
            o[u] = SS_MFMA_32x32x16(vc[u].v, pC.v, o[u], 0, 0, 0);
            o[u] = SS_MFMA_32x32x16(vd[u].v, pD.v, o[u], 0, 0, 0);
        }
    }
    l += __shfl_xor(l, 32, 64);
    if (valid) {
        const float inv = 1.0f / l;
        bf16_t* op = out + (size_t)(q_begin + qi) * ((size_t)n_q * D) + (size_t)a * D;
#pragma unroll
        for (int u = 0; u < DT; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                vec8 w;
                w.w[0] = pack_bf16x2(o[u][4 * j] * inv, o[u][4 * j + 1] * inv);
                w.w[1] = pack_bf16x2(o[u][4 * j + 2] * inv, o[u][4 * j + 3] * inv);
                *reinterpret_cast<vec8*>(op + u * 32 + 8 * j + 4 * g2) = w;
            }
    }
    }   // items
}

hipError_t attn_generic(int dt, const void* qkv, void* out, int n_q, int n_kv, const BatchMeta& bm,
                        const KvLayer& kv, hipStream_t s);

hipError_t attn_prefill(int dt, const void* qkv, void* out, int n_q, int n_kv, const BatchMeta& bm,
                        const KvLayer& kv, bool force_generic, hipStream_t s) {
    if (bm.T <= 0 || bm.n_seqs <= 0) return hipSuccess;
    if (dt != BF16 || force_generic || kv.d != 128) return attn_generic(dt, qkv, out, n_q, n_kv, bm, kv, s);
    if (kv.page_size != 16 || n_kv <= 0 || n_q % n_kv != 0 || kv.n_heads != n_kv) return hipErrorInvalidValue;
    if (bm.n_seqs > 65535 || n_q > 65535) return hipErrorInvalidValue;
    const float sl2 = 1.4426950408889634f / sqrtf((float)kv.d);
    if (bm.max_q_len <= 64 || !bm.pf_items || bm.pf_blocks <= 0) {       // short prompts (or no work lists): per-wave operand loads, no ring to fill
        dim3 grid((bm.max_q_len + 127) / 128, n_q, bm.n_seqs);
        attn_prefill_mfma_kernel<128, 1><<<grid, 256, 0, s>>>((const bf16_t*)qkv, (bf16_t*)out, n_q, n_kv, bm,
                                                               (const bf16_t*)kv.k_pool, (const bf16_t*)kv.v_pool, sl2);
        return hipGetLastError();
    }
    constexpr int LDS = 3 * 32768;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)attn_prefill_lds_kernel<128>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    attn_prefill_lds_kernel<128><<<(unsigned)bm.pf_blocks, 512, LDS, s>>>((const bf16_t*)qkv, (bf16_t*)out, n_q, n_kv, bm,
                                                        (const bf16_t*)kv.k_pool, (const bf16_t*)kv.v_pool, sl2);
    return hipGetLastError();
}

// ======================================================================
// Decode.  One wave per (work item, kv head).  A work item is a run of pages of
// one sequence.  All G = n_q / n_kv (<= 16) query heads that share the kv head
// form the 16 query columns of v_mfma_f32_16x16x32_bf16 (unused columns are
// zero), so K and V are read from HBM once per group:
//   accumulator register v of lane l <-> token 4*(l/16) + v, query l%16.
// Each step covers two pages; k-slot e of lane group g4 is token 4*g4 + e of
// page A for e < 4 and token 4*g4 + e - 4 of page B for e >= 4.
// Partial (max, sum, O) of every item go to scratch and are merged per sequence.
// scratch layout: float [n_items][n_q][D + 4]  (O[D], running max, running sum)
// ======================================================================
template <int D>
__global__ __launch_bounds__(64) void attn_decode_mfma_kernel(const bf16_t* __restrict__ qkv, int n_q, int n_kv,
                                                              BatchMeta bm, DecodeWork wk,
                                                              const bf16_t* __restrict__ k_pool,
                                                              const bf16_t* __restrict__ v_pool,
                                                              float* __restrict__ scratch, float scale_log2e) {
    constexpr int KS = D / 32;
    constexpr int DT = D / 16;
    const int item = wk.item_order[blockIdx.x / n_kv], g = blockIdx.x % n_kv;     // the heads of an item side by side
    const int G = n_q / n_kv;
    const int sq = wk.item_seq[item];
    // an item is pages page0, page0 + stride, ... (npg of them) of its sequence: the items of a sequence interleave
    const int page0 = wk.item_page0[item], npg = wk.item_npages[item] & 0xffff;
    const int stride = (wk.item_npages[item] >> 16) > 0 ? (wk.item_npages[item] >> 16) : 1;
    const int kv_len = bm.kv_before[sq] + 1;
    const int lane = threadIdx.x;
    const int lq = lane & 15, g4 = lane >> 4;
    const size_t row_stride = (size_t)(n_q + 2 * n_kv) * D;

    Frag qf[KS];
    if (lq < G) {
        const bf16_t* qp = qkv + (size_t)bm.cu_q[sq] * row_stride + (size_t)(g * G + lq) * D + g4 * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks].q = *reinterpret_cast<const vec16*>(qp + ks * 32);
    } else {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks].w[0] = qf[ks].w[1] = qf[ks].w[2] = qf[ks].w[3] = 0u;
    }
    f32x4_t o[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t) o[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f;

    const int32_t* pt = bm.page_tables + (size_t)sq * bm.pt_stride + page0;
    const size_t page_elems = (size_t)n_kv * 16 * D;
    const size_t head_off = (size_t)g * 16 * D;
    // tokens 4*g4 .. 4*g4+3 sit at piece ((g4 & 1) << 1 | g4 >> 1) of a V^T row, in rows with bit 3 of the row
    // index set in the other half of the row (see vpos)
    const int vpiece = (((g4 & 1) << 1) | (g4 >> 1)) ^ (((lq >> 3) & 1) << 1);
    const size_t k_lane = head_off + (size_t)lq * D + g4 * 8, v_lane = head_off + (size_t)lq * 16 + 4 * vpiece;
    // The loop is software-pipelined over page pairs: the K fragments of the next pair (8 KB per wave) are
    // requested right after the score product of this pair has consumed its own, and the V^T fragments of
    // this pair before that product, so that a wave always has 8 to 16 KB on their way instead of the 2 KB
    // the plain order (load two fragments, multiply, load the next two) keeps in flight.  Past the last
    // pair the prefetch repeats the last page (a cache hit), which keeps the loop free of a branch that
    // would make the load counter's bookkeeping conservative.
    auto pair_pages = [&](int pi, int& pgA, int& pgB) {
        const int ia = pi < npg ? pi : npg - 1, ib = pi + 1 < npg ? pi + 1 : npg - 1;
        pgA = pt[ia * stride];
        pgB = pt[ib * stride];
    };
    auto load_k = [&](int pgA, int pgB, Frag* fa, Frag* fb) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            fa[ks].q = *reinterpret_cast<const vec16*>(k_pool + (size_t)pgA * page_elems + k_lane + ks * 32);
            fb[ks].q = *reinterpret_cast<const vec16*>(k_pool + (size_t)pgB * page_elems + k_lane + ks * 32);
        }
    };
    // one pair of pages: fragments ka / kb hold its K, na / nb receive the K of the next pair
    auto step = [&](auto prefetch, int pi, int pA, int pB, const Frag* ka, const Frag* kb, int nA, int nB, Frag* na, Frag* nb) {
        const bool hasB = pi + 1 < npg;
        const bf16_t* vA = v_pool + (size_t)pA * page_elems + v_lane;
        const bf16_t* vB = v_pool + (size_t)pB * page_elems + v_lane;
        Frag vf[DT];
#pragma unroll
        for (int t = 0; t < DT; ++t) {
            vf[t].h[0] = *reinterpret_cast<const vec8*>(vA + t * 16 * 16);
            vf[t].h[1] = *reinterpret_cast<const vec8*>(vB + t * 16 * 16);
        }
        __builtin_amdgcn_sched_barrier(0);
        f32x4_t sA = {0.f, 0.f, 0.f, 0.f}, sB = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            sA = SS_MFMA_16x16x32(ka[ks].v, qf[ks].v, sA, 0, 0, 0);
            sB = SS_MFMA_16x16x32(kb[ks].v, qf[ks].v, sB, 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (decltype(prefetch)::value) load_k(nA, nB, na, nb);
        __builtin_amdgcn_sched_barrier(0);
        const int posA = (page0 + pi * stride) * 16 + 4 * g4, posB = posA + 16 * stride;
        float mx = m;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            sA[v] = (posA + v < kv_len) ? sA[v] * scale_log2e : -INFINITY;
            sB[v] = (hasB && posB + v < kv_len) ? sB[v] * scale_log2e : -INFINITY;
            mx = fmaxf(mx, fmaxf(sA[v], sB[v]));
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        // the first page of an item always holds a visible token: mx is finite
        const float alpha = fast_exp2(m - mx);
        m = mx;
        float rs = 0.f;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            sA[v] = fast_exp2(sA[v] - mx);
            sB[v] = fast_exp2(sB[v] - mx);
            rs += sA[v] + sB[v];
        }
        l = l * alpha + rs;
        Frag pf;
        pf.w[0] = pack_bf16x2(sA[0], sA[1]);
        pf.w[1] = pack_bf16x2(sA[2], sA[3]);
        pf.w[2] = pack_bf16x2(sB[0], sB[1]);
        pf.w[3] = pack_bf16x2(sB[2], sB[3]);
#pragma unroll
        for (int t = 0; t < DT; ++t) {
#pragma unroll
            for (int v = 0; v < 4; ++v) o[t][v] *= alpha;
            o[t] = SS_MFMA_16x16x32(vf[t].v, pf.v, o[t], 0, 0, 0);
        }
    };
    // two steps per trip, the two fragment sets changing roles, so that no set is ever copied; a last
    // single pair runs without a prefetch
    int pA, pB;
    pair_pages(0, pA, pB);
    Frag k0a[KS], k0b[KS], k1a[KS], k1b[KS];
    load_k(pA, pB, k0a, k0b);
    int pi = 0;
    for (; pi + 2 < npg; pi += 4) {
        int nA, nB;
        pair_pages(pi + 2, nA, nB);
        step(std::true_type{}, pi, pA, pB, k0a, k0b, nA, nB, k1a, k1b);
        pair_pages(pi + 4, pA, pB);
        step(std::true_type{}, pi + 2, nA, nB, k1a, k1b, pA, pB, k0a, k0b);
    }
    if (pi < npg) step(std::false_type{}, pi, pA, pB, k0a, k0b, pA, pB, k1a, k1b);
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    if (lq < G) {
        float* sp = scratch + ((size_t)item * n_q + (size_t)(g * G + lq)) * (D + 4);
#pragma unroll
        for (int t = 0; t < DT; ++t)
            *reinterpret_cast<f32x4_t*>(sp + t * 16 + 4 * g4) = o[t];
        if (g4 == 0) { sp[D] = m; sp[D + 1] = l; }
    }
}

// Merge of the per-item partials: D threads per (q head, sequence), HB heads per block.
template <int D, int HB>
__global__ __launch_bounds__(D * HB) void attn_decode_merge_kernel(const float* __restrict__ scratch,
                                                                   bf16_t* __restrict__ out, int n_q, BatchMeta bm,
                                                                   DecodeWork wk) {
    const int a = blockIdx.x * HB + threadIdx.x / D, sq = blockIdx.y, e = threadIdx.x % D;
    if (a >= n_q) return;
    const int i0 = wk.seq_item0[sq], i1 = wk.seq_item0[sq + 1];
    float M = -INFINITY;
    for (int i = i0; i < i1; ++i) M = fmaxf(M, scratch[((size_t)i * n_q + a) * (D + 4) + D]);
    float num = 0.f, den = 0.f;
    for (int i = i0; i < i1; ++i) {
        const float* sp = scratch + ((size_t)i * n_q + a) * (D + 4);
        const float w = fast_exp2(sp[D] - M);
        num += w * sp[e];
        den += w * sp[D + 1];
    }
    out[(size_t)bm.cu_q[sq] * ((size_t)n_q * D) + (size_t)a * D + e] = f2bf(num / den);
}

size_t attn_decode_scratch_floats(int n_items, int n_q, int d) { return (size_t)n_items * n_q * (d + 4); }

hipError_t attn_decode(int dt, const void* qkv, void* out, int n_q, int n_kv, const BatchMeta& bm,
                       const KvLayer& kv, const DecodeWork& wk, float* scratch, bool force_generic,
                       hipStream_t s) {
    if (bm.n_seqs <= 0) return hipSuccess;
    if (n_kv <= 0 || n_q % n_kv != 0) return hipErrorInvalidValue;
    const int G = n_q / n_kv;
    if (dt != BF16 || force_generic || kv.d != 128 || G > 16) return attn_generic(dt, qkv, out, n_q, n_kv, bm, kv, s);
    if (kv.page_size != 16 || kv.n_heads != n_kv || !scratch || wk.n_items <= 0) return hipErrorInvalidValue;
    if (n_kv > 65535 || bm.n_seqs > 65535) return hipErrorInvalidValue;
    const float sl2 = 1.4426950408889634f / sqrtf((float)kv.d);
    if ((long long)wk.n_items * n_kv > 0x7fffffffll) return hipErrorInvalidValue;
    dim3 grid((unsigned)(wk.n_items * n_kv));
    attn_decode_mfma_kernel<128><<<grid, 64, 0, s>>>((const bf16_t*)qkv, n_q, n_kv, bm, wk,
                                                     (const bf16_t*)kv.k_pool, (const bf16_t*)kv.v_pool, scratch, sl2);
    dim3 mgrid((n_q + 7) / 8, bm.n_seqs);
    attn_decode_merge_kernel<128, 8><<<mgrid, 1024, 0, s>>>(scratch, (bf16_t*)out, n_q, bm, wk);
    return hipGetLastError();
}

}  // namespace SS_NS
