// bf16 MFMA GEMM for gfx950: C[M,N] = A[M,K] * Wt[N,K]^T, fp32 accumulate.
//
// Both operands are K-contiguous, so every MFMA operand fragment (8 consecutive
// k of one row) is a single 16-byte LDS read.  A block owns a BM x BN output
// tile and walks K in slices of 64: the next slice is fetched from global
// memory into registers while the current one is multiplied out of LDS, then
// stored to the other LDS buffer (one barrier per slice).  LDS rows are 128
// bytes; the 16-byte chunk index is XOR-swizzled with the row so that the 32
// rows read by one fragment load spread over all banks.
//
// v_mfma_f32_32x32x16_bf16 operand layout (64-lane wave): lane l supplies row
// (l % 32) of A / column (l % 32) of B with the 8 k-values of group (l / 32);
// accumulator register v of lane l is C[8*(v/4) + 4*(l/32) + v%4][l % 32].
//
// The 1-D grid is remapped so that each of the 8 XCDs (blocks are dealt to them
// round-robin) works on a contiguous run of tiles, and runs are ordered in
// groups of 8 tile rows, so that the A and Wt slices an XCD touches at one time
// stay in its own L2.
#include <cstdlib>

#include "ss_device.h"
#include "ss_kernels.h"

namespace SS_NS {
using namespace ssk;

typedef half8_t bf16x8_t;       // MFMA operand: 8 elements of the 16-bit type
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
constexpr int EPI_PARTIAL = 100;   // internal: fp32 split-K partials

// silu(g) * u with the exponential and the reciprocal on the hardware units (about 1 ulp each; the
// result is rounded to bf16).  A plain `/` expands to the IEEE division sequence, a dozen VALU
// operations per element in the epilogue.
__device__ __forceinline__ float swiglu_act(float g, float u) {
    const float e = __builtin_amdgcn_exp2f(g * -1.4426950408889634f);
    return g * __builtin_amdgcn_rcpf(1.0f + e) * u;
}

__device__ __forceinline__ int lds_chunk_off(int row, int kc) {
    // byte offset of 16-byte chunk kc (0..7) of a 128-byte row
    const int sw = (row & 7) ^ ((row >> 3) & 1);
    return row * 128 + ((kc ^ sw) << 4);
}

template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(64 * WM * WN) void gemm_mfma_kernel(const bf16_t* __restrict__ A, int lda,
                                                                 const bf16_t* __restrict__ Wt,
                                                                 bf16_t* __restrict__ C, int ldc,
                                                                 const bf16_t* __restrict__ R, int M, int N, int K,
                                                                 int tiles_m, int tiles_n, int per_xcd, int ksplit,
                                                                 const float* __restrict__ RS) {
    constexpr int NT = 64 * WM * WN;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int A_CH = BM * 8 / NT, B_CH = BN * 8 / NT;   // 16-byte chunks per thread per slice
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "loader mapping");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    uint8_t* As = smem;                       // [2][BM * 128]
    uint8_t* Bs = smem + 2 * BM * 128;        // [2][BN * 128]

    // ---- block -> tile
    const int xcd = blockIdx.x & 7;
    const int logical = xcd * per_xcd + (blockIdx.x >> 3);
    if ((blockIdx.x >> 3) >= per_xcd || logical >= tiles_m * tiles_n) return;
    constexpr int GM = 8;
    const int group_size = GM * tiles_n;
    const int group = logical / group_size;
    const int first_m = group * GM;
    const int gm = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
    const int in_group = logical - group * group_size;
    const int tile_m = first_m + in_group % gm;
    const int tile_n = in_group / gm;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // ---- global -> register staging (rows beyond the matrix are clamped; their
    // products are never stored)
    const bf16_t* a_src[A_CH];
    const bf16_t* b_src[B_CH];
    int a_dst[A_CH], b_dst[B_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        const int c = tid + i * NT, row = c >> 3, kc = c & 7;
        int gr = m0 + row;
        gr = gr < M ? gr : M - 1;
        a_src[i] = A + (size_t)gr * lda + kc * 8;
        a_dst[i] = lds_chunk_off(row, kc);
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
        const int c = tid + i * NT, row = c >> 3, kc = c & 7;
        int gr = n0 + row;
        gr = gr < N ? gr : N - 1;
        b_src[i] = Wt + (size_t)gr * K + kc * 8;
        b_dst[i] = lds_chunk_off(row, kc);
    }
    // two register sets: the loads of two slices are in flight while a third is multiplied.  At decode sizes the
    // kernel does little but stream weights; twice the bytes in flight per block gained 3-4 % on the shapes of
    // tensor-parallel shards and nothing on the 7B shape (the chain of steps of one iteration bounds it)
    u32x4_t a_reg[2][A_CH], b_reg[2][B_CH];

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // split-K: blockIdx.y owns K slices [kt0, kt0 + nk)
    const int nk = K / 64 / ksplit;
    const int kt0 = blockIdx.y * nk;
    const int lrow = lane & 31, lgrp = lane >> 5;

    auto fetch = [&](int kt, u32x4_t* ar, u32x4_t* br) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) ar[i] = *reinterpret_cast<const u32x4_t*>(a_src[i] + (size_t)(kt0 + kt) * 64);
#pragma unroll
        for (int i = 0; i < B_CH; ++i) br[i] = *reinterpret_cast<const u32x4_t*>(b_src[i] + (size_t)(kt0 + kt) * 64);
    };
    auto stash = [&](int buf, const u32x4_t* ar, const u32x4_t* br) {
        uint8_t* An = As + buf * BM * 128;
        uint8_t* Bn = Bs + buf * BN * 128;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) *reinterpret_cast<u32x4_t*>(An + a_dst[i]) = ar[i];
#pragma unroll
        for (int i = 0; i < B_CH; ++i) *reinterpret_cast<u32x4_t*>(Bn + b_dst[i]) = br[i];
    };
    // Fragments of k-step ks+1 are read from LDS while the MFMAs of k-step ks run
    // (two register sets); scheduling barriers keep the compiler from sinking the
    // reads (or the global prefetch) down to their first use.
    auto load_frags = [&](const uint8_t* Ab, const uint8_t* Bb, int ks, bf16x8_t* af, bf16x8_t* bfr) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
            af[i] = *reinterpret_cast<const bf16x8_t*>(Ab + lds_chunk_off(wm * (BM / WM) + i * 32 + lrow, ks * 2 + lgrp));
#pragma unroll
        for (int j = 0; j < TN; ++j)
            bfr[j] = *reinterpret_cast<const bf16x8_t*>(Bb + lds_chunk_off(wn * (BN / WN) + j * 32 + lrow, ks * 2 + lgrp));
    };
    auto multiply = [&](int buf) {
        const uint8_t* Ab = As + buf * BM * 128;
        const uint8_t* Bb = Bs + buf * BN * 128;
        bf16x8_t af[2][TM], bfr[2][TN];
        load_frags(Ab, Bb, 0, af[0], bfr[0]);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks < 3) load_frags(Ab, Bb, ks + 1, af[(ks + 1) & 1], bfr[(ks + 1) & 1]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = SS_MFMA_32x32x16(af[ks & 1][i], bfr[ks & 1][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // slice kt is multiplied out of LDS stage kt & 1 while slice kt + 1 (register set (kt + 1) & 1) and slice
    // kt + 2 (set kt & 1, free since slice kt was stashed) are on their way; the loop is unrolled by two so that
    // the sets are named at compile time
    fetch(0, a_reg[0], b_reg[0]);
    if (nk > 1) fetch(1, a_reg[1], b_reg[1]);
    stash(0, a_reg[0], b_reg[0]);
    __syncthreads();
    auto step = [&](int kt, u32x4_t* a_same, u32x4_t* b_same, u32x4_t* a_next, u32x4_t* b_next) {
        if (kt + 2 < nk) fetch(kt + 2, a_same, b_same);
        __builtin_amdgcn_sched_barrier(0);
        multiply(kt & 1);
        stash((kt + 1) & 1, a_next, b_next);
        __syncthreads();
    };
    int kt = 0;
    for (; kt + 2 < nk; kt += 2) {
        step(kt, a_reg[0], b_reg[0], a_reg[1], b_reg[1]);
        step(kt + 1, a_reg[1], b_reg[1], a_reg[0], b_reg[0]);
    }
    if (kt + 1 < nk) step(kt, a_reg[0], b_reg[0], a_reg[1], b_reg[1]);
    multiply((nk - 1) & 1);

    // ---- epilogue
    const int col_in = lane & 31;
    if (EPI == EPI_PARTIAL) {      // fp32 partial sums of this K range: [split][M][N]
        float* P = reinterpret_cast<float*>(C) + (size_t)blockIdx.y * M * N;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int rbase = m0 + wm * (BM / WM) + i * 32 + 4 * lgrp;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int c = n0 + wn * (BN / WN) + j * 32 + col_in;
                if (c >= N) continue;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = rbase + 8 * (v >> 2) + (v & 3);
                    if (r < M) P[(size_t)r * N + c] = acc[i][j][v];
                }
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int rbase = m0 + wm * (BM / WM) + i * 32 + 4 * lgrp;
        if (EPI == EPI_SWIGLU) {
#pragma unroll
            for (int j = 0; j < TN; j += 2) {
                const int nb = n0 + wn * (BN / WN) + j * 32;        // multiple of 64: gate block, then up block
                const int oc = (nb >> 1) + col_in;
                if (nb + col_in >= N) continue;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = rbase + 8 * (v >> 2) + (v & 3);
                    if (r >= M) continue;
                    const float rs = RS ? RS[r] : 1.0f;
                    const float g = acc[i][j][v] * rs, u = acc[i][j + 1][v] * rs;
                    C[(size_t)r * ldc + oc] = f2bf(swiglu_act(g, u));
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int c = n0 + wn * (BN / WN) + j * 32 + col_in;
                if (c >= N) continue;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = rbase + 8 * (v >> 2) + (v & 3);
                    if (r >= M) continue;
                    float o = acc[i][j][v];
                    if (RS) o *= RS[r];
                    if (EPI == EPI_RESIDUAL) o += bf2f(R[(size_t)r * ldc + c]);
                    C[(size_t)r * ldc + c] = f2bf(o);
                }
            }
        }
    }
}


// ----------------------------------------------------------------------------
// Large-output kernel: persistent, direct global->LDS loads, two-stage ring.
//
// One block (4 waves, 2 x 2, wave tile 128 x 128 = 8 x 8 tiles of v_mfma_f32_16x16x32_bf16,
// 256 fp32 accumulators per lane) per CU walks that CU's share of the 256 x 256 output
// tiles.  Under the chip's power limit the 16x16x32 shape sustains 10-20 % more than
// 32x32x16 on random data (half the accumulator traffic per flop).  Its operand layout:
// lane l supplies row (l % 16) of the row operand / column (l % 16) of the column operand
// with the 8 k-values of group (l / 16); accumulator register v of lane l is
// D[4*(l/16) + v][l % 16].
//
// K is cut in slices of 64: a row of a slice is one 128-byte line, so every request to L2
// moves a whole line (slices of 32 ask for every line twice, and the number of requests,
// not their bytes, is what the L2 channels run out of).  `global_load_lds_dwordx4` moves
// 16 bytes per lane straight into LDS (lane j of a wave lands at M0 + 16*j): no registers
// are spent on staging.  The ring has two stages of 64 KB and runs on across tile
// boundaries, so the first slices of the next tile are already in flight while the current
// tile is finished and written out.
//
// Per slice (2 k-steps of 32, 64 MFMAs per wave each):
//   k-step 0  multiply out of the current stage; the 16 fragments of k-step 1 are read one
//             at a time behind every other one of the first 32 MFMAs (a burst of reads
//             fills the LDS command queue and holds up the MFMAs issued behind it)
//   k-step 1  wait until the own loads of the next slice have landed, barrier (the next
//             stage is complete, the current one is free), then request the slice after
//             the next into the freed stage: 16 loads per wave, one behind every 4th MFMA
//             (the L1 -> LDS path moves 64 bytes per clock, a 64 KB slice keeps it busy for
//             half of the slice's MFMA time; requests queued faster than that stall the
//             issuing wave), and read the fragments of the next slice's k-step 0
// Completion is tracked with vmcnt by hand (the loads are issued from inline asm), and a
// bare s_barrier publishes a stage; only loads of this one kind are in flight in the main
// loop, so they complete in issue order.  The MFMAs are inline asm too, with the
// accumulators constrained to the accumulation registers: left to itself the register
// allocator moves accumulators between the two register files inside the loop in some
// instantiations.
//
// LDS rows are 128 bytes (8 chunks of 16 bytes); chunk position = kc ^ ((row>>1)&7), which
// spreads the 16 rows that one pass of a fragment read touches over all banks.  A
// wave-level load covers 8 consecutive rows: lane j supplies row j/8, position j%8, and
// therefore fetches global chunk (j%8) ^ ((row>>1)&7).
//
// The product is formed transposed (weight fragment as the row operand): a lane ends up
// with 4 consecutive output columns of one token, which go through an 8 KB per wave fp32
// staging tile (outside the ring) to come out as 16-byte, full-line stores.  Outputs are
// written with the nontemporal hint: they are not read again by this kernel and would
// otherwise push the operand slices out of L2.
// ----------------------------------------------------------------------------
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
template <int V> struct VmcntImm { static constexpr int value = (V & 15) | ((V >> 4) << 14) | 0x0F70; };

template <int EPI>
__global__ __launch_bounds__(256) void gemm_mfma_stream_kernel(const bf16_t* __restrict__ A, int lda,
                                                               const bf16_t* __restrict__ Wt, bf16_t* __restrict__ C,
                                                               int ldc, const bf16_t* __restrict__ R, int M, int N,
                                                               int K, int tiles_m, int tiles_n, int sync_walk,
                                                               int cus_per_xcd, int it0, int max_it, int GM,
                                                               int pf_dist, const float* __restrict__ RS, int ksplit) {
    constexpr int BM = 256, BN = 256;
    constexpr int STAGE = (BM + BN) * 128;       // bytes per ring stage
    constexpr int LPS = 16;                      // loads per wave per slice
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // ---- this block's tiles.  Tiles are ordered in groups of GM tile rows (inside a group: column by column), so
    // that the 32 blocks of an XCD (blocks are dealt to the XCDs round-robin) work on GM rows x 32/GM columns at a
    // time and the slices they touch stay in that XCD's L2.  XCD x owns `gpx` whole groups, [x gpx, (x+1) gpx):
    // all eight XCDs then sweep the columns in step, each over its own rows, so a weight slice is asked for by
    // the eight L2s at about the same time and comes from HBM once (the other seven find it in the memory-side
    // cache), and the 8 GM rows of tokens in use stay in that cache over the whole sweep.  The rows that are
    // left over (fewer than 8 whole groups) are dealt to the XCDs as eight contiguous runs.  A block takes every
    // cus_per_xcd-th tile of its XCD's list; this launch covers rounds [it0, it0 + max_it) of that walk.
    const int xcd = blockIdx.x & 7, cu = blockIdx.x >> 3;
    const int group_size = GM * tiles_n;
    const int gpx = sync_walk ? (tiles_m / GM) / 8 : 0;
    const int main_tiles = gpx * group_size;
    const int rem_row0 = 8 * gpx * GM;
    const int rem_tiles = (tiles_m - rem_row0) * tiles_n;
    const int rem_per_xcd = (rem_tiles + 7) / 8;
    int my_rem = rem_tiles - xcd * rem_per_xcd;
    my_rem = my_rem < rem_per_xcd ? my_rem : rem_per_xcd;
    my_rem = my_rem > 0 ? my_rem : 0;
    const int my_tiles = main_tiles + my_rem;
    // Split K (outputs of too few tiles to occupy the chip): the list of the XCD is walked ksplit times, once per
    // K range; entry l is K range l / my_tiles of tile l % my_tiles, and the product of a range goes to plane
    // `range` of the fp32 partial sums [ksplit][M][N] (EPI_PARTIAL, C is that buffer), which a second kernel sums.
    const int my_entries = my_tiles * ksplit;
    const int first = cu + it0 * cus_per_xcd;          // index in this XCD's list
    if (first >= my_entries) return;
    int nt_local = (my_entries - first + cus_per_xcd - 1) / cus_per_xcd;
    nt_local = nt_local < max_it ? nt_local : max_it;
    // (r, c) = the tile's row inside its group and its column: the CUs of an XCD that work on one group row
    // at a time differ in c, those on one column in r
    int tile_r = 0, tile_c = 0, tile_gm = 1, tile_range = 0;
    auto tile_origin = [&](int it, int& m0, int& n0) {
        int l = first + it * cus_per_xcd;
        tile_range = 0;
        if (ksplit > 1) {
            tile_range = l / my_tiles;
            l -= tile_range * my_tiles;
        }
        int row0, logical;
        if (l < main_tiles) {
            row0 = xcd * gpx * GM;
            logical = l;
        } else {
            row0 = rem_row0;
            logical = xcd * rem_per_xcd + (l - main_tiles);
        }
        const int group = logical / group_size;
        const int first_m = row0 + group * GM;
        const int gm = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
        const int in_group = logical - group * group_size;
        tile_r = in_group % gm;
        tile_c = in_group / gm;
        tile_gm = gm;
        m0 = (first_m + tile_r) * BM;
        n0 = tile_c * BN;
    };

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const uint32_t lds_base = (uint32_t)(uintptr_t)smem;

    // ---- loads: waves 0-1 bring A rows [128w, 128w+128), waves 2-3 bring Wt rows [128(w-2), ...);
    // one load = 8 rows.  tbase = first row of the tile whose slices are being requested (a 64-bit scalar
    // address, so operands of any size are addressed), roff[i] = byte offset of this lane's 16 bytes inside
    // slice 0 of that tile (rows beyond the matrix are clamped: their products are never stored), plus the
    // 3 KB - (i % 4) KB that `issue1_load` takes back out
    const bool isA = wave < 2;
    const int row_base = (wave & 1) * 128;
    const uint8_t* gbase = reinterpret_cast<const uint8_t*>(isA ? A : Wt);
    const int ld = isA ? lda : K;
    const int row_lim = isA ? M : N;
    uint32_t roff[LPS];
    const uint8_t* tbase = gbase;
    // L2 prefetch (see `prefetch` below): this wave asks for the lines of a later slice in every pf_period-th
    // slice, starting at slice 1 + pf_phase of a tile
    // (only for tiles whose 256 operand rows all exist: the touch then needs no per-lane arithmetic)
    int pf_period = 1 << 30, pf_phase = 0, pf_next = -1;
    bool pf_full = false;
    auto set_roff = [&](int it) {
        int m0, n0;
        tile_origin(it < nt_local ? it : nt_local - 1, m0, n0);
        const int row0 = isA ? m0 : n0;
        tbase = gbase + (size_t)row0 * (size_t)ld * 2 + (size_t)tile_range * (size_t)(K / 64 / ksplit) * 128;
        pf_full = row0 + 256 <= row_lim;
        if (pf_dist > 0) {
            const int sharers = cus_per_xcd / GM > 0 ? cus_per_xcd / GM : 1;      // CUs of the XCD on one group row
            pf_period = isA ? sharers : tile_gm;
            pf_phase = isA ? tile_c % sharers : tile_r;
        }
#pragma unroll
        for (int i = 0; i < LPS; ++i) {
            const int row = row_base + i * 8 + (lane >> 3);
            const int kc = (lane & 7) ^ ((row >> 1) & 7);
            int gr = row0 + row;
            gr = gr < row_lim ? gr : row_lim - 1;
            roff[i] = (uint32_t)(gr - row0) * (uint32_t)ld * 2u + (uint32_t)kc * 16u + 3072u - (uint32_t)(i & 3) * 1024u;
        }
    };
    const uint32_t dst0 = lds_base + (isA ? 0 : BM * 128) + row_base * 128;
    const int nsl = K / 64 / ksplit;             // slices of one K range
    const int g_last = nt_local * nsl - 1;       // last slice of this block's stream
    auto issue1 = [&](int stage, int ksl, int i) {
        const uint8_t* sb = tbase + (size_t)ksl * 128 - 3072 + (i & 3) * 1024;
        const uint32_t d = dst0 + (uint32_t)stage * STAGE + i * 1024;
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(roff[i]), "s"(sb), "s"(d) : "memory");
    };
    // Inside the K loop the load comes in two parts with a matrix instruction between them, and one write of M0 (the
    // LDS address) serves four loads.  The scalar instructions of a wave that runs alone on its SIMD are paid for
    // in matrix-pipe time (a write of M0 directly in front of the load that reads it holds the wave for some ten
    // cycles; counters: 6.7 % of the wave's cycles went to scalar instructions with three of them per load, 4 % now).
    // The immediate offset of the load, (i % 4) KB, moves the LDS address and the global address alike: roff[i]
    // carries 3 KB minus that and the scalar base is lowered by the 3 KB, so the global address is unchanged.
    // All-zero operands (full clock): the K = 28672 projection 0.62 -> 0.72 of the matrix peak, K = 8192 unchanged;
    // on random data (clock set by the power limit) +0.5 %.
    auto issue1_m0 = [&](int stage, int i) {
        const uint32_t d = dst0 + (uint32_t)stage * STAGE + i * 1024;
        asm volatile("s_mov_b32 m0, %0" ::"s"(d) : "memory");
    };
    auto issue1_load = [&](int ksl, int i) {
        const uint8_t* sb = tbase + (size_t)ksl * 128 - 3072;
        switch (i & 3) {
            case 0: asm volatile("global_load_lds_dwordx4 %0, %1" ::"v"(roff[i]), "s"(sb) : "memory"); break;
            case 1: asm volatile("global_load_lds_dwordx4 %0, %1 offset:1024" ::"v"(roff[i]), "s"(sb) : "memory"); break;
            case 2: asm volatile("global_load_lds_dwordx4 %0, %1 offset:2048" ::"v"(roff[i]), "s"(sb) : "memory"); break;
            default: asm volatile("global_load_lds_dwordx4 %0, %1 offset:3072" ::"v"(roff[i]), "s"(sb) : "memory"); break;
        }
    };

    // L2 prefetch.  Of the 32 CUs of an XCD, cus_per_xcd / GM read the same token rows and GM the same weight rows
    // at about the same time; whichever asks first waits for the line to come from beyond L2, the others wait with
    // it, and with a two-stage ring a request has at most one slice time to land: too little for a miss.  So the
    // CUs take turns (by their column for token rows, by their row in the group for weight rows): in its slice a
    // wave touches one dword of each of the 128 lines of its loading share of slice `ksl`, pf_dist slices ahead of
    // the slice being multiplied, which brings the lines into L2 for all sharers.  The dwords land in the wave's
    // epilogue staging tile (unused inside the K loop) and are never read.  Loads of a wave return in order, so
    // the requests of the next slice queue behind these two; the mid-slice wait of the slice that issued them
    // leaves them outstanding (vmcnt 2), every other wait takes them in.
    // The touch is two instructions with a scalar base and one per-lane offset (row `lane` of a run of 64 rows)
    // that is formed on the spot from the lane number, inside the assembly: a value kept in a register over the
    // whole kernel for this rare use is what the register allocator spills first, the reload is a vector memory
    // operation, and the wait the compiler puts in front of the first use counts the loads of this loop, which it
    // does not know of, as well (seen: a vmcnt(0) in front of every touch, 2.7 % of the GEMM time).
    const uint32_t pf_dst = lds_base + 2 * STAGE + wave * 8192;
    const uint32_t ld_bytes = (uint32_t)ld * 2u;
    auto prefetch = [&](int ksl) {
        uint32_t off;
        asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0\n\tv_mul_lo_u32 %0, %0, %1" : "=v"(off) : "s"(ld_bytes));
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint8_t* sb = tbase + (size_t)ksl * 128 + (size_t)(row_base + h * 64) * (size_t)ld * 2;
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(off), "s"(sb), "s"(pf_dst) : "memory");
        }
    };

    // The residual rows of the tile being finished, brought into L2 the same way three slices before the epilogue
    // reads them: this wave's 128 x 128 piece is 128 rows of 256 bytes = 256 lines, one per lane and request.
    // (tiles that lie wholly inside the output; scalar base + a per-lane offset formed on the spot as above: lane l
    // is row l / 2, half l % 2 of a run of 32 rows)
    auto prefetch_residual = [&](int it) -> bool {
        if (EPI != EPI_RESIDUAL) return false;
        int m0, n0;
        tile_origin(it, m0, n0);
        if (m0 + 256 > M || n0 + 256 > N) return false;
        const uint32_t ldc_bytes = (uint32_t)ldc * 2u;
        uint32_t lane_res_off, half;
        asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0\n\tv_and_b32 %1, 1, %0\n\tv_lshrrev_b32 %0, 1, %0\n\t"
                     "v_mul_lo_u32 %0, %0, %2\n\tv_lshl_add_u32 %0, %1, 7, %0" : "=&v"(lane_res_off), "=&v"(half) : "s"(ldc_bytes));
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            const uint8_t* sb = reinterpret_cast<const uint8_t*>(R) + (size_t)(m0 + wm * 128 + h * 32) * (size_t)ldc * 2 +
                                (size_t)(n0 + wn * 128) * 2;
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(lane_res_off), "s"(sb), "s"(pf_dst) : "memory");
        }
        return true;
    };

    f32x4_t acc[8][8];       // [n tile][m tile] of 16 x 16
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;

    // fragment of a 16-row tile: lane supplies row l % 16, 16-byte chunk 4 ks + l / 16 of the 128-byte row
    const int l16 = lane & 15, lk = lane >> 4;
    int koff[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) koff[ks] = l16 * 128 + ((((ks * 4 + lk) ^ ((l16 >> 1) & 7))) << 4);
    const int a_base = wm * 128 * 128, b_base = BM * 128 + wn * 128 * 128;
    bf16x8_t af[2][8], bfr[2][8];
    // t-th of the 16 fragment reads of a k-step: token fragments first (the first MFMAs need them all)
    auto read_one = [&](const uint8_t* st, int ks, int par, int t) {
        if (t < 8) af[par][t] = *reinterpret_cast<const bf16x8_t*>(st + a_base + t * 2048 + koff[ks]);
        else bfr[par][t - 8] = *reinterpret_cast<const bf16x8_t*>(st + b_base + (t - 8) * 2048 + koff[ks]);
    };
    // 64 MFMAs on set `par`; behind every other one of the first 32 a fragment read of (rst, rks) into the other
    // set; when `loads`, one load behind every 4th MFMA
    auto mfma_step = [&](int par, const uint8_t* rst, int rks, bool loads, int stage, int ksl) {
#pragma unroll
        for (int t = 0; t < 64; ++t) {
            const int nt = t >> 3, mt = t & 7;
            // accumulators pinned to the accumulation registers, fragments to the ordinary ones
            asm volatile(SS_MFMA_16x16x32_ASM " %0, %1, %2, %0" : "+a"(acc[nt][mt]) : "v"(bfr[par][nt]), "v"(af[par][mt]));
            if (t < 32 && (t & 1)) {
                __builtin_amdgcn_sched_barrier(0);
                read_one(rst, rks, par ^ 1, t >> 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (loads && (t & 15) == 1) {
                __builtin_amdgcn_sched_barrier(0);
                issue1_m0(stage, t >> 2);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (loads && (t & 3) == 2) {
                __builtin_amdgcn_sched_barrier(0);
                issue1_load(ksl, t >> 2);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    float* stg = reinterpret_cast<float*>(smem + 2 * STAGE + wave * 8192);
    // Epilogue of one tile.  A pass covers 32 tokens x 64 output columns: the lanes' 4-column pieces go
    // into the fp32 staging tile [32][64] (row stride 256 B, 16-byte chunk index XORed with the row) and
    // come back as 8 consecutive columns per lane.  Passes are software-pipelined: the staging writes of
    // pass p+1 (and its residual loads) are issued behind the read-back of pass p -- LDS executes a wave's
    // operations in order, so the read-back still sees pass p -- and run while pass p is packed and stored.
    auto epilogue = [&](int it) {
        int m0, n0;
        tile_origin(it, m0, n0);
        if (EPI == EPI_PARTIAL) {                // fp32 sums of this K range, straight from the accumulators
            float* P = reinterpret_cast<float*>(C) + (size_t)tile_range * (size_t)M * (size_t)N;
#pragma unroll
            for (int mt = 0; mt < 8; ++mt) {
                const int gr = m0 + wm * 128 + mt * 16 + l16;
                if (gr >= M) continue;
#pragma unroll
                for (int nt = 0; nt < 8; ++nt) {
                    const int gc = n0 + wn * 128 + nt * 16 + 4 * lk;
                    if (gc < N) *reinterpret_cast<f32x4_t*>(P + (size_t)gr * N + gc) = acc[nt][mt];
                }
            }
            return;
        }
        constexpr int NH = (EPI == EPI_SWIGLU) ? 1 : 2;
        constexpr int NP = 4 * NH;
        const int n_out = (EPI == EPI_SWIGLU) ? (N >> 1) : N;
        const int row_l = lane >> 3, g8 = lane & 7;
        // RMSNorm factor of the token rows this lane holds products of (row 16 mt + lane % 16 of the wave's 128):
        // norm(x) W = r * (x (g W)), the gains are in the weight rows already
        float rsv[8];
#pragma unroll
        for (int mt = 0; mt < 8; ++mt) {
            int gr = m0 + wm * 128 + mt * 16 + l16;
            gr = gr < M ? gr : M - 1;
            rsv[mt] = (EPI != EPI_RESIDUAL && RS) ? RS[gr] : 1.0f;
        }
        auto write_pass = [&](int p) {
            const int q = p / NH, h = p % NH;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int c4 = 0; c4 < 4; ++c4) {
                    f32x4_t o;
                    if (EPI == EPI_SWIGLU) {             // n tiles (0,1) gate, (2,3) up, (4,5) gate, (6,7) up
                        const int gt = (c4 >> 1) * 4 + (c4 & 1);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float g = acc[gt][2 * q + mt][e] * rsv[2 * q + mt], u = acc[gt + 2][2 * q + mt][e] * rsv[2 * q + mt];
                            o[e] = swiglu_act(g, u);
                        }
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            o[e] = acc[4 * h + c4][2 * q + mt][e];
                            if (EPI != EPI_RESIDUAL) o[e] *= rsv[2 * q + mt];
                        }
                    }
                    const int row = mt * 16 + l16;
                    const int c = c4 * 4 + lk;
                    *reinterpret_cast<f32x4_t*>(stg + row * 64 + ((c ^ (row & 15)) << 2)) = o;
                }
        };
        auto out_ptr = [&](int p, int r8, bool& ok) -> size_t {
            const int q = p / NH, h = p % NH;
            const int oc0 = (EPI == EPI_SWIGLU) ? ((n0 + wn * 128) >> 1) : (n0 + wn * 128 + 64 * h);
            const int gr = m0 + wm * 128 + q * 32 + r8 * 8 + row_l;
            const int gc = oc0 + g8 * 8;
            ok = gr < M && gc < n_out;
            return (size_t)gr * ldc + gc;
        };
        constexpr int RD = 4;                    // residual loads run RD-1 passes ahead
        u32x4_t rres[RD][4];
        auto load_res = [&](int p) {
            if (EPI != EPI_RESIDUAL) return;
#pragma unroll
            for (int r8 = 0; r8 < 4; ++r8) {
                bool ok;
                const size_t off = out_ptr(p, r8, ok);
                rres[p % RD][r8] = *reinterpret_cast<const u32x4_t*>(R + (ok ? off : 0));    // no branch: out-of-range lanes read element 0
            }
        };
#pragma unroll
        for (int p = 0; p < RD - 1 && p < NP; ++p) load_res(p);
        write_pass(0);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            f32x4_t lo[4], hi[4];
#pragma unroll
            for (int r8 = 0; r8 < 4; ++r8) {
                const int row = r8 * 8 + row_l;
                lo[r8] = *reinterpret_cast<const f32x4_t*>(stg + row * 64 + (((2 * g8) ^ (row & 15)) << 2));
                hi[r8] = *reinterpret_cast<const f32x4_t*>(stg + row * 64 + (((2 * g8 + 1) ^ (row & 15)) << 2));
            }
            __builtin_amdgcn_sched_barrier(0);
            if (p + RD - 1 < NP) load_res(p + RD - 1);
            if (p + 1 < NP) write_pass(p + 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int r8 = 0; r8 < 4; ++r8) {
                bool ok;
                const size_t off = out_ptr(p, r8, ok);
                if (ok) {
                    float o[8] = {lo[r8][0], lo[r8][1], lo[r8][2], lo[r8][3], hi[r8][0], hi[r8][1], hi[r8][2], hi[r8][3]};
                    if (EPI == EPI_RESIDUAL) {
                        const u32x4_t rv = rres[p % RD][r8];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            float r0, r1;
                            unpack_bf16x2(rv[e], r0, r1);
                            o[2 * e] += r0;
                            o[2 * e + 1] += r1;
                        }
                    }
                    u32x4_t pv;
#pragma unroll
                    for (int e = 0; e < 4; ++e) pv[e] = pack_bf16x2(o[2 * e], o[2 * e + 1]);
                    // streaming stores are acknowledged late, and the residual loads behind them in the
                    // memory counter would wait for that: plain stores when there is a residual to read
                    if (EPI == EPI_RESIDUAL) *reinterpret_cast<u32x4_t*>(C + off) = pv;
                    else __builtin_nontemporal_store(pv, reinterpret_cast<u32x4_t*>(C + off));
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    set_roff(0);
#pragma unroll
    for (int i = 0; i < LPS; ++i) issue1(0, 0, i);
#pragma unroll
    for (int i = 0; i < LPS; ++i) issue1(1, 1, i);
    __builtin_amdgcn_s_waitcnt(VmcntImm<LPS>::value);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < 16; ++t) read_one(smem, 0, 0, t);

    int g = 0;
    for (int it = 0; it < nt_local; ++it) {
        for (int s = 0; s < nsl; ++s, ++g) {
            const uint8_t* st = smem + (g & 1) * STAGE;
            const uint8_t* stn = smem + ((g + 1) & 1) * STAGE;
            int k2 = s + 2;
            if (k2 >= nsl) k2 -= nsl;
            if (g + 2 > g_last) k2 = nsl - 1;
            // no prefetch in slice 0 (stores of the previous tile's epilogue may still be outstanding, and those
            // do not return in order with the loads) nor where the target lies beyond this tile's K range
            if (s == 0) pf_next = pf_dist > 0 ? 1 + pf_phase : -1;
            bool prefetched = false;
            if (s == pf_next) {
                pf_next += pf_period;
                if (s + pf_dist < nsl - 1 && pf_full) {
                    prefetch(s + pf_dist);
                    prefetched = true;
                }
            }
            bool res_prefetched = false;
            if (EPI == EPI_RESIDUAL && pf_dist > 0 && !prefetched && s == nsl - 3 && s > 0) res_prefetched = prefetch_residual(it);
            __builtin_amdgcn_sched_barrier(0);
            mfma_step(0, st, 1, false, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (s == nsl - 2) set_roff(it + 1);
            __builtin_amdgcn_s_waitcnt(0xC07F);
            if (prefetched) __builtin_amdgcn_s_waitcnt(VmcntImm<2>::value);
            else if (res_prefetched) __builtin_amdgcn_s_waitcnt(VmcntImm<4>::value);
            else __builtin_amdgcn_s_waitcnt(0x0F70);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            mfma_step(1, stn, 0, true, g & 1, k2);
            __builtin_amdgcn_sched_barrier(0);
        }
        // the MFMAs are issued from inline asm, so the compiler does not place the wait states an
        // accumulator read behind a matrix instruction needs: the last products are written before they are read
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
        epilogue(it);
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
        asm volatile("s_nop 7" ::: "memory");        // ... and the zeros are in place before the next product reads them
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
}


constexpr size_t STREAM_LDS = (size_t)2 * 512 * 128 + 4 * 8192;     // ring + staging = 160 KB

bool gemm_mfma_stream_supported(const void* C, const void* R, int ldc, int M, int N, int K, int lda, int epi) {
    if (K % 64 != 0 || K < 128 || N % 16 != 0 || ldc % 8 != 0) return false;
    if (((uintptr_t)C & 15) != 0 || (epi == EPI_RESIDUAL && ((uintptr_t)R & 15) != 0)) return false;
    // 32-bit byte offsets inside one 256-row tile of an operand
    if ((long long)256 * lda * 2 >= (1ll << 32) || (long long)256 * K * 2 >= (1ll << 32)) return false;
    (void)M;
    return true;
}

// Blocks of the persistent kernel own their CU (all registers, all LDS) until they are done, so a kernel
// of another stream can only start at a launch boundary.  `max_rounds` > 0 cuts the walk into launches
// of at most that many tiles per block, for callers that have latency-bound work on other streams.
// With ksplit > 1 the kernel writes fp32 partial sums [ksplit][M][N] into `partial` (EPI_PARTIAL) and the caller
// sums them.
static hipError_t launch_stream(const bf16_t* A, int lda, const bf16_t* Wt, bf16_t* C, int ldc, const bf16_t* R, int M,
                                int N, int K, int epi, hipStream_t s, int max_rounds, const float* rs, int ksplit = 1,
                                float* partial = nullptr) {
    if (rs && epi == EPI_RESIDUAL) return hipErrorInvalidValue;      // no caller scales a product that adds a residual
    if (ksplit < 1 || (K / 64) % ksplit != 0 || K / 64 / ksplit < 2 || (ksplit > 1 && !partial)) return hipErrorInvalidValue;
    if (ksplit > 1) {
        epi = EPI_PARTIAL;
        C = reinterpret_cast<bf16_t*>(partial);
        rs = nullptr;
    }
    const int tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
    const long long n_tiles = (long long)tiles_m * tiles_n;
    if (n_tiles > (1ll << 30)) return hipErrorInvalidValue;
    static int n_cus = 0;
    if (!n_cus) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        e = hipDeviceGetAttribute(&n_cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        if (n_cus < 8) n_cus = 8;
    }
    const int cus_per_xcd = n_cus / 8;
    // Tile rows per group of the walk: the 32 CUs of an XCD cover GM x 32/GM tiles at a time, so an XCD re-fetches
    // its token slices (tiles_n * GM / 32) times and the weight slices once per group from beyond its L2; with the
    // eight XCDs sweeping the columns in step those re-fetches are served by the memory-side cache (the 8 GM tile
    // rows in use and the 32/GM tile columns of weights fit it), and HBM sees the weights once per 8 GM tile rows.
    // Measured (fraction of the MFMA peak over the four GEMMs of a layer, GM = 2 / 4 / 8 / 16): 70B-shape slice of
    // 75 k tokens 0.518 / 0.529 / 0.501 / 0.477, 13B shape 0.503 / 0.510 / 0.518 / 0.457, 7B shape of 20 k tokens
    // 0.524 / 0.516 / 0.508 / 0.488; without the XCDs in step (each on a contiguous run of tiles): 0.499 on the
    // 70B shape.  Groups of 4, of 2 for wide outputs of few tile rows.
    static const int gm_env = getenv("SS_GEMM_GROUP_ROWS") ? atoi(getenv("SS_GEMM_GROUP_ROWS")) : 0;
    const int gm_rows = gm_env > 0 ? gm_env : (tiles_n >= 64 && tiles_m < 100 ? 2 : 4);
    // the longest list of an XCD: its whole groups plus its share of the left-over rows (same arithmetic as the kernel)
    static const int sync_walk = getenv("SS_GEMM_SYNC_WALK") ? atoi(getenv("SS_GEMM_SYNC_WALK")) : 1;
    // L2 prefetch distance in slices (0 = off; the kernel needs at least 2).  Measured on the 70B-shape slice
    // (fraction of the MFMA peak over a layer's four GEMMs, one box): off 0.488-0.494, 2: 0.541-0.555, 3: 0.539-0.551,
    // 4: 0.515, 6: 0.509; weight lines only 0.541-0.544, token lines only 0.489.  A larger distance gains nothing:
    // the requests behind a prefetch in the same wave wait for it (loads return in order), and at distance 2
    // those are requests for the very lines it asked for.
    static const int pf_env = getenv("SS_GEMM_PREFETCH") ? atoi(getenv("SS_GEMM_PREFETCH")) : 2;
    const int pf_dist = pf_env >= 2 && pf_env < 64 ? pf_env : 0;
    const int gpx = sync_walk ? (tiles_m / gm_rows) / 8 : 0;
    const long long main_tiles = (long long)gpx * gm_rows * tiles_n;
    const long long rem_tiles = (long long)(tiles_m - 8 * gpx * gm_rows) * tiles_n;
    const int per_xcd = (int)(main_tiles + (rem_tiles + 7) / 8) * ksplit;       // entries of the longest list
    const unsigned grid = 8 * (unsigned)(per_xcd < cus_per_xcd ? per_xcd : cus_per_xcd);
    const int rounds_total = (per_xcd + cus_per_xcd - 1) / cus_per_xcd;
    const int step = max_rounds > 0 ? max_rounds : rounds_total;
#define SS_LAUNCH(E)                                                                                            \
    {                                                                                                           \
        auto kfn = gemm_mfma_stream_kernel<E>;                                                                  \
        static bool attr_set = false;                                                                           \
        if (!attr_set) {                                                                                        \
            hipError_t e = hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize,   \
                                               (int)STREAM_LDS);                                                \
            if (e != hipSuccess) return e;                                                                      \
            attr_set = true;                                                                                    \
        }                                                                                                       \
        for (int it0 = 0; it0 < rounds_total; it0 += step)                                                      \
            kfn<<<grid, 256, STREAM_LDS, s>>>(A, lda, Wt, C, ldc, R, M, N, K, tiles_m, tiles_n, sync_walk,      \
                                              cus_per_xcd, it0, step, gm_rows, pf_dist, rs, ksplit);            \
    }
    switch (epi) {
        case EPI_STORE: SS_LAUNCH(EPI_STORE) break;
        case EPI_RESIDUAL:
            if (!R) return hipErrorInvalidValue;
            SS_LAUNCH(EPI_RESIDUAL) break;
        case EPI_SWIGLU: SS_LAUNCH(EPI_SWIGLU) break;
        case EPI_PARTIAL: SS_LAUNCH(EPI_PARTIAL) break;
        default: return hipErrorInvalidValue;
    }
#undef SS_LAUNCH
    return hipGetLastError();
}

bool gemm_mfma_supported(int M, int N, int K, int lda, int ldc, int epi) {
    if (K % 64 != 0 || lda % 8 != 0) return false;
    if (epi == EPI_STORE_F32 && ldc != N) return false;      // written as plane 0 of the fp32 partials: dense rows
    if (epi == EPI_SWIGLU && (N % 64 != 0)) return false;
    (void)M;
    return true;
}

// Sums the split-K partials [S][M][N] and applies the epilogue.
template <int EPI>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ P, int S, bf16_t* __restrict__ C,
                                                            int ldc, const bf16_t* __restrict__ R, int M, int N,
                                                            const float* __restrict__ RS) {
    const int n_out = (EPI == EPI_SWIGLU) ? N / 2 : N;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)M * n_out) return;
    const int m = (int)(idx / n_out), j = (int)(idx % n_out);
    const size_t plane = (size_t)M * N;
    const float rs = RS ? RS[m] : 1.0f;
    if (EPI == EPI_SWIGLU) {
        const int ng = (j >> 5) * 64 + (j & 31);
        float g = 0.f, u = 0.f;
        for (int s = 0; s < S; ++s) { g += P[s * plane + (size_t)m * N + ng]; u += P[s * plane + (size_t)m * N + ng + 32]; }
        C[(size_t)m * ldc + j] = f2bf(swiglu_act(g * rs, u * rs));
    } else {
        float o = 0.f;
        for (int s = 0; s < S; ++s) o += P[s * plane + (size_t)m * N + j];
        o *= rs;
        if (EPI == EPI_RESIDUAL) o += bf2f(R[(size_t)m * ldc + j]);
        if (EPI == EPI_STORE_F32) reinterpret_cast<float*>(C)[(size_t)m * ldc + j] = o;
        else C[(size_t)m * ldc + j] = f2bf(o);
    }
}

static hipError_t reduce_partials(const float* ws, int ksplit, bf16_t* C, int ldc, const bf16_t* R, int M, int N, int epi,
                                  const float* rs, hipStream_t s) {
    const size_t n_out = (size_t)M * (epi == EPI_SWIGLU ? N / 2 : N);
    const unsigned rgrid = (unsigned)((n_out + 255) / 256);
    switch (epi) {
        case EPI_STORE: splitk_reduce_kernel<EPI_STORE><<<rgrid, 256, 0, s>>>(ws, ksplit, C, ldc, R, M, N, rs); break;
        case EPI_RESIDUAL:
            if (!R) return hipErrorInvalidValue;
            splitk_reduce_kernel<EPI_RESIDUAL><<<rgrid, 256, 0, s>>>(ws, ksplit, C, ldc, R, M, N, rs);
            break;
        case EPI_SWIGLU: splitk_reduce_kernel<EPI_SWIGLU><<<rgrid, 256, 0, s>>>(ws, ksplit, C, ldc, R, M, N, rs); break;
        case EPI_STORE_F32: splitk_reduce_kernel<EPI_STORE_F32><<<rgrid, 256, 0, s>>>(ws, ksplit, C, ldc, R, M, N, rs); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch_cfg(const bf16_t* A, int lda, const bf16_t* Wt, bf16_t* C, int ldc, const bf16_t* R, int M,
                             int N, int K, int epi, hipStream_t s, int ksplit = 1, float* ws = nullptr,
                             const float* rs = nullptr) {
    constexpr int NT = 64 * WM * WN;
    constexpr size_t LDS = (size_t)2 * (BM + BN) * 128;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const long long n_tiles = (long long)tiles_m * tiles_n;
    if (n_tiles > (1ll << 30)) return hipErrorInvalidValue;
    if (ksplit < 1 || (K / 64) % ksplit != 0 || (ksplit > 1 && !ws)) return hipErrorInvalidValue;
    const int per_xcd = (int)((n_tiles + 7) / 8);
    const dim3 grid((unsigned)per_xcd * 8, ksplit);
#define SS_LAUNCH(E, OUT)                                                                                       \
    {                                                                                                           \
        auto kfn = gemm_mfma_kernel<BM, BN, WM, WN, E>;                                                         \
        static bool attr_set = false;                                                                           \
        if (!attr_set) {                                                                                        \
            hipError_t e = hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS); \
            if (e != hipSuccess) return e;                                                                      \
            attr_set = true;                                                                                    \
        }                                                                                                       \
        kfn<<<grid, NT, LDS, s>>>(A, lda, Wt, OUT, ldc, R, M, N, K, tiles_m, tiles_n, per_xcd, ksplit, rs);     \
    }
    if (ksplit > 1) {
        SS_LAUNCH(EPI_PARTIAL, reinterpret_cast<bf16_t*>(ws))
        return reduce_partials(ws, ksplit, C, ldc, R, M, N, epi, rs, s);
    }
    switch (epi) {
        case EPI_STORE_F32:                                       // one K range: plane 0 of the partials is the fp32 result
            if (rs) return hipErrorInvalidValue;
            SS_LAUNCH(EPI_PARTIAL, C) break;
        case EPI_STORE: SS_LAUNCH(EPI_STORE, C) break;
        case EPI_RESIDUAL:
            if (!R) return hipErrorInvalidValue;
            SS_LAUNCH(EPI_RESIDUAL, C) break;
        case EPI_SWIGLU: SS_LAUNCH(EPI_SWIGLU, C) break;
        default: return hipErrorInvalidValue;
    }
#undef SS_LAUNCH
    return hipGetLastError();
}

hipError_t gemm_mfma_bf16(const void* A, int lda, const void* Wt, void* C, int ldc, const void* R, int M, int N,
                          int K, int epi, hipStream_t s, float* ws, size_t ws_bytes, int max_rounds, const float* rs) {
    const bf16_t* a = (const bf16_t*)A;
    const bf16_t* w = (const bf16_t*)Wt;
    bf16_t* c = (bf16_t*)C;
    const bf16_t* r = (const bf16_t*)R;
    // Prefill-sized outputs (at least one 256 x 256 tile per CU): the persistent direct-to-LDS kernel.
    // Smaller outputs (decode batches) are bound by streaming the weights: 128 x 128 tiles with split-K
    // (partials in fp32, summed by a small second kernel).
    const long long big = (long long)((M + 255) / 256) * ((N + 255) / 256);
    static const long long stream_min = getenv("SS_GEMM_STREAM_MIN_TILES") ? atoll(getenv("SS_GEMM_STREAM_MIN_TILES")) : 256;
    if (big >= stream_min && epi != EPI_STORE_F32 && gemm_mfma_stream_supported(C, R, ldc, M, N, K, lda, epi))
        return launch_stream(a, lda, w, c, ldc, r, M, N, K, epi, s, max_rounds, rs);
    // In between (a thousand tokens or so, as in the decode step of a tensor-parallel shard): too few 256 x 256
    // tiles for the chip, but long contractions.  The persistent kernel with K cut into ranges, so that tiles x
    // ranges fill the CUs, with fp32 partial sums and the reduce kernel of the small-tile path; only while the
    // partial sums stay below the weight bytes (as below) and at least half the CUs get a block.  Measured with
    // 1024 tokens on the shapes of the k = 8 shard of the 70B layer: gate/up (7168 x 8192) 150 -> 113 us; the
    // down projection (K = 3584) would lose (73 -> 83 us: its partial sums outweigh its weights) and is excluded
    // by the rule, as are outputs too narrow to fill the chip even when split (QKV of the shard: 20 tiles).  At 256
    // tokens (one tile row) the four GEMMs of the 7B layer together go from 232 to 217 us.
    static const int stream_split = getenv("SS_GEMM_STREAM_SPLIT") ? atoi(getenv("SS_GEMM_STREAM_SPLIT")) : 1;
    static const int stream_split_min_m = getenv("SS_GEMM_STREAM_SPLIT_MIN_M") ? atoi(getenv("SS_GEMM_STREAM_SPLIT_MIN_M")) : 256;
    if (stream_split && M >= stream_split_min_m && big >= 8 && big < 256 && epi != EPI_STORE_F32 && ws &&
        gemm_mfma_stream_supported(C, R, ldc, M, N, K, lda, epi) && ((uintptr_t)ws & 15) == 0) {
        int ks = 1;
        constexpr int min_slices = 16, min_blocks = 128;      // (64 blocks: the 7B-shape decode GEMMs 217 -> 260 us)
        while (ks < 8 && big * (ks * 2) <= 288 && (K / 64) % (ks * 2) == 0 && K / 64 / (ks * 2) >= min_slices &&
               (long long)(ks * 2) * 4 * M <= K && (size_t)(ks * 2) * M * N * sizeof(float) <= ws_bytes)
            ks *= 2;
        if (ks > 1 && big * ks >= min_blocks) {
            hipError_t e = launch_stream(a, lda, w, c, ldc, r, M, N, K, epi, s, max_rounds, rs, ks, ws);
            if (e != hipSuccess) return e;
            return reduce_partials(ws, ks, c, ldc, r, M, N, epi, rs, s);
        }
    }
    const long long mid = (long long)((M + 127) / 128) * ((N + 127) / 128);
    // split K until every CU has a block, but only while the fp32 partials (8*S*M*N bytes written and
    // read back) stay below twice the weight bytes (2*N*K) they help to stream: S <= K / (2 M).  (With the bound at
    // the weight bytes themselves, S <= K / (4 M), the QKV projection of the k = 8 shard of the 70B layer with 1024
    // tokens stopped at two ranges: 57 us, with four 47 us; the same for the QKV and down projections of the 13B
    // k = 4 shard with 512 tokens, 44 -> 41 and 46 -> 43 us; the 7B shapes with 256 tokens choose as before.)
    int split = 1;
    while (split < 8 && mid * split < 256 && (K / 64) % (split * 2) == 0 && (long long)(split * 2) * 2 * M <= K &&
           (size_t)(split * 2) * M * N * sizeof(float) <= ws_bytes && ws)
        split *= 2;
    return launch_cfg<128, 128, 2, 2>(a, lda, w, c, ldc, r, M, N, K, epi, s, split, ws, rs);
}

}  // namespace SS_NS
