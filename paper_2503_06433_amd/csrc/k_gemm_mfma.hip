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
#include "ss_device.h"
#include "ss_kernels.h"

namespace ssk {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

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
                                                                 int tiles_m, int tiles_n, int per_xcd) {
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
    u32x4_t a_reg[A_CH], b_reg[B_CH];

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nk = K / 64;
    const int lrow = lane & 31, lgrp = lane >> 5;

    auto fetch = [&](int kt) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) a_reg[i] = *reinterpret_cast<const u32x4_t*>(a_src[i] + (size_t)kt * 64);
#pragma unroll
        for (int i = 0; i < B_CH; ++i) b_reg[i] = *reinterpret_cast<const u32x4_t*>(b_src[i] + (size_t)kt * 64);
    };
    auto stash = [&](int buf) {
        uint8_t* An = As + buf * BM * 128;
        uint8_t* Bn = Bs + buf * BN * 128;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) *reinterpret_cast<u32x4_t*>(An + a_dst[i]) = a_reg[i];
#pragma unroll
        for (int i = 0; i < B_CH; ++i) *reinterpret_cast<u32x4_t*>(Bn + b_dst[i]) = b_reg[i];
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
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][i], bfr[ks & 1][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    fetch(0);
    stash(0);
    __syncthreads();
    for (int kt = 0; kt + 1 < nk; ++kt) {
        fetch(kt + 1);          // global loads of the next slice fly while this one is multiplied
        __builtin_amdgcn_sched_barrier(0);
        multiply(kt & 1);
        stash((kt + 1) & 1);
        __syncthreads();
    }
    multiply((nk - 1) & 1);

    // ---- epilogue
    const int col_in = lane & 31;
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
                    const float g = acc[i][j][v], u = acc[i][j + 1][v];
                    C[(size_t)r * ldc + oc] = f2bf(g / (1.0f + __expf(-g)) * u);
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
                    if (EPI == EPI_RESIDUAL) o += bf2f(R[(size_t)r * ldc + c]);
                    C[(size_t)r * ldc + c] = f2bf(o);
                }
            }
        }
    }
}

bool gemm_mfma_supported(int M, int N, int K, int lda, int ldc, int epi) {
    if (K % 64 != 0 || lda % 8 != 0) return false;
    if (epi == EPI_STORE_F32) return false;
    if (epi == EPI_SWIGLU && (N % 64 != 0)) return false;
    (void)M; (void)ldc;
    return true;
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch_cfg(const bf16_t* A, int lda, const bf16_t* Wt, bf16_t* C, int ldc, const bf16_t* R, int M,
                             int N, int K, int epi, hipStream_t s) {
    constexpr int NT = 64 * WM * WN;
    constexpr size_t LDS = (size_t)2 * (BM + BN) * 128;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const long long n_tiles = (long long)tiles_m * tiles_n;
    if (n_tiles > (1ll << 30)) return hipErrorInvalidValue;
    const int per_xcd = (int)((n_tiles + 7) / 8);
    const unsigned grid = (unsigned)per_xcd * 8;
#define SS_LAUNCH(E)                                                                                            \
    {                                                                                                           \
        auto kfn = gemm_mfma_kernel<BM, BN, WM, WN, E>;                                                         \
        static bool attr_set = false;                                                                           \
        if (!attr_set) {                                                                                        \
            hipError_t e = hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS); \
            if (e != hipSuccess) return e;                                                                      \
            attr_set = true;                                                                                    \
        }                                                                                                       \
        kfn<<<grid, NT, LDS, s>>>(A, lda, Wt, C, ldc, R, M, N, K, tiles_m, tiles_n, per_xcd);                   \
    }
    switch (epi) {
        case EPI_STORE: SS_LAUNCH(EPI_STORE) break;
        case EPI_RESIDUAL:
            if (!R) return hipErrorInvalidValue;
            SS_LAUNCH(EPI_RESIDUAL) break;
        case EPI_SWIGLU: SS_LAUNCH(EPI_SWIGLU) break;
        default: return hipErrorInvalidValue;
    }
#undef SS_LAUNCH
    return hipGetLastError();
}

hipError_t gemm_mfma_bf16(const void* A, int lda, const void* Wt, void* C, int ldc, const void* R, int M, int N,
                          int K, int epi, hipStream_t s) {
    const bf16_t* a = (const bf16_t*)A;
    const bf16_t* w = (const bf16_t*)Wt;
    bf16_t* c = (bf16_t*)C;
    const bf16_t* r = (const bf16_t*)R;
    // Tile choice: the large tile when it still yields a few waves of blocks per
    // CU, smaller tiles to keep all 256 CUs streaming weights at decode sizes.
    const long long big = (long long)((M + 255) / 256) * ((N + 255) / 256);
    const long long mid = (long long)((M + 127) / 128) * ((N + 127) / 128);
    if (big >= 512) return launch_cfg<256, 256, 2, 4>(a, lda, w, c, ldc, r, M, N, K, epi, s);
    if (mid >= 512) return launch_cfg<128, 128, 2, 2>(a, lda, w, c, ldc, r, M, N, K, epi, s);
    return launch_cfg<64, 64, 2, 1>(a, lda, w, c, ldc, r, M, N, K, epi, s);
}

}  // namespace ssk

// Tuning hook (not part of the C ABI): run one named tile configuration.
namespace ssk {
hipError_t gemm_mfma_bf16_cfg(int cfg, const void* A, int lda, const void* Wt, void* C, int ldc, const void* R,
                              int M, int N, int K, int epi, hipStream_t s) {
    const bf16_t* a = (const bf16_t*)A;
    const bf16_t* w = (const bf16_t*)Wt;
    bf16_t* c = (bf16_t*)C;
    const bf16_t* r = (const bf16_t*)R;
    switch (cfg) {
        case 0: return launch_cfg<256, 256, 2, 4>(a, lda, w, c, ldc, r, M, N, K, epi, s);
        case 1: return launch_cfg<128, 128, 2, 2>(a, lda, w, c, ldc, r, M, N, K, epi, s);
        case 2: return launch_cfg<64, 64, 2, 1>(a, lda, w, c, ldc, r, M, N, K, epi, s);
        default: return hipErrorInvalidValue;
    }
}
}  // namespace ssk
