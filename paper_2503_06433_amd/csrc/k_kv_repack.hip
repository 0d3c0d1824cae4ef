// KV repack between the paged device cache and heads-major staging
//   staging unit (one sequence, one local layer): [K|V][head][position][d]
// the layout the host tier keeps (heads x seq_len x head_dim per layer and K|V),
// so that a tensor-parallel shard's heads are contiguous runs.
//
// Pure data movement, HBM-bound: every byte is read once and written once with
// 16-byte accesses.  One block per (page, unit, head).  K page chunks ([16][d] per
// head) are already position-major and are copied straight through; V page
// chunks are stored transposed in the page ([d][16], token order see vpos) and go through a small
// LDS tile to be turned back into [position][d] (and the reverse on scatter).
#include "ss_device.h"
#include "ss_kernels.h"

namespace SS_NS {
using namespace ssk;

template <typename E, bool GATHER>
__global__ __launch_bounds__(256) void kv_repack_kernel(void* const* __restrict__ k_pools,
                                                        void* const* __restrict__ v_pools, int n_heads, int d,
                                                        RepackUnits u, E* __restrict__ staging) {
    constexpr int PS = 16;
    constexpr int EV = 16 / (int)sizeof(E);          // elements per 16-byte vector
    const int unit = blockIdx.y, pg = blockIdx.x;
    const int len = u.unit_len[unit];
    if (pg * PS >= len) return;
    const int page = u.pages[u.unit_pt[unit] + pg];
    const int layer = u.unit_layer[unit];
    const int p0 = pg * PS;
    const int nvalid = (len - p0) < PS ? (len - p0) : PS;
    E* kpool = reinterpret_cast<E*>(k_pools[layer]);
    E* vpool = reinterpret_cast<E*>(v_pools[layer]);
    const size_t chunk = (size_t)PS * d;             // elements of one head's page chunk
    E* st = staging + u.unit_off[unit];
    const int vec_per_row = d / EV;                  // 16-byte vectors per position row
    const int vec_per_chunk = PS * vec_per_row;

    // ---- K: straight copy of the valid rows (one head per block: blockIdx.z)
    const int g = blockIdx.z;
    for (int r = threadIdx.x; r < vec_per_chunk; r += 256) {
        const int tok = r / vec_per_row;
        if (tok >= nvalid) continue;
        E* pgp = kpool + ((size_t)page * n_heads + g) * chunk + (size_t)r * EV;
        E* stp = st + ((size_t)g * len + p0) * d + (size_t)r * EV;
        if (GATHER) st16_stream(stp, ld16_stream(pgp));
        else st16_stream(pgp, ld16_stream(stp));
    }

    // ---- V: [d][16] in the page <-> [position][d] in staging
    __shared__ E tile[128][PS + 1];   // odd row stride: the transposed element reads of 16 lanes fall on 16 banks
    E* stv = st + (size_t)n_heads * len * d;          // V half of the unit
    constexpr int VPR = PS / EV;                      // vectors per d-row of the page chunk
    {
        E* pgp = vpool + ((size_t)page * n_heads + g) * chunk;
        E* stp = stv + ((size_t)g * len + p0) * d;
        if (GATHER) {
            for (int i = threadIdx.x; i < d * VPR; i += 256) {
                const int e = i / VPR, t0 = (i % VPR) * EV;
                union { vec16 v; E x[EV]; } w;
                w.v = ld16_stream(pgp + (size_t)e * PS + t0);
#pragma unroll
                for (int j = 0; j < EV; ++j) tile[e][t0 + j] = w.x[j];
            }
            __syncthreads();
            for (int o = threadIdx.x; o < nvalid * vec_per_row; o += 256) {
                const int tok = o / vec_per_row, e0 = (o % vec_per_row) * EV;
                union { vec16 v; E x[EV]; } w;
#pragma unroll
                for (int j = 0; j < EV; ++j) w.x[j] = tile[e0 + j][vpos(tok, e0 + j)];
                st16_stream(stp + (size_t)tok * d + e0, w.v);
            }
        } else {
            for (int o = threadIdx.x; o < PS * vec_per_row; o += 256) {
                const int tok = o / vec_per_row, e0 = (o % vec_per_row) * EV;
                union { vec16 v; E x[EV]; } w;
                if (tok < nvalid) w.v = ld16_stream(stp + (size_t)tok * d + e0);
                else w.v = vec16{{0u, 0u, 0u, 0u}};
#pragma unroll
                for (int j = 0; j < EV; ++j) tile[e0 + j][vpos(tok, e0 + j)] = w.x[j];
            }
            __syncthreads();
            for (int i = threadIdx.x; i < d * VPR; i += 256) {
                const int e = i / VPR, t0 = (i % VPR) * EV;
                union { vec16 v; E x[EV]; } w;
#pragma unroll
                for (int j = 0; j < EV; ++j) w.x[j] = tile[e][t0 + j];
                st16_stream(pgp + (size_t)e * PS + t0, w.v);
            }
        }
        __syncthreads();
    }
}

template <bool GATHER>
static hipError_t launch_repack(int dt, void* const* k_pools, void* const* v_pools, int n_heads, int d,
                                int page_size, const RepackUnits& u, void* staging, hipStream_t s) {
    if (u.n_units <= 0 || u.max_pages <= 0) return hipSuccess;
    if (page_size != 16 || d > 128 || d % 8 != 0 || n_heads <= 0 || n_heads > 65535 || u.n_units > 65535) return hipErrorInvalidValue;
    dim3 grid(u.max_pages, u.n_units, n_heads);
    if (dt == F32)
        kv_repack_kernel<uint32_t, GATHER><<<grid, 256, 0, s>>>(k_pools, v_pools, n_heads, d, u, (uint32_t*)staging);
    else
        kv_repack_kernel<uint16_t, GATHER><<<grid, 256, 0, s>>>(k_pools, v_pools, n_heads, d, u, (uint16_t*)staging);
    return hipGetLastError();
}

hipError_t kv_gather(int dt, void* const* k_pools, void* const* v_pools, int n_heads, int d, int page_size,
                     const RepackUnits& u, void* staging, hipStream_t s) {
    return launch_repack<true>(dt, k_pools, v_pools, n_heads, d, page_size, u, staging, s);
}

hipError_t kv_scatter(int dt, void* const* k_pools, void* const* v_pools, int n_heads, int d, int page_size,
                      const RepackUnits& u, const void* staging, hipStream_t s) {
    return launch_repack<false>(dt, k_pools, v_pools, n_heads, d, page_size, u, const_cast<void*>(staging), s);
}

}  // namespace SS_NS
