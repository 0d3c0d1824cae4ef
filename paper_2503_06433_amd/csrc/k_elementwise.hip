// RMSNorm, SwiGLU (unfused form), embedding gather, rotary embedding + KV page
// write, and the load-time weight slicing.  All of these are HBM-bound
// element-wise passes: one wave-coalesced read and write per element.
#include "ss_device.h"
#include "ss_kernels.h"

namespace ssk {

// ---------------------------------------------------------------- RMSNorm
// One 256-thread block per token row.  Two passes over the row (the second hits
// the vector L1): sum of squares with a wave + LDS reduction, then scale.
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const T* __restrict__ x, const T* __restrict__ g,
                                                      T* __restrict__ out, int H, float eps) {
    constexpr int V = VecOf<T>::N;
    const int t = blockIdx.x;
    const T* row = x + (size_t)t * H;
    T* orow = out + (size_t)t * H;
    float ss = 0.f;
    const bool vec = (H % V) == 0;
    if (vec) {
        for (int i = threadIdx.x * V; i < H; i += 256 * V) {
            vec16 v = *reinterpret_cast<const vec16*>(row + i);
            float f[V];
            unpack16<T>(v, f);
#pragma unroll
            for (int j = 0; j < V; ++j) ss += f[j] * f[j];
        }
    } else {
        for (int i = threadIdx.x; i < H; i += 256) { float f = ldf(row + i); ss += f * f; }
    }
    __shared__ float part[4];
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = part[0] + part[1] + part[2] + part[3];
    const float r = 1.0f / sqrtf(tot / (float)H + eps);
    if (vec) {
        for (int i = threadIdx.x * V; i < H; i += 256 * V) {
            vec16 v = *reinterpret_cast<const vec16*>(row + i);
            vec16 gv = *reinterpret_cast<const vec16*>(g + i);
            float f[V], gf[V];
            unpack16<T>(v, f);
            unpack16<T>(gv, gf);
#pragma unroll
            for (int j = 0; j < V; ++j) f[j] = f[j] * r * gf[j];
            *reinterpret_cast<vec16*>(orow + i) = pack16<T>(f);
        }
    } else {
        for (int i = threadIdx.x; i < H; i += 256) stf(orow + i, ldf(row + i) * r * ldf(g + i));
    }
}

hipError_t rmsnorm(int dt, const void* x, const void* g, void* out, int T, int H, float eps, hipStream_t s) {
    if (T <= 0) return hipSuccess;
    if (H <= 0) return hipErrorInvalidValue;
    if (dt == F32)
        rmsnorm_kernel<float><<<T, 256, 0, s>>>((const float*)x, (const float*)g, (float*)out, H, eps);
    else
        rmsnorm_kernel<bf16_t><<<T, 256, 0, s>>>((const bf16_t*)x, (const bf16_t*)g, (bf16_t*)out, H, eps);
    return hipGetLastError();
}

// ---------------------------------------------------------------- SwiGLU (unfused)
template <typename T>
__global__ __launch_bounds__(256) void swiglu_kernel(const T* __restrict__ gu, T* __restrict__ out, int F) {
    const int t = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= F) return;
    const float a = ldf(gu + (size_t)t * 2 * F + j);
    const float b = ldf(gu + (size_t)t * 2 * F + F + j);
    stf(out + (size_t)t * F + j, a / (1.0f + expf(-a)) * b);
}

hipError_t swiglu(int dt, const void* gu, void* out, int T, int F, hipStream_t s) {
    if (T <= 0) return hipSuccess;
    if (F <= 0 || T > 65535 * 16) return hipErrorInvalidValue;
    // grid.y is limited to 65535: fold tokens in chunks
    for (int t0 = 0; t0 < T; t0 += 65535) {
        int n = T - t0 < 65535 ? T - t0 : 65535;
        dim3 grid((F + 255) / 256, n);
        if (dt == F32)
            swiglu_kernel<float><<<grid, 256, 0, s>>>((const float*)gu + (size_t)t0 * 2 * F, (float*)out + (size_t)t0 * F, F);
        else
            swiglu_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t*)gu + (size_t)t0 * 2 * F, (bf16_t*)out + (size_t)t0 * F, F);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------- embedding gather
template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const T* __restrict__ table, const int32_t* __restrict__ ids,
                                                    T* __restrict__ out, int H) {
    const int t = blockIdx.x;
    const T* src = table + (size_t)ids[t] * H;
    for (int i = threadIdx.x; i < H; i += 256) out[(size_t)t * H + i] = src[i];
}

hipError_t embed_rows(int dt, const void* table, const int32_t* ids, void* out, int n, int H, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    if (dt == F32)
        embed_kernel<float><<<n, 256, 0, s>>>((const float*)table, ids, (float*)out, H);
    else
        embed_kernel<bf16_t><<<n, 256, 0, s>>>((const bf16_t*)table, ids, (bf16_t*)out, H);
    return hipGetLastError();
}

// ---------------------------------------------------------------- RoPE + KV page write
// One block per token.  Work items are 16-byte chunk pairs (element i.. and
// i + d/2 ..) of the q and k heads, and 16-byte chunks of the v heads.
// K lands in its page as [head][slot][d]; V lands transposed, [head][d][vslot(slot)].
template <typename T>
__global__ __launch_bounds__(256) void rope_kvwrite_kernel(T* __restrict__ qkv, int n_q, int n_kv, int d,
                                                           const float* __restrict__ rope, BatchMeta bm,
                                                           T* __restrict__ k_pool, T* __restrict__ v_pool,
                                                           int page_size) {
    constexpr int V = VecOf<T>::N;
    const int t = blockIdx.x;
    const int pos = bm.tok_pos[t];
    const int sq = bm.tok_seq[t];
    const int page = bm.page_tables[(size_t)sq * bm.pt_stride + pos / page_size];
    const int slot = pos % page_size;
    const int half = d / 2;
    const int cph = half / V;                     // chunk pairs per head
    const size_t row_stride = (size_t)(n_q + 2 * n_kv) * d;
    T* row = qkv + (size_t)t * row_stride;
    const float* cs = rope + (size_t)pos * d;     // [half][2] = cos, sin interleaved
    const size_t page_elems = (size_t)n_kv * page_size * d;

    const int n_rot = (n_q + n_kv) * cph;
    for (int w = threadIdx.x; w < n_rot; w += 256) {
        const int head = w / cph;
        const int i0 = (w % cph) * V;
        T* lo_p = row + (size_t)head * d + i0;
        T* hi_p = lo_p + half;
        float lo[V], hi[V], olo[V], ohi[V];
        unpack16<T>(*reinterpret_cast<const vec16*>(lo_p), lo);
        unpack16<T>(*reinterpret_cast<const vec16*>(hi_p), hi);
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const float c = cs[2 * (i0 + j)], sn = cs[2 * (i0 + j) + 1];
            olo[j] = lo[j] * c - hi[j] * sn;
            ohi[j] = hi[j] * c + lo[j] * sn;
        }
        const vec16 plo = pack16<T>(olo), phi = pack16<T>(ohi);
        if (head < n_q) {
            *reinterpret_cast<vec16*>(lo_p) = plo;
            *reinterpret_cast<vec16*>(hi_p) = phi;
        } else {
            const int g = head - n_q;
            T* dst = k_pool + (size_t)page * page_elems + ((size_t)g * page_size + slot) * d + i0;
            *reinterpret_cast<vec16*>(dst) = plo;
            *reinterpret_cast<vec16*>(dst + half) = phi;
        }
    }
    // V: element (g, e) -> v_pool[page][g][e][slot]
    const T* vrow = row + (size_t)(n_q + n_kv) * d;
    T* vdst = v_pool + (size_t)page * page_elems + vslot(slot);
    const int n_v = n_kv * d;
    for (int w = threadIdx.x; w < n_v; w += 256) vdst[(size_t)w * page_size] = vrow[w];
}

hipError_t rope_kvwrite(int dt, void* qkv, int n_q, int n_kv, const float* rope_table, const BatchMeta& bm,
                        const KvLayer& kv, hipStream_t s) {
    if (bm.T <= 0) return hipSuccess;
    const int V = dt == F32 ? 4 : 8;
    if (kv.d % (2 * V) != 0 || kv.n_heads != n_kv || kv.page_size <= 0) return hipErrorInvalidValue;
    if (dt == F32)
        rope_kvwrite_kernel<float><<<bm.T, 256, 0, s>>>((float*)qkv, n_q, n_kv, kv.d, rope_table, bm,
                                                        (float*)kv.k_pool, (float*)kv.v_pool, kv.page_size);
    else
        rope_kvwrite_kernel<bf16_t><<<bm.T, 256, 0, s>>>((bf16_t*)qkv, n_q, n_kv, kv.d, rope_table, bm,
                                                         (bf16_t*)kv.k_pool, (bf16_t*)kv.v_pool, kv.page_size);
    return hipGetLastError();
}

// ---------------------------------------------------------------- weight slicing
// 32x32 tile transpose through LDS: src[K, ld] columns c0.. -> dst rows.
template <typename T>
__global__ __launch_bounds__(256) void slice_transpose_kernel(const T* __restrict__ src, int64_t ld, int K, int c0,
                                                              int n, T* __restrict__ dst, int blk, int blk_stride,
                                                              int row_off) {
    __shared__ T tile[32][33];
    const int k0 = blockIdx.x * 32, j0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
    for (int r = ty; r < 32; r += 8) {
        const int k = k0 + r, j = j0 + tx;
        if (k < K && j < n) tile[r][tx] = src[(size_t)k * ld + c0 + j];
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int j = j0 + r, k = k0 + tx;
        if (j < n && k < K) {
            const size_t drow = (size_t)(j / blk) * blk_stride + (j % blk) + row_off;
            dst[drow * K + k] = tile[tx][r];
        }
    }
}

hipError_t slice_transpose(int dt, const void* src, int64_t ld_src, int K, int c0, int n, void* dst, int blk,
                           int blk_stride, int row_off, hipStream_t s) {
    if (K <= 0 || n <= 0) return hipSuccess;
    if (blk <= 0) return hipErrorInvalidValue;
    dim3 grid((K + 31) / 32, (n + 31) / 32);
    if (grid.y > 65535) return hipErrorInvalidValue;
    if (dt == F32)
        slice_transpose_kernel<float><<<grid, 256, 0, s>>>((const float*)src, ld_src, K, c0, n, (float*)dst, blk,
                                                           blk_stride, row_off);
    else
        slice_transpose_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t*)src, ld_src, K, c0, n, (bf16_t*)dst, blk,
                                                            blk_stride, row_off);
    return hipGetLastError();
}

template <typename T>
__global__ void copy_kernel(const T* __restrict__ src, T* __restrict__ dst, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

hipError_t copy_elems(int dt, const void* src, void* dst, int64_t n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    const unsigned grid = (unsigned)((n + 255) / 256);
    if (dt == F32)
        copy_kernel<float><<<grid, 256, 0, s>>>((const float*)src, (float*)dst, n);
    else
        copy_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t*)src, (bf16_t*)dst, n);
    return hipGetLastError();
}

}  // namespace ssk
