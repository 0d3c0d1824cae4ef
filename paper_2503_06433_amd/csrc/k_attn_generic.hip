// Plain (non-MFMA) paged causal attention, any dtype, head_dim 64 or 128.
// Serves the fp32 configuration, and prefill and decode alike: a decode batch
// is a batch whose sequences each bring one query.
//
// One 256-thread block per (64-query tile, q head, sequence).  Four threads
// share a query row, each owning a quarter of the head dimension.  The block
// walks the sequence's pages in order; a page's K [16][D] and V^T [D][16]
// chunks are staged through LDS as floats; softmax is the streaming
// (running max / running sum) form in fp32.
#include "ss_device.h"
#include "ss_kernels.h"

namespace SS_NS {
using namespace ssk;

template <typename T, int D>
__global__ __launch_bounds__(256) void attn_generic_kernel(const T* __restrict__ qkv, T* __restrict__ out, int n_q,
                                                           int n_kv, BatchMeta bm, const T* __restrict__ k_pool,
                                                           const T* __restrict__ v_pool, float scale) {
    constexpr int PS = 16;
    constexpr int DS = D / 4;
    __shared__ float Ks[PS][D];
    __shared__ float Vs[D][PS + 1];
    const int sq = blockIdx.z, a = blockIdx.y, tile = blockIdx.x;
    const int q_begin = bm.cu_q[sq], q_len = bm.cu_q[sq + 1] - q_begin;
    if (tile * 64 >= q_len) return;
    const int before = bm.kv_before[sq];
    const int g = a / (n_q / n_kv);
    const int r = threadIdx.x >> 2, sub = threadIdx.x & 3;
    const int qi = tile * 64 + r;
    const bool valid = qi < q_len;
    const int p = before + (valid ? qi : 0);              // absolute position of this row's query
    const int last_q = (tile * 64 + 63 < q_len ? tile * 64 + 63 : q_len - 1);
    const int n_pages = (before + last_q) / PS + 1;
    const size_t row_stride = (size_t)(n_q + 2 * n_kv) * D;
    const T* qp = qkv + (size_t)(q_begin + (valid ? qi : 0)) * row_stride + (size_t)a * D + sub * DS;
    float q[DS], acc[DS];
#pragma unroll
    for (int e = 0; e < DS; ++e) { q[e] = ldf(qp + e) * scale; acc[e] = 0.f; }
    float m = -INFINITY, l = 0.f;
    const int32_t* pt = bm.page_tables + (size_t)sq * bm.pt_stride;
    const size_t page_elems = (size_t)n_kv * PS * D;
    for (int j = 0; j < n_pages; ++j) {
        const T* kp = k_pool + (size_t)pt[j] * page_elems + (size_t)g * PS * D;
        const T* vp = v_pool + (size_t)pt[j] * page_elems + (size_t)g * PS * D;
        for (int i = threadIdx.x; i < PS * D; i += 256) {
            (&Ks[0][0])[i] = ldf(kp + i);
            Vs[i / PS][i % PS] = ldf(vp + i);
        }
        __syncthreads();
        float s[PS];
        float mx = m;
#pragma unroll
        for (int jj = 0; jj < PS; ++jj) {
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < DS; ++e) d = fmaf(q[e], Ks[jj][sub * DS + e], d);
            d += __shfl_xor(d, 1, 64);
            d += __shfl_xor(d, 2, 64);
            s[jj] = (j * PS + jj <= p) ? d : -INFINITY;
            mx = fmaxf(mx, s[jj]);
        }
        // page 0 always holds position 0, which every query sees: mx is finite
        const float alpha = __expf(m - mx);
        l *= alpha;
#pragma unroll
        for (int e = 0; e < DS; ++e) acc[e] *= alpha;
#pragma unroll
        for (int jj = 0; jj < PS; ++jj) {
            const float pj = __expf(s[jj] - mx);
            l += pj;
#pragma unroll
            for (int e = 0; e < DS; ++e) acc[e] = fmaf(pj, Vs[sub * DS + e][vpos(jj, sub * DS + e)], acc[e]);
        }
        m = mx;
        __syncthreads();
    }
    if (valid) {
        T* op = out + (size_t)(q_begin + qi) * ((size_t)n_q * D) + (size_t)a * D + sub * DS;
        const float inv = 1.0f / l;
#pragma unroll
        for (int e = 0; e < DS; ++e) stf(op + e, acc[e] * inv);
    }
}

hipError_t attn_generic(int dt, const void* qkv, void* out, int n_q, int n_kv, const BatchMeta& bm,
                        const KvLayer& kv, hipStream_t s) {
    if (bm.T <= 0 || bm.n_seqs <= 0) return hipSuccess;
    if (kv.page_size != 16 || (kv.d != 64 && kv.d != 128) || n_kv <= 0 || n_q % n_kv != 0 || kv.n_heads != n_kv)
        return hipErrorInvalidValue;
    if (bm.n_seqs > 65535 || n_q > 65535) return hipErrorInvalidValue;
    dim3 grid((bm.max_q_len + 63) / 64, n_q, bm.n_seqs);
    const float scale = 1.0f / sqrtf((float)kv.d);
#define SS_GO(TT, DD)                                                                                       \
    attn_generic_kernel<TT, DD><<<grid, 256, 0, s>>>((const TT*)qkv, (TT*)out, n_q, n_kv, bm,               \
                                                     (const TT*)kv.k_pool, (const TT*)kv.v_pool, scale)
    if (dt == F32) {
        if (kv.d == 64) SS_GO(float, 64); else SS_GO(float, 128);
    } else {
        if (kv.d == 64) SS_GO(bf16_t, 64); else SS_GO(bf16_t, 128);
    }
#undef SS_GO
    return hipGetLastError();
}

}  // namespace SS_NS
