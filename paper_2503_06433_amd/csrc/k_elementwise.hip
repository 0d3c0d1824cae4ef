// RMSNorm, SwiGLU (unfused form), embedding gather, rotary embedding + KV page
// write, and the load-time weight slicing.  All of these are HBM-bound
// element-wise passes: one wave-coalesced read and write per element.
#include "ss_device.h"
#include "ss_kernels.h"

namespace SS_NS {
using namespace ssk;

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

// ---------------------------------------------------------------- RMSNorm statistics
// r[t] = 1 / sqrt(mean(x[t,:]^2) + eps): the per-row factor of RMSNorm.  The gains are folded into the rows
// of the weight matrix that follows and the factor is applied in that product's epilogue
// (norm(x) W = r * (x (g W))), so the normalised activations are never written.  One read of x, T floats out.
// One wave per row, four rows per block.
template <typename T>
__global__ __launch_bounds__(256) void row_scale_kernel(const T* __restrict__ x, float* __restrict__ r, int n_rows, int H,
                                                        float eps) {
    constexpr int V = VecOf<T>::N;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= n_rows) return;
    const int lane = threadIdx.x & 63;
    const T* row = x + (size_t)t * H;
    float ss = 0.f;
    if ((H % V) == 0) {
        for (int i = lane * V; i < H; i += 64 * V) {
            vec16 v = *reinterpret_cast<const vec16*>(row + i);
            float f[V];
            unpack16<T>(v, f);
#pragma unroll
            for (int j = 0; j < V; ++j) ss += f[j] * f[j];
        }
    } else {
        for (int i = lane; i < H; i += 64) { float f = ldf(row + i); ss += f * f; }
    }
    ss = wave_sum(ss);
    if (lane == 0) r[t] = 1.0f / sqrtf(ss / (float)H + eps);
}

hipError_t row_scale(int dt, const void* x, float* r, int T, int H, float eps, hipStream_t s) {
    if (T <= 0) return hipSuccess;
    if (H <= 0) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)((T + 3) / 4);
    if (dt == F32) row_scale_kernel<float><<<grid, 256, 0, s>>>((const float*)x, r, T, H, eps);
    else row_scale_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t*)x, r, T, H, eps);
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

// ---------------------------------------------------------------- greedy token choice
// out[r] = index of the largest of logits[r, 0..V); the lowest index wins a tie.  One block per row.
__global__ __launch_bounds__(256) void argmax_rows_kernel(const float* __restrict__ logits, int V, int32_t* __restrict__ out) {
    const float* row = logits + (size_t)blockIdx.x * V;
    float best = -INFINITY;
    int bi = 0x7fffffff;
    for (int i = threadIdx.x; i < V; i += 256) {
        const float v = row[i];
        if (v > best || (v == best && i < bi)) { best = v; bi = i; }
    }
    __shared__ float sv[256];
    __shared__ int si[256];
    sv[threadIdx.x] = best;
    si[threadIdx.x] = bi;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) {
            const float v = sv[threadIdx.x + o];
            const int i = si[threadIdx.x + o];
            if (v > sv[threadIdx.x] || (v == sv[threadIdx.x] && i < si[threadIdx.x])) { sv[threadIdx.x] = v; si[threadIdx.x] = i; }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) out[blockIdx.x] = si[0] == 0x7fffffff ? 0 : si[0];
}

hipError_t argmax_rows(const float* logits, int n, int V, int32_t* out, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    if (V <= 0) return hipErrorInvalidValue;
    argmax_rows_kernel<<<n, 256, 0, s>>>(logits, V, out);
    return hipGetLastError();
}

// ---------------------------------------------------------------- RoPE + KV page write
// One block per (page unit, HB kv heads): the new tokens of one sequence that fall into one page (up to 16),
// with the q heads of those kv heads' groups, the k heads and the v heads (several heads per block at
// prefill sizes: a thread loads the cos / sin values of its token and chunk once and reuses them over the
// heads, and has several independent rows in flight).  q is rotated in place; the rotated
// k rows land in the page as [slot][d] (one contiguous run); v lands transposed, [d][vpos(slot, d)].  A full
// page of v goes through an LDS tile and is written as one contiguous 16-byte-per-lane run; partial pages
// (the first and last page of a prompt, every decode step) write element by element.
template <typename T, int HB>
__global__ __launch_bounds__(256) void rope_kvwrite_kernel(T* __restrict__ qkv, int n_q, int n_kv, int d,
                                                           const float* __restrict__ rope, BatchMeta bm,
                                                           T* __restrict__ k_pool, T* __restrict__ v_pool) {
    constexpr int V = VecOf<T>::N;
    constexpr int PS = 16;
    // the head groups of a page unit are adjacent blocks: together they read whole rows of the qkv buffer
    const int n_hg = (n_kv + HB - 1) / HB;
    const int u = blockIdx.x / n_hg, g0 = (blockIdx.x % n_hg) * HB;          // HB kv heads per block
    const int sq = bm.unit_seq[u], tok0 = bm.unit_tok0[u], pos0 = bm.unit_pos0[u], cnt = bm.unit_cnt[u];
    const int page = bm.page_tables[(size_t)sq * bm.pt_stride + pos0 / PS];
    const int slot0 = pos0 % PS;
    const int G = n_q / n_kv;
    const int half = d / 2;
    const int cph = half / V;                     // 16-byte chunk pairs per head row
    const size_t row_stride = (size_t)(n_q + 2 * n_kv) * d;
    const size_t page_elems = (size_t)n_kv * PS * d;
    const int nh = (n_kv - g0) < HB ? (n_kv - g0) : HB;      // kv heads of this block

    // ---- rotation: a thread keeps one (token, chunk pair) and its cos / sin values and walks over the
    // head slots (the G q heads and the k head of each kv head of the block)
    const int per_head = cnt * cph;               // <= 128 for d <= 128
    const int lanes = per_head < 256 ? per_head : 256;
    const int stride_h = 256 / (lanes > 0 ? lanes : 1);      // head slots processed side by side
    if (per_head > 0 && (int)threadIdx.x < lanes * stride_h) {
        const int r = threadIdx.x % lanes, h_first = threadIdx.x / lanes;
        const int tl = r / cph, i0 = (r % cph) * V;
        const float* cs = rope + (size_t)(pos0 + tl) * d + 2 * i0;    // [half][2] = cos, sin interleaved
        float c[V], sn[V];
#pragma unroll
        for (int j = 0; j < V; ++j) { c[j] = cs[2 * j]; sn[j] = cs[2 * j + 1]; }
        const int slots = nh * (G + 1);
        T* row = qkv + (size_t)(tok0 + tl) * row_stride + i0;
#pragma unroll 4
        for (int hs = h_first; hs < slots; hs += stride_h) {
            const int gl = hs / (G + 1), hh = hs % (G + 1);
            const int g = g0 + gl;
            const int head = hh < G ? g * G + hh : n_q + g;      // column block of the qkv row
            T* lo_p = row + (size_t)head * d;
            T* hi_p = lo_p + half;
            float lo[V], hi[V], olo[V], ohi[V];
            unpack16<T>(*reinterpret_cast<const vec16*>(lo_p), lo);
            unpack16<T>(*reinterpret_cast<const vec16*>(hi_p), hi);
#pragma unroll
            for (int j = 0; j < V; ++j) {
                olo[j] = lo[j] * c[j] - hi[j] * sn[j];
                ohi[j] = hi[j] * c[j] + lo[j] * sn[j];
            }
            const vec16 plo = pack16<T>(olo), phi = pack16<T>(ohi);
            if (hh < G) {
                *reinterpret_cast<vec16*>(lo_p) = plo;
                *reinterpret_cast<vec16*>(hi_p) = phi;
            } else {
                T* dst = k_pool + (size_t)page * page_elems + (size_t)g * PS * d + (size_t)(slot0 + tl) * d + i0;
                *reinterpret_cast<vec16*>(dst) = plo;
                *reinterpret_cast<vec16*>(dst + half) = phi;
            }
        }
    }

    // ---- v: element (token tl, e) of head g -> vpage[e][vpos(slot0 + tl, e)]
    __shared__ T tile[HB][PS][128 + V];
    if (cnt == PS && d == 128) {                   // block-uniform: whole pages go through LDS
        constexpr int CPR = 128 / V;               // 16-byte chunks per row
        for (int w = threadIdx.x; w < nh * PS * CPR; w += 256) {
            const int gl = w / (PS * CPR), tl = (w / CPR) % PS, cc = w % CPR;
            const T* vcol = qkv + (size_t)(tok0 + tl) * row_stride + (size_t)(n_q + n_kv + g0 + gl) * d;
            *reinterpret_cast<vec16*>(&tile[gl][tl][cc * V]) = *reinterpret_cast<const vec16*>(vcol + cc * V);
        }
        __syncthreads();
        // 16-byte piece `pc` of row e holds positions [V*pc, V*pc + V); position p of row e is token vtok(p, e)
        constexpr int PPR = PS / V;
        for (int w = threadIdx.x; w < nh * 128 * PPR; w += 256) {
            const int gl = w / (128 * PPR), e = (w / PPR) % 128, pc = w % PPR;
            union { vec16 v; T x[V]; } o;
#pragma unroll
            for (int j = 0; j < V; ++j) o.x[j] = tile[gl][vtok(pc * V + j, e)][e];
            T* vpage = v_pool + (size_t)page * page_elems + (size_t)(g0 + gl) * PS * d;
            *reinterpret_cast<vec16*>(vpage + (size_t)e * PS + pc * V) = o.v;
        }
    } else {
        for (int w = threadIdx.x; w < nh * cnt * d; w += 256) {
            const int gl = w / (cnt * d), tl = (w / d) % cnt, e = w % d;
            const T* vcol = qkv + (size_t)(tok0 + tl) * row_stride + (size_t)(n_q + n_kv + g0 + gl) * d;
            T* vpage = v_pool + (size_t)page * page_elems + (size_t)(g0 + gl) * PS * d;
            vpage[(size_t)e * PS + vpos(slot0 + tl, e)] = vcol[e];
        }
    }
}

hipError_t rope_kvwrite(int dt, void* qkv, int n_q, int n_kv, const float* rope_table, const BatchMeta& bm,
                        const KvLayer& kv, hipStream_t s) {
    if (bm.T <= 0 || bm.n_units <= 0) return hipSuccess;
    const int V = dt == F32 ? 4 : 8;
    if (kv.d % (2 * V) != 0 || kv.n_heads != n_kv || kv.page_size != 16 || n_kv <= 0 || n_q % n_kv != 0 || n_kv > 65535)
        return hipErrorInvalidValue;
    if (kv.d > 128 || (long long)bm.n_units * n_kv > 0x7fffffffll) return hipErrorInvalidValue;
    if (dt == F32) {
        dim3 grid((unsigned)(bm.n_units * n_kv));
        rope_kvwrite_kernel<float, 1><<<grid, 256, 0, s>>>((float*)qkv, n_q, n_kv, kv.d, rope_table, bm,
                                                           (float*)kv.k_pool, (float*)kv.v_pool);
    } else if (n_kv >= 4 && bm.n_units >= 256) {    // prefill-sized: several kv heads per block (cos / sin reused)
        dim3 grid((unsigned)(bm.n_units * ((n_kv + 3) / 4)));
        rope_kvwrite_kernel<bf16_t, 4><<<grid, 256, 0, s>>>((bf16_t*)qkv, n_q, n_kv, kv.d, rope_table, bm,
                                                            (bf16_t*)kv.k_pool, (bf16_t*)kv.v_pool);
    } else {
        dim3 grid((unsigned)(bm.n_units * n_kv));
        rope_kvwrite_kernel<bf16_t, 1><<<grid, 256, 0, s>>>((bf16_t*)qkv, n_q, n_kv, kv.d, rope_table, bm,
                                                            (bf16_t*)kv.k_pool, (bf16_t*)kv.v_pool);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------- weight slicing
// 32x32 tile transpose through LDS: src[K, ld] columns c0.. -> dst rows.  With `gain`, source row k is
// multiplied by gain[k] on the way (the product of two stored values is formed in fp32 and rounded once to
// the storage type): the RMSNorm gains folded into the matrix that consumes the normalised activations.
template <typename T>
__global__ __launch_bounds__(256) void slice_transpose_kernel(const T* __restrict__ src, int64_t ld, int K, int c0,
                                                              int n, T* __restrict__ dst, int blk, int blk_stride,
                                                              int row_off, const T* __restrict__ gain) {
    __shared__ T tile[32][33];
    const int k0 = blockIdx.x * 32, j0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
    for (int r = ty; r < 32; r += 8) {
        const int k = k0 + r, j = j0 + tx;
        if (k < K && j < n) {
            T v = src[(size_t)k * ld + c0 + j];
            if (gain) {
                T w;
                stf(&w, ldf(&v) * ldf(gain + k));
                v = w;
            }
            tile[r][tx] = v;
        }
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
                           int blk_stride, int row_off, hipStream_t s, const void* gain) {
    if (K <= 0 || n <= 0) return hipSuccess;
    if (blk <= 0) return hipErrorInvalidValue;
    dim3 grid((K + 31) / 32, (n + 31) / 32);
    if (grid.y > 65535) return hipErrorInvalidValue;
    if (dt == F32)
        slice_transpose_kernel<float><<<grid, 256, 0, s>>>((const float*)src, ld_src, K, c0, n, (float*)dst, blk,
                                                           blk_stride, row_off, (const float*)gain);
    else
        slice_transpose_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t*)src, ld_src, K, c0, n, (bf16_t*)dst, blk,
                                                            blk_stride, row_off, (const bf16_t*)gain);
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

}  // namespace SS_NS
