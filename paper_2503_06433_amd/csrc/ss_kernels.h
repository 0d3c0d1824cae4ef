// Internal launcher interface between the runtime (ss_runtime.hip) and the
// kernel files.  Everything here is device pointers + sizes; every launcher
// validates what its kernel assumes and returns hipErrorInvalidValue instead of
// launching a grid that would not fit.
#include <hip/hip_runtime.h>
#include <stdint.h>

// Shared types live in namespace ssk, once.  The launcher declarations follow in the namespace of the
// build: ssk for the brain-float build of the kernel files, ssk16 for the IEEE-half build (see
// ss_device.h).  A translation unit that calls both (the runtime) includes this file a second time with
// SS_DECL_NS set to the other namespace.
#ifndef SS_KERNELS_TYPES_H
#define SS_KERNELS_TYPES_H
namespace ssk {

enum Dtype { F32 = 0, BF16 = 1 };
inline size_t esize(int dt) { return dt == F32 ? 4 : 2; }

enum Epilogue {
    EPI_STORE = 0,      // C = acc
    EPI_RESIDUAL = 1,   // C = acc + R   (R has C's shape and leading dimension)
    EPI_SWIGLU = 2,     // weight rows come in blocks of 32 gate rows followed by the
                        // matching 32 up rows; C[m, j] = silu(gate_j) * up_j, C has N/2 columns
    EPI_STORE_F32 = 3,  // C is float regardless of the input dtype
};

// Paged cache geometry of one shard and one layer.
//   K page: [n_heads][page_size][d]   (token-major, d contiguous)
//   V page: [n_heads][d][page_size]   (transposed inside the page: token contiguous, in the
//           order 0-3, 8-11, 4-7, 12-15, the two halves swapped in rows d with bit 3 set, see vpos() in ss_device.h)
// page p of the pool starts at element p * n_heads * page_size * d.
struct KvLayer {
    void* k_pool;
    void* v_pool;
    int n_heads;     // local kv heads
    int d;
    int page_size;
};

// Per-token metadata of a batch (device arrays): tok_seq[t] = index of the
// sequence inside the batch, tok_pos[t] = absolute position.  page_tables is
// [n_seqs, pt_stride] int32.
struct BatchMeta {
    const int32_t* tok_seq;
    const int32_t* tok_pos;
    const int32_t* page_tables;
    int pt_stride;
    const int32_t* cu_q;        // [n_seqs+1] first token of each sequence in the batch
    const int32_t* kv_before;   // [n_seqs]
    int n_seqs;
    int T;
    int max_q_len;
    // page units of the new tokens: unit u = the tokens of sequence unit_seq[u] that fall into one of its
    // pages: batch tokens [unit_tok0[u], +unit_cnt[u]), absolute positions from unit_pos0[u]
    const int32_t* unit_seq;
    const int32_t* unit_tok0;
    const int32_t* unit_pos0;
    const int32_t* unit_cnt;
    int n_units;
    // work lists of the LDS-staged prefill attention (null for decode batches): block b of pf_blocks walks the
    // items pf_items[(b * pf_stride + j) * 8 .. +7] = (sequence, q head, first query of a block of 256, first batch
    // token of the sequence, its new tokens, its cached tokens, 0, 0), j = 0, 1, ... up to a sequence of -1 (32-byte
    // records, 32-byte aligned).  All items that read the pages of one (sequence, kv head) are in lists of blocks
    // with the same b % 8; within a list the item with the most cached tokens to visit comes first.
    const int32_t* pf_items;
    int pf_stride;
    int pf_blocks;
};

// One query token per sequence.  work items (seq, first page, n pages) split long
// sequences; partial results go through `scratch` (floats) and are merged.
struct DecodeWork {
    const int32_t* item_seq;    // [n_items]
    const int32_t* item_page0;  // [n_items] first page index within the sequence
    const int32_t* item_npages; // [n_items] low 16 bits: number of pages; high 16 bits: stride between them in pages
                                //           (0 = 1): pages page0, page0 + stride, ...
    const int32_t* seq_item0;   // [n_seqs+1] first item of each sequence
    const int32_t* item_order;  // [n_items] launch order (block x works on item item_order[x])
    int n_items;
    int max_items_per_seq;
};

// KV repack between pages and heads-major staging.
// unit u = one (sequence, local layer): a staging block [2][n_heads][len][d] at
// element offset unit_off[u]; its page list starts at pages[unit_pt[u]]; the
// layer's pools are k_pools[unit_layer[u]] / v_pools[unit_layer[u]].
struct RepackUnits {
    const int64_t* unit_off;
    const int32_t* unit_len;
    const int32_t* unit_pt;      // offset into `pages`
    const int32_t* unit_layer;   // local layer index
    const int32_t* pages;        // concatenated page lists
    int n_units;
    int max_pages;               // most pages of any unit
};

}  // namespace ssk
#endif

#ifndef SS_DECL_NS
#ifdef SS_HALF_F16
#define SS_DECL_NS ssk16
#else
#define SS_DECL_NS ssk
#endif
#endif
namespace SS_DECL_NS {
using namespace ssk;

// C[M,N] = A[M,K] * Wt[N,K]^T.  A row-major with leading dimension lda, Wt
// row-major [N,K] (K contiguous), C row-major with leading dimension ldc.
// force_generic selects the plain LDS-tiled FMA kernel (any shape, any dtype);
// otherwise bf16 with K % 64 == 0 runs on the MFMA kernel.
// `ws` is an optional float workspace of ws_bytes for split-K partial sums (used
// when the output has too few tiles to occupy the chip, as at decode batch sizes).
// The large-output bf16 kernel runs as persistent blocks that own their CUs until the launch is done;
// max_rounds > 0 cuts it into launches of at most that many output tiles per block, so that kernels of
// other streams (the KV movers' repack kernels) get the chip at the boundaries; 0 = one launch.
// row_scale (optional, M floats): row m of the product is multiplied by row_scale[m] before the epilogue's
// activation or store: the RMSNorm factor of token m when A holds the raw activations and the gains are
// folded into the weight rows.  Not combined with EPI_RESIDUAL or EPI_STORE_F32 by the large-output and
// fp32-output kernels (refused there).
hipError_t gemm_nt(int dt, const void* A, int lda, const void* Wt, void* C, int ldc,
                   const void* R, int M, int N, int K, int epi, bool force_generic,
                   hipStream_t s, float* ws = nullptr, size_t ws_bytes = 0, int max_rounds = 0,
                   const float* row_scale = nullptr);

// out[t,:] = x[t,:] * rsqrt(mean(x[t,:]^2) + eps) * g
hipError_t rmsnorm(int dt, const void* x, const void* g, void* out, int T, int H, float eps,
                   hipStream_t s);

// r[t] = rsqrt(mean(x[t,:]^2) + eps)
hipError_t row_scale(int dt, const void* x, float* r, int T, int H, float eps, hipStream_t s);

// out[t, j] = silu(gu[t, j]) * gu[t, F + j]   (unfused form used by the generic GEMM path)
hipError_t swiglu(int dt, const void* gu, void* out, int T, int F, hipStream_t s);

// Gathers rows of an embedding table.
hipError_t embed_rows(int dt, const void* table, const int32_t* ids, void* out, int n, int H,
                      hipStream_t s);

// Rotates q and k in place inside qkv [T, (n_q + 2 n_kv) d] by the token's
// position (half-split pairing, angles from the fp32 table rope[pos][d/2][cos,sin]),
// then writes the rotated k and the v of every token into the pages.
hipError_t rope_kvwrite(int dt, void* qkv, int n_q, int n_kv, const float* rope_table,
                        const BatchMeta& bm, const KvLayer& kv, hipStream_t s);

// Causal attention of the batch's new tokens against the paged cache (which
// already holds them).  q is read from qkv (row stride (n_q + 2 n_kv) d), out is
// [T, n_q d].  Query at absolute position p sees cache positions 0..p.
hipError_t attn_prefill(int dt, const void* qkv, void* out, int n_q, int n_kv,
                        const BatchMeta& bm, const KvLayer& kv, bool force_generic, hipStream_t s);

size_t attn_decode_scratch_floats(int n_items, int n_q, int d);

hipError_t attn_decode(int dt, const void* qkv, void* out, int n_q, int n_kv,
                       const BatchMeta& bm, const KvLayer& kv, const DecodeWork& wk,
                       float* scratch, bool force_generic, hipStream_t s);

hipError_t kv_gather(int dt, void* const* k_pools, void* const* v_pools, int n_heads, int d,
                     int page_size, const RepackUnits& u, void* staging, hipStream_t s);

hipError_t kv_scatter(int dt, void* const* k_pools, void* const* v_pools, int n_heads, int d,
                      int page_size, const RepackUnits& u, const void* staging, hipStream_t s);

// Weight slicing at load time: column j (0 <= j < n) of src[K, ld_src], taken from
// column c0 + j, becomes row  (j / blk) * blk_stride + (j % blk) + row_off  of
// dst[*, K] (K contiguous).  blk = n, row_off = 0 gives the plain transpose.  With `gain` (K values of the
// model dtype) element [k, j] is multiplied by gain[k] and rounded once to the storage type.
hipError_t slice_transpose(int dt, const void* src, int64_t ld_src, int K, int c0, int n,
                           void* dst, int blk, int blk_stride, int row_off, hipStream_t s,
                           const void* gain = nullptr);

// out[r] = argmax of logits[r, 0..V), lowest index on ties (greedy decoding).
hipError_t argmax_rows(const float* logits, int n, int V, int32_t* out, hipStream_t s);

// dst[i] = src[i] for i < n (elements of the model dtype); used for gains.
hipError_t copy_elems(int dt, const void* src, void* dst, int64_t n, hipStream_t s);



}  // namespace SS_DECL_NS
#undef SS_DECL_NS
