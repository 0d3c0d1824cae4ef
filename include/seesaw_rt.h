/*
 * seesaw_rt.h - C ABI of the MI355X (gfx950) hot path of re-sharded LLM inference:
 * one GPU's share of a LLaMA-style decoder layer in the pipeline-parallel layout
 * used for prefill and in the tensor-parallel layout used for decode, plus the
 * KV-cache movement through a host-DRAM tier that converts one into the other.
 *
 * Conventions shared by every call
 *   - returns 0 (SS_OK) or a negative SS_E* code; never throws or aborts across
 *     the ABI; ss_last_error() gives the text of the last failure of a context.
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP
 *     device memory of the context's GPU; every argument says which it is.
 *   - activations are row-major [tokens, hidden] in the model dtype (SS_F32:
 *     IEEE float, SS_BF16: 16-bit brain float, SS_F16: IEEE half, raw bits;
 *     the 16-bit types accumulate in fp32) and are CALLER-owned
 *     device buffers; weights are copied by the library at load time; KV pages,
 *     the host tier, the pinned staging ring and the side stream are
 *     library-owned.
 *   - `stream` is a hipStream_t (0 = the null stream).  Layer calls are
 *     asynchronous on it.  KV movement runs on the library's side stream, driven
 *     by a library-owned host thread, and is complete after ss_sync().
 *   - one context per GPU, calls on one context come from one thread at a time.
 *   - ONE compute stream per context: the layer calls, ss_embed, ss_lm_head and
 *     the device-side export / import of a context share its workspaces and
 *     cached batch metadata, which are ordered by stream order alone.  Pass the
 *     same stream to all of them (or synchronise the device between calls that
 *     use different streams).  The `stream` arguments of ss_kv_swap,
 *     ss_kv_reshard and ss_reshard_weights only name what the movement has to
 *     come after; they may be any stream.
 *   - ss_kv_swap(SS_IN) and ss_kv_import_dev are all or nothing: when the pages
 *     of the listed sequences do not fit the pool together, SS_ENOMEM is
 *     returned, no page is taken and no sequence becomes resident.
 */
#ifndef SEESAW_RT_H
#define SEESAW_RT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { SS_F32 = 0, SS_BF16 = 1, SS_F16 = 2 };     /* model dtype (the paper runs in IEEE half, section 6.1) */
enum { SS_PP = 0, SS_TP = 1 };                    /* shard mode */
enum { SS_ATTN = 1, SS_MLP = 2, SS_BOTH = 3,      /* phase */
       SS_NO_RESIDUAL = 4 };                      /* flag OR-ed into phase */
enum { SS_OUT = 0, SS_IN = 1 };                   /* swap direction */
enum { SS_HOST = 0, SS_DEVICE = 1 };              /* where weight pointers live */
enum { SS_OK = 0, SS_EINVAL = -1, SS_ENOMEM = -2, SS_ENOENT = -3, SS_EHIP = -4 };

typedef struct ss_ctx ss_ctx;

/* Model shape.  head_dim must be 64 or 128; page_size must be 16. */
typedef struct {
    int32_t hidden, n_q_heads, n_kv_heads, head_dim, ffn, n_layers, vocab;
    float rms_eps, rope_base;
    int32_t dtype;       /* SS_F32 | SS_BF16 | SS_F16 */
    int32_t page_size;   /* tokens per KV page */
} ss_model_cfg;

typedef struct {
    int64_t gpu_kv_pages;    /* pages in the pool of EACH shard descriptor used */
    int64_t host_tier_bytes; /* capacity of the host tier (complete caches); allocated page-locked up to 64 GiB
                                (environment SS_TIER_PIN_MAX_GB), pageable above */
    int64_t pinned_bytes;    /* pinned staging: two lanes (out, in) of two slots each; used for every movement
                                into a pageable tier and for runs shorter than 256 KiB into a page-locked one */
    int32_t device;          /* HIP device ordinal */
    int32_t max_seq_len;     /* longest sequence (rotary table size) */
} ss_runtime_cfg;

/*
 * What one GPU holds (paper section 3.1, Observations 1 and 2; Appendix A.3).
 *   SS_PP: layers [layer_begin, layer_end), all heads, all FFN columns;
 *          k and shard are ignored except that k must be >= 1.
 *   SS_TP: layers [layer_begin, layer_end), q heads [shard*n_q/k, (shard+1)*n_q/k),
 *          kv heads [shard*n_kv/k, ...), FFN columns [shard*ffn/k, ...).
 *          k must divide n_q_heads, n_kv_heads and ffn (k > n_kv_heads is refused).
 * Every distinct descriptor owns its own weights, page pool and page tables, as
 * a distinct GPU would.
 */
typedef struct { int32_t mode, k, shard, layer_begin, layer_end; } ss_shard_desc;

/* A batch of sequences: host arrays, caller-owned, read during the call only.
 * Tokens of the batch are concatenated in this order in the activation buffers.
 * q_lens[i] new tokens of sequence i sit at positions kv_lens_before[i] ... */
typedef struct {
    int32_t n_seqs;
    const int64_t* seq_ids;
    const int32_t* q_lens;
    const int32_t* kv_lens_before;
} ss_batch;

/* Full (unsharded) weights of one layer, row-major [in_features, out_features],
 * model dtype; g1/g2 are the two RMSNorm gains [hidden].
 * wq [H, n_q*d]  wk, wv [H, n_kv*d]  wo [n_q*d, H]  wg, wu [H, ffn]  wd [ffn, H] */
typedef struct {
    const void *g1, *wq, *wk, *wv, *wo, *g2, *wg, *wu, *wd;
    int32_t location;    /* SS_HOST | SS_DEVICE: applies to all nine pointers */
} ss_layer_weights;

/* ---- life cycle ------------------------------------------------------- */
int ss_create(const ss_model_cfg* model, const ss_runtime_cfg* rt, ss_ctx** out);
int ss_destroy(ss_ctx* ctx);
const char* ss_last_error(ss_ctx* ctx);   /* valid until the next failing call */

/* Slices the shard's part out of the full layer and keeps a device copy
 * (the pointers may be released on return).  The gains are folded into the
 * matrices that follow the norms (see ss_weights_read). */
int ss_load_layer(ss_ctx*, const ss_shard_desc*, int layer, const ss_layer_weights* full);

/* ---- weight re-sharding (paper section 4.1 "Dynamic Model Re-sharding",
 * Figure 5: at a switch between the prefill strategy and the decode strategy
 * the weights are re-partitioned by reloading the shards the new strategy needs
 * from a copy of the model in CPU memory; section 4.2: that cost does not
 * depend on the batch size; Appendix A.3 for what a shard holds: 1/k of every
 * matrix under tensor parallelism, whole layers under pipeline parallelism) ---
 *
 * ss_host_weights_put: copies the nine full tensors of `layer` (host or device
 *   pointers, released on return) into the library's page-locked CPU copy of
 *   the model, replacing an earlier copy of that layer.
 * ss_reshard_weights(from, to, stream): every layer of `to`'s range receives
 *   the shard's slices of the CPU copy.  Asynchronous: the copies run on the
 *   library's weight stream after everything enqueued on `stream` (device
 *   stream handle or NULL) before the call, and move exactly the shard's bytes
 *   over PCIe (a row range of a matrix is one contiguous copy, a column range
 *   one strided copy; a device kernel then lays the slice out for the GEMMs).
 *   Layer calls on `to` issued later wait for the load on the GPU, the host
 *   does not block.  `from` (may be NULL; ignored when it names the same shard
 *   as `to`, which is then simply reloaded) loses its device weights once the
 *   work enqueued on `stream` before the call has finished: its layer calls
 *   fail with SS_EINVAL until it is loaded again; its KV pages are untouched.
 *   The memory itself returns to the device at the next ss_reshard_weights,
 *   ss_sync or ss_destroy after that point.  SS_ENOENT if a layer of `to` has
 *   no CPU copy.
 * ss_weights_wait: blocks the host until the descriptor's pending load is done.
 * ss_weights_shard_bytes: bytes one (re)load of the descriptor moves (all its
 *   layers: matrices / k plus the two gain vectors), or a negative code.
 * ss_weights_read: inspection (slow): slice `which` (SS_W_*) that the shard
 *   holds for `layer`, in [in_features, out_features] orientation as in
 *   ss_layer_weights but with the shard's columns / rows only, into host_out.
 *   The matrices are returned as the library keeps them: RMSNorm is fused
 *   into the products that follow it (norm(x) W = r (x (g W)) with r the
 *   per-token factor rsqrt(mean(x^2) + eps), applied in the epilogue), so the
 *   rows of wq, wk, wv carry the gains g1 and the rows of wg, wu the gains g2:
 *   element [h, j] is w[h, j] * g[h], formed in fp32 and rounded once to the
 *   model dtype.  g1, g2, wo and wd are kept as given.
 */
enum { SS_W_G1 = 0, SS_W_Q = 1, SS_W_K = 2, SS_W_V = 3, SS_W_O = 4, SS_W_G2 = 5, SS_W_G = 6, SS_W_U = 7, SS_W_D = 8 };
int ss_host_weights_put(ss_ctx*, int layer, const ss_layer_weights* full);
int ss_reshard_weights(ss_ctx*, const ss_shard_desc* from, const ss_shard_desc* to, void* stream);
int ss_weights_wait(ss_ctx*, const ss_shard_desc*);
int64_t ss_weights_shard_bytes(ss_ctx*, const ss_shard_desc*);
int ss_weights_read(ss_ctx*, const ss_shard_desc*, int layer, int which, void* host_out);

/* ---- the layer (paper section 2.1: linear layers around one attention layer;
 * prefill handles all prompt tokens at once, decode one token per sequence
 * against its KV cache) ------------------------------------------------------
 *
 * x_in [T, hidden] device, out [T, hidden] device; out must not alias x_in.
 * T = sum of q_lens (prefill) or n_seqs (decode, every q_len must be 1).
 *
 * phase SS_ATTN: RMSNorm, QKV projection, rotary embedding, K/V written into
 *   the shard's paged cache (pages allocated on demand), causal attention, O
 *   projection.  out = x_in + o when k == 1, else the shard's partial o
 *   WITHOUT residual (the k partials are summed by the caller: that sum is
 *   where tensor parallelism places its first all-reduce, paper Table 3).
 * phase SS_MLP: x_in is the reduced x1.  RMSNorm, gate/up projection, SwiGLU,
 *   down projection.  out = x1 + y when k == 1, else the partial y.
 * phase SS_BOTH: both, k == 1 only.
 * SS_NO_RESIDUAL forces the partial form for k == 1 as well.
 */
int ss_layer_prefill(ss_ctx*, const ss_shard_desc*, int layer, int phase, const ss_batch*,
                     const void* x_in, void* out, void* stream);
int ss_layer_decode(ss_ctx*, const ss_shard_desc*, int layer, int phase, const ss_batch*,
                    const void* x_in, void* out, void* stream);

/* All layers of the descriptor's range, both phases each, chained on the device
 * in one call (what a worker does with its stage of the model, paper section
 * 2.2; for decode this is one step of the stage): layer l reads what layer
 * l - 1 wrote (two library-owned buffers of T x hidden in between), the first
 * layer reads x_in, the last writes out.  k == 1 only (SS_EINVAL otherwise:
 * with k > 1 the partial sums of every layer have to be reduced over the shards
 * between the phases, which one shard cannot do on its own).  The result is the
 * one the same layers give when called one by one with SS_BOTH. */
int ss_layers_prefill(ss_ctx*, const ss_shard_desc*, const ss_batch*, const void* x_in, void* out, void* stream);
int ss_layers_decode(ss_ctx*, const ss_shard_desc*, const ss_batch*, const void* x_in, void* out, void* stream);

/* ---- KV movement (paper section 4.2 "tiered KV cache buffering" and the
 * re-sharding paragraph; section 5.2 two-stage swap-out, asynchronous swap-in,
 * heads-major host layout) ---------------------------------------------------
 *
 * Host tier: per sequence one slot holding the COMPLETE cache of exactly s
 * tokens, element (layer l, c in {0:K,1:V}, kv head g, position p, e) at
 *   ((((l*2 + c)*n_kv + g)*s + p)*head_dim + e
 * elements from the slot's base.  Slots are placed first-fit at the lowest free
 * address and freed blocks merge with their neighbours, so when the last live
 * sequence is released the tier is empty and allocation restarts at 0.
 *
 * ss_kv_swap(SS_OUT): gathers the descriptor's layers/heads of the listed
 *   sequences from its pages into heads-major staging, copies to the pinned
 *   ring (asynchronous DMA on the side stream), then host-copies into the tier
 *   (stage two, on the library's host thread).  Pages stay allocated: release
 *   them with ss_kv_free (which waits for the movements that still read them).  SS_ENOMEM when
 *   the tier is full.
 * ss_kv_swap(SS_IN): allocates pages in the descriptor's pool (in call order,
 *   lowest free id first) and fills them with the descriptor's layers/heads
 *   taken from the tier.  SS_ENOENT if a sequence is not in the tier.
 * Ordering: the side stream first waits for everything enqueued on `stream`
 *   before the call.  Compute that uses swapped-in pages must follow ss_sync().
 * ss_kv_reshard(from, to) = swap-out under `from`, then swap-in under `to`.
 */
int ss_kv_swap(ss_ctx*, const ss_shard_desc*, int dir, const int64_t* seq_ids, int n, void* stream);
int ss_kv_reshard(ss_ctx*, const ss_shard_desc* from, const ss_shard_desc* to,
                  const int64_t* seq_ids, int n, void* stream);
int ss_sync(ss_ctx*);                       /* drains the host thread and the side stream */
/* Completion of individual movements (the notification the asynchronous prefetcher gives the
 * scheduler, paper section 5.2): every ss_kv_swap enqueues one job (ss_kv_reshard two), jobs
 * complete in order.  ss_kv_jobs_issued returns how many were enqueued so far; ss_kv_wait(n)
 * returns once the first n have completed (data visible to later compute on any stream). */
int64_t ss_kv_jobs_issued(ss_ctx*);
int ss_kv_wait(ss_ctx*, int64_t n_jobs);
int ss_kv_free(ss_ctx*, const ss_shard_desc*, const int64_t* seq_ids, int n);  /* pages back to the pool */
int ss_host_tier_release(ss_ctx*, const int64_t* seq_ids, int n);

/* Device-side halves of the movement, without the PCIe leg: staging is a device
 * buffer laid out [seq][layer_local][K|V][head_local][position][head_dim],
 * sequences back to back at exact lengths, model dtype.  Export gathers pages
 * into it; import allocates pages for (seq_ids, lens) and scatters into them.
 * Both run on `stream`. */
int ss_kv_export_dev(ss_ctx*, const ss_shard_desc*, const int64_t* seq_ids, int n, void* staging, void* stream);
int ss_kv_import_dev(ss_ctx*, const ss_shard_desc*, const int64_t* seq_ids, const int32_t* lens, int n,
                     const void* staging, void* stream);

/* ---- inspection (tests) ------------------------------------------------ */
/* pages [*n_inout] receives the page ids of seq; *n_inout returns the count. */
int ss_kv_page_table(ss_ctx*, const ss_shard_desc*, int64_t seq, int32_t* pages, int32_t* n_inout);
int ss_kv_seq_len(ss_ctx*, const ss_shard_desc*, int64_t seq, int32_t* len_out);
/* host_out [2][heads_local][s][head_dim], model dtype; synchronises the device. */
int ss_kv_read(ss_ctx*, const ss_shard_desc*, int64_t seq, int layer, void* host_out);
/* host_out [2][n_kv][s][head_dim] of one layer straight from the tier. */
int ss_host_tier_read(ss_ctx*, int64_t seq, int layer, void* host_out);
int64_t ss_host_tier_used_bytes(ss_ctx*);
int64_t ss_kv_free_pages(ss_ctx*, const ss_shard_desc*);

/* ---- helpers for the tiny whole-model configuration --------------------- */
/* embed [vocab, H], gf [H], wlm [H, vocab]; host pointers, model dtype. */
int ss_load_head(ss_ctx*, const void* embed, const void* gf, const void* wlm);
int ss_embed(ss_ctx*, const int32_t* token_ids_host, int n, void* x_out, void* stream);
/* logits [n, vocab] float32 device = RMSNorm(x; gf) * wlm */
int ss_lm_head(ss_ctx*, const void* x, int n, float* logits, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid it): ss_lm_head with its scratch --
 * the normed rows and the split-K partial sums of the GEMM -- in a fixed 32 MiB
 * device array that every GPU the library runs on holds until the process ends,
 * instead of workspaces that grow on demand.  Same arguments and result as
 * ss_lm_head; calls no hipMalloc / hipFree and no allocating library routine.
 * Limit: n * hidden * (bytes per element) <= 8 MiB (e.g. 512 rows of hidden 8192
 * in a 16-bit type); above it SS_EINVAL with the sizes in ss_last_error, and
 * nothing is launched.  All calls on one GPU (from any context) share that GPU's
 * array: calls that overlap in time on one GPU race; issue them on one stream or
 * order them with events. */
int ss_lm_head_noalloc(ss_ctx*, const void* x, int n, float* logits, void* stream);

/* The shapes the context was created with. */
int ss_get_config(ss_ctx*, ss_model_cfg* model_out, ss_runtime_cfg* rt_out);

/* ---- offline engine loop (paper section 4.2 "Tiered KV Cache Buffering and
 * Transition-minimizing Scheduling", Figure 6; section 5.2 "Asynchronous
 * swap-in") -------------------------------------------------------------------
 *
 * Runs a list of requests to completion on one GPU with greedy decoding,
 * switching between a prefill strategy and a decode strategy only when the
 * CPU store (the host tier) is full, respectively has been emptied onto the
 * GPU.  Host control only: all work is issued through the entry points above.
 * The rules (the paper fixes the triggers; the rest is stated so that the order
 * of actions is unique):
 *   prefill stage: requests in arrival order; a batch takes requests while
 *     the prompt tokens stay within max_prefill_tokens (a longer prompt alone)
 *     and the prompts' pages fit gpu_kv_pages;
 *     every batch's cache is swapped out behind it; the stage ends when the
 *     next prompt does not fit in the store (host_tier_bytes / bytes per token
 *     over all layers) or nothing is left to prefill.  A request that wants one
 *     token is finished by its prefill and never enters the store.
 *   decode stage, per iteration: caches requested in the previous iteration
 *     come on board; while the head of the store fits (pages of its final
 *     length, prompt + outputs - 1 tokens, next to those promised to admitted
 *     sequences within gpu_kv_pages; at most max_decode_seqs admitted; at most
 *     swap_in_group per iteration, 0 = no limit, so that decoding can begin
 *     while the rest of the store is still on its way) its swap-in is requested; every sequence on board gets one token; finished
 *     ones free their pages.  When the store is empty and nothing is arriving:
 *     back to prefilling if requests wait (sequences still decoding keep their
 *     pages and continue in the next decode stage), else on until all are done.
 * Both descriptors must cover all layers with k == 1 (one GPU runs whole
 * layers) and be distinct (one SS_PP, one SS_TP).  With reshard_weights != 0
 * the stage's weights are reloaded from the CPU copy at every switch
 * (ss_reshard_weights; needs ss_host_weights_put for every layer); with 0 both
 * descriptors must already be loaded and stay resident.  Needs ss_load_head.
 *
 * prompt_tokens: the prompts back to back; tokens_out: out_lens[i] tokens per
 * request back to back (token 1 comes from the prefill).  trace (may be NULL):
 * int32 records  code, n, id_0 .. id_{n-1}  with code 1 prefill batch,
 * 2 switch to decode, 3 swap-in requested, 4 decode step, 5 switch to prefill,
 * 6 finished; *trace_len receives the length needed (SS_ENOMEM if above
 * trace_cap).  All pointers are host memory.  SS_ENOMEM if a request can never
 * fit the CPU store or the GPU store. */
typedef struct {
    ss_shard_desc prefill, decode;
    int32_t max_prefill_tokens, max_decode_seqs;
    int32_t reshard_weights;
    int32_t swap_in_group;
} ss_offline_cfg;
typedef struct {
    int64_t prefill_batches, decode_steps, to_decode, to_prefill, tokens;
    double prefill_seconds, decode_seconds, switch_seconds, total_seconds;
} ss_offline_stats;
int ss_offline_run(ss_ctx*, const ss_offline_cfg*, int32_t n_requests, const int32_t* prompt_lens,
                   const int32_t* prompt_tokens, const int32_t* out_lens, int32_t* tokens_out, int32_t* trace,
                   int64_t trace_cap, int64_t* trace_len, ss_offline_stats* stats, void* stream);

/* ---- timing hooks (bench) ------------------------------------------------ */
/* Average duration in ms of the kernels of one class since the last reset,
 * measured with HIP events on the stream they were launched on; enabled with
 * ss_prof_enable(ctx, 1).  cls: 0 GEMM, 1 prefill attention, 2 decode
 * attention, 3 KV gather/scatter, 4 everything else.  Returns the number of
 * launches counted through *n_out. */
int ss_prof_enable(ss_ctx*, int on);
int ss_prof_read(ss_ctx*, int cls, double* total_ms_out, int64_t* n_out);
int ss_prof_reset(ss_ctx*);

#ifdef __cplusplus
}
#endif
#endif
