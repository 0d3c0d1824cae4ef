// Offline engine loop: transition-minimizing scheduling over the tiered KV buffer (paper section 4.2,
// Figure 6) with the asynchronous swap-in of section 5.2, on one GPU.  Host control only: every piece of
// work it issues is one of the library's own entry points (layer calls, KV swaps, weight re-shards), plus
// the token choice (argmax) and the row gather in front of the LM head.
//
// The policy, as deterministic rules (the paper fixes the triggers, the rest is this library's reading):
//   prefill stage   requests in arrival order; a batch takes requests while the prompt tokens stay within
//                   max_prefill_tokens (a longer prompt alone) and the prompts' pages fit the GPU store; the
//                   cache of every batch is swapped out to the CPU store behind the batch; the stage ends when
//                   the next prompt does not fit in the store ("full") or nothing is left to prefill.  A request that wants a single token is
//                   finished by its prefill and never enters the store.
//   decode stage    per iteration: (1) the caches requested in the previous iteration come on board;
//                   (2) while the head of the store fits (pages of its final length next to those promised
//                   to admitted sequences, at most max_decode_seqs admitted, at most swap_in_group per
//                   iteration) its swap-in is requested;
//                   (3) one token for every sequence on board; finished ones leave and free their pages;
//                   (4) when the store is empty and nothing is arriving: back to prefilling if requests are
//                   waiting (sequences still decoding keep their pages and continue in the next decode
//                   stage), else on until all are finished.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdio>
#include <deque>
#include <string>
#include <vector>

#include "../../include/seesaw_rt.h"
#include "ss_kernels.h"
#define SS_DECL_NS ssk16
#include "ss_kernels.h"

namespace {

enum { T_PREFILL = 1, T_TO_DECODE = 2, T_SWAP_IN = 3, T_DECODE = 4, T_TO_PREFILL = 5, T_FINISH = 6 };

double now_s() { return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count(); }

struct Trace {
    int32_t* buf;
    int64_t cap, len = 0;
    bool overflow = false;
    void add(int code, const std::vector<int>& ids) {
        const int64_t need = 2 + (int64_t)ids.size();
        if (!buf || len + need > cap) { overflow = overflow || buf != nullptr; len += need; return; }
        buf[len++] = code;
        buf[len++] = (int32_t)ids.size();
        for (int i : ids) buf[len++] = i;
    }
};

struct Bufs {
    void *x = nullptr, *y = nullptr, *rows = nullptr;
    float* logits = nullptr;
    int32_t *d_idx = nullptr, *d_tok = nullptr, *h_tok = nullptr, *h_idx = nullptr;
    ~Bufs() {
        for (void* p : {x, y, rows, (void*)logits, (void*)d_idx, (void*)d_tok}) if (p) (void)hipFree(p);
        if (h_tok) (void)hipHostFree(h_tok);
        if (h_idx) (void)hipHostFree(h_idx);
    }
};

}  // namespace

extern "C" int ss_offline_set_error(ss_ctx*, const char*);   // ss_runtime.hip: text for ss_last_error

#define OFF_FAIL(code, ...)                                         \
    do {                                                            \
        char _b[384];                                               \
        snprintf(_b, sizeof _b, __VA_ARGS__);                       \
        ss_offline_set_error(c, _b);                                \
        return (code);                                              \
    } while (0)
#define OFF_HIP(expr)                                                                            \
    do {                                                                                         \
        hipError_t _e = (expr);                                                                  \
        if (_e != hipSuccess) OFF_FAIL(SS_EHIP, "offline loop: %s: %s", #expr, hipGetErrorString(_e)); \
    } while (0)
#define OFF_TRY(expr)                  \
    do {                               \
        int _rc = (expr);              \
        if (_rc != SS_OK) return _rc;  \
    } while (0)

extern "C" int ss_offline_run(ss_ctx* c, const ss_offline_cfg* cfg, int32_t n, const int32_t* prompt_lens,
                              const int32_t* prompt_tokens, const int32_t* out_lens, int32_t* tokens_out, int32_t* trace_buf,
                              int64_t trace_cap, int64_t* trace_len, ss_offline_stats* stats, void* stream) {
    if (!c) return SS_EINVAL;
    if (!cfg || n < 0 || (n > 0 && (!prompt_lens || !prompt_tokens || !out_lens || !tokens_out)))
        OFF_FAIL(SS_EINVAL, "offline loop: null argument");
    ss_model_cfg m;
    ss_runtime_cfg rt;
    OFF_TRY(ss_get_config(c, &m, &rt));
    const ss_shard_desc P = cfg->prefill, D = cfg->decode;
    for (const ss_shard_desc* d : {&P, &D}) {
        const int k = d->mode == SS_TP ? d->k : 1;
        if (k != 1 || d->layer_begin != 0 || d->layer_end != m.n_layers)
            OFF_FAIL(SS_EINVAL, "offline loop: one GPU runs whole layers: both strategies need k == 1 over all layers");
    }
    if (P.mode == D.mode) OFF_FAIL(SS_EINVAL, "offline loop: the two strategies must be distinct descriptors");
    if (cfg->max_prefill_tokens < 1 || cfg->max_decode_seqs < 1) OFF_FAIL(SS_EINVAL, "offline loop: bad batch limits");
    if (m.vocab < 1) OFF_FAIL(SS_EINVAL, "offline loop: the model has no vocabulary (ss_load_head)");
    hipStream_t st = (hipStream_t)stream;
    const int ps = m.page_size;
    const size_t es = m.dtype == SS_F32 ? 4 : 2;
    const int64_t tok_bytes = (int64_t)2 * m.n_kv_heads * m.head_dim * (int64_t)es * m.n_layers;
    const int64_t tier_tokens = rt.host_tier_bytes / tok_bytes;
    const int64_t gpu_pages = rt.gpu_kv_pages;
    auto pages_of = [&](int64_t tokens) { return (tokens + ps - 1) / ps; };
    auto final_pages = [&](int r) { return pages_of((int64_t)prompt_lens[r] + out_lens[r] - 1); };
    std::vector<int64_t> p_off(n + 1, 0), o_off(n + 1, 0);
    int longest = 1;
    for (int i = 0; i < n; ++i) {
        if (prompt_lens[i] < 1 || out_lens[i] < 1) OFF_FAIL(SS_EINVAL, "offline loop: request %d has a non-positive length", i);
        if (prompt_lens[i] + out_lens[i] - 1 > rt.max_seq_len) OFF_FAIL(SS_EINVAL, "offline loop: request %d exceeds max_seq_len", i);
        if (out_lens[i] > 1 && prompt_lens[i] > tier_tokens) OFF_FAIL(SS_ENOMEM, "offline loop: request %d does not fit the CPU store", i);
        if (out_lens[i] > 1 && final_pages(i) > gpu_pages) OFF_FAIL(SS_ENOMEM, "offline loop: request %d does not fit the GPU store", i);
        if (pages_of(prompt_lens[i]) > gpu_pages) OFF_FAIL(SS_ENOMEM, "offline loop: prompt %d does not fit the GPU store", i);
        p_off[i + 1] = p_off[i] + prompt_lens[i];
        o_off[i + 1] = o_off[i] + out_lens[i];
        longest = std::max(longest, prompt_lens[i]);
    }
    const int max_T = std::max(std::max(cfg->max_prefill_tokens, longest), cfg->max_decode_seqs);
    const int max_rows = std::max(cfg->max_decode_seqs, std::min(n, max_T));
    Bufs b;
    OFF_HIP(hipMalloc(&b.x, (size_t)max_T * m.hidden * es));
    OFF_HIP(hipMalloc(&b.y, (size_t)max_T * m.hidden * es));
    OFF_HIP(hipMalloc(&b.rows, (size_t)max_rows * m.hidden * es));
    OFF_HIP(hipMalloc((void**)&b.logits, (size_t)max_rows * m.vocab * sizeof(float)));
    OFF_HIP(hipMalloc((void**)&b.d_idx, (size_t)max_rows * sizeof(int32_t)));
    OFF_HIP(hipMalloc((void**)&b.d_tok, (size_t)max_rows * sizeof(int32_t)));
    OFF_HIP(hipHostMalloc((void**)&b.h_tok, (size_t)max_rows * sizeof(int32_t), hipHostMallocDefault));
    OFF_HIP(hipHostMalloc((void**)&b.h_idx, (size_t)max_rows * sizeof(int32_t), hipHostMallocDefault));

    Trace tr{trace_buf, trace_cap};
    ss_offline_stats s{};
    const double t_start = now_s();
    std::vector<int> produced(n, 0), last_tok(n, 0);
    std::deque<int> waiting, store;
    for (int i = 0; i < n; ++i) waiting.push_back(i);
    std::vector<int> running, arriving;
    int64_t arriving_job = 0;
    int64_t store_used = 0, promised = 0;

    // the whole model on `ids` (tokens concatenated): embed, every layer, final norm + LM head on the
    // rows listed in h_idx, argmax; the chosen tokens land in h_tok
    auto forward = [&](const ss_shard_desc& d, const std::vector<int>& ids, const std::vector<int32_t>& toks,
                       const std::vector<int32_t>& q_lens, const std::vector<int32_t>& before, bool decode) -> int {
        const int T = (int)toks.size(), nb = (int)ids.size();
        std::vector<int64_t> sid(ids.begin(), ids.end());
        ss_batch bt{nb, sid.data(), q_lens.data(), before.data()};
        OFF_TRY(ss_embed(c, toks.data(), T, b.x, st));
        void *in = b.x, *out = b.y;
        for (int l = 0; l < m.n_layers; ++l) {
            if (decode) OFF_TRY(ss_layer_decode(c, &d, l, SS_BOTH, &bt, in, out, st));
            else OFF_TRY(ss_layer_prefill(c, &d, l, SS_BOTH, &bt, in, out, st));
            std::swap(in, out);
        }
        const void* rows = in;
        if (!decode) {                       // the last token of every prompt
            int t = 0;
            for (int i = 0; i < nb; ++i) { t += q_lens[i]; b.h_idx[i] = t - 1; }
            OFF_HIP(hipMemcpyAsync(b.d_idx, b.h_idx, (size_t)nb * sizeof(int32_t), hipMemcpyHostToDevice, st));
            hipError_t e = m.dtype == SS_F16 ? ssk16::embed_rows(ssk::BF16, in, b.d_idx, b.rows, nb, m.hidden, st)
                                             : ssk::embed_rows(m.dtype, in, b.d_idx, b.rows, nb, m.hidden, st);
            if (e != hipSuccess) OFF_FAIL(SS_EHIP, "offline loop: row gather: %s", hipGetErrorString(e));
            rows = b.rows;
        }
        OFF_TRY(ss_lm_head(c, rows, nb, b.logits, st));
        hipError_t e = ssk::argmax_rows(b.logits, nb, m.vocab, b.d_tok, st);
        if (e != hipSuccess) OFF_FAIL(SS_EHIP, "offline loop: argmax: %s", hipGetErrorString(e));
        OFF_HIP(hipMemcpyAsync(b.h_tok, b.d_tok, (size_t)nb * sizeof(int32_t), hipMemcpyDeviceToHost, st));
        OFF_HIP(hipStreamSynchronize(st));
        return SS_OK;
    };
    auto emit = [&](int r, int tok) {
        tokens_out[o_off[r] + produced[r]] = tok;
        produced[r]++;
        last_tok[r] = tok;
        s.tokens++;
    };
    auto free_ids = [&](const ss_shard_desc& d, const std::vector<int>& ids) -> int {
        if (ids.empty()) return SS_OK;
        std::vector<int64_t> sid(ids.begin(), ids.end());
        return ss_kv_free(c, &d, sid.data(), (int)sid.size());
    };

    if (cfg->reshard_weights) OFF_TRY(ss_reshard_weights(c, nullptr, &P, st));
    std::deque<std::vector<int>> out_batches;      // prefill batches whose pages are still allocated
    while (!waiting.empty() || !store.empty() || !running.empty() || !arriving.empty()) {
        // ------------------------------------------------------------ prefill stage
        double t0 = now_s();
        bool full = false;
        while (!waiting.empty() && !full) {
            std::vector<int> batch;
            int64_t tokens = 0, need_pages = 0;
            while (!waiting.empty()) {
                const int r = waiting.front();
                const int64_t need = out_lens[r] > 1 ? prompt_lens[r] : 0;
                if (store_used + need > tier_tokens) { full = true; break; }
                if (!batch.empty() && tokens + prompt_lens[r] > cfg->max_prefill_tokens) break;
                if (!batch.empty() && need_pages + pages_of(prompt_lens[r]) > gpu_pages) break;
                waiting.pop_front();
                batch.push_back(r);
                tokens += prompt_lens[r];
                need_pages += pages_of(prompt_lens[r]);
                store_used += need;
            }
            if (batch.empty()) break;
            // pages for the batch: earlier batches give theirs back once their swap-out has read them
            while (!out_batches.empty() && ss_kv_free_pages(c, &P) < need_pages) {
                OFF_TRY(free_ids(P, out_batches.front()));
                out_batches.pop_front();
            }
            tr.add(T_PREFILL, batch);
            s.prefill_batches++;
            std::vector<int32_t> toks, q_lens, before;
            for (int r : batch) {
                toks.insert(toks.end(), prompt_tokens + p_off[r], prompt_tokens + p_off[r + 1]);
                q_lens.push_back(prompt_lens[r]);
                before.push_back(0);
            }
            OFF_TRY(forward(P, batch, toks, q_lens, before, false));
            std::vector<int> done, keep;
            for (size_t i = 0; i < batch.size(); ++i) {
                emit(batch[i], b.h_tok[i]);
                (out_lens[batch[i]] == 1 ? done : keep).push_back(batch[i]);
            }
            if (!keep.empty()) {
                std::vector<int64_t> sid(keep.begin(), keep.end());
                OFF_TRY(ss_kv_swap(c, &P, SS_OUT, sid.data(), (int)sid.size(), st));
                for (int r : keep) store.push_back(r);
            }
            out_batches.push_back(batch);
            if (!done.empty()) tr.add(T_FINISH, done);
        }
        s.prefill_seconds += now_s() - t0;
        if (store.empty() && running.empty() && arriving.empty()) continue;
        // ------------------------------------------------------------ switch to the decode strategy
        t0 = now_s();
        tr.add(T_TO_DECODE, {});
        s.to_decode++;
        while (!out_batches.empty()) {          // the prefill pool is empty while decoding
            OFF_TRY(free_ids(P, out_batches.front()));
            out_batches.pop_front();
        }
        if (cfg->reshard_weights) OFF_TRY(ss_reshard_weights(c, &P, &D, st));
        s.switch_seconds += now_s() - t0;
        // ------------------------------------------------------------ decode stage
        t0 = now_s();
        for (;;) {
            if (!arriving.empty()) {             // the prefetcher's notification
                OFF_TRY(ss_kv_wait(c, arriving_job));
                std::vector<int64_t> sid(arriving.begin(), arriving.end());
                OFF_TRY(ss_host_tier_release(c, sid.data(), (int)sid.size()));
                for (int r : arriving) { running.push_back(r); store_used -= prompt_lens[r]; }
                arriving.clear();
            }
            std::vector<int> asked;
            while (!store.empty() && promised + final_pages(store.front()) <= gpu_pages &&
                   (int)(running.size() + asked.size()) < cfg->max_decode_seqs &&
                   (cfg->swap_in_group <= 0 || (int)asked.size() < cfg->swap_in_group)) {
                const int r = store.front();
                store.pop_front();
                promised += final_pages(r);
                asked.push_back(r);
            }
            if (!asked.empty()) {
                tr.add(T_SWAP_IN, asked);
                std::vector<int64_t> sid(asked.begin(), asked.end());
                OFF_TRY(ss_kv_swap(c, &D, SS_IN, sid.data(), (int)sid.size(), st));
                arriving_job = ss_kv_jobs_issued(c);
                arriving = asked;
            }
            const bool stepped = !running.empty();
            if (stepped) {
                tr.add(T_DECODE, running);
                s.decode_steps++;
                std::vector<int32_t> toks, q_lens, before;
                for (int r : running) {
                    toks.push_back(last_tok[r]);
                    q_lens.push_back(1);
                    before.push_back(prompt_lens[r] + produced[r] - 1);
                }
                OFF_TRY(forward(D, running, toks, q_lens, before, true));
                std::vector<int> done, keep;
                for (size_t i = 0; i < running.size(); ++i) {
                    const int r = running[i];
                    emit(r, b.h_tok[i]);
                    (produced[r] == out_lens[r] ? done : keep).push_back(r);
                }
                if (!done.empty()) {
                    tr.add(T_FINISH, done);
                    OFF_TRY(free_ids(D, done));
                    for (int r : done) promised -= final_pages(r);
                    running = keep;
                }
            }
            if (store.empty() && arriving.empty()) {
                if (!waiting.empty()) {
                    tr.add(T_TO_PREFILL, {});
                    s.to_prefill++;
                    break;
                }
                if (running.empty()) break;
            } else if (!stepped && asked.empty()) {
                OFF_FAIL(SS_EINVAL, "offline loop: no progress (the head of the CPU store cannot be admitted)");
            }
        }
        s.decode_seconds += now_s() - t0;
        if (!waiting.empty() && cfg->reshard_weights) {
            t0 = now_s();
            OFF_TRY(ss_reshard_weights(c, &D, &P, st));
            s.switch_seconds += now_s() - t0;
        }
    }
    while (!out_batches.empty()) {
        OFF_TRY(free_ids(P, out_batches.front()));
        out_batches.pop_front();
    }
    OFF_TRY(ss_sync(c));
    s.total_seconds = now_s() - t_start;
    if (stats) *stats = s;
    if (trace_len) *trace_len = tr.len;
    if (tr.overflow) OFF_FAIL(SS_ENOMEM, "offline loop: trace buffer too small (%lld entries needed)", (long long)tr.len);
    return SS_OK;
}
