// Host runtime behind the C ABI of include/seesaw_rt.h: shard state (sliced
// weights, page pools, page tables), the layer pipelines, the host tier, and the
// asynchronous KV mover (side stream + host thread + pinned two-slot ring).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <functional>
#include <map>
#include <mutex>
#include <queue>
#include <string>
#include <thread>
#include <unordered_map>
#include <vector>

#include <hsa/hsa.h>
#include <hsa/hsa_ext_amd.h>

#include "../../include/seesaw_rt.h"
#include "ss_kernels.h"
#define SS_DECL_NS ssk16
#include "ss_kernels.h"

// The kernel files exist twice: built for brain-float (namespace ssk; also serves fp32 models) and for IEEE
// half (namespace ssk16, where the 16-bit dtype code means half).  Every launcher takes the dtype first.
#define SSK_CALL(c, fn, ...) \
    ((c)->dt == SS_F16 ? ssk16::fn(ssk::BF16, __VA_ARGS__) : ssk::fn((c)->dt, __VA_ARGS__))

namespace {

struct DevBuf {
    void* p = nullptr;
    size_t cap = 0;
};

struct LayerW {
    void *g1 = nullptr, *g2 = nullptr, *wqkv_t = nullptr, *wo_t = nullptr, *wgu_t = nullptr, *wd_t = nullptr;
    bool loaded = false;
    bool gu_interleaved = false;
};

// CPU copy of one layer's full weights (page-locked): the nine tensors in the order of
// ss_layer_weights, [in_features, out_features] orientation, at byte offsets off[i] from base.
struct HostLayer {
    uint8_t* base = nullptr;
    size_t off[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
};

// Device buffers whose release waits for the work that may still read them.
struct DeferredFree {
    hipEvent_t ev = nullptr;
    std::vector<void*> ptrs;
};

struct SeqState {
    std::vector<int32_t> pages;
    int32_t len = 0;
};

struct Shard {
    ss_shard_desc desc{};
    int nq_l = 0, nkv_l = 0, f_l = 0, q0 = 0, g0 = 0, f0 = 0, n_layers_l = 0;
    std::vector<LayerW> w;
    std::vector<void*> k_pool, v_pool;
    void** d_k_pools = nullptr;
    void** d_v_pools = nullptr;
    bool pools_ready = false;
    std::priority_queue<int32_t, std::vector<int32_t>, std::greater<int32_t>> free_pages;
    std::unordered_map<int64_t, SeqState> seqs;
    uint64_t version = 0;     // bumped on every page-table change
    hipEvent_t w_ready = nullptr;   // recorded on the weight stream behind the shard's last (re)load
    bool w_pending = false;         // ... which layer calls still have to wait for
};

struct DescKey {
    int32_t v[5];
    bool operator<(const DescKey& o) const { return std::lexicographical_compare(v, v + 5, o.v, o.v + 5); }
};

// One slot of batch metadata: pinned host image + device copy + "last use" event.
struct MetaSlot {
    uint8_t* host = nullptr;
    uint8_t* dev = nullptr;
    size_t cap = 0;
    hipEvent_t done = nullptr;
    bool in_flight = false;
    // cache key
    Shard* shard = nullptr;
    uint64_t version = 0;
    bool decode = false;
    std::vector<int64_t> seq_ids;
    std::vector<int32_t> q_lens, kv_before;
    ssk::BatchMeta bm{};
    ssk::DecodeWork wk{};
};

struct SeqJob {
    int64_t seq;
    int32_t len;
    std::vector<int32_t> pages;
    size_t tier_off;   // bytes
};

struct Job {
    int dir;
    Shard* sh;
    std::vector<SeqJob> seqs;
    hipEvent_t after = nullptr;
    int64_t id = 0;            // 1-based issue order over both lanes
    int64_t needs_out = 0;     // swap-in: number of swap-out jobs that must have completed first
};

// Device-to-host copies on the DMA engines, issued through the HSA runtime.  The HIP runtime that a process gets
// when PyTorch is loaded first (the 7.0 runtime bundled with the wheel) executes hipMemcpyAsync from device memory
// into page-locked host memory as a copy kernel on the compute units (`__amd_rocclr_copyBuffer` in a kernel trace:
// no device-to-host entry in the memory-copy trace), while the same call under the system's 7.2 runtime goes to a
// DMA engine; host-to-device copies use the engines under both.  A copy kernel needs compute units, which the
// persistent GEMM blocks hold, so the swap-out both slowed the layer down and waited for it.
// hsa_amd_memory_async_copy addresses the engines directly and works the same under either runtime: both are
// the process's one HSA runtime (same library, reference-counted hsa_init), and the buffers HIP allocated
// (hipMalloc, hipHostMalloc) are HSA allocations that the agents already may access.
struct HsaCopy {
    bool ok = false;
    hsa_agent_t gpu{}, cpu{};
    hsa_signal_t done{};
    static hsa_status_t pick(hsa_agent_t a, void* data) {
        HsaCopy* h = (HsaCopy*)data;
        hsa_device_type_t t;
        if (hsa_agent_get_info(a, HSA_AGENT_INFO_DEVICE, &t) != HSA_STATUS_SUCCESS) return HSA_STATUS_SUCCESS;
        if (t == HSA_DEVICE_TYPE_CPU && !h->cpu.handle) h->cpu = a;
        if (t == HSA_DEVICE_TYPE_GPU) {
            uint32_t bdf = 0;
            if (hsa_agent_get_info(a, (hsa_agent_info_t)HSA_AMD_AGENT_INFO_BDFID, &bdf) != HSA_STATUS_SUCCESS) return HSA_STATUS_SUCCESS;
            if ((int)((bdf >> 8) & 0xff) == h->want_bus && (int)((bdf >> 3) & 0x1f) == h->want_dev) h->gpu = a;
        }
        return HSA_STATUS_SUCCESS;
    }
    int want_bus = -1, want_dev = -1;
    // finds the HSA agents of HIP device `device` (matched by PCI bus and device number) and of the host
    void init(int device) {
        const char* e = getenv("SS_HSA_COPY");
        if (e && e[0] == '0') return;
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, device) != hipSuccess) { (void)hipGetLastError(); return; }
        want_bus = prop.pciBusID;
        want_dev = prop.pciDeviceID;
        if (hsa_init() != HSA_STATUS_SUCCESS) return;
        if (hsa_iterate_agents(pick, this) != HSA_STATUS_SUCCESS || !gpu.handle || !cpu.handle) { (void)hsa_shut_down(); return; }
        if (hsa_signal_create(0, 0, nullptr, &done) != HSA_STATUS_SUCCESS) { (void)hsa_shut_down(); return; }
        // An engine of its own for this direction.  Left to the HSA runtime, these copies and the host-to-device
        // copies of the swap-in (issued by the HIP runtime) queue up on the same engines and the two PCIe
        // directions take turns; and not every engine the runtime lists reaches the host link at full rate
        // (measured on the pipelined step of the 7B-shape layer, ms per step: engines 0 / 1 / 2 / 3: 13.9 / 12.0 /
        // 9.0 / 9.0, runtime's choice 12.0, engines 4 and above 26 - 47).  So every listed engine copies 16 MB once,
        // and of those within 10 % of the fastest the highest-numbered one is taken (the HIP runtime starts from
        // the lowest).  SS_HSA_ENGINE = bit index overrides, -1 leaves the choice to the HSA runtime.
        uint32_t st_out = 0;
        (void)hsa_amd_memory_copy_engine_status(cpu, gpu, &st_out);
        int bit = -1;
        if (const char* eb = getenv("SS_HSA_ENGINE")) {
            bit = atoi(eb);
        } else {
            const size_t probe = (size_t)16 << 20;
            void *d = nullptr, *h = nullptr;
            if (hipMalloc(&d, probe) == hipSuccess && hipHostMalloc(&h, probe, hipHostMallocDefault) == hipSuccess &&
                hipMemset(d, 0, probe) == hipSuccess && hipDeviceSynchronize() == hipSuccess) {
                double best = 1e30, t[16];
                for (int b = 0; b < 16; ++b) {
                    t[b] = 1e30;
                    if (!(st_out & (1u << b))) continue;
                    for (int rep = 0; rep < 2; ++rep) {                  // the first copy on an engine sets it up
                        hsa_signal_store_relaxed(done, 1);
                        const auto t0 = std::chrono::steady_clock::now();
                        if (hsa_amd_memory_async_copy_on_engine(h, cpu, d, gpu, probe, 0, nullptr, done,
                                                                (hsa_amd_sdma_engine_id_t)(1u << b), false) != HSA_STATUS_SUCCESS) break;
                        if (hsa_signal_wait_scacquire(done, HSA_SIGNAL_CONDITION_LT, 1, 2000000000ull, HSA_WAIT_STATE_BLOCKED) != 0) break;
                        if (rep) t[b] = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
                    }
                    best = std::min(best, t[b]);
                }
                for (int b = 0; b < 16; ++b)
                    if (t[b] <= 1.1 * best) bit = b;
            }
            (void)hipGetLastError();
            if (d) (void)hipFree(d);
            if (h) (void)hipHostFree(h);
        }
        engine = bit >= 0 && bit < 16 ? (1u << bit) : 0;
        if (getenv("SS_TRACE_MOVER"))
            fprintf(stderr, "[mover] DMA engines listed for device->host: 0x%x; using 0x%x\n", st_out, engine);
        ok = true;
    }
    uint32_t engine = 0;                 // hsa_amd_sdma_engine_id_t of the device -> host copies, 0 = the runtime's choice
    void shutdown() {
        if (!ok) return;
        (void)hsa_signal_destroy(done);
        (void)hsa_shut_down();
        ok = false;
    }
    struct Run { void* host; const void* dev; size_t bytes; };
    // all runs device -> host, then waits for them; false on any error (the caller falls back to hipMemcpyAsync)
    bool copy_out(const std::vector<Run>& runs) {
        if (!ok) return false;
        if (runs.empty()) return true;
        hsa_signal_store_relaxed(done, (hsa_signal_value_t)runs.size());
        size_t issued = 0;
        for (const Run& r : runs) {
            const hsa_status_t st = engine
                ? hsa_amd_memory_async_copy_on_engine(r.host, cpu, r.dev, gpu, r.bytes, 0, nullptr, done, (hsa_amd_sdma_engine_id_t)engine, false)
                : hsa_amd_memory_async_copy(r.host, cpu, r.dev, gpu, r.bytes, 0, nullptr, done);
            if (st != HSA_STATUS_SUCCESS) break;
            ++issued;
        }
        if (issued < runs.size())       // account for the copies that were never issued, then drain the others
            hsa_signal_add_relaxed(done, -(hsa_signal_value_t)(runs.size() - issued));
        hsa_signal_value_t v;
        do {
            v = hsa_signal_wait_scacquire(done, HSA_SIGNAL_CONDITION_LT, 1, UINT64_MAX, HSA_WAIT_STATE_BLOCKED);
        } while (v > 0);
        return issued == runs.size() && v == 0;
    }
};

// One mover lane: a host thread, a side stream, a two-slot pinned ring with its
// device staging twin, and a metadata region.  Lane 0 carries swap-outs, lane 1
// swap-ins, so that the two PCIe directions (and their host copies) overlap.
struct Lane {
    hipStream_t side = nullptr;
    hipStream_t copy = nullptr;                  // the swap-out's device-to-host copies (when the HSA path is off)
    HsaCopy hsa;                                 // the swap-out's device-to-host copies on the DMA engines
    hipEvent_t copy_ev[2] = {nullptr, nullptr};
    uint8_t* pinned = nullptr;
    uint8_t* dev_staging = nullptr;
    size_t dev_cap = 0;                          // bytes of dev_staging
    uint8_t* mv_meta_host = nullptr;
    uint8_t* mv_meta_dev = nullptr;
    hipEvent_t mv_ev[2] = {nullptr, nullptr};
    std::thread worker;
    std::deque<Job> jobs;
    bool busy = false;
    const Job* running = nullptr;
};

struct TierSlot {
    size_t off;     // bytes
    int32_t len;    // tokens
};

struct ProfRec {
    int cls;
    hipEvent_t a, b;
};

// Fixed scratch of the entry point that allocates nothing (ss_lm_head_noalloc): the normed rows and the
// split-K partial sums of its GEMM.  One copy per GPU the library runs on, held until the process ends.  In
// host code the array's name is only a handle for hipGetSymbolAddress: the device address of each GPU's copy
// is looked up once per device (ss_create) and kept in g_noalloc_scratch; kernels and copies get that pointer.
constexpr size_t NOALLOC_SCRATCH_BYTES = (size_t)32 << 20;
constexpr size_t NOALLOC_ROWS_BYTES = (size_t)8 << 20;        // first part: normed rows; the rest: partial sums
constexpr int NOALLOC_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];
void* g_noalloc_scratch[NOALLOC_MAX_DEVICES] = {};
std::mutex g_noalloc_mu;

}  // namespace

struct ss_ctx {
    ss_model_cfg m{};
    ss_runtime_cfg rt{};
    int dt = 0;
    size_t es = 2;
    bool force_generic = false;
    int gemm_rounds_busy = 8;                    // GEMM launch granularity while mover jobs are pending
    int gemm_rounds_idle = 8;                    // ... and while none are: the blocks of a long persistent launch drift
                                                 // apart and lose the sharing of operand slices in L2; a launch
                                                 // boundary every few tiles brings them back in step (70B-shape
                                                 // GEMMs: 0.52 of the MFMA peak in one launch, 0.547 in launches of 8,
                                                 // 16 or 32 tiles per block; shorter GEMMs are not affected)
    int gemm_rounds = 0;                         // ... of the layer call in progress (0 = one launch)
    int copy_threads = 4;
    int n_cus = 256;                             // compute units of the device (blocks of the persistent kernels)
    size_t copy_max_bytes = (size_t)8 << 20;      // adjacent runs of the direct tier path are merged up to this size
    bool trace_mover = false;
    std::string err;
    std::map<DescKey, Shard*> shards;
    float* d_rope = nullptr;
    DevBuf ws_h, ws_qkv, ws_attn, ws_gu, ws_act, ws_x1, ws_scratch, ws_splitk, ws_rs, ws_chain[2];
    MetaSlot meta[4];
    int meta_next = 0;
    void *d_embed = nullptr, *d_gf = nullptr, *d_wlm_t = nullptr;
    int32_t* d_ids = nullptr;
    size_t d_ids_cap = 0;
    // host tier
    uint8_t* tier = nullptr;
    bool tier_pinned = false;                    // page-locked: the DMA engines address it directly
    size_t tier_cap = 0, tier_used = 0;
    std::map<size_t, size_t> tier_free;          // offset -> length of every free block (coalesced)
    std::unordered_map<int64_t, TierSlot> tier_slots;
    // mover
    Lane lane[2];
    size_t slot_bytes = 0;             // per lane: two slots of this size
    size_t mv_meta_cap = 0;            // per lane
    std::mutex mu;                     // guards the lanes' queues and the counters below
    std::condition_variable cv, cv_idle;
    bool stop = false;
    int64_t jobs_issued = 0, jobs_done = 0;      // jobs_done: all jobs with id <= jobs_done completed
    std::vector<int64_t> done_ids;               // completed out of order, above jobs_done
    int64_t out_issued = 0, out_done = 0;
    std::string worker_err;
    int worker_rc = 0;
    // weight re-sharding: CPU copy of the model, the stream its reloads run on, their staging
    std::vector<HostLayer> hw;
    hipStream_t wstream = nullptr;
    DevBuf w_staging;
    std::vector<DeferredFree> deferred;
    // profiling
    bool prof_on = false;
    std::vector<ProfRec> prof;
    std::mutex prof_mu;
};

namespace {

// The mover thread reports into its own string (read by ss_sync); everything
// else reports into the context's.
thread_local std::string* tl_err = nullptr;

int fail(ss_ctx* c, int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (tl_err) *tl_err = buf;
    else if (c) c->err = buf;
    return code;
}

#define HIP_TRY(c, expr)                                                                        \
    do {                                                                                        \
        hipError_t e_ = (expr);                                                                 \
        if (e_ != hipSuccess)                                                                   \
            return fail((c), e_ == hipErrorOutOfMemory ? SS_ENOMEM : SS_EHIP, "%s: %s (%s:%d)", #expr, \
                        hipGetErrorString(e_), __FILE__, __LINE__);                             \
    } while (0)

struct ProfScope {
    ss_ctx* c;
    int cls;
    hipStream_t s;
    hipEvent_t a = nullptr, b = nullptr;
    ProfScope(ss_ctx* c_, int cls_, hipStream_t s_) : c(c_), cls(cls_), s(s_) {
        if (c->prof_on) {
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { a = b = nullptr; return; }
            (void)hipEventRecord(a, s);
        }
    }
    ~ProfScope() {
        if (a && b) {
            (void)hipEventRecord(b, s);
            std::lock_guard<std::mutex> lk(c->prof_mu);
            c->prof.push_back({cls, a, b});
        }
    }
};

int ensure_buf(ss_ctx* c, DevBuf& b, size_t bytes) {
    if (bytes <= b.cap) return SS_OK;
    if (b.p) {
        HIP_TRY(c, hipDeviceSynchronize());
        HIP_TRY(c, hipFree(b.p));
        b.p = nullptr;
        b.cap = 0;
    }
    size_t want = bytes + bytes / 8 + 256;
    HIP_TRY(c, hipMalloc(&b.p, want));
    b.cap = want;
    return SS_OK;
}

int check_desc(ss_ctx* c, const ss_shard_desc* d) {
    if (!d) return fail(c, SS_EINVAL, "null shard descriptor");
    const ss_model_cfg& m = c->m;
    if (d->mode != SS_PP && d->mode != SS_TP) return fail(c, SS_EINVAL, "bad shard mode %d", d->mode);
    if (d->k < 1) return fail(c, SS_EINVAL, "shard degree k=%d < 1", d->k);
    if (d->layer_begin < 0 || d->layer_end > m.n_layers || d->layer_begin >= d->layer_end)
        return fail(c, SS_EINVAL, "bad layer range [%d,%d) of %d", d->layer_begin, d->layer_end, m.n_layers);
    if (d->mode == SS_TP) {
        if (d->shard < 0 || d->shard >= d->k) return fail(c, SS_EINVAL, "shard %d outside [0,%d)", d->shard, d->k);
        if (d->k > m.n_kv_heads) return fail(c, SS_EINVAL, "k=%d exceeds n_kv_heads=%d", d->k, m.n_kv_heads);
        if (m.n_q_heads % d->k || m.n_kv_heads % d->k || m.ffn % d->k)
            return fail(c, SS_EINVAL, "k=%d must divide n_q_heads, n_kv_heads and ffn", d->k);
    }
    return SS_OK;
}

int get_shard(ss_ctx* c, const ss_shard_desc* d, Shard** out) {
    int rc = check_desc(c, d);
    if (rc) return rc;
    DescKey key;
    key.v[0] = d->mode;
    key.v[1] = d->mode == SS_TP ? d->k : 1;
    key.v[2] = d->mode == SS_TP ? d->shard : 0;
    key.v[3] = d->layer_begin;
    key.v[4] = d->layer_end;
    auto it = c->shards.find(key);
    if (it != c->shards.end()) { *out = it->second; return SS_OK; }
    Shard* s = new Shard();
    s->desc = *d;
    const int k = key.v[1], i = key.v[2];
    s->nq_l = c->m.n_q_heads / k;
    s->nkv_l = c->m.n_kv_heads / k;
    s->f_l = c->m.ffn / k;
    s->q0 = i * s->nq_l;
    s->g0 = i * s->nkv_l;
    s->f0 = i * s->f_l;
    s->n_layers_l = d->layer_end - d->layer_begin;
    s->w.resize(s->n_layers_l);
    c->shards[key] = s;
    *out = s;
    return SS_OK;
}

size_t page_bytes(ss_ctx* c, Shard* s) { return (size_t)s->nkv_l * c->m.page_size * c->m.head_dim * c->es; }

int ensure_pools(ss_ctx* c, Shard* s) {
    if (s->pools_ready) return SS_OK;
    const size_t bytes = page_bytes(c, s) * (size_t)c->rt.gpu_kv_pages;
    s->k_pool.assign(s->n_layers_l, nullptr);
    s->v_pool.assign(s->n_layers_l, nullptr);
    for (int l = 0; l < s->n_layers_l; ++l) {
        HIP_TRY(c, hipMalloc(&s->k_pool[l], bytes));
        HIP_TRY(c, hipMalloc(&s->v_pool[l], bytes));
        // finite contents everywhere: masked slots are multiplied by exact zeros
        HIP_TRY(c, hipMemset(s->k_pool[l], 0, bytes));
        HIP_TRY(c, hipMemset(s->v_pool[l], 0, bytes));
    }
    HIP_TRY(c, hipMalloc((void**)&s->d_k_pools, sizeof(void*) * s->n_layers_l));
    HIP_TRY(c, hipMalloc((void**)&s->d_v_pools, sizeof(void*) * s->n_layers_l));
    HIP_TRY(c, hipMemcpy(s->d_k_pools, s->k_pool.data(), sizeof(void*) * s->n_layers_l, hipMemcpyHostToDevice));
    HIP_TRY(c, hipMemcpy(s->d_v_pools, s->v_pool.data(), sizeof(void*) * s->n_layers_l, hipMemcpyHostToDevice));
    for (int64_t p = 0; p < c->rt.gpu_kv_pages; ++p) s->free_pages.push((int32_t)p);
    s->pools_ready = true;
    return SS_OK;
}

// Grow a sequence's page list to cover `length` tokens: lowest free id first.
// A sequence the shard does not know yet is entered only once its pages are certain.
int ensure_pages(ss_ctx* c, Shard* s, int64_t seq, int32_t length) {
    const int ps = c->m.page_size;
    const size_t need = (size_t)((length + ps - 1) / ps);
    {
        auto it = s->seqs.find(seq);
        const size_t have = it == s->seqs.end() ? 0 : it->second.pages.size();
        if (need > have && need - have > s->free_pages.size())
            return fail(c, SS_ENOMEM, "page pool exhausted: sequence %lld needs %zu more pages, %zu free",
                        (long long)seq, need - have, s->free_pages.size());
    }
    SeqState& st = s->seqs[seq];
    if (need > st.pages.size()) {
        while (st.pages.size() < need) {
            st.pages.push_back(s->free_pages.top());
            s->free_pages.pop();
        }
        s->version++;
    }
    if (length > st.len) st.len = length;
    return SS_OK;
}

// All or nothing for calls that bring whole sequences on board (swap-in, device import): the pages of
// every listed sequence must fit together, otherwise nothing is allocated and no sequence is entered.
int check_new_seqs_fit(ss_ctx* c, Shard* s, const int32_t* lens, int n) {
    const int ps = c->m.page_size;
    size_t need = 0;
    for (int i = 0; i < n; ++i) need += (size_t)((lens[i] + ps - 1) / ps);
    if (need > s->free_pages.size())
        return fail(c, SS_ENOMEM, "page pool exhausted: the %d sequences need %zu pages, %zu free", n, need,
                    s->free_pages.size());
    return SS_OK;
}

ssk::KvLayer kv_layer(ss_ctx* c, Shard* s, int ll) {
    ssk::KvLayer k;
    k.k_pool = s->k_pool[ll];
    k.v_pool = s->v_pool[ll];
    k.n_heads = s->nkv_l;
    k.d = c->m.head_dim;
    k.page_size = c->m.page_size;
    return k;
}

// Pages per decode work item.  Longer items mean fewer partial results to write and merge and less
// per-wave set-up (measured on the 7B-shape batch: 5.2 TB/s at 8 pages, 5.6 at 64; on the GQA shard
// with one kv head: 3.9 TB/s at 8 pages, 4.6 at 64, 3.7 at 128), but the batch must still split into a
// couple of thousand waves (items x kv heads): within [16, 64] pages.  SS_DECODE_ITEM_PAGES overrides
// the choice (tuning).
static int decode_item_pages(int64_t total_pages, int n_kv_local) {
    static const int forced = [] {
        const char* e = getenv("SS_DECODE_ITEM_PAGES");
        const int n = e ? atoi(e) : 0;
        return n >= 2 && n <= 4096 ? (n & ~1) : 0;
    }();
    if (forced) return forced;
    int64_t n = total_pages * n_kv_local / 2048;
    n = std::max<int64_t>(16, std::min<int64_t>(64, n));
    return (int)(n & ~1);
}

// Builds (or reuses) the device metadata of a batch.  Returns the slot.
int prepare_batch(ss_ctx* c, Shard* s, const ss_batch* b, bool decode, hipStream_t stream, MetaSlot** out) {
    const int n = b->n_seqs;
    // ---- validation + page allocation (idempotent)
    int64_t T = 0;
    int max_q = 0;
    for (int i = 0; i < n; ++i) {
        const int ql = b->q_lens[i], before = b->kv_lens_before[i];
        if (ql <= 0 || before < 0) return fail(c, SS_EINVAL, "sequence %d: q_len=%d kv_len_before=%d", i, ql, before);
        if (decode && ql != 1) return fail(c, SS_EINVAL, "decode needs q_len == 1 (sequence %d has %d)", i, ql);
        if (before + ql > c->rt.max_seq_len)
            return fail(c, SS_EINVAL, "sequence %d reaches length %d > max_seq_len %d", i, before + ql, c->rt.max_seq_len);
        if (before > 0) {
            auto it = s->seqs.find(b->seq_ids[i]);
            if (it == s->seqs.end() || it->second.len < before)
                return fail(c, SS_ENOENT, "sequence %lld has no %d cached tokens in this shard",
                            (long long)b->seq_ids[i], before);
        }
        T += ql;
        max_q = std::max(max_q, ql);
    }
    if (T > (1 << 30)) return fail(c, SS_EINVAL, "batch too large");
    {   // all or nothing: a batch that does not fit leaves no sequence with pages it did not have before
        size_t more = 0;
        const int ps = c->m.page_size;
        for (int i = 0; i < n; ++i) {
            const size_t need = (size_t)((b->kv_lens_before[i] + b->q_lens[i] + ps - 1) / ps);
            auto it = s->seqs.find(b->seq_ids[i]);
            const size_t have = it == s->seqs.end() ? 0 : it->second.pages.size();
            if (need > have) more += need - have;
        }
        if (more > s->free_pages.size())
            return fail(c, SS_ENOMEM, "page pool exhausted: the batch needs %zu more pages, %zu free", more,
                        s->free_pages.size());
    }
    for (int i = 0; i < n; ++i) {
        int rc = ensure_pages(c, s, b->seq_ids[i], b->kv_lens_before[i] + b->q_lens[i]);
        if (rc) return rc;
    }
    // ---- cache lookup
    for (auto& ms : c->meta) {
        if (ms.shard == s && ms.version == s->version && ms.decode == decode && (int)ms.seq_ids.size() == n &&
            !memcmp(ms.seq_ids.data(), b->seq_ids, sizeof(int64_t) * n) &&
            !memcmp(ms.q_lens.data(), b->q_lens, sizeof(int32_t) * n) &&
            !memcmp(ms.kv_before.data(), b->kv_lens_before, sizeof(int32_t) * n)) {
            *out = &ms;
            return SS_OK;
        }
    }
    // ---- build
    MetaSlot& ms = c->meta[c->meta_next];
    c->meta_next = (c->meta_next + 1) % 4;
    if (ms.in_flight) {
        HIP_TRY(c, hipEventSynchronize(ms.done));
        ms.in_flight = false;
    }
    ms.shard = nullptr;
    int pt_stride = 1;
    std::vector<const SeqState*> sts(n);
    for (int i = 0; i < n; ++i) {
        sts[i] = &s->seqs[b->seq_ids[i]];
        pt_stride = std::max<int>(pt_stride, (int)sts[i]->pages.size());
    }
    // decode work items
    std::vector<int32_t> item_seq, item_page0, item_np, seq_item0;
    int max_items = 0;
    if (decode) {
        seq_item0.resize(n + 1);
        int64_t total_pages = 0;
        for (int i = 0; i < n; ++i) total_pages += (b->kv_lens_before[i] + 1 + c->m.page_size - 1) / c->m.page_size;
        const int ipp = decode_item_pages(total_pages, s->nkv_l);
        for (int i = 0; i < n; ++i) {
            seq_item0[i] = (int32_t)item_seq.size();
            const int used = (b->kv_lens_before[i] + 1 + c->m.page_size - 1) / c->m.page_size;
            // near-equal items (even page counts: the kernel walks pages in pairs) instead of full items
            // and a short remainder
            const int cnt = (used + ipp - 1) / ipp;
            const int per = (((used + cnt - 1) / cnt) + 1) & ~1;
            // The items of a sequence interleave (item j takes pages j, j + cnt, ...): the waves that work on one
            // sequence then read neighbouring pages at about the same time (7B shape: 0.715 -> 0.73 of the HBM rate;
            // the one-kv-head shard is unchanged).  SS_DECODE_STRIDED=0 gives contiguous runs of pages instead.
            static const int strided = getenv("SS_DECODE_STRIDED") ? atoi(getenv("SS_DECODE_STRIDED")) : 1;
            if (strided && cnt > 1 && cnt < 65536) {
                for (int j = 0; j < cnt && j < used; ++j) {
                    item_seq.push_back(i);
                    item_page0.push_back(j);
                    item_np.push_back(((used - j + cnt - 1) / cnt) | (cnt << 16));
                }
            } else
            for (int p0 = 0; p0 < used; p0 += per) {
                item_seq.push_back(i);
                item_page0.push_back(p0);
                item_np.push_back(std::min(per, used - p0));
            }
            max_items = std::max(max_items, cnt);
        }
        seq_item0[n] = (int32_t)item_seq.size();
    }
    // page units of the new tokens (for the RoPE + cache-write kernel)
    std::vector<int32_t> unit_seq, unit_tok0, unit_pos0, unit_cnt;
    {
        int t0 = 0;
        const int ps = c->m.page_size;
        for (int i = 0; i < n; ++i) {
            const int b0 = b->kv_lens_before[i], e0 = b0 + b->q_lens[i];
            for (int pg = b0 / ps; pg * ps < e0; ++pg) {
                const int p0 = std::max(b0, pg * ps), p1 = std::min(e0, pg * ps + ps);
                unit_seq.push_back(i);
                unit_tok0.push_back(t0 + (p0 - b0));
                unit_pos0.push_back(p0);
                unit_cnt.push_back(p1 - p0);
            }
            t0 += b->q_lens[i];
        }
    }
    const size_t n_units = unit_seq.size();
    const size_t n_items = item_seq.size();
    // Prefill attention work lists.  An item is (sequence, q head, block of 256 queries); its cost is the
    // number of 64-token tiles it visits plus a fixed part.  The blocks of the kernel (one per compute unit)
    // are dealt to the 8 XCDs round-robin by their index, so the items of one (sequence, kv head) -- which
    // read the same K and V pages -- all go to blocks of one residue modulo 8 and find those pages in one
    // L2.  Within a residue the items are taken sequence by sequence (longest first), kv head by kv head, last
    // query block first, and each goes to the block with the least work so far: the items of one (sequence,
    // kv head) then start at about the same time on different blocks and share the pages while they are in
    // the L2 (taking all items heaviest first balances 2 % better and reads twice as much from beyond L2).
    std::vector<int32_t> pf_items;
    int pf_stride = 0, pf_blocks = 0;
    if (!decode && max_q > 64) {
        struct PfItem { int32_t sq, a, qb, cost, len; };
        const int G = s->nq_l / s->nkv_l;
        const int per_x = std::max(1, c->n_cus / 8);
        std::vector<std::vector<PfItem>> by_x(8);
        for (int i = 0; i < n; ++i) {
            const int nqb_i = (b->q_lens[i] + 255) / 256;
            for (int g = 0; g < s->nkv_l; ++g) {
                const int x = (int)(((int64_t)i * s->nkv_l + g) % 8);
                for (int jg = 0; jg < G; ++jg)
                    for (int qb = 0; qb < nqb_i; ++qb) {
                        const int last = b->kv_lens_before[i] + std::min(qb * 256 + 255, b->q_lens[i] - 1);
                        by_x[x].push_back({i, g * G + jg, qb, last / 64 + 1 + 2, b->kv_lens_before[i] + b->q_lens[i]});
                    }
            }
        }
        std::vector<std::vector<PfItem>> lists((size_t)8 * per_x);
        for (int x = 0; x < 8; ++x) {
            std::stable_sort(by_x[x].begin(), by_x[x].end(), [G](const PfItem& p, const PfItem& q) {
                if (p.len != q.len) return p.len > q.len;
                if (p.sq != q.sq) return p.sq < q.sq;
                if (p.a / G != q.a / G) return p.a / G < q.a / G;
                if (p.qb != q.qb) return p.qb > q.qb;
                return p.a < q.a;
            });
            std::priority_queue<std::pair<int64_t, int>, std::vector<std::pair<int64_t, int>>, std::greater<std::pair<int64_t, int>>> load;
            for (int k = 0; k < per_x; ++k) load.push({0, k});
            for (const PfItem& it : by_x[x]) {
                auto top = load.top();
                load.pop();
                lists[(size_t)top.second * 8 + x].push_back(it);
                load.push({top.first + it.cost, top.second});
            }
        }
        pf_blocks = 8 * per_x;
        size_t longest = 0;
        for (const auto& l : lists) longest = std::max(longest, l.size());
        pf_stride = (int)longest + 1;
        // one 32-byte record per item, everything the block needs to start on it: sequence (-1 ends the
        // list), q head, first query of the block, first token of the sequence in the batch, its number of
        // new tokens, its number of cached tokens
        pf_items.assign((size_t)pf_blocks * pf_stride * 8, -1);
        int t0 = 0;
        std::vector<int> q_begin(n);
        for (int i = 0; i < n; ++i) { q_begin[i] = t0; t0 += b->q_lens[i]; }
        for (int blk = 0; blk < pf_blocks; ++blk)
            for (size_t j = 0; j < lists[blk].size(); ++j) {
                int32_t* r = &pf_items[((size_t)blk * pf_stride + j) * 8];
                const PfItem& it = lists[blk][j];
                r[0] = it.sq; r[1] = it.a; r[2] = it.qb * 256; r[3] = q_begin[it.sq]; r[4] = b->q_lens[it.sq];
                r[5] = b->kv_lens_before[it.sq]; r[6] = 0; r[7] = 0;
            }
    }
    // launch order: longest items first, so that the last waves of the grid are the short ones
    std::vector<int32_t> item_order(n_items);
    for (size_t i = 0; i < n_items; ++i) item_order[i] = (int32_t)i;
    std::stable_sort(item_order.begin(), item_order.end(), [&](int32_t a, int32_t b2) { return (item_np[a] & 0xffff) > (item_np[b2] & 0xffff); });
    auto al = [](size_t x) { return (x + 63) & ~(size_t)63; };
    size_t off_tok_seq = 0;
    size_t off_tok_pos = off_tok_seq + al(4 * (size_t)T);
    size_t off_cu = off_tok_pos + al(4 * (size_t)T);
    size_t off_before = off_cu + al(4 * (size_t)(n + 1));
    size_t off_pt = off_before + al(4 * (size_t)n);
    size_t off_iseq = off_pt + al(4 * (size_t)n * pt_stride);
    size_t off_ip0 = off_iseq + al(4 * n_items);
    size_t off_inp = off_ip0 + al(4 * n_items);
    size_t off_si0 = off_inp + al(4 * n_items);
    size_t off_iord = off_si0 + al(4 * (size_t)(n + 1));
    size_t off_useq = off_iord + al(4 * n_items);
    size_t off_utok = off_useq + al(4 * n_units);
    size_t off_upos = off_utok + al(4 * n_units);
    size_t off_ucnt = off_upos + al(4 * n_units);
    size_t off_pf = off_ucnt + al(4 * n_units);
    size_t total = off_pf + al(4 * pf_items.size());
    if (total > ms.cap) {
        if (ms.host) { HIP_TRY(c, hipHostFree(ms.host)); ms.host = nullptr; }
        if (ms.dev) { HIP_TRY(c, hipFree(ms.dev)); ms.dev = nullptr; }
        ms.cap = total + total / 4 + 4096;
        HIP_TRY(c, hipHostMalloc((void**)&ms.host, ms.cap, hipHostMallocDefault));
        HIP_TRY(c, hipMalloc((void**)&ms.dev, ms.cap));
    }
    int32_t* tok_seq = (int32_t*)(ms.host + off_tok_seq);
    int32_t* tok_pos = (int32_t*)(ms.host + off_tok_pos);
    int32_t* cu = (int32_t*)(ms.host + off_cu);
    int32_t* before = (int32_t*)(ms.host + off_before);
    int32_t* pt = (int32_t*)(ms.host + off_pt);
    int t = 0;
    for (int i = 0; i < n; ++i) {
        cu[i] = t;
        before[i] = b->kv_lens_before[i];
        for (int j = 0; j < b->q_lens[i]; ++j, ++t) {
            tok_seq[t] = i;
            tok_pos[t] = b->kv_lens_before[i] + j;
        }
        const auto& pg = sts[i]->pages;
        int32_t* row = pt + (size_t)i * pt_stride;
        std::copy(pg.begin(), pg.end(), row);
        std::fill(row + pg.size(), row + pt_stride, pg.empty() ? 0 : pg.back());
    }
    cu[n] = t;
    if (decode) {
        memcpy(ms.host + off_iseq, item_seq.data(), 4 * n_items);
        memcpy(ms.host + off_ip0, item_page0.data(), 4 * n_items);
        memcpy(ms.host + off_inp, item_np.data(), 4 * n_items);
        memcpy(ms.host + off_si0, seq_item0.data(), 4 * (size_t)(n + 1));
        memcpy(ms.host + off_iord, item_order.data(), 4 * n_items);
    }
    memcpy(ms.host + off_useq, unit_seq.data(), 4 * n_units);
    memcpy(ms.host + off_utok, unit_tok0.data(), 4 * n_units);
    memcpy(ms.host + off_upos, unit_pos0.data(), 4 * n_units);
    memcpy(ms.host + off_ucnt, unit_cnt.data(), 4 * n_units);
    if (!pf_items.empty()) memcpy(ms.host + off_pf, pf_items.data(), 4 * pf_items.size());
    HIP_TRY(c, hipMemcpyAsync(ms.dev, ms.host, total, hipMemcpyHostToDevice, stream));
    ms.bm.tok_seq = (const int32_t*)(ms.dev + off_tok_seq);
    ms.bm.tok_pos = (const int32_t*)(ms.dev + off_tok_pos);
    ms.bm.cu_q = (const int32_t*)(ms.dev + off_cu);
    ms.bm.kv_before = (const int32_t*)(ms.dev + off_before);
    ms.bm.page_tables = (const int32_t*)(ms.dev + off_pt);
    ms.bm.pt_stride = pt_stride;
    ms.bm.n_seqs = n;
    ms.bm.T = (int)T;
    ms.bm.max_q_len = max_q;
    ms.bm.unit_seq = (const int32_t*)(ms.dev + off_useq);
    ms.bm.unit_tok0 = (const int32_t*)(ms.dev + off_utok);
    ms.bm.unit_pos0 = (const int32_t*)(ms.dev + off_upos);
    ms.bm.unit_cnt = (const int32_t*)(ms.dev + off_ucnt);
    ms.bm.n_units = (int)n_units;
    ms.bm.pf_items = pf_items.empty() ? nullptr : (const int32_t*)(ms.dev + off_pf);
    ms.bm.pf_stride = pf_stride;
    ms.bm.pf_blocks = pf_blocks;
    ms.wk.item_seq = (const int32_t*)(ms.dev + off_iseq);
    ms.wk.item_page0 = (const int32_t*)(ms.dev + off_ip0);
    ms.wk.item_npages = (const int32_t*)(ms.dev + off_inp);
    ms.wk.seq_item0 = (const int32_t*)(ms.dev + off_si0);
    ms.wk.item_order = (const int32_t*)(ms.dev + off_iord);
    ms.wk.n_items = (int)n_items;
    ms.wk.max_items_per_seq = max_items;
    ms.shard = s;
    ms.version = s->version;
    ms.decode = decode;
    ms.seq_ids.assign(b->seq_ids, b->seq_ids + n);
    ms.q_lens.assign(b->q_lens, b->q_lens + n);
    ms.kv_before.assign(b->kv_lens_before, b->kv_lens_before + n);
    *out = &ms;
    return SS_OK;
}

int mark_meta_used(ss_ctx* c, MetaSlot* ms, hipStream_t stream) {
    if (!ms->done) HIP_TRY(c, hipEventCreateWithFlags(&ms->done, hipEventDisableTiming));
    HIP_TRY(c, hipEventRecord(ms->done, stream));
    ms->in_flight = true;
    return SS_OK;
}

#define K_TRY(c, expr)                                                                                       \
    do {                                                                                                     \
        hipError_t e_ = (expr);                                                                              \
        if (e_ != hipSuccess)                                                                                \
            return fail((c), e_ == hipErrorInvalidValue ? SS_EINVAL : SS_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

int run_attn_phase(ss_ctx* c, Shard* s, int ll, const ss_batch* b, bool decode, const void* x_in, void* out,
                   bool residual, hipStream_t st) {
    const ss_model_cfg& m = c->m;
    const LayerW& w = s->w[ll];
    MetaSlot* ms = nullptr;
    int rc = prepare_batch(c, s, b, decode, st, &ms);
    if (rc) return rc;
    const int T = ms->bm.T, H = m.hidden, d = m.head_dim;
    const int nqkv = (s->nq_l + 2 * s->nkv_l) * d;
    if ((rc = ensure_buf(c, c->ws_rs, (size_t)T * sizeof(float)))) return rc;
    if ((rc = ensure_buf(c, c->ws_qkv, (size_t)T * nqkv * c->es))) return rc;
    if ((rc = ensure_buf(c, c->ws_attn, (size_t)T * s->nq_l * d * c->es))) return rc;
    if (decode) {
        size_t fl = ssk::attn_decode_scratch_floats(ms->wk.n_items, s->nq_l, d);
        if ((rc = ensure_buf(c, c->ws_scratch, fl * sizeof(float)))) return rc;
    }
    if (c->dt != SS_F32 && T <= 2048 && (rc = ensure_buf(c, c->ws_splitk, (size_t)128 << 20))) return rc;
    const ssk::KvLayer kv = kv_layer(c, s, ll);
    // RMSNorm is not a pass of its own: the gains are folded into the rows of Wqkv at load time, the product
    // runs on the raw activations and its epilogue multiplies every token row by rsqrt(mean(x^2) + eps), which
    // a read-only pass over x provides (T floats)
    {
        ProfScope ps(c, 4, st);
        K_TRY(c, SSK_CALL(c, row_scale, x_in, (float*)c->ws_rs.p, T, H, m.rms_eps, st));
    }
    {
        ProfScope ps(c, 0, st);
        K_TRY(c, SSK_CALL(c, gemm_nt, x_in, H, w.wqkv_t, c->ws_qkv.p, nqkv, nullptr, T, nqkv, H, ssk::EPI_STORE,
                              c->force_generic, st, (float*)c->ws_splitk.p, c->ws_splitk.cap, c->gemm_rounds,
                              (const float*)c->ws_rs.p));
    }
    {
        ProfScope ps(c, 4, st);
        K_TRY(c, SSK_CALL(c, rope_kvwrite, c->ws_qkv.p, s->nq_l, s->nkv_l, c->d_rope, ms->bm, kv, st));
    }
    if (decode) {
        ProfScope ps(c, 2, st);
        K_TRY(c, SSK_CALL(c, attn_decode, c->ws_qkv.p, c->ws_attn.p, s->nq_l, s->nkv_l, ms->bm, kv, ms->wk,
                                  (float*)c->ws_scratch.p, c->force_generic, st));
    } else {
        ProfScope ps(c, 1, st);
        K_TRY(c, SSK_CALL(c, attn_prefill, c->ws_qkv.p, c->ws_attn.p, s->nq_l, s->nkv_l, ms->bm, kv,
                                   c->force_generic, st));
    }
    {
        ProfScope ps(c, 0, st);
        K_TRY(c, SSK_CALL(c, gemm_nt, c->ws_attn.p, s->nq_l * d, w.wo_t, out, H, residual ? x_in : nullptr, T, H,
                              s->nq_l * d, residual ? ssk::EPI_RESIDUAL : ssk::EPI_STORE, c->force_generic, st, (float*)c->ws_splitk.p, c->ws_splitk.cap, c->gemm_rounds));
    }
    return mark_meta_used(c, ms, st);
}

int run_mlp_phase(ss_ctx* c, Shard* s, int ll, int T, const void* x1, void* out, bool residual, hipStream_t st) {
    const ss_model_cfg& m = c->m;
    const LayerW& w = s->w[ll];
    const int H = m.hidden, F = s->f_l;
    int rc;
    if ((rc = ensure_buf(c, c->ws_rs, (size_t)T * sizeof(float)))) return rc;
    if ((rc = ensure_buf(c, c->ws_act, (size_t)T * F * c->es))) return rc;
    if (c->dt != SS_F32 && T <= 2048 && (rc = ensure_buf(c, c->ws_splitk, (size_t)128 << 20))) return rc;
    {
        ProfScope ps(c, 4, st);
        K_TRY(c, SSK_CALL(c, row_scale, x1, (float*)c->ws_rs.p, T, H, m.rms_eps, st));      // as in the attention phase
    }
    if (w.gu_interleaved) {
        ProfScope ps(c, 0, st);
        K_TRY(c, SSK_CALL(c, gemm_nt, x1, H, w.wgu_t, c->ws_act.p, F, nullptr, T, 2 * F, H, ssk::EPI_SWIGLU,
                              false, st, (float*)c->ws_splitk.p, c->ws_splitk.cap, c->gemm_rounds, (const float*)c->ws_rs.p));
    } else {
        if ((rc = ensure_buf(c, c->ws_gu, (size_t)T * 2 * F * c->es))) return rc;
        {
            ProfScope ps(c, 0, st);
            K_TRY(c, SSK_CALL(c, gemm_nt, x1, H, w.wgu_t, c->ws_gu.p, 2 * F, nullptr, T, 2 * F, H,
                                  ssk::EPI_STORE, c->force_generic, st, (float*)c->ws_splitk.p, c->ws_splitk.cap, c->gemm_rounds,
                                  (const float*)c->ws_rs.p));
        }
        ProfScope ps(c, 4, st);
        K_TRY(c, SSK_CALL(c, swiglu, c->ws_gu.p, c->ws_act.p, T, F, st));
    }
    {
        ProfScope ps(c, 0, st);
        K_TRY(c, SSK_CALL(c, gemm_nt, c->ws_act.p, F, w.wd_t, out, H, residual ? x1 : nullptr, T, H, F,
                              residual ? ssk::EPI_RESIDUAL : ssk::EPI_STORE, c->force_generic, st, (float*)c->ws_splitk.p, c->ws_splitk.cap, c->gemm_rounds));
    }
    return SS_OK;
}

int layer_call(ss_ctx* c, const ss_shard_desc* d, int layer, int phase, const ss_batch* b, const void* x_in,
               void* out, void* stream, bool decode) {
    if (!c) return SS_EINVAL;
    if (!b || !x_in || !out || b->n_seqs <= 0 || !b->seq_ids || !b->q_lens || !b->kv_lens_before)
        return fail(c, SS_EINVAL, "null or empty batch / buffers");
    if (x_in == out) return fail(c, SS_EINVAL, "out must not alias x_in");
    Shard* s = nullptr;
    int rc = get_shard(c, d, &s);
    if (rc) return rc;
    if (layer < d->layer_begin || layer >= d->layer_end)
        return fail(c, SS_EINVAL, "layer %d outside the shard's range [%d,%d)", layer, d->layer_begin, d->layer_end);
    const int ll = layer - d->layer_begin;
    if (!s->w[ll].loaded) return fail(c, SS_EINVAL, "layer %d not loaded for this shard", layer);
    if (s->w_pending) {      // a reload on the weight stream: the caller's stream waits for it, the host does not
        HIP_TRY(c, hipStreamWaitEvent((hipStream_t)stream, s->w_ready, 0));
        if (hipEventQuery(s->w_ready) == hipSuccess) s->w_pending = false;
        else (void)hipGetLastError();
    }
    const bool nores = (phase & SS_NO_RESIDUAL) != 0;
    const int ph = phase & 3;
    if (ph == 0) return fail(c, SS_EINVAL, "bad phase %d", phase);
    const int k = d->mode == SS_TP ? d->k : 1;
    if (ph == SS_BOTH && (k != 1 || nores)) return fail(c, SS_EINVAL, "SS_BOTH needs k == 1 and residuals");
    const bool residual = (k == 1) && !nores;
    if ((rc = ensure_pools(c, s))) return rc;
    hipStream_t st = (hipStream_t)stream;
    int64_t T = 0;
    for (int i = 0; i < b->n_seqs; ++i) T += b->q_lens[i];
    {   // the movers' repack kernels need launch boundaries to get onto the chip between persistent GEMM blocks
        std::lock_guard<std::mutex> lk(c->mu);
        c->gemm_rounds = c->jobs_done < c->jobs_issued ? c->gemm_rounds_busy : c->gemm_rounds_idle;
    }
    if (ph == SS_ATTN) return run_attn_phase(c, s, ll, b, decode, x_in, out, residual, st);
    if (ph == SS_MLP) {
        if (T <= 0 || T > (1 << 30)) return fail(c, SS_EINVAL, "bad token count");
        return run_mlp_phase(c, s, ll, (int)T, x_in, out, residual, st);
    }
    if ((rc = ensure_buf(c, c->ws_x1, (size_t)T * c->m.hidden * c->es))) return rc;
    if ((rc = run_attn_phase(c, s, ll, b, decode, x_in, c->ws_x1.p, true, st))) return rc;
    return run_mlp_phase(c, s, ll, (int)T, c->ws_x1.p, out, true, st);
}

// The layers of the shard's range one after the other, the output of one the input of the next.
int layers_call(ss_ctx* c, const ss_shard_desc* d, const ss_batch* b, const void* x_in, void* out, void* stream, bool decode) {
    if (!c) return SS_EINVAL;
    if (!d || !b || !x_in || !out || b->n_seqs <= 0 || !b->q_lens) return fail(c, SS_EINVAL, "null or empty batch / buffers");
    if (d->k != 1) return fail(c, SS_EINVAL, "layers can only be chained on the device for k == 1");
    if (d->layer_end <= d->layer_begin) return fail(c, SS_EINVAL, "empty layer range");
    int64_t T = 0;
    for (int i = 0; i < b->n_seqs; ++i) T += b->q_lens[i];
    if (T <= 0 || T > (1 << 30)) return fail(c, SS_EINVAL, "bad token count");
    const int n = d->layer_end - d->layer_begin;
    int rc;
    for (int j = 0; j < (n > 2 ? 2 : n - 1); ++j)
        if ((rc = ensure_buf(c, c->ws_chain[j], (size_t)T * c->m.hidden * c->es))) return rc;
    const void* in = x_in;
    for (int j = 0; j < n; ++j) {
        void* o = j == n - 1 ? out : c->ws_chain[j & 1].p;
        if ((rc = layer_call(c, d, d->layer_begin + j, SS_BOTH, b, in, o, stream, decode))) return rc;
        in = o;
    }
    return SS_OK;
}

// ------------------------------------------------------------------ mover
struct Unit {
    int seq_idx;     // index into job.seqs
    int ll;          // local layer
    size_t bytes;
};

// Fills the repack metadata of units [u0,u1) into host image `h`; returns the
// device-side struct (pointers relative to `dbase`).  Staging offsets are
// relative to the chunk start.
size_t build_units(ss_ctx* c, Shard* s, const std::vector<SeqJob>& seqs, const std::vector<Unit>& units, size_t u0,
                   size_t u1, uint8_t* h, uint8_t* dbase, size_t cap, ssk::RepackUnits* ru) {
    const size_t n = u1 - u0;
    // page lists: one per distinct sequence in the chunk
    std::vector<int> seq_first;   // seq_idx of units, compacted
    size_t n_pages = 0;
    std::unordered_map<int, size_t> pt_off;
    for (size_t u = u0; u < u1; ++u) {
        const int si = units[u].seq_idx;
        if (!pt_off.count(si)) {
            pt_off[si] = n_pages;
            seq_first.push_back(si);
            n_pages += (seqs[si].len + c->m.page_size - 1) / c->m.page_size;
        }
    }
    auto al = [](size_t x) { return (x + 63) & ~(size_t)63; };
    const size_t o_off = 0, o_len = o_off + al(8 * n), o_pt = o_len + al(4 * n), o_layer = o_pt + al(4 * n);
    const size_t o_pages = o_layer + al(4 * n), total = o_pages + al(4 * n_pages);
    if (total > cap) return 0;
    int64_t* uoff = (int64_t*)(h + o_off);
    int32_t* ulen = (int32_t*)(h + o_len);
    int32_t* upt = (int32_t*)(h + o_pt);
    int32_t* ulay = (int32_t*)(h + o_layer);
    int32_t* pages = (int32_t*)(h + o_pages);
    for (int si : seq_first) {
        const size_t np = (seqs[si].len + c->m.page_size - 1) / c->m.page_size;
        std::copy(seqs[si].pages.begin(), seqs[si].pages.begin() + np, pages + pt_off[si]);
    }
    size_t off_elems = 0;
    int max_pages = 0;
    for (size_t u = u0; u < u1; ++u) {
        const SeqJob& sj = seqs[units[u].seq_idx];
        uoff[u - u0] = (int64_t)off_elems;
        ulen[u - u0] = sj.len;
        upt[u - u0] = (int32_t)pt_off[units[u].seq_idx];
        ulay[u - u0] = units[u].ll;
        off_elems += units[u].bytes / c->es;
        max_pages = std::max(max_pages, (sj.len + c->m.page_size - 1) / c->m.page_size);
    }
    ru->unit_off = (const int64_t*)(dbase + o_off);
    ru->unit_len = (const int32_t*)(dbase + o_len);
    ru->unit_pt = (const int32_t*)(dbase + o_pt);
    ru->unit_layer = (const int32_t*)(dbase + o_layer);
    ru->pages = (const int32_t*)(dbase + o_pages);
    ru->n_units = (int)n;
    ru->max_pages = max_pages;
    (void)s;
    return total;
}

std::vector<Unit> make_units(ss_ctx* c, Shard* s, const std::vector<SeqJob>& seqs) {
    std::vector<Unit> units;
    for (size_t i = 0; i < seqs.size(); ++i)
        for (int ll = 0; ll < s->n_layers_l; ++ll)
            units.push_back({(int)i, ll, (size_t)2 * s->nkv_l * seqs[i].len * c->m.head_dim * c->es});
    return units;
}

// Host tier address of the run (layer, c, first local head) of a sequence.
uint8_t* tier_run(ss_ctx* c, Shard* s, const SeqJob& sj, int ll, int kv) {
    const size_t layer = (size_t)(s->desc.layer_begin + ll);
    const size_t elems = (((layer * 2 + kv) * c->m.n_kv_heads + s->g0) * (size_t)sj.len) * c->m.head_dim;
    return c->tier + sj.tier_off + elems * c->es;
}

int worker_job(ss_ctx* c, Lane& L, Job& job) {
    Shard* s = job.sh;
    if (job.after) {
        HIP_TRY(c, hipStreamWaitEvent(L.side, job.after, 0));
    }
    const std::vector<Unit> units = make_units(c, s, job.seqs);
    const size_t run_elems_bytes = c->es * c->m.head_dim;   // per token per head
    // chunks of consecutive units fitting one slot
    std::vector<std::pair<size_t, size_t>> chunks;
    for (size_t u = 0; u < units.size();) {
        size_t bytes = 0, v = u;
        while (v < units.size() && bytes + units[v].bytes <= c->slot_bytes && v - u < 65535) bytes += units[v++].bytes;
        if (v == u) return fail(c, SS_ENOMEM, "pinned slot (%zu bytes) smaller than one sequence-layer unit (%zu bytes)",
                                c->slot_bytes, units[u].bytes);
        chunks.push_back({u, v});
        u = v;
    }
    // Stage two (pinned <-> tier) is plain host memcpy; large chunks are split over a few helper
    // threads so that one core's copy rate does not become the ceiling of the whole movement.
    auto host_copy = [&](size_t ci, bool to_tier, int slot) {
        struct Piece { uint8_t* tier; uint8_t* pin; size_t bytes; };
        std::vector<Piece> pieces;
        uint8_t* p = L.pinned + (size_t)slot * c->slot_bytes;
        size_t total = 0;
        for (size_t u = chunks[ci].first; u < chunks[ci].second; ++u) {
            const SeqJob& sj = job.seqs[units[u].seq_idx];
            const size_t run = (size_t)s->nkv_l * sj.len * run_elems_bytes;
            for (int kv = 0; kv < 2; ++kv) {
                pieces.push_back({tier_run(c, s, sj, units[u].ll, kv), p, run});
                p += run;
                total += run;
            }
        }
        auto work = [&](size_t b, size_t e) {
            for (size_t i = b; i < e; ++i) {
                if (to_tier) memcpy(pieces[i].tier, pieces[i].pin, pieces[i].bytes);
                else memcpy(pieces[i].pin, pieces[i].tier, pieces[i].bytes);
            }
        };
        const int nth = (total >= ((size_t)8 << 20)) ? std::min<int>(c->copy_threads, (int)pieces.size()) : 1;
        if (nth <= 1) { work(0, pieces.size()); return; }
        std::vector<std::thread> th;
        // contiguous ranges of pieces with roughly equal bytes
        size_t begin = 0, acc = 0;
        int made = 0;
        for (size_t i = 0; i < pieces.size(); ++i) {
            acc += pieces[i].bytes;
            const bool last = i + 1 == pieces.size();
            if (last || (acc >= total / nth * (made + 1) && made + 1 < nth)) {
                th.emplace_back(work, begin, i + 1);
                begin = i + 1;
                ++made;
            }
        }
        for (auto& t : th) t.join();
    };
    auto chunk_bytes = [&](size_t ci) {
        size_t b = 0;
        for (size_t u = chunks[ci].first; u < chunks[ci].second; ++u) b += units[u].bytes;
        return b;
    };
    // Device staging holds a group of consecutive chunks (a whole job when it fits): one repack kernel per
    // group instead of one per chunk, so that the copies of a group run back to back on the lane's stream
    // without a kernel (that has to find room on a chip busy with the caller's kernels) between them.
    // out: gather(group) -> for each chunk: DMA staging -> pinned slot | stage two of the previous chunk
    // in:  for each chunk: stage two into the pinned slot | DMA pinned slot -> staging; then scatter(group)
    constexpr size_t DEV_CAP_MAX = (size_t)2 << 30;
    size_t job_bytes = 0;
    for (const Unit& u : units) job_bytes += u.bytes;
    {
        const size_t want = std::min(std::max(job_bytes, 2 * c->slot_bytes), DEV_CAP_MAX);
        if (want > L.dev_cap) {              // the lane's stream is idle between jobs
            if (L.dev_staging) HIP_TRY(c, hipFree(L.dev_staging));
            L.dev_staging = nullptr;
            L.dev_cap = 0;
            HIP_TRY(c, hipMalloc((void**)&L.dev_staging, want));
            L.dev_cap = want;
        }
    }
    size_t n_dma = 0;                        // chunks whose DMA has been issued (pinned slot = n_dma & 1)
    const bool fine = c->trace_mover && getenv("SS_TRACE_MOVER")[0] == '2';
    auto now_ms = [] { return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count(); };
    const double tj0 = now_ms();
    auto mark = [&](const char* what, size_t ci) { if (fine) fprintf(stderr, "[mover-fine] %s dir %d chunk %zu at %.3f ms\n", what, job.dir, ci, now_ms() - tj0); };
    for (size_t g0 = 0; g0 < chunks.size();) {
        size_t g1 = g0, gbytes = 0;
        while (g1 < chunks.size() && gbytes + chunk_bytes(g1) <= L.dev_cap &&
               chunks[g1].second - chunks[g0].first <= 65535) gbytes += chunk_bytes(g1++);
        if (g1 == g0) return fail(c, SS_ENOMEM, "device staging smaller than one chunk");
        if (g0 > 0) HIP_TRY(c, hipStreamSynchronize(L.side));    // the previous group is through: metadata is free
        ssk::RepackUnits ru{};
        const size_t mbytes = build_units(c, s, job.seqs, units, chunks[g0].first, chunks[g1 - 1].second, L.mv_meta_host,
                                          L.mv_meta_dev, c->mv_meta_cap, &ru);
        if (!mbytes) return fail(c, SS_ENOMEM, "KV mover metadata region too small");
        HIP_TRY(c, hipMemcpyAsync(L.mv_meta_dev, L.mv_meta_host, mbytes, hipMemcpyHostToDevice, L.side));
        if (job.dir == SS_OUT) {
            ProfScope ps(c, 3, L.side);
            K_TRY(c, SSK_CALL(c, kv_gather, s->d_k_pools, s->d_v_pools, s->nkv_l, c->m.head_dim, c->m.page_size, ru,
                                    L.dev_staging, L.side));
        }
        // runs of this group: (unit, K|V) -> contiguous in staging and in the tier
        size_t min_run = SIZE_MAX;
        for (size_t u = chunks[g0].first; u < chunks[g1 - 1].second; ++u) min_run = std::min(min_run, units[u].bytes / 2);
        const bool direct = c->tier_pinned && min_run >= ((size_t)256 << 10);
        if (direct) {
            // runs that follow each other both in staging and in the tier (K and V of a shard that owns all
            // kv heads, consecutive layers, sequences whose tier slots are adjacent) go as one copy
            size_t uoff = 0, cur_bytes = 0;
            uint8_t *cur_t = nullptr, *cur_d = nullptr;
            // The device-to-host copies of a swap-out go to a stream of their own, ordered behind the gather
            // by an event: measured, the pipelined step (prefill + re-shard + decode) is 4 % shorter and its
            // time steadier than with the copies on the gather's stream.  The runtime executes them as copy
            // kernels either way.
            hipStream_t out_stream = L.side;
            const bool via_hsa = job.dir == SS_OUT && L.hsa.ok;
            std::vector<HsaCopy::Run> hsa_runs;
            if (job.dir == SS_OUT && !via_hsa && L.copy) {
                HIP_TRY(c, hipEventRecord(L.copy_ev[0], L.side));
                HIP_TRY(c, hipStreamWaitEvent(L.copy, L.copy_ev[0], 0));
                out_stream = L.copy;
            }
            // merged runs: up to copy_max_bytes for copies the HIP runtime carries out, 64 MB on the DMA engines
            const size_t merge_max = via_hsa ? std::max(c->copy_max_bytes, (size_t)64 << 20) : c->copy_max_bytes;
            auto flush = [&]() -> int {
                if (!cur_bytes) return SS_OK;
                if (via_hsa) hsa_runs.push_back({cur_t, cur_d, cur_bytes});
                else if (job.dir == SS_OUT) HIP_TRY(c, hipMemcpyAsync(cur_t, cur_d, cur_bytes, hipMemcpyDeviceToHost, out_stream));
                else HIP_TRY(c, hipMemcpyAsync(cur_d, cur_t, cur_bytes, hipMemcpyHostToDevice, L.side));
                cur_bytes = 0;
                return SS_OK;
            };
            for (size_t u = chunks[g0].first; u < chunks[g1 - 1].second; ++u) {
                const SeqJob& sj = job.seqs[units[u].seq_idx];
                const size_t run = units[u].bytes / 2;
                for (int kv = 0; kv < 2; ++kv) {
                    uint8_t* t = tier_run(c, s, sj, units[u].ll, kv);
                    uint8_t* d = L.dev_staging + uoff + (size_t)kv * run;
                    if (cur_bytes && cur_bytes + run <= merge_max && t == cur_t + cur_bytes && d == cur_d + cur_bytes) {
                        cur_bytes += run;
                    } else {
                        int rc = flush();
                        if (rc) return rc;
                        cur_t = t; cur_d = d; cur_bytes = run;
                    }
                }
                uoff += units[u].bytes;
            }
            int rc = flush();
            if (rc) return rc;
            if (via_hsa) {
                // the gather kernel has written the staging buffer; then the engines copy while this thread waits
                HIP_TRY(c, hipStreamSynchronize(L.side));
                if (!L.hsa.copy_out(hsa_runs)) {
                    L.hsa.ok = false;                 // once: from here on (and for these runs) the HIP runtime's copies
                    for (const HsaCopy::Run& r : hsa_runs)
                        HIP_TRY(c, hipMemcpyAsync(r.host, r.dev, r.bytes, hipMemcpyDeviceToHost, L.side));
                }
            }
            if (out_stream != L.side) {
                HIP_TRY(c, hipEventRecord(L.copy_ev[1], L.copy));
                HIP_TRY(c, hipStreamWaitEvent(L.side, L.copy_ev[1], 0));
            }
        }
        size_t off = 0;
        size_t pending = SIZE_MAX;               // out: chunk whose stage two has not run yet
        for (size_t ci = g0; !direct && ci < g1; ++ci, ++n_dma) {
            const int slot = (int)(n_dma & 1);
            uint8_t* pin = L.pinned + (size_t)slot * c->slot_bytes;
            const size_t bytes = chunk_bytes(ci);
            if (job.dir == SS_OUT) {
                // the pinned slot is free: stage two of the chunk before the previous one has run
                HIP_TRY(c, hipMemcpyAsync(pin, L.dev_staging + off, bytes, hipMemcpyDeviceToHost, L.side));
                HIP_TRY(c, hipEventRecord(L.mv_ev[slot], L.side));
                if (pending != SIZE_MAX) {   // stage two of the previous chunk overlaps this chunk's DMA
                    mark("wait-dma", pending);
                    HIP_TRY(c, hipEventSynchronize(L.mv_ev[slot ^ 1]));
                    mark("dma-done", pending);
                    host_copy(pending, true, slot ^ 1);
                    mark("host-copied", pending);
                }
                pending = ci;
            } else {
                mark("wait-slot", ci);
                if (n_dma >= 2) HIP_TRY(c, hipEventSynchronize(L.mv_ev[slot]));   // the DMA of chunk ci-2 has read the slot
                mark("slot-free", ci);
                host_copy(ci, false, slot);   // overlaps the previous chunk's DMA
                mark("host-copied", ci);
                HIP_TRY(c, hipMemcpyAsync(L.dev_staging + off, pin, bytes, hipMemcpyHostToDevice, L.side));
                HIP_TRY(c, hipEventRecord(L.mv_ev[slot], L.side));
            }
            off += bytes;
        }
        if (pending != SIZE_MAX) {
            const int slot = (int)((n_dma - 1) & 1);
            HIP_TRY(c, hipEventSynchronize(L.mv_ev[slot]));
            mark("dma-done", pending);
            host_copy(pending, true, slot);
            mark("host-copied", pending);
        }
        if (job.dir == SS_IN) {
            ProfScope ps(c, 3, L.side);
            K_TRY(c, SSK_CALL(c, kv_scatter, s->d_k_pools, s->d_v_pools, s->nkv_l, c->m.head_dim, c->m.page_size, ru,
                                     L.dev_staging, L.side));
        }
        g0 = g1;
    }
    mark("wait-stream", chunks.size());
    HIP_TRY(c, hipStreamSynchronize(L.side));
    mark("stream-done", chunks.size());
    return SS_OK;
}

void worker_main(ss_ctx* c, int li) {
    Lane& L = c->lane[li];
    (void)hipSetDevice(c->rt.device);
    std::string local_err;
    tl_err = &local_err;
    for (;;) {
        Job job;
        {
            std::unique_lock<std::mutex> lk(c->mu);
            // a swap-in starts only after the swap-outs issued before it have filled the tier
            c->cv.wait(lk, [&] { return c->stop || (!L.jobs.empty() && c->out_done >= L.jobs.front().needs_out); });
            if (L.jobs.empty()) return;                      // stop requested and queue drained
            if (c->out_done < L.jobs.front().needs_out) {    // stopping: the other lane drains first
                c->cv.wait(lk, [&] { return c->out_done >= L.jobs.front().needs_out; });
            }
            job = std::move(L.jobs.front());
            L.jobs.pop_front();
            L.busy = true;
            L.running = &job;
        }
        local_err.clear();
        const auto t_job0 = std::chrono::steady_clock::now();
        const int rc = worker_job(c, L, job);
        if (c->trace_mover) {
            const double ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_job0).count();
            size_t bytes = 0;
            for (const SeqJob& sj : job.seqs)
                bytes += (size_t)2 * job.sh->nkv_l * sj.len * c->m.head_dim * c->es * job.sh->n_layers_l;
            fprintf(stderr, "[mover] job %lld %s: %.2f ms, %.1f MB, %.1f GB/s\n", (long long)job.id,
                    job.dir == SS_OUT ? "out" : "in", ms, bytes / 1e6, bytes / ms / 1e6);
        }
        if (job.after) (void)hipEventDestroy(job.after);
        {
            std::lock_guard<std::mutex> lk(c->mu);
            if (rc && !c->worker_rc) {
                c->worker_rc = rc;
                c->worker_err = local_err;
            }
            L.busy = false;
            L.running = nullptr;
            if (job.dir == SS_OUT) c->out_done++;
            c->done_ids.push_back(job.id);
            for (bool moved = true; moved;) {
                moved = false;
                for (size_t i = 0; i < c->done_ids.size(); ++i)
                    if (c->done_ids[i] == c->jobs_done + 1) {
                        c->jobs_done++;
                        c->done_ids.erase(c->done_ids.begin() + i);
                        moved = true;
                        break;
                    }
            }
        }
        c->cv_idle.notify_all();
        c->cv.notify_all();
    }
}

}  // namespace

// =====================================================================
// C ABI
// =====================================================================
namespace {

void wait_idle(ss_ctx* c) {
    std::unique_lock<std::mutex> lk(c->mu);
    c->cv_idle.wait(lk, [&] {
        return c->lane[0].jobs.empty() && !c->lane[0].busy && c->lane[1].jobs.empty() && !c->lane[1].busy;
    });
}

int upload_matrix(ss_ctx* c, const void* src, int location, size_t bytes, void** tmp_out, const void** dev_src) {
    *tmp_out = nullptr;
    if (location == SS_DEVICE) { *dev_src = src; return SS_OK; }
    HIP_TRY(c, hipMalloc(tmp_out, bytes));
    hipError_t e = hipMemcpy(*tmp_out, src, bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) { (void)hipFree(*tmp_out); *tmp_out = nullptr; return fail(c, SS_EHIP, "weight upload: %s", hipGetErrorString(e)); }
    *dev_src = *tmp_out;
    return SS_OK;
}

// dst rows <- columns [c0, c0+n) of src[K, ld] (one full matrix staged at a time)
// (`gain`: device vector of K values folded into the rows, or null)
int slice_into(ss_ctx* c, const void* src, int location, size_t src_rows, size_t ld, size_t row0, int K, int c0, int n,
               void* dst, int blk, int blk_stride, int row_off, const void* gain = nullptr) {
    void* tmp = nullptr;
    const void* dsrc = nullptr;
    int rc = upload_matrix(c, src, location, src_rows * ld * c->es, &tmp, &dsrc);
    if (rc) return rc;
    const uint8_t* base = (const uint8_t*)dsrc + row0 * ld * c->es;
    hipError_t e = SSK_CALL(c, slice_transpose, base, (int64_t)ld, K, c0, n, dst, blk, blk_stride, row_off, 0, gain);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (tmp) (void)hipFree(tmp);
    if (e != hipSuccess) return fail(c, SS_EHIP, "weight slicing: %s", hipGetErrorString(e));
    return SS_OK;
}

int copy_vec(ss_ctx* c, const void* src, int location, size_t n, void** dst) {
    if (!*dst) HIP_TRY(c, hipMalloc(dst, n * c->es));
    HIP_TRY(c, hipMemcpy(*dst, src, n * c->es, location == SS_DEVICE ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice));
    return SS_OK;
}

int enqueue_job(ss_ctx* c, Job&& job, hipStream_t stream) {
    HIP_TRY(c, hipEventCreateWithFlags(&job.after, hipEventDisableTiming));
    HIP_TRY(c, hipEventRecord(job.after, stream));
    {
        std::lock_guard<std::mutex> lk(c->mu);
        job.id = ++c->jobs_issued;
        if (job.dir == SS_OUT) c->out_issued++;
        else job.needs_out = c->out_issued;
        c->lane[job.dir == SS_OUT ? 0 : 1].jobs.push_back(std::move(job));
    }
    c->cv.notify_all();
    return SS_OK;
}

// Blocks until no queued or running mover job touches any of the listed sequences
// (of shard `sh`, or of any shard when sh is null).
void wait_seqs_idle(ss_ctx* c, const Shard* sh, const int64_t* ids, int n) {
    std::unique_lock<std::mutex> lk(c->mu);
    auto touches = [&](const Job& j) {
        if (sh && j.sh != sh) return false;
        for (const SeqJob& sj : j.seqs)
            for (int i = 0; i < n; ++i)
                if (sj.seq == ids[i]) return true;
        return false;
    };
    c->cv_idle.wait(lk, [&] {
        for (const Lane& L : c->lane) {
            if (L.running && touches(*L.running)) return false;
            for (const Job& j : L.jobs)
                if (touches(j)) return false;
        }
        return true;
    });
}

size_t seq_tier_bytes(ss_ctx* c, int32_t len) {
    return (size_t)c->m.n_layers * 2 * c->m.n_kv_heads * (size_t)len * c->m.head_dim * c->es;
}

// Host tier slots: first fit at the lowest address; freed blocks merge with their
// neighbours, so an empty tier is one block again and allocation restarts at 0.
bool tier_alloc(ss_ctx* c, size_t bytes, size_t* off) {
    for (auto it = c->tier_free.begin(); it != c->tier_free.end(); ++it) {
        if (it->second < bytes) continue;
        *off = it->first;
        const size_t rest = it->second - bytes;
        c->tier_free.erase(it);
        if (rest) c->tier_free[*off + bytes] = rest;
        c->tier_used += bytes;
        return true;
    }
    return false;
}

void tier_release(ss_ctx* c, size_t off, size_t bytes) {
    auto it = c->tier_free.emplace(off, bytes).first;
    auto nx = std::next(it);
    if (nx != c->tier_free.end() && it->first + it->second == nx->first) {
        it->second += nx->second;
        c->tier_free.erase(nx);
    }
    if (it != c->tier_free.begin()) {
        auto pv = std::prev(it);
        if (pv->first + pv->second == it->first) {
            pv->second += it->second;
            c->tier_free.erase(it);
        }
    }
    c->tier_used -= bytes;
}

// ------------------------------------------------------------------ weights
size_t tensor_elems(const ss_model_cfg& m, int which) {
    const size_t H = m.hidden, qd = (size_t)m.n_q_heads * m.head_dim, kd = (size_t)m.n_kv_heads * m.head_dim, F = m.ffn;
    switch (which) {
        case SS_W_G1: case SS_W_G2: return H;
        case SS_W_Q: return H * qd;
        case SS_W_K: case SS_W_V: return H * kd;
        case SS_W_O: return qd * H;
        case SS_W_G: case SS_W_U: return H * F;
        case SS_W_D: return F * H;
    }
    return 0;
}

int alloc_layer_buffers(ss_ctx* c, Shard* s, LayerW& L) {
    const size_t H = c->m.hidden, nq = (size_t)s->nq_l * c->m.head_dim, nkv = (size_t)s->nkv_l * c->m.head_dim, F = s->f_l;
    const size_t es = c->es;
    auto alloc = [&](void** p, size_t bytes) -> int {
        if (!*p) HIP_TRY(c, hipMalloc(p, bytes));
        return SS_OK;
    };
    int rc;
    if ((rc = alloc(&L.g1, H * es))) return rc;
    if ((rc = alloc(&L.g2, H * es))) return rc;
    if ((rc = alloc(&L.wqkv_t, (nq + 2 * nkv) * H * es))) return rc;
    if ((rc = alloc(&L.wo_t, H * nq * es))) return rc;
    if ((rc = alloc(&L.wgu_t, 2 * F * H * es))) return rc;
    if ((rc = alloc(&L.wd_t, H * F * es))) return rc;
    return SS_OK;
}

// Frees the buffers whose guarding event has completed (all of them, waiting, when `wait`).
int release_deferred(ss_ctx* c, bool wait) {
    for (size_t i = 0; i < c->deferred.size();) {
        DeferredFree& df = c->deferred[i];
        if (wait) HIP_TRY(c, hipEventSynchronize(df.ev));
        const hipError_t q = hipEventQuery(df.ev);
        if (q == hipSuccess) {
            for (void* p : df.ptrs) HIP_TRY(c, hipFree(p));
            (void)hipEventDestroy(df.ev);
            c->deferred.erase(c->deferred.begin() + i);
        } else {
            (void)hipGetLastError();
            ++i;
        }
    }
    return SS_OK;
}

// One layer of shard s from the CPU copy, on the weight stream.  PCIe carries exactly the slice: a row
// range is one contiguous copy, a column range one strided (2D) copy; a device kernel then lays the
// staged slice out the way the GEMMs read it (transposed, gate/up interleaved).
int reload_layer(ss_ctx* c, Shard* s, int ll) {
    const ss_model_cfg& m = c->m;
    const HostLayer& hl = c->hw[s->desc.layer_begin + ll];
    LayerW& L = s->w[ll];
    int rc = alloc_layer_buffers(c, s, L);
    if (rc) return rc;
    const size_t es = c->es;
    const int H = m.hidden, dh = m.head_dim;
    const int nq = s->nq_l * dh, nkv = s->nkv_l * dh, F = s->f_l;
    const size_t qd = (size_t)m.n_q_heads * dh, kd = (size_t)m.n_kv_heads * dh;
    hipStream_t ws = c->wstream;
    HIP_TRY(c, hipMemcpyAsync(L.g1, hl.base + hl.off[SS_W_G1], (size_t)H * es, hipMemcpyHostToDevice, ws));
    HIP_TRY(c, hipMemcpyAsync(L.g2, hl.base + hl.off[SS_W_G2], (size_t)H * es, hipMemcpyHostToDevice, ws));
    // columns [c0, c0+n) of the host matrix [K, ld] -> dense staging [K, n] -> dst rows
    auto cols = [&](int which, int K, size_t ld, size_t c0, int n, void* dst, int blk, int blk_stride, int row_off,
                    const void* gain) -> int {
        const uint8_t* src = hl.base + hl.off[which] + c0 * es;
        if ((size_t)n == ld) HIP_TRY(c, hipMemcpyAsync(c->w_staging.p, src, (size_t)K * n * es, hipMemcpyHostToDevice, ws));
        else HIP_TRY(c, hipMemcpy2DAsync(c->w_staging.p, (size_t)n * es, src, ld * es, (size_t)n * es, (size_t)K,
                                         hipMemcpyHostToDevice, ws));
        K_TRY(c, SSK_CALL(c, slice_transpose, c->w_staging.p, (int64_t)n, K, 0, n, dst, blk, blk_stride, row_off, ws, gain));
        return SS_OK;
    };
    // rows [r0, r0+K) of the host matrix [*, n] (contiguous) -> staging [K, n] -> dst = its transpose
    auto rows = [&](int which, size_t r0, int K, int n, void* dst) -> int {
        const uint8_t* src = hl.base + hl.off[which] + r0 * (size_t)n * es;
        HIP_TRY(c, hipMemcpyAsync(c->w_staging.p, src, (size_t)K * n * es, hipMemcpyHostToDevice, ws));
        K_TRY(c, SSK_CALL(c, slice_transpose, c->w_staging.p, (int64_t)n, K, 0, n, dst, n, n, 0, ws));
        return SS_OK;
    };
    uint8_t* qkv = (uint8_t*)L.wqkv_t;
    // gains folded as in ss_load_layer (they were copied on this stream just above)
    if ((rc = cols(SS_W_Q, H, qd, (size_t)s->q0 * dh, nq, qkv, nq, nq, 0, L.g1))) return rc;
    if ((rc = cols(SS_W_K, H, kd, (size_t)s->g0 * dh, nkv, qkv + (size_t)nq * H * es, nkv, nkv, 0, L.g1))) return rc;
    if ((rc = cols(SS_W_V, H, kd, (size_t)s->g0 * dh, nkv, qkv + (size_t)(nq + nkv) * H * es, nkv, nkv, 0, L.g1))) return rc;
    if ((rc = rows(SS_W_O, (size_t)s->q0 * dh, nq, H, L.wo_t))) return rc;
    L.gu_interleaved = (c->dt != SS_F32) && !c->force_generic && (F % 32 == 0) && (H % 64 == 0);
    if (L.gu_interleaved) {
        if ((rc = cols(SS_W_G, H, m.ffn, s->f0, F, L.wgu_t, 32, 64, 0, L.g2))) return rc;
        if ((rc = cols(SS_W_U, H, m.ffn, s->f0, F, L.wgu_t, 32, 64, 32, L.g2))) return rc;
    } else {
        if ((rc = cols(SS_W_G, H, m.ffn, s->f0, F, L.wgu_t, F, F, 0, L.g2))) return rc;
        if ((rc = cols(SS_W_U, H, m.ffn, s->f0, F, L.wgu_t, F, F, F, L.g2))) return rc;
    }
    if ((rc = rows(SS_W_D, (size_t)s->f0, F, H, L.wd_t))) return rc;
    L.loaded = true;
    return SS_OK;
}

}  // namespace

extern "C" {

int ss_create(const ss_model_cfg* model, const ss_runtime_cfg* rt, ss_ctx** out) {
    if (!model || !rt || !out) return SS_EINVAL;
    *out = nullptr;
    const ss_model_cfg& m = *model;
    if (m.hidden <= 0 || m.n_q_heads <= 0 || m.n_kv_heads <= 0 || m.ffn <= 0 || m.n_layers <= 0) return SS_EINVAL;
    if ((m.head_dim != 64 && m.head_dim != 128) || m.page_size != 16) return SS_EINVAL;
    if (m.n_q_heads % m.n_kv_heads) return SS_EINVAL;
    if (m.dtype != SS_F32 && m.dtype != SS_BF16 && m.dtype != SS_F16) return SS_EINVAL;
    if (rt->gpu_kv_pages <= 0 || rt->gpu_kv_pages > (1ll << 30) || rt->max_seq_len <= 0 || rt->host_tier_bytes < 0 ||
        rt->pinned_bytes < 0)
        return SS_EINVAL;
    if (hipSetDevice(rt->device) != hipSuccess) return SS_EHIP;
    if (rt->device < 0 || rt->device >= NOALLOC_MAX_DEVICES) return SS_EINVAL;
    {   // this device's copy of the fixed scratch array: address looked up once, with the device current
        std::lock_guard<std::mutex> lk(g_noalloc_mu);
        if (!g_noalloc_scratch[rt->device]) {
            void* p = nullptr;
            const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !p) {
                fprintf(stderr, "ss_create: hipGetSymbolAddress(scratch): %s\n", hipGetErrorString(e));
                return SS_EHIP;
            }
            g_noalloc_scratch[rt->device] = p;
        }
    }
    ss_ctx* c = new ss_ctx();
    c->m = m;
    c->rt = *rt;
    c->dt = m.dtype;
    c->es = m.dtype == SS_F32 ? 4 : 2;
    const char* fg = getenv("SS_FORCE_GENERIC");
    c->force_generic = fg && fg[0] == '1';
    c->trace_mover = getenv("SS_TRACE_MOVER") != nullptr;
    if (const char* gr = getenv("SS_GEMM_ROUNDS")) c->gemm_rounds_busy = std::max(0, atoi(gr));
    if (const char* gr = getenv("SS_GEMM_ROUNDS_IDLE")) c->gemm_rounds_idle = std::max(0, atoi(gr));
    if (const char* cm = getenv("SS_COPY_MAX_MB")) c->copy_max_bytes = (size_t)std::max(1, atoi(cm)) << 20;
    if (const char* ct = getenv("SS_COPY_THREADS")) c->copy_threads = std::max(1, std::min(16, atoi(ct)));
    {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, rt->device) == hipSuccess && n >= 8) c->n_cus = n;
        else (void)hipGetLastError();
    }
    int rc = SS_OK;
    auto boot = [&]() -> int {
        // rotary table: cos/sin of p * base^(-2i/d), evaluated in double, stored as float pairs
        const int half = m.head_dim / 2;
        std::vector<float> tab((size_t)rt->max_seq_len * half * 2);
        for (int p = 0; p < rt->max_seq_len; ++p)
            for (int i = 0; i < half; ++i) {
                const double ang = (double)p * std::pow((double)m.rope_base, -2.0 * i / m.head_dim);
                tab[((size_t)p * half + i) * 2] = (float)std::cos(ang);
                tab[((size_t)p * half + i) * 2 + 1] = (float)std::sin(ang);
            }
        HIP_TRY(c, hipMalloc((void**)&c->d_rope, tab.size() * sizeof(float)));
        HIP_TRY(c, hipMemcpy(c->d_rope, tab.data(), tab.size() * sizeof(float), hipMemcpyHostToDevice));
        if (rt->host_tier_bytes > 0) {
            // Page-locked when it is of moderate size (SS_TIER_PIN_MAX_GB, default 64): the movers then copy
            // between device staging and the tier directly, one DMA per (sequence, layer, K|V) run, and
            // stage two through the pinned ring (a host memcpy per chunk, which doubles the host-memory
            // traffic of a movement) is only taken for short runs.  Larger tiers are pageable.
            double pin_max_gb = 64.0;
            if (const char* e = getenv("SS_TIER_PIN_MAX_GB")) pin_max_gb = atof(e);
            if ((double)rt->host_tier_bytes <= pin_max_gb * (double)(1ull << 30)) {
                void* pt = nullptr;
                if (hipHostMalloc(&pt, (size_t)rt->host_tier_bytes, hipHostMallocDefault) == hipSuccess) {
                    c->tier = (uint8_t*)pt;
                    c->tier_pinned = true;
                } else {
                    (void)hipGetLastError();
                }
            }
            if (!c->tier) c->tier = (uint8_t*)malloc((size_t)rt->host_tier_bytes);
            if (!c->tier) return fail(c, SS_ENOMEM, "host tier allocation failed");
            c->tier_cap = (size_t)rt->host_tier_bytes;
            c->tier_free[0] = c->tier_cap;
        }
        c->slot_bytes = ((size_t)rt->pinned_bytes / 4) & ~(size_t)255;
        c->mv_meta_cap = 16u << 20;
        for (Lane& L : c->lane) {
            if (c->slot_bytes) {
                HIP_TRY(c, hipHostMalloc((void**)&L.pinned, 2 * c->slot_bytes, hipHostMallocDefault));
                HIP_TRY(c, hipMalloc((void**)&L.dev_staging, 2 * c->slot_bytes));
                L.dev_cap = 2 * c->slot_bytes;
            }
            HIP_TRY(c, hipHostMalloc((void**)&L.mv_meta_host, c->mv_meta_cap, hipHostMallocDefault));
            HIP_TRY(c, hipMalloc((void**)&L.mv_meta_dev, c->mv_meta_cap));
            HIP_TRY(c, hipStreamCreateWithFlags(&L.side, hipStreamNonBlocking));
            HIP_TRY(c, hipStreamCreateWithFlags(&L.copy, hipStreamNonBlocking));
            if (&L == &c->lane[0]) L.hsa.init(rt->device);
            for (hipEvent_t& e : L.copy_ev) HIP_TRY(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
            for (int i = 0; i < 2; ++i) HIP_TRY(c, hipEventCreateWithFlags(&L.mv_ev[i], hipEventDisableTiming));
        }
        return SS_OK;
    };
    rc = boot();
    if (rc) { fprintf(stderr, "ss_create: %s\n", c->err.c_str()); delete c; return rc; }
    for (int li = 0; li < 2; ++li) c->lane[li].worker = std::thread(worker_main, c, li);
    *out = c;
    return SS_OK;
}

int ss_destroy(ss_ctx* c) {
    if (!c) return SS_EINVAL;
    {
        std::lock_guard<std::mutex> lk(c->mu);
        c->stop = true;
    }
    c->cv.notify_all();
    for (Lane& L : c->lane)
        if (L.worker.joinable()) L.worker.join();
    (void)hipSetDevice(c->rt.device);
    (void)hipDeviceSynchronize();
    for (auto& kv : c->shards) {
        Shard* s = kv.second;
        for (auto& w : s->w) {
            for (void* p : {w.g1, w.g2, w.wqkv_t, w.wo_t, w.wgu_t, w.wd_t})
                if (p) (void)hipFree(p);
        }
        for (void* p : s->k_pool) if (p) (void)hipFree(p);
        for (void* p : s->v_pool) if (p) (void)hipFree(p);
        if (s->d_k_pools) (void)hipFree(s->d_k_pools);
        if (s->d_v_pools) (void)hipFree(s->d_v_pools);
        if (s->w_ready) (void)hipEventDestroy(s->w_ready);
        delete s;
    }
    for (DevBuf* b : {&c->ws_h, &c->ws_qkv, &c->ws_attn, &c->ws_gu, &c->ws_act, &c->ws_x1, &c->ws_scratch, &c->ws_splitk, &c->ws_rs,
                      &c->ws_chain[0], &c->ws_chain[1]})
        if (b->p) (void)hipFree(b->p);
    for (auto& ms : c->meta) {
        if (ms.host) (void)hipHostFree(ms.host);
        if (ms.dev) (void)hipFree(ms.dev);
        if (ms.done) (void)hipEventDestroy(ms.done);
    }
    for (Lane& L : c->lane) {
        if (L.dev_staging) (void)hipFree(L.dev_staging);
        if (L.mv_meta_dev) (void)hipFree(L.mv_meta_dev);
        if (L.pinned) (void)hipHostFree(L.pinned);
        if (L.mv_meta_host) (void)hipHostFree(L.mv_meta_host);
        for (int i = 0; i < 2; ++i) if (L.mv_ev[i]) (void)hipEventDestroy(L.mv_ev[i]);
        if (L.side) (void)hipStreamDestroy(L.side);
        if (L.copy) (void)hipStreamDestroy(L.copy);
        L.hsa.shutdown();
        for (hipEvent_t e : L.copy_ev) if (e) (void)hipEventDestroy(e);
    }
    for (void* p : {(void*)c->d_rope, c->d_embed, c->d_gf, c->d_wlm_t, (void*)c->d_ids})
        if (p) (void)hipFree(p);
    for (DeferredFree& df : c->deferred) {
        for (void* p : df.ptrs) (void)hipFree(p);
        if (df.ev) (void)hipEventDestroy(df.ev);
    }
    for (HostLayer& hl : c->hw) if (hl.base) (void)hipHostFree(hl.base);
    if (c->w_staging.p) (void)hipFree(c->w_staging.p);
    if (c->wstream) (void)hipStreamDestroy(c->wstream);
    for (auto& r : c->prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    if (c->tier_pinned) (void)hipHostFree(c->tier);
    else free(c->tier);
    delete c;
    return SS_OK;
}

const char* ss_last_error(ss_ctx* c) { return c ? c->err.c_str() : "null context"; }

int ss_load_layer(ss_ctx* c, const ss_shard_desc* d, int layer, const ss_layer_weights* w) {
    if (!c) return SS_EINVAL;
    if (!w || !w->g1 || !w->wq || !w->wk || !w->wv || !w->wo || !w->g2 || !w->wg || !w->wu || !w->wd)
        return fail(c, SS_EINVAL, "null weight pointer");
    if (w->location != SS_HOST && w->location != SS_DEVICE) return fail(c, SS_EINVAL, "bad weight location");
    Shard* s = nullptr;
    int rc = get_shard(c, d, &s);
    if (rc) return rc;
    if (layer < d->layer_begin || layer >= d->layer_end) return fail(c, SS_EINVAL, "layer %d outside the shard", layer);
    LayerW& L = s->w[layer - d->layer_begin];
    const ss_model_cfg& m = c->m;
    const int H = m.hidden, dh = m.head_dim;
    const int nq = s->nq_l * dh, nkv = s->nkv_l * dh, F = s->f_l;
    const size_t es = c->es;
    auto alloc = [&](void** p, size_t bytes) -> int {
        if (!*p) HIP_TRY(c, hipMalloc(p, bytes));
        return SS_OK;
    };
    if ((rc = alloc(&L.wqkv_t, (size_t)(nq + 2 * nkv) * H * es))) return rc;
    if ((rc = alloc(&L.wo_t, (size_t)H * nq * es))) return rc;
    if ((rc = alloc(&L.wgu_t, (size_t)2 * F * H * es))) return rc;
    if ((rc = alloc(&L.wd_t, (size_t)H * F * es))) return rc;
    if ((rc = copy_vec(c, w->g1, w->location, H, &L.g1))) return rc;
    if ((rc = copy_vec(c, w->g2, w->location, H, &L.g2))) return rc;
    uint8_t* qkv = (uint8_t*)L.wqkv_t;
    const size_t qd = (size_t)m.n_q_heads * dh, kd = (size_t)m.n_kv_heads * dh;
    // the RMSNorm gains are folded into the matrices that read the normalised activations (Q, K, V: g1; gate, up: g2)
    if ((rc = slice_into(c, w->wq, w->location, H, qd, 0, H, s->q0 * dh, nq, qkv, nq, nq, 0, L.g1))) return rc;
    if ((rc = slice_into(c, w->wk, w->location, H, kd, 0, H, s->g0 * dh, nkv, qkv + (size_t)nq * H * es, nkv, nkv, 0, L.g1))) return rc;
    if ((rc = slice_into(c, w->wv, w->location, H, kd, 0, H, s->g0 * dh, nkv, qkv + (size_t)(nq + nkv) * H * es, nkv, nkv, 0, L.g1))) return rc;
    // Wo rows of this shard's heads -> Wo^T [H, nq]
    if ((rc = slice_into(c, w->wo, w->location, qd, H, (size_t)s->q0 * dh, nq, 0, H, L.wo_t, H, H, 0))) return rc;
    // gate / up: interleaved in blocks of 32 rows when the fused SwiGLU epilogue can run
    L.gu_interleaved = (c->dt != SS_F32) && !c->force_generic && (F % 32 == 0) && (H % 64 == 0);
    if (L.gu_interleaved) {
        if ((rc = slice_into(c, w->wg, w->location, H, m.ffn, 0, H, s->f0, F, L.wgu_t, 32, 64, 0, L.g2))) return rc;
        if ((rc = slice_into(c, w->wu, w->location, H, m.ffn, 0, H, s->f0, F, L.wgu_t, 32, 64, 32, L.g2))) return rc;
    } else {
        if ((rc = slice_into(c, w->wg, w->location, H, m.ffn, 0, H, s->f0, F, L.wgu_t, F, F, 0, L.g2))) return rc;
        if ((rc = slice_into(c, w->wu, w->location, H, m.ffn, 0, H, s->f0, F, L.wgu_t, F, F, F, L.g2))) return rc;
    }
    if ((rc = slice_into(c, w->wd, w->location, m.ffn, H, (size_t)s->f0, F, 0, H, L.wd_t, H, H, 0))) return rc;
    L.loaded = true;
    return SS_OK;
}

int ss_host_weights_put(ss_ctx* c, int layer, const ss_layer_weights* w) {
    if (!c) return SS_EINVAL;
    if (!w || !w->g1 || !w->wq || !w->wk || !w->wv || !w->wo || !w->g2 || !w->wg || !w->wu || !w->wd)
        return fail(c, SS_EINVAL, "null weight pointer");
    if (w->location != SS_HOST && w->location != SS_DEVICE) return fail(c, SS_EINVAL, "bad weight location");
    if (layer < 0 || layer >= c->m.n_layers) return fail(c, SS_EINVAL, "bad layer %d", layer);
    if (c->hw.empty()) c->hw.resize(c->m.n_layers);
    HostLayer& hl = c->hw[layer];
    if (!hl.base) {
        size_t total = 0;
        for (int i = 0; i < 9; ++i) {
            hl.off[i] = total;
            total += (tensor_elems(c->m, i) * c->es + 255) & ~(size_t)255;
        }
        HIP_TRY(c, hipHostMalloc((void**)&hl.base, total, hipHostMallocDefault));
    } else if (c->wstream) {
        HIP_TRY(c, hipStreamSynchronize(c->wstream));       // no reload is reading the copy that is replaced
    }
    const void* src[9] = {w->g1, w->wq, w->wk, w->wv, w->wo, w->g2, w->wg, w->wu, w->wd};
    for (int i = 0; i < 9; ++i) {
        const size_t bytes = tensor_elems(c->m, i) * c->es;
        if (w->location == SS_HOST) memcpy(hl.base + hl.off[i], src[i], bytes);
        else HIP_TRY(c, hipMemcpy(hl.base + hl.off[i], src[i], bytes, hipMemcpyDeviceToHost));
    }
    return SS_OK;
}

int ss_reshard_weights(ss_ctx* c, const ss_shard_desc* from, const ss_shard_desc* to, void* stream) {
    if (!c) return SS_EINVAL;
    if (!to) return fail(c, SS_EINVAL, "null target descriptor");
    Shard *sf = nullptr, *st = nullptr;
    int rc = get_shard(c, to, &st);
    if (rc) return rc;
    if (from && (rc = get_shard(c, from, &sf))) return rc;
    for (int l = to->layer_begin; l < to->layer_end; ++l)
        if ((size_t)l >= c->hw.size() || !c->hw[l].base)
            return fail(c, SS_ENOENT, "layer %d has no CPU copy (ss_host_weights_put)", l);
    if (!c->wstream) HIP_TRY(c, hipStreamCreateWithFlags(&c->wstream, hipStreamNonBlocking));
    if ((rc = release_deferred(c, false))) return rc;
    hipStream_t cs = (hipStream_t)stream;
    if (sf && sf != st) {
        // the old shard's buffers go once everything enqueued on the caller's stream so far has run
        if (sf->w_pending) {
            HIP_TRY(c, hipEventSynchronize(sf->w_ready));
            sf->w_pending = false;
        }
        DeferredFree df;
        for (LayerW& L : sf->w) {
            for (void** p : {&L.g1, &L.g2, &L.wqkv_t, &L.wo_t, &L.wgu_t, &L.wd_t})
                if (*p) { df.ptrs.push_back(*p); *p = nullptr; }
            L.loaded = false;
        }
        if (!df.ptrs.empty()) {
            HIP_TRY(c, hipEventCreateWithFlags(&df.ev, hipEventDisableTiming));
            HIP_TRY(c, hipEventRecord(df.ev, cs));
            c->deferred.push_back(std::move(df));
        }
    }
    // staging for the largest slice of the target
    {
        const size_t H = c->m.hidden;
        const size_t widest = std::max<size_t>((size_t)st->nq_l * c->m.head_dim, (size_t)st->f_l);
        const size_t need = H * widest * c->es;
        if (need > c->w_staging.cap) {
            HIP_TRY(c, hipStreamSynchronize(c->wstream));
            if (c->w_staging.p) HIP_TRY(c, hipFree(c->w_staging.p));
            c->w_staging.p = nullptr;
            c->w_staging.cap = 0;
            HIP_TRY(c, hipMalloc(&c->w_staging.p, need));
            c->w_staging.cap = need;
        }
    }
    // a reload into buffers that layer calls already enqueued on the caller's stream still read comes after them
    {
        hipEvent_t e = nullptr;
        HIP_TRY(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
        hipError_t er = hipEventRecord(e, cs);
        if (er == hipSuccess) er = hipStreamWaitEvent(c->wstream, e, 0);
        (void)hipEventDestroy(e);
        if (er != hipSuccess) return fail(c, SS_EHIP, "weight re-shard ordering: %s", hipGetErrorString(er));
    }
    for (int ll = 0; ll < st->n_layers_l; ++ll)
        if ((rc = reload_layer(c, st, ll))) return rc;
    if (!st->w_ready) HIP_TRY(c, hipEventCreateWithFlags(&st->w_ready, hipEventDisableTiming));
    HIP_TRY(c, hipEventRecord(st->w_ready, c->wstream));
    st->w_pending = true;
    return SS_OK;
}

int ss_weights_wait(ss_ctx* c, const ss_shard_desc* d) {
    if (!c) return SS_EINVAL;
    Shard* s = nullptr;
    int rc = get_shard(c, d, &s);
    if (rc) return rc;
    if (s->w_pending) {
        HIP_TRY(c, hipEventSynchronize(s->w_ready));
        s->w_pending = false;
    }
    return SS_OK;
}

int64_t ss_weights_shard_bytes(ss_ctx* c, const ss_shard_desc* d) {
    if (!c) return SS_EINVAL;
    Shard* s = nullptr;
    if (get_shard(c, d, &s)) return SS_EINVAL;
    const int64_t H = c->m.hidden, dh = c->m.head_dim;
    const int64_t per_layer = H * (s->nq_l + 2 * s->nkv_l) * dh + s->nq_l * dh * H + 3 * H * s->f_l + 2 * H;
    return per_layer * s->n_layers_l * (int64_t)c->es;
}

int ss_weights_read(ss_ctx* c, const ss_shard_desc* d, int layer, int which, void* host_out) {
    if (!c || !host_out) return SS_EINVAL;
    Shard* s = nullptr;
    int rc = get_shard(c, d, &s);
    if (rc) return rc;
    if (layer < d->layer_begin || layer >= d->layer_end) return fail(c, SS_EINVAL, "layer %d outside the shard", layer);
    if (which < 0 || which > SS_W_D) return fail(c, SS_EINVAL, "bad tensor index %d", which);
    const LayerW& L = s->w[layer - d->layer_begin];
    if (!L.loaded) return fail(c, SS_ENOENT, "layer %d not loaded for this shard", layer);
    if ((rc = ss_weights_wait(c, d))) return rc;
    HIP_TRY(c, hipDeviceSynchronize());
    const size_t es = c->es, H = c->m.hidden, dh = c->m.head_dim;
    const size_t nq = (size_t)s->nq_l * dh, nkv = (size_t)s->nkv_l * dh, F = s->f_l;
    uint8_t* out = (uint8_t*)host_out;
    if (which == SS_W_G1 || which == SS_W_G2) {
        HIP_TRY(c, hipMemcpy(out, which == SS_W_G1 ? L.g1 : L.g2, H * es, hipMemcpyDeviceToHost));
        return SS_OK;
    }
    // device image -> host, then back to [in, out] orientation element by element
    const void* dev = nullptr;
    size_t rows_t = 0, cols_t = 0;        // device image [rows_t][cols_t]
    switch (which) {
        case SS_W_Q: case SS_W_K: case SS_W_V: dev = L.wqkv_t; rows_t = nq + 2 * nkv; cols_t = H; break;
        case SS_W_O: dev = L.wo_t; rows_t = H; cols_t = nq; break;
        case SS_W_G: case SS_W_U: dev = L.wgu_t; rows_t = 2 * F; cols_t = H; break;
        default: dev = L.wd_t; rows_t = H; cols_t = F; break;
    }
    std::vector<uint8_t> img(rows_t * cols_t * es);
    HIP_TRY(c, hipMemcpy(img.data(), dev, img.size(), hipMemcpyDeviceToHost));
    auto put = [&](size_t o, size_t r, size_t cc) { memcpy(out + o * es, img.data() + (r * cols_t + cc) * es, es); };
    if (which == SS_W_Q || which == SS_W_K || which == SS_W_V) {
        const size_t n = which == SS_W_Q ? nq : nkv, r0 = which == SS_W_Q ? 0 : (which == SS_W_K ? nq : nq + nkv);
        for (size_t h = 0; h < H; ++h)
            for (size_t j = 0; j < n; ++j) put(h * n + j, r0 + j, h);
    } else if (which == SS_W_O) {
        for (size_t j = 0; j < nq; ++j)
            for (size_t h = 0; h < H; ++h) put(j * H + h, h, j);
    } else if (which == SS_W_G || which == SS_W_U) {
        const bool up = which == SS_W_U;
        for (size_t h = 0; h < H; ++h)
            for (size_t j = 0; j < F; ++j) {
                const size_t r = L.gu_interleaved ? (j / 32) * 64 + (j % 32) + (up ? 32 : 0) : j + (up ? F : 0);
                put(h * F + j, r, h);
            }
    } else {
        for (size_t f = 0; f < F; ++f)
            for (size_t h = 0; h < H; ++h) put(f * H + h, h, f);
    }
    return SS_OK;
}

int ss_layer_prefill(ss_ctx* c, const ss_shard_desc* d, int layer, int phase, const ss_batch* b, const void* x_in,
                     void* out, void* stream) {
    return layer_call(c, d, layer, phase, b, x_in, out, stream, false);
}

int ss_layer_decode(ss_ctx* c, const ss_shard_desc* d, int layer, int phase, const ss_batch* b, const void* x_in,
                    void* out, void* stream) {
    return layer_call(c, d, layer, phase, b, x_in, out, stream, true);
}

int ss_layers_prefill(ss_ctx* c, const ss_shard_desc* d, const ss_batch* b, const void* x_in, void* out, void* stream) {
    return layers_call(c, d, b, x_in, out, stream, false);
}

int ss_layers_decode(ss_ctx* c, const ss_shard_desc* d, const ss_batch* b, const void* x_in, void* out, void* stream) {
    return layers_call(c, d, b, x_in, out, stream, true);
}

int ss_kv_swap(ss_ctx* c, const ss_shard_desc* d, int dir, const int64_t* seq_ids, int n, void* stream) {
    if (!c) return SS_EINVAL;
    if (n < 0 || (n > 0 && !seq_ids)) return fail(c, SS_EINVAL, "bad sequence list");
    if (dir != SS_OUT && dir != SS_IN) return fail(c, SS_EINVAL, "bad direction %d", dir);
    if (!c->tier || !c->slot_bytes) return fail(c, SS_EINVAL, "context was created without a host tier / pinned ring");
    Shard* s = nullptr;
    int rc = get_shard(c, d, &s);
    if (rc) return rc;
    if ((rc = ensure_pools(c, s))) return rc;
    if (n == 0) return SS_OK;
    Job job;
    job.dir = dir;
    job.sh = s;
    if (dir == SS_OUT) {
        for (int i = 0; i < n; ++i) {
            auto it = s->seqs.find(seq_ids[i]);
            if (it == s->seqs.end()) return fail(c, SS_ENOENT, "sequence %lld not resident in this shard", (long long)seq_ids[i]);
            auto ts = c->tier_slots.find(seq_ids[i]);
            if (ts != c->tier_slots.end() && ts->second.len != it->second.len)
                return fail(c, SS_EINVAL, "sequence %lld is in the tier with length %d, shard holds %d",
                            (long long)seq_ids[i], ts->second.len, it->second.len);
        }
        std::vector<int64_t> placed;
        for (int i = 0; i < n; ++i) {
            const SeqState& st = s->seqs[seq_ids[i]];
            auto ts = c->tier_slots.find(seq_ids[i]);
            if (ts == c->tier_slots.end()) {
                size_t off = 0;
                if (!tier_alloc(c, seq_tier_bytes(c, st.len), &off)) {
                    for (int64_t id : placed) {     // all or nothing
                        tier_release(c, c->tier_slots[id].off, seq_tier_bytes(c, c->tier_slots[id].len));
                        c->tier_slots.erase(id);
                    }
                    return fail(c, SS_ENOMEM, "host tier full: sequence %lld needs %zu bytes, %zu in use of %zu",
                                (long long)seq_ids[i], seq_tier_bytes(c, st.len), c->tier_used, c->tier_cap);
                }
                ts = c->tier_slots.emplace(seq_ids[i], TierSlot{off, st.len}).first;
                placed.push_back(seq_ids[i]);
            }
        }
        for (int i = 0; i < n; ++i) {
            const SeqState& st = s->seqs[seq_ids[i]];
            job.seqs.push_back({seq_ids[i], st.len, st.pages, c->tier_slots[seq_ids[i]].off});
        }
    } else {
        for (int i = 0; i < n; ++i) {
            if (!c->tier_slots.count(seq_ids[i]))
                return fail(c, SS_ENOENT, "sequence %lld not in the host tier", (long long)seq_ids[i]);
            if (s->seqs.count(seq_ids[i]))
                return fail(c, SS_EINVAL, "sequence %lld already resident in this shard", (long long)seq_ids[i]);
        }
        {
            std::vector<int32_t> lens(n);
            for (int i = 0; i < n; ++i) {
                lens[i] = c->tier_slots[seq_ids[i]].len;
                for (int j = 0; j < i; ++j)
                    if (seq_ids[j] == seq_ids[i]) return fail(c, SS_EINVAL, "sequence %lld listed twice", (long long)seq_ids[i]);
            }
            if ((rc = check_new_seqs_fit(c, s, lens.data(), n))) return rc;
        }
        for (int i = 0; i < n; ++i) {
            const TierSlot& ts = c->tier_slots[seq_ids[i]];
            if ((rc = ensure_pages(c, s, seq_ids[i], ts.len))) return rc;
            const SeqState& st = s->seqs[seq_ids[i]];
            job.seqs.push_back({seq_ids[i], ts.len, st.pages, ts.off});
        }
    }
    return enqueue_job(c, std::move(job), (hipStream_t)stream);
}

int ss_kv_reshard(ss_ctx* c, const ss_shard_desc* from, const ss_shard_desc* to, const int64_t* seq_ids, int n,
                  void* stream) {
    int rc = ss_kv_swap(c, from, SS_OUT, seq_ids, n, stream);
    if (rc) return rc;
    return ss_kv_swap(c, to, SS_IN, seq_ids, n, stream);
}

int ss_sync(ss_ctx* c) {
    if (!c) return SS_EINVAL;
    wait_idle(c);
    for (Lane& L : c->lane) HIP_TRY(c, hipStreamSynchronize(L.side));
    if (c->wstream) HIP_TRY(c, hipStreamSynchronize(c->wstream));
    {
        int rc = release_deferred(c, false);
        if (rc) return rc;
    }
    std::lock_guard<std::mutex> lk(c->mu);
    if (c->worker_rc) {
        const int rc = c->worker_rc;
        c->err = "KV mover: " + c->worker_err;
        c->worker_rc = 0;
        c->worker_err.clear();
        return rc;
    }
    return SS_OK;
}

int64_t ss_kv_jobs_issued(ss_ctx* c) {
    if (!c) return SS_EINVAL;
    std::lock_guard<std::mutex> lk(c->mu);
    return c->jobs_issued;
}

int ss_kv_wait(ss_ctx* c, int64_t n_jobs) {
    if (!c) return SS_EINVAL;
    std::unique_lock<std::mutex> lk(c->mu);
    c->cv_idle.wait(lk, [&] { return c->jobs_done >= n_jobs || c->jobs_done >= c->jobs_issued; });
    if (c->worker_rc) {
        const int rc = c->worker_rc;
        c->err = "KV mover: " + c->worker_err;
        c->worker_rc = 0;
        c->worker_err.clear();
        return rc;
    }
    return SS_OK;
}

int ss_kv_free(ss_ctx* c, const ss_shard_desc* d, const int64_t* seq_ids, int n) {
    if (!c) return SS_EINVAL;
    Shard* s = nullptr;
    int rc = get_shard(c, d, &s);
    if (rc) return rc;
    wait_seqs_idle(c, s, seq_ids, n);
    for (int i = 0; i < n; ++i)
        if (!s->seqs.count(seq_ids[i])) return fail(c, SS_ENOENT, "sequence %lld not resident", (long long)seq_ids[i]);
    for (int i = 0; i < n; ++i) {
        auto it = s->seqs.find(seq_ids[i]);
        if (it == s->seqs.end()) continue;   // listed twice
        for (int32_t p : it->second.pages) s->free_pages.push(p);
        s->seqs.erase(it);
    }
    s->version++;
    return SS_OK;
}

int ss_host_tier_release(ss_ctx* c, const int64_t* seq_ids, int n) {
    if (!c) return SS_EINVAL;
    wait_seqs_idle(c, nullptr, seq_ids, n);
    for (int i = 0; i < n; ++i)
        if (!c->tier_slots.count(seq_ids[i])) return fail(c, SS_ENOENT, "sequence %lld not in the host tier", (long long)seq_ids[i]);
    for (int i = 0; i < n; ++i) {
        auto it = c->tier_slots.find(seq_ids[i]);
        if (it == c->tier_slots.end()) continue;   // listed twice
        tier_release(c, it->second.off, seq_tier_bytes(c, it->second.len));
        c->tier_slots.erase(it);
    }
    return SS_OK;
}

static int xfer_dev(ss_ctx* c, const ss_shard_desc* d, const int64_t* seq_ids, const int32_t* lens, int n, void* staging,
                    void* stream, bool import) {
    if (!c) return SS_EINVAL;
    if (n < 0 || (n > 0 && (!seq_ids || !staging))) return fail(c, SS_EINVAL, "bad arguments");
    Shard* s = nullptr;
    int rc = get_shard(c, d, &s);
    if (rc) return rc;
    if ((rc = ensure_pools(c, s))) return rc;
    if (n == 0) return SS_OK;
    std::vector<SeqJob> seqs;
    if (import) {
        if (!lens) return fail(c, SS_EINVAL, "import needs lengths");
        for (int i = 0; i < n; ++i) {
            if (lens[i] <= 0) return fail(c, SS_EINVAL, "sequence %d has length %d", i, lens[i]);
            if (s->seqs.count(seq_ids[i])) return fail(c, SS_EINVAL, "sequence %lld already resident", (long long)seq_ids[i]);
        }
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < i; ++j)
                if (seq_ids[j] == seq_ids[i]) return fail(c, SS_EINVAL, "sequence %lld listed twice", (long long)seq_ids[i]);
        if ((rc = check_new_seqs_fit(c, s, lens, n))) return rc;
        for (int i = 0; i < n; ++i) {
            if ((rc = ensure_pages(c, s, seq_ids[i], lens[i]))) return rc;
            seqs.push_back({seq_ids[i], lens[i], s->seqs[seq_ids[i]].pages, 0});
        }
    } else {
        for (int i = 0; i < n; ++i) {
            auto it = s->seqs.find(seq_ids[i]);
            if (it == s->seqs.end()) return fail(c, SS_ENOENT, "sequence %lld not resident", (long long)seq_ids[i]);
            seqs.push_back({seq_ids[i], it->second.len, it->second.pages, 0});
        }
    }
    const std::vector<Unit> units = make_units(c, s, seqs);
    hipStream_t st = (hipStream_t)stream;
    // metadata goes through a pageable image and a synchronous copy; the device
    // image must outlive the kernels, so it is only rewritten after they finished
    HIP_TRY(c, hipStreamSynchronize(st));
    std::vector<uint8_t> img(c->mv_meta_cap / 2);
    static_assert(sizeof(size_t) == 8, "64-bit only");
    wait_idle(c);   // shares lane 0's device metadata region with the mover, which is idle from here on
    uint8_t* md = c->lane[0].mv_meta_dev;
    size_t stage_off = 0;
    for (size_t u0 = 0; u0 < units.size(); u0 += 32768) {
        const size_t u1 = std::min(units.size(), u0 + 32768);
        ssk::RepackUnits ru{};
        const size_t mbytes = build_units(c, s, seqs, units, u0, u1, img.data(), md, img.size(), &ru);
        if (!mbytes) return fail(c, SS_ENOMEM, "repack metadata region too small");
        HIP_TRY(c, hipMemcpy(md, img.data(), mbytes, hipMemcpyHostToDevice));
        uint8_t* stg = (uint8_t*)staging + stage_off;
        {
            ProfScope ps(c, 3, st);
            if (import)
                K_TRY(c, SSK_CALL(c, kv_scatter, s->d_k_pools, s->d_v_pools, s->nkv_l, c->m.head_dim, c->m.page_size, ru, stg, st));
            else
                K_TRY(c, SSK_CALL(c, kv_gather, s->d_k_pools, s->d_v_pools, s->nkv_l, c->m.head_dim, c->m.page_size, ru, stg, st));
        }
        for (size_t u = u0; u < u1; ++u) stage_off += units[u].bytes;
        if (u1 < units.size()) HIP_TRY(c, hipStreamSynchronize(st));
    }
    return SS_OK;
}

int ss_kv_export_dev(ss_ctx* c, const ss_shard_desc* d, const int64_t* seq_ids, int n, void* staging, void* stream) {
    return xfer_dev(c, d, seq_ids, nullptr, n, staging, stream, false);
}

int ss_kv_import_dev(ss_ctx* c, const ss_shard_desc* d, const int64_t* seq_ids, const int32_t* lens, int n,
                     const void* staging, void* stream) {
    return xfer_dev(c, d, seq_ids, lens, n, const_cast<void*>(staging), stream, true);
}

int ss_kv_page_table(ss_ctx* c, const ss_shard_desc* d, int64_t seq, int32_t* pages, int32_t* n_inout) {
    if (!c || !n_inout) return SS_EINVAL;
    Shard* s = nullptr;
    int rc = get_shard(c, d, &s);
    if (rc) return rc;
    auto it = s->seqs.find(seq);
    if (it == s->seqs.end()) return fail(c, SS_ENOENT, "sequence %lld not resident", (long long)seq);
    const int32_t have = (int32_t)it->second.pages.size();
    if (pages) std::copy(it->second.pages.begin(), it->second.pages.begin() + std::min(have, *n_inout), pages);
    *n_inout = have;
    return SS_OK;
}

int ss_kv_seq_len(ss_ctx* c, const ss_shard_desc* d, int64_t seq, int32_t* len_out) {
    if (!c || !len_out) return SS_EINVAL;
    Shard* s = nullptr;
    int rc = get_shard(c, d, &s);
    if (rc) return rc;
    auto it = s->seqs.find(seq);
    if (it == s->seqs.end()) return fail(c, SS_ENOENT, "sequence %lld not resident", (long long)seq);
    *len_out = it->second.len;
    return SS_OK;
}

int ss_kv_read(ss_ctx* c, const ss_shard_desc* d, int64_t seq, int layer, void* host_out) {
    if (!c || !host_out) return SS_EINVAL;
    Shard* s = nullptr;
    int rc = get_shard(c, d, &s);
    if (rc) return rc;
    if (layer < d->layer_begin || layer >= d->layer_end) return fail(c, SS_EINVAL, "layer %d outside the shard", layer);
    auto it = s->seqs.find(seq);
    if (it == s->seqs.end()) return fail(c, SS_ENOENT, "sequence %lld not resident", (long long)seq);
    if (!s->pools_ready) return fail(c, SS_ENOENT, "shard has no cache yet");
    wait_idle(c);
    HIP_TRY(c, hipDeviceSynchronize());
    std::vector<SeqJob> seqs{{seq, it->second.len, it->second.pages, 0}};
    std::vector<Unit> units{{0, layer - d->layer_begin, (size_t)2 * s->nkv_l * it->second.len * c->m.head_dim * c->es}};
    std::vector<uint8_t> img(1 << 20);
    ssk::RepackUnits ru{};
    const size_t mbytes = build_units(c, s, seqs, units, 0, 1, img.data(), c->lane[0].mv_meta_dev, img.size(), &ru);
    if (!mbytes) return fail(c, SS_ENOMEM, "sequence too long for the inspection path");
    HIP_TRY(c, hipMemcpy(c->lane[0].mv_meta_dev, img.data(), mbytes, hipMemcpyHostToDevice));
    void* tmp = nullptr;
    HIP_TRY(c, hipMalloc(&tmp, units[0].bytes));
    hipError_t e = SSK_CALL(c, kv_gather, s->d_k_pools, s->d_v_pools, s->nkv_l, c->m.head_dim, c->m.page_size, ru, tmp, 0);
    if (e == hipSuccess) e = hipMemcpy(host_out, tmp, units[0].bytes, hipMemcpyDeviceToHost);
    (void)hipFree(tmp);
    if (e != hipSuccess) return fail(c, SS_EHIP, "kv read: %s", hipGetErrorString(e));
    return SS_OK;
}

int ss_host_tier_read(ss_ctx* c, int64_t seq, int layer, void* host_out) {
    if (!c || !host_out) return SS_EINVAL;
    if (layer < 0 || layer >= c->m.n_layers) return fail(c, SS_EINVAL, "bad layer %d", layer);
    auto it = c->tier_slots.find(seq);
    if (it == c->tier_slots.end()) return fail(c, SS_ENOENT, "sequence %lld not in the host tier", (long long)seq);
    wait_idle(c);
    const size_t per_layer = (size_t)2 * c->m.n_kv_heads * it->second.len * c->m.head_dim * c->es;
    memcpy(host_out, c->tier + it->second.off + per_layer * layer, per_layer);
    return SS_OK;
}

int64_t ss_host_tier_used_bytes(ss_ctx* c) { return c ? (int64_t)c->tier_used : -1; }

int64_t ss_kv_free_pages(ss_ctx* c, const ss_shard_desc* d) {
    if (!c) return SS_EINVAL;
    Shard* s = nullptr;
    int rc = get_shard(c, d, &s);
    if (rc) return rc;
    if (!s->pools_ready) return c->rt.gpu_kv_pages;
    return (int64_t)s->free_pages.size();
}

int ss_load_head(ss_ctx* c, const void* embed, const void* gf, const void* wlm) {
    if (!c || !embed || !gf || !wlm) return SS_EINVAL;
    if (c->m.vocab <= 0) return fail(c, SS_EINVAL, "model has no vocabulary");
    const size_t V = c->m.vocab, H = c->m.hidden;
    int rc;
    if ((rc = copy_vec(c, embed, SS_HOST, V * H, &c->d_embed))) return rc;
    if ((rc = copy_vec(c, gf, SS_HOST, H, &c->d_gf))) return rc;
    if (!c->d_wlm_t) HIP_TRY(c, hipMalloc(&c->d_wlm_t, V * H * c->es));
    return slice_into(c, wlm, SS_HOST, H, V, 0, (int)H, 0, (int)V, c->d_wlm_t, (int)V, (int)V, 0);
}

int ss_embed(ss_ctx* c, const int32_t* ids, int n, void* x_out, void* stream) {
    if (!c || !ids || !x_out || n <= 0) return SS_EINVAL;
    if (!c->d_embed) return fail(c, SS_EINVAL, "head weights not loaded");
    for (int i = 0; i < n; ++i)
        if (ids[i] < 0 || ids[i] >= c->m.vocab) return fail(c, SS_EINVAL, "token id %d out of range", ids[i]);
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(c, hipStreamSynchronize(st));
    if ((size_t)n > c->d_ids_cap) {
        if (c->d_ids) HIP_TRY(c, hipFree(c->d_ids));
        c->d_ids = nullptr;
        HIP_TRY(c, hipMalloc((void**)&c->d_ids, sizeof(int32_t) * (size_t)n * 2));
        c->d_ids_cap = (size_t)n * 2;
    }
    HIP_TRY(c, hipMemcpy(c->d_ids, ids, sizeof(int32_t) * (size_t)n, hipMemcpyHostToDevice));
    K_TRY(c, SSK_CALL(c, embed_rows, c->d_embed, c->d_ids, x_out, n, c->m.hidden, st));
    return SS_OK;
}

int ss_lm_head(ss_ctx* c, const void* x, int n, float* logits, void* stream) {
    if (!c || !x || !logits || n <= 0) return SS_EINVAL;
    if (!c->d_wlm_t) return fail(c, SS_EINVAL, "head weights not loaded");
    hipStream_t st = (hipStream_t)stream;
    int rc = ensure_buf(c, c->ws_h, (size_t)n * c->m.hidden * c->es);
    if (rc) return rc;
    K_TRY(c, SSK_CALL(c, rmsnorm, x, c->d_gf, c->ws_h.p, n, c->m.hidden, c->m.rms_eps, st));
    K_TRY(c, SSK_CALL(c, gemm_nt, c->ws_h.p, c->m.hidden, c->d_wlm_t, logits, c->m.vocab, nullptr, n, c->m.vocab,
                          c->m.hidden, ssk::EPI_STORE_F32, c->force_generic, st, (float*)c->ws_splitk.p, c->ws_splitk.cap));
    return SS_OK;
}

int ss_lm_head_noalloc(ss_ctx* c, const void* x, int n, float* logits, void* stream) {
    if (!c || !x || !logits || n <= 0) return SS_EINVAL;
    if (!c->d_wlm_t) return fail(c, SS_EINVAL, "head weights not loaded");
    uint8_t* base = (uint8_t*)g_noalloc_scratch[c->rt.device];
    if (!base) return fail(c, SS_EHIP, "no fixed scratch on device %d", c->rt.device);
    const size_t rows_bytes = (size_t)n * c->m.hidden * c->es;
    if (rows_bytes > NOALLOC_ROWS_BYTES)
        return fail(c, SS_EINVAL, "ss_lm_head_noalloc: %d rows of %d elements need %zu bytes of scratch, the fixed limit is %zu",
                    n, c->m.hidden, rows_bytes, NOALLOC_ROWS_BYTES);
    hipStream_t st = (hipStream_t)stream;
    void* rows = base;
    float* partials = (float*)(base + NOALLOC_ROWS_BYTES);
    const size_t partial_bytes = NOALLOC_SCRATCH_BYTES - NOALLOC_ROWS_BYTES;
    // nothing in the scratch has to start at zero: the norm writes every row before the GEMM reads it, and the
    // GEMM writes every partial sum it later adds up
    K_TRY(c, SSK_CALL(c, rmsnorm, x, c->d_gf, rows, n, c->m.hidden, c->m.rms_eps, st));
    K_TRY(c, SSK_CALL(c, gemm_nt, rows, c->m.hidden, c->d_wlm_t, logits, c->m.vocab, nullptr, n, c->m.vocab,
                          c->m.hidden, ssk::EPI_STORE_F32, c->force_generic, st, partials, partial_bytes));
    return SS_OK;
}

int ss_get_config(ss_ctx* c, ss_model_cfg* model_out, ss_runtime_cfg* rt_out) {
    if (!c) return SS_EINVAL;
    if (model_out) *model_out = c->m;
    if (rt_out) *rt_out = c->rt;
    return SS_OK;
}

// for the offline loop (ss_offline.hip), which reports through the context's error text
int ss_offline_set_error(ss_ctx* c, const char* text) {
    if (!c || !text) return SS_EINVAL;
    c->err = text;
    return SS_OK;
}

int ss_prof_enable(ss_ctx* c, int on) {
    if (!c) return SS_EINVAL;
    c->prof_on = on != 0;
    return SS_OK;
}

int ss_prof_reset(ss_ctx* c) {
    if (!c) return SS_EINVAL;
    wait_idle(c);
    HIP_TRY(c, hipDeviceSynchronize());
    std::lock_guard<std::mutex> lk(c->prof_mu);
    for (auto& r : c->prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    c->prof.clear();
    return SS_OK;
}

int ss_prof_read(ss_ctx* c, int cls, double* total_ms_out, int64_t* n_out) {
    if (!c || !total_ms_out || !n_out) return SS_EINVAL;
    wait_idle(c);
    HIP_TRY(c, hipDeviceSynchronize());
    std::lock_guard<std::mutex> lk(c->prof_mu);
    double tot = 0;
    int64_t cnt = 0;
    for (auto& r : c->prof) {
        if (r.cls != cls) continue;
        float ms = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&ms, r.a, r.b));
        tot += ms;
        ++cnt;
    }
    *total_ms_out = tot;
    *n_out = cnt;
    return SS_OK;
}

}  // extern "C"
