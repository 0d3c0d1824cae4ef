"""Benchmark of the hot path on one MI355X.

The headline step (no flags: configuration 5, the largest one a single GPU holds) is one pass of the whole
path over one batch of the LLaMA-3-70B-shape pipeline slice (bf16, ten full layers, 17 GB of weights):
    layer_prefill of 64 prompts (lengths lognormal(7, 0.6) clipped to [128, 4096], 68 044 tokens) through the
        ten layers of the slice,
    kv_reshard of those prompts' caches (2.79 GB) to the k = 8 head-sharded decode layout: pages -> heads-major
        staging -> page-locked host tier -> pages of the decode shard, on the side streams, overlapped with the
        prefill of the next batch.
value = prompt tokens through the slice per second, everything resident in HBM when the timed region starts.
`--config 2|3|4` put the headline on the other configurations (2: prefill + re-shard + decode of one 7B-shape
layer; 3: 13B-shape pipeline prefill + k = 4 shard decode; 4: the 70B-shape k = 8 GQA shard decode); `--config 1`
runs the tiny fp32 model (prefill + 8 greedy steps).

Prints ONE JSON line.  `roofline` is the prefill GEMM class of the headline configuration (MFMA-bound; for
configuration 4, which has no prefill, the decode attention); `rooflines` holds every bounded kernel class of
configurations 2-5 as "<config>.<class>", each timed with HIP events on the stream its kernels are launched on.
`cpu_baseline` times the CPU oracle on a bounded sample of the headline workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # dense bf16 MFMA, MI355X
PEAK_HBM_GBS = 8000.0

CLS_GEMM, CLS_PATTN, CLS_DATTN, CLS_REPACK, CLS_OTHER = 0, 1, 2, 3, 4


def measured_traffic():
    """HBM-side bytes per layer call (per launch for the repack) from the rocprofv3 --pmc runs that
    `python -m paper_2503_06433_amd.profile_summary` condensed into bench_traffic.json ({} if absent)."""
    path = os.path.join(ROOT, "bench_traffic.json")
    if not os.path.exists(path):
        return {}
    with open(path) as f:
        return json.load(f)


def oracle_threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] + [1]))
    except Exception:
        return int(os.cpu_count() or 1)


def host_weights(dev_w, wl, hz, dtype):
    return {k: wl.storage_to_f64(hz.to_raw(v, dtype), dtype) for k, v in dev_w.items()}


def cpu_baseline_layer(work, vals, wl, budget_flop, n_decode, layers_in_step, seed):
    """Times the oracle as it stands on a bounded sample: one layer over the shortest prompts of the workload
    (as many as fit `budget_flop` of GEMM work) and, when the workload decodes, `n_decode` decode sequences.
    The rate is scaled to the metric's unit: tokens through all `layers_in_step` layers of the step per second."""
    from oracle import layer_math as lm
    cfg = work.cfg
    secs, toks, parts = 0.0, 0, []
    if work.prefill_lens is not None:
        per_tok = 2.0 * cfg.layer_params()
        lens = []
        for i in np.argsort(work.prefill_lens):
            n = int(work.prefill_lens[i])
            if lens and (sum(lens) + n) * per_tok > budget_flop:
                break
            lens.append(n)
        T = sum(lens)
        xv, _ = wl.make_activations((T, cfg.hidden), seed, cfg.dtype)
        t0 = time.perf_counter()
        lm.layer_forward(cfg, vals, xv, [(i, n, 0) for i, n in enumerate(lens)], lm.KVCache(cfg), 0)
        secs += time.perf_counter() - t0
        toks += T
        parts.append("prefill of the %d shortest prompts (%d tokens)" % (len(lens), T))
    if work.decode_kv_lens is not None and n_decode:
        k = work.k
        dlens = [int(v) for v in work.decode_kv_lens[:n_decode]]
        rng = np.random.default_rng(seed + 1)
        cache = lm.KVCache(cfg)
        for i, n in enumerate(dlens):            # caches are inputs: filled outside the timed region
            cache.ensure(i, n + 1)
            cache.data[i][:] = rng.standard_normal(cache.data[i].shape)
        dx, _ = wl.make_activations((n_decode, cfg.hidden), seed + 2, cfg.dtype)
        batch = [(i, 1, n) for i, n in enumerate(dlens)]
        t0 = time.perf_counter()
        o = lm.attn_block(cfg, vals, dx, batch, cache, 0, k, 0)
        lm.mlp_block(cfg, vals, dx + o, k, 0)
        secs += time.perf_counter() - t0
        toks += n_decode
        parts.append("decode of %d sequences%s" % (n_decode, " (shard 0 of %d)" % k if k > 1 else ""))
    return {"value": toks / (secs * layers_in_step), "unit": "tokens/s", "cores": oracle_threads(), "kind": "oracle",
            "sample": " + ".join(parts) + ", one layer in fp64 numpy; rate divided by the %d layer(s) of a step"
                      % layers_in_step,
            "seconds": secs}


# ----------------------------------------------------------------------------------------------------------
class Bench:
    def __init__(self, args, torch, wl, ss, hz):
        self.args, self.torch, self.wl, self.ss, self.hz = args, torch, wl, ss, hz
        self.stream = torch.cuda.current_stream().cuda_stream
        self.traffic = measured_traffic()
        self.rooflines = {}

    # ---- helpers
    def timed(self, ctx, fn, reps):
        """Per-class kernel time over `reps` calls of fn: {class: (total ms, launches)}."""
        ctx.prof_reset()
        ctx.prof_enable(True)
        for _ in range(reps):
            fn()
        self.torch.cuda.synchronize()
        ctx.sync()
        ctx.prof_enable(False)
        return {c: ctx.prof_read(c) for c in range(5)}

    def mfma(self, flops_per_call, ms_total, calls, key):
        a = flops_per_call * calls / (ms_total * 1e-3) / 1e12 if ms_total > 0 else 0.0
        return {"bound": "mfma", "achieved": a, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": a / PEAK_BF16_TFLOPS,
                "traffic": self.traffic.get(key), "avg_ms_per_call": ms_total / max(calls, 1)}

    def hbm(self, bytes_per_call, ms_total, calls, key):
        a = bytes_per_call * calls / (ms_total * 1e-3) / 1e9 if ms_total > 0 else 0.0
        return {"bound": "hbm", "achieved": a, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": a / PEAK_HBM_GBS,
                "traffic": self.traffic.get(key), "avg_ms_per_call": ms_total / max(calls, 1)}

    def weights_on_device(self, cfg, seed):
        return self.wl.device_layer_weights(cfg, seed)

    def prefill_classes(self, tag, ctx, desc, layer, ids, lens, x, y, reps, k=1):
        """Kernel classes of one prefill layer call (pages are given back after every call)."""
        cfg_T = sum(lens)
        zeros = [0] * len(ids)

        def fn():
            ctx.layer_prefill(desc, layer, self.ss.SS_BOTH, ids, lens, zeros, x, y, self.stream)
            ctx.kv_free(desc, ids)

        fn()
        pf = self.timed(ctx, fn, reps)
        m = ctx.model
        W = m.hidden * (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim + m.n_q_heads * m.head_dim * m.hidden + 3 * m.hidden * m.ffn
        self.rooflines[tag + ".prefill_gemms"] = self.mfma(2.0 * W / k * cfg_T, pf[CLS_GEMM][0], reps, tag + ".prefill_gemms")
        self.rooflines[tag + ".prefill_attention"] = self.mfma(
            2.0 * m.n_q_heads * m.head_dim * float(sum(n * n for n in lens)), pf[CLS_PATTN][0], reps, tag + ".prefill_attention")
        call_ms = sum(v[0] for v in pf.values()) / reps
        return {"prefill_call_ms": call_ms, "prefill_tokens_per_s": cfg_T / (call_ms * 1e-3),
                "prefill_other_kernels_ms": pf[CLS_OTHER][0] / reps}

    def decode_classes(self, tag, ctx, desc, layer, ids, lens, x, y, reps, k, phases_fused):
        ss = self.ss

        def fn():
            if phases_fused:
                ctx.layer_decode(desc, layer, ss.SS_BOTH, ids, lens, x, y, self.stream)
            else:       # a k > 1 shard returns partials: the two phases are separate calls (the all-reduce sits between)
                ctx.layer_decode(desc, layer, ss.SS_ATTN, ids, lens, x, y, self.stream)
                ctx.layer_decode(desc, layer, ss.SS_MLP, ids, lens, x, y2, self.stream)

        y2 = self.torch.empty_like(y)
        fn()
        dc = self.timed(ctx, fn, reps)
        m = ctx.model
        B = len(ids)
        kv_tok = 2 * (m.n_kv_heads // k) * m.head_dim * 2
        W = m.hidden * (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim + m.n_q_heads * m.head_dim * m.hidden + 3 * m.hidden * m.ffn
        attn_bytes = float(sum(lens) + B) * kv_tok + B * 4.0 * (m.n_q_heads // k) * m.head_dim
        self.rooflines[tag + ".decode_attention"] = self.hbm(attn_bytes, dc[CLS_DATTN][0], reps, tag + ".decode_attention")
        gemm_ms = dc[CLS_GEMM][0]
        self.rooflines[tag + ".decode_gemms"] = self.hbm(2.0 * W / k, gemm_ms, reps, tag + ".decode_gemms")
        # at M >= ~300 rows the same GEMMs are bounded by the MFMA pipes rather than the weight stream: report both
        fl = 2.0 * W / k * B
        self.rooflines[tag + ".decode_gemms"]["mfma_tflops"] = fl * reps / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
        call_ms = sum(v[0] for v in dc.values()) / reps
        return {"decode_call_ms": call_ms, "decode_tokens_per_s": B / (call_ms * 1e-3),
                "decode_other_kernels_ms": dc[CLS_OTHER][0] / reps}

    def import_decode_caches(self, ctx, desc, cfg, k, lens, seed, first_id):
        kv_tok_elems = 2 * (cfg.n_kv_heads // k) * cfg.head_dim
        ids = list(range(first_id, first_id + len(lens)))
        stg = self.wl.device_normal((sum(lens) * kv_tok_elems,), seed, cfg.dtype)
        ctx.kv_import_dev(desc, ids, lens, stg)
        self.torch.cuda.synchronize()
        del stg
        return ids

    # ---- configuration 2: one 7B-shape layer, prefill + re-shard + decode
    def config2(self, headline):
        torch, wl, ss, hz, args = self.torch, self.wl, self.ss, self.hz, self.args
        work = wl.config2()
        cfg = work.cfg
        cfg.dtype = wl.F16 if args.dtype == "f16" else wl.BF16
        p_lens = [int(v) for v in work.prefill_lens]
        d_lens = [int(v) for v in work.decode_kv_lens]
        Tp, B = sum(p_lens), len(d_lens)
        kv_tok_bytes = 2 * cfg.n_kv_heads * cfg.head_dim * 2
        N_SETS = 3
        pages = sum(-(-(n + 1) // 16) for n in d_lens) + N_SETS * sum(-(-n // 16) for n in p_lens) + 64
        tier_bytes = N_SETS * Tp * kv_tok_bytes * cfg.n_layers + (1 << 20)
        ctx = hz.make_context(cfg, pages=pages, tier_bytes=tier_bytes, pinned_bytes=args.pinned_mb << 20, max_seq_len=4096)
        w = self.weights_on_device(cfg, 2001)
        pp, tp = hz.pp_desc(cfg), hz.tp_desc(cfg, 1, 0)
        ctx.load_layer(pp, 0, w, ss.SS_DEVICE)
        ctx.load_layer(tp, 0, w, ss.SS_DEVICE)
        x_p = wl.device_normal((Tp, cfg.hidden), 2002, cfg.dtype)
        y_p, x1_p = torch.empty_like(x_p), torch.empty_like(x_p)
        x_d = wl.device_normal((B, cfg.hidden), 2003, cfg.dtype)
        y_d = torch.empty_like(x_d)
        d_ids = self.import_decode_caches(ctx, tp, cfg, 1, d_lens, 2004, 1000)
        id_sets = [list(range(16 * j, 16 * j + 16)) for j in range(N_SETS)]
        tickets = [None] * N_SETS
        zeros = [0] * 16
        stream = self.stream
        out = {}
        if headline:
            # Alternating id sets for the prefill batch: the re-shard of batch i (swap-out, host tier, swap-in) runs on
            # the side streams and the mover threads while the following batches are prefilled, as the cache of a
            # prefilled batch is not needed until its decode begins (paper section 5.2).  The swap-out is requested as
            # soon as the attention half of the layer has written the cache.
            def retire(s):
                if tickets[s] is not None:
                    ctx.kv_wait(tickets[s])
                    ctx.kv_free(tp, id_sets[s])
                    ctx.host_tier_release(id_sets[s])
                    ctx.kv_free(pp, id_sets[s])
                    tickets[s] = None

            def step(i):
                s = i % N_SETS
                ids = id_sets[s]
                if not args.no_reshard:
                    retire(s)
                    ctx.layer_prefill(pp, 0, ss.SS_ATTN, ids, p_lens, zeros, x_p, x1_p, stream)
                    ctx.kv_reshard(pp, tp, ids, stream)
                    tickets[s] = ctx.kv_jobs_issued()
                    ctx.layer_prefill(pp, 0, ss.SS_MLP, ids, p_lens, zeros, x1_p, y_p, stream)
                else:
                    ctx.layer_prefill(pp, 0, ss.SS_BOTH, ids, p_lens, zeros, x_p, y_p, stream)
                ctx.layer_decode(tp, 0, ss.SS_BOTH, d_ids, d_lens, x_d, y_d, stream)
                if args.no_reshard:
                    ctx.kv_free(pp, ids)

            for i in range(args.warmup):
                step(i)
            torch.cuda.synchronize()
            ctx.sync()
            t0 = time.perf_counter()
            for i in range(args.warmup, args.warmup + args.steps):
                step(i)
            torch.cuda.synchronize()
            ctx.sync()                      # every re-shard issued in the timed region has completed
            elapsed = time.perf_counter() - t0
            for j in range(N_SETS):
                retire(j)
            out = {"elapsed": elapsed, "tokens_per_step": Tp + B,
                   "config": {"workload": work.name, "prefill_tokens": Tp, "prefill_prompts": len(p_lens), "decode_seqs": B,
                              "decode_kv_tokens": sum(d_lens), "k": 1, "layers": 1, "reshard_in_step": not args.no_reshard}}
        reps = args.class_reps
        phase = self.prefill_classes("c2", ctx, pp, 0, id_sets[0], p_lens, x_p, y_p, reps)
        phase.update(self.decode_classes("c2", ctx, tp, 0, d_ids, d_lens, x_d, y_d, reps, 1, True))
        # repack alone: export the prefill batch's pages into device staging
        ctx.layer_prefill(pp, 0, ss.SS_BOTH, id_sets[0], p_lens, zeros, x_p, y_p, stream)
        stg = torch.empty(Tp * kv_tok_bytes // 2, device="cuda", dtype=torch.bfloat16)
        rp = self.timed(ctx, lambda: ctx.kv_export_dev(pp, id_sets[0], stg, stream), reps)
        ctx.kv_free(pp, id_sets[0])
        self.rooflines["c2.kv_repack"] = self.hbm(2.0 * Tp * kv_tok_bytes, rp[CLS_REPACK][0], rp[CLS_REPACK][1], "c2.kv_repack")
        out["phase"] = phase
        if headline:
            # weight re-shard (outside the timed steps): reload of the decode strategy's slices of this layer from the
            # page-locked CPU copy; k = 1 moves whole matrices, k = 4 the strided column / row slices
            ctx.host_weights_put(0, w, ss.SS_DEVICE)
            wr = {}
            for label, desc in (("k1", tp), ("k4_shard0", hz.tp_desc(cfg, 4, 0))):
                ctx.reshard_weights(None, desc, stream)                  # first call allocates
                ctx.weights_wait(desc)
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                for _ in range(3):
                    ctx.reshard_weights(None, desc, stream)
                ctx.weights_wait(desc)
                dt_w = (time.perf_counter() - t1) / 3
                nbytes = ctx.weights_shard_bytes(desc)
                wr[label] = {"bytes": nbytes, "ms": dt_w * 1e3, "GB/s": nbytes / dt_w / 1e9}
            out["weight_reshard"] = wr
            if not args.no_cpu_baseline:
                out["cpu_baseline"] = cpu_baseline_layer(work, host_weights(w, wl, hz, cfg.dtype), wl, 6.6e12, 32, 1, 2101)
        ctx.destroy()
        del w
        torch.cuda.empty_cache()
        return out

    # ---- configuration 3: 13B shape, pipeline prefill of the full layer + decode of one k = 4 shard
    def config3(self, headline):
        torch, wl, ss, hz, args = self.torch, self.wl, self.ss, self.hz, self.args
        work = wl.config3()
        cfg, k = work.cfg, work.k
        p_lens = [int(v) for v in work.prefill_lens]
        d_lens = [int(v) for v in work.decode_kv_lens]
        Tp, B = sum(p_lens), len(d_lens)
        pages = max(sum(-(-(n + 1) // 16) for n in d_lens), sum(-(-n // 16) for n in p_lens)) + 64
        ctx = hz.make_context(cfg, pages=pages, max_seq_len=4608)
        w = self.weights_on_device(cfg, 3001)
        pp, tp = hz.pp_desc(cfg), hz.tp_desc(cfg, k, 0)
        ctx.load_layer(pp, 0, w, ss.SS_DEVICE)
        ctx.load_layer(tp, 0, w, ss.SS_DEVICE)
        x_p = wl.device_normal((Tp, cfg.hidden), 3002, cfg.dtype)
        y_p = torch.empty_like(x_p)
        x_d = wl.device_normal((B, cfg.hidden), 3003, cfg.dtype)
        y_d, y2_d = torch.empty_like(x_d), torch.empty_like(x_d)
        d_ids = self.import_decode_caches(ctx, tp, cfg, k, d_lens, 3004, 1000)
        p_ids = list(range(len(p_lens)))
        zeros = [0] * len(p_ids)
        stream = self.stream
        out = {}
        if headline:
            def step(_):
                ctx.layer_prefill(pp, 0, ss.SS_BOTH, p_ids, p_lens, zeros, x_p, y_p, stream)
                ctx.kv_free(pp, p_ids)
                ctx.layer_decode(tp, 0, ss.SS_ATTN, d_ids, d_lens, x_d, y_d, stream)
                ctx.layer_decode(tp, 0, ss.SS_MLP, d_ids, d_lens, x_d, y2_d, stream)

            for i in range(args.warmup):
                step(i)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(args.steps):
                step(i)
            torch.cuda.synchronize()
            out = {"elapsed": time.perf_counter() - t0, "tokens_per_step": Tp + B,
                   "config": {"workload": work.name, "prefill_tokens": Tp, "prefill_prompts": len(p_lens), "prefill_k": 1,
                              "decode_seqs": B, "decode_kv_tokens": sum(d_lens), "decode_k": k, "decode_shard": 0, "layers": 1}}
        reps = args.class_reps
        phase = self.prefill_classes("c3", ctx, pp, 0, p_ids, p_lens, x_p, y_p, reps)
        phase.update(self.decode_classes("c3", ctx, tp, 0, d_ids, d_lens, x_d, y_d, reps, k, False))
        out["phase"] = phase
        if headline and not args.no_cpu_baseline:
            out["cpu_baseline"] = cpu_baseline_layer(work, host_weights(w, wl, hz, cfg.dtype), wl, 8.0e12, 32, 1, 3101)
        ctx.destroy()
        del w
        torch.cuda.empty_cache()
        return out

    # ---- configuration 4: 70B shape with GQA, decode of one k = 8 shard (8 q heads, 1 kv head)
    def config4(self, headline):
        torch, wl, ss, hz, args = self.torch, self.wl, self.ss, self.hz, self.args
        work = wl.config4()
        cfg, k = work.cfg, work.k
        d_lens = [int(v) for v in work.decode_kv_lens]
        B = len(d_lens)
        ctx = hz.make_context(cfg, pages=sum(-(-(n + 1) // 16) for n in d_lens) + 64, max_seq_len=4608)
        w = self.weights_on_device(cfg, 4001)
        tp = hz.tp_desc(cfg, k, 0)
        ctx.load_layer(tp, 0, w, ss.SS_DEVICE)
        x_d = wl.device_normal((B, cfg.hidden), 4003, cfg.dtype)
        y_d, y2_d = torch.empty_like(x_d), torch.empty_like(x_d)
        d_ids = self.import_decode_caches(ctx, tp, cfg, k, d_lens, 4004, 1000)
        stream = self.stream
        out = {}
        if headline:
            def step(_):
                ctx.layer_decode(tp, 0, ss.SS_ATTN, d_ids, d_lens, x_d, y_d, stream)
                ctx.layer_decode(tp, 0, ss.SS_MLP, d_ids, d_lens, x_d, y2_d, stream)

            for i in range(args.warmup):
                step(i)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(args.steps):
                step(i)
            torch.cuda.synchronize()
            out = {"elapsed": time.perf_counter() - t0, "tokens_per_step": B,
                   "config": {"workload": work.name, "decode_seqs": B, "decode_kv_tokens": sum(d_lens), "k": k, "shard": 0,
                              "layers": 1}}
        out["phase"] = self.decode_classes("c4", ctx, tp, 0, d_ids, d_lens, x_d, y_d, args.class_reps, k, False)
        if headline and not args.no_cpu_baseline:
            out["cpu_baseline"] = cpu_baseline_layer(work, host_weights(w, wl, hz, cfg.dtype), wl, 0.0, 256, 1, 4101)
        ctx.destroy()
        del w
        torch.cuda.empty_cache()
        return out

    # ---- configuration 5: ten 70B-shape layers (the k = 8 pipeline slice), prefill + overlapped re-shard
    def config5(self, headline):
        torch, wl, ss, hz, args = self.torch, self.wl, self.ss, self.hz, self.args
        work = wl.config5()
        cfg = work.cfg
        L = cfg.n_layers
        lens_a = [int(v) for v in work.prefill_lens]
        lens_b = [int(v) for v in work.notes["next_batch_lens"]]
        Ta, Tb = sum(lens_a), sum(lens_b)
        kv_tok_bytes = 2 * cfg.n_kv_heads * cfg.head_dim * 2           # K and V, one layer
        shard = 0
        pages = sum(-(-n // 16) for n in lens_a) + sum(-(-n // 16) for n in lens_b) + 64
        tier_bytes = (Ta + Tb) * kv_tok_bytes * L + (1 << 20)
        ctx = hz.make_context(cfg, pages=pages, tier_bytes=tier_bytes, pinned_bytes=args.pinned_mb << 20, max_seq_len=4096)
        pp, tp = hz.pp_desc(cfg), hz.tp_desc(cfg, work.k, shard)
        w0 = None
        for l in range(L):
            w = self.weights_on_device(cfg, 5100 + l)
            ctx.load_layer(pp, l, w, ss.SS_DEVICE)
            if l == 0 and headline and not args.no_cpu_baseline:
                w0 = host_weights(w, wl, hz, cfg.dtype)
            del w
        torch.cuda.empty_cache()
        # two batches alternate (the workload's batch and its "next batch"), so that the re-shard of one overlaps the
        # prefill of the other, as the swap-out of a prefilled batch does in the paper (section 5.2)
        sets = [(list(range(len(lens_a))), lens_a, wl.device_normal((Ta, cfg.hidden), 5002, cfg.dtype)),
                (list(range(1000, 1000 + len(lens_b))), lens_b, wl.device_normal((Tb, cfg.hidden), 5003, cfg.dtype))]
        tmax = max(Ta, Tb)
        buf = [torch.empty((tmax, cfg.hidden), device="cuda", dtype=torch.bfloat16)]
        tickets = [None, None]
        stream = self.stream
        out = {}

        def run_slice(ids, lens, x):
            # the slice's ten layers chained on the device in one call
            ctx.layers_prefill(pp, ids, lens, [0] * len(ids), x, buf[0][:sum(lens)], stream)

        def retire(s):
            if tickets[s] is not None:
                ctx.kv_wait(tickets[s])
                ctx.kv_free(tp, sets[s][0])
                ctx.host_tier_release(sets[s][0])
                ctx.kv_free(pp, sets[s][0])
                tickets[s] = None

        def step(i):
            s = i & 1
            ids, lens, x = sets[s]
            retire(s)
            run_slice(ids, lens, x)
            if not args.no_reshard:
                ctx.kv_reshard(pp, tp, ids, stream)
                tickets[s] = ctx.kv_jobs_issued()
            else:
                ctx.kv_free(pp, ids)

        if headline:
            for i in range(args.warmup):
                step(i)
            torch.cuda.synchronize()
            ctx.sync()
            # the kernel classes are timed inside the timed region itself (HIP events on the launch streams)
            ctx.prof_reset()
            ctx.prof_enable(True)
            t0 = time.perf_counter()
            for i in range(args.warmup, args.warmup + args.steps):
                step(i)
            torch.cuda.synchronize()
            ctx.sync()                      # every re-shard issued in the timed region has completed
            elapsed = time.perf_counter() - t0
            ctx.prof_enable(False)
            live = {c: ctx.prof_read(c) for c in range(5)}
            for j in range(2):
                retire(j)
            toks = sum(sum(sets[i & 1][1]) for i in range(args.warmup, args.warmup + args.steps))
            W = cfg.layer_params()
            calls = args.steps * L
            mean_T = toks / args.steps
            self.rooflines["c5.prefill_gemms"] = self.mfma(2.0 * W * mean_T, live[CLS_GEMM][0], calls, "c5.prefill_gemms")
            sq = sum(sum(n * n for n in sets[i & 1][1]) for i in range(args.warmup, args.warmup + args.steps)) / args.steps
            self.rooflines["c5.prefill_attention"] = self.mfma(2.0 * cfg.n_q_heads * cfg.head_dim * float(sq),
                                                               live[CLS_PATTN][0], calls, "c5.prefill_attention")
            self.rooflines["c5.prefill_gemms"]["timed"] = "inside the timed steps, re-shard running beside them"
            out = {"elapsed": elapsed, "tokens_per_step": mean_T,
                   "config": {"workload": work.name, "prefill_prompts": len(lens_a), "prefill_tokens": Ta,
                              "next_batch_tokens": Tb, "layers": L, "weights_GB": W * L * 2 / 1e9, "prefill_k": 1,
                              "reshard_to": "k=%d shard %d" % (work.k, shard), "reshard_GB_per_batch": Ta * kv_tok_bytes * L / 1e9,
                              "reshard_in_step": not args.no_reshard},
                   "phase": {"gemm_ms_per_step": live[CLS_GEMM][0] / args.steps, "attention_ms_per_step": live[CLS_PATTN][0] / args.steps,
                             "other_kernels_ms_per_step": live[CLS_OTHER][0] / args.steps,
                             "repack_kernels_ms_per_step": live[CLS_REPACK][0] / args.steps}}
        else:
            ids, lens, x = sets[0]
            y = buf[0][:Ta]
            self.prefill_classes("c5", ctx, pp, 0, ids, lens, x, y, max(2, args.class_reps // 2))
        # the repack of one batch alone: all ten layers' pages of batch A into device staging
        ids, lens, x = sets[0]
        run_slice(ids, lens, x)
        stg = torch.empty(Ta * kv_tok_bytes * L // 2, device="cuda", dtype=torch.bfloat16)
        rp = self.timed(ctx, lambda: ctx.kv_export_dev(pp, ids, stg, stream), 3)
        self.rooflines["c5.kv_repack"] = self.hbm(2.0 * Ta * kv_tok_bytes * L, rp[CLS_REPACK][0], rp[CLS_REPACK][1], "c5.kv_repack")
        del stg
        if headline:
            # the PCIe legs of the re-shard alone, nothing else running: the batch's caches out of the pipeline layout
            # into the host tier, then the tensor-parallel shard's heads of them in; next to what a plain copy between
            # the device and page-locked memory reaches on this machine (the link differs a lot from box to box)
            torch.cuda.synchronize()
            ctx.sync()
            t0 = time.perf_counter()
            ctx.kv_swap(pp, ss.SS_OUT, ids, stream)
            ctx.kv_wait(ctx.kv_jobs_issued())
            t_out = time.perf_counter() - t0
            t0 = time.perf_counter()
            ctx.kv_swap(tp, ss.SS_IN, ids, stream)
            ctx.kv_wait(ctx.kv_jobs_issued())
            t_in = time.perf_counter() - t0
            ctx.kv_free(tp, ids)
            ctx.host_tier_release(ids)
            b_out, b_in = Ta * kv_tok_bytes * L, Ta * kv_tok_bytes * L // work.k
            n = 512 << 20
            dev = torch.empty(n, dtype=torch.uint8, device="cuda")
            pin = torch.empty(n, dtype=torch.uint8, pin_memory=True)
            rates = {}
            for label, dst, src in (("d2h", pin, dev), ("h2d", dev, pin)):
                dst.copy_(src, non_blocking=True)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                dst.copy_(src, non_blocking=True)
                torch.cuda.synchronize()
                rates[label + "_GB/s"] = n / (time.perf_counter() - t0) / 1e9
            del dev, pin
            out["kv_movement"] = {"swap_out": {"bytes": b_out, "ms": t_out * 1e3, "GB/s": b_out / t_out / 1e9},
                                  "swap_in": {"bytes": b_in, "ms": t_in * 1e3, "GB/s": b_in / t_in / 1e9},
                                  "plain_pinned_copy_512MB": rates}
        ctx.kv_free(pp, ids)
        if headline and w0 is not None:
            out["cpu_baseline"] = cpu_baseline_layer(work, w0, wl, 2.0e13, 0, L, 5101)
        ctx.destroy()
        del sets, buf
        torch.cuda.empty_cache()
        return out

    # ---- configuration 1: the tiny fp32 model end to end (prefill + 8 greedy steps, pipeline layout)
    def config1(self, headline):
        torch, wl, ss, hz, args = self.torch, self.wl, self.ss, self.hz, self.args
        work = wl.config1()
        cfg = work.cfg
        steps_dec = work.notes["decode_steps"]
        ws = [wl.make_layer_weights(cfg, 1001 + l) for l in range(cfg.n_layers)]
        hv, hr = wl.make_head_weights(cfg, 1099)
        ctx = hz.make_context(cfg, pages=64)
        pp = hz.pp_desc(cfg)
        for l in range(cfg.n_layers):
            ctx.load_layer(pp, l, ws[l][1])
        ctx.load_head(hr["embed"], hr["gf"], hr["wlm"])
        rng = np.random.default_rng(1001)
        prompts = [rng.integers(0, cfg.vocab, size=int(n)) for n in work.prefill_lens]
        n = len(prompts)
        lens = [len(p) for p in prompts]
        T = sum(lens)
        ids = list(range(n))
        a = torch.empty((T, cfg.hidden), device="cuda", dtype=torch.float32)
        b = torch.empty_like(a)
        logits = torch.empty((n, cfg.vocab), device="cuda", dtype=torch.float32)
        last = torch.tensor(np.cumsum(lens) - 1, device="cuda")
        stream = self.stream

        def layers(fn, cur_lens, q_lens, x, y):
            for l in range(cfg.n_layers):
                fn(pp, l, ss.SS_BOTH, ids, *q_lens, cur_lens, x, y, stream)
                x, y = y, x
            return x

        def generate():
            ctx.embed(np.concatenate(prompts), a, stream)
            x = layers(ctx.layer_prefill, [0] * n, (lens,), a, b)
            ctx.lm_head(x[last].contiguous(), n, logits, stream)
            tok = torch.argmax(logits, dim=-1).cpu().numpy()
            cur = list(lens)
            for _ in range(steps_dec):
                ctx.embed(tok, a[:n], stream)
                x = layers(ctx.layer_decode, cur, (), a[:n], b[:n])
                ctx.lm_head(x, n, logits, stream)
                tok = torch.argmax(logits, dim=-1).cpu().numpy()
                cur = [v + 1 for v in cur]
            ctx.kv_free(pp, ids)

        for _ in range(args.warmup):
            generate()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            generate()
        torch.cuda.synchronize()
        out = {"elapsed": time.perf_counter() - t0, "tokens_per_step": T + n * steps_dec,
               "config": {"workload": work.name, "prompts": n, "prompt_tokens": T, "decode_steps": steps_dec, "layers": cfg.n_layers}}
        if not args.no_cpu_baseline:
            from oracle import layer_math as lm
            t1 = time.perf_counter()
            lm.generate(cfg, [w[0] for w in ws], hv, prompts, steps_dec)
            secs = time.perf_counter() - t1
            out["cpu_baseline"] = {"value": (T + n * steps_dec) / secs, "unit": "tokens/s", "cores": oracle_threads(),
                                   "kind": "oracle", "sample": "the whole configuration (fp64 numpy)", "seconds": secs}
        ctx.destroy()
        return out


def offline_loop_bench(torch, wl, ss, hz):
    """Constant-length requests (prompt 3000 tokens, as in the paper's study of the prompt : output ratio,
    section 6.5; 64 output tokens), two layers of the configuration-2 shape with a small vocabulary, greedy
    decoding.  The CPU store holds all, a quarter or a sixteenth of the requests: the smaller it is, the more
    often the engine changes stage (and reloads its weights)."""
    base = wl.config2().cfg
    cfg = wl.ModelCfg(hidden=base.hidden, n_q_heads=base.n_q_heads, n_kv_heads=base.n_kv_heads, head_dim=base.head_dim,
                      ffn=base.ffn, n_layers=2, vocab=2048, dtype=wl.BF16)
    n_req, p_len, o_len = 64, 3000, 64
    raws = [wl.make_layer_weights(cfg, 6001 + l)[1] for l in range(cfg.n_layers)]
    _, hr = wl.make_head_weights(cfg, 6099)
    rng = np.random.default_rng(6100)
    prompts = [rng.integers(0, cfg.vocab, size=p_len).astype(np.int32) for _ in range(n_req)]
    tok_bytes = 2 * cfg.n_kv_heads * cfg.head_dim * 2 * cfg.n_layers
    per_seq_pages = -(-(p_len + o_len) // 16)
    compute = torch.cuda.Stream()
    torch.cuda.synchronize()
    runs = {}
    for label, in_store, group in (("store_all", n_req, 0), ("store_all_swap_in_groups_of_4", n_req, 4),
                                   ("store_quarter", n_req // 4, 0), ("store_sixteenth", n_req // 16, 0)):
        ctx = hz.make_context(cfg, pages=n_req * per_seq_pages, tier_bytes=in_store * p_len * tok_bytes,
                              pinned_bytes=256 << 20, max_seq_len=4096)
        ctx.load_head(hr["embed"], hr["gf"], hr["wlm"])
        for l in range(cfg.n_layers):
            ctx.host_weights_put(l, raws[l])
        P, D = hz.pp_desc(cfg), hz.tp_desc(cfg, 1, 0)
        for rep in range(2):                                 # the first run allocates pools, staging and workspaces
            _, _, st = ctx.offline_run(P, D, prompts, [o_len] * n_req, 8 * p_len, n_req, True, compute.cuda_stream,
                                       swap_in_group=group)
        total_tokens = n_req * (p_len + o_len)
        runs[label] = {"tokens_per_s": total_tokens / st["total_seconds"], "output_tokens_per_s": st["tokens"] / st["total_seconds"],
                       "switches": st["to_decode"] + st["to_prefill"], "prefill_batches": st["prefill_batches"],
                       "decode_steps": st["decode_steps"], "prefill_s": st["prefill_seconds"],
                       "decode_s": st["decode_seconds"], "switch_s": st["switch_seconds"], "total_s": st["total_seconds"]}
        ctx.destroy()
    print(json.dumps({"metric": "offline loop, prompt+output tokens/s", "unit": "tokens/s", "n_gpus": 1, "dtype": "bf16",
                      "data": "synthetic", "config": {"workload": "c2_shape_2_layers_const_3000_in_64_out", "requests": n_req,
                                                      "weight_reshard_at_every_switch": True},
                      "value": runs["store_all"]["tokens_per_s"], "runs": runs}))


def library_gemm_yardstick(torch, wl, config):
    """The vendor library's GEMM on the shapes of the configuration's prefill projections (tokens = the mean of the two
    alternating batches where there are two): the same contractions as this library's prefill GEMMs without the
    fused epilogues.  One JSON line; fractions are of the 2.5 PFLOP/s bf16 peak."""
    w = {2: wl.config2, 3: wl.config3, 5: wl.config5}.get(config)
    if w is None:
        print("bench.py: --library-gemm needs a configuration with a prefill batch (2, 3 or 5)", file=sys.stderr)
        sys.exit(2)
    w = w()
    cfg = w.cfg
    T = int(sum(w.prefill_lens))
    if w.notes and "next_batch_lens" in w.notes:
        T = (T + int(sum(w.notes["next_batch_lens"]))) // 2
    d = cfg.head_dim
    shapes = [("qkv", (cfg.n_q_heads + 2 * cfg.n_kv_heads) * d, cfg.hidden), ("o", cfg.hidden, cfg.n_q_heads * d),
              ("gate_up", 2 * cfg.ffn, cfg.hidden), ("down", cfg.hidden, cfg.ffn)]
    out = {"library_gemm": {"workload": w.name, "tokens": T, "peak_tflops": 2500.0, "reps": 5}}
    for data in ("random", "zeros"):
        rows, total_ms, total_fl = {}, 0.0, 0.0
        for name, N, K in shapes:
            if data == "zeros":
                a = torch.zeros((T, K), device="cuda", dtype=torch.bfloat16)
                wt = torch.zeros((N, K), device="cuda", dtype=torch.bfloat16)
            else:
                a = wl.device_normal((T, K), 9101, wl.BF16)
                wt = wl.device_normal((N, K), 9102, wl.BF16, std=0.02)
            c = torch.empty((T, N), device="cuda", dtype=torch.bfloat16)
            for _ in range(2):
                torch.matmul(a, wt.t(), out=c)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                torch.matmul(a, wt.t(), out=c)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 5
            fl = 2.0 * T * N * K
            rows[name] = {"N": N, "K": K, "ms": ms, "frac": fl / ms / 1e9 / 2500.0}
            total_ms += ms
            total_fl += fl
            del a, wt, c
        rows["all"] = {"ms": total_ms, "frac": total_fl / total_ms / 1e9 / 2500.0}
        out["library_gemm"][data] = rows
    print(json.dumps(out))


DEFAULT_STEPS = {1: (20, 3), 2: (20, 6), 3: (10, 3), 4: (50, 5), 5: (8, 2)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--config", type=int, default=5, choices=[1, 2, 3, 4, 5],
                    help="configuration the headline step runs (default 5, the largest single-GPU one)")
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--class-reps", type=int, default=5, help="calls per kernel-class timing pass")
    ap.add_argument("--only", action="store_true", help="leave the kernel classes of the other configurations out")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-reshard", action="store_true", help="leave the KV re-shard out of the step (configurations 2 and 5)")
    ap.add_argument("--pinned-mb", type=int, default=256, help="pinned staging ring of the KV movers (two lanes x two slots)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--dtype", choices=["bf16", "f16"], default="bf16",
                    help="16-bit storage type of configuration 2 (bf16: the type the benchmark is defined on; f16: the paper's own)")
    ap.add_argument("--zero-data", action="store_true",
                    help="power probe, not a benchmark: weights, gains and inputs are all zero, so the same instruction streams run "
                         "without toggling the data paths (the clock the chip then holds shows how far the package power limit, "
                         "not the kernels' issue rate, sets the speed on real data)")
    ap.add_argument("--offline-loop", action="store_true",
                    help="instead of the layer step: the whole offline engine loop (scheduler, swaps, weight re-shards) on a "
                         "two-layer model of the configuration-2 layer shape, for three sizes of the CPU store")
    ap.add_argument("--library-gemm", action="store_true",
                    help="yardstick, not a benchmark of this library: the vendor library's plain GEMM (torch.matmul, no fused "
                         "epilogue) on the four projection shapes of the configuration's prefill batch, on random data and on zeros")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    if args.steps is None:
        args.steps = DEFAULT_STEPS[args.config][0]
    if args.warmup is None:
        args.warmup = DEFAULT_STEPS[args.config][1]

    import torch
    import workloads as wl
    import paper_2503_06433_amd as ss
    from paper_2503_06433_amd import harness as hz

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    if args.zero_data:
        draw_normal, draw_weights = wl.device_normal, wl.device_layer_weights
        wl.device_normal = lambda *a, **k: draw_normal(*a, **k).zero_()
        wl.device_layer_weights = lambda *a, **k: {name: t.zero_() for name, t in draw_weights(*a, **k).items()}
        args.no_cpu_baseline = True
    if args.calibrate_copy:
        src = torch.ones(1 << 29, dtype=torch.bfloat16, device="cuda")      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.offline_loop:
        offline_loop_bench(torch, wl, ss, hz)
        return
    if args.library_gemm:
        library_gemm_yardstick(torch, wl, args.config)
        return
    b = Bench(args, torch, wl, ss, hz)
    runs = {1: b.config1, 2: b.config2, 3: b.config3, 4: b.config4, 5: b.config5}
    head = runs[args.config](True)
    others = {}
    if not args.only and args.config != 1:
        for n in (2, 3, 4, 5):
            if n != args.config:
                others["c%d" % n] = runs[n](False).get("phase")
    elapsed = head["elapsed"]
    main_key = {2: "c2.prefill_gemms", 3: "c3.prefill_gemms", 4: "c4.decode_attention", 5: "c5.prefill_gemms"}.get(args.config)
    roof = dict(b.rooflines[main_key]) if main_key else None
    if roof is not None:
        roof["kernel"] = {"c4.decode_attention": "paged decode attention (GQA, 8 q heads on 1 kv head)"}.get(
            main_key, "prefill GEMMs (QKV, O, gate/up, down)")
    out = {
        "metric": "prefill+decode tokens/s per GPU shard", "value": head["tokens_per_step"] * args.steps / elapsed,
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if args.config == 1 else (args.dtype if args.config == 2 else "bf16"),
        "data": "zeros (power probe, not a benchmark result)" if args.zero_data else "synthetic",
        "config": head["config"], "roofline": roof, "rooflines": b.rooflines,
        "phase_ms": dict({"c%d" % args.config: head.get("phase")}, **others),
    }
    for key in ("weight_reshard", "kv_movement", "cpu_baseline"):
        if key in head:
            out[key] = head[key]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
