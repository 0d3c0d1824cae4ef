"""Benchmark of the hot path on one MI355X.

A step is one pass of the whole path over one batch of the LLaMA-2-7B-shape
single-layer workload (bf16, k = 1):
    layer_prefill of 16 prompts (lengths uniform[512, 2048], 20 018 tokens)
    kv_reshard of those prompts' KV: pages -> heads-major staging -> pinned ->
        host tier -> pinned -> pages of the decode-layout shard (side stream)
    layer_decode of 256 resident sequences (KV lengths uniform[512, 2560])
value = (prefill tokens + decode tokens) * steps / elapsed, everything resident
in HBM when the timed region starts.

Prints ONE JSON line.  `roofline` is the prefill GEMM class (MFMA-bound); the
other bounded kernels are reported under `rooflines`.  `cpu_baseline` times the
CPU oracle on a bounded sample of the same workload.
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


def measured_traffic():
    """HBM bytes per launch from the rocprofv3 --pmc runs recorded in profiles/ (None if not recorded)."""
    path = os.path.join(ROOT, "bench_traffic.json")
    if not os.path.exists(path):
        return {}
    with open(path) as f:
        return json.load(f)


def gemm_flops_per_token(cfg, k=1):
    return 2.0 * cfg.layer_params() / k


def cpu_baseline(work, vals, budget_tokens=16384, n_decode=32):
    """Times the oracle as it stands on a bounded sample: the first `budget_tokens`
    worth of the shortest prompts for prefill and `n_decode` decode sequences."""
    from oracle import layer_math as lm
    import workloads as wl
    cfg = work.cfg
    order = np.argsort(work.prefill_lens)
    lens = []
    for i in order:
        if sum(lens) + int(work.prefill_lens[i]) > budget_tokens and lens:
            break
        lens.append(int(work.prefill_lens[i]))
    T = sum(lens)
    xv, _ = wl.make_activations((T, cfg.hidden), 2101, cfg.dtype)
    batch = [(i, n, 0) for i, n in enumerate(lens)]
    cache = lm.KVCache(cfg)
    t0 = time.perf_counter()
    lm.layer_forward(cfg, vals, xv, batch, cache, 0)
    t_prefill = time.perf_counter() - t0
    # decode leg: caches are inputs (filled outside the timed region)
    dlens = [int(v) for v in work.decode_kv_lens[:n_decode]]
    rng = np.random.default_rng(2102)
    dcache = lm.KVCache(cfg)
    for i, n in enumerate(dlens):
        dcache.ensure(i, n + 1)
        dcache.data[i][:] = rng.standard_normal(dcache.data[i].shape)
    dx, _ = wl.make_activations((n_decode, cfg.hidden), 2103, cfg.dtype)
    t2 = time.perf_counter()
    lm.layer_forward(cfg, vals, dx, [(i, 1, n) for i, n in enumerate(dlens)], dcache, 0)
    t_decode = time.perf_counter() - t2
    secs = t_prefill + t_decode
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    return {"value": (T + n_decode) / secs, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "prefill of the %d shortest prompts (%d tokens) + decode of %d sequences, one layer, fp64 numpy"
                      % (len(lens), T, n_decode),
            "seconds": secs}


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=6)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-reshard", action="store_true", help="leave the KV re-shard out of the step")
    ap.add_argument("--pinned-mb", type=int, default=256, help="pinned staging ring of the KV movers (two lanes x two slots)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--dtype", choices=["bf16", "f16"], default="bf16",
                    help="16-bit storage type of the model (bf16: the configuration BASELINE.json names; f16: the paper's own)")
    ap.add_argument("--offline-loop", action="store_true",
                    help="instead of the layer step: the whole offline engine loop (scheduler, swaps, weight re-shards) on a "
                         "two-layer model of the configuration-2 layer shape, for three sizes of the CPU store")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as wl
    import paper_2503_06433_amd as ss
    from paper_2503_06433_amd import harness as hz

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
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
    work = wl.config2()
    cfg = work.cfg
    cfg.dtype = wl.F16 if args.dtype == "f16" else wl.BF16
    p_lens = [int(v) for v in work.prefill_lens]
    d_lens = [int(v) for v in work.decode_kv_lens]
    Tp, B = sum(p_lens), len(d_lens)
    kv_tok_bytes = 2 * cfg.n_kv_heads * cfg.head_dim * 2          # K and V, bf16, per token per layer
    decode_tokens = sum(d_lens)
    N_SETS = 3
    pages = sum(-(-(n + 1) // 16) for n in d_lens) + N_SETS * sum(-(-n // 16) for n in p_lens) + 64
    tier_bytes = N_SETS * Tp * kv_tok_bytes * cfg.n_layers + (1 << 20)
    ctx = hz.make_context(cfg, pages=pages, tier_bytes=tier_bytes, pinned_bytes=args.pinned_mb << 20, max_seq_len=4096)
    vals, raws = wl.make_layer_weights(cfg, 2001)
    pp = hz.pp_desc(cfg)
    tp = hz.tp_desc(cfg, 1, 0)
    ctx.load_layer(pp, 0, raws)
    ctx.load_layer(tp, 0, raws)
    _, xr = wl.make_activations((Tp, cfg.hidden), 2002, cfg.dtype)
    x_p = hz.to_device(xr, cfg.dtype)
    y_p = torch.empty_like(x_p)
    _, dr = wl.make_activations((B, cfg.hidden), 2003, cfg.dtype)
    x_d = hz.to_device(dr, cfg.dtype)
    y_d = torch.empty_like(x_d)
    # resident decode caches: K, V ~ N(0,1), drawn on the device, scattered into pages
    d_ids = list(range(1000, 1000 + B))
    stg = wl.device_normal((decode_tokens * kv_tok_bytes // 2,), 2004, cfg.dtype)
    ctx.kv_import_dev(tp, d_ids, d_lens, stg)
    torch.cuda.synchronize()
    del stg
    # Alternating id sets for the prefill batch: the re-shard of batch i (swap-out, host tier, swap-in)
    # runs on the side streams and the mover threads while the following batches are prefilled, as the
    # KV of a prefilled batch is not needed until its decode begins (paper section 5.2).  The swap-out
    # is requested as soon as the attention half of the layer has written the cache.
    id_sets = [list(range(16 * j, 16 * j + 16)) for j in range(N_SETS)]
    tickets = [None] * N_SETS
    x1_p = torch.empty_like(x_p)
    p_ids = id_sets[0]
    zeros = [0] * len(p_ids)
    stream = torch.cuda.current_stream().cuda_stream

    def retire(s):
        if tickets[s] is not None:
            ctx.kv_wait(tickets[s])
            ctx.kv_free(tp, id_sets[s])
            ctx.host_tier_release(id_sets[s])
            ctx.kv_free(pp, id_sets[s])
            tickets[s] = None

    def step(i, reshard=True):
        s = i % N_SETS
        ids = id_sets[s]
        if reshard:
            retire(s)
            ctx.layer_prefill(pp, 0, ss.SS_ATTN, ids, p_lens, zeros, x_p, x1_p, stream)
            ctx.kv_reshard(pp, tp, ids, stream)
            tickets[s] = ctx.kv_jobs_issued()
            ctx.layer_prefill(pp, 0, ss.SS_MLP, ids, p_lens, zeros, x1_p, y_p, stream)
        else:
            ctx.layer_prefill(pp, 0, ss.SS_BOTH, ids, p_lens, zeros, x_p, y_p, stream)
        ctx.layer_decode(tp, 0, ss.SS_BOTH, d_ids, d_lens, x_d, y_d, stream)
        if not reshard:
            ctx.kv_free(pp, ids)

    do_reshard = not args.no_reshard
    for i in range(args.warmup):
        step(i, do_reshard)
    torch.cuda.synchronize()
    ctx.sync()
    t0 = time.perf_counter()
    for i in range(args.warmup, args.warmup + args.steps):
        step(i, do_reshard)
    torch.cuda.synchronize()
    ctx.sync()                      # every re-shard issued in the timed region has completed
    elapsed = time.perf_counter() - t0
    for j in range(N_SETS):
        retire(j)
    ms_per_step = elapsed * 1e3 / args.steps
    value = (Tp + B) * args.steps / elapsed

    # ---- per-kernel-class timing with HIP events on the launch stream (separate passes)
    def timed(fn, reps):
        ctx.prof_reset()
        ctx.prof_enable(True)
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        ctx.sync()
        ctx.prof_enable(False)
        return {c: ctx.prof_read(c) for c in range(5)}

    def prefill_only():
        ctx.layer_prefill(pp, 0, ss.SS_BOTH, p_ids, p_lens, zeros, x_p, y_p, stream)
        ctx.kv_free(pp, p_ids)

    def decode_only():
        ctx.layer_decode(tp, 0, ss.SS_BOTH, d_ids, d_lens, x_d, y_d, stream)

    reps = max(3, min(args.steps, 10))
    pf = timed(prefill_only, reps)
    dc = timed(decode_only, reps)
    # repack alone: export the prefill batch's pages into device staging
    ctx.layer_prefill(pp, 0, ss.SS_BOTH, p_ids, p_lens, zeros, x_p, y_p, stream)
    stg = torch.empty(Tp * kv_tok_bytes // 2, device="cuda", dtype=torch.bfloat16)
    rp = timed(lambda: ctx.kv_export_dev(pp, p_ids, stg, stream), reps)
    ctx.kv_free(pp, p_ids)

    gemm_ms, gemm_n = pf[0]
    gemm_flops = gemm_flops_per_token(cfg) * Tp                      # per prefill call (4 launches)
    gemm_tflops = gemm_flops * reps / (gemm_ms * 1e-3) / 1e12
    attn_ms, _ = pf[1]
    attn_flops = 2.0 * cfg.n_q_heads * cfg.head_dim * float(sum(n * n for n in p_lens))
    dattn_ms, dattn_n = dc[2]
    dattn_bytes = float(decode_tokens + B) * kv_tok_bytes + B * 4.0 * cfg.n_q_heads * cfg.head_dim
    dgemm_ms, _ = dc[0]
    dgemm_bytes = 2.0 * cfg.layer_params()
    rp_ms, rp_n = rp[3]
    rp_bytes = 2.0 * Tp * kv_tok_bytes

    traffic = measured_traffic()

    def hbm(bytes_per_launch, ms_total, n, traffic=None):
        a = bytes_per_launch * n / (ms_total * 1e-3) / 1e9 if ms_total > 0 else 0.0
        return {"bound": "hbm", "achieved": a, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": a / PEAK_HBM_GBS,
                "traffic": traffic, "avg_ms": ms_total / max(n, 1)}

    out = {
        "metric": "prefill+decode tokens/s per GPU shard", "value": value, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": work.name, "prefill_tokens": Tp, "prefill_prompts": len(p_lens),
                   "decode_seqs": B, "decode_kv_tokens": decode_tokens, "k": 1, "layers": 1,
                   "reshard_in_step": do_reshard},
        "roofline": {"bound": "mfma", "achieved": gemm_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": gemm_tflops / PEAK_BF16_TFLOPS, "traffic": traffic.get("prefill_gemms"),
                     "kernel": "prefill GEMMs (QKV, O, gate/up, down)", "avg_ms_per_call": gemm_ms / reps},
        "rooflines": {
            "prefill_attention": {"bound": "mfma", "achieved": attn_flops * reps / (attn_ms * 1e-3) / 1e12,
                                  "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                                  "frac": attn_flops * reps / (attn_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                                  "avg_ms": attn_ms / reps},
            "decode_attention": hbm(dattn_bytes, dattn_ms, dattn_n, traffic.get("decode_attention")),
            "decode_gemms": hbm(dgemm_bytes, dgemm_ms, reps, traffic.get("decode_gemms")),
            "kv_repack": hbm(rp_bytes, rp_ms, rp_n, traffic.get("kv_repack")),
        },
        "phase_ms": {"prefill_call": sum(v[0] for v in pf.values()) / reps,
                     "decode_call": sum(v[0] for v in dc.values()) / reps,
                     "prefill_tokens_per_s": Tp * reps / (sum(v[0] for v in pf.values()) * 1e-3),
                     "decode_tokens_per_s": B * reps / (sum(v[0] for v in dc.values()) * 1e-3)},
    }
    # ---- weight re-shard (outside the timed steps): reload of the decode strategy's slices of this layer
    # from the page-locked CPU copy; k = 1 moves whole matrices, k = 4 the strided column / row slices
    ctx.host_weights_put(0, raws)
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
        out["cpu_baseline"] = cpu_baseline(work, vals)
    print(json.dumps(out))
    ctx.destroy()


if __name__ == "__main__":
    main()
