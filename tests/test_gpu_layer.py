"""GPU parity of the layer calls against the CPU oracle, through the C ABI.

Element-by-element comparisons on seeded inputs at sizes that span several
tiles and ragged tails; the acceptance metric is max|gpu - oracle| / max|oracle|
per output tensor, <= 2e-2 for bf16 and <= 1e-4 for fp32.
"""
import os

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import layer_math as lm

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2503_06433_amd as ss
    from paper_2503_06433_amd.harness import (make_context, to_device, to_f64, empty_like_acts, rel_err, tol, parity, ROW_TOL_FULL,
                                              pp_desc, tp_desc)


def _load(ctx, desc, cfg, raws):
    for l in range(desc.layer_begin, desc.layer_end):
        ctx.load_layer(desc, l, raws[l])


def _weights(cfg, seed):
    vals, raws = [], []
    for l in range(cfg.n_layers):
        v, r = wl.make_layer_weights(cfg, seed + l)
        vals.append(v)
        raws.append(r)
    return vals, raws


def _round_kv(cfg):
    if cfg.dtype == wl.F32:
        return None
    return lambda a: wl.round_to_storage(a, cfg.dtype)


SMALL = {
    "mha_d128": dict(hidden=512, n_q_heads=4, n_kv_heads=4, head_dim=128, ffn=1024),
    "gqa4_d128": dict(hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=1536),
    "gqa8_d128": dict(hidden=1024, n_q_heads=8, n_kv_heads=1, head_dim=128, ffn=1024),
    "mha_d64_generic": dict(hidden=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn=688),
}


@pytest.mark.parametrize("name,dtype,k", [
    ("mha_d128", wl.BF16, 1), ("mha_d128", wl.BF16, 2), ("gqa4_d128", wl.BF16, 2), ("gqa8_d128", wl.BF16, 1),
    ("mha_d64_generic", wl.BF16, 2), ("mha_d64_generic", wl.F32, 1), ("mha_d128", wl.F32, 2),
    ("mha_d128", wl.F16, 1), ("gqa4_d128", wl.F16, 2), ("mha_d64_generic", wl.F16, 2),
])
def test_prefill_then_decode_matches_oracle(name, dtype, k):
    cfg = wl.ModelCfg(n_layers=1, dtype=dtype, **SMALL[name])
    vals, raws = _weights(cfg, 100)
    lens = [1, 17, 130, 300, 32]
    T = sum(lens)
    xv, xr = wl.make_activations((T, cfg.hidden), 7, dtype)
    ctx = make_context(cfg, pages=64)
    batch = [(10 + i, n, 0) for i, n in enumerate(lens)]
    ids = [b[0] for b in batch]
    cache = lm.KVCache(cfg)
    x = to_device(xr, dtype)
    eps = tol(dtype)
    descs = [pp_desc(cfg)] if k == 1 else [tp_desc(cfg, k, i) for i in range(k)]
    for d in descs:
        _load(ctx, d, cfg, raws)
    starts = np.concatenate([[0], np.cumsum(lens)])
    spans = [(int(starts[i]), int(starts[i + 1])) for i in range(len(lens))]     # compared per sequence as well
    tag = "%s/%s/k%d " % (name, {wl.F32: "f32", wl.BF16: "bf16", wl.F16: "f16"}[dtype], k)

    # ---- prefill, attention block partials (no residual) and the cache they leave behind
    o_sum = np.zeros((T, cfg.hidden))
    for i, d in enumerate(descs):
        out = empty_like_acts(T, cfg.hidden, dtype)
        ctx.layer_prefill(d, 0, ss.SS_ATTN | ss.SS_NO_RESIDUAL, ids, lens, [0] * len(lens), x, out)
        torch.cuda.synchronize()
        ref = lm.attn_block(cfg, vals[0], xv, batch, cache, 0, k, i, _round_kv(cfg))
        got = to_f64(out, dtype)
        parity(got, ref, dtype, tag + "prefill attention partial of shard %d" % i, spans)
        o_sum += got
    # cache contents: rotated K and V of every shard
    (_, _), (g0, g1), _ = lm.shard_ranges(cfg, k, 0)
    for i, d in enumerate(descs):
        nh = cfg.n_kv_heads // k
        for sid, n in zip(ids, lens):
            raw = ctx.kv_read(d, sid, 0, nh)
            got = wl.storage_to_f64(raw, dtype)
            ref = cache.data[sid][0, :, i * nh:(i + 1) * nh]
            parity(got, ref, dtype, tag + "cached K/V of sequence %d (%d tokens) shard %d" % (sid, n, i))
    # ---- MLP partials on the oracle's x1
    x1v = xv + sum(lm.attn_block(cfg, vals[0], xv, batch, lm.KVCache(cfg), 0, k, i) for i in range(k))
    x1q, x1r = wl.quantize(x1v, dtype)
    x1 = to_device(x1r, dtype)
    for i, d in enumerate(descs):
        out = empty_like_acts(T, cfg.hidden, dtype)
        ctx.layer_prefill(d, 0, ss.SS_MLP | ss.SS_NO_RESIDUAL, ids, lens, [0] * len(lens), x1, out)
        torch.cuda.synchronize()
        ref = lm.mlp_block(cfg, vals[0], x1q, k, i)
        parity(to_f64(out, dtype), ref, dtype, tag + "prefill MLP partial of shard %d" % i, spans)
    # ---- residual forms for k == 1
    if k == 1:
        d = descs[0]
        out = empty_like_acts(T, cfg.hidden, dtype)
        ctx.layer_prefill(d, 0, ss.SS_BOTH, ids, lens, [0] * len(lens), x, out)
        torch.cuda.synchronize()
        _, ref2 = lm.layer_forward(cfg, vals[0], xv, batch, lm.KVCache(cfg), 0)
        parity(to_f64(out, dtype), ref2, dtype, tag + "prefill layer output", spans)
    # ---- three decode steps (the sequence of length 32 crosses a page boundary at once)
    cur = list(lens)
    for step in range(3):
        dv, dr = wl.make_activations((len(lens), cfg.hidden), 50 + step, dtype)
        dx = to_device(dr, dtype)
        dbatch = [(sid, 1, n) for sid, n in zip(ids, cur)]
        total = np.zeros((len(lens), cfg.hidden))
        for i, d in enumerate(descs):
            out = empty_like_acts(len(lens), cfg.hidden, dtype)
            ctx.layer_decode(d, 0, ss.SS_ATTN | ss.SS_NO_RESIDUAL, ids, cur, dx, out)
            torch.cuda.synchronize()
            ref = lm.attn_block(cfg, vals[0], dv, dbatch, cache, 0, k, i, _round_kv(cfg))
            parity(to_f64(out, dtype), ref, dtype, tag + "decode step %d shard %d" % (step, i),
                   [(j, j + 1) for j in range(len(lens))])
        cur = [n + 1 for n in cur]
    for d in descs:
        assert len(ctx.kv_page_table(d, ids[4])) == 3     # 32 + 3 tokens -> 3 pages of 16
    ctx.destroy()


def test_chunked_prefill_and_long_decode_split():
    """Prefill in two chunks (second chunk has kv_lens_before > 0), then a decode step on
    a sequence long enough to be split into several work items (> 256 tokens)."""
    cfg = wl.ModelCfg(n_layers=1, dtype=wl.BF16, **SMALL["gqa4_d128"])
    vals, raws = _weights(cfg, 200)
    d = pp_desc(cfg)
    ctx = make_context(cfg, pages=128)
    _load(ctx, d, cfg, raws)
    lens = [700, 45]
    xv, xr = wl.make_activations((sum(lens), cfg.hidden), 8, cfg.dtype)
    cache = lm.KVCache(cfg)
    # oracle: whole prefill at once
    batch = [(0, lens[0], 0), (1, lens[1], 0)]
    ref = lm.attn_block(cfg, vals[0], xv, batch, cache, 0, round_kv=_round_kv(cfg))
    # gpu: first 400 + 45, then the remaining 300 of sequence 0
    first = np.concatenate([xr[:400], xr[700:]])
    out1 = empty_like_acts(445, cfg.hidden, cfg.dtype)
    ctx.layer_prefill(d, 0, ss.SS_ATTN | ss.SS_NO_RESIDUAL, [0, 1], [400, 45], [0, 0], to_device(first, cfg.dtype), out1)
    out2 = empty_like_acts(300, cfg.hidden, cfg.dtype)
    ctx.layer_prefill(d, 0, ss.SS_ATTN | ss.SS_NO_RESIDUAL, [0], [300], [400], to_device(xr[400:700], cfg.dtype), out2)
    torch.cuda.synchronize()
    got = np.concatenate([to_f64(out1, cfg.dtype)[:400], to_f64(out2, cfg.dtype), to_f64(out1, cfg.dtype)[400:]])
    parity(got, ref, cfg.dtype, "chunked prefill (400 + 45, then 300 behind 400)", [(0, 400), (400, 700), (700, 745)])
    dv, dr = wl.make_activations((2, cfg.hidden), 9, cfg.dtype)
    out = empty_like_acts(2, cfg.hidden, cfg.dtype)
    ctx.layer_decode(d, 0, ss.SS_ATTN | ss.SS_NO_RESIDUAL, [0, 1], lens, to_device(dr, cfg.dtype), out)
    torch.cuda.synchronize()
    ref = lm.attn_block(cfg, vals[0], dv, [(0, 1, 700), (1, 1, 45)], cache, 0, round_kv=_round_kv(cfg))
    parity(to_f64(out, cfg.dtype), ref, cfg.dtype, "decode over split work items (700 and 45 tokens)", [(0, 1), (1, 2)])
    ctx.destroy()


@pytest.mark.parametrize("name,dtype", [("gqa4_d128", wl.BF16), ("mha_d128", wl.F16), ("mha_d64_generic", wl.F32)])
def test_mixed_batch_of_prompt_chunks_and_decode_tokens(name, dtype):
    """One layer call over a batch that mixes whole prompts, chunks of prompts and single decode tokens (the batches
    a chunked-prefill engine forms, paper section 6.1 "Baselines" and section 7.1): a decode token is a sequence
    with one new token behind its cached ones, so `ss_layer_prefill` takes the mix as it is.  Compared with the
    oracle on the same batches, and with the same work issued as separate prefill and decode calls."""
    cfg = wl.ModelCfg(n_layers=1, dtype=dtype, **SMALL[name])
    vals, raws = _weights(cfg, 400)
    d = pp_desc(cfg)
    ctx = make_context(cfg, pages=160)
    twin = make_context(cfg, pages=160)                  # the same work as separate calls
    for c in (ctx, twin):
        _load(c, d, cfg, raws)
    cache = lm.KVCache(cfg)
    rk = _round_kv(cfg)

    def run(c, fn_name, batch, xr):
        ids = [b[0] for b in batch]
        T = sum(b[1] for b in batch)
        out = empty_like_acts(T, cfg.hidden, dtype)
        x = to_device(xr, dtype)
        if fn_name == "prefill":
            c.layer_prefill(d, 0, ss.SS_BOTH, ids, [b[1] for b in batch], [b[2] for b in batch], x, out)
        else:
            c.layer_decode(d, 0, ss.SS_BOTH, ids, [b[2] for b in batch], x, out)
        torch.cuda.synchronize()
        return to_f64(out, dtype)

    def spans_of(batch):
        st = np.concatenate([[0], np.cumsum([b[1] for b in batch])])
        return [(int(st[i]), int(st[i + 1])) for i in range(len(batch))]

    # two sequences are on board already (100 and 300 tokens)
    warm = [(1, 100, 0), (2, 300, 0)]
    xv, xr = wl.make_activations((400, cfg.hidden), 31, dtype)
    for c in (ctx, twin):
        run(c, "prefill", warm, xr)
    lm.layer_forward(cfg, vals[0], xv, warm, cache, 0, round_kv=rk)
    # mixed call 1: decode token of 1, a whole new prompt 3 (200), decode token of 2, first chunk (64 of 150) of prompt 4
    # mixed call 2: the rest of prompt 4 behind its first chunk, the next decode token of 1, a one-token prompt 5
    calls = [[(1, 1, 100), (3, 200, 0), (2, 1, 300), (4, 64, 0)],
             [(4, 86, 64), (1, 1, 101), (5, 1, 0)]]
    for n_call, batch in enumerate(calls):
        T = sum(b[1] for b in batch)
        xv, xr = wl.make_activations((T, cfg.hidden), 32 + n_call, dtype)
        got = run(ctx, "prefill", batch, xr)
        _, ref = lm.layer_forward(cfg, vals[0], xv, batch, cache, 0, round_kv=rk)
        sp = spans_of(batch)
        parity(got, ref, dtype, "mixed batch %d (%s) against the oracle" % (n_call, name), sp)
        # the same rows from separate calls: the prompt parts in one prefill call, the decode tokens in one decode call
        pre = [i for i, b in enumerate(batch) if not (b[1] == 1 and b[2] > 0)]
        dec = [i for i, b in enumerate(batch) if b[1] == 1 and b[2] > 0]
        rows = lambda idx: np.concatenate([np.arange(sp[i][0], sp[i][1]) for i in idx])
        sep = np.zeros_like(got)
        sep[rows(pre)] = run(twin, "prefill", [batch[i] for i in pre], xr[rows(pre)])
        sep[rows(dec)] = run(twin, "decode", [batch[i] for i in dec], xr[rows(dec)])
        parity(got, sep, dtype, "mixed batch %d (%s) against separate calls" % (n_call, name), sp)
    # the caches the two ways leave behind hold the same tokens
    for sid, n in ((1, 102), (2, 301), (3, 200), (4, 150), (5, 1)):
        a = wl.storage_to_f64(ctx.kv_read(d, sid, 0, cfg.n_kv_heads), dtype)
        assert a.shape[2] == n
        parity(a, cache.data[sid][0], dtype, "mixed batches (%s), cached K/V of sequence %d" % (name, sid))
        b = wl.storage_to_f64(twin.kv_read(d, sid, 0, cfg.n_kv_heads), dtype)     # (split-K choices differ with the batch size)
        parity(a, b, dtype, "mixed batches (%s), cache of sequence %d against separate calls" % (name, sid))
    ctx.destroy()
    twin.destroy()


@pytest.mark.parametrize("name,dtype", [("gqa4_d128", wl.BF16), ("mha_d64_generic", wl.F32)])
def test_layers_chained_in_one_call_equal_layer_by_layer_calls_and_the_oracle(name, dtype):
    """ss_layers_prefill / ss_layers_decode over a three-layer stage: the same bits as the layers called one by
    one on a twin context (outputs and every layer's cache), the oracle's result within the tolerance, the
    descriptor's own range (layers 1 and 2 of 3) respected, and k > 1 refused."""
    cfg = wl.ModelCfg(n_layers=3, dtype=dtype, **SMALL[name])
    vals, raws = _weights(cfg, 900)
    lens = [5, 70, 33]
    ids = [3, 4, 9]
    T = sum(lens)
    xv, xr = wl.make_activations((T, cfg.hidden), 31, dtype)
    x = to_device(xr, dtype)
    zeros = [0] * len(lens)
    stage = pp_desc(cfg)
    one, twin = make_context(cfg, pages=64), make_context(cfg, pages=64)
    for ctx in (one, twin):
        _load(ctx, stage, cfg, raws)
    # ---- prefill
    y = empty_like_acts(T, cfg.hidden, dtype)
    one.layers_prefill(stage, ids, lens, zeros, x, y)
    cur = x
    for l in range(cfg.n_layers):
        nxt = empty_like_acts(T, cfg.hidden, dtype)
        twin.layer_prefill(stage, l, ss.SS_BOTH, ids, lens, zeros, cur, nxt)
        cur = nxt
    torch.cuda.synchronize()
    assert torch.equal(y, cur)
    cache = lm.KVCache(cfg)
    batch = [(sid, n, 0) for sid, n in zip(ids, lens)]
    ref = lm.run_layers(cfg, vals, xv, batch, cache, 0, cfg.n_layers, round_kv=_round_kv(cfg))
    starts = np.concatenate([[0], np.cumsum(lens)])
    spans = [(int(starts[i]), int(starts[i + 1])) for i in range(len(lens))]
    parity(to_f64(y, dtype), ref, dtype, "three chained layers, prefill output", spans)
    for l in range(cfg.n_layers):
        for sid in ids:
            assert np.array_equal(one.kv_read(stage, sid, l, cfg.n_kv_heads), twin.kv_read(stage, sid, l, cfg.n_kv_heads))
    # ---- two decode steps
    now = list(lens)
    for step in range(2):
        dv, dr = wl.make_activations((len(ids), cfg.hidden), 60 + step, dtype)
        dx = to_device(dr, dtype)
        y = empty_like_acts(len(ids), cfg.hidden, dtype)
        one.layers_decode(stage, ids, now, dx, y)
        cur = dx
        for l in range(cfg.n_layers):
            nxt = empty_like_acts(len(ids), cfg.hidden, dtype)
            twin.layer_decode(stage, l, ss.SS_BOTH, ids, now, cur, nxt)
            cur = nxt
        torch.cuda.synchronize()
        assert torch.equal(y, cur)
        dbatch = [(sid, 1, n) for sid, n in zip(ids, now)]
        ref = lm.run_layers(cfg, vals, dv, dbatch, cache, 0, cfg.n_layers, round_kv=_round_kv(cfg))
        parity(to_f64(y, dtype), ref, dtype, "three chained layers, decode step %d" % step,
               [(j, j + 1) for j in range(len(ids))])
        now = [n + 1 for n in now]
    # ---- a stage of layers 1 and 2 only, and the refusal for k > 1
    part = pp_desc(cfg, 1, 3)
    _load(one, part, cfg, raws)
    y = empty_like_acts(T, cfg.hidden, dtype)
    one.layers_prefill(part, [100, 101, 102], lens, zeros, x, y)
    mid = empty_like_acts(T, cfg.hidden, dtype)
    last = empty_like_acts(T, cfg.hidden, dtype)
    _load(twin, part, cfg, raws)
    twin.layer_prefill(part, 1, ss.SS_BOTH, [100, 101, 102], lens, zeros, x, mid)
    twin.layer_prefill(part, 2, ss.SS_BOTH, [100, 101, 102], lens, zeros, mid, last)
    torch.cuda.synchronize()
    assert torch.equal(y, last)
    if cfg.n_kv_heads % 2 == 0:
        shard = tp_desc(cfg, 2, 0)
        _load(one, shard, cfg, raws)
        with pytest.raises(ss.SeesawError) as e:
            one.layers_prefill(shard, [200], [4], [0], x[:4], y[:4])
        assert e.value.code == ss.SS_EINVAL
    one.destroy()
    twin.destroy()


def test_generic_kernels_forced_for_bf16():
    os.environ["SS_FORCE_GENERIC"] = "1"
    try:
        cfg = wl.ModelCfg(n_layers=1, dtype=wl.BF16, **SMALL["mha_d128"])
        vals, raws = _weights(cfg, 300)
        d = pp_desc(cfg)
        ctx = make_context(cfg, pages=64)
    finally:
        del os.environ["SS_FORCE_GENERIC"]
    _load(ctx, d, cfg, raws)
    lens = [70, 5]
    xv, xr = wl.make_activations((75, cfg.hidden), 10, cfg.dtype)
    out = empty_like_acts(75, cfg.hidden, cfg.dtype)
    ctx.layer_prefill(d, 0, ss.SS_BOTH, [0, 1], lens, [0, 0], to_device(xr, cfg.dtype), out)
    torch.cuda.synchronize()
    _, ref = lm.layer_forward(cfg, vals[0], xv, [(0, 70, 0), (1, 5, 0)], lm.KVCache(cfg), 0)
    parity(to_f64(out, cfg.dtype), ref, cfg.dtype, "generic kernels forced, layer output", [(0, 70), (70, 75)])
    ctx.destroy()


@pytest.mark.parametrize("k", [1, 2])
def test_config1_tiny_model_greedy_decode(k):
    """Configuration 1: 2 layers, hidden 256, 4x64 heads, FFN 688, vocab 512, fp32; 4 prompts of 32
    tokens, prefill emits token 1, then 8 decode steps.  PP (one shard, both layers) and TP k=2 (both
    shards run in turn, partials summed on the host)."""
    work = wl.config1()
    cfg = work.cfg
    vals, raws = _weights(cfg, 1001)
    hv, hr = wl.make_head_weights(cfg, 1099)
    rng = np.random.default_rng(work.notes["seed"])
    prompts = [rng.integers(0, cfg.vocab, size=int(n)) for n in work.prefill_lens]
    steps = work.notes["decode_steps"]
    ref_toks, ref_logits, _ = lm.generate(cfg, vals, hv, prompts, steps, k=1)

    ctx = make_context(cfg, pages=32)
    ctx.load_head(hr["embed"], hr["gf"], hr["wlm"])
    descs = [pp_desc(cfg)] if k == 1 else [tp_desc(cfg, k, i) for i in range(k)]
    for d in descs:
        _load(ctx, d, cfg, raws)
    ids = list(range(len(prompts)))

    def forward(tokens, q_lens, before, decode):
        T = len(tokens)
        x = empty_like_acts(T, cfg.hidden, cfg.dtype)
        ctx.embed(tokens, x)
        for l in range(cfg.n_layers):
            if k == 1:
                y = empty_like_acts(T, cfg.hidden, cfg.dtype)
                if decode:
                    ctx.layer_decode(descs[0], l, ss.SS_BOTH, ids, before, x, y)
                else:
                    ctx.layer_prefill(descs[0], l, ss.SS_BOTH, ids, q_lens, before, x, y)
                x = y
            else:
                for phase in (ss.SS_ATTN, ss.SS_MLP):
                    acc = x.clone()
                    for d in descs:
                        part = empty_like_acts(T, cfg.hidden, cfg.dtype)
                        if decode:
                            ctx.layer_decode(d, l, phase, ids, before, x, part)
                        else:
                            ctx.layer_prefill(d, l, phase, ids, q_lens, before, x, part)
                        torch.cuda.synchronize()
                        # host-side sum of the partials: the stand-in for the all-reduce
                        acc = torch.from_numpy(acc.cpu().numpy() + part.cpu().numpy()).cuda()
                    x = acc
        return x

    lens = [len(p) for p in prompts]
    x = forward(np.concatenate(prompts), lens, [0] * len(lens), False)
    last = torch.tensor(np.cumsum(lens) - 1, device="cuda")
    logits = torch.empty((len(prompts), cfg.vocab), device="cuda", dtype=torch.float32)
    ctx.lm_head(x[last].contiguous(), len(prompts), logits)
    torch.cuda.synchronize()
    got_logits = [logits.cpu().numpy().astype(np.float64)]
    toks = [lm.greedy(got_logits[0])]
    for s in range(steps):
        # teacher forcing on the oracle's token keeps the two runs on the same path
        x = forward(ref_toks[:, s], [1] * len(lens), lens, True)
        ctx.lm_head(x, len(prompts), logits)
        torch.cuda.synchronize()
        got_logits.append(logits.cpu().numpy().astype(np.float64))
        toks.append(lm.greedy(got_logits[-1]))
        lens = [n + 1 for n in lens]
    for s, (g, r) in enumerate(zip(got_logits, ref_logits)):
        assert rel_err(g, r) <= 1e-4, "logits at step %d" % s
        top2 = np.sort(r, axis=-1)[:, -2:]
        decisive = (top2[:, 1] - top2[:, 0]) > 10 * 1e-4 * np.max(np.abs(r))
        assert np.array_equal(toks[s][decisive], ref_toks[decisive, s])
    assert len(ctx.kv_page_table(descs[0], 0)) == 3      # 32 + 8 tokens -> 3 pages of 16
    ctx.destroy()


def test_descriptor_and_argument_errors():
    cfg = wl.ModelCfg(n_layers=2, dtype=wl.BF16, **SMALL["gqa4_d128"])
    ctx = make_context(cfg, pages=4)
    vals, raws = _weights(cfg, 400)
    x = empty_like_acts(4, cfg.hidden, cfg.dtype)
    y = empty_like_acts(4, cfg.hidden, cfg.dtype)
    with pytest.raises(ss.SeesawError) as e:        # k does not divide the kv heads
        ctx.load_layer(ss.ShardDesc(ss.SS_TP, 4, 0, 0, 2), 0, raws[0])
    assert e.value.code == ss.SS_EINVAL
    with pytest.raises(ss.SeesawError) as e:        # layer outside the range
        ctx.load_layer(ss.ShardDesc(ss.SS_PP, 1, 0, 0, 1), 1, raws[1])
    assert e.value.code == ss.SS_EINVAL
    d = pp_desc(cfg)
    with pytest.raises(ss.SeesawError) as e:        # not loaded
        ctx.layer_prefill(d, 0, ss.SS_BOTH, [0], [4], [0], x, y)
    assert e.value.code == ss.SS_EINVAL
    _load(ctx, d, cfg, raws)
    with pytest.raises(ss.SeesawError) as e:        # unknown sequence with cached tokens claimed
        ctx.layer_decode(d, 0, ss.SS_BOTH, [5], [3], x[:1], y[:1])
    assert e.value.code == ss.SS_ENOENT
    with pytest.raises(ss.SeesawError) as e:        # pool of 4 pages cannot hold 80 tokens
        big = empty_like_acts(80, cfg.hidden, cfg.dtype)
        ctx.layer_prefill(d, 0, ss.SS_BOTH, [0], [80], [0], big, empty_like_acts(80, cfg.hidden, cfg.dtype))
    assert e.value.code == ss.SS_ENOMEM
    assert ctx.kv_free_pages(d) == 4
    with pytest.raises(ss.SeesawError) as e:        # 2 + 3 pages: the batch fails as a whole and keeps no page
        xb = empty_like_acts(70, cfg.hidden, cfg.dtype)
        ctx.layer_prefill(d, 0, ss.SS_BOTH, [1, 2], [30, 40], [0, 0], xb, empty_like_acts(70, cfg.hidden, cfg.dtype))
    assert e.value.code == ss.SS_ENOMEM
    assert ctx.kv_free_pages(d) == 4
    td = tp_desc(cfg, 2, 0)
    _load(ctx, td, cfg, raws)
    with pytest.raises(ss.SeesawError) as e:        # fused phases need k == 1
        ctx.layer_prefill(td, 0, ss.SS_BOTH, [1], [4], [0], x, y)
    assert e.value.code == ss.SS_EINVAL
    ctx.destroy()


@pytest.mark.parametrize("n_rows,vocab", [(5, 256), (70, 2048), (300, 1024)])
def test_lm_head_bf16_matches_oracle(n_rows, vocab):
    """Final norm + LM head of a bf16 model (fp32 logits out of the MFMA GEMM, with and without split-K)."""
    cfg = wl.ModelCfg(hidden=512, n_q_heads=4, n_kv_heads=4, head_dim=128, ffn=1024, n_layers=1, vocab=vocab, dtype=wl.BF16)
    hv, hr = wl.make_head_weights(cfg, 77)
    ctx = make_context(cfg, pages=4)
    ctx.load_head(hr["embed"], hr["gf"], hr["wlm"])
    xv, xr = wl.make_activations((n_rows, cfg.hidden), 78, cfg.dtype)
    logits = torch.empty((n_rows, vocab), device="cuda", dtype=torch.float32)
    for rep in range(2):                      # the second call finds the split-K workspace of the layer calls, if any
        ctx.lm_head(to_device(xr, cfg.dtype), n_rows, logits)
        torch.cuda.synchronize()
        ref = lm.lm_logits(cfg, hv, xv)
        assert rel_err(logits.cpu().numpy(), ref) <= tol(cfg.dtype)
    ctx.destroy()


def test_prefill_many_pages_six_kv_heads_cache_matches_oracle():
    """A prompt batch of more than 256 page units with a kv head count that is not a multiple of four: the
    RoPE + page-write kernel takes four kv heads per block at this size, the last block two; the attention
    block's output and the cache it leaves behind are compared with the oracle."""
    cfg = wl.ModelCfg(hidden=768, n_q_heads=12, n_kv_heads=6, head_dim=128, ffn=1024, n_layers=1, dtype=wl.BF16)
    vals, raws = _weights(cfg, 910)
    lens = [1500, 1307, 1390, 5]
    T = sum(lens)
    xv, xr = wl.make_activations((T, cfg.hidden), 911, cfg.dtype)
    ctx = make_context(cfg, pages=300)
    d = pp_desc(cfg)
    _load(ctx, d, cfg, raws)
    ids = [3, 4, 5, 6]
    batch = [(s, n, 0) for s, n in zip(ids, lens)]
    out = empty_like_acts(T, cfg.hidden, cfg.dtype)
    ctx.layer_prefill(d, 0, ss.SS_ATTN, ids, lens, [0] * 4, to_device(xr, cfg.dtype), out)
    torch.cuda.synchronize()
    cache = lm.KVCache(cfg)
    ref = xv + lm.attn_block(cfg, vals[0], xv, batch, cache, 0, 1, 0, _round_kv(cfg))
    starts = np.concatenate([[0], np.cumsum(lens)])
    parity(to_f64(out, cfg.dtype), ref, cfg.dtype, "six kv heads, attention block with residual",
           [(int(starts[i]), int(starts[i + 1])) for i in range(4)])
    for sid, n in zip(ids, lens):
        got = wl.storage_to_f64(ctx.kv_read(d, sid, 0, cfg.n_kv_heads), cfg.dtype)
        parity(got, cache.data[sid][0], cfg.dtype, "six kv heads, cached K/V of sequence %d" % sid)
    ctx.destroy()


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F16])
def test_prefill_wide_score_range_matches_oracle(dtype):
    """Weights three times the usual scale make the attention scores nine times as wide (standard deviation
    about 2.7 in the exponent's base-2 units, row maxima near 9): the running maximum of a row then grows both
    in small steps and by more than the slack the prefill kernel allows its reference maximum before it rescales
    the accumulated output, so both branches of that rule are exercised on rows of up to 57 steps."""
    cfg = wl.ModelCfg(n_layers=1, dtype=dtype, **SMALL["mha_d128"])
    v, r = wl.make_layer_weights(cfg, 300, std=0.06)
    lens = [900, 300, 77]
    T = sum(lens)
    xv, xr = wl.make_activations((T, cfg.hidden), 17, dtype)
    ctx = make_context(cfg, pages=128)
    d = pp_desc(cfg)
    ctx.load_layer(d, 0, r)
    ids = [5, 6, 7]
    out = empty_like_acts(T, cfg.hidden, dtype)
    ctx.layer_prefill(d, 0, ss.SS_ATTN | ss.SS_NO_RESIDUAL, ids, lens, [0] * 3, to_device(xr, dtype), out)
    torch.cuda.synchronize()
    ref = lm.attn_block(cfg, v, xv, [(i, n, 0) for i, n in zip(ids, lens)], lm.KVCache(cfg), 0, round_kv=_round_kv(cfg))
    parity(to_f64(out, dtype), ref, dtype, "wide score range, attention partial (dtype %d)" % dtype,
           [(0, 900), (900, 1200), (1200, 1277)], ROW_TOL_FULL[dtype])
    ctx.destroy()


def test_prefill_prompt_longer_than_64_tiles_matches_oracle():
    """A prompt of 4500 tokens is 71 tiles of 64 cached tokens for its last queries: the prefill attention keeps
    the page-table entries of 64 tiles in a register and has to refill it once; a second, short prompt shares
    the batch.  Then one decode step on the long sequence (several work items)."""
    cfg = wl.ModelCfg(n_layers=1, dtype=wl.BF16, **SMALL["gqa4_d128"])
    v, r = wl.make_layer_weights(cfg, 500)
    lens = [4500, 90]
    T = sum(lens)
    xv, xr = wl.make_activations((T, cfg.hidden), 23, cfg.dtype)
    ctx = make_context(cfg, pages=300, max_seq_len=4608)
    d = pp_desc(cfg)
    ctx.load_layer(d, 0, r)
    ids = [3, 4]
    out = empty_like_acts(T, cfg.hidden, cfg.dtype)
    ctx.layer_prefill(d, 0, ss.SS_ATTN | ss.SS_NO_RESIDUAL, ids, lens, [0, 0], to_device(xr, cfg.dtype), out)
    torch.cuda.synchronize()
    cache = lm.KVCache(cfg)
    ref = lm.attn_block(cfg, v, xv, [(i, n, 0) for i, n in zip(ids, lens)], cache, 0, round_kv=_round_kv(cfg))
    got = to_f64(out, cfg.dtype)
    parity(got, ref, cfg.dtype, "prompt of 4500 tokens next to one of 90", [(0, lens[0]), (lens[0], T)])
    dv, dr = wl.make_activations((2, cfg.hidden), 24, cfg.dtype)
    out = empty_like_acts(2, cfg.hidden, cfg.dtype)
    ctx.layer_decode(d, 0, ss.SS_ATTN | ss.SS_NO_RESIDUAL, ids, lens, to_device(dr, cfg.dtype), out)
    torch.cuda.synchronize()
    ref = lm.attn_block(cfg, v, dv, [(3, 1, 4500), (4, 1, 90)], cache, 0, round_kv=_round_kv(cfg))
    parity(to_f64(out, cfg.dtype), ref, cfg.dtype, "decode behind the 4500-token prompt", [(0, 1), (1, 2)])
    ctx.destroy()
