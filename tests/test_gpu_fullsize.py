"""Parity at the full sizes of configurations 2-5, in the launch configuration
bench.py times.  The GPU runs the whole batch; the oracle (which cannot run a
whole batch in reasonable time) recomputes sampled sequences one by one from the
same inputs: a layer treats sequences independently, so the oracle's result for
one sequence, given that sequence's rows of the input, is exactly what the full
batch must contain in those rows (teacher forcing on the layer input for
multi-layer runs).  Data movement at full size is checked bit for bit.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import kv_tier as kt
from oracle import layer_math as lm

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2503_06433_amd as ss
    from paper_2503_06433_amd.harness import (make_context, to_device, to_f64, to_raw, empty_like_acts, rel_err, ROW_TOL_FULL,
                                              pp_desc, tp_desc)
    from paper_2503_06433_amd.harness import parity as _parity

TOL = 2e-2


def parity(got, ref, dtype, label, spans=None):
    """the harness check with the per-row bound of the full-size class"""
    return _parity(got, ref, dtype, label, spans, ROW_TOL_FULL[dtype])


def _round_kv(a):
    return wl.bf16_to_f32(wl.bf16_bits(a.astype(np.float32))).astype(np.float64)


def _sample(lens, n_extra, seed):
    """shortest, median, longest + a few seeded others"""
    order = np.argsort(lens)
    picks = {int(order[0]), int(order[len(order) // 2]), int(order[-1])}
    rng = np.random.default_rng(seed)
    while len(picks) < min(len(lens), 3 + n_extra):
        picks.add(int(rng.integers(0, len(lens))))
    return sorted(picks)


def _pages_for(lens, extra=0):
    return int(sum(-(-(int(n) + extra) // 16) for n in lens)) + 8


def _host_weights_from_device(dev_w):
    return {k: wl.bf16_to_f32(to_raw(v, wl.BF16)).astype(np.float64) for k, v in dev_w.items()}


def _seq_kv_from_staging(stg, offs, i, n_layers_l, n_heads_l, s, d):
    """logical cache [layers, 2, heads, s, d] (float64) of sequence i out of the device staging tensor"""
    raw = to_raw(stg[int(offs[i]):int(offs[i + 1])], wl.BF16)
    return wl.bf16_to_f32(raw).astype(np.float64).reshape(n_layers_l, 2, n_heads_l, s, d)


def test_config2_prefill_full_batch_sampled_rows():
    work = wl.config2()
    cfg = work.cfg
    vals, raws = wl.make_layer_weights(cfg, 2001)
    lens = [int(v) for v in work.prefill_lens]
    T = sum(lens)
    assert T == 20018
    xv, xr = wl.make_activations((T, cfg.hidden), 2002, cfg.dtype)
    ctx = make_context(cfg, pages=_pages_for(lens), max_seq_len=4096)
    desc = pp_desc(cfg)
    ctx.load_layer(desc, 0, raws)
    ids = list(range(len(lens)))
    out = empty_like_acts(T, cfg.hidden, cfg.dtype)
    ctx.layer_prefill(desc, 0, ss.SS_BOTH, ids, lens, [0] * len(lens), to_device(xr, cfg.dtype), out)
    part = empty_like_acts(T, cfg.hidden, cfg.dtype)
    ctx.layer_prefill(desc, 0, ss.SS_ATTN | ss.SS_NO_RESIDUAL, ids, lens, [0] * len(lens), to_device(xr, cfg.dtype), part)
    torch.cuda.synchronize()
    got, got_o = to_f64(out, cfg.dtype), to_f64(part, cfg.dtype)
    starts = np.concatenate([[0], np.cumsum(lens)])
    for i in _sample(lens, 0, 1):
        a, b = int(starts[i]), int(starts[i + 1])
        cache = lm.KVCache(cfg)
        o = lm.attn_block(cfg, vals, xv[a:b], [(i, lens[i], 0)], cache, 0, round_kv=_round_kv)
        x1 = xv[a:b] + o
        x2 = x1 + lm.mlp_block(cfg, vals, x1)
        parity(got_o[a:b], o, cfg.dtype, "C2 prefill attention block, sequence %d (%d tokens)" % (i, lens[i]))
        parity(got[a:b], x2, cfg.dtype, "C2 prefill layer output, sequence %d (%d tokens)" % (i, lens[i]))
        kv = wl.storage_to_f64(ctx.kv_read(desc, i, 0, cfg.n_kv_heads), cfg.dtype)
        parity(kv, cache.data[i][0], cfg.dtype, "C2 prefill cached K/V, sequence %d" % i)
    ctx.destroy()


def _run_decode_case(work, k, shard, w_seed, kv_seed, x_seed, n_extra):
    cfg = work.cfg
    vals, raws = wl.make_layer_weights(cfg, w_seed)
    lens = [int(v) for v in work.decode_kv_lens]
    B, d = len(lens), cfg.head_dim
    nh = cfg.n_kv_heads // k
    desc = tp_desc(cfg, k, shard)
    ctx = make_context(cfg, pages=_pages_for(lens, 1), max_seq_len=4608)
    ctx.load_layer(desc, 0, raws)
    ids = list(range(5000, 5000 + B))
    offs = kt.staging_offsets(lens, 1, nh, d)
    stg = wl.device_normal((int(offs[-1]),), kv_seed, cfg.dtype)
    ctx.kv_import_dev(desc, ids, lens, stg)
    dv, dr = wl.make_activations((B, cfg.hidden), x_seed, cfg.dtype)
    dx = to_device(dr, cfg.dtype)
    o_part = empty_like_acts(B, cfg.hidden, cfg.dtype)
    ctx.layer_decode(desc, 0, ss.SS_ATTN | ss.SS_NO_RESIDUAL, ids, lens, dx, o_part)
    y_part = empty_like_acts(B, cfg.hidden, cfg.dtype)
    ctx.layer_decode(desc, 0, ss.SS_MLP | ss.SS_NO_RESIDUAL, ids, lens, dx, y_part)
    torch.cuda.synchronize()
    got_o, got_y = to_f64(o_part, cfg.dtype), to_f64(y_part, cfg.dtype)
    (_, _), (g0, g1), _ = lm.shard_ranges(cfg, k, shard)
    picks = _sample(lens, n_extra, kv_seed)
    ref_o = np.zeros((len(picks), cfg.hidden))
    for j, i in enumerate(picks):
        cache = lm.KVCache(cfg)
        cache.ensure(i, lens[i] + 1)
        cache.data[i][0, :, g0:g1, :lens[i]] = _seq_kv_from_staging(stg, offs, i, 1, nh, lens[i], d)[0]
        ref_o[j] = lm.attn_block(cfg, vals, dv[i:i + 1], [(i, 1, lens[i])], cache, 0, k, shard, _round_kv)[0]
        # the step appended the new token's K and V at position lens[i]
        kv = wl.storage_to_f64(ctx.kv_read(desc, ids[i], 0, nh), cfg.dtype)
        assert kv.shape[2] == lens[i] + 1
        parity(kv[:, :, lens[i]], cache.data[i][0, :, g0:g1, lens[i]], cfg.dtype,
               "%s decode, appended K/V of sequence %d" % (work.name, i))
    each = [(j, j + 1) for j in range(len(picks))]
    parity(got_o[picks], ref_o, cfg.dtype, "%s decode attention partial (%d sampled sequences)" % (work.name, len(picks)), each)
    ref_y = lm.mlp_block(cfg, vals, dv[picks], k, shard)
    parity(got_y[picks], ref_y, cfg.dtype, "%s decode MLP partial" % work.name, each)
    if k == 1:
        out = empty_like_acts(B, cfg.hidden, cfg.dtype)
        ctx.layer_decode(desc, 0, ss.SS_BOTH, ids, lens, dx, out)
        torch.cuda.synchronize()
        x1 = dv[picks] + ref_o
        x2 = x1 + lm.mlp_block(cfg, vals, x1)
        parity(to_f64(out, cfg.dtype)[picks], x2, cfg.dtype, "%s decode layer output" % work.name, each)
    ctx.destroy()


def test_config2_decode_256_sequences():
    _run_decode_case(wl.config2(), 1, 0, 2001, 2004, 2003, 5)


def test_config3_tp4_shard_decode_512_sequences():
    _run_decode_case(wl.config3(), 4, 1, 3001, 3004, 3003, 3)


def test_config4_gqa_tp8_shard_decode_1024_sequences():
    _run_decode_case(wl.config4(), 8, 3, 4001, 4004, 4003, 3)


def test_config3_pp_prefill_full_layer_sampled_rows():
    work = wl.config3()
    cfg = work.cfg
    vals, raws = wl.make_layer_weights(cfg, 3001)
    lens = [int(v) for v in work.prefill_lens]
    T = sum(lens)
    xv, xr = wl.make_activations((T, cfg.hidden), 3002, cfg.dtype)
    ctx = make_context(cfg, pages=_pages_for(lens), max_seq_len=4096)
    desc = pp_desc(cfg)
    ctx.load_layer(desc, 0, raws)
    ids = list(range(len(lens)))
    out = empty_like_acts(T, cfg.hidden, cfg.dtype)
    ctx.layer_prefill(desc, 0, ss.SS_BOTH, ids, lens, [0] * len(lens), to_device(xr, cfg.dtype), out)
    torch.cuda.synchronize()
    got = to_f64(out, cfg.dtype)
    starts = np.concatenate([[0], np.cumsum(lens)])
    order = np.argsort(lens)
    for i in (int(order[0]), int(order[len(order) // 2]), int(order[-1])):      # shortest, median, longest prompt
        a, b = int(starts[i]), int(starts[i + 1])
        _, x2 = lm.layer_forward(cfg, vals, xv[a:b], [(i, lens[i], 0)], lm.KVCache(cfg), 0, round_kv=_round_kv)
        parity(got[a:b], x2, cfg.dtype, "C3 prefill layer output, sequence %d (%d tokens)" % (i, lens[i]))
    ctx.destroy()


def test_config5_pp_slice_prefill_and_overlapped_reshard():
    """Ten 70B-shape layers on one GPU (the k = 8 pipeline slice): prefill of 64 prompts, re-shard of
    their caches to the k = 8 head-sharded layout through the host tier while the next batch is
    prefilled, layer outputs checked by teacher forcing on sampled layers and sequences."""
    work = wl.config5()
    cfg = work.cfg
    lens = [int(v) for v in work.prefill_lens]
    lens2 = [int(v) for v in work.notes["next_batch_lens"]]
    T, T2 = sum(lens), sum(lens2)
    L, d, n_kv = cfg.n_layers, cfg.head_dim, cfg.n_kv_heads
    tier_bytes = T * L * 2 * n_kv * d * 2 + (1 << 20)
    ctx = make_context(cfg, pages=_pages_for(lens) + _pages_for(lens2), tier_bytes=tier_bytes,
                       pinned_bytes=512 << 20, max_seq_len=4096)
    pp = pp_desc(cfg)
    shard = 5
    tp = tp_desc(cfg, 8, shard)
    check_layers = (0, L - 1)
    host_w = {}
    for l in range(L):
        w = wl.device_layer_weights(cfg, 5100 + l)
        ctx.load_layer(pp, l, w, ss.SS_DEVICE)
        if l in check_layers:
            host_w[l] = _host_weights_from_device(w)
        del w
    torch.cuda.empty_cache()
    ids = list(range(len(lens)))
    ids2 = list(range(1000, 1000 + len(lens2)))
    x = wl.device_normal((T, cfg.hidden), 5002, cfg.dtype)
    x2 = wl.device_normal((T2, cfg.hidden), 5003, cfg.dtype)

    def run_slice(xin, sids, slens, keep):
        cur, kept = xin, {}
        for l in range(L):
            nxt = torch.empty_like(cur)
            ctx.layer_prefill(pp, l, ss.SS_BOTH, sids, slens, [0] * len(slens), cur, nxt)
            if l in keep:
                kept[l] = (cur, nxt)
            cur = nxt
        return cur, kept

    out, kept = run_slice(x, ids, lens, check_layers)
    torch.cuda.synchronize()
    # ---- layer parity by teacher forcing: the oracle gets the GPU's input of that layer
    starts = np.concatenate([[0], np.cumsum(lens)])
    order = np.argsort(lens)
    for l in check_layers:
        xin, xout = kept[l]
        for i in (int(order[0]), int(order[2])):
            a, b = int(starts[i]), int(starts[i + 1])
            cache = lm.KVCache(cfg)
            _, ref = lm.layer_forward(cfg, host_w[l], to_f64(xin[a:b], cfg.dtype), [(i, lens[i], 0)], cache, l,
                                      round_kv=_round_kv)
            parity(to_f64(xout[a:b], cfg.dtype), ref, cfg.dtype,
                   "C5 layer %d output, sequence %d (%d tokens)" % (l, i, lens[i]))
            kv = wl.storage_to_f64(ctx.kv_read(pp, i, l, n_kv), cfg.dtype)
            parity(kv, cache.data[i][l], cfg.dtype, "C5 layer %d cached K/V, sequence %d" % (l, i))
    w0 = host_w[0]
    del kept, host_w
    # ---- re-shard of batch 1 overlapped with the prefill of batch 2
    alone, _ = run_slice(x2, ids2, lens2, ())
    torch.cuda.synchronize()
    alone = alone.clone()
    # ---- a long prompt at the 70B GQA shape (the next batch holds one of 3931 tokens; the first batch none above
    # 2627): the attention block of layer 0 and the cache it writes.  The MLP of that many tokens at this width
    # would take the CPU minutes; it is per token and is covered by the short sequences above.
    order2 = np.argsort(lens2)
    long_i = int(order2[-1])
    assert lens2[long_i] >= 3000
    starts2 = np.concatenate([[0], np.cumsum(lens2)])
    part = torch.empty_like(x2)
    ctx.layer_prefill(pp, 0, ss.SS_ATTN | ss.SS_NO_RESIDUAL, ids2, lens2, [0] * len(lens2), x2, part)
    torch.cuda.synchronize()
    a, b = int(starts2[long_i]), int(starts2[long_i + 1])
    cache = lm.KVCache(cfg)
    ref_o = lm.attn_block(cfg, w0, to_f64(x2[a:b], cfg.dtype), [(long_i, lens2[long_i], 0)], cache, 0,
                          round_kv=_round_kv)
    parity(to_f64(part[a:b], cfg.dtype), ref_o, cfg.dtype,
           "C5 layer 0 attention block, long sequence (%d tokens)" % lens2[long_i])
    kv = wl.storage_to_f64(ctx.kv_read(pp, ids2[long_i], 0, n_kv), cfg.dtype)
    parity(kv, cache.data[long_i][0], cfg.dtype, "C5 layer 0 cached K/V, long sequence")
    del part, w0, ref_o, kv, cache
    ctx.kv_free(pp, ids2)
    snap = {i: [ctx.kv_read(pp, i, l, n_kv) for l in (0, L - 1)] for i in (int(order[0]), int(order[-1]))}
    ctx.kv_reshard(pp, tp, ids)
    overl, _ = run_slice(x2, ids2, lens2, ())
    torch.cuda.synchronize()
    ctx.sync()
    assert torch.equal(overl, alone), "prefill output changed under the overlapped re-shard"
    # the head-sharded copy equals the head slice of what the pipeline slice held (any size: property)
    for i, per_layer in snap.items():
        for l, full in zip((0, L - 1), per_layer):
            assert np.array_equal(ctx.kv_read(tp, i, l, 1), full[:, shard:shard + 1])
    assert ctx.host_tier_used_bytes() == tier_bytes - (1 << 20)
    ctx.destroy()


def test_config5_reshard_all_bytes_synthetic_cache():
    """The same movement with seeded random caches, every byte compared with the oracle's index
    formula (tier image) and with the head slice (shard content)."""
    work = wl.config5()
    cfg = work.cfg
    lens = [int(v) for v in work.prefill_lens]
    L, d, n_kv = cfg.n_layers, cfg.head_dim, cfg.n_kv_heads
    T = sum(lens)
    per_tok = L * 2 * n_kv * d
    tier_bytes = T * per_tok * 2
    ctx = make_context(cfg, pages=_pages_for(lens), tier_bytes=tier_bytes, pinned_bytes=256 << 20, max_seq_len=4096)
    pp = pp_desc(cfg)
    ids = list(range(len(lens)))
    offs = kt.staging_offsets(lens, L, n_kv, d)
    stg = wl.device_normal((int(offs[-1]),), 5004, cfg.dtype)
    ctx.kv_import_dev(pp, ids, lens, stg)
    torch.cuda.synchronize()
    shard = 2
    tp = tp_desc(cfg, 8, shard)
    ctx.kv_reshard(pp, tp, ids)
    ctx.sync()
    order = np.argsort(lens)
    oracle_checked = {int(order[0]), int(order[1]), int(order[len(order) // 2])}
    for i in ids:
        content = to_raw(stg[int(offs[i]):int(offs[i + 1])], cfg.dtype).reshape(L, 2, n_kv, lens[i], d)
        if i in oracle_checked:
            n = kt.tier_seq_elems(L, n_kv, d, lens[i])
            tier = np.zeros(n, dtype=np.uint16)
            kt.tier_put(tier, 0, content, n_kv, (0, L), (0, n_kv))
            want = kt.tier_get(tier, 0, lens[i], n_kv, d, (0, L), (shard, shard + 1))
            per_layer = 2 * n_kv * lens[i] * d
            for l in range(L):
                assert np.array_equal(ctx.host_tier_read(i, l, lens[i]).reshape(-1), tier[l * per_layer:(l + 1) * per_layer])
        else:
            want = content[:, :, shard:shard + 1]
        for l in range(L):
            assert np.array_equal(ctx.kv_read(tp, i, l, 1), want[l]), "sequence %d layer %d" % (i, l)
    ctx.destroy()


def test_config3_weight_reshard_pp_layer_to_tp4_shard_bit_exact():
    """The weight half of the configuration-3 switch at full layer size (13B shape: 317 M parameters per
    layer): one layer of the pipeline stage is replaced by shard 2 of 4 of the same layer, reloaded from
    the CPU copy; every tensor the shard then holds is compared bit for bit with the oracle's slice."""
    from oracle import weight_shard as ows
    from paper_2503_06433_amd.binding import W_NAMES
    from paper_2503_06433_amd.harness import stored_form
    cfg = wl.config3().cfg
    _, raws = wl.make_layer_weights(cfg, 3301)
    ctx = make_context(cfg, pages=8)
    ctx.host_weights_put(0, raws)
    stage, shard = pp_desc(cfg, 0, 1), tp_desc(cfg, 4, 2, 0, 1)
    ctx.reshard_weights(None, stage)
    ctx.reshard_weights(stage, shard)
    assert ctx.weights_shard_bytes(shard) == ows.reload_elems(cfg, 4, 0, 1) * 2
    ref = stored_form(ows.shard_weights(cfg, raws, 4, 2), cfg.dtype)      # gains folded into wq, wk, wv, wg, wu
    for which, name in enumerate(W_NAMES):
        got = ctx.weights_read(shard, 0, which, ref[name].size)
        assert np.array_equal(got, ref[name].reshape(-1)), name
    ctx.destroy()


def test_many_tokens_on_a_narrow_layer_short_contractions_on_the_large_output_kernel():
    """70 000 tokens through a layer of hidden size 256: every projection has enough output tiles for the
    persistent large-output GEMM but contractions of only 4 or 5 slices (K = 256, 320) and ragged output widths
    (gate/up: 640 columns), the corner where that kernel's prefetches, waits and tile boundaries lie closest
    together.  700 prompts of 100 tokens; eight of them recomputed by the oracle."""
    cfg = wl.ModelCfg(n_layers=1, dtype=wl.BF16, hidden=256, n_q_heads=2, n_kv_heads=2, head_dim=128, ffn=320)
    vals, raws = wl.make_layer_weights(cfg, 7301)
    lens = [100] * 700
    T = sum(lens)
    xv, xr = wl.make_activations((T, cfg.hidden), 7302, cfg.dtype)
    ctx = make_context(cfg, pages=_pages_for(lens), max_seq_len=256)
    desc = pp_desc(cfg)
    ctx.load_layer(desc, 0, raws)
    ids = list(range(len(lens)))
    out = empty_like_acts(T, cfg.hidden, cfg.dtype)
    ctx.layer_prefill(desc, 0, ss.SS_BOTH, ids, lens, [0] * len(lens), to_device(xr, cfg.dtype), out)
    torch.cuda.synchronize()
    got = to_f64(out, cfg.dtype)
    assert np.isfinite(got).all()
    for i in (0, 1, 255, 256, 349, 511, 698, 699):             # around tile boundaries of 256 tokens, first and last
        a, b = 100 * i, 100 * (i + 1)
        _, ref = lm.layer_forward(cfg, vals, xv[a:b], [(i, 100, 0)], lm.KVCache(cfg), 0)
        parity(got[a:b], ref, cfg.dtype, "narrow layer, sequence %d" % i)
    ctx.destroy()


@pytest.mark.parametrize("hidden,n_q,n_kv,ffn,T", [(8192, 16, 8, 2048, 777), (4096, 8, 8, 8192, 777), (8192, 16, 8, 2048, 1000)])
def test_ragged_token_count_on_the_projections_cut_along_the_contraction(hidden, n_q, n_kv, ffn, T):
    """Between a decode batch and a prefill batch (some hundreds of tokens, a count that is no multiple of any tile)
    wide layers send their projections to the large-output GEMM with the contraction cut into ranges and fp32
    partial sums: with hidden 8192 the QKV product (plain store) and the gate/up product (SwiGLU), with
    hidden 4096 and an inner width of 8192 the down projection (residual).  Single-token sequences, so the
    attention is the identity on V and the oracle can afford every row."""
    cfg = wl.ModelCfg(n_layers=1, dtype=wl.BF16, hidden=hidden, n_q_heads=n_q, n_kv_heads=n_kv, head_dim=128, ffn=ffn)
    vals, raws = wl.make_layer_weights(cfg, 7401)
    lens = [1] * T
    xv, xr = wl.make_activations((T, cfg.hidden), 7402, cfg.dtype)
    ctx = make_context(cfg, pages=T + 8, max_seq_len=64)
    desc = pp_desc(cfg)
    ctx.load_layer(desc, 0, raws)
    ids = list(range(T))
    out = empty_like_acts(T, cfg.hidden, cfg.dtype)
    ctx.layer_prefill(desc, 0, ss.SS_BOTH, ids, lens, [0] * T, to_device(xr, cfg.dtype), out)
    torch.cuda.synchronize()
    got = to_f64(out, cfg.dtype)
    assert np.isfinite(got).all()
    _, ref = lm.layer_forward(cfg, vals, xv, [(i, 1, 0) for i in range(T)], lm.KVCache(cfg), 0)
    parity(got, ref, cfg.dtype, "ragged %d tokens, hidden %d" % (T, hidden))
    ctx.destroy()
