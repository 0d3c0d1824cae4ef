"""GPU parity of the offline engine loop (transition-minimizing scheduling over
the tiered KV buffer, weight and KV re-sharding at every switch) against the
CPU oracles, through the C ABI.

Decisions are integers: the trace of actions must equal the scheduling oracle's
exactly.  Tokens are greedy choices over fp32 logits: they must equal the layer
oracle's own greedy run of each request wherever the oracle's choice is decisive
(top-2 logit gap above ten times the logit tolerance); behind a non-decisive
step of a request the two runs may legitimately part, so that request is
compared no further.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import layer_math as lm
from oracle import scheduler as sc

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2503_06433_amd as ss
    from paper_2503_06433_amd.harness import make_context, pp_desc, tp_desc


def _model(cfg, seed):
    vals, raws = [], []
    for l in range(cfg.n_layers):
        v, r = wl.make_layer_weights(cfg, seed + l)
        vals.append(v)
        raws.append(r)
    hv, hr = wl.make_head_weights(cfg, seed + 99)
    return vals, raws, hv, hr


def _tok_bytes(cfg):
    es = 4 if cfg.dtype == wl.F32 else 2
    return 2 * cfg.n_kv_heads * cfg.head_dim * es * cfg.n_layers


def _check_tokens(cfg, vals, hv, prompts, out_lens, got, logit_tol):
    compared = 0
    for i, (p, o) in enumerate(zip(prompts, out_lens)):
        ref, logits, _ = lm.generate(cfg, vals, hv, [np.asarray(p)], o - 1)
        for s in range(o):
            r = logits[s][0]
            top2 = np.sort(r)[-2:]
            decisive = (top2[1] - top2[0]) > 10 * logit_tol * np.max(np.abs(r))
            if got[i][s] != ref[0, s]:
                assert not decisive, "request %d token %d: %d instead of %d" % (i, s, got[i][s], ref[0, s])
                break
            compared += 1
    return compared


def _run(cfg, seed, prompts, out_lens, tier_tokens, gpu_pages, mpt, mds, reshard, stream=0, group=0):
    vals, raws, hv, hr = _model(cfg, seed)
    ctx = make_context(cfg, pages=gpu_pages, tier_bytes=tier_tokens * _tok_bytes(cfg) + 7, pinned_bytes=4 << 20,
                       max_seq_len=512)
    ctx.load_head(hr["embed"], hr["gf"], hr["wlm"])
    P, D = pp_desc(cfg), tp_desc(cfg, 1, 0)
    if reshard:
        for l in range(cfg.n_layers):
            ctx.host_weights_put(l, raws[l])
    else:
        for d in (P, D):
            for l in range(cfg.n_layers):
                ctx.load_layer(d, l, raws[l])
    toks, trace, stats = ctx.offline_run(P, D, prompts, out_lens, mpt, mds, reshard_weights=reshard, stream=stream,
                                         swap_in_group=group)
    ref_trace, ref_stats = sc.simulate([len(p) for p in prompts], out_lens, tier_tokens, gpu_pages, mpt, mds, cfg.page_size,
                                       group)
    assert trace == ref_trace
    for key in ("prefill_batches", "decode_steps", "to_decode", "to_prefill", "tokens"):
        assert stats[key] == ref_stats[key], key
    assert ctx.host_tier_used_bytes() == 0                 # everything that went to the store came back
    assert ctx.kv_free_pages(D) == gpu_pages and ctx.kv_free_pages(P) == gpu_pages
    ctx.destroy()
    return vals, hv, toks, stats


def _requests(cfg, n, seed, p_lo, p_hi, o_lo, o_hi):
    rng = np.random.default_rng(seed)
    prompts = [rng.integers(0, cfg.vocab, size=int(rng.integers(p_lo, p_hi + 1))).astype(np.int32) for _ in range(n)]
    out_lens = [int(v) for v in rng.integers(o_lo, o_hi + 1, n)]
    return prompts, out_lens


@pytest.mark.parametrize("reshard", [True, False])
def test_loop_matches_the_oracles_on_config1_model(reshard):
    cfg = wl.config1().cfg
    prompts, out_lens = _requests(cfg, 14, 41, 3, 70, 1, 9)
    out_lens[3] = 1                                         # finishes at its prefill
    # a store of 150 tokens fills several times; 9 pages throttle admission; batches of at most 96 tokens
    vals, hv, toks, stats = _run(cfg, 1001, prompts, out_lens, tier_tokens=150, gpu_pages=9, mpt=96, mds=5, reshard=reshard)
    assert stats["to_decode"] >= 3 and stats["to_prefill"] >= 2
    compared = _check_tokens(cfg, vals, hv, prompts, out_lens, toks, 1e-4)
    assert compared >= 0.9 * sum(out_lens)


def test_loop_with_a_store_that_holds_everything_switches_once():
    cfg = wl.config1().cfg
    prompts, out_lens = _requests(cfg, 8, 42, 10, 40, 2, 6)
    compute = torch.cuda.Stream()
    torch.cuda.synchronize()
    vals, hv, toks, stats = _run(cfg, 1002, prompts, out_lens, tier_tokens=100000, gpu_pages=64, mpt=64, mds=64, reshard=True,
                                 stream=compute.cuda_stream, group=3)
    assert (stats["to_decode"], stats["to_prefill"]) == (1, 0)
    assert _check_tokens(cfg, vals, hv, prompts, out_lens, toks, 1e-4) >= 0.9 * sum(out_lens)


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F16])
def test_loop_16bit_model_trace_and_counts(dtype):
    # 16-bit storage, head_dim 128 (the MFMA kernels): the order of actions is what is compared; tokens of such
    # a run are not expected to equal those of the float64 oracle beyond the first few
    cfg = wl.ModelCfg(hidden=512, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn=1024, n_layers=2, vocab=256, dtype=dtype)
    prompts, out_lens = _requests(cfg, 10, 43, 5, 90, 2, 12)
    _run(cfg, 1003, prompts, out_lens, tier_tokens=200, gpu_pages=12, mpt=128, mds=4, reshard=True)
    _run(cfg, 1003, prompts, out_lens, tier_tokens=400, gpu_pages=24, mpt=128, mds=8, reshard=True, group=2)


def test_loop_argument_errors():
    cfg = wl.config1().cfg
    vals, raws, hv, hr = _model(cfg, 1004)
    ctx = make_context(cfg, pages=4, tier_bytes=64 * _tok_bytes(cfg), pinned_bytes=4 << 20, max_seq_len=512)
    ctx.load_head(hr["embed"], hr["gf"], hr["wlm"])
    for l in range(cfg.n_layers):
        ctx.host_weights_put(l, raws[l])
    P, D = pp_desc(cfg), tp_desc(cfg, 1, 0)
    one = [np.arange(10, dtype=np.int32)]
    with pytest.raises(ss.SeesawError) as e:                # prompt larger than the CPU store
        ctx.offline_run(P, D, [np.zeros(65, dtype=np.int32)], [4], 128, 4)
    assert e.value.code == ss.SS_ENOMEM
    with pytest.raises(ss.SeesawError) as e:                # final length needs 5 pages, the GPU store has 4
        ctx.offline_run(P, D, [np.zeros(60, dtype=np.int32)], [8], 128, 4)
    assert e.value.code == ss.SS_ENOMEM
    with pytest.raises(ss.SeesawError) as e:                # both strategies the same descriptor
        ctx.offline_run(P, P, one, [2], 128, 4)
    assert e.value.code == ss.SS_EINVAL
    with pytest.raises(ss.SeesawError) as e:                # a tensor-parallel shard needs its partners
        ctx.offline_run(P, tp_desc(cfg, 2, 0), one, [2], 128, 4)
    assert e.value.code == ss.SS_EINVAL
    with pytest.raises(ss.SeesawError) as e:
        ctx.offline_run(P, D, one, [0], 128, 4)
    assert e.value.code == ss.SS_EINVAL
    with pytest.raises(ss.SeesawError) as e:                # trace buffer too small
        ctx.offline_run(P, D, one, [3], 128, 4, trace_cap=4)
    assert e.value.code == ss.SS_ENOMEM
    toks, trace, stats = ctx.offline_run(P, D, one, [3], 128, 4)    # and the context is still usable
    assert stats["tokens"] == 3 and len(toks[0]) == 3
    toks, trace, stats = ctx.offline_run(P, D, [], [], 128, 4)      # nothing to do
    assert toks == [] and trace == [] and stats["tokens"] == 0
    ctx.destroy()
