"""GPU parity of weight re-sharding (reload of the new strategy's shards from the
CPU copy of the model) against the CPU oracle, through the C ABI.

Data movement: what a shard holds after the switch is compared bit for bit with
the oracle's slices of the same seeded weights; layer outputs computed with the
re-sharded weights are compared bit for bit with those of a shard loaded
directly, and with the layer oracle within the floating-point tolerance.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import layer_math as lm
from oracle import weight_shard as ows

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2503_06433_amd as ss
    from paper_2503_06433_amd.binding import W_NAMES
    from paper_2503_06433_amd.harness import (make_context, to_device, to_f64, to_raw, empty_like_acts, rel_err, tol,
                                              pp_desc, tp_desc, stored_form)

SHAPES = {
    "mha_d128": dict(hidden=512, n_q_heads=4, n_kv_heads=4, head_dim=128, ffn=1024),      # gate/up interleaved layout
    "gqa4_d128": dict(hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=1536),
    "mha_d64_ragged": dict(hidden=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn=688),  # ffn/k not a multiple of 32
}


def _model(cfg, seed):
    vals, raws = [], []
    for l in range(cfg.n_layers):
        v, r = wl.make_layer_weights(cfg, seed + l)
        vals.append(v)
        raws.append(r)
    return vals, raws


def _check_shard(ctx, cfg, raws, desc, k, i):
    """Every tensor the shard holds == the oracle's slice of the raw storage bits (the matrices behind a norm
    with that norm's gains folded into their rows, see harness.stored_form)."""
    for l in range(desc.layer_begin, desc.layer_end):
        ref = stored_form(ows.shard_weights(cfg, raws[l], k, i), cfg.dtype)
        for which, name in enumerate(W_NAMES):
            got = ctx.weights_read(desc, l, which, ref[name].size)
            assert np.array_equal(got, ref[name].reshape(-1)), (l, name)


@pytest.mark.parametrize("name,dtype,k", [
    ("mha_d128", wl.BF16, 2), ("mha_d128", wl.BF16, 4), ("gqa4_d128", wl.BF16, 2), ("mha_d64_ragged", wl.BF16, 2),
    ("mha_d64_ragged", wl.F32, 2), ("mha_d128", wl.F32, 1), ("mha_d128", wl.F16, 2),
])
def test_resharded_slices_are_bit_exact(name, dtype, k):
    cfg = wl.ModelCfg(n_layers=3, dtype=dtype, **SHAPES[name])
    _, raws = _model(cfg, 500)
    ctx = make_context(cfg, pages=8)
    for l in range(cfg.n_layers):
        ctx.host_weights_put(l, raws[l])
    es = 4 if dtype == wl.F32 else 2
    stage = pp_desc(cfg, 1, 3)                          # a pipeline stage: whole layers 1 and 2
    ctx.reshard_weights(None, stage)
    assert ctx.weights_shard_bytes(stage) == ows.reload_elems(cfg, 1, 1, 3) * es
    _check_shard(ctx, cfg, raws, stage, 1, 0)
    for i in range(k):                                  # the switch to the decode strategy: every shard in turn
        shard = tp_desc(cfg, k, i)
        ctx.reshard_weights(stage if i == 0 else None, shard)
        assert ctx.weights_shard_bytes(shard) == ows.reload_elems(cfg, k, 0, cfg.n_layers) * es
        _check_shard(ctx, cfg, raws, shard, k, i)
    # the stage's weights are gone, its layer calls say so
    x = empty_like_acts(4, cfg.hidden, dtype)
    with pytest.raises(ss.SeesawError) as e:
        ctx.layer_prefill(stage, 1, ss.SS_BOTH, [0], [4], [0], x, torch.empty_like(x))
    assert e.value.code == ss.SS_EINVAL
    with pytest.raises(ss.SeesawError) as e:
        ctx.weights_read(stage, 1, 1, 1)
    assert e.value.code == ss.SS_ENOENT
    ctx.sync()
    # ... and back (the next prefill phase): reloaded, identical
    ctx.reshard_weights(tp_desc(cfg, k, 0), stage)
    _check_shard(ctx, cfg, raws, stage, 1, 0)
    ctx.destroy()


@pytest.mark.parametrize("name,dtype,k", [("mha_d128", wl.BF16, 2), ("gqa4_d128", wl.BF16, 2), ("mha_d64_ragged", wl.F32, 2),
                                          ("gqa4_d128", wl.F16, 2)])
def test_layer_after_reshard_equals_direct_load_and_oracle(name, dtype, k):
    cfg = wl.ModelCfg(n_layers=2, dtype=dtype, **SHAPES[name])
    vals, raws = _model(cfg, 600)
    lens = [5, 33, 130]
    T = sum(lens)
    xv, xr = wl.make_activations((T, cfg.hidden), 8, dtype)
    x = to_device(xr, dtype)
    ids, zeros = [0, 1, 2], [0, 0, 0]
    batch = [(s, n, 0) for s, n in zip(ids, lens)]
    compute = torch.cuda.Stream()
    torch.cuda.synchronize()

    # context A: shards loaded directly
    direct = []
    ctx = make_context(cfg, pages=64)
    for i in range(k):
        d = tp_desc(cfg, k, i)
        for l in range(cfg.n_layers):
            ctx.load_layer(d, l, raws[l])
        outs = []
        for l in range(cfg.n_layers):
            y = empty_like_acts(T, cfg.hidden, dtype)
            ctx.layer_prefill(d, l, ss.SS_ATTN, ids, lens, zeros, x, y)
            z = empty_like_acts(T, cfg.hidden, dtype)
            ctx.layer_prefill(d, l, ss.SS_MLP, ids, lens, zeros, x, z)
            outs.append((y, z))
        torch.cuda.synchronize()
        direct.append([(to_raw(y, dtype).copy(), to_raw(z, dtype).copy()) for y, z in outs])
    ctx.destroy()

    # context B: a pipeline stage runs first, then the switch; the layer calls on the new shard are issued
    # right behind the re-shard request, on a stream of their own, without waiting on the host
    ctx = make_context(cfg, pages=64)
    for l in range(cfg.n_layers):
        ctx.host_weights_put(l, raws[l])
    stage = pp_desc(cfg)
    ctx.reshard_weights(None, stage, compute.cuda_stream)
    y_pp = empty_like_acts(T, cfg.hidden, dtype)
    ctx.layer_prefill(stage, 0, ss.SS_BOTH, ids, lens, zeros, x, y_pp, compute.cuda_stream)
    for i in range(k):
        d = tp_desc(cfg, k, i)
        ctx.reshard_weights(stage if i == 0 else None, d, compute.cuda_stream)
        outs = []
        for l in range(cfg.n_layers):
            y = empty_like_acts(T, cfg.hidden, dtype)
            ctx.layer_prefill(d, l, ss.SS_ATTN, ids, lens, zeros, x, y, compute.cuda_stream)
            z = empty_like_acts(T, cfg.hidden, dtype)
            ctx.layer_prefill(d, l, ss.SS_MLP, ids, lens, zeros, x, z, compute.cuda_stream)
            outs.append((y, z))
        torch.cuda.synchronize()
        ctx.sync()
        for l, (y, z) in enumerate(outs):
            assert np.array_equal(to_raw(y, dtype), direct[i][l][0]), (i, l, "attention half")
            assert np.array_equal(to_raw(z, dtype), direct[i][l][1]), (i, l, "mlp half")
            rk = None if dtype == wl.F32 else (lambda a: wl.round_to_storage(a, dtype))
            ref_a = lm.attn_block(cfg, vals[l], xv, batch, lm.KVCache(cfg), l, k, i, rk)
            ref_m = lm.mlp_block(cfg, vals[l], xv, k, i)
            assert rel_err(to_f64(y, dtype), ref_a) <= tol(dtype)
            assert rel_err(to_f64(z, dtype), ref_m) <= tol(dtype)
    # the stage's output was computed before its weights were released
    cache = lm.KVCache(cfg)
    _, ref = lm.layer_forward(cfg, vals[0], xv, batch, cache, 0, 1,
                              None if dtype == wl.F32 else (lambda a: wl.round_to_storage(a, dtype)))
    assert rel_err(to_f64(y_pp, dtype), ref) <= tol(dtype)
    ctx.destroy()


def test_reshard_error_paths():
    cfg = wl.ModelCfg(n_layers=2, dtype=wl.BF16, **SHAPES["mha_d128"])
    _, raws = _model(cfg, 700)
    ctx = make_context(cfg, pages=8)
    with pytest.raises(ss.SeesawError) as e:            # nothing in the CPU copy yet
        ctx.reshard_weights(None, pp_desc(cfg))
    assert e.value.code == ss.SS_ENOENT
    ctx.host_weights_put(0, raws[0])
    with pytest.raises(ss.SeesawError) as e:            # layer 1 still missing
        ctx.reshard_weights(None, pp_desc(cfg))
    assert e.value.code == ss.SS_ENOENT
    ctx.reshard_weights(None, pp_desc(cfg, 0, 1))       # layer 0 alone is fine
    with pytest.raises(ss.SeesawError) as e:
        ctx.host_weights_put(2, raws[0])                # no such layer
    assert e.value.code == ss.SS_EINVAL
    with pytest.raises(ss.SeesawError) as e:            # k does not divide the heads
        ctx.reshard_weights(None, ss.ShardDesc(ss.SS_TP, 3, 0, 0, 1))
    assert e.value.code == ss.SS_EINVAL
    ctx.destroy()


def test_mixed_layout_weight_shares_bit_exact():
    """A device's share under a mixed strategy is a tensor-parallel shard of a run of layers: re-sharding
    from a (2 shards x 2 stages) share to a (4 shards, all layers) share and on to a (4 x 2) share."""
    cfg = wl.ModelCfg(n_layers=4, dtype=wl.BF16, **SHAPES["mha_d128"])
    _, raws = _model(cfg, 800)
    ctx = make_context(cfg, pages=8)
    for l in range(cfg.n_layers):
        ctx.host_weights_put(l, raws[l])
    a = tp_desc(cfg, 2, 1, 2, 4)                # shard 1 of 2, second stage
    b = tp_desc(cfg, 4, 3)                      # shard 3 of 4, all layers
    c = tp_desc(cfg, 4, 0, 0, 2)                # shard 0 of 4, first stage
    ctx.reshard_weights(None, a)
    _check_shard(ctx, cfg, raws, a, 2, 1)
    ctx.reshard_weights(a, b)
    _check_shard(ctx, cfg, raws, b, 4, 3)
    ctx.reshard_weights(b, c)
    _check_shard(ctx, cfg, raws, c, 4, 0)
    assert ctx.weights_shard_bytes(c) * 2 == ctx.weights_shard_bytes(b)
    ctx.destroy()
