"""GPU parity of the KV-cache movement (repack, swap, re-shard, paging) against
the CPU oracle's index formulas, through the C ABI.  Everything here is data
movement: comparisons are bit for bit.  Cache contents are seeded random bit
patterns, never values produced by the layer kernels.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import kv_tier as kt

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2503_06433_amd as ss
    from paper_2503_06433_amd.harness import make_context, to_device, to_raw, pp_desc, tp_desc


def _cfg(dtype, d=128, n_kv=4, n_layers=3):
    return wl.ModelCfg(hidden=256, n_q_heads=n_kv * 2, n_kv_heads=n_kv, head_dim=d, ffn=512,
                       n_layers=n_layers, dtype=dtype)


def _rand_bits(shape, seed, dtype):
    rng = np.random.default_rng(seed)
    if dtype == wl.F32:
        # finite float32 bit patterns
        return rng.standard_normal(shape, dtype=np.float32)
    return wl.bf16_bits(rng.standard_normal(shape, dtype=np.float32))


def _import(ctx, desc, cfg, ids, contents):
    flat = np.concatenate([c.reshape(-1) for c in contents])
    lens = [c.shape[3] for c in contents]
    ctx.kv_import_dev(desc, ids, lens, to_device(flat, cfg.dtype))
    torch.cuda.synchronize()


@pytest.mark.parametrize("dtype,d", [(wl.BF16, 128), (wl.BF16, 64), (wl.F32, 64), (wl.F32, 128), (wl.F16, 128)])
def test_import_read_export_round_trip(dtype, d):
    cfg = _cfg(dtype, d=d)
    desc = pp_desc(cfg)
    ctx = make_context(cfg, pages=64)
    lens = [1, 15, 16, 17, 300]
    ids = [100 + i for i in range(len(lens))]
    contents = [_rand_bits((cfg.n_layers, 2, cfg.n_kv_heads, n, d), 10 + i, dtype) for i, n in enumerate(lens)]
    _import(ctx, desc, cfg, ids, contents)
    store = kt.PagedStore(64, cfg.n_layers, cfg.n_kv_heads, d, contents[0].dtype)
    for sid, c in zip(ids, contents):
        store.write(sid, c)
    for sid, c in zip(ids, contents):
        assert list(ctx.kv_page_table(desc, sid)) == store.alloc.tables[sid]
        assert ctx.kv_seq_len(desc, sid) == c.shape[3]
        for l in range(cfg.n_layers):
            assert np.array_equal(ctx.kv_read(desc, sid, l, cfg.n_kv_heads), store.read(sid)[l])
    # export of a subset, in a different order, in the documented staging layout
    order = [4, 1, 3]
    off = kt.staging_offsets([lens[i] for i in order], cfg.n_layers, cfg.n_kv_heads, d)
    stg = torch.zeros(int(off[-1]), device="cuda", dtype=torch.float32 if dtype == wl.F32 else torch.int16)
    ctx.kv_export_dev(desc, [ids[i] for i in order], stg)
    torch.cuda.synchronize()
    raw = to_raw(stg, dtype)
    for j, i in enumerate(order):
        assert np.array_equal(raw[off[j]:off[j + 1]].reshape(contents[i].shape), contents[i])
    assert ctx.kv_free_pages(desc) == len(store.alloc.free)
    ctx.destroy()


def test_page_policy_matches_oracle_through_growth_and_free():
    cfg = _cfg(wl.BF16, n_layers=1)
    desc = pp_desc(cfg)
    ctx = make_context(cfg, pages=12)
    alloc = kt.PageAllocator(12)
    mk = lambda n, s: _rand_bits((1, 2, cfg.n_kv_heads, n, 128), s, wl.BF16)
    _import(ctx, desc, cfg, [1, 2, 3], [mk(20, 1), mk(40, 2), mk(5, 3)])
    for sid, n in ((1, 20), (2, 40), (3, 5)):
        alloc.ensure(sid, n)
    ctx.kv_free(desc, [2])
    alloc.release(2)
    _import(ctx, desc, cfg, [4], [mk(70, 4)])
    alloc.ensure(4, 70)
    for sid in (1, 3, 4):
        assert list(ctx.kv_page_table(desc, sid)) == alloc.tables[sid]
    assert ctx.kv_free_pages(desc) == len(alloc.free)
    free_before = ctx.kv_free_pages(desc)
    with pytest.raises(ss.SeesawError) as e:
        _import(ctx, desc, cfg, [5], [mk(16 * 6, 5)])
    assert e.value.code == ss.SS_ENOMEM
    # a refused import leaves nothing behind: no pages taken, the sequence unknown, the others untouched
    assert ctx.kv_free_pages(desc) == free_before
    with pytest.raises(ss.SeesawError) as e:
        ctx.kv_seq_len(desc, 5)
    assert e.value.code == ss.SS_ENOENT
    # ... also when an earlier sequence of the same call would have fitted alone
    with pytest.raises(ss.SeesawError) as e:
        _import(ctx, desc, cfg, [6, 5], [mk(16, 6), mk(16 * 6, 5)])
    assert e.value.code == ss.SS_ENOMEM
    assert ctx.kv_free_pages(desc) == free_before
    for sid in (5, 6):
        with pytest.raises(ss.SeesawError) as e:
            ctx.kv_seq_len(desc, sid)
        assert e.value.code == ss.SS_ENOENT
    # once pages are free again the same call goes through, with the pages the policy gives
    ctx.kv_free(desc, [4])
    alloc.release(4)
    c6, c5 = mk(16, 6), mk(16 * 6, 5)
    _import(ctx, desc, cfg, [6, 5], [c6, c5])
    alloc.ensure(6, 16)
    alloc.ensure(5, 96)
    for sid, cont in ((6, c6), (5, c5)):
        assert list(ctx.kv_page_table(desc, sid)) == alloc.tables[sid]
        assert np.array_equal(ctx.kv_read(desc, sid, 0, cfg.n_kv_heads), cont[0])
    with pytest.raises(ss.SeesawError) as e:
        ctx.kv_free(desc, [99])
    assert e.value.code == ss.SS_ENOENT
    ctx.destroy()


def test_swap_in_that_does_not_fit_is_all_or_nothing():
    """A swap-in whose sequences do not all fit the shard's pool is refused as a whole: no pages are taken, no
    sequence becomes resident, and the same call succeeds once pages have been freed."""
    cfg = _cfg(wl.BF16, n_layers=2)
    L, n_kv, d = 2, cfg.n_kv_heads, 128
    lens = {1: 40, 2: 100, 3: 30}                       # 3 + 7 + 2 pages
    complete = {s: _rand_bits((L, 2, n_kv, n, d), 50 + s, wl.BF16) for s, n in lens.items()}
    ctx = make_context(cfg, pages=14, tier_bytes=8 << 20, pinned_bytes=4 << 20)
    src, dst = pp_desc(cfg), tp_desc(cfg, 2, 1)
    ids = list(lens)
    _import(ctx, src, cfg, ids, [complete[s] for s in ids])
    ctx.kv_swap(src, ss.SS_OUT, ids)
    ctx.sync()
    blocker = _rand_bits((L, 2, n_kv // 2, 16 * 4, d), 60, wl.BF16)     # 4 of the 14 pages of the target pool
    _import(ctx, dst, cfg, [900], [blocker])
    assert ctx.kv_free_pages(dst) == 10
    with pytest.raises(ss.SeesawError) as e:
        ctx.kv_swap(dst, ss.SS_IN, ids)                 # needs 12
    assert e.value.code == ss.SS_ENOMEM
    ctx.sync()
    assert ctx.kv_free_pages(dst) == 10
    for s in ids:
        with pytest.raises(ss.SeesawError) as e:
            ctx.kv_seq_len(dst, s)
        assert e.value.code == ss.SS_ENOENT
    with pytest.raises(ss.SeesawError) as e:
        ctx.kv_swap(dst, ss.SS_IN, [1, 1])              # listed twice
    assert e.value.code == ss.SS_EINVAL
    ctx.kv_free(dst, [900])
    ctx.kv_swap(dst, ss.SS_IN, ids)
    ctx.sync()
    alloc = kt.PageAllocator(14)
    for s in ids:
        alloc.ensure(s, lens[s])
    for s in ids:
        assert list(ctx.kv_page_table(dst, s)) == alloc.tables[s]
        for l in range(L):
            assert np.array_equal(ctx.kv_read(dst, s, l, n_kv // 2), complete[s][l][:, n_kv // 2:])
    ctx.destroy()


@pytest.mark.parametrize("dtype,pinned_kib", [(wl.BF16, 8192), (wl.BF16, 1280), (wl.F32, 1280)])
def test_reshard_pp_stages_to_tp_shards_bit_exact(dtype, pinned_kib):
    """Two pipeline stages push their layer slices into the host tier; the tier then holds the complete
    cache at the closed-form offsets; every tensor-parallel shard pulls its heads.  A small pinned ring
    forces the two-slot pipeline through many chunks."""
    d, n_kv, L = (128, 4, 4) if dtype == wl.BF16 else (64, 4, 4)
    cfg = _cfg(dtype, d=d, n_kv=n_kv, n_layers=L)
    es = 2 if dtype == wl.BF16 else 4
    lens = {7: 33, 8: 16, 9: 1, 12: 150}
    complete = {s: _rand_bits((L, 2, n_kv, n, d), 20 + s, dtype) for s, n in lens.items()}
    tier_bytes = sum(kt.tier_seq_elems(L, n_kv, d, n) for n in lens.values()) * es
    ctx = make_context(cfg, pages=32, tier_bytes=tier_bytes, pinned_bytes=pinned_kib * 1024)
    ids = list(lens)
    stages = [pp_desc(cfg, 0, 2), pp_desc(cfg, 2, 4)]
    for j, st in enumerate(stages):
        _import(ctx, st, cfg, ids, [complete[s][2 * j:2 * j + 2] for s in ids])
    for st in stages:
        ctx.kv_swap(st, ss.SS_OUT, ids)
    ctx.sync()
    # the tier image, by the oracle's index formula
    tier = np.zeros(tier_bytes // es, dtype=complete[7].dtype)
    talloc = kt.TierAllocator(tier.size)
    for s in ids:
        base = talloc.place(s, kt.tier_seq_elems(L, n_kv, d, lens[s]))
        for j in range(2):
            kt.tier_put(tier, base, complete[s][2 * j:2 * j + 2], n_kv, (2 * j, 2 * j + 2), (0, n_kv))
    assert ctx.host_tier_used_bytes() == talloc.used * es
    for s in ids:
        base = talloc.base[s][0]
        per_layer = 2 * n_kv * lens[s] * d
        for l in range(L):
            got = ctx.host_tier_read(s, l, lens[s])
            assert np.array_equal(got.reshape(-1), tier[base + l * per_layer: base + (l + 1) * per_layer])
    # tier full: one more sequence does not fit
    extra = _rand_bits((2, 2, n_kv, 40, d), 99, dtype)
    _import(ctx, stages[0], cfg, [500], [extra])
    with pytest.raises(ss.SeesawError) as e:
        ctx.kv_swap(stages[0], ss.SS_OUT, [500])
    assert e.value.code == ss.SS_ENOMEM
    # swap-in under the decode layout: k = 2 and k = 4 shards, all layers
    for k in (2, 4):
        nh = n_kv // k
        for i in range(k):
            td = tp_desc(cfg, k, i)
            order = ids[::-1]
            ctx.kv_swap(td, ss.SS_IN, order)
            ctx.sync()
            alloc = kt.PageAllocator(32)
            for s in order:
                alloc.ensure(s, lens[s])
            for s in ids:
                assert list(ctx.kv_page_table(td, s)) == alloc.tables[s]
                want = kt.tier_get(tier, talloc.base[s][0], lens[s], n_kv, d, (0, L), (i * nh, (i + 1) * nh))
                for l in range(L):
                    assert np.array_equal(ctx.kv_read(td, s, l, nh), want[l])
                    assert np.array_equal(want[l], complete[s][l][:, i * nh:(i + 1) * nh])
    with pytest.raises(ss.SeesawError) as e:
        ctx.kv_swap(tp_desc(cfg, 2, 0), ss.SS_IN, [7])          # already resident
    assert e.value.code == ss.SS_EINVAL
    with pytest.raises(ss.SeesawError) as e:
        ctx.kv_swap(tp_desc(cfg, 2, 1), ss.SS_IN, [4242])       # not in the tier
    assert e.value.code == ss.SS_ENOENT
    # drain: releasing every sequence empties the tier and restarts allocation at 0
    ctx.host_tier_release(ids)
    assert ctx.host_tier_used_bytes() == 0
    ctx.destroy()


def test_kv_reshard_single_call_and_pp_round_trip():
    cfg = _cfg(wl.BF16, n_layers=2)
    L, n_kv, d = 2, cfg.n_kv_heads, 128
    lens = {1: 47, 2: 260}
    complete = {s: _rand_bits((L, 2, n_kv, n, d), 30 + s, wl.BF16) for s, n in lens.items()}
    ctx = make_context(cfg, pages=40, tier_bytes=8 << 20, pinned_bytes=4 << 20)
    src = pp_desc(cfg)
    ids = list(lens)
    _import(ctx, src, cfg, ids, [complete[s] for s in ids])
    dst = tp_desc(cfg, 4, 3)
    ctx.kv_reshard(src, dst, ids)
    ctx.sync()
    for s in ids:
        for l in range(L):
            assert np.array_equal(ctx.kv_read(dst, s, l, 1), complete[s][l][:, 3:4])
    # PP -> tier -> PP is the identity: free the pages, pull the full shard back
    ctx.kv_free(src, ids)
    assert ctx.kv_free_pages(src) == 40
    ctx.kv_swap(src, ss.SS_IN, ids)
    ctx.sync()
    for s in ids:
        for l in range(L):
            assert np.array_equal(ctx.kv_read(src, s, l, n_kv), complete[s][l])
    ctx.destroy()


def test_mixed_layout_tp2pp2_to_tp4_shares_bit_exact():
    """Mixed strategies (the paper's TP2PP2 -> TP4 style of switch, section 6.2): a device's share is a
    tensor-parallel shard of a run of layers.  Four devices of the prefill layout (2 stages x 2 shards) push
    their layers x heads blocks into the tier, where they form the complete cache; the devices of the decode
    layout (4 shards, all layers) and of a second mixed layout (2 stages x 4 shards) pull theirs."""
    dtype, d, n_kv, L = wl.BF16, 128, 4, 4
    cfg = _cfg(dtype, d=d, n_kv=n_kv, n_layers=L)
    lens = {3: 40, 5: 17, 6: 130}
    ids = list(lens)
    complete = {s: _rand_bits((L, 2, n_kv, n, d), 70 + s, dtype) for s, n in lens.items()}
    tier_bytes = sum(kt.tier_seq_elems(L, n_kv, d, n) for n in lens.values()) * 2
    ctx = make_context(cfg, pages=32, tier_bytes=tier_bytes, pinned_bytes=2 << 20)
    for stage in range(2):
        for shard in range(2):
            desc = tp_desc(cfg, 2, shard, 2 * stage, 2 * stage + 2)
            _import(ctx, desc, cfg, ids, [complete[s][2 * stage:2 * stage + 2, :, 2 * shard:2 * shard + 2] for s in ids])
            ctx.kv_swap(desc, ss.SS_OUT, ids)
    ctx.sync()
    for s in ids:                                            # the tier holds the complete cache, layer by layer
        for l in range(L):
            assert np.array_equal(ctx.host_tier_read(s, l, lens[s]).reshape(2, n_kv, lens[s], d), complete[s][l])
    targets = [(4, i, 0, L) for i in range(4)] + [(4, i, 2 * st, 2 * st + 2) for st in range(2) for i in range(4)]
    for k, i, lb, le in targets:
        desc = tp_desc(cfg, k, i, lb, le)
        ctx.kv_swap(desc, ss.SS_IN, ids)
        ctx.sync()
        nh = n_kv // k
        for s in ids:
            for l in range(lb, le):
                assert np.array_equal(ctx.kv_read(desc, s, l, nh), complete[s][l][:, i * nh:(i + 1) * nh])
    ctx.host_tier_release(ids)
    assert ctx.host_tier_used_bytes() == 0
    ctx.destroy()
