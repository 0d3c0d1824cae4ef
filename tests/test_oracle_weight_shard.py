"""Pins for the weight re-sharding oracle (CPU only).

The paper states what re-sharding must achieve (every device ends up with the
part of the weights its new strategy needs, reloaded from the CPU copy; section
4.1) and what a tensor-parallel device holds only through its cost model (1/k
of every matrix, partial results summed; Appendix A.3).  The pins are therefore
properties: the shards partition every matrix exactly once, computing with the
slices and summing reproduces the unsharded products, the element counts are
the paper's W / k, and the slicing agrees with the one the layer oracle uses.
"""
import numpy as np
import pytest

import workloads as wl
from oracle import layer_math as lm
from oracle import weight_shard as ws


def cfg_of(n_q=8, n_kv=4, d=4, hidden=12, ffn=16, n_layers=4):
    return wl.ModelCfg(hidden=hidden, n_q_heads=n_q, n_kv_heads=n_kv, head_dim=d, ffn=ffn, n_layers=n_layers,
                       vocab=16, dtype=wl.F32)


def labelled_weights(cfg):
    """Every element is a distinct integer that encodes (matrix, row, column)."""
    shapes = {"wq": (cfg.hidden, cfg.q_dim), "wk": (cfg.hidden, cfg.kv_dim), "wv": (cfg.hidden, cfg.kv_dim),
              "wo": (cfg.q_dim, cfg.hidden), "wg": (cfg.hidden, cfg.ffn), "wu": (cfg.hidden, cfg.ffn),
              "wd": (cfg.ffn, cfg.hidden)}
    w = {}
    for mi, (name, (r, c)) in enumerate(shapes.items()):
        w[name] = (mi * 1_000_000 + np.arange(r * c).reshape(r, c)).astype(np.int64)
    w["g1"] = np.arange(cfg.hidden, dtype=np.int64) + 7_000_000
    w["g2"] = np.arange(cfg.hidden, dtype=np.int64) + 8_000_000
    return w


@pytest.mark.parametrize("k", [1, 2, 4])
def test_shards_partition_every_matrix_exactly_once(k):
    cfg = cfg_of()
    w = labelled_weights(cfg)
    shards = [ws.shard_weights(cfg, w, k, i) for i in range(k)]
    d = cfg.head_dim
    # brute force, element by element: which shard holds (r, c) and where
    for name in ws.MATRICES:
        full = w[name]
        seen = np.zeros(full.shape, dtype=np.int64)
        for i, sh in enumerate(shards):
            part = sh[name]
            for r in range(part.shape[0]):
                for c in range(part.shape[1]):
                    if name in ("wq",):
                        fr, fc = r, i * (cfg.n_q_heads // k) * d + c
                    elif name in ("wk", "wv"):
                        fr, fc = r, i * (cfg.n_kv_heads // k) * d + c
                    elif name == "wo":
                        fr, fc = i * (cfg.n_q_heads // k) * d + r, c
                    elif name in ("wg", "wu"):
                        fr, fc = r, i * (cfg.ffn // k) + c
                    else:
                        fr, fc = i * (cfg.ffn // k) + r, c
                    assert part[r, c] == full[fr, fc]
                    seen[fr, fc] += 1
        assert np.all(seen == 1), name
    for sh in shards:                                   # gains are replicated
        assert np.array_equal(sh["g1"], w["g1"]) and np.array_equal(sh["g2"], w["g2"])


def test_concatenating_the_shards_gives_back_the_matrices():
    cfg = cfg_of()
    w = wl.make_layer_weights(cfg, 11, std=0.5)[0]
    k = 4
    sh = [ws.shard_weights(cfg, w, k, i) for i in range(k)]
    for name in ("wq", "wk", "wv", "wg", "wu"):
        assert np.array_equal(np.concatenate([s[name] for s in sh], axis=1), w[name])
    for name in ("wo", "wd"):
        assert np.array_equal(np.concatenate([s[name] for s in sh], axis=0), w[name])


@pytest.mark.parametrize("k", [2, 4])
def test_products_with_the_slices_sum_to_the_unsharded_products(k):
    # column-parallel first matrix, row-parallel second matrix: sum_i f(h W1_i) W2_i = f(h W1) W2 for an
    # elementwise f; a slice taken along the wrong axis or with mismatched ranges breaks the identity.
    cfg = cfg_of()
    w = wl.make_layer_weights(cfg, 12, std=0.5)[0]
    rng = np.random.default_rng(3)
    h = rng.standard_normal((5, cfg.hidden))
    full = (np.tanh(h @ w["wg"]) * (h @ w["wu"])) @ w["wd"]
    part = sum((np.tanh(h @ s["wg"]) * (h @ s["wu"])) @ s["wd"] for s in (ws.shard_weights(cfg, w, k, i) for i in range(k)))
    assert np.allclose(part, full, rtol=1e-12, atol=1e-12)
    a = rng.standard_normal((5, cfg.q_dim))                 # any per-head attention output
    d = cfg.head_dim
    part = 0.0
    for i in range(k):
        s = ws.shard_weights(cfg, w, k, i)
        (q0, q1), (g0, g1), _ = ws.head_and_ffn_ranges(cfg, k, i)
        assert np.array_equal(h @ s["wq"], (h @ w["wq"])[:, q0 * d:q1 * d])
        assert np.array_equal(h @ s["wk"], (h @ w["wk"])[:, g0 * d:g1 * d])
        assert np.array_equal(h @ s["wv"], (h @ w["wv"])[:, g0 * d:g1 * d])
        part = part + a[:, q0 * d:q1 * d] @ s["wo"]
    assert np.allclose(part, a @ w["wo"], rtol=1e-12, atol=1e-12)


def test_query_heads_stay_with_their_kv_head():
    # grouped-query attention: query head j reads kv head j // (n_q / n_kv); a shard must hold both
    cfg = cfg_of(n_q=8, n_kv=2)
    for k in (1, 2):
        for i in range(k):
            (q0, q1), (g0, g1), _ = ws.head_and_ffn_ranges(cfg, k, i)
            for j in range(q0, q1):
                assert g0 <= j // (cfg.n_q_heads // cfg.n_kv_heads) < g1


@pytest.mark.parametrize("k", [1, 2, 4])
def test_element_counts_are_the_model_size_over_k(k):
    cfg = cfg_of()
    assert ws.shard_matrix_elems(cfg, k) * k == cfg.layer_params()
    w = labelled_weights(cfg)
    held = sum(ws.shard_weights(cfg, w, k, 0)[n].size for n in ws.MATRICES)
    assert held == ws.shard_matrix_elems(cfg, k)
    # a pipeline slice of L/k whole layers and a tensor shard of all L layers hold the same number of matrix
    # elements: the switch replaces one k-th of the model by another
    L = cfg.n_layers
    if L % k == 0:
        pp = ws.reload_elems(cfg, 1, 0, L // k) - 2 * cfg.hidden * (L // k)
        tp = ws.reload_elems(cfg, k, 0, L) - 2 * cfg.hidden * L
        assert pp == tp == L * cfg.layer_params() // k


def test_slicing_agrees_with_the_layer_oracle():
    # the layer oracle run on the full weights with (k, i) must equal the layer oracle run unsharded on a
    # model that consists of the shard's slices only
    cfg = cfg_of(n_q=4, n_kv=2, d=8, hidden=16, ffn=24, n_layers=1)
    w = wl.make_layer_weights(cfg, 13, std=0.3)[0]
    rng = np.random.default_rng(5)
    x = rng.standard_normal((6, cfg.hidden))
    batch = [(0, 4, 0), (1, 2, 0)]
    k = 2
    small = wl.ModelCfg(hidden=cfg.hidden, n_q_heads=cfg.n_q_heads // k, n_kv_heads=cfg.n_kv_heads // k,
                        head_dim=cfg.head_dim, ffn=cfg.ffn // k, n_layers=1, vocab=16, dtype=wl.F32)
    for i in range(k):
        sw = ws.shard_weights(cfg, w, k, i)
        a_full = lm.attn_block(cfg, w, x, batch, lm.KVCache(cfg), 0, k, i)
        a_small = lm.attn_block(small, sw, x, batch, lm.KVCache(small), 0, 1, 0)
        assert np.array_equal(a_full, a_small)
        assert np.array_equal(lm.mlp_block(cfg, w, x, k, i), lm.mlp_block(small, sw, x, 1, 0))


def test_reshard_depends_only_on_the_cpu_copy_and_the_target():
    cfg = cfg_of()
    model = [wl.make_layer_weights(cfg, 20 + l, std=0.5)[0] for l in range(cfg.n_layers)]
    held = ws.reshard(cfg, model, 2, 1, 0, cfg.n_layers)
    assert sorted(held) == list(range(cfg.n_layers))
    for l in held:
        ref = ws.shard_weights(cfg, model[l], 2, 1)
        assert all(np.array_equal(held[l][n], ref[n]) for n in ws.MATRICES + ws.GAINS)
    stage = ws.reshard(cfg, model, 1, 0, 2, 4)             # a pipeline stage: whole layers 2 and 3
    assert sorted(stage) == [2, 3]
    assert all(np.array_equal(stage[3][n], model[3][n]) for n in ws.MATRICES)


def test_bad_shard_arguments():
    cfg = cfg_of()
    with pytest.raises(ValueError):
        ws.head_and_ffn_ranges(cfg, 3, 0)
    with pytest.raises(ValueError):
        ws.head_and_ffn_ranges(cfg, 2, 2)


def _golden(name):
    import os
    out = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#") and "=" in line:
                k, v = (x.strip() for x in line.split("=", 1))
                out[k] = v
    return out


def test_weight_count_of_the_70b_model_matches_the_size_the_paper_prints():
    """Section 3.3 prints the one absolute model size of the paper: the 70B model's float16 weights take 140 GiB and
    need at least four 40 GiB GPUs.  The oracle's element count of a layer (the paper's W, which every cost term of
    Appendix A and every re-shard volume here is built on) times the layers, plus the two vocabulary matrices, must
    give that size; a dropped or doubled matrix in the count moves it by 8 % or more."""
    g = _golden("section3_3_model_weight_bytes.txt")
    cfg = wl.ModelCfg(hidden=int(g["hidden"]), n_q_heads=int(g["n_q_heads"]), n_kv_heads=int(g["n_kv_heads"]),
                      head_dim=int(g["head_dim"]), ffn=int(g["ffn"]), n_layers=int(g["n_layers"]), vocab=int(g["vocab"]),
                      dtype=wl.F16)
    per_layer = ws.shard_matrix_elems(cfg, 1) + 2 * cfg.hidden
    # the count agrees with the shapes the layer oracle multiplies with
    assert per_layer == sum(int(np.prod(s)) for s in wl.layer_weight_shapes(cfg).values())
    total = (per_layer * cfg.n_layers + 2 * cfg.vocab * cfg.hidden + cfg.hidden) * int(g["bytes_per_element"])
    printed, tol = float(g["printed_weight_bytes"]), float(g["relative_tolerance"])
    assert abs(total - printed) <= tol * printed, (total, printed)
    # "at least four GPUs (160 GiB) are needed to fit the model weights"
    gib40 = 40 * 2 ** 30
    assert -(-total // gib40) == int(g["min_gpus_of_40GiB"])
    # and a tensor-parallel shard holds W / k of the matrices (Appendix A.3)
    for k in (2, 4, 8):
        assert ws.shard_matrix_elems(cfg, k) * k == ws.shard_matrix_elems(cfg, 1)
