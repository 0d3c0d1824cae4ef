"""Pins for the CPU oracle: closed forms, invariants, brute force, and library
routines it must reduce to.  None of the expected values here comes from the
oracle itself or from the HIP path.  (CPU only.)

The paper prints no worked numerical example of the layer math or of the cache
movement, so there are no paper-printed values to pin against; what the paper
does state as properties (shards sum to the whole, shards form the complete
cache, consecutive layers chain) appears below as invariants.
"""
import math

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import kv_tier as kt
from oracle import layer_math as lm


def tiny_cfg(n_q=4, n_kv=2, d=8, hidden=16, ffn=24, n_layers=2):
    return wl.ModelCfg(hidden=hidden, n_q_heads=n_q, n_kv_heads=n_kv, head_dim=d, ffn=ffn,
                       n_layers=n_layers, vocab=32, dtype=wl.F32)


def rand_weights(cfg, seed):
    return [wl.make_layer_weights(cfg, seed + l, std=0.3)[0] for l in range(cfg.n_layers)]


# ---------------------------------------------------------------- RoPE
def test_rope_position_zero_is_identity():
    u = np.random.default_rng(0).standard_normal((3, 2, 8))
    assert np.array_equal(lm.rope(u, [0, 0, 0], 10000.0), u)


def test_rope_two_dim_closed_form():
    # d = 2: the single pair rotates (1, 0) by p radians, any base.
    for p in (1, 2, 7):
        out = lm.rope(np.array([[[1.0, 0.0]]]), [p], 123.0)
        assert np.allclose(out[0, 0], [math.cos(p), math.sin(p)], atol=1e-15)


def test_rope_pairing_and_frequencies_d4():
    # d = 4, base 100: pairs are (0,2) with theta 1 and (1,3) with theta 100^(-2/4) = 0.1.
    p = 3
    u = np.array([[[1.0, 2.0, 3.0, 4.0]]])
    out = lm.rope(u, [p], 100.0)[0, 0]
    c0, s0, c1, s1 = math.cos(3.0), math.sin(3.0), math.cos(0.3), math.sin(0.3)
    want = [1 * c0 - 3 * s0, 2 * c1 - 4 * s1, 3 * c0 + 1 * s0, 4 * c1 + 2 * s1]
    assert np.allclose(out, want, atol=1e-14)


def test_rope_complex_multiplication_form():
    # (u_i + j u_{i+d/2}) * exp(j p theta_i), evaluated with torch complex ops.
    rng = np.random.default_rng(1)
    d, base = 16, 10000.0
    u = rng.standard_normal((5, 3, d))
    pos = np.array([0, 1, 17, 300, 4095])
    z = torch.complex(torch.tensor(u[..., : d // 2]), torch.tensor(u[..., d // 2:]))
    theta = torch.tensor([base ** (-2.0 * i / d) for i in range(d // 2)], dtype=torch.float64)
    rot = torch.polar(torch.ones(5, d // 2, dtype=torch.float64), torch.tensor(pos, dtype=torch.float64)[:, None] * theta)
    zr = z * rot[:, None, :]
    want = torch.cat([zr.real, zr.imag], dim=-1).numpy()
    assert np.allclose(lm.rope(u, pos, base), want, atol=1e-12)


def test_rope_norm_and_relative_position():
    rng = np.random.default_rng(2)
    q = rng.standard_normal((1, 1, 32))
    k = rng.standard_normal((1, 1, 32))
    assert np.allclose(np.linalg.norm(lm.rope(q, [77], 1e4)), np.linalg.norm(q))
    dots = [np.sum(lm.rope(q, [5 + c], 1e4) * lm.rope(k, [2 + c], 1e4)) for c in (0, 1, 40, 1000)]
    assert np.allclose(dots, dots[0], atol=1e-10)
    # and it does depend on the relative offset
    other = np.sum(lm.rope(q, [6], 1e4) * lm.rope(k, [2], 1e4))
    assert abs(other - dots[0]) > 1e-6


# ---------------------------------------------------------------- norm / activation
def test_rmsnorm_closed_forms():
    g = np.array([0.5, 1.0, 2.0, -1.0])
    c, eps = 3.0, 1e-5
    out = lm.rmsnorm(np.full((2, 4), c), g, eps)
    assert np.allclose(out, g * c / math.sqrt(c * c + eps), atol=1e-15)
    assert np.array_equal(lm.rmsnorm(np.zeros((1, 4)), g, eps), np.zeros((1, 4)))
    x = np.random.default_rng(3).standard_normal((6, 4))
    want = torch.nn.functional.rms_norm(torch.tensor(x), (4,), torch.tensor(g), eps).numpy()
    assert np.allclose(lm.rmsnorm(x, g, eps), want, atol=1e-14)


def test_silu_values():
    assert lm.silu(0.0) == 0.0
    assert np.isclose(lm.silu(1.0), 1.0 / (1.0 + math.exp(-1.0)), atol=1e-16)
    assert np.isclose(lm.silu(40.0), 40.0, rtol=1e-15)
    assert abs(lm.silu(-40.0)) < 1e-15
    z = np.linspace(-6, 6, 25)
    assert np.allclose(lm.silu(z), torch.nn.functional.silu(torch.tensor(z)).numpy(), atol=1e-15)


# ---------------------------------------------------------------- attention
def _qkv(seed, T, n_q, n_kv, d):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((T, n_q, d)), rng.standard_normal((n_kv, T, d)),
            rng.standard_normal((n_kv, T, d)))


def test_attention_first_position_returns_v0():
    q, K, V = _qkv(4, 5, 2, 2, 4)
    out = lm.attention_one_sequence(q, K, V, np.arange(5))
    assert np.allclose(out[0], V[:, 0, :], atol=1e-15)


def test_attention_zero_query_gives_running_mean():
    _, K, V = _qkv(5, 6, 2, 1, 4)
    out = lm.attention_one_sequence(np.zeros((6, 2, 4)), K, V, np.arange(6))
    for t in range(6):
        assert np.allclose(out[t, 0], V[0, : t + 1].mean(axis=0), atol=1e-14)
        assert np.allclose(out[t, 1], V[0, : t + 1].mean(axis=0), atol=1e-14)


def test_attention_is_causal_bitwise():
    q, K, V = _qkv(6, 7, 2, 2, 4)
    base = lm.attention_one_sequence(q, K, V, np.arange(7))
    K2, V2 = K.copy(), V.copy()
    K2[:, 4:] += 100.0
    V2[:, 4:] -= 50.0
    pert = lm.attention_one_sequence(q, K2, V2, np.arange(7))
    assert np.array_equal(base[:4], pert[:4])
    assert not np.allclose(base[4:], pert[4:])


def test_attention_brute_force_loops():
    T, n_q, n_kv, d = 5, 4, 2, 3
    q, K, V = _qkv(7, T, n_q, n_kv, d)
    out = lm.attention_one_sequence(q, K, V, np.arange(T))
    for t in range(T):
        for a in range(n_q):
            g = a // 2
            sc = [sum(q[t, a, e] * K[g, j, e] for e in range(d)) / math.sqrt(d) for j in range(t + 1)]
            m = max(sc)
            w = [math.exp(v - m) for v in sc]
            z = sum(w)
            for e in range(d):
                want = sum(w[j] / z * V[g, j, e] for j in range(t + 1))
                assert abs(out[t, a, e] - want) < 1e-13


def test_attention_matches_torch_sdpa_with_gqa():
    T, n_q, n_kv, d = 9, 4, 2, 8
    q, K, V = _qkv(8, T, n_q, n_kv, d)
    out = lm.attention_one_sequence(q, K, V, np.arange(T))
    tq = torch.tensor(q).permute(1, 0, 2)[None]                          # [1, n_q, T, d]
    tk = torch.tensor(K).repeat_interleave(n_q // n_kv, dim=0)[None]
    tv = torch.tensor(V).repeat_interleave(n_q // n_kv, dim=0)[None]
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    assert np.allclose(out, want[0].permute(1, 0, 2).numpy(), atol=1e-12)


def test_attention_decode_query_against_longer_cache():
    # a single query at position p sees exactly keys 0..p even if the arrays are longer
    q, K, V = _qkv(9, 8, 2, 2, 4)
    full = lm.attention_one_sequence(q, K, V, np.arange(8))
    one = lm.attention_one_sequence(q[5:6], K, V, np.array([5]))
    assert np.allclose(one[0], full[5], atol=1e-15)


# ---------------------------------------------------------------- whole layer
def _torch_layer(cfg, w, x, lens):
    """Independent statement of the layer with torch library routines
    (rms_norm, linear, scaled_dot_product_attention, silu); RoPE via complex
    multiplication.  Prefill only, sequences of the given lengths."""
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    F = torch.nn.functional
    d, H = cfg.head_dim, cfg.hidden
    x = t(x)
    h = F.rms_norm(x, (H,), t(w["g1"]), cfg.rms_eps)
    q = F.linear(h, t(w["wq"]).T).reshape(-1, cfg.n_q_heads, d)
    k = F.linear(h, t(w["wk"]).T).reshape(-1, cfg.n_kv_heads, d)
    v = F.linear(h, t(w["wv"]).T).reshape(-1, cfg.n_kv_heads, d)
    pos = torch.cat([torch.arange(n, dtype=torch.float64) for n in lens])
    theta = torch.tensor([cfg.rope_base ** (-2.0 * i / d) for i in range(d // 2)], dtype=torch.float64)
    rot = torch.polar(torch.ones(len(pos), d // 2, dtype=torch.float64), pos[:, None] * theta)[:, None, :]

    def rope(u):
        z = torch.complex(u[..., : d // 2], u[..., d // 2:]) * rot
        return torch.cat([z.real, z.imag], dim=-1)

    q, k = rope(q), rope(k)
    rep = cfg.n_q_heads // cfg.n_kv_heads
    outs, t0 = [], 0
    for n in lens:
        qs = q[t0:t0 + n].permute(1, 0, 2)[None]
        ks = k[t0:t0 + n].permute(1, 0, 2).repeat_interleave(rep, dim=0)[None]
        vs = v[t0:t0 + n].permute(1, 0, 2).repeat_interleave(rep, dim=0)[None]
        o = F.scaled_dot_product_attention(qs, ks, vs, is_causal=True)[0].permute(1, 0, 2)
        outs.append(o.reshape(n, -1))
        t0 += n
    x1 = x + F.linear(torch.cat(outs), t(w["wo"]).T)
    h2 = F.rms_norm(x1, (H,), t(w["g2"]), cfg.rms_eps)
    y = F.linear(F.silu(F.linear(h2, t(w["wg"]).T)) * F.linear(h2, t(w["wu"]).T), t(w["wd"]).T)
    return x1.numpy(), (x1 + y).numpy()


@pytest.mark.parametrize("n_q,n_kv", [(4, 4), (4, 2), (8, 1)])
def test_layer_matches_torch_library_composition(n_q, n_kv):
    cfg = tiny_cfg(n_q=n_q, n_kv=n_kv, d=8, hidden=16, ffn=24, n_layers=1)
    w = rand_weights(cfg, 10)[0]
    lens = [5, 1, 9]
    x = np.random.default_rng(11).standard_normal((sum(lens), cfg.hidden))
    batch = [(i, n, 0) for i, n in enumerate(lens)]
    x1, x2 = lm.layer_forward(cfg, w, x, batch, lm.KVCache(cfg), 0)
    w1, w2 = _torch_layer(cfg, w, x, lens)
    assert np.allclose(x1, w1, atol=1e-11)
    assert np.allclose(x2, w2, atol=1e-11)


def test_gqa_equals_mha_with_replicated_kv_heads():
    cfg_g = tiny_cfg(n_q=4, n_kv=2, n_layers=1)
    cfg_m = tiny_cfg(n_q=4, n_kv=4, n_layers=1)
    w = rand_weights(cfg_g, 20)[0]
    d = cfg_g.head_dim
    wm = dict(w)
    rep = lambda m: np.repeat(m.reshape(cfg_g.hidden, 2, d), 2, axis=1).reshape(cfg_g.hidden, 4 * d)
    wm["wk"], wm["wv"] = rep(w["wk"]), rep(w["wv"])
    x = np.random.default_rng(21).standard_normal((7, cfg_g.hidden))
    batch = [(0, 7, 0)]
    a = lm.layer_forward(cfg_g, w, x, batch, lm.KVCache(cfg_g), 0)[1]
    b = lm.layer_forward(cfg_m, wm, x, batch, lm.KVCache(cfg_m), 0)[1]
    assert np.allclose(a, b, atol=1e-12)


@pytest.mark.parametrize("k", [1, 2, 4])
def test_tp_partials_sum_to_unsharded_layer(k):
    cfg = tiny_cfg(n_q=8, n_kv=4, d=8, hidden=32, ffn=48, n_layers=1)
    w = rand_weights(cfg, 30)[0]
    x = np.random.default_rng(31).standard_normal((11, cfg.hidden))
    batch = [(0, 4, 0), (1, 7, 0)]
    ref1, ref2 = lm.layer_forward(cfg, w, x, batch, lm.KVCache(cfg), 0, k=1)
    cache = lm.KVCache(cfg)
    got1, got2 = lm.layer_forward(cfg, w, x, batch, cache, 0, k=k)
    assert np.max(np.abs(got1 - ref1)) <= 1e-12 * np.max(np.abs(ref1))
    assert np.max(np.abs(got2 - ref2)) <= 1e-12 * np.max(np.abs(ref2))
    # every partial is a genuine fraction (no shard returns the whole)
    if k > 1:
        part = lm.attn_block(cfg, w, x, batch, lm.KVCache(cfg), 0, k, 0)
        assert np.max(np.abs(part - (ref1 - x))) > 1e-3


def test_tp_caches_equal_slices_of_unsharded_cache():
    # the cache a TP shard computes directly == the head slice of the cache the
    # unsharded (pipeline) layout computes: layer 0 to round-off of the matmul.
    cfg = tiny_cfg(n_q=4, n_kv=4, n_layers=1)
    w = rand_weights(cfg, 40)[0]
    x = np.random.default_rng(41).standard_normal((6, cfg.hidden))
    batch = [(0, 6, 0)]
    full = lm.KVCache(cfg)
    lm.attn_block(cfg, w, x, batch, full, 0)
    for i in range(2):
        part = lm.KVCache(cfg)
        lm.attn_block(cfg, w, x, batch, part, 0, k=2, i=i)
        sl = slice(2 * i, 2 * i + 2)
        assert np.allclose(part.data[0][:, :, sl], full.data[0][:, :, sl], atol=1e-13)
        other = slice(2 * (1 - i), 2 * (1 - i) + 2)
        assert np.all(part.data[0][:, :, other] == 0)


def test_pp_stage_split_is_exact():
    cfg = tiny_cfg(n_layers=4)
    ws = rand_weights(cfg, 50)
    x = np.random.default_rng(51).standard_normal((5, cfg.hidden))
    batch = [(0, 5, 0)]
    c1, c2 = lm.KVCache(cfg), lm.KVCache(cfg)
    whole = lm.run_layers(cfg, ws, x, batch, c1, 0, 4)
    half = lm.run_layers(cfg, ws, x, batch, c2, 0, 2)
    split = lm.run_layers(cfg, ws, half, batch, c2, 2, 4)
    assert np.array_equal(whole, split)
    assert np.array_equal(c1.data[0], c2.data[0])


def test_prefill_then_decode_equals_longer_prefill():
    cfg = tiny_cfg(n_layers=2)
    ws = rand_weights(cfg, 60)
    x = np.random.default_rng(61).standard_normal((9, cfg.hidden))
    ca, cb = lm.KVCache(cfg), lm.KVCache(cfg)
    full = lm.run_layers(cfg, ws, x, [(0, 9, 0)], ca, 0, 2)
    lm.run_layers(cfg, ws, x[:8], [(0, 8, 0)], cb, 0, 2)
    step = lm.run_layers(cfg, ws, x[8:9], [(0, 1, 8)], cb, 0, 2)
    assert np.allclose(step[0], full[8], atol=1e-12)
    assert np.allclose(ca.data[0], cb.data[0], atol=1e-12)


def test_chunked_prefill_equals_whole_prefill():
    cfg = tiny_cfg(n_layers=1)
    ws = rand_weights(cfg, 62)
    x = np.random.default_rng(63).standard_normal((10, cfg.hidden))
    ca, cb = lm.KVCache(cfg), lm.KVCache(cfg)
    full = lm.run_layers(cfg, ws, x, [(0, 10, 0)], ca, 0, 1)
    a = lm.run_layers(cfg, ws, x[:6], [(0, 6, 0)], cb, 0, 1)
    b = lm.run_layers(cfg, ws, x[6:], [(0, 4, 6)], cb, 0, 1)
    assert np.allclose(np.concatenate([a, b]), full, atol=1e-12)


def test_batch_order_independence():
    cfg = tiny_cfg(n_layers=1)
    w = rand_weights(cfg, 64)[0]
    rng = np.random.default_rng(65)
    xa, xb = rng.standard_normal((3, cfg.hidden)), rng.standard_normal((5, cfg.hidden))
    ab = lm.layer_forward(cfg, w, np.concatenate([xa, xb]), [(0, 3, 0), (1, 5, 0)], lm.KVCache(cfg), 0)[1]
    ba = lm.layer_forward(cfg, w, np.concatenate([xb, xa]), [(1, 5, 0), (0, 3, 0)], lm.KVCache(cfg), 0)[1]
    assert np.allclose(ab[:3], ba[5:], atol=1e-13) and np.allclose(ab[3:], ba[:5], atol=1e-13)


def test_swiglu_reduces_to_silu_when_up_is_one():
    cfg = tiny_cfg(n_layers=1)
    w = dict(rand_weights(cfg, 66)[0])
    x1 = np.random.default_rng(67).standard_normal((4, cfg.hidden))
    h2 = lm.rmsnorm(x1, w["g2"], cfg.rms_eps)
    # choose Wu by least squares so that h2 @ Wu == 1 for these rows (4 rows, 16 unknowns)
    col = np.linalg.lstsq(h2, np.ones(4), rcond=None)[0]
    w["wu"] = np.repeat(col[:, None], cfg.ffn, axis=1)
    want = lm.silu(h2 @ w["wg"]) @ w["wd"]
    assert np.allclose(lm.mlp_block(cfg, w, x1), want, atol=1e-11)


def test_config1_pp_and_tp2_agree_end_to_end():
    work = wl.config1()
    cfg = work.cfg
    ws = [wl.make_layer_weights(cfg, 1001 + l)[0] for l in range(cfg.n_layers)]
    head = wl.make_head_weights(cfg, 1099)[0]
    rng = np.random.default_rng(1001)
    prompts = [rng.integers(0, cfg.vocab, size=8) for _ in range(2)]
    t1, l1, c1 = lm.generate(cfg, ws, head, prompts, 3, k=1)
    t2, l2, c2 = lm.generate(cfg, ws, head, prompts, 3, k=2)
    assert np.array_equal(t1, t2)
    for a, b in zip(l1, l2):
        assert np.max(np.abs(a - b)) <= 1e-10 * np.max(np.abs(a))
    assert c1.length(0) == 8 + 3 and t1.shape == (2, 4)


# ---------------------------------------------------------------- whole model (embedding, LM head, greedy, generate)
def test_embed_is_a_row_lookup_on_a_labelled_table():
    # table entry (t, j) = 100 t + j: every output element names its token and its column
    vocab, hidden = 7, 5
    table = 100.0 * np.arange(vocab)[:, None] + np.arange(hidden)[None, :]
    toks = np.array([3, 0, 6, 3])
    out = lm.embed({"embed": table}, toks)
    assert out.shape == (4, hidden)
    for r, t in enumerate(toks):
        for j in range(hidden):
            assert out[r, j] == 100.0 * t + j


def test_lm_logits_hand_values_and_torch_library_form():
    # hand-worked: H = 2, vocab = 3, row (3, 4): mean square 12.5, eps 0 -> h = (3, 4) / sqrt(12.5) * gf
    cfg = wl.ModelCfg(hidden=2, n_q_heads=1, n_kv_heads=1, head_dim=2, ffn=2, vocab=3, dtype=wl.F32, rms_eps=0.0)
    head = {"gf": np.array([2.0, 0.5]), "wlm": np.array([[1.0, 0.0, 2.0], [0.0, 1.0, -1.0]])}
    r = math.sqrt(12.5)
    h0, h1 = 3.0 / r * 2.0, 4.0 / r * 0.5
    got = lm.lm_logits(cfg, head, np.array([[3.0, 4.0]]))
    assert got.shape == (1, 3)
    assert np.allclose(got[0], [h0, h1, 2.0 * h0 - h1], atol=1e-15)
    # library form on a non-square head [H, vocab] (a transposed operand cannot even multiply)
    cfg = wl.ModelCfg(hidden=12, n_q_heads=1, n_kv_heads=1, head_dim=4, ffn=8, vocab=29, dtype=wl.F32)
    rng = np.random.default_rng(70)
    head = {"gf": 1.0 + 0.3 * rng.standard_normal(12), "wlm": rng.standard_normal((12, 29))}
    x = rng.standard_normal((6, 12))
    want = torch.nn.functional.linear(
        torch.nn.functional.rms_norm(torch.tensor(x), (12,), torch.tensor(head["gf"]), cfg.rms_eps),
        torch.tensor(head["wlm"]).T.contiguous())
    assert np.allclose(lm.lm_logits(cfg, head, x), want.numpy(), atol=1e-12)


def test_greedy_takes_the_lowest_index_among_equal_maxima():
    logits = np.array([[0.5, 2.0, -1.0, 2.0, 2.0],      # three equal maxima -> the first of them
                       [-3.0, -3.0, -7.0, -3.0, -9.0],  # negative values, tie at 0, 1, 3
                       [1.0, 1.5, 1.25, 1.5, 9.0]])     # unique maximum at the end
    assert lm.greedy(logits).tolist() == [1, 0, 4]


def permutation_model(vocab, n_layers, seed):
    """A model whose greedy continuation is known in closed form: the output projections Wo and Wd are zero,
    so every layer is the identity on the residual stream (the attention and MLP blocks still run); the
    embedding of token t is c_t * e_t (one scaled unit vector per token); the final gain is 1 and the LM head
    sends unit vector t to unit vector pi(t).  RMSNorm keeps the direction of c_t * e_t, so the largest logit
    after token t sits at pi(t): every emitted token is pi of the token before it."""
    cfg = wl.ModelCfg(hidden=vocab, n_q_heads=2, n_kv_heads=1, head_dim=4, ffn=6, n_layers=n_layers, vocab=vocab,
                      dtype=wl.F32)
    ws = []
    for l in range(n_layers):
        w = dict(wl.make_layer_weights(cfg, seed + l, std=0.3)[0])
        w["wo"] = np.zeros_like(w["wo"])
        w["wd"] = np.zeros_like(w["wd"])
        ws.append(w)
    rng = np.random.default_rng(seed + 100)
    pi = rng.permutation(vocab)
    head = {"embed": np.diag(1.0 + rng.random(vocab)), "gf": np.ones(vocab), "wlm": np.zeros((vocab, vocab))}
    head["wlm"][np.arange(vocab), pi] = 1.0
    return cfg, ws, head, pi


def test_generate_follows_the_permutation_closed_form_on_ragged_prompts():
    cfg, ws, head, pi = permutation_model(vocab=11, n_layers=2, seed=71)
    # unequal lengths, and every prompt ends in a token whose image differs from that of any other prompt row a
    # wrong "last position" index could pick (row 0 of the batch, the first token of the next prompt, ...)
    prompts = [np.array([4, 9, 1]), np.array([7]), np.array([2, 2, 5, 0, 8]), np.array([3, 6])]
    steps = 6
    toks, logits, cache = lm.generate(cfg, ws, head, prompts, steps)
    assert toks.shape == (4, steps + 1) and len(logits) == steps + 1
    for s, p in enumerate(prompts):
        want, t = [], p[-1]
        for _ in range(steps + 1):           # token 1 comes from the prefill (last prompt position), then `steps` more
            t = pi[t]
            want.append(t)
        assert toks[s].tolist() == want
        assert cache.length(s) == len(p) + steps     # the last emitted token is not fed back


def test_generate_equals_recomputation_of_every_step_from_the_whole_prefix():
    # Every step's logits must equal those of a fresh prefill over prompt + tokens emitted so far (run_layers on
    # an empty cache, last row), which uses neither generate's bookkeeping of lengths nor its cache.
    cfg = tiny_cfg()
    ws = rand_weights(cfg, 72)
    head = wl.make_head_weights(cfg, 73, std=0.3)[0]
    rng = np.random.default_rng(74)
    prompts = [rng.integers(0, cfg.vocab, size=n) for n in (5, 1, 9)]
    steps = 4
    toks, logits, cache = lm.generate(cfg, ws, head, prompts, steps)
    for s, p in enumerate(prompts):
        for j in range(steps + 1):
            prefix = np.concatenate([p, toks[s, :j]])
            run = lm.run_layers(cfg, ws, lm.embed(head, prefix), [(0, len(prefix), 0)], lm.KVCache(cfg), 0,
                                    cfg.n_layers)
            want = lm.lm_logits(cfg, head, run[-1:])[0]
            assert np.allclose(logits[j][s], want, atol=1e-10), (s, j)
            assert toks[s, j] == int(np.argmax(want))
        assert cache.length(s) == len(p) + steps


# ---------------------------------------------------------------- tier / paging
def test_tier_index_is_c_order_of_layer_kv_head_pos_dim():
    L, n_kv, s, d = 3, 4, 5, 2
    n = kt.tier_seq_elems(L, n_kv, d, s)
    assert n == L * 2 * n_kv * s * d
    ref = np.arange(n).reshape(L, 2, n_kv, s, d)       # numpy's own C-order
    for (l, c, g, p, e) in [(0, 0, 0, 0, 0), (2, 1, 3, 4, 1), (1, 0, 2, 3, 0), (0, 1, 0, 0, 0)]:
        assert kt.tier_index(n_kv, d, s, l, c, g, p, e) == ref[l, c, g, p, e]
    # heads-major inside each (layer, K|V): one head's whole sequence is contiguous
    assert kt.tier_index(n_kv, d, s, 1, 1, 2, 1, 0) - kt.tier_index(n_kv, d, s, 1, 1, 2, 0, 0) == d
    assert kt.tier_index(n_kv, d, s, 1, 1, 3, 0, 0) - kt.tier_index(n_kv, d, s, 1, 1, 2, 0, 0) == s * d


def test_pp_shards_form_complete_cache_and_tp_shards_are_head_slices():
    L, n_kv, s, d = 4, 4, 7, 3
    rng = np.random.default_rng(70)
    complete = rng.integers(0, 2 ** 16, size=(L, 2, n_kv, s, d)).astype(np.uint16)
    n = kt.tier_seq_elems(L, n_kv, d, s)
    tier = np.zeros(100 + n, dtype=np.uint16)
    for j in range(2):                                   # two pipeline stages push layer slices
        kt.tier_put(tier, 100, complete[2 * j:2 * j + 2], n_kv, (2 * j, 2 * j + 2), (0, n_kv))
    assert np.array_equal(tier[100:].reshape(L, 2, n_kv, s, d), complete)
    assert np.all(tier[:100] == 0)
    for i in range(4):                                   # four TP shards pull one head each
        got = kt.tier_get(tier, 100, s, n_kv, d, (0, L), (i, i + 1))
        assert np.array_equal(got, complete[:, :, i:i + 1])
    got = kt.tier_get(tier, 100, s, n_kv, d, (1, 3), (2, 4))
    assert np.array_equal(got, complete[1:3, :, 2:4])


def test_page_allocator_policy():
    a = kt.PageAllocator(8, page_size=16)
    assert a.ensure(10, 1) == [0]
    assert a.ensure(11, 33) == [1, 2, 3]
    assert a.ensure(10, 16) == [0]            # still fits one page
    assert a.ensure(10, 17) == [0, 4]         # grows by appending the lowest free id
    a.release(11)
    assert a.free == [1, 2, 3, 5, 6, 7]
    assert a.ensure(12, 40) == [1, 2, 3]
    with pytest.raises(MemoryError):
        a.ensure(13, 16 * 4)
    assert a.pages_needed(0) == 0 and a.pages_needed(16) == 1 and a.pages_needed(17) == 2


def test_paged_store_round_trip_and_slot_addressing():
    rng = np.random.default_rng(71)
    st = kt.PagedStore(n_pages=6, n_layers_local=2, n_heads_local=3, d=4, dtype=np.uint16)
    a = rng.integers(0, 2 ** 16, size=(2, 2, 3, 20, 4)).astype(np.uint16)
    b = rng.integers(0, 2 ** 16, size=(2, 2, 3, 5, 4)).astype(np.uint16)
    st.write(0, a[:, :, :, :9])
    st.write(1, b)
    st.write(0, a[:, :, :, 9:], start=9)     # grows across a page boundary
    assert st.alloc.tables == {0: [0, 2], 1: [1]}
    assert np.array_equal(st.read(0), a) and np.array_equal(st.read(1), b)
    # token 17 of sequence 0 sits in its second page, slot 1
    assert np.array_equal(st.pool[1, 0, 2, 2, 1], a[1, 0, 2, 17])


def test_tier_allocator_full_and_empty_cycle():
    t = kt.TierAllocator(100)
    assert t.place(5, 40) == 0 and t.place(6, 50) == 40 and t.place(5, 40) == 0
    with pytest.raises(MemoryError):
        t.place(7, 20)                        # 10 free: full
    t.release(5)
    assert t.used == 50 and t.free == [(0, 40), (90, 10)]
    assert t.place(9, 30) == 0                # first fit, lowest address
    with pytest.raises(MemoryError):
        t.place(10, 15)                       # holes of 10 and 10 do not add up
    assert t.place(11, 10) == 30
    t.release(6)
    t.release(9)
    t.release(11)
    assert t.used == 0 and t.free == [(0, 100)] and t.place(8, 100) == 0   # empty again: restart at 0


def test_reshard_pp_to_tp_union_is_identity():
    L, n_kv, d = 4, 4, 2
    lens = {3: 21, 9: 16, 4: 1}
    rng = np.random.default_rng(72)
    complete = {s: rng.integers(0, 2 ** 16, size=(L, 2, n_kv, n, d)).astype(np.uint16) for s, n in lens.items()}
    tier = np.zeros(sum(kt.tier_seq_elems(L, n_kv, d, n) for n in lens.values()), dtype=np.uint16)
    talloc = kt.TierAllocator(tier.size)
    stages = []
    for j in range(2):
        st = kt.PagedStore(8, 2, n_kv, d, np.uint16)
        for s in lens:
            st.write(s, complete[s][2 * j:2 * j + 2])
        stages.append(st)
    shards = [kt.PagedStore(8, L, 2, d, np.uint16) for _ in range(2)]
    # both stages push, then both TP shards pull
    for j, st in enumerate(stages):
        for s in lens:
            base = talloc.place(s, kt.tier_seq_elems(L, n_kv, d, lens[s]))
            kt.tier_put(tier, base, st.read(s), n_kv, (2 * j, 2 * j + 2), (0, n_kv))
    for i, sh in enumerate(shards):
        for s in lens:
            sh.write(s, kt.tier_get(tier, talloc.base[s][0], lens[s], n_kv, d, (0, L), (2 * i, 2 * i + 2)))
    for s in lens:
        union = np.concatenate([shards[0].read(s), shards[1].read(s)], axis=2)
        assert np.array_equal(union, complete[s])
    # single-stage helper agrees with the hand-rolled sequence above
    tier2 = np.zeros_like(tier)
    src = kt.PagedStore(8, L, n_kv, d, np.uint16)
    for s in lens:
        src.write(s, complete[s])
    dst = kt.PagedStore(8, L, 1, d, np.uint16)
    kt.reshard(src, dst, tier2, kt.TierAllocator(tier2.size), list(lens), L, n_kv, d,
               (0, L), (0, n_kv), (0, L), (3, 4))
    for s in lens:
        assert np.array_equal(dst.read(s), complete[s][:, :, 3:4])
    assert np.array_equal(tier2, tier)


def test_staging_offsets():
    off = kt.staging_offsets([3, 5], n_layers_local=2, n_heads_local=4, d=8)
    assert list(off) == [0, 3 * 2 * 2 * 4 * 8, 8 * 2 * 2 * 4 * 8]


# ---------------------------------------------------------------- input helpers
def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, 1.0 + 3 * 2 ** -8, -2.5, 0.0], dtype=np.float32)
    bits = wl.bf16_bits(x)
    back = wl.bf16_to_f32(bits)
    assert list(back) == [1.0, 1.0, 1.0 + 2 ** -7, 1.0 + 2 ** -6, -2.5, 0.0]
    t = torch.tensor(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, t)
