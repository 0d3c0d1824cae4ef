"""CPU oracle for the decoder-layer math.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package; the product path (the HIP library and its Python binding) never
does, and shares no code with it.

What is computed.  The paper says of a decoder layer only that it is made of
linear layers around one attention layer, with grouped-query attention in the
models it runs (section 2.1 "Transformer Architecture", section 6.1 "Model"),
and gives no formulas; the
LLaMA-style definitions below (RMSNorm, rotary embedding in the half-split
pairing, 1/sqrt(d) scaled causal softmax attention, SwiGLU, pre-norm residual
layout, no biases) are the reading this build fixes.  What the paper does fix
is followed literally:
  * prefill processes every prompt token at once, decode one new token per
    sequence against the cached K and V (section 2.1 "Auto-regressive
    Generation");
  * tensor parallelism shards the weights, every device computes a portion and
    the partial results are summed (section 2.2 "Parallelism"; section 3.1
    Observation 1; Appendix A.3 "Tensor parallelism");
  * pipeline parallelism gives each device a run of consecutive layers
    (section 3.1 Observation 2; Appendix A.3 "Pipeline parallelism").

Everything is float64 numpy, written as the plain definitions: no blocking, no
fusion, no online softmax.  numpy's matmul is the only library primitive used
as a step.
"""
import numpy as np


# --------------------------------------------------------------------------
# elementwise pieces
# --------------------------------------------------------------------------
def rmsnorm(x, g, eps):
    """y = x * (mean_j x_j^2 + eps)^(-1/2) * g, row by row."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(g, dtype=np.float64)


def silu(z):
    z = np.asarray(z, dtype=np.float64)
    return z / (1.0 + np.exp(-z))


def rope_angles(pos, d, base):
    """theta_i = base^(-2i/d), i in [0, d/2); returns p*theta as [len(pos), d/2]."""
    i = np.arange(d // 2, dtype=np.float64)
    theta = np.power(float(base), -2.0 * i / d)
    return np.asarray(pos, dtype=np.float64)[:, None] * theta[None, :]


def rope(u, pos, base):
    """Rotate every head vector of u [T, n_heads, d] by its token's position.

    Half-split pairing: element i is paired with element i + d/2."""
    u = np.asarray(u, dtype=np.float64)
    d = u.shape[-1]
    ang = rope_angles(pos, d, base)
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    lo, hi = u[..., : d // 2], u[..., d // 2:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def softmax_rows(s):
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def attention_one_sequence(q, K, V, q_pos):
    """Causal attention of one sequence.

    q [Tq, n_q, d] (already rotated), K and V [n_kv, S, d] hold cache positions
    0..S-1, q_pos [Tq] are the absolute positions of the queries.  Query at
    position p sees keys 0..p inclusive.  q head a uses kv head a // (n_q/n_kv).
    Returns [Tq, n_q, d]."""
    Tq, n_q, d = q.shape
    n_kv, S, _ = K.shape
    group = n_q // n_kv
    out = np.zeros((Tq, n_q, d), dtype=np.float64)
    key_pos = np.arange(S)
    visible = key_pos[None, :] <= np.asarray(q_pos)[:, None]          # [Tq, S]
    for a in range(n_q):
        g = a // group
        s = (q[:, a, :] @ K[g].T) / np.sqrt(float(d))
        s = np.where(visible, s, -np.inf)
        out[:, a, :] = softmax_rows(s) @ V[g]
    return out


# --------------------------------------------------------------------------
# shard geometry (paper: TP holds 1/k of the weights, PP holds whole layers)
# --------------------------------------------------------------------------
def shard_ranges(cfg, k, i):
    """Head and FFN-column ranges of tensor-parallel shard i of k."""
    if cfg.n_q_heads % k or cfg.n_kv_heads % k or cfg.ffn % k:
        raise ValueError("k must divide n_q_heads, n_kv_heads and ffn")
    nq, nkv, f = cfg.n_q_heads // k, cfg.n_kv_heads // k, cfg.ffn // k
    return (i * nq, (i + 1) * nq), (i * nkv, (i + 1) * nkv), (i * f, (i + 1) * f)


class KVCache:
    """Complete logical cache: seq id -> float64 array [n_layers, 2, n_kv, len, d]."""

    def __init__(self, cfg):
        self.cfg = cfg
        self.data = {}

    def ensure(self, seq, length):
        cfg = self.cfg
        cur = self.data.get(seq)
        if cur is None:
            self.data[seq] = np.zeros((cfg.n_layers, 2, cfg.n_kv_heads, length, cfg.head_dim))
        elif cur.shape[3] < length:
            grown = np.zeros((cfg.n_layers, 2, cfg.n_kv_heads, length, cfg.head_dim))
            grown[:, :, :, : cur.shape[3]] = cur
            self.data[seq] = grown

    def length(self, seq):
        return self.data[seq].shape[3]


def batch_positions(batch):
    """batch: list of (seq_id, q_len, kv_len_before).  Returns per-token positions
    and the [start, end) token range of every sequence in the concatenated batch."""
    pos, spans, t = [], [], 0
    for _, q_len, before in batch:
        pos.extend(range(before, before + q_len))
        spans.append((t, t + q_len))
        t += q_len
    return np.array(pos, dtype=np.int64), spans


# --------------------------------------------------------------------------
# the two halves of a layer, per shard
# --------------------------------------------------------------------------
def attn_block(cfg, w, x, batch, cache, layer, k=1, i=0, round_kv=None):
    """Shard i's partial of the attention block, WITHOUT the residual.

    x [T, H] is the (replicated) layer input for the concatenated batch.  The
    shard projects only its heads, writes its K/V heads into `cache`, attends,
    and multiplies by its rows of Wo.  Summing the k partials gives the
    unsharded block output.  `round_kv`, if given, is applied to K and V before
    they are cached (models a cache kept in a narrower storage type)."""
    (q0, q1), (g0, g1), _ = shard_ranges(cfg, k, i)
    d = cfg.head_dim
    x = np.asarray(x, dtype=np.float64)
    T = x.shape[0]
    pos, spans = batch_positions(batch)
    h = rmsnorm(x, w["g1"], cfg.rms_eps)
    q = (h @ w["wq"][:, q0 * d:q1 * d]).reshape(T, q1 - q0, d)
    kk = (h @ w["wk"][:, g0 * d:g1 * d]).reshape(T, g1 - g0, d)
    v = (h @ w["wv"][:, g0 * d:g1 * d]).reshape(T, g1 - g0, d)
    q = rope(q, pos, cfg.rope_base)
    kk = rope(kk, pos, cfg.rope_base)
    if round_kv is not None:
        kk, v = round_kv(kk), round_kv(v)
    attn = np.zeros((T, q1 - q0, d))
    for (seq, q_len, before), (t0, t1) in zip(batch, spans):
        cache.ensure(seq, before + q_len)
        store = cache.data[seq]
        store[layer, 0, g0:g1, before:before + q_len] = kk[t0:t1].transpose(1, 0, 2)
        store[layer, 1, g0:g1, before:before + q_len] = v[t0:t1].transpose(1, 0, 2)
        S = before + q_len
        attn[t0:t1] = attention_one_sequence(q[t0:t1], store[layer, 0, g0:g1, :S],
                                             store[layer, 1, g0:g1, :S], pos[t0:t1])
    return attn.reshape(T, (q1 - q0) * d) @ w["wo"][q0 * d:q1 * d, :]


def mlp_block(cfg, w, x1, k=1, i=0):
    """Shard i's partial of the SwiGLU block, WITHOUT the residual."""
    _, _, (f0, f1) = shard_ranges(cfg, k, i)
    h2 = rmsnorm(x1, w["g2"], cfg.rms_eps)
    a = silu(h2 @ w["wg"][:, f0:f1]) * (h2 @ w["wu"][:, f0:f1])
    return a @ w["wd"][f0:f1, :]


def layer_forward(cfg, w, x, batch, cache, layer, k=1, round_kv=None):
    """Full layer as the sum of k shard partials; the two sums are where the
    tensor-parallel all-reduces sit (paper Table 3, T_nw column)."""
    x = np.asarray(x, dtype=np.float64)
    x1 = x + sum(attn_block(cfg, w, x, batch, cache, layer, k, i, round_kv) for i in range(k))
    x2 = x1 + sum(mlp_block(cfg, w, x1, k, i) for i in range(k))
    return x1, x2


def run_layers(cfg, weights, x, batch, cache, layer_begin, layer_end, k=1, round_kv=None):
    """A pipeline stage: consecutive layers [layer_begin, layer_end)."""
    for l in range(layer_begin, layer_end):
        _, x = layer_forward(cfg, weights[l], x, batch, cache, l, k, round_kv)
    return x


# --------------------------------------------------------------------------
# tiny whole model (embedding, layers, final norm, LM head, greedy)
# --------------------------------------------------------------------------
def embed(head, tokens):
    return np.asarray(head["embed"], dtype=np.float64)[np.asarray(tokens)]


def lm_logits(cfg, head, x):
    return rmsnorm(x, head["gf"], cfg.rms_eps) @ np.asarray(head["wlm"], dtype=np.float64)


def greedy(logits):
    """Lowest index among equal maxima."""
    return np.argmax(logits, axis=-1)


def generate(cfg, weights, head, prompts, steps, k=1):
    """Prefill every prompt (emits token 1 from the last prompt position), then
    `steps` decode steps.  Returns (tokens [n, steps+1], list of logits arrays,
    cache)."""
    cache = KVCache(cfg)
    n = len(prompts)
    batch = [(s, len(p), 0) for s, p in enumerate(prompts)]
    x = embed(head, np.concatenate(prompts))
    x = run_layers(cfg, weights, x, batch, cache, 0, cfg.n_layers, k)
    last = np.cumsum([len(p) for p in prompts]) - 1
    logits = lm_logits(cfg, head, x[last])
    all_logits = [logits]
    toks = [greedy(logits)]
    lens = [len(p) for p in prompts]
    for _ in range(steps):
        batch = [(s, 1, lens[s]) for s in range(n)]
        x = embed(head, toks[-1])
        x = run_layers(cfg, weights, x, batch, cache, 0, cfg.n_layers, k)
        logits = lm_logits(cfg, head, x)
        all_logits.append(logits)
        toks.append(greedy(logits))
        lens = [v + 1 for v in lens]
    return np.stack(toks, axis=1), all_logits, cache
