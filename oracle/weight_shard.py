"""CPU oracle for weight re-sharding.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package; the product path never does, and shares no code with it.

What is computed.  The paper re-partitions the model weights at every switch
between the prefill strategy c_p and the decode strategy c_d by reloading the
shards the new strategy needs from a copy of the model kept in CPU memory
(section 4.1 "Dynamic Model Re-sharding", Figure 5), and notes that this cost
does not depend on the batch size (section 4.2, overhead paragraph).  It does
not spell out which part of which matrix a device holds; the reading fixed here
is the one its cost model implies (Appendix A.3: a tensor-parallel device holds
and multiplies 1/k of every weight matrix and the partial results are summed;
a pipeline-parallel device holds whole layers):

  * tensor parallel, shard i of k: the columns of Wq, Wk, Wv of its heads, the
    rows of Wo of its query heads, the columns of Wg, Wu and the rows of Wd of
    its FFN range; both gain vectors in full (replicated);
  * pipeline parallel: every matrix of the layers [layer_begin, layer_end) in
    full (k = 1 below).

Plain numpy slicing on the caller's arrays: data movement only, so results are
exact in any dtype.
"""
import numpy as np

MATRICES = ("wq", "wk", "wv", "wo", "wg", "wu", "wd")
GAINS = ("g1", "g2")


def head_and_ffn_ranges(cfg, k, i):
    """[begin, end) of shard i's query heads, kv heads and FFN columns."""
    if k < 1 or not 0 <= i < k:
        raise ValueError("shard index outside [0, k)")
    if cfg.n_q_heads % k or cfg.n_kv_heads % k or cfg.ffn % k:
        raise ValueError("k must divide n_q_heads, n_kv_heads and ffn")
    nq, nkv, f = cfg.n_q_heads // k, cfg.n_kv_heads // k, cfg.ffn // k
    return (i * nq, i * nq + nq), (i * nkv, i * nkv + nkv), (i * f, i * f + f)


def shard_weights(cfg, w, k, i):
    """The part of one layer's weights that shard i of k holds.

    w maps the nine names to the full arrays in [in_features, out_features]
    orientation; the result uses the same orientation."""
    (q0, q1), (g0, g1), (f0, f1) = head_and_ffn_ranges(cfg, k, i)
    d = cfg.head_dim
    return {
        "g1": np.asarray(w["g1"]).copy(),
        "g2": np.asarray(w["g2"]).copy(),
        "wq": np.asarray(w["wq"])[:, q0 * d:q1 * d].copy(),
        "wk": np.asarray(w["wk"])[:, g0 * d:g1 * d].copy(),
        "wv": np.asarray(w["wv"])[:, g0 * d:g1 * d].copy(),
        "wo": np.asarray(w["wo"])[q0 * d:q1 * d, :].copy(),
        "wg": np.asarray(w["wg"])[:, f0:f1].copy(),
        "wu": np.asarray(w["wu"])[:, f0:f1].copy(),
        "wd": np.asarray(w["wd"])[f0:f1, :].copy(),
    }


def shard_matrix_elems(cfg, k):
    """Matrix elements one shard holds per layer: the paper's W / k."""
    d, H = cfg.head_dim, cfg.hidden
    nq, nkv, f = cfg.n_q_heads // k, cfg.n_kv_heads // k, cfg.ffn // k
    return H * (nq + 2 * nkv) * d + nq * d * H + 3 * H * f


def reload_elems(cfg, k_to, layer_begin, layer_end):
    """Elements (matrices + gains) a device loads from the CPU copy when it
    becomes shard (k_to, *) of the layers [layer_begin, layer_end): independent
    of what it held before and of the batch size."""
    return (layer_end - layer_begin) * (shard_matrix_elems(cfg, k_to) + 2 * cfg.hidden)


def reshard(cfg, cpu_model, to_k, to_i, layer_begin, layer_end):
    """What the device holds after the switch: {layer: shard_weights(...)}.

    cpu_model is the list of full per-layer weight dicts kept in CPU memory; the
    result depends on nothing else (reloading, not device-to-device exchange)."""
    return {l: shard_weights(cfg, cpu_model[l], to_k, to_i) for l in range(layer_begin, layer_end)}
