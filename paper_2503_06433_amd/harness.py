"""Helpers shared by the GPU parity tests, smoke() and bench.py: turning seeded
numpy inputs into device buffers and back, and building contexts from a
workload description.  torch is used for device memory only; nothing here
computes anything of the method, and nothing here touches the CPU oracle."""
import numpy as np
import torch

import workloads as wl

from . import binding as ss


def model_cfg(cfg):
    return ss.ModelCfg(cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.ffn, cfg.n_layers,
                       cfg.vocab, cfg.rms_eps, cfg.rope_base, cfg.dtype, cfg.page_size)


def make_context(cfg, pages, tier_bytes=0, pinned_bytes=0, max_seq_len=4608):
    rt = ss.RuntimeCfg(pages, tier_bytes, pinned_bytes, 0, max_seq_len)
    return ss.Context(model_cfg(cfg), rt)


def torch_dtype(dtype):
    return {wl.F32: torch.float32, wl.BF16: torch.bfloat16, wl.F16: torch.float16}[dtype]


def to_device(raw, dtype):
    """raw storage array (float32 or uint16 bf16 bits) -> cuda tensor of the model dtype."""
    raw = np.ascontiguousarray(raw)
    if dtype == wl.F32:
        return torch.from_numpy(raw).cuda()
    return torch.from_numpy(raw.view(np.int16)).cuda().view(torch_dtype(dtype))


def to_f64(t, dtype):
    """cuda tensor of the model dtype -> float64 numpy."""
    if dtype == wl.F32:
        return t.detach().cpu().numpy().astype(np.float64)
    bits = t.detach().view(torch.int16).cpu().numpy().view(np.uint16)
    return wl.storage_to_f64(bits, dtype)


def to_raw(t, dtype):
    if dtype == wl.F32:
        return t.detach().cpu().numpy()
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)


def empty_like_acts(T, width, dtype):
    return torch.empty((T, width), device="cuda", dtype=torch_dtype(dtype))


def rel_err(got, ref):
    """max |got - ref| / max |ref| : the metric of the acceptance thresholds."""
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - ref)) / max(np.max(np.abs(ref)), 1e-30))


def tol(dtype):
    return 1e-4 if dtype == wl.F32 else 2e-2


def row_errs(got, ref):
    """Per-row relative error in the 2-norm, rows = vectors along the last axis (a token's hidden vector,
    a cached head vector): |got_r - ref_r|_2 / |ref_r|_2."""
    ref = np.asarray(ref, dtype=np.float64)
    dif = np.asarray(got, dtype=np.float64) - ref
    num = np.sqrt(np.sum(dif * dif, axis=-1))
    den = np.sqrt(np.sum(ref * ref, axis=-1))
    return (num / np.maximum(den, 1e-30)).reshape(-1)


# Bounds on the per-row error.  The acceptance metric (rel_err, one maximum per tensor) lets a single row be far
# off its own magnitude; this one does not.  Every bound is three times the largest value observed for its class
# over the GPU suite (`parity` records them, the test session lists them at its end):
#   small shapes (hidden <= 1024, rows of a few hundred tokens): bf16 5.7e-3, half 7.3e-4, fp32 1.0e-6;
#   the full-size configurations and the wide-score case (hidden 4096-8192, attention rows over thousands of
#   tokens, layer outputs in which the MLP block sees the attention block's error): bf16 1.7e-2, half 1.9e-3.
# The errors are rounding of the intermediates kept in the storage type (normed input, q/k/v, softmax weights,
# attention output, x1, SwiGLU output): the half build, with three more significand bits, sits 8 times lower
# on every check.
ROW_TOL = {wl.F32: 4e-6, wl.BF16: 1.7e-2, wl.F16: 2.2e-3}
ROW_TOL_FULL = {wl.F32: 4e-6, wl.BF16: 5e-2, wl.F16: 6e-3}

OBSERVED = []     # (label, rel_err, worst row error, median row error, rows)


def parity(got, ref, dtype, label, spans=None, row_tol=None):
    """Acceptance check plus the tighter ones: rel_err over the tensor, rel_err per sequence (spans = list of
    (begin, end) row ranges), and the per-row 2-norm error.  Records what was observed."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, "%s: shape %s vs %s" % (label, got.shape, ref.shape)
    e = rel_err(got, ref)
    r = row_errs(got, ref)
    OBSERVED.append((label, e, float(np.max(r)), float(np.median(r)), int(r.size)))
    assert e <= tol(dtype), "%s: max|d|/max|ref| = %.3e" % (label, e)
    for a, b in (spans or []):
        es = rel_err(got[a:b], ref[a:b])
        assert es <= tol(dtype), "%s rows [%d, %d): max|d|/max|ref| = %.3e" % (label, a, b, es)
    worst = int(np.argmax(r))
    bound = ROW_TOL[dtype] if row_tol is None else row_tol
    assert r[worst] <= bound, "%s: row %d is off by %.3e of its norm (bound %.1e)" % (label, worst, r[worst], bound)
    return e


def pp_desc(cfg, lb=0, le=None):
    return ss.ShardDesc(ss.SS_PP, 1, 0, lb, cfg.n_layers if le is None else le)


def tp_desc(cfg, k, i, lb=0, le=None):
    return ss.ShardDesc(ss.SS_TP, k, i, lb, cfg.n_layers if le is None else le)


def staging_from_logical(content_by_seq, dtype):
    """content_by_seq: list of raw arrays [n_layers_local, 2, heads_local, s, d] ->
    one flat raw staging array in the export/import layout (sequences back to back)."""
    return np.concatenate([np.ascontiguousarray(c).reshape(-1) for c in content_by_seq])


def stored_form(ref, dtype):
    """What the library keeps (and ss_weights_read returns) for a shard whose raw slices are `ref` (name -> storage
    array, matrices in [in, out] orientation): the RMSNorm gains are folded into the rows of the matrices that
    read normalised activations (wq, wk, wv: g1; wg, wu: g2).  Element [h, j] * gain[h] is formed in float32
    (exact for the 16-bit types: the factors have at most 11 significant bits each) and rounded once, to nearest
    even, to the storage type; everything else is kept as it is."""
    def f32(a):
        if dtype == wl.F32:
            return np.asarray(a, dtype=np.float32)
        if dtype == wl.F16:
            return np.ascontiguousarray(a, dtype=np.uint16).view(np.float16).astype(np.float32)
        return wl.bf16_to_f32(a)

    def store(a):
        if dtype == wl.F32:
            return a
        if dtype == wl.F16:
            return a.astype(np.float16).view(np.uint16)
        return wl.bf16_bits(a)

    out = dict(ref)
    for names, gain in ((("wq", "wk", "wv"), "g1"), (("wg", "wu"), "g2")):
        g = f32(ref[gain]).reshape(-1, 1)
        for n in names:
            w = f32(ref[n])
            out[n] = store((w.reshape(g.shape[0], -1) * g).astype(np.float32)).reshape(np.shape(ref[n]))
    return out
