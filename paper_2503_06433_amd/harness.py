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


def pp_desc(cfg, lb=0, le=None):
    return ss.ShardDesc(ss.SS_PP, 1, 0, lb, cfg.n_layers if le is None else le)


def tp_desc(cfg, k, i, lb=0, le=None):
    return ss.ShardDesc(ss.SS_TP, k, i, lb, cfg.n_layers if le is None else le)


def staging_from_logical(content_by_seq, dtype):
    """content_by_seq: list of raw arrays [n_layers_local, 2, heads_local, s, d] ->
    one flat raw staging array in the export/import layout (sequences back to back)."""
    return np.concatenate([np.ascontiguousarray(c).reshape(-1) for c in content_by_seq])
