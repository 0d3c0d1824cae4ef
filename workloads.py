"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds no arithmetic of the method: it only draws random numbers,
rounds them to the storage type, and describes the shapes of the five
evaluation configurations.  Both the CPU oracle and the HIP library receive
exactly the values produced here (the oracle as float64 arrays, the library as
raw fp32 / bf16 bits), so that neither side's inputs ever come from the other.

The length distributions stand in for the offline workloads the paper measures
on (a chat-like set with comparable input and output lengths, a summarisation
set with long inputs and short outputs, and constant-length prompts; paper
section 6.1 "Workload" and section 6.5).  None of those datasets' records is
reproduced here: only the shape of the length mix.
"""
from dataclasses import dataclass, field

import numpy as np

F32 = 0
BF16 = 1
F16 = 2          # IEEE half, the paper's own precision (section 6.1)


@dataclass
class ModelCfg:
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    n_layers: int = 1
    vocab: int = 0
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    dtype: int = BF16
    page_size: int = 16

    @property
    def q_dim(self):
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self):
        return self.n_kv_heads * self.head_dim

    def layer_params(self):
        """Number of weight-matrix parameters of one full layer (the paper's W)."""
        H, F = self.hidden, self.ffn
        return H * (self.q_dim + 2 * self.kv_dim) + self.q_dim * H + 3 * H * F


# ---------------------------------------------------------------------------
# storage-type rounding (input preparation only)
# ---------------------------------------------------------------------------
def bf16_bits(x):
    """float32 array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_to_f32(bits):
    """uint16 bf16 bit patterns -> float32 array (exact)."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def quantize(x, dtype):
    """Round x to the storage type; returns (values as float64, raw storage array).

    The float64 values are exactly the numbers the raw bits encode, so the
    oracle and the library start from identical inputs."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == F32:
        return x32.astype(np.float64), x32
    if dtype == F16:
        h = x32.astype(np.float16)                      # numpy rounds to nearest even
        return h.astype(np.float64), h.view(np.uint16)
    bits = bf16_bits(x32)
    return bf16_to_f32(bits).astype(np.float64), bits


def storage_to_f64(raw, dtype):
    if dtype == F32:
        return np.asarray(raw, dtype=np.float32).astype(np.float64)
    if dtype == F16:
        return np.ascontiguousarray(raw, dtype=np.uint16).view(np.float16).astype(np.float64)
    return bf16_to_f32(raw).astype(np.float64)


def round_to_storage(a, dtype):
    """float64 array rounded to the storage type and back (what a cache kept in that type holds)."""
    if dtype == F32:
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    return quantize(np.asarray(a, dtype=np.float32), dtype)[0]


def storage_np_dtype(dtype):
    return np.float32 if dtype == F32 else np.uint16


# ---------------------------------------------------------------------------
# weights
# ---------------------------------------------------------------------------
WEIGHT_NAMES = ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd")


def layer_weight_shapes(cfg):
    H, F = cfg.hidden, cfg.ffn
    return {
        "g1": (H,), "wq": (H, cfg.q_dim), "wk": (H, cfg.kv_dim), "wv": (H, cfg.kv_dim),
        "wo": (cfg.q_dim, H), "g2": (H,), "wg": (H, F), "wu": (H, F), "wd": (F, H),
    }


def make_layer_weights(cfg, seed, std=0.02):
    """One layer's weights: matrices N(0, std), norm gains 1 + N(0, std).

    Returns (values, raw): two dicts keyed by WEIGHT_NAMES; matrices are
    row-major [in_features, out_features]."""
    rng = np.random.default_rng(seed)
    vals, raws = {}, {}
    for name, shape in layer_weight_shapes(cfg).items():
        w = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
        if name in ("g1", "g2"):
            w = w + np.float32(1.0)
        vals[name], raws[name] = quantize(w, cfg.dtype)
    return vals, raws


def make_head_weights(cfg, seed, std=0.02):
    """Embedding table [vocab, H], final norm gain [H], LM head [H, vocab] (untied)."""
    rng = np.random.default_rng(seed)
    out_v, out_r = {}, {}
    for name, shape in (("embed", (cfg.vocab, cfg.hidden)), ("gf", (cfg.hidden,)),
                        ("wlm", (cfg.hidden, cfg.vocab))):
        w = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
        if name == "gf":
            w = w + np.float32(1.0)
        if name == "embed":
            w = w * np.float32(1.0 / std)  # unit-scale activations
        out_v[name], out_r[name] = quantize(w, cfg.dtype)
    return out_v, out_r


def make_activations(shape, seed, dtype, std=1.0):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
    return quantize(x, dtype)


# ---------------------------------------------------------------------------
# length mixes
# ---------------------------------------------------------------------------
def uniform_lengths(n, lo, hi, seed):
    rng = np.random.default_rng(seed)
    return rng.integers(lo, hi + 1, size=n).astype(np.int32)


def lognormal_lengths(n, mu, sigma, lo, hi, seed):
    rng = np.random.default_rng(seed)
    v = np.rint(rng.lognormal(mu, sigma, size=n))
    return np.clip(v, lo, hi).astype(np.int32)


# ---------------------------------------------------------------------------
# the five configurations
# ---------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    cfg: ModelCfg
    k: int = 1                      # shard degree the decode part runs at
    prefill_lens: np.ndarray = None
    decode_kv_lens: np.ndarray = None
    notes: dict = field(default_factory=dict)


def config1():
    cfg = ModelCfg(hidden=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn=688,
                   n_layers=2, vocab=512, dtype=F32)
    return Workload("c1_tiny_fp32", cfg, k=2,
                    prefill_lens=np.full(4, 32, dtype=np.int32),
                    notes={"decode_steps": 8, "seed": 1001})


def config2():
    cfg = ModelCfg(hidden=4096, n_q_heads=32, n_kv_heads=32, head_dim=128, ffn=11008)
    return Workload("c2_llama2_7b_layer", cfg, k=1,
                    prefill_lens=uniform_lengths(16, 512, 2048, 2002),
                    decode_kv_lens=uniform_lengths(256, 512, 2560, 2003))


def config3():
    cfg = ModelCfg(hidden=5120, n_q_heads=40, n_kv_heads=40, head_dim=128, ffn=13824)
    return Workload("c3_llama2_13b_tp4", cfg, k=4,
                    prefill_lens=uniform_lengths(32, 256, 2048, 3002),
                    decode_kv_lens=uniform_lengths(512, 256, 4096, 3003))


def config4():
    cfg = ModelCfg(hidden=8192, n_q_heads=64, n_kv_heads=8, head_dim=128, ffn=28672)
    return Workload("c4_llama3_70b_tp8", cfg, k=8,
                    decode_kv_lens=uniform_lengths(1024, 512, 4096, 4003))


def config5():
    cfg = ModelCfg(hidden=8192, n_q_heads=64, n_kv_heads=8, head_dim=128, ffn=28672,
                   n_layers=10)
    return Workload("c5_llama3_70b_pp8_slice", cfg, k=8,
                    prefill_lens=lognormal_lengths(64, 7.0, 0.6, 128, 4096, 5002),
                    notes={"next_batch_lens": lognormal_lengths(64, 7.0, 0.6, 128, 4096, 5003)})


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


# ---------------------------------------------------------------------------
# large inputs drawn directly in device memory (torch's seeded generator is the
# random source; the values are inputs like any other and are copied to the host
# whenever the oracle needs them)
# ---------------------------------------------------------------------------
def device_normal(shape, seed, dtype, std=1.0, device="cuda"):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    t = torch.empty(shape, device=device, dtype={F32: torch.float32, BF16: torch.bfloat16, F16: torch.float16}[dtype])
    t.normal_(0.0, std, generator=g)
    return t


def device_layer_weights(cfg, seed, std=0.02, device="cuda"):
    """Same shapes and distributions as make_layer_weights, drawn on the device."""
    out = {}
    for j, (name, shape) in enumerate(layer_weight_shapes(cfg).items()):
        w = device_normal(shape, seed * 16 + j, cfg.dtype, std, device)
        if name in ("g1", "g2"):
            w += 1.0
        out[name] = w
    return out
