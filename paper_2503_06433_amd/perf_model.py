"""The paper's analytical performance model (Appendix A; Table 3; the inverse-throughput
equation of Appendix A.3) as plain functions, with MI355X numbers to evaluate it on.

Pure arithmetic on Python floats: nothing here touches the GPU library.  It answers the question the
appendix is written for -- which of tensor, pipeline and data parallelism gives the highest throughput
in the prefill and in the decode stage -- for a node of MI355X GPUs, once with the data-sheet rates and
once with the rates this repository's kernels were measured at (`MI355X_MEASURED`).

Notation as in the appendix: W parameters of one layer, L layers, h_q / h_kv query / kv heads, d head
dimension, b global batch, s sequence length, TP / PP / DP degrees; storage is 2 bytes per element.
Readings: the attention flop counts are printed with d squared; the algorithmic counts (one d) are used,
with the causal half for the prefill.  The all-reduce bandwidth B_ar(TP) is not given as a formula; for
the fully connected xGMI node a reduce-scatter + all-gather moves 2 (TP-1)/TP of the data per GPU over
TP-1 links in parallel, so B_ar(TP) = link_bw * TP / 2 (per byte of activation).
"""
from dataclasses import dataclass


@dataclass
class Model:
    W: float        # parameters of one layer
    L: int
    h_q: int
    h_kv: int
    d: int


@dataclass
class Hardware:
    hbm_bw: float               # bytes/s
    flops: float                # flop/s, dense 16-bit
    link_bw: float              # bytes/s per direction of one inter-GPU link
    mem_bytes: float            # per GPU
    eff_linear_prefill: float = 1.0     # fraction of `flops` the prefill GEMMs reach
    eff_linear_decode: float = 1.0      # fraction of `hbm_bw` the decode GEMMs reach streaming weights
    eff_attn_prefill: float = 1.0       # fraction of `flops`, prefill attention
    eff_attn_decode: float = 1.0        # fraction of `hbm_bw`, decode attention


MI355X_PEAK = Hardware(hbm_bw=8e12, flops=2.5e15, link_bw=153e9 / 2, mem_bytes=288e9)
# Fallback when no bench record is at hand: the fractions of one bench.py run of this repository (configuration 2).
# `hardware_from_bench` replaces them by those of a record, so that the model follows the kernels.
MI355X_MEASURED = Hardware(hbm_bw=8e12, flops=2.5e15, link_bw=153e9 / 2, mem_bytes=288e9, eff_linear_prefill=0.52,
                           eff_linear_decode=0.22, eff_attn_prefill=0.23, eff_attn_decode=0.72)

# which configuration of bench.py measures the kernels of which model shape: (prefill, decode)
BENCH_CONFIG_OF = {"LLaMA-2-7B": ("c2", "c2"), "LLaMA-2-13B": ("c3", "c3"), "LLaMA-3-70B": ("c5", "c4")}


def hardware_from_bench(record, model_name, base=MI355X_PEAK):
    """Hardware whose four efficiencies are the roofline fractions of a bench.py record (the parsed JSON line, or
    the path of a file that holds it, alone or under the key "parsed") for the configurations that measure
    `model_name`'s shapes.  A class the record lacks keeps the fallback value."""
    import dataclasses
    import json
    if isinstance(record, str):
        with open(record) as f:
            record = json.load(f)
    if "parsed" in record and "rooflines" not in record:
        record = record["parsed"]
    roofs = record.get("rooflines", {})
    pre, dec = BENCH_CONFIG_OF[model_name]
    pick = lambda key, fallback: float(roofs[key]["frac"]) if key in roofs and roofs[key].get("frac") else fallback
    fb = MI355X_MEASURED
    return dataclasses.replace(base,
                               eff_linear_prefill=pick(pre + ".prefill_gemms", fb.eff_linear_prefill),
                               eff_attn_prefill=pick(pre + ".prefill_attention", fb.eff_attn_prefill),
                               eff_linear_decode=pick(dec + ".decode_gemms", fb.eff_linear_decode),
                               eff_attn_decode=pick(dec + ".decode_attention", fb.eff_attn_decode))

LLAMA2_7B = Model(W=202.4e6, L=32, h_q=32, h_kv=32, d=128)
LLAMA2_13B = Model(W=317.2e6, L=40, h_q=40, h_kv=40, d=128)
LLAMA3_70B = Model(W=855.6e6, L=80, h_q=64, h_kv=8, d=128)


def allreduce_bw(hw, tp):
    """Bytes of activation all-reduced per second per GPU on a fully connected node (see the header)."""
    return float("inf") if tp <= 1 else hw.link_bw * tp / 2.0


def components(m, hw, stage, b, s, tp=1):
    """The five terms of Table 3 for ONE layer on ONE GPU holding the whole layer (before the parallelism
    scaling of Appendix A.3): dict with dm_lin, comp_lin, dm_attn, comp_attn, nw (seconds)."""
    if stage == "prefill":
        return {
            "dm_lin": 2 * m.W / hw.hbm_bw,
            "comp_lin": 2 * b * m.W * s / (hw.flops * hw.eff_linear_prefill),
            "dm_attn": 2 * b * s * (m.h_q + 2 * m.h_kv) * m.d / hw.hbm_bw,
            "comp_attn": 2 * b * m.h_q * s * s * m.d / (hw.flops * hw.eff_attn_prefill),
            "nw": 4 * b * s * m.h_q * m.d / allreduce_bw(hw, tp),
        }
    if stage == "decode":
        return {
            "dm_lin": 2 * m.W / (hw.hbm_bw * hw.eff_linear_decode),
            "comp_lin": 2 * b * m.W / hw.flops,
            "dm_attn": 4 * b * s * m.h_kv * m.d / (hw.hbm_bw * hw.eff_attn_decode),
            "comp_attn": 4 * b * m.h_q * s * m.d / hw.flops,
            "nw": 4 * b * m.h_q * m.d / allreduce_bw(hw, tp),
        }
    raise ValueError("stage must be 'prefill' or 'decode'")


def layer_time(c):
    """T_L = max(T_dm_lin, T_comp_lin) + max(T_dm_attn, T_comp_attn) + T_nw."""
    return max(c["dm_lin"], c["comp_lin"]) + max(c["dm_attn"], c["comp_attn"]) + c["nw"]


def max_batch(m, hw, s, tp=1, pp=1, dp=1):
    """Largest global batch the KV cache leaves room for: DP (M TP PP - 2 L W) / (4 L h_kv d s)."""
    return dp * (hw.mem_bytes * tp * pp - 2 * m.L * m.W) / (4 * m.L * m.h_kv * m.d * s)


def inv_throughput(m, hw, stage, b, s, tp=1, pp=1, dp=1):
    """Seconds per request of the whole cluster: the inverse-throughput equation of Appendix A.3."""
    c = components(m, hw, stage, b, s, tp)
    g = dp * tp * pp
    return m.L / b * (max(c["dm_lin"] / tp, c["comp_lin"] / g) + max(c["dm_attn"], c["comp_attn"]) / g + c["nw"] / (pp * dp))


def best_strategy(m, hw, stage, b, s, n_gpus):
    """(tp, pp, seconds per request) with tp * pp == n_gpus that minimises inv_throughput, dp = 1."""
    best = None
    for tp in range(1, n_gpus + 1):
        if n_gpus % tp or m.h_kv % tp:
            continue
        t = inv_throughput(m, hw, stage, b, s, tp=tp, pp=n_gpus // tp)
        if best is None or t < best[2]:
            best = (tp, n_gpus // tp, t)
    return best


def request_time(m, hw, n_gpus, s_in, s_out, prefill_tp, decode_tp, host_bw=None, b_prefill=16):
    """Seconds per request of an offline job with prompts of s_in and outputs of s_out tokens on n_gpus GPUs:
    prefill under (TP = prefill_tp, PP = n / prefill_tp), decode under (decode_tp, n / decode_tp), both at the
    batch sizes the model gives them.  When the two strategies differ the job re-shards (paper section 4): per
    request its cache crosses the host link twice (4 L h_kv d s_in bytes each way, swap-out and swap-in), and
    per switch every GPU reloads its weight shard (2 W L / n bytes), amortised over the requests the CPU store
    holds between two switches (section 4.2; `host_bw` bytes/s per GPU, store of 80 GB per GPU as in section 6.1).
    Both movements overlap compute in the method (section 5.2), so this charge is an upper bound."""
    s_dec = s_in + s_out / 2.0
    b_dec = min(max_batch(m, hw, s_in + s_out, tp=decode_tp, pp=n_gpus // decode_tp), 4096.0)
    if b_dec < 1:
        return float("inf")
    t = inv_throughput(m, hw, "prefill", b_prefill, s_in, tp=prefill_tp, pp=n_gpus // prefill_tp)
    t += s_out * inv_throughput(m, hw, "decode", b_dec, s_dec, tp=decode_tp, pp=n_gpus // decode_tp)
    if prefill_tp != decode_tp and host_bw:
        kv_bytes = 4.0 * m.L * m.h_kv * m.d * s_in
        t += 2.0 * kv_bytes / (host_bw * n_gpus)
        per_switch = 2.0 * m.W * m.L / n_gpus / host_bw
        store_requests = max(1.0, 80e9 * n_gpus / kv_bytes)
        t += 2.0 * per_switch / store_requests
    return t


def link_sweep(m, hw, n_gpus, s_in=3000, s_out=300, factors=(0.1, 0.2, 0.5, 1, 2, 5, 10, 20, 50), host_bw=50e9):
    """The sensitivity study of section 6.5 on this model: for inter-GPU links of `factors` times hw.link_bw,
    the best strategy that stays fixed over both stages against the best pair (prefill strategy, decode
    strategy) with re-sharding between them.  Rows: (factor, fixed tp, fixed s/request, prefill tp, decode tp,
    re-sharded s/request, gain = fixed / re-sharded)."""
    import dataclasses
    rows = []
    tps = [tp for tp in range(1, n_gpus + 1) if n_gpus % tp == 0 and m.h_kv % tp == 0]
    for f in factors:
        h = dataclasses.replace(hw, link_bw=hw.link_bw * f)
        fixed = min(((request_time(m, h, n_gpus, s_in, s_out, tp, tp), tp) for tp in tps))
        pair = min(((request_time(m, h, n_gpus, s_in, s_out, a, b, host_bw), a, b) for a in tps for b in tps))
        rows.append((f, fixed[1], fixed[0], pair[1], pair[2], pair[0], fixed[0] / pair[0]))
    return rows


def report(bench=None):
    lines = []
    for name, m, n in (("LLaMA-2-7B", LLAMA2_7B, 2), ("LLaMA-2-13B", LLAMA2_13B, 4), ("LLaMA-3-70B", LLAMA3_70B, 8)):
        measured = hardware_from_bench(bench, name) if bench is not None else MI355X_MEASURED
        for label, hw in (("data-sheet rates", MI355X_PEAK), ("measured kernel rates", measured)):
            s_in, s_dec = 3000, 3100
            b_dec = min(max_batch(m, hw, s_dec, tp=n), 4096.0)
            p = best_strategy(m, hw, "prefill", 16, s_in, n)
            d = best_strategy(m, hw, "decode", b_dec, s_dec, n)
            lines.append("%s on %d GPUs, %s: prefill best TP%d PP%d (%.3f ms/request), decode best TP%d PP%d "
                         "(%.4f ms/request/token at b = %d)" % (name, n, label, p[0], p[1], p[2] * 1e3, d[0], d[1], d[2] * 1e3, b_dec))
    # where the switch between a prefill and a decode strategy pays, against the link bandwidth (section 6.5)
    for name, m, n in (("LLaMA-2-13B", LLAMA2_13B, 4), ("LLaMA-3-70B", LLAMA3_70B, 8)):
        hw = hardware_from_bench(bench, name) if bench is not None else MI355X_MEASURED
        lines.append("%s on %d GPUs, prompts 3000 / outputs 300, measured kernel rates; link = factor x %.0f GB/s per direction:"
                     % (name, n, hw.link_bw / 1e9))
        for f, ftp, ft, ptp, dtp, pt, gain in link_sweep(m, hw, n):
            lines.append("  x%-5g fixed TP%d PP%d %.2f ms/request | prefill TP%d PP%d -> decode TP%d PP%d %.2f ms/request | gain %.3f"
                         % (f, ftp, n // ftp, ft * 1e3, ptp, n // ptp, dtp, n // dtp, pt * 1e3, gain))
    return "\n".join(lines)


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser(description="Appendix A of the paper evaluated for MI355X")
    ap.add_argument("--bench", help="file with a bench.py JSON line (or a driver record holding it under 'parsed'): its "
                                    "roofline fractions replace the built-in efficiencies")
    print(report(ap.parse_args().bench))
