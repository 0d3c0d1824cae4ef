"""CPU oracle: plain float64 numpy statements of what the hot path computes.

TEST INFRASTRUCTURE ONLY.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py import this package.  It shares no code with the
HIP library or its binding and never imports them.

  layer_math  decoder-layer math per tensor-parallel shard, pipeline stages,
              the tiny whole model used by the fp32 configuration
  kv_tier     paged store model, host-tier index formula, swap-out / swap-in
"""
