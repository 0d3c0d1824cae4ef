"""The entry point that allocates nothing (ss_lm_head_noalloc, for callers that cannot call hipMalloc) against
the entry point it is a variant of (ss_lm_head), through the C ABI: two calls in a row on one GPU, the second
with a smaller input, both sharing the GPU's fixed scratch array; then the size limit."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import layer_math as lm

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2503_06433_amd as ss
    from paper_2503_06433_amd.harness import make_context, to_device, rel_err, tol


@pytest.mark.parametrize("dtype,hidden,vocab,rows", [(wl.BF16, 1024, 2048, (70, 9)), (wl.BF16, 512, 1024, (300, 40)),
                                                     (wl.F32, 256, 512, (33, 4))])
def test_lm_head_noalloc_equals_lm_head_on_two_calls_in_a_row(dtype, hidden, vocab, rows):
    cfg = wl.ModelCfg(hidden=hidden, n_q_heads=4, n_kv_heads=4, head_dim=128 if dtype != wl.F32 else 64, ffn=1024,
                      n_layers=1, vocab=vocab, dtype=dtype)
    hv, hr = wl.make_head_weights(cfg, 77)
    ctx = make_context(cfg, pages=4)
    ctx.load_head(hr["embed"], hr["gf"], hr["wlm"])
    for j, n in enumerate(rows):                          # the second call is smaller and finds the first one's leftovers
        xv, xr = wl.make_activations((n, hidden), 80 + j, dtype)
        x = to_device(xr, dtype)
        want = torch.empty((n, vocab), device="cuda", dtype=torch.float32)
        ctx.lm_head(x, n, want)
        torch.cuda.synchronize()
        got = torch.full((n, vocab), float("nan"), device="cuda", dtype=torch.float32)
        ctx.lm_head_noalloc(x, n, got)
        torch.cuda.synchronize()
        g, w = got.cpu().numpy(), want.cpu().numpy()
        assert np.isfinite(g).all()
        # same kernels on the same inputs; only the number of split-K parts (fp32 summation order) may differ
        assert rel_err(g, w) <= 1e-5, "call %d (%d rows)" % (j, n)
        assert rel_err(g, lm.lm_logits(cfg, hv, xv)) <= tol(dtype)
    ctx.destroy()


def test_lm_head_noalloc_refuses_sizes_beyond_the_fixed_scratch():
    cfg = wl.ModelCfg(hidden=4096, n_q_heads=4, n_kv_heads=4, head_dim=128, ffn=1024, n_layers=1, vocab=256, dtype=wl.BF16)
    _, hr = wl.make_head_weights(cfg, 78)
    ctx = make_context(cfg, pages=4)
    ctx.load_head(hr["embed"], hr["gf"], hr["wlm"])
    n_ok, n_big = 1024, 1025                               # 1024 rows * 4096 * 2 B = 8 MiB exactly
    x = torch.zeros((n_big, cfg.hidden), device="cuda", dtype=torch.bfloat16)
    out = torch.empty((n_big, cfg.vocab), device="cuda", dtype=torch.float32)
    ctx.lm_head_noalloc(x, n_ok, out)
    torch.cuda.synchronize()
    with pytest.raises(ss.SeesawError) as e:
        ctx.lm_head_noalloc(x, n_big, out)
    assert e.value.code == ss.SS_EINVAL and "fixed limit" in str(e.value)
    ctx.destroy()
