"""skv_decode_step_noalloc (the decode step on the library's static device scratch, for callers that cannot allocate)
against skv_decode_step with a context, through the C ABI: the selection bit for bit and out / lse bit for bit (both
run the same kernels in the same launch shapes; only the workspace differs), on two calls in a row, the second with a
smaller input, and on a small ragged batch.  Collected last on purpose."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2504_00970_amd as skv
from paper_2504_00970_amd import binding
from workload import gen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def U():
    import gpu_util
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return gpu_util


def _both_ways(U, wl, seed, sentinel):
    """One layer of a ragged batch through skv_decode_step (context) and skv_decode_step_noalloc; returns both results."""
    inp = gen.ragged_inputs(wl, seed=seed, device=U.DEV, resident_layers=1)
    B, H, Hq, D = wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.head_dim
    T_total, S_total = int(inp.cu_tok[-1]), int(inp.cu_sent[-1])
    budget = int(inp.budget.max())
    desc = skv.Desc(n_layers=1, n_q_heads=Hq, n_kv_heads=H, kv_dtype=skv.dtype_code(wl.torch_dtype), max_tokens=T_total,
                    max_sentences=S_total, max_budget=budget, max_batch=B)
    ctx = skv.Context(desc)
    sv = torch.zeros(1, H, S_total, D, device=U.DEV)
    ctx.build_semvec(inp.K, U.i32(gen.offsets_of(inp.sent_len)), S_total, sv)
    d = [U.i32(x) for x in (inp.cu_tok, inp.cu_sent, inp.sent_off, inp.sent_len, inp.budget)]
    q = inp.q[0]
    res = []
    for how in ("ctx", "noalloc"):
        out = torch.full((B, Hq, D), sentinel, device=U.DEV)
        lse = torch.full((B, Hq), sentinel, device=U.DEV)
        tok_idx = U.empty_i32(B, H, budget, fill=-1)
        n_tok = U.empty_i32(B, H, fill=-1)
        if how == "ctx":
            ctx.decode_step(0, B, q, q, inp.K, inp.V, T_total, sv, S_total, *d, out, lse, tok_idx, n_tok)
        else:
            skv.decode_step_noalloc(desc, 0, B, q, q, inp.K, inp.V, T_total, sv, S_total, *d, out, lse, tok_idx, n_tok)
        torch.cuda.synchronize()
        res.append((out, lse, tok_idx, n_tok))
    return res


def _same(a, b, exact):
    out_a, lse_a, idx_a, n_a = a
    out_b, lse_b, idx_b, n_b = b
    assert torch.equal(n_a, n_b) and torch.equal(idx_a, idx_b)           # selection bit for bit
    assert bool((n_a >= 0).all())
    if exact:
        assert torch.equal(out_a, out_b) and torch.equal(lse_a, lse_b)
    else:                                                                  # streaming kernel: tiles in arrival order
        assert float((out_a - out_b).abs().max()) <= 2e-2 / 4
        fin = torch.isfinite(lse_a)
        assert torch.equal(fin, torch.isfinite(lse_b)) and float((lse_a[fin] - lse_b[fin]).abs().max()) <= 2e-2 / 4


def test_noalloc_step_equals_context_step_two_calls_second_smaller(U):
    print("noalloc: cfg1 shapes, 12000 tokens, budget 1024, then 3000 tokens, budget 200", flush=True)
    big = gen.CFG1.scaled(n_layers=1, batch=1, t_range=(12000, 12000), budgets=(1024,))
    a, b = _both_ways(U, big, seed=5, sentinel=3.0)
    _same(a, b, exact=True)
    small = gen.CFG1.scaled(n_layers=1, batch=1, t_range=(3000, 3000), budgets=(200,))
    a, b = _both_ways(U, small, seed=6, sentinel=4.0)
    _same(a, b, exact=True)
    print("noalloc: fp32 pool, then a ragged bf16 batch of 3", flush=True)
    a, b = _both_ways(U, gen.CFG0.scaled(n_layers=1, batch=1, t_range=(4096, 4096), budgets=(512,)), seed=7, sentinel=5.0)
    _same(a, b, exact=True)
    a, b = _both_ways(U, gen.CFG4.scaled(n_layers=1, batch=3, t_range=(500, 4000), budgets=(512,)), seed=8, sentinel=6.0)
    _same(a, b, exact=True)
    print("noalloc: batch of 12 on the streaming kernel, fp32 batch of 9 through tok_idx", flush=True)
    a, b = _both_ways(U, gen.CFG4.scaled(n_layers=1, n_q_heads=8, batch=12, t_range=(900, 5000), budgets=(1500,)), seed=9,
                      sentinel=7.0)
    _same(a, b, exact=False)
    a, b = _both_ways(U, gen.CFG4.scaled(n_layers=1, n_q_heads=32, batch=9, t_range=(200, 3000), budgets=(700,), dtype="f32"),
                      seed=10, sentinel=8.0)
    _same(a, b, exact=True)


def test_noalloc_step_rejects_what_does_not_fit_the_static_scratch(U):
    lib = binding._lib()
    wl = gen.CFG4
    desc = binding._Desc(1, 64, 8, 128, skv.SKV_BF16, 600000, 24000, 2048, 16, skv.SKV_F32)     # 16 MB of split-K partials
    dummy = torch.zeros(64, device=U.DEV)
    p = ctypes.c_void_p(dummy.data_ptr())
    rc = lib.skv_decode_step_noalloc(ctypes.byref(desc), None, 0, 16, p, p, p, p, 600000, p, 24000, p, p, p, p, p, p, None,
                                     None, None)
    assert rc == skv.SKV_ECAPACITY
    bad = binding._Desc(1, 64, 8, 64, skv.SKV_BF16, 100, 10, 16, 1, skv.SKV_F32)                 # head_dim 64
    assert lib.skv_decode_step_noalloc(ctypes.byref(bad), None, 0, 1, p, p, p, p, 100, p, 10, p, p, p, p, p, p, None, None,
                                       None) == skv.SKV_EINVAL
    assert lib.skv_decode_step_noalloc(None, None, 0, 1, p, p, p, p, 100, p, 10, p, p, p, p, p, p, None, None, None) == skv.SKV_EINVAL
