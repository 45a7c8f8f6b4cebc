"""Error behaviour of the C entry points on a live context: every documented SKV_EINVAL / SKV_ECAPACITY condition is
reported by the host-side checks, before any kernel is launched (so none of these calls touches device memory)."""
import ctypes

import pytest
import torch

import paper_2504_00970_amd as skv
from paper_2504_00970_amd import binding
from workload import gen

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def env():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    ctx = skv.Context(skv.Desc(n_layers=2, n_q_heads=32, n_kv_heads=8, kv_dtype=skv.SKV_BF16, max_tokens=1000, max_sentences=50,
                               max_budget=64, max_batch=2))
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device=DEV)
    return ctx, binding._lib(), buf.data_ptr()


def test_query_update_errors(env):
    ctx, lib, p = env
    h = ctx._h
    assert lib.skv_query_update(h, 0, p, p, p, 64, p, p, p) == skv.SKV_EINVAL          # B < 1
    assert lib.skv_query_update(h, 1, p, p, p, 0, p, p, p) == skv.SKV_EINVAL           # vocab <= 0
    assert lib.skv_query_update(h, 1, None, p, p, 64, p, p, p) == skv.SKV_EINVAL       # null pointer
    assert lib.skv_query_update(h, 1, p + 4, p, p, 64, p, p, p) == skv.SKV_EINVAL      # misaligned pointer
    assert lib.skv_query_update(h, 3, p, p, p, 64, p, p, p) == skv.SKV_ECAPACITY       # B > max_batch


def test_token_importance_errors(env):
    ctx, lib, p = env
    h = ctx._h
    need = lib.skv_token_importance_work_bytes(h, 1000, 32)
    assert need > 0
    assert lib.skv_token_importance_work_bytes(h, 1000, 0) == -1
    assert lib.skv_token_importance_work_bytes(h, 32, 32) == -1                            # no token before the window
    assert lib.skv_token_importance_work_bytes(h, 1000, 65) == -1                          # G * N > 256
    assert lib.skv_token_importance(h, p, p, 1000, 0, p, p, need) == skv.SKV_EINVAL
    assert lib.skv_token_importance(h, p, p, 32, 32, p, p, need) == skv.SKV_EINVAL
    assert lib.skv_token_importance(h, p, p, 1000, 65, p, p, 1 << 20) == skv.SKV_ECAPACITY
    assert lib.skv_token_importance(h, p, p, 1001, 32, p, p, 1 << 20) == skv.SKV_ECAPACITY   # T > max_tokens
    assert lib.skv_token_importance(h, p, p, 1000, 32, p, p, need - 1) == skv.SKV_EINVAL      # scratch too small
    assert lib.skv_token_importance(h, p, None, 1000, 32, p, p, need) == skv.SKV_EINVAL
    assert lib.skv_token_importance(h, p, p, 1000, 32, p, None, need) == skv.SKV_EINVAL


def test_retain_compact_semvec_layers_errors(env):
    ctx, lib, p = env
    h = ctx._h
    assert lib.skv_retain(h, p, 0, 4, p, 10, p, p, p, p) == skv.SKV_EINVAL                # Tp < 1
    assert lib.skv_retain(h, p, 100, -1, p, 10, p, p, p, p) == skv.SKV_EINVAL             # k < 0
    assert lib.skv_retain(h, p, 100, 4, p, 0, p, p, p, p) == skv.SKV_EINVAL               # S < 1
    assert lib.skv_retain(h, p, 100, 4, None, 10, p, p, p, p) == skv.SKV_EINVAL
    assert lib.skv_retain(h, p, 1001, 4, p, 10, p, p, p, p) == skv.SKV_ECAPACITY
    assert lib.skv_retain(h, p, 100, 4, p, 51, p, p, p, p) == skv.SKV_ECAPACITY
    assert lib.skv_compact_pool(h, p, p, 0, p, 4, p, p, p) == skv.SKV_EINVAL
    assert lib.skv_compact_pool(h, p, p, 100, p, -1, p, p, p) == skv.SKV_EINVAL
    assert lib.skv_compact_pool(h, p, None, 100, p, 4, p, p, p) == skv.SKV_EINVAL
    assert lib.skv_compact_pool(h, p, p, 1001, p, 4, p, p, p) == skv.SKV_ECAPACITY
    assert lib.skv_compact_pool(h, None, None, 100, None, 0, None, None, None) == skv.SKV_OK    # k == 0: nothing to copy
    assert lib.skv_build_semvec_layers(h, p, -1, p, 4, p) == skv.SKV_EINVAL
    assert lib.skv_build_semvec_layers(h, p, 100, None, 4, p) == skv.SKV_EINVAL
    assert lib.skv_build_semvec_layers(h, p, 100, p, 51, p) == skv.SKV_ECAPACITY
    assert lib.skv_build_semvec_layers(h, None, 100, None, 0, None) == skv.SKV_OK               # S == 0 is a no-op


def test_merge_lse_errors(env):
    ctx, lib, p = env
    h = ctx._h
    assert lib.skv_merge_lse(h, 0, p, p, p, p, p, p) == skv.SKV_EINVAL
    assert lib.skv_merge_lse(h, 8, p, p, None, p, p, p) == skv.SKV_EINVAL
    assert lib.skv_merge_lse(h, 8, p, p, p, p, p, p + 4) == skv.SKV_EINVAL                 # misaligned optional output
    assert lib.skv_merge_lse(h, 2 * 32 + 1, p, p, p, p, p, p) == skv.SKV_ECAPACITY         # more heads than max_batch * Hq


def test_decode_entry_point_errors(env):
    ctx, lib, p = env
    h = ctx._h
    assert lib.skv_score(h, 2, p, p, 10, p) == skv.SKV_EINVAL                              # layer out of range
    assert lib.skv_score(h, 0, p, p, 51, p) == skv.SKV_ECAPACITY
    assert lib.skv_select(h, p, p, p, 10, 65, p, p, p, p) == skv.SKV_ECAPACITY             # budget > max_budget
    assert lib.skv_gather(h, 0, p, p, 100, 2, p, p, 16, p, p) == skv.SKV_EINVAL            # pool_in_host not 0/1
    assert lib.skv_attend(h, p, p, p, p, 65, p, None) == skv.SKV_ECAPACITY
    assert lib.skv_decode_step(h, 0, 3, p, p, p, p, 100, p, 10, p, p, p, p, p, p, None, None, None) == skv.SKV_ECAPACITY
    assert lib.skv_decode_step(h, 0, 1, p, p, p, p, 100, p, 10, None, p, p, p, p, p, None, None, None) == skv.SKV_EINVAL


def test_single_launch_step_gives_up_cleanly_and_recovers():
    """The single-launch decode step with a wait limit of zero: every block that waits for another block's words gives up
    at once (the host forces the condition; the kernel itself ends normally), the outputs are NaN, the next step on the
    context reports SKV_EHIP, and skv_set_wait_limit clears the condition: the same step then equals a fresh context's."""
    import numpy as np
    from workload import gen
    import gpu_util as U
    wl = gen.CFG1.scaled(n_layers=1, batch=1, t_range=(6000, 6000), budgets=(512,))
    inp = gen.ragged_inputs(wl, seed=11, device=DEV, resident_layers=1)
    H, Hq, D = wl.n_kv_heads, wl.n_q_heads, wl.head_dim
    T, S = int(inp.cu_tok[-1]), int(inp.cu_sent[-1])
    d = [U.i32(x) for x in (inp.cu_tok, inp.cu_sent, inp.sent_off, inp.sent_len, inp.budget)]

    def fresh():
        c = U.make_ctx(wl, T, S, 512)
        sv = torch.zeros(1, H, S, D, device=DEV)
        c.build_semvec(inp.K, U.i32(gen.offsets_of(inp.sent_len)), S, sv)
        return c, sv

    def step(c, sv, out, n_tok):
        c.decode_step(0, 1, inp.q[0], inp.q[0], inp.K, inp.V, T, sv, S, *d, out, None, None, n_tok)
        torch.cuda.synchronize()

    ref_ctx, sv = fresh()
    ref, ref_n = torch.zeros(1, Hq, D, device=DEV), U.empty_i32(1, H, fill=-1)
    step(ref_ctx, sv, ref, ref_n)
    assert bool(torch.isfinite(ref).all())

    ctx, sv2 = fresh()
    ctx.set_wait_limit(0)
    out, n_tok = torch.zeros(1, Hq, D, device=DEV), U.empty_i32(1, H, fill=-1)
    print("decode step with a wait limit of zero", flush=True)
    step(ctx, sv2, out, n_tok)                               # runs to its end; every waiting block gave up
    assert bool(torch.isnan(out).all())
    with pytest.raises(skv.SkvError) as e:                   # the give-up is reported by the next call
        step(ctx, sv2, out, n_tok)
    assert e.value.status == skv.SKV_EHIP
    ctx.set_wait_limit(200000)                               # clears the condition
    step(ctx, sv2, out, n_tok)
    assert torch.equal(out, ref) and torch.equal(n_tok, ref_n)
    step(ctx, sv2, out, n_tok)
    assert torch.equal(out, ref)
