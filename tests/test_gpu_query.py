"""GPU parity of skv_query_update (Sec. 4.2 "Sentence-level query aggregation", Eq. 2; Alg. 1 decoding phase)
against the oracle's literal sentence cache Q_s.

Gate: bit-exact.  Both sides add the same float values in the order of generation, divide once (IEEE) and
round once to the storage type, so q-bar, the running sum and the count must agree bit for bit.
"""
import numpy as np
import pytest
import torch

from workload import gen

pytestmark = pytest.mark.gpu

TERM, OTHER, VOCAB = 7, 3, 64


@pytest.fixture(scope="module")
def U():
    import gpu_util
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return gpu_util


def _bitmap():
    bm = np.zeros(2, dtype=np.uint32)
    bm[0] = 1 << TERM
    return bm


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("Hq,B", [(32, 1), (8, 3), (64, 5)])
def test_query_update_bit_exact_over_a_generated_run(U, oracle32, dtype, Hq, B):
    print("query_update", dtype, "Hq", Hq, "B", B, flush=True)
    D, n_steps = 128, 48
    per = Hq * D
    wl = gen.CFG0.scaled(n_layers=1, n_q_heads=Hq, n_kv_heads=8 if Hq % 8 == 0 else 1, dtype=dtype)
    ctx = U.make_ctx(wl, 16, 4, 16, batch=B)
    q = gen.queries(n_steps * B, Hq, D, wl.torch_dtype, seed=11 + Hq + B).view(n_steps, B, Hq, D)
    rng = np.random.default_rng(Hq * 100 + B)
    is_term = rng.random((n_steps, B)) < 0.2
    is_term[5:7, 0] = True                                        # a run of terminators in sequence 0
    is_term[n_steps - 1, B - 1] = True                            # the run ends on a boundary for the last sequence
    tok = np.where(is_term, TERM, OTHER).astype(np.int32)
    tok[3, 0] = VOCAB + TERM                                      # outside the vocabulary: never a terminator
    tok[4, 0] = -1
    is_term[3, 0] = is_term[4, 0] = False

    d_bm = torch.as_tensor(_bitmap().view(np.int32)).to(U.DEV)
    q_sum = torch.zeros(B, Hq, D, dtype=torch.float32, device=U.DEV)
    q_cnt = torch.zeros(max(B, 4), dtype=torch.int32, device=U.DEV)
    q_bar = torch.zeros(B, Hq, D, dtype=wl.torch_dtype, device=U.DEV)
    caches = [oracle32.query_cache(per, n_steps + 1) for _ in range(B)]
    qd = q.to(U.DEV)
    resets = 0
    for t in range(n_steps):
        ctx.query_update(B, qd[t], U.i32(tok[t]), d_bm, VOCAB, q_sum, q_cnt, q_bar)
        torch.cuda.synchronize()
        got = U.np_of(q_bar)
        cnt = q_cnt.cpu().numpy()
        for b in range(B):
            _, want = caches[b].step(gen.to_numpy(q[t, b]).reshape(-1), int(tok[t, b]), _bitmap(), VOCAB)
            assert np.array_equal(got[b].reshape(-1).view(want.dtype), want), (t, b)
            assert cnt[b] == len(caches[b])
            resets += int(is_term[t, b])
        live = np.array([len(c) for c in caches]) > 0
        s = q_sum.cpu().numpy().reshape(B, -1)
        assert np.all(s[~live] == 0)                              # cleared state after a boundary
    assert resets >= B


def test_query_update_feeds_decode_step(U, oracle32):
    """q-bar from skv_query_update handed to skv_decode_step as q_score: the step's selection equals the oracle's
    selection from the oracle's own q-bar (up to documented score ties), end to end."""
    wl = gen.CFG0.scaled(n_layers=1)
    inp = gen.decode_inputs(wl, seed=3, device=U.DEV)
    S, T, L = len(inp.lengths), wl.n_tokens, 0
    Hq, H, D = wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    budget = wl.budgets[0]
    ctx = U.make_ctx(wl, T, S, budget)
    sv = torch.zeros(1, H, S, D, dtype=torch.float32, device=U.DEV)
    ctx.build_semvec(inp.K, U.i32(inp.sent_off), S, sv)
    qs = gen.queries(4, Hq, D, wl.torch_dtype, seed=77, device=U.DEV)
    d_bm = torch.as_tensor(_bitmap().view(np.int32)).to(U.DEV)
    q_sum = torch.zeros(1, Hq, D, dtype=torch.float32, device=U.DEV)
    q_cnt = torch.zeros(4, dtype=torch.int32, device=U.DEV)
    q_bar = torch.zeros(1, Hq, D, dtype=wl.torch_dtype, device=U.DEV)
    cache = oracle32.query_cache(Hq * D, 8)
    out = torch.zeros(Hq, D, dtype=torch.float32, device=U.DEV)
    tok_idx = U.empty_i32(H, budget, fill=-1)
    n_tok = U.empty_i32(max(H, 4), fill=-5)
    K, V = gen.to_numpy(inp.K[L]), gen.to_numpy(inp.V[L])
    sv_np = sv.cpu().numpy()[0]
    n_ties = 0
    for t in range(4):
        print("query_update -> decode_step, token", t, flush=True)
        ctx.query_update(1, qs[t], U.i32([OTHER]), d_bm, VOCAB, q_sum, q_cnt, q_bar)
        ctx.decode_step(L, 1, q_bar[0], qs[t], inp.K, inp.V, T, sv, S, U.i32([0, T]), U.i32([0, S]),
                        U.i32(inp.sent_off), U.i32(inp.lengths), U.i32([budget]), out, None, tok_idx, n_tok)
        torch.cuda.synchronize()
        _, qbar_ref = cache.step(U.np_of(qs[t]).reshape(-1), OTHER, _bitmap(), VOCAB)
        assert np.array_equal(U.np_of(q_bar[0]).reshape(-1).view(qbar_ref.dtype), qbar_ref)
        g_n, g_idx = n_tok.cpu().numpy()[:H], tok_idx.cpu().numpy()
        # the GPU's mean query is bit-exact (checked above), so both sides rank with the same query; the selection gate
        # is the usual one: oracle rule on the GPU's scores bit for bit, documented ties only against the oracle's scores
        sc = oracle32.score(qbar_ref.reshape(Hq, D), sv_np)
        sc_gpu = U.gpu_scores(ctx, L, q_bar[0], sv, S, H)
        n_ties += U.check_selection(oracle32, sc, sc_gpu, inp.sent_off, inp.lengths, budget, g_idx, g_n, what=f"token {t}")
        tok_g = np.where(g_idx < 0, 0, g_idx).astype(np.int32)
        o_ref, _ = oracle32.attend(U.np_of(qs[t]), oracle32.gather(K, tok_g, g_n.astype(np.int32)),
                                   oracle32.gather(V, tok_g, g_n.astype(np.int32)), g_n.astype(np.int32))
        tol = 1e-4 if wl.dtype == "f32" else 2e-2
        assert np.abs(out.cpu().numpy() - o_ref).max() <= tol
    assert n_ties <= U.MAX_TIES_PER_TEST, n_ties
