"""GPU parity of the prefill-side token retention (Sec. 4.1; App. "Effect of Sentence Length") against the oracle:
skv_token_importance, skv_retain, skv_compact_pool, skv_build_semvec_layers, and the decode step on the retained pool.

Gates: importance within 2e-4 relative (+1e-7 of the largest value): both sides form the same exact bf16 products
(fp32 inputs: products exact to 2^-23) and differ in summation order and in exp2 vs exp; the retained set must equal
the oracle's rule applied to the GPU's own importance bit for bit, and may differ from the oracle's end-to-end set only
in tokens whose oracle importance is within 5e-4 relative of the cut ("documented tie"); offsets, lengths and compacted
rows bit-exact; decode on the retained pool to the usual attention tolerance.
"""
import numpy as np
import pytest
import torch

from workload import gen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def U():
    import gpu_util
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return gpu_util


def _say(*a):
    print(*a, flush=True)


def _gpu_importance(U, ctx, q_obs, K, T, N):
    L = K.shape[0]
    alpha = torch.full((L, T - N), -5.0, dtype=torch.float32, device=U.DEV)
    nbytes = ctx.token_importance_work_bytes(T, N)
    assert nbytes > 0
    work = torch.empty(nbytes, dtype=torch.uint8, device=U.DEV)
    ctx.token_importance(q_obs, K, T, N, alpha, work)
    torch.cuda.synchronize()
    return alpha


IMP_CASES = [("bf16", 32, 8, 32, 1500), ("bf16", 8, 8, 32, 700), ("bf16", 16, 8, 32, 513), ("bf16", 64, 8, 32, 1100),
             ("bf16", 32, 8, 7, 530), ("bf16", 32, 8, 1, 300), ("f32", 32, 8, 16, 600), ("f32", 8, 2, 32, 257)]


@pytest.mark.parametrize("dtype,Hq,H,N,T", IMP_CASES, ids=[f"{c[0]}-Hq{c[1]}-H{c[2]}-N{c[3]}-T{c[4]}" for c in IMP_CASES])
def test_token_importance_matches_oracle(U, oracle32, dtype, Hq, H, N, T):
    _say("importance", dtype, Hq, H, N, T)
    L = 2
    wl = gen.CFG3.scaled(n_layers=L, n_q_heads=Hq, n_kv_heads=H, n_tokens=T, dtype=dtype, len_dist=("uniform", 5, 30))
    lens = gen.sentence_lengths(wl.len_dist, T, seed=3)
    K = torch.stack([gen.kv_layer(lens, H, 128, wl.torch_dtype, 3, l)[0] for l in range(L)]).to(U.DEV)
    q_obs = gen.queries(L * Hq, N, 128, wl.torch_dtype, seed=4, device=U.DEV).view(L, Hq, N, 128)
    ctx = U.make_ctx(wl, T, len(lens), 16)
    alpha = _gpu_importance(U, ctx, q_obs, K, T, N).cpu().numpy()
    for l in range(L):
        ref = oracle32.token_importance(U.np_of(q_obs[l]), U.np_of(K[l]))
        err = np.abs(alpha[l] - ref)
        assert np.all(err <= 2e-4 * ref + 1e-7 * ref.max()), (l, float((err / (ref + 1e-30)).max()))
        assert np.all(alpha[l] >= 0)


FULL_IMP_CASES = [("bf16", 32, 8, 32, 32768), ("f32", 32, 8, 32, 32768), ("bf16", 8, 2, 32, 40100), ("f32", 4, 1, 32, 70001)]


@pytest.mark.parametrize("dtype,Hq,H,N,T", FULL_IMP_CASES, ids=[f"{c[0]}-Hq{c[1]}-H{c[2]}-N{c[3]}-T{c[4]}" for c in FULL_IMP_CASES])
def test_token_importance_and_retention_at_benchmark_size(U, oracle32, dtype, Hq, H, N, T):
    """The size the retention benchmark times (32768 tokens, 32/8 heads, a 32-token window: 64 key chunks of 512 per
    head) and prompts beyond it, where the per-row combine walks its chunks in several strides of 64 (40100 tokens: 79
    chunks; 70001: 137) and most sweeps lie wholly before the window (no masking): one layer against the oracle, then
    the k = 4096 best tokens by the oracle's rule on the GPU's own importance, bit for bit."""
    _say("importance at size", dtype, Hq, H, N, T)
    wl = gen.CFG3.scaled(n_layers=1, n_q_heads=Hq, n_kv_heads=H, n_tokens=T, dtype=dtype)
    lens = gen.sentence_lengths(wl.len_dist, T, seed=5)
    K = gen.kv_layer(lens, H, 128, wl.torch_dtype, 5, 0)[0][None].to(U.DEV)
    q_obs = gen.queries(Hq, N, 128, wl.torch_dtype, seed=6, device=U.DEV).view(1, Hq, N, 128)
    S = len(lens)
    ctx = U.make_ctx(wl, T, S, 16)
    alpha_dev = _gpu_importance(U, ctx, q_obs, K, T, N)
    alpha = alpha_dev.cpu().numpy()
    ref = oracle32.token_importance(U.np_of(q_obs[0]), U.np_of(K[0]))
    err = np.abs(alpha[0] - ref)
    assert np.all(err <= 2e-4 * ref + 1e-7 * ref.max()), float((err / (ref + 1e-30)).max())
    assert np.all(alpha[0] >= 0)
    k, Tp = 4096, T - N
    seg = np.repeat(np.arange(S), lens).astype(np.int32)[:T]
    keep, n_keep, off, ln = _gpu_retain(U, ctx, alpha_dev, k, seg, S)
    want_keep, want_off, want_len = oracle32.retain(alpha[0], k, seg, S)
    assert n_keep[0] == len(want_keep) == min(k, Tp)
    assert np.array_equal(keep[0, :n_keep[0]], want_keep)
    assert np.array_equal(off[0], want_off) and np.array_equal(ln[0], want_len)
    # end to end against the oracle's own importance: the two sets may differ only in tokens at the cut
    ref_keep, _, _ = oracle32.retain(ref, k, seg, S)
    diff = np.setxor1d(want_keep, ref_keep)
    if len(diff):
        cut = np.sort(ref)[::-1][k - 1]
        _say(f"  retained sets differ in {len(diff)} tokens at the cut")
        assert np.all(np.abs(ref[diff] - cut) <= 5e-4 * cut), float(np.abs(ref[diff] - cut).max() / cut)


def _gpu_retain(U, ctx, alpha_dev, k, seg_id, S):
    L, Tp = alpha_dev.shape
    keep = U.empty_i32(L, max(k, 1), fill=-9)
    n_keep = U.empty_i32(max(L, 4), fill=-9)
    off = U.empty_i32(L, S + 1, fill=-9)
    ln = U.empty_i32(L, S, fill=-9)
    ctx.retain(alpha_dev, Tp, k, U.i32(seg_id), S, keep, n_keep, off, ln)
    torch.cuda.synchronize()
    return keep.cpu().numpy(), n_keep.cpu().numpy()[:L], off.cpu().numpy(), ln.cpu().numpy()


@pytest.mark.parametrize("Tp", [1, 2, 63, 1023, 1024, 1025, 5000, 40001])
def test_retain_bit_exact(U, oracle32, Tp):
    _say("retain Tp", Tp)
    L = 3
    rng = np.random.default_rng(Tp)
    alpha = rng.random((L, Tp)).astype(np.float32)
    alpha[1] = rng.choice(np.array([0.0, 0.125, 0.5, 2.0], np.float32), size=Tp)        # many exact ties
    alpha[2, rng.integers(0, Tp, max(Tp // 50, 1))] = np.nan
    alpha[2, rng.integers(0, Tp, max(Tp // 50, 1))] = -0.0
    lens = gen.sentence_lengths(("uniform", 1, 40), Tp + 8, seed=Tp)
    seg = np.repeat(np.arange(len(lens)), lens).astype(np.int32)
    S = len(lens)
    wl = gen.CFG3.scaled(n_layers=L)
    ctx = U.make_ctx(wl, Tp + 8, S, 16)
    a_dev = torch.from_numpy(alpha).to(U.DEV)
    for k in sorted({0, 1, Tp // 7, Tp // 2, Tp - 1, Tp, Tp + 3}):
        if k < 0:
            continue
        keep, n_keep, off, ln = _gpu_retain(U, ctx, a_dev, k, seg, S)
        for l in range(L):
            want_keep, want_off, want_len = oracle32.retain(alpha[l], k, seg, S)
            assert n_keep[l] == len(want_keep) == min(k, Tp)
            assert np.array_equal(keep[l, :n_keep[l]], want_keep), (k, l)
            assert np.all(keep[l, n_keep[l]:] == -9)                                       # nothing written past n_keep
            assert np.array_equal(off[l], want_off) and np.array_equal(ln[l], want_len), (k, l)


@pytest.mark.parametrize("S", [50, 3000, 7000])
def test_select_ignores_buckets_without_tokens(U, oracle32, S):
    """Zero-length buckets (a retained pool has them) are never listed, in both the register and the re-read path of
    the selection (S above 6144 takes the latter)."""
    _say("select with empty buckets, S", S)
    rng = np.random.default_rng(S)
    H = 8
    lens = rng.integers(0, 6, size=S).astype(np.int32)
    lens[rng.integers(0, S, S // 3)] = 0
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(off[-1])
    score = rng.standard_normal((H, S)).astype(np.float32)
    score[0, lens == 0] = 50.0                                        # empty buckets at the very top of a ranking
    score[1] = np.round(score[1] * 2) / 2                             # ties
    wl = gen.CFG1.scaled(n_layers=1)
    for budget in (7, 300, T + 5):
        ctx = U.make_ctx(wl, T, S, budget)
        sel = U.empty_i32(H, ctx.desc.max_sel, fill=-1)
        n_sel, n_tok = U.empty_i32(8, fill=-5), U.empty_i32(8, fill=-5)
        tok_idx = U.empty_i32(H, budget, fill=-1)
        ctx.select(torch.from_numpy(score).to(U.DEV), U.i32(off[:-1]), U.i32(lens), S, budget, sel, n_sel, tok_idx, n_tok)
        torch.cuda.synchronize()
        r_sel, r_nsel, r_tok, r_ntok = oracle32.select(score, off[:-1], lens, budget)
        g_sel, g_nsel, g_tok, g_ntok = sel.cpu().numpy(), n_sel.cpu().numpy(), tok_idx.cpu().numpy(), n_tok.cpu().numpy()
        for h in range(H):
            assert g_ntok[h] == r_ntok[h] and np.array_equal(g_tok[h, :r_ntok[h]], r_tok[h, :r_ntok[h]]), (budget, h)
            m = min(int(r_nsel[h]), ctx.desc.max_sel)
            assert g_nsel[h] == m and np.array_equal(g_sel[h, :m], r_sel[h, :m])
            assert np.all(lens[g_sel[h, :m]] > 0)


@pytest.mark.parametrize("dtype,T,N,k,budget", [("bf16", 6000, 32, 1024, 512), ("f32", 2500, 16, 600, 256)])
def test_retention_pipeline_then_decode(U, oracle32, dtype, T, N, k, budget):
    """segment -> importance -> retain -> compact -> mean keys of the retained tokens -> fused decode step on the
    retained pool, every stage against the oracle (later stages on the GPU's retained set)."""
    _say("retention pipeline", dtype, T, N, k, budget)
    L, Hq, H, D = 2, 32, 8, 128
    wl = gen.CFG1.scaled(n_layers=L, n_tokens=T, dtype=dtype)
    p = gen.prefill_inputs(gen.CFG3.scaled(n_layers=L, n_tokens=T, dtype=dtype), seed=11, device=U.DEV)
    seg_ref, off_ref, len_ref, S = oracle32.segment(p.tok, p.bitmap, gen.CFG3.vocab)
    ctx = U.make_ctx(wl, T, S, budget)                          # tok_idx rows are max_budget wide
    seg, off, ln, S_host, _ = U.gpu_segment(ctx, p.tok, p.bitmap, gen.CFG3.vocab, S)
    assert S_host == S and np.array_equal(seg, seg_ref)
    K = p.K
    V = torch.stack([gen.kv_layer(p.lengths, H, D, wl.torch_dtype, 12, l, device=U.DEV)[1] for l in range(L)])
    q_obs = gen.queries(L * Hq, N, D, wl.torch_dtype, seed=13, device=U.DEV).view(L, Hq, N, D)
    Tp = T - N
    alpha = _gpu_importance(U, ctx, q_obs, K, T, N)
    a_np = alpha.cpu().numpy()
    keep, n_keep, r_off, r_len = _gpu_retain(U, ctx, alpha, k, seg, S)
    K_ret = torch.zeros(L, H, k, D, dtype=wl.torch_dtype, device=U.DEV)
    V_ret = torch.zeros_like(K_ret)
    ctx.compact_pool(K, V, T, U.i32(keep), k, U.i32(np.concatenate([n_keep, np.zeros(4, np.int32)])), K_ret, V_ret)
    sv = torch.full((L, H, S, D), 3.0, dtype=torch.float32, device=U.DEV)
    ctx.build_semvec_layers(K_ret, U.i32(r_off), S, sv)
    torch.cuda.synchronize()
    qd = gen.queries(L, Hq, D, wl.torch_dtype, seed=14, device=U.DEV)
    out = torch.zeros(Hq, D, dtype=torch.float32, device=U.DEV)
    tok_idx, n_tok = U.empty_i32(H, budget, fill=-1), U.empty_i32(8, fill=-5)
    n_diff = 0
    for l in range(L):
        # importance and the retained set
        a_ref = oracle32.token_importance(U.np_of(q_obs[l]), U.np_of(K[l]))
        assert np.all(np.abs(a_np[l] - a_ref) <= 2e-4 * a_ref + 1e-7 * a_ref.max())
        keep_same, off_same, len_same = oracle32.retain(a_np[l], k, seg, S)
        assert n_keep[l] == k and np.array_equal(keep[l], keep_same)
        assert np.array_equal(r_off[l], off_same) and np.array_equal(r_len[l], len_same)
        keep_e2e, _, _ = oracle32.retain(a_ref, k, seg, S)
        diff = np.setxor1d(keep_e2e, keep[l])
        if len(diff):
            cut = np.sort(a_ref)[::-1][k - 1]
            assert np.all(np.abs(a_ref[diff] - cut) <= 5e-4 * cut), (l, diff)
            n_diff += len(diff)
        assert (r_len[l] == 0).any()                              # the case does contain vanished buckets
        # compacted rows and mean keys
        Kl, Vl = U.np_of(K[l]), U.np_of(V[l])
        assert np.array_equal(U.np_of(K_ret[l]), Kl[:, keep[l]]) and np.array_equal(U.np_of(V_ret[l]), Vl[:, keep[l]])
        sv_ref = oracle32.semvec(np.ascontiguousarray(Kl[:, keep[l]])[None], r_off[l])[0]
        got = sv[l].cpu().numpy()
        kmax = float(np.abs(K[l].float().cpu().numpy()).max())
        bound = (2.0 * np.maximum(r_len[l] - 1, 0) * 2.0 ** -24 * kmax + 2.0 ** -22 * kmax)[None, :, None]
        assert np.all(np.abs(got - sv_ref) <= bound)
        assert np.all(got[:, r_len[l] == 0] == 0)
        # decode on the retained pool
        ctx.decode_step(l, 1, qd[l], qd[l], K_ret, V_ret, k, sv, S, U.i32([0, k]), U.i32([0, S]), U.i32(r_off[l]),
                        U.i32(r_len[l]), U.i32([budget]), out, None, tok_idx, n_tok)
        torch.cuda.synchronize()
        q = U.np_of(qd[l])
        ref = oracle32.decode_step(q, q, np.ascontiguousarray(Kl[:, keep[l]]), np.ascontiguousarray(Vl[:, keep[l]]), got,
                                   r_off[l][:-1], r_len[l], budget)
        g_n, g_idx = n_tok.cpu().numpy()[:H], tok_idx.cpu().numpy()
        for h in range(H):
            assert g_n[h] == ref["n_tok"][h] and np.array_equal(g_idx[h, :g_n[h]], ref["tok_idx"][h, :g_n[h]]), (l, h)
        tol = 1e-4 if dtype == "f32" else 2e-2
        assert np.abs(out.cpu().numpy() - ref["out"]).max() <= tol
    _say("  retained-set differences from the oracle's end-to-end set (documented ties):", n_diff)
