"""GPU parity: every C entry point of libsentencekv against the CPU oracle on the same seeded inputs.

Gates: segment ids, offsets, lengths, selected bucket ids, token indices and gathered rows bit-exact;
scores within 1e-5 of the score scale; the GPU's selection must equal the oracle's selection rule
applied to the GPU's own scores bit for bit, and may differ from the oracle's end-to-end selection
only through documented score ties (< 1e-5 relative); attention within 1e-4 (fp32) / 2e-2 (bf16)
max-abs on identical gathered tokens.
"""
import math

import numpy as np
import pytest
import torch

from workload import gen

pytestmark = pytest.mark.gpu

ATT_TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def U():
    import gpu_util
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return gpu_util


def _say(*a):
    print(*a, flush=True)


# ----------------------------------------------------------------------------- segment

SEG_SIZES = [0, 1, 2, 63, 64, 1023, 1024, 1025, 4096, 32768, 100001]


@pytest.mark.parametrize("T", SEG_SIZES)
def test_segment_bit_exact(U, oracle32, T):
    _say("segment T", T)
    wl = gen.CFG3.scaled(n_tokens=T)
    p = gen.prefill_inputs(wl, seed=T + 1, with_keys=False)
    seg_ref, off_ref, len_ref, S_ref = oracle32.segment(p.tok, p.bitmap, wl.vocab)
    ctx = U.make_ctx(wl.scaled(n_layers=1), T, max(S_ref, 1) + 3, 16)
    seg, off, ln, S_host, S_dev = U.gpu_segment(ctx, p.tok, p.bitmap, wl.vocab, max(S_ref, 1) + 3)
    assert S_host == S_ref == S_dev
    assert np.array_equal(seg, seg_ref)
    assert np.array_equal(off[:S_ref + 1], off_ref)
    assert np.array_equal(ln[:S_ref], len_ref)
    assert np.all(off[S_ref + 1:] == -7) and np.all(ln[S_ref:] == -7)      # nothing written past S


_STREAMS = {"no_term": "aaaa", "all_term": "....", "term_last": "aaa.", "term_first": ".aaa", "one_tok": "a",
            "one_term": ".", "alternating": "a.a.a.a.", "run_of_terms": "aa..a", "2050_terms": "." * 2050,
            "3000_then_term": "a" * 3000 + "."}


@pytest.mark.parametrize("text", list(_STREAMS.values()), ids=list(_STREAMS.keys()))
def test_segment_hand_built_streams(U, oracle32, text):
    tok = np.array([7 if c == "." else 3 for c in text], dtype=np.int32)
    bitmap = np.zeros(2, dtype=np.uint32)
    bitmap[0] = 1 << 7
    seg_ref, off_ref, len_ref, S_ref = oracle32.segment(tok, bitmap, 64)
    wl = gen.CFG3.scaled(n_layers=1)
    ctx = U.make_ctx(wl, len(tok), len(tok), 16)
    seg, off, ln, S_host, _ = U.gpu_segment(ctx, tok, bitmap, 64, len(tok))
    assert S_host == S_ref and np.array_equal(seg, seg_ref)
    assert np.array_equal(off[:S_ref + 1], off_ref) and np.array_equal(ln[:S_ref], len_ref)


def test_segment_reports_capacity_overflow(U, oracle32):
    import paper_2504_00970_amd as skv
    tok = np.array([7] * 50, dtype=np.int32)
    bitmap = np.zeros(2, dtype=np.uint32)
    bitmap[0] = 1 << 7
    ctx = U.make_ctx(gen.CFG3.scaled(n_layers=1), 64, 10, 16)
    with pytest.raises(skv.SkvError) as e:
        U.gpu_segment(ctx, tok, bitmap, 64, 10)
    assert e.value.status == skv.SKV_ECAPACITY


# ----------------------------------------------------------------------------- semvec

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("dist", [("geometric", 0.05), ("uniform", 8, 40), ("fixed", 1), ("fixed", 257)])
def test_semvec_matches_oracle(U, oracle32, dtype, dist):
    _say("semvec", dtype, dist)
    wl = gen.CFG3.scaled(n_layers=3, n_kv_heads=2, n_q_heads=8, n_tokens=3001, dtype=dtype, len_dist=dist)
    lens = gen.sentence_lengths(wl.len_dist, wl.n_tokens, seed=5)
    off = gen.offsets_of(lens)
    S = len(lens)
    K = torch.stack([gen.kv_layer(lens, wl.n_kv_heads, 128, wl.torch_dtype, 5, l)[0] for l in range(wl.n_layers)])
    ref = oracle32.semvec(gen.to_numpy(K), off)
    ctx = U.make_ctx(wl, wl.n_tokens, S, 16)
    sv = torch.full((wl.n_layers, wl.n_kv_heads, S, 128), 9.0, dtype=torch.float32, device=U.DEV)
    ctx.build_semvec(K.to(U.DEV), U.i32(off), S, sv)
    torch.cuda.synchronize()
    got = sv.cpu().numpy()
    # both sides sum the same len values in fp32 in different orders: |diff| <= 2 (len-1) u max|k| (+1 ulp of the divide)
    kmax = float(K.float().abs().max())
    bound = (2.0 * np.maximum(lens - 1, 0) * 2.0 ** -24 * kmax + 2.0 ** -22 * kmax)[None, None, :, None]
    assert np.all(np.abs(got - ref) <= bound), float(np.abs(got - ref).max())
    one = lens == 1
    assert np.array_equal(got[:, :, one], ref[:, :, one])          # length-1 buckets are exact copies


# ----------------------------------------------------------------------------- decode chain, per stage

def _chain_case(U, oracle32, wl, seed, budget, pool_in_host=False, layers=None, sv_dtype="f32"):
    """Runs the 4-call chain on the GPU for some layers and checks each stage against the oracle."""
    inp = gen.decode_inputs(wl, seed=seed, device=U.DEV)          # generated on the GPU; the oracle reads copies
    S, T = len(inp.lengths), wl.n_tokens
    ctx = U.make_ctx(wl, T, S, budget, sv_dtype=sv_dtype)
    if pool_in_host:
        Kd = torch.empty(inp.K.shape, dtype=inp.K.dtype, pin_memory=True).copy_(inp.K)
        Vd = torch.empty(inp.V.shape, dtype=inp.V.dtype, pin_memory=True).copy_(inp.V)
        Kdev_for_semvec = inp.K.to(U.DEV)
    else:
        Kd, Vd = inp.K.to(U.DEV), inp.V.to(U.DEV)
        Kdev_for_semvec = Kd
    qd = inp.q.to(U.DEV)
    sv = torch.zeros(wl.n_layers, wl.n_kv_heads, max(S, 1), 128, dtype=U.sv_torch_dtype(sv_dtype), device=U.DEV)
    ctx.build_semvec(Kdev_for_semvec, U.i32(inp.sent_off), S, sv)
    torch.cuda.synchronize()
    sv_np = U.np_of(sv)[:, :, :S]
    n_ties = 0
    for l in (layers if layers is not None else range(wl.n_layers)):
        _say("chain", wl.name, "seed", seed, "budget", budget, "layer", l, "host_pool", pool_in_host)
        K, V, q = gen.to_numpy(inp.K[l]), gen.to_numpy(inp.V[l]), gen.to_numpy(inp.q[l])
        g = U.gpu_decode_chain(ctx, wl, l, qd[l], Kd, Vd, sv, inp.sent_off, inp.lengths, budget, pool_in_host)
        # (2) scores, on the GPU's own semantic vectors (stage parity) ...
        sc_ref_same_sv = oracle32.score(q, sv_np[l])
        assert np.all(np.abs(g["score"] - sc_ref_same_sv) <= U.score_tolerance(sc_ref_same_sv))
        # ... and end to end from the oracle's semantic vectors
        sv_ref = oracle32.semvec(K[None], inp.sent_off, sv_dtype=sv_dtype)[0]
        sc_ref = oracle32.score(q, sv_ref)
        if sv_dtype == "f32":
            assert np.all(np.abs(g["score"] - sc_ref) <= 2 * U.score_tolerance(sc_ref))
        else:                               # the two reduced tables round fp32 means that differ in summation order
            if sv_dtype == "bf16":
                assert U.bf16_table_close(sv_np[l], sv_ref)
            else:
                assert U.e4m3_table_close(sv_np[l], sv_ref, oracle32.e4m3_decode)
            one = inp.lengths == 1
            assert np.array_equal(sv_np[l][:, one], sv_ref[:, one])
        # (3) selection: the oracle's rule on the GPU's scores, bit for bit
        sel, n_sel, tok_idx, n_tok = oracle32.select(g["score"], inp.sent_off, inp.lengths, budget)
        assert np.array_equal(g["n_sel"], n_sel) and np.array_equal(g["n_tok"], n_tok)
        for h in range(wl.n_kv_heads):
            assert np.array_equal(g["sel_sent"][h, :n_sel[h]], sel[h, :n_sel[h]])
            assert np.array_equal(g["tok_idx"][h, :n_tok[h]], tok_idx[h, :n_tok[h]])
            assert n_tok[h] <= budget
        # end-to-end selection may differ only through documented ties
        sel_e, n_sel_e, tok_idx_e, n_tok_e = oracle32.select(sc_ref, inp.sent_off, inp.lengths, budget)
        for h in range(wl.n_kv_heads):
            if sv_dtype == "f32" and (n_sel_e[h] != n_sel[h] or not np.array_equal(sel_e[h, :n_sel_e[h]], sel[h, :n_sel[h]])):
                ok, a, b, gap = U.documented_tie(sc_ref[h], g["score"][h], upto=int(max(n_sel_e[h], n_sel[h])) + 1)
                _say(f"  documented tie: layer {l} head {h} buckets {a},{b} relative gap {gap:.3e}")
                assert ok, (l, h, a, b, gap)
                n_ties += 1
        # (4) gather: bit copy of the rows the GPU selected
        Ks_ref, Vs_ref = oracle32.gather(K, tok_idx, n_tok), oracle32.gather(V, tok_idx, n_tok)
        for h in range(wl.n_kv_heads):
            assert np.array_equal(g["K_sel"][h, :n_tok[h]], Ks_ref[h, :n_tok[h]])
            assert np.array_equal(g["V_sel"][h, :n_tok[h]], Vs_ref[h, :n_tok[h]])
            assert not g["K_sel"][h, n_tok[h]:].any()                  # rows past n_tok untouched
        # (5) attention on identical gathered tokens
        out_ref, lse_ref = oracle32.attend(q, Ks_ref, Vs_ref, n_tok)
        err = float(np.abs(g["out"] - out_ref).max())
        assert err <= ATT_TOL[wl.dtype], err
        fin = np.isfinite(lse_ref)
        assert np.array_equal(np.isfinite(g["lse"]), fin)
        assert not fin.any() or np.abs(g["lse"][fin] - lse_ref[fin]).max() <= ATT_TOL[wl.dtype]
    return n_ties


def test_chain_cfg0_fp32_4k(U, oracle32):
    _chain_case(U, oracle32, gen.CFG0, seed=0, budget=512)


@pytest.mark.parametrize("budget", [1024, 2048])
def test_chain_cfg1_shape_bf16_small_context(U, oracle32, budget):
    # cfg1's heads, dtype and length distribution at a context the oracle handles for several layers
    _chain_case(U, oracle32, gen.CFG1.scaled(n_layers=3, n_tokens=9000), seed=1, budget=budget)


@pytest.mark.parametrize("T,budget", [(1, 4), (37, 5), (300, 64), (1000, 63), (1000, 65), (1000, 4000), (2500, 129)])
def test_chain_ragged_tails_and_edges(U, oracle32, T, budget):
    for dtype in ("f32", "bf16"):
        _chain_case(U, oracle32, gen.CFG0.scaled(n_tokens=T, dtype=dtype, n_layers=2), seed=T, budget=budget)


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (16, 8), (64, 8), (4, 1)])
def test_chain_group_sizes(U, oracle32, Hq, Hkv):
    _chain_case(U, oracle32, gen.CFG1.scaled(n_layers=1, n_tokens=3000, n_q_heads=Hq, n_kv_heads=Hkv), seed=9, budget=256)


def test_chain_pinned_host_pool(U, oracle32):
    _chain_case(U, oracle32, gen.CFG1.scaled(n_layers=2, n_tokens=5000), seed=3, budget=512, pool_in_host=True)


# ----------------------------------------------------------------------------- selection on hand-made scores

def _gpu_select(U, ctx, score, off, lens, budget):
    H, S = score.shape
    sel = U.empty_i32(H, ctx.desc.max_sel, fill=-1)
    n_sel, n_tok = U.empty_i32(max(H, 4), fill=-5), U.empty_i32(max(H, 4), fill=-5)
    tok_idx = U.empty_i32(H, max(budget, 1), fill=-1)
    ctx.select(torch.as_tensor(score).to(U.DEV), U.i32(off), U.i32(lens), S, budget, sel, n_sel, tok_idx, n_tok)
    torch.cuda.synchronize()
    return sel.cpu().numpy(), n_sel.cpu().numpy()[:H], tok_idx.cpu().numpy(), n_tok.cpu().numpy()[:H]


def _check_select(U, oracle32, score, lens, budget):
    score = np.ascontiguousarray(score, dtype=np.float32)
    lens = np.asarray(lens, dtype=np.int32)
    off = gen.offsets_of(lens)
    H, S = score.shape
    wl = gen.CFG0.scaled(n_kv_heads=H, n_q_heads=H)
    ctx = U.make_ctx(wl, int(lens.sum()), S, budget)
    sel, n_sel, tok_idx, n_tok = _gpu_select(U, ctx, score, off, lens, budget)
    sel_r, n_sel_r, tok_idx_r, n_tok_r = oracle32.select(score, off, lens, budget)
    assert np.array_equal(n_sel, n_sel_r), (n_sel, n_sel_r)
    assert np.array_equal(n_tok, n_tok_r)
    for h in range(H):
        assert np.array_equal(sel[h, :n_sel[h]], sel_r[h, :n_sel[h]])
        assert np.array_equal(tok_idx[h, :n_tok[h]], tok_idx_r[h, :n_tok[h]])


def test_select_hand_made_scores(U, oracle32):
    rng = np.random.default_rng(11)
    nan, inf = float("nan"), float("inf")
    _say("select: ties / zeros / nan")
    _check_select(U, oracle32, [[1, 1, 1, 1], [2, 1, 2, 1]], [2, 2, 2, 2], 5)
    _check_select(U, oracle32, [[0.0, -0.0, -1], [-0.0, 0.0, -1]], [1, 1, 1], 1)
    _check_select(U, oracle32, [[nan, -inf, 1], [nan, nan, 1], [inf, nan, -inf]], [1, 1, 1], 2)
    _check_select(U, oracle32, [[9, 8, 7]], [10, 1, 1], 5)          # top bucket too long: nothing
    _check_select(U, oracle32, [[9, 8, 7]], [2, 10, 1], 5)          # stop at the first overflow
    _check_select(U, oracle32, [[3, 2, 1]], [4, 4, 4], 0)
    _say("select: all equal scores, several chunks of 1024 buckets")
    for S in (1, 1023, 1024, 1025, 5000):
        lens = rng.integers(1, 9, size=S)
        for budget in (1, 7, int(lens.sum()) // 3, int(lens.sum()), int(lens.sum()) + 10):
            _check_select(U, oracle32, np.zeros((2, S)), lens, budget)
    _say("select: coarse scores (many ties at the cut), random budgets")
    for trial in range(40):
        S = int(rng.integers(1, 3000))
        lens = rng.integers(1, 40, size=S)
        score = rng.integers(-6, 7, size=(3, S)) / 4.0
        _check_select(U, oracle32, score, lens, int(rng.integers(1, 2049)))
    _say("select: scores that differ only in low mantissa bits / tiny and huge magnitudes")
    for trial in range(10):
        S = int(rng.integers(2, 2000))
        lens = rng.integers(1, 30, size=S)
        base = np.float32(1.0) + rng.integers(0, 50, size=(2, S)).astype(np.float32) * np.float32(2.0 ** -23)
        _check_select(U, oracle32, base, lens, int(rng.integers(1, 1500)))
        wide = (rng.standard_normal((2, S)) * 10.0 ** rng.integers(-30, 30, size=(2, S))).astype(np.float32)
        _check_select(U, oracle32, wide, lens, int(rng.integers(1, 1500)))


# ----------------------------------------------------------------------------- attention edge cases

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_attend_ragged_counts(U, oracle32, dtype):
    wl = gen.CFG0.scaled(dtype=dtype)
    H, Hq, D, budget = 8, 32, 128, 200
    g = torch.Generator().manual_seed(3)
    q = torch.randn(Hq, D, generator=g).to(wl.torch_dtype)
    Ks = torch.randn(H, budget, D, generator=g).to(wl.torch_dtype)
    Vs = torch.randn(H, budget, D, generator=g).to(wl.torch_dtype)
    n_tok = np.array([0, 1, 63, 64, 65, 128, 199, 200], dtype=np.int32)
    ctx = U.make_ctx(wl, 4096, 64, budget)
    out = torch.full((Hq, D), 5.0, device=U.DEV)
    lse = torch.full((Hq,), 5.0, device=U.DEV)
    for rep in range(2):                                   # second call checks the arrival counters were reset
        ctx.attend(q.to(U.DEV), Ks.to(U.DEV), Vs.to(U.DEV), U.i32(n_tok), budget, out, lse)
        torch.cuda.synchronize()
        out_ref, lse_ref = oracle32.attend(gen.to_numpy(q), gen.to_numpy(Ks), gen.to_numpy(Vs), n_tok)
        assert np.abs(out.cpu().numpy() - out_ref).max() <= ATT_TOL[dtype]
        assert np.all(np.isneginf(lse.cpu().numpy()[:4])) and not out.cpu().numpy()[:4].any()
        assert np.abs(lse.cpu().numpy()[4:] - lse_ref[4:]).max() <= ATT_TOL[dtype]


def test_attend_large_logits_do_not_overflow(U, oracle32):
    wl = gen.CFG0
    H, Hq, D, budget = 8, 32, 128, 130
    g = torch.Generator().manual_seed(4)
    q = torch.randn(Hq, D, generator=g) * 30.0
    Ks = torch.randn(H, budget, D, generator=g) * 30.0
    Vs = torch.randn(H, budget, D, generator=g)
    n_tok = np.full(H, budget, dtype=np.int32)
    ctx = U.make_ctx(wl, 4096, 64, budget)
    out = torch.zeros(Hq, D, device=U.DEV)
    lse = torch.zeros(Hq, device=U.DEV)
    ctx.attend(q.to(U.DEV), Ks.to(U.DEV), Vs.to(U.DEV), U.i32(n_tok), budget, out, lse)
    torch.cuda.synchronize()
    out_ref, lse_ref = oracle32.attend(q.numpy(), Ks.numpy(), Vs.numpy(), n_tok)
    assert np.isfinite(out.cpu().numpy()).all()
    assert np.abs(out.cpu().numpy() - out_ref).max() <= 1e-4
    assert np.abs(lse.cpu().numpy() - lse_ref).max() <= 1e-3 * np.abs(lse_ref).max()


# ----------------------------------------------------------------------------- fused step

# Descriptor max_budget values that steer a bf16 batch of 8 sequences x 8 KV heads (64 pairs, 4 blocks per pair in the
# single-launch step: budgets up to 1024 run there, in 256-token blocks); beyond that the library picks the attention kernel
# from block counts, pairs x ceil(max_budget / 256) <= 256 compute units: 256-token fused blocks; else the streaming
# kernel, in 512-token blocks while pairs x ceil(max_budget / 1024) <= 128, else in 1024-token blocks.
STREAM_CAPACITY = 9000      # 1024-token streaming blocks
HALF_CAPACITY = 1500        # 512-token streaming blocks (for 64 pairs; 72 pairs need 1024)


def _fused_case(U, oracle32, wl, seed, layers, sv_dtype="f32", seq_tokens=None, budgets=None, capacity=0):
    """One skv_decode_step per layer against the oracle, sequence by sequence.  `capacity` raises the context's
    max_budget above the budgets in use: the library sizes its grids by it, and a bf16 batch whose 256-token blocks
    (pairs x ceil(max_budget / 256)) outnumber the compute units takes the streaming kernel instead of the fused one,
    so the same inputs reach both kernels."""
    inp = gen.ragged_inputs(wl, seed=seed, device=U.DEV, resident_layers=len(layers), seq_tokens=seq_tokens, budgets=budgets)
    B, H, Hq, D = wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.head_dim
    T_total, S_total = int(inp.cu_tok[-1]), int(inp.cu_sent[-1])
    max_budget = max(int(inp.budget.max()), capacity)
    ctx = U.make_ctx(wl.scaled(n_layers=len(layers)), T_total, S_total, max_budget, batch=B, sv_dtype=sv_dtype)
    Kd, Vd, qd = inp.K.to(U.DEV), inp.V.to(U.DEV), inp.q.to(U.DEV)
    # semantic vectors of the concatenated stream: bucket boundaries are the concatenation of the sequences'
    glob_off = gen.offsets_of(inp.sent_len)
    sv = torch.zeros(len(layers), H, S_total, D, dtype=U.sv_torch_dtype(sv_dtype), device=U.DEV)
    ctx.build_semvec(Kd, U.i32(glob_off), S_total, sv)
    out = torch.full((B, Hq, D), 7.0, device=U.DEV)
    lse = torch.full((B, Hq), 7.0, device=U.DEV)
    tok_idx = U.empty_i32(B, H, max_budget, fill=-1)
    n_tok = U.empty_i32(B, H, fill=-1)
    d = dict(cu_tok=U.i32(inp.cu_tok), cu_sent=U.i32(inp.cu_sent), sent_off=U.i32(inp.sent_off),
             sent_len=U.i32(inp.sent_len), budget=U.i32(inp.budget))
    n_ties = 0
    for li, l in enumerate(layers):
        _say("fused", wl.name, "B", B, "layer", li)
        ctx.decode_step(li, B, qd[li], qd[li], Kd, Vd, T_total, sv, S_total, d["cu_tok"], d["cu_sent"], d["sent_off"],
                        d["sent_len"], d["budget"], out, lse, tok_idx, n_tok)
        torch.cuda.synchronize()
        sv_l = U.np_of(sv[li])
        o, ls, ti, nt = out.cpu().numpy(), lse.cpu().numpy(), tok_idx.cpu().numpy(), n_tok.cpu().numpy()
        for b in range(B):
            t0, t1, s0, s1 = inp.cu_tok[b], inp.cu_tok[b + 1], inp.cu_sent[b], inp.cu_sent[b + 1]
            K = gen.to_numpy(inp.K[li, :, t0:t1]); V = gen.to_numpy(inp.V[li, :, t0:t1]); q = gen.to_numpy(inp.q[li, b])
            off_b, len_b = inp.sent_off[s0 + b: s1 + b + 1], inp.sent_len[s0:s1]
            # selection: the oracle's rule on the GPU's own scores bit for bit; against the oracle's scores only a
            # documented tie may change it (U.check_selection).  Attention is then compared on the GPU's tokens.
            sc = oracle32.score(q, sv_l[:, s0:s1])
            sc_gpu = U.gpu_scores(ctx, li, qd[li, b], sv, S_total, H)[:, s0:s1]
            n_ties += U.check_selection(oracle32, sc, sc_gpu, off_b, len_b, int(inp.budget[b]), ti[b], nt[b],
                                        what=f"{wl.name} layer {li} sequence {b}")
            n_ref = nt[b].astype(np.int32)
            tok_ref = np.where(ti[b] < 0, 0, ti[b]).astype(np.int32)
            Ks, Vs = oracle32.gather(K, tok_ref, n_ref), oracle32.gather(V, tok_ref, n_ref)
            o_ref, l_ref = oracle32.attend(q, Ks, Vs, n_ref)
            assert np.abs(o[b] - o_ref).max() <= ATT_TOL[wl.dtype]
            fin = np.isfinite(l_ref)
            assert not fin.any() or np.abs(ls[b][fin] - l_ref[fin]).max() <= ATT_TOL[wl.dtype]
        # without the optional outputs the result is the same
        out2 = torch.zeros_like(out)
        ctx.decode_step(li, B, qd[li], qd[li], Kd, Vd, T_total, sv, S_total, d["cu_tok"], d["cu_sent"], d["sent_off"],
                        d["sent_len"], d["budget"], out2, None, None, None)
        torch.cuda.synchronize()
        if wl.dtype == "bf16" and B * H * math.ceil(max_budget / 256) > 256:
            # the streaming kernel (bf16, more 256-token blocks than compute units) hands its
            # 16-token tiles to whichever wave is free: the summation order, and with it the last bits of the output,
            # differ from call to call
            assert (out - out2).abs().max().item() <= ATT_TOL[wl.dtype] / 4
        else:
            assert torch.equal(out, out2)
    if n_ties:
        _say(f"  fused {wl.name}: {n_ties} documented ties")
    assert n_ties <= U.MAX_TIES_PER_TEST, n_ties
    return n_ties


@pytest.mark.parametrize("capacity", [0, 5000, STREAM_CAPACITY, 20000])
def test_fused_single_sequence_matches_oracle(U, oracle32, capacity):
    """One sequence through the forms of the step: single launch in 128-token blocks, in 256-token blocks (capacity 5000: 8 heads x
    40 blocks of 128 tokens no longer fit the chip at once), 512- and 1024-token streaming blocks (capacities 9000 and
    20000: beyond 32 blocks x 256 tokens per head, and 8 x 36 > 256 blocks of 256 tokens); fp32 runs the single launch on the
    plain ALUs, and selection + attention through the positions for the large capacities."""
    wl = gen.CFG1.scaled(n_layers=2, batch=1, t_range=(6000, 6000), budgets=(1024,))
    _fused_case(U, oracle32, wl, seed=2, layers=[0, 1], capacity=capacity)
    wl = gen.CFG0.scaled(n_layers=1, batch=1, t_range=(4096, 4096), budgets=(512,))
    _fused_case(U, oracle32, wl, seed=3, layers=[0], capacity=capacity)


@pytest.mark.parametrize("tokens,budget", [(700, 2048), (2500, 2048), (3000, 1)])
@pytest.mark.parametrize("B", [1, 3])
def test_fused_single_launch_with_idle_blocks(U, oracle32, tokens, budget, B):
    """The single-launch step when the retrieved tokens do not fill the blocks the budget provides: a context smaller than
    the budget (every bucket is taken: 6 of 16 blocks hold tokens), a selection that ends a block or two short of the
    budget's last one, and a budget no bucket fits (nothing retrieved).  The blocks without tokens run the selection too,
    and block 0 of a pair waits for their word before it ends the pair's launch."""
    wl = gen.CFG1.scaled(n_layers=1, batch=B, t_range=(tokens, tokens), budgets=(budget,), len_dist=("uniform", 2, 300))
    _fused_case(U, oracle32, wl, seed=61, layers=[0])
    _fused_case(U, oracle32, wl, seed=62, layers=[0])                 # again, on a fresh context


@pytest.mark.parametrize("budget", [3000, 6000])
def test_fused_single_sequence_large_budget(U, oracle32, budget):
    """Budgets of thousands of tokens for one sequence, single launch: 128-token blocks (3000: 8 x 24 blocks of 128 tokens still
    fit the 32 blocks of a head; 6000 takes 256-token blocks) with every block full of retrieved tokens."""
    wl = gen.CFG1.scaled(n_layers=1, batch=1, t_range=(9000, 9000), budgets=(budget,))
    _fused_case(U, oracle32, wl, seed=5, layers=[0])


def test_fused_ragged_batch_70b_heads(U, oracle32):
    wl = gen.CFG4.scaled(n_layers=2, batch=5, t_range=(500, 4000), budgets=(512,))
    _fused_case(U, oracle32, wl, seed=4, layers=[0, 1])


@pytest.mark.parametrize("capacity", [0, 1024, STREAM_CAPACITY])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("Hq", [8, 16, 32, 64])
def test_fused_batch_path_many_heads(U, oracle32, Hq, dtype, capacity):
    """Nine sequences x 8 KV heads, for every group size: bf16 pools run the selection inside 256-token fused MFMA blocks
    or, with the larger capacities, inside 512-token and 1024-token streaming MFMA blocks; fp32 pools run select_kernel
    and 256-token blocks through tok_idx."""
    wl = gen.CFG4.scaled(n_layers=1, n_q_heads=Hq, batch=9, t_range=(200, 3000), budgets=(700,), dtype=dtype)
    _fused_case(U, oracle32, wl, seed=6, layers=[0], capacity=capacity)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("budget", [100, 200, 700])
def test_fused_two_launch_small_blocks(U, oracle32, budget, dtype):
    """More than 64 (sequence, head) pairs with small budgets: too many pairs for the single-launch step, few enough blocks
    for the two-launch step's fused blocks of 64 tokens (budget 100), 128 tokens (200) and 256 tokens (700) (fp32 pools of
    64 pairs or more: selection kernel + attention through the positions)."""
    wl = gen.CFG4.scaled(n_layers=1, n_q_heads=32, batch=9, t_range=(300, 2500), budgets=(budget,), dtype=dtype)
    _fused_case(U, oracle32, wl, seed=51, layers=[0])


@pytest.mark.parametrize("capacity", [0, HALF_CAPACITY, STREAM_CAPACITY])
@pytest.mark.parametrize("budget", [512, 513, 1024, 1025, 1500, 2048])
def test_fused_batch_path_two_blocks_per_head(U, oracle32, budget, capacity):
    """Budgets around the 512- and 1024-token blocks of the bf16 streaming kernel: a full block, one token in the next
    block, a block whose last waves have nothing to stream, two full blocks; contexts shorter than the budget too.
    (Without a capacity budgets up to 1024 run 256-token fused blocks, the others 512-token streaming blocks.)"""
    wl = gen.CFG4.scaled(n_layers=1, n_q_heads=32, batch=8, t_range=(900, 5000), budgets=(budget,))
    _fused_case(U, oracle32, wl, seed=8, layers=[0], capacity=capacity)


@pytest.mark.parametrize("capacity", [0, HALF_CAPACITY, STREAM_CAPACITY])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B", [2, 3, 8])
def test_fused_batch_with_empty_and_tiny_sequences(U, oracle32, dtype, B, capacity):
    """Sequences without tokens, with one token and with one bucket next to ordinary ones, budgets from 0 to more than the
    context, in the single-launch step (B = 2: 128-token blocks; B = 3: 256-token blocks; B = 8 without a capacity) and on the
    batch paths (B = 8 with a capacity: 256-token fused blocks or the streaming kernel; fp32: selection kernel + indirect
    attention)."""
    toks = [0, 1, 1500, 0, 37, 2300, 5, 0][:B]
    buds = [64, 64, 700, 0, 1000, 0, 3, 9][:B]
    if B == 2:
        toks, buds = [1500, 0], [700, 64]
    wl = gen.CFG4.scaled(n_layers=1, n_q_heads=32, batch=B, budgets=(1000,), dtype=dtype)
    _fused_case(U, oracle32, wl, seed=12, layers=[0], seq_tokens=toks, budgets=buds, capacity=capacity)


@pytest.mark.parametrize("capacity", [0, 2048])
@pytest.mark.parametrize("sv_dtype", ["f32", "bf16", "fp8"])
@pytest.mark.parametrize("B", [2, 7, 8, 9, 21, 70])
def test_fused_batch_sequence_boundaries_inside_a_wave(U, oracle32, B, sv_dtype, capacity):
    """The score kernel's waves own 8, 16 or 32 consecutive buckets of the concatenated batch (fp32, bf16, E4M3 table)
    and look up the sequences they fall in.  Sequences of a handful of tokens, some without tokens, put several
    boundaries inside one wave; a long sequence in between spans many waves; batch sizes lie on both sides of the
    lookup's eight-entry step.  (With a capacity of 2048 the two largest batches take the streaming kernel's 2048-token
    blocks, the others 512-token blocks or the fused kernel.)"""
    rng = np.random.default_rng(100 + B)
    toks = rng.integers(0, 90, size=B)
    toks[rng.integers(0, B, size=max(1, B // 5))] = 0
    toks[B // 2] = 2100
    toks[-1] = int(rng.integers(1, 30))
    buds = rng.integers(0, 400, size=B)
    wl = gen.CFG4.scaled(n_layers=1, n_q_heads=32, batch=B, budgets=(400,), dtype="bf16")
    _fused_case(U, oracle32, wl, seed=40 + B, layers=[0], sv_dtype=sv_dtype, seq_tokens=toks.tolist(), budgets=buds.tolist(),
                capacity=capacity)


@pytest.mark.parametrize("Hq", [8, 32, 64])
@pytest.mark.parametrize("budget", [1025, 1500, 2048, 2049, 3000])
def test_fused_batch_2048_token_blocks(U, oracle32, budget, Hq):
    """20 sequences x 8 KV heads with budgets above 1024: the 1024-token streaming blocks would need two rounds on 256
    compute units, so the kernel runs 2048-token blocks (two positions per thread), each writing its result directly
    while one block covers the budget, and through the split-K merge from 2049 tokens on; contexts shorter and longer
    than the budget."""
    wl = gen.CFG4.scaled(n_layers=1, n_q_heads=Hq, batch=20, t_range=(900, 4500), budgets=(budget,))
    _fused_case(U, oracle32, wl, seed=31, layers=[0])


def test_fused_batch_of_hundreds_of_short_sequences(U, oracle32):
    """600 sequences of 0..60 tokens (4800 (sequence, head) pairs): the sequence lookup of the score kernel bisects seven
    levels deep before its eight-entry step, most waves span several sequences, the attention grid has thousands of rows."""
    B = 600
    rng = np.random.default_rng(77)
    toks = rng.integers(0, 61, size=B)
    buds = rng.integers(0, 80, size=B)
    wl = gen.CFG4.scaled(n_layers=1, n_q_heads=32, batch=B, budgets=(80,), dtype="bf16")
    _fused_case(U, oracle32, wl, seed=77, layers=[0], seq_tokens=toks.tolist(), budgets=buds.tolist())
    _fused_case(U, oracle32, wl, seed=78, layers=[0], seq_tokens=toks.tolist(), budgets=buds.tolist(), capacity=2048)   # 2048-token blocks


@pytest.mark.parametrize("capacity", [0, HALF_CAPACITY, STREAM_CAPACITY])
@pytest.mark.parametrize("dtype,budget", [("f32", 700), ("bf16", 2), ("bf16", 256), ("bf16", 257), ("bf16", 5000)])
def test_fused_batch_path_edges(U, oracle32, dtype, budget, capacity):
    """Batch paths (fp32: the VALU kernel through tok_idx; bf16: 256-token fused blocks, and the streaming kernel with the
    large capacity or the 5000-token budget) with a budget no bucket fits (empty selections), budgets at and just past
    one 256-token block, and a budget above every context length (all tokens retrieved)."""
    wl = gen.CFG4.scaled(n_layers=1, n_q_heads=32, batch=8, t_range=(150, 2500), budgets=(budget,), dtype=dtype)
    _fused_case(U, oracle32, wl, seed=9, layers=[0], capacity=capacity)


def test_attend_batch_path_direct_rows(U, oracle32):
    """skv_attend with n_kv_heads = 64 (>= the batch-path threshold): 256-token blocks on K_sel/V_sel."""
    wl = gen.CFG0.scaled(dtype="bf16", n_q_heads=64, n_kv_heads=64)
    H, Hq, D, budget = 64, 64, 128, 700
    g = torch.Generator().manual_seed(5)
    q = torch.randn(Hq, D, generator=g).to(wl.torch_dtype)
    Ks = torch.randn(H, budget, D, generator=g).to(wl.torch_dtype)
    Vs = torch.randn(H, budget, D, generator=g).to(wl.torch_dtype)
    n_tok = np.array([(37 * i) % 701 for i in range(H)], dtype=np.int32)
    n_tok[:4] = [0, 1, 256, 700]
    ctx = U.make_ctx(wl, 4096, 64, budget)
    out = torch.full((Hq, D), 5.0, device=U.DEV)
    lse = torch.full((Hq,), 5.0, device=U.DEV)
    for rep in range(2):
        ctx.attend(q.to(U.DEV), Ks.to(U.DEV), Vs.to(U.DEV), U.i32(n_tok), budget, out, lse)
        torch.cuda.synchronize()
        out_ref, lse_ref = oracle32.attend(gen.to_numpy(q), gen.to_numpy(Ks), gen.to_numpy(Vs), n_tok)
        assert np.abs(out.cpu().numpy() - out_ref).max() <= ATT_TOL["bf16"]
        fin = np.isfinite(lse_ref)
        assert np.array_equal(np.isfinite(lse.cpu().numpy()), fin)
        assert np.abs(lse.cpu().numpy()[fin] - lse_ref[fin]).max() <= ATT_TOL["bf16"]


# ----------------------------------------------------------------------------- full benchmark sizes

def test_full_size_cfg1_sampled_layers(U, oracle32):
    """cfg1 at its real size (32 layers, 32768 tokens, bf16, budgets 1024 and 2048): every stage checked
    against the oracle on three layers of the 32-layer pool, through the same calls bench.py times."""
    wl = gen.CFG1
    total_ties = 0
    for budget in wl.budgets:
        total_ties += _chain_case(U, oracle32, wl, seed=0, budget=budget, layers=[0, 13, 31])
    _say("full-size cfg1 documented ties:", total_ties)


def test_full_size_cfg2_128k_sampled_layers(U, oracle32):
    """cfg2 at its real size (32 layers x 131072 tokens, budget 2048): the 4-call chain on two layers of the
    17 GB pool, and the fused decode step (selection with more than 2048 buckets per head) on two layers."""
    _chain_case(U, oracle32, gen.CFG2, seed=0, budget=2048, layers=[0, 31])
    torch.cuda.empty_cache()
    wl = gen.CFG2.scaled(n_layers=2, batch=1, t_range=(131072, 131072), budgets=(2048,))
    _fused_case(U, oracle32, wl, seed=1, layers=[0, 1])
    # the same sequence through the streaming kernel (a context sized for budgets up to 20000 takes 1024-token blocks)
    _fused_case(U, oracle32, wl.scaled(n_layers=1), seed=1, layers=[0], capacity=20000)
    # and with a budget of 8192 tokens: 256-token fused blocks, each full of retrieved tokens
    _fused_case(U, oracle32, wl.scaled(n_layers=1, budgets=(8192,)), seed=1, layers=[0])


def test_full_size_cfg3_prefill(U, oracle32):
    """cfg3 at its real size: 32768-token stream over a 128k vocabulary, keys [32][8][32768][128] bf16; segment ids,
    offsets and lengths bit-exact, mean keys of three sampled layers against the oracle."""
    wl = gen.CFG3
    p = gen.prefill_inputs(wl, seed=0, device=U.DEV)
    seg_ref, off_ref, len_ref, S_ref = oracle32.segment(p.tok, p.bitmap, wl.vocab)
    ctx = U.make_ctx(wl, wl.n_tokens, S_ref + 8, 16)
    seg, off, ln, S_host, S_dev = U.gpu_segment(ctx, p.tok, p.bitmap, wl.vocab, S_ref + 8)
    assert S_host == S_ref == S_dev == len(p.lengths)
    assert np.array_equal(seg, seg_ref) and np.array_equal(off[:S_ref + 1], off_ref) and np.array_equal(ln[:S_ref], len_ref)
    sv = torch.zeros(wl.n_layers, wl.n_kv_heads, S_ref, 128, dtype=torch.float32, device=U.DEV)
    ctx.build_semvec(p.K, U.i32(off[:S_ref + 1]), S_ref, sv)
    torch.cuda.synchronize()
    for l in (0, 17, 31):
        _say("cfg3 semvec layer", l)
        ref = oracle32.semvec(gen.to_numpy(p.K[l:l + 1]), off_ref)[0]
        got = sv[l].cpu().numpy()
        kmax = float(p.K[l].float().abs().max())
        bound = (2.0 * np.maximum(len_ref - 1, 0) * 2.0 ** -24 * kmax + 2.0 ** -22 * kmax)[None, :, None]
        assert np.all(np.abs(got - ref) <= bound), float(np.abs(got - ref).max())


def test_full_size_cfg4_ragged_batch(U, oracle32):
    """cfg4 at its real shapes (64 q heads / 8 KV heads, 16 sequences of 8192..65536 tokens, budget 2048) on two
    resident layers: every sequence's selection and attention output against the oracle."""
    _fused_case(U, oracle32, gen.CFG4.scaled(n_layers=2), seed=0, layers=[0, 1])


def test_full_size_cfg1_batched(U, oracle32):
    """The batched extras of bench.py at their real shapes, one layer: 16 sequences of 32768 tokens (1024-token streaming
    blocks) and 24 sequences (2048-token blocks, one per (sequence, head)), budget 2048, every sequence against the oracle."""
    for B in (16, 24):
        wl = gen.CFG1.scaled(n_layers=1, batch=B, t_range=(32768, 32768), budgets=(2048,))
        _fused_case(U, oracle32, wl, seed=3, layers=[0])
        torch.cuda.empty_cache()


# ----------------------------------------------------------------------------- budget hint

@pytest.mark.parametrize("B,dtype", [(1, "bf16"), (1, "f32"), (4, "bf16"), (9, "bf16"), (9, "f32")])
def test_budget_hint_makes_a_large_context_plan_like_a_small_one(U, oracle32, B, dtype):
    """A context created for budgets up to 8192 and told (skv_set_budget_hint) that the budgets in use are at most 700
    runs the step exactly as a context created for 700 does: same selection, same output bits (the streaming kernel,
    nine bf16 sequences with the unhinted capacity, is the one form whose last bits vary between calls); budgets above
    the hint are treated as the hint; 0 restores the capacity."""
    wl = gen.CFG4.scaled(n_layers=1, n_q_heads=32, batch=B, t_range=(1500, 4000), budgets=(700,), dtype=dtype)
    inp = gen.ragged_inputs(wl, seed=17, device=U.DEV, resident_layers=1)
    H, Hq, D = wl.n_kv_heads, wl.n_q_heads, wl.head_dim
    T, S = int(inp.cu_tok[-1]), int(inp.cu_sent[-1])
    d = [U.i32(x) for x in (inp.cu_tok, inp.cu_sent, inp.sent_off, inp.sent_len)]
    q = inp.q[0]

    def run(ctx, sv, budgets, cap):
        out = torch.full((B, Hq, D), 3.0, device=U.DEV)
        lse = torch.full((B, Hq), 3.0, device=U.DEV)
        tok_idx = U.empty_i32(B, H, cap, fill=-1)
        n_tok = U.empty_i32(B, H, fill=-1)
        ctx.decode_step(0, B, q, q, inp.K, inp.V, T, sv, S, *d, U.i32(budgets), out, lse, tok_idx, n_tok)
        torch.cuda.synchronize()
        return out, lse, tok_idx[:, :, :700].clone(), n_tok

    def make(cap):
        ctx = U.make_ctx(wl, T, S, cap, batch=B)
        sv = torch.zeros(1, H, S, D, device=U.DEV)
        ctx.build_semvec(inp.K, U.i32(gen.offsets_of(inp.sent_len)), S, sv)
        return ctx, sv

    small, sv_s = make(700)
    big, sv_b = make(8192)
    ref = run(small, sv_s, [700] * B, 700)
    big.set_budget_hint(700)
    _say("budget hint: capacity 8192, hint 700, B", B, dtype)
    got = run(big, sv_b, [700] * B, 8192)
    for a, b in zip(ref, got):
        assert torch.equal(a, b)
    got = run(big, sv_b, [5000] * B, 8192)                  # budgets above the hint count as the hint
    for a, b in zip(ref, got):
        assert torch.equal(a, b)
    big.set_budget_hint(0)                                  # back to the capacity: the larger budget now applies
    full = run(big, sv_b, [5000] * B, 8192)
    assert bool((full[3] >= ref[3]).all()) and int(full[3].max()) > 700
    with pytest.raises(Exception):
        big.set_budget_hint(9000)


@pytest.mark.parametrize("B,dtype", [(1, "bf16"), (3, "bf16"), (1, "f32")])
def test_single_launch_can_be_turned_off(U, oracle32, B, dtype):
    """skv_set_single_launch(ctx, 0): the step takes the two-launch form (for callers whose steps overlap with other work
    on the GPU); the selection is the same bit for bit, the outputs agree to the attention tolerance, and turning the
    form on again brings the single launch's own bits back."""
    wl = gen.CFG1.scaled(n_layers=1, batch=B, t_range=(5000, 7000), budgets=(1024,), dtype=dtype)
    inp = gen.ragged_inputs(wl, seed=23, device=U.DEV, resident_layers=1)
    H, Hq, D = wl.n_kv_heads, wl.n_q_heads, wl.head_dim
    T, S = int(inp.cu_tok[-1]), int(inp.cu_sent[-1])
    d = [U.i32(x) for x in (inp.cu_tok, inp.cu_sent, inp.sent_off, inp.sent_len, inp.budget)]
    ctx = U.make_ctx(wl, T, S, 1024, batch=B)
    sv = torch.zeros(1, H, S, D, device=U.DEV)
    ctx.build_semvec(inp.K, U.i32(gen.offsets_of(inp.sent_len)), S, sv)

    def run():
        out = torch.full((B, Hq, D), 3.0, device=U.DEV)
        lse = torch.full((B, Hq), 3.0, device=U.DEV)
        tok_idx = U.empty_i32(B, H, 1024, fill=-1)
        n_tok = U.empty_i32(B, H, fill=-1)
        ctx.decode_step(0, B, inp.q[0], inp.q[0], inp.K, inp.V, T, sv, S, *d, out, lse, tok_idx, n_tok)
        torch.cuda.synchronize()
        return out, lse, tok_idx, n_tok

    one = run()
    ctx.set_single_launch(False)
    _say("single launch off, B", B, dtype)
    two = run()
    assert torch.equal(one[2], two[2]) and torch.equal(one[3], two[3])
    assert (one[0] - two[0]).abs().max().item() <= ATT_TOL[dtype] and (one[1] - two[1]).abs().max().item() <= ATT_TOL[dtype]
    ctx.set_single_launch(True)
    again = run()
    for a, b in zip(one, again):
        assert torch.equal(a, b)


# ----------------------------------------------------------------------------- local window merge, equal chunks

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_decode_plus_local_window_merge(U, oracle32, dtype):
    """Retrieved prompt tokens (fused decode step) merged by lse with a contiguous window of recent tokens attended by
    skv_attend: equals the oracle's attention over the union of both token sets; empty sides handled."""
    wl = gen.CFG1.scaled(n_layers=1, n_tokens=5000, dtype=dtype)
    inp = gen.decode_inputs(wl, seed=21, device=U.DEV)
    S, T, H, Hq, D, budget, W = len(inp.lengths), wl.n_tokens, wl.n_kv_heads, wl.n_q_heads, 128, 512, 100
    ctx = U.make_ctx(wl, T, S, budget)
    sv = torch.zeros(1, H, S, D, dtype=torch.float32, device=U.DEV)
    ctx.build_semvec(inp.K, U.i32(inp.sent_off), S, sv)
    q = inp.q[0]
    g = torch.Generator(device=U.DEV).manual_seed(5)
    Kw = torch.randn(H, budget, D, generator=g, device=U.DEV).to(wl.torch_dtype)      # the window's rows (first W used)
    Vw = torch.randn(H, budget, D, generator=g, device=U.DEV).to(wl.torch_dtype)
    out_r, lse_r = torch.zeros(Hq, D, device=U.DEV), torch.zeros(Hq, device=U.DEV)
    out_w, lse_w = torch.zeros(Hq, D, device=U.DEV), torch.zeros(Hq, device=U.DEV)
    out, lse = torch.zeros(Hq, D, device=U.DEV), torch.zeros(Hq, device=U.DEV)
    tok_idx, n_tok = U.empty_i32(H, budget, fill=-1), U.empty_i32(8, fill=-5)
    for w_len, bud in ((W, budget), (0, budget), (W, 2)):                                # both, window empty, retrieval empty
        _say("local window merge", dtype, "window", w_len, "budget", bud)
        ctx.decode_step(0, 1, q, q, inp.K, inp.V, T, sv, S, U.i32([0, T]), U.i32([0, S]), U.i32(inp.sent_off),
                        U.i32(inp.lengths), U.i32([bud]), out_r, lse_r, tok_idx, n_tok)
        ctx.attend(q, Kw, Vw, U.i32([w_len] * 8), budget, out_w, lse_w)
        ctx.merge_lse(Hq, out_r, lse_r, out_w, lse_w, out, lse)
        torch.cuda.synchronize()
        nt, ti = n_tok.cpu().numpy()[:H], tok_idx.cpu().numpy()
        K, V = gen.to_numpy(inp.K[0]), gen.to_numpy(inp.V[0])
        Ks = np.zeros((H, budget + W, D), dtype=K.dtype)
        Vs = np.zeros_like(Ks)
        for h in range(H):                                             # union: the GPU's retrieved rows, then the window
            Ks[h, :nt[h]], Vs[h, :nt[h]] = K[h, ti[h, :nt[h]]], V[h, ti[h, :nt[h]]]
            Ks[h, nt[h]:nt[h] + w_len], Vs[h, nt[h]:nt[h] + w_len] = U.np_of(Kw[h, :w_len]), U.np_of(Vw[h, :w_len])
        ref, lref = oracle32.attend(U.np_of(q), Ks, Vs, (nt + w_len).astype(np.int32))
        assert np.abs(out.cpu().numpy() - ref).max() <= ATT_TOL[dtype]
        fin = np.isfinite(lref)
        assert np.array_equal(np.isfinite(lse.cpu().numpy()), fin)
        assert np.abs(lse.cpu().numpy()[fin] - lref[fin]).max() <= ATT_TOL[dtype]
        # the merge itself against the oracle's merge of the GPU's partial results: fp32 arithmetic on both sides
        m_ref, ml_ref = oracle32.merge_lse(out_r.cpu().numpy(), lse_r.cpu().numpy(), out_w.cpu().numpy(), lse_w.cpu().numpy())
        assert np.abs(out.cpu().numpy() - m_ref).max() <= 1e-5
    # both sides empty
    ctx.decode_step(0, 1, q, q, inp.K, inp.V, T, sv, S, U.i32([0, T]), U.i32([0, S]), U.i32(inp.sent_off),
                    U.i32(inp.lengths), U.i32([2]), out_r, lse_r, None, None)
    ctx.attend(q, Kw, Vw, U.i32([0] * 8), budget, out_w, lse_w)
    out.fill_(9.0)
    ctx.merge_lse(Hq, out_r, lse_r, out_w, lse_w, out, lse)
    torch.cuda.synchronize()
    assert torch.all(out == 0) and torch.all(torch.isinf(lse) & (lse < 0))


def test_equal_size_chunk_mode(U, oracle32):
    """The paper's equal-size-chunk ablation is the same path with uniform bucket offsets (16-token chunks)."""
    wl = gen.CFG1.scaled(n_layers=1, n_tokens=4096 + 7, len_dist=("fixed", 16))
    _chain_case(U, oracle32, wl, seed=23, budget=512)
    _fused_case(U, oracle32, wl.scaled(batch=1, t_range=(4103, 4103), budgets=(512,)), seed=23, layers=[0])


# ----------------------------------------------------------------------------- bf16 table of mean key vectors

@pytest.mark.parametrize("sv_dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_reduced_semvec_table_chain(U, oracle32, dtype, sv_dtype):
    """Mixed-precision sentence vectors (semvec_dtype = bf16 or E4M3): table within one step of the oracle's, scores from
    the GPU's own table to the usual tolerance, selection bit-exact on those scores, through the 4-call chain."""
    wl = gen.CFG1.scaled(n_layers=2, n_tokens=9000, dtype=dtype)
    _chain_case(U, oracle32, wl, seed=31, budget=700, sv_dtype=sv_dtype)


@pytest.mark.parametrize("sv_dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("Hq,B", [(32, 1), (64, 9), (8, 3), (16, 2)])
def test_reduced_semvec_table_fused(U, oracle32, Hq, B, sv_dtype):
    """The fused decode step (single sequence, small batch, batch path) on a reduced table, every group size."""
    wl = gen.CFG4.scaled(n_layers=1, n_q_heads=Hq, batch=B, t_range=(300, 3500), budgets=(600,))
    _fused_case(U, oracle32, wl, seed=33, layers=[0], sv_dtype=sv_dtype)


def test_e4m3_table_every_code_scores_like_the_oracle(U, oracle32):
    """A hand-filled E4M3 table holding every finite code (both signs, subnormals, 448) scored by the GPU and by the oracle:
    pins the kernel's decoding of the format, for bf16 and fp32 queries."""
    H, S, D = 2, 37, 128
    codes = np.array([c for c in range(256) if (c & 0x7f) != 0x7f], dtype=np.uint8)
    rng = np.random.default_rng(3)
    table = codes[rng.integers(0, len(codes), size=(1, H, S, D))]
    table[0, 0].reshape(-1)[:len(codes)] = codes                          # every code at least once, in order
    for dtype in ("bf16", "f32"):
        wl = gen.CFG1.scaled(n_layers=1, n_q_heads=8, n_kv_heads=H, n_tokens=64, dtype=dtype)
        ctx = U.make_ctx(wl, 64, S, 8, sv_dtype="fp8")
        q = gen.queries(1, 8, D, wl.torch_dtype, 5, U.DEV)[0]
        score = torch.zeros(H, S, device=U.DEV)
        ctx.score(0, q, torch.from_numpy(table).to(U.DEV), S, score)
        torch.cuda.synchronize()
        ref = oracle32.score(gen.to_numpy(q), table[0])
        assert np.all(np.abs(score.cpu().numpy() - ref) <= U.score_tolerance(ref))


@pytest.mark.parametrize("dtype,B", [("bf16", 1), ("f32", 1), ("bf16", 3)])
def test_fused_many_buckets_per_sequence(U, oracle32, dtype, B):
    """More than 1024 buckets per sequence: the step runs 128-token split blocks (two 64-position pieces per block,
    buckets spanning both pieces) and the selection with up to 6 buckets per thread in registers."""
    wl = gen.CFG1.scaled(n_layers=1, batch=B, t_range=(5800, 6400), budgets=(700,), len_dist=("uniform", 1, 3), dtype=dtype)
    _fused_case(U, oracle32, wl, seed=41, layers=[0])
    wl = gen.CFG1.scaled(n_layers=1, batch=B, t_range=(9000, 9100), budgets=(130,), len_dist=("uniform", 1, 200), dtype=dtype)
    _fused_case(U, oracle32, wl, seed=42, layers=[0])          # few, long buckets: S small, 64-token blocks; long spans
    wl = gen.CFG1.scaled(n_layers=1, batch=B, t_range=(40000, 40100), budgets=(1000,), len_dist=("uniform", 1, 30), dtype=dtype)
    _fused_case(U, oracle32, wl, seed=43, layers=[0])          # S > 2048 with buckets that span the 64-position pieces
    wl = gen.CFG1.scaled(n_layers=1, batch=B, t_range=(16000, 16500), budgets=(600,), len_dist=("uniform", 1, 3), dtype=dtype)
    _fused_case(U, oracle32, wl, seed=44, layers=[0])          # S > 6144: buckets beyond the six a thread keeps in registers


# ----------------------------------------------------------------------------- seeded sweeps over shapes

_LEN_DISTS = [("uniform", 1, 3), ("uniform", 8, 40), ("lognormal", 20, 0.7, 3, 120), ("uniform", 1, 300)]


@pytest.mark.parametrize("sweep_seed", [1, 7])
def test_fused_step_seeded_shape_sweep(U, oracle32, sweep_seed):
    """The fused step over a seeded sample of (batch, group size, pool type, table type, budget, context range, bucket
    length distribution): every launch path (single launch, fused and streaming blocks of the two-launch step, the fp32 batch path) with
    shapes no hand-written case has."""
    rng = np.random.default_rng(sweep_seed)
    for it in range(14):
        B = int(rng.choice([1, 2, 3, 8, 9, 16, 20]))
        Hq = int(rng.choice([8, 16, 32, 64]))
        dtype = str(rng.choice(["bf16", "bf16", "f32"]))
        sv = str(rng.choice(["f32", "bf16", "fp8"]))
        budget = int(rng.choice([1, 17, 64, 200, 700, 1024, 1100, 2048, 3000]))
        lo = int(rng.choice([1, 50, 400, 2000]))
        hi = lo + int(rng.choice([0, 100, 3000, 9000]))
        if B >= 16:
            hi = min(hi, 3000)
        ld = _LEN_DISTS[int(rng.integers(0, 4))]
        wl = gen.CFG4.scaled(n_layers=1, n_q_heads=Hq, batch=B, t_range=(lo, hi), budgets=(budget,), dtype=dtype, len_dist=ld)
        _say(f"sweep {sweep_seed}/{it}: B={B} Hq={Hq} {dtype} table={sv} budget={budget} T=[{lo},{hi}] len={ld}")
        _fused_case(U, oracle32, wl, seed=100 * sweep_seed + it, layers=[0], sv_dtype=sv)


@pytest.mark.parametrize("sweep_seed", [3, 11])
def test_chain_seeded_shape_sweep(U, oracle32, sweep_seed):
    """The 4-call chain over a seeded sample of head layouts, pool and table types, budgets around the block sizes of the
    attention kernel (64, 128, 256 tokens) and contexts from one token up."""
    rng = np.random.default_rng(sweep_seed)
    for it in range(14):
        Hq, Hkv = [(32, 8), (8, 8), (16, 8), (64, 8), (4, 1), (8, 2)][int(rng.integers(0, 6))]
        dtype = str(rng.choice(["bf16", "bf16", "f32"]))
        sv = str(rng.choice(["f32", "bf16", "fp8"]))
        budget = int(rng.choice([1, 17, 64, 127, 128, 129, 700, 1024, 2048, 4096, 5000]))
        Tn = int(rng.choice([1, 2, 63, 500, 3000, 9000, 20000]))
        ld = _LEN_DISTS[int(rng.integers(0, 4))]
        wl = gen.CFG1.scaled(n_layers=1, n_q_heads=Hq, n_kv_heads=Hkv, n_tokens=Tn, dtype=dtype, len_dist=ld)
        _say(f"sweep {sweep_seed}/{it}: Hq={Hq}/{Hkv} {dtype} table={sv} budget={budget} T={Tn} len={ld}")
        _chain_case(U, oracle32, wl, seed=200 * sweep_seed + it, budget=budget, sv_dtype=sv)


# ----------------------------------------------------------------------------- repeated launches

@pytest.mark.parametrize("case", ["single", "small_batch", "batch_bf16", "batch_f32"])
def test_repeated_launches_reproduce_their_results(U, oracle32, case):
    """The split-K partials and the arrival counter travel between blocks inside one launch: many back-to-back launches
    (nothing but the launches themselves between two checks) must keep reproducing the first result of the same inputs --
    bit for bit where the summation order is fixed, within the attention tolerance for the bf16 batch kernel, whose waves
    take their tiles in arrival order.  (A missing wait for the partial stores before the arrival showed up as wrong outputs
    about once in 1600 launches of the full-size batch.)"""
    wl, iters, exact = {
        "single": (gen.CFG1.scaled(n_layers=1, batch=1, t_range=(32768, 32768), budgets=(2048,)), 1500, True),
        "small_batch": (gen.CFG4.scaled(n_layers=1, batch=3, t_range=(3000, 9000), budgets=(1024,)), 1500, True),
        "batch_bf16": (gen.CFG4.scaled(n_layers=1, t_range=(8192, 32768)), 3000, False),
        "batch_f32": (gen.CFG4.scaled(n_layers=1, dtype="f32", batch=8, t_range=(3000, 9000)), 800, True),
    }[case]
    inp = gen.ragged_inputs(wl, seed=0, device=U.DEV, resident_layers=1)
    B, H, Hq, D = wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.head_dim
    T_total, S_total = int(inp.cu_tok[-1]), int(inp.cu_sent[-1])
    budget = int(inp.budget.max())
    ctx = U.make_ctx(wl, T_total, S_total, budget, batch=B)
    sv = torch.zeros(1, H, S_total, D, device=U.DEV)
    ctx.build_semvec(inp.K, U.i32(gen.offsets_of(inp.sent_len)), S_total, sv)
    d = [U.i32(x) for x in (inp.cu_tok, inp.cu_sent, inp.sent_off, inp.sent_len, inp.budget)]
    NQ = 4
    q = gen.queries(NQ * B, Hq, D, wl.torch_dtype, 1, U.DEV).view(NQ, B, Hq, D)
    out = torch.empty(B, Hq, D, device=U.DEV)
    lse = torch.empty(B, Hq, device=U.DEV)
    nt = U.empty_i32(B, H, fill=-1)

    def step(k):
        ctx.decode_step(0, B, q[k], q[k], inp.K, inp.V, T_total, sv, S_total, *d, out, lse, None, nt)

    ref = []
    for k in range(NQ):
        step(k)
        torch.cuda.synchronize()
        ref.append((out.clone(), lse.clone(), nt.clone()))
    _say("repeated launches:", case, "B", B, "tokens", T_total, "iters", iters)
    for it in range(iters):
        step(it % NQ)
        if it % 8 == 7 or it == iters - 1:
            torch.cuda.synchronize()
            o, l, n = ref[it % NQ]
            assert torch.equal(nt, n), it
            if exact:
                assert torch.equal(out, o) and torch.equal(lse, l), it
            else:
                assert float((out - o).abs().max()) <= ATT_TOL[wl.dtype] / 4, it
                assert float((lse - l).abs().max()) <= ATT_TOL[wl.dtype] / 4, it
