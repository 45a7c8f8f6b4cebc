"""Pins for the oracle's decode steps: similarity score (Sec. 4.2), ranking + budgeted retrieval
(Sec. 4.2, App. "Effect of Sentence Length"), K/V load (Alg. 1) and sparse attention (Eq. 3).

Independent references used here: float64 brute force from the RAW keys (linearity of the mean),
hand-worked selection cases from tests/golden, an O(S^2) characterisation of the selection that
uses no sort, and dense softmax attention in float64 (the budget covers the whole context).
"""
import math
import os

import numpy as np
import pytest
import torch

from workload import gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _randn(shape, seed, dtype=torch.float32):
    return torch.randn(*shape, generator=torch.Generator().manual_seed(seed)).to(dtype)


# ----------------------------------------------------------------------------- score

@pytest.mark.parametrize("dtype,G", [(torch.float32, 4), (torch.bfloat16, 4), (torch.bfloat16, 8), (torch.float32, 1)])
def test_score_equals_mean_of_raw_key_dots(oracle32, dtype, G):
    """q-bar^T k-bar = (1/len) sum_x q-bar^T k_x, summed over the G heads of the group."""
    H, D = 2, 128
    lens = np.array([3, 1, 40, 7, 25, 12], dtype=np.int32)
    off = gen.offsets_of(lens)
    K = _randn((1, H, int(lens.sum()), D), 21, dtype)
    q = _randn((H * G, D), 22, dtype)
    sv = oracle32.semvec(gen.to_numpy(K), off)[0]
    got = oracle32.score(gen.to_numpy(q), sv)
    Kd, qd = K[0].to(torch.float64).numpy(), q.to(torch.float64).numpy()
    for h in range(H):
        qsum = qd[h * G:(h + 1) * G].sum(axis=0)
        for s in range(len(lens)):
            want = (Kd[h, off[s]:off[s + 1]] @ qsum).mean()
            mag = np.abs(Kd[h, off[s]:off[s + 1]]).mean(axis=0) @ np.abs(qd[h * G:(h + 1) * G]).sum(axis=0)
            assert abs(got[h, s] - want) <= 1e-5 * abs(want) + 2e-6 * mag


def test_score_special_queries(oracle32):
    H, G, D, S = 3, 4, 128, 10
    sv = _randn((H, S, D), 5).numpy()
    assert np.all(oracle32.score(np.zeros((H * G, D), np.float32), sv) == 0.0)
    # a one-hot query in one head of the group picks one coordinate of k-bar; no scaling is applied
    for (j, d) in [(0, 0), (5, 17), (11, 127)]:
        q = np.zeros((H * G, D), np.float32)
        q[j, d] = 2.0
        sc = oracle32.score(q, sv)
        want = np.zeros((H, S), np.float32)
        want[j // G] = 2.0 * sv[j // G, :, d]
        assert np.array_equal(sc, want)
    # heads of one group add up; heads of other groups do not leak in
    q = np.zeros((H * G, D), np.float32)
    q[4:8, 3] = 1.0
    sc = oracle32.score(q, sv)
    assert np.allclose(sc[1], 4.0 * sv[1, :, 3], rtol=1e-6) and np.all(sc[0] == 0) and np.all(sc[2] == 0)


# ----------------------------------------------------------------------------- select

def _select_cases():
    out = []
    for line in open(os.path.join(GOLDEN, "select_cases.txt")):
        if line.startswith("#") or ";" not in line:
            continue
        sc, ln, b, want = [x.strip() for x in line.rstrip("\n").split(";")]
        out.append(([float(x) for x in sc.split()], [int(x) for x in ln.split()], int(b),
                    [int(x) for x in want.split()]))
    return out


@pytest.mark.parametrize("scores,lens,budget,want", _select_cases())
def test_select_hand_worked_cases(oracle32, scores, lens, budget, want):
    lens = np.array(lens, dtype=np.int32)
    off = gen.offsets_of(lens)
    sel, n_sel, tok_idx, n_tok = oracle32.select(np.array([scores], dtype=np.float32), off, lens, budget,
                                                 budget_stride=max(budget, 1))
    assert n_sel[0] == len(want)
    assert sel[0, :n_sel[0]].tolist() == want
    toks = [x for s in want for x in range(off[s], off[s + 1])]
    assert n_tok[0] == len(toks) and tok_idx[0, :n_tok[0]].tolist() == toks


def _selected_without_sorting(score, lens, budget):
    """Bucket i is in the retrieved prefix iff the buckets ranked before it, plus itself, fit the budget
    (lengths are positive, so the running total along the ranking is increasing)."""
    S = len(score)
    chosen = []
    for i in range(S):
        ahead = 0
        for j in range(S):
            better = (score[j] > score[i]) or (score[j] == score[i] and j < i)
            if better:
                ahead += int(lens[j])
        if ahead + int(lens[i]) <= budget:
            chosen.append(i)
    return chosen


def test_select_matches_sort_free_characterisation_on_random_inputs(oracle32):
    rng = np.random.default_rng(7)
    for trial in range(300):
        S = int(rng.integers(1, 40))
        lens = rng.integers(1, 12, size=S).astype(np.int32)
        # coarse scores force many exact ties
        score = (rng.integers(-4, 5, size=(3, S)) / 2.0).astype(np.float32)
        if trial % 3 == 0:
            score = rng.standard_normal((3, S)).astype(np.float32)
        budget = int(rng.integers(0, lens.sum() + 5))
        off = gen.offsets_of(lens)
        sel, n_sel, tok_idx, n_tok = oracle32.select(score, off, lens, budget, budget_stride=max(budget, 1))
        for h in range(3):
            want = _selected_without_sorting(score[h], lens, budget)
            assert sel[h, :n_sel[h]].tolist() == want, (trial, h)
            assert n_tok[h] == sum(int(lens[s]) for s in want)


def test_select_invariants_on_workload_shapes(oracle32):
    lens = gen.sentence_lengths(gen.CFG1.len_dist, 32768, seed=2)
    off = gen.offsets_of(lens)
    S = len(lens)
    score = np.random.default_rng(3).standard_normal((8, S)).astype(np.float32)
    for budget in (1024, 2048):
        sel, n_sel, tok_idx, n_tok = oracle32.select(score, off, lens, budget)
        for h in range(8):
            ids = sel[h, :n_sel[h]]
            t = tok_idx[h, :n_tok[h]]
            assert n_tok[h] <= budget                                   # budget never exceeded
            assert np.all(np.diff(ids) > 0) and np.all(np.diff(t) > 0)  # ascending, no duplicates
            assert n_tok[h] == lens[ids].sum()                          # whole sentences only
            assert np.array_equal(t, np.concatenate([np.arange(off[s], off[s + 1]) for s in ids]))
            order = np.lexsort((np.arange(S), -score[h].astype(np.float64)))
            assert set(order[:n_sel[h]].tolist()) == set(ids.tolist())  # a prefix of the ranking
            if n_sel[h] < S:                                            # maximal: the next bucket overflows
                assert n_tok[h] + lens[order[n_sel[h]]] > budget
    # budget >= context: everything is taken and tok_idx is the identity
    sel, n_sel, tok_idx, n_tok = oracle32.select(score[:1], off, lens, 40000)
    assert n_sel[0] == S and n_tok[0] == 32768 and np.array_equal(tok_idx[0, :32768], np.arange(32768))


def test_select_empty_inputs(oracle32):
    sel, n_sel, tok_idx, n_tok = oracle32.select(np.zeros((2, 0), np.float32), np.zeros(1, np.int32),
                                                 np.zeros(0, np.int32), 16)
    assert n_sel.tolist() == [0, 0] and n_tok.tolist() == [0, 0]


# ----------------------------------------------------------------------------- gather

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_gather_is_direct_indexing(oracle32, dtype):
    H, T, D = 3, 50, 128
    pool = _randn((H, T, D), 9, dtype)
    tok_idx = np.full((H, 16), -1, dtype=np.int32)
    n_tok = np.array([16, 0, 5], dtype=np.int32)
    rng = np.random.default_rng(1)
    for h in range(H):
        tok_idx[h, :n_tok[h]] = np.sort(rng.choice(T, size=n_tok[h], replace=False))
    got = oracle32.gather(gen.to_numpy(pool), tok_idx, n_tok)
    ref = gen.to_numpy(pool)
    for h in range(H):
        assert np.array_equal(got[h, :n_tok[h]], ref[h, tok_idx[h, :n_tok[h]]])
        assert not got[h, n_tok[h]:].any()


# ----------------------------------------------------------------------------- attend

def _dense_attention64(q, K, V, G):
    """Textbook softmax(q K^T / sqrt(d)) V in float64, q head j on KV head j // G."""
    Hq, D = q.shape
    out = np.zeros((Hq, D))
    lse = np.zeros(Hq)
    for j in range(Hq):
        logits = K[j // G] @ q[j] / math.sqrt(D)
        m = logits.max()
        p = np.exp(logits - m)
        out[j] = (p[:, None] * V[j // G]).sum(axis=0) / p.sum()
        lse[j] = m + math.log(p.sum())
    return out, lse


@pytest.mark.parametrize("dtype,tol", [(torch.float32, 2e-5), (torch.bfloat16, 2e-5)])
def test_full_budget_chain_equals_dense_attention(oracle32, oracle64, dtype, tol):
    """Budget >= context: score -> select -> gather -> attend must reproduce plain dense attention."""
    wl = gen.CFG0.scaled(n_tokens=700, dtype="f32" if dtype == torch.float32 else "bf16")
    inp = gen.decode_inputs(wl, seed=4)
    K, V, q = gen.to_numpy(inp.K[0]), gen.to_numpy(inp.V[0]), gen.to_numpy(inp.q[0])
    want, want_lse = _dense_attention64(inp.q[0].double().numpy(), inp.K[0].double().numpy(),
                                        inp.V[0].double().numpy(), wl.group)
    for orc, t in ((oracle32, tol), (oracle64, 1e-6)):
        sv = orc.semvec(K[None], inp.sent_off)[0]
        r = orc.decode_step(q, q, K, V, sv, inp.sent_off, inp.lengths, budget=700)
        assert r["n_tok"].tolist() == [700] * wl.n_kv_heads
        assert np.abs(r["out"] - want).max() <= t
        assert np.abs(r["lse"] - want_lse).max() <= 10 * t


def test_attend_on_a_subset_equals_dense_attention_on_that_subset(oracle32):
    H, G, D, T = 2, 4, 128, 300
    K, V, q = _randn((H, T, D), 1), _randn((H, T, D), 2), _randn((H * G, D), 3)
    rng = np.random.default_rng(0)
    n_tok = np.array([37, 120], dtype=np.int32)
    tok_idx = np.full((H, 128), -1, dtype=np.int32)
    for h in range(H):
        tok_idx[h, :n_tok[h]] = np.sort(rng.choice(T, size=n_tok[h], replace=False))
    Ks, Vs = oracle32.gather(K.numpy(), tok_idx, n_tok), oracle32.gather(V.numpy(), tok_idx, n_tok)
    out, lse = oracle32.attend(q.numpy(), Ks, Vs, n_tok)
    for h in range(H):
        idx = tok_idx[h, :n_tok[h]]
        want, want_lse = _dense_attention64(q[h * G:(h + 1) * G].double().numpy(), K[h:h + 1, idx].double().numpy(),
                                            V[h:h + 1, idx].double().numpy(), G)
        assert np.abs(out[h * G:(h + 1) * G] - want).max() <= 2e-5
        assert np.abs(lse[h * G:(h + 1) * G] - want_lse).max() <= 2e-5


def test_attend_special_cases(oracle32):
    H, G, D = 2, 4, 128
    q = _randn((H * G, D), 3).numpy()
    V = _randn((H, 8, D), 4).numpy()
    K = _randn((H, 8, D), 5).numpy()
    # one token: the output is its value row exactly and lse is its logit
    out, lse = oracle32.attend(q, K, V, np.array([1, 1], np.int32))
    for j in range(H * G):
        assert np.array_equal(out[j], V[j // G, 0])
        assert abs(lse[j] - float(K[j // G, 0].astype(np.float64) @ q[j] / math.sqrt(D))) < 1e-5
    # equal keys: uniform weights, the output is the mean of the values
    Keq = np.broadcast_to(K[:, :1], K.shape).copy()
    out, _ = oracle32.attend(q, Keq, V, np.array([8, 5], np.int32))
    assert np.allclose(out[0], V[0, :8].mean(axis=0), atol=1e-6)
    assert np.allclose(out[G], V[1, :5].mean(axis=0), atol=1e-6)
    # empty selection
    out, lse = oracle32.attend(q, K, V, np.array([0, 3], np.int32))
    assert not out[:G].any() and np.all(np.isneginf(lse[:G])) and np.isfinite(lse[G:]).all()
    # the 1/sqrt(d) factor: scaling q by c and K by 1/c changes nothing; a missing scale would
    # show against the float64 dense reference above, a doubled one here
    out1, _ = oracle32.attend(q, K, V, np.array([8, 8], np.int32))
    out2, _ = oracle32.attend(q * 2, K / 2, V, np.array([8, 8], np.int32))
    assert np.allclose(out1, out2, atol=1e-6)
    # order of the gathered tokens does not matter beyond rounding
    perm = np.random.default_rng(0).permutation(8)
    out3, _ = oracle32.attend(q, K[:, perm], V[:, perm], np.array([8, 8], np.int32))
    assert np.allclose(out1, out3, atol=1e-6)


# ----------------------------------------------------------------------------- figures the paper prints

def test_pool_bytes_per_token_reproduce_the_papers_kv_cache_size():
    kv = {}
    for line in open(os.path.join(GOLDEN, "paper_byte_accounting.txt")):
        if line.startswith("#") or "=" not in line:
            continue
        k, v = line.strip().split("=")
        kv[k] = float(v)
    wl = gen.CFG1
    assert (wl.n_layers, wl.n_kv_heads, wl.head_dim, wl.elt_bytes) == (kv["layers"], kv["kv_heads"], kv["head_dim"],
                                                                      kv["elt_bytes"])
    per_token = wl.n_layers * wl.n_kv_heads * wl.head_dim * 2 * wl.elt_bytes
    assert abs(per_token * kv["context_tokens_256k"] / 1e9 - kv["kv_cache_gb_256k"]) < 0.01
    assert math.floor(kv["r"] * kv["tau"]) == kv["retained"]


# ----------------------------------------------------------------------------- merge of partial results

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_merge_lse_equals_attention_over_the_union(oracle32, oracle64, dtype):
    """Eq. 3 over A u B from the two partial results == Eq. 3 computed on the concatenated rows."""
    Hq, H, D, nA, nB = 8, 2, 128, 37, 90
    q = _randn((Hq, D), 40, dtype)
    K, V = _randn((H, nA + nB, D), 41, dtype), _randn((H, nA + nB, D), 42, dtype)
    qn, Kn, Vn = gen.to_numpy(q), gen.to_numpy(K), gen.to_numpy(V)
    for o, tol in ((oracle64, 2e-6), (oracle32, 2e-5)):
        oa, la = o.attend(qn, np.ascontiguousarray(Kn[:, :nA]), np.ascontiguousarray(Vn[:, :nA]), np.full(H, nA, np.int32))
        ob, lb = o.attend(qn, np.ascontiguousarray(Kn[:, nA:]), np.ascontiguousarray(Vn[:, nA:]), np.full(H, nB, np.int32))
        want, lw = o.attend(qn, Kn, Vn, np.full(H, nA + nB, np.int32))
        got, lg = o.merge_lse(oa, la, ob, lb)
        assert np.abs(got - want).max() <= tol and np.abs(lg - lw).max() <= tol * 10
    # against scipy on the raw logits
    from scipy.special import logsumexp
    logits = np.einsum("jd,jtd->jt", q.double().numpy(), K.double().numpy()[np.repeat(np.arange(H), Hq // H)]) / math.sqrt(D)
    assert np.abs(lg - logsumexp(logits, axis=1)).max() <= 1e-4


def test_merge_lse_empty_sides(oracle32):
    rng = np.random.default_rng(3)
    oa, ob = rng.standard_normal((4, 128)).astype(np.float32), rng.standard_normal((4, 128)).astype(np.float32)
    la = np.array([0.5, -np.inf, -np.inf, 3.0], np.float32)
    lb = np.array([-np.inf, 1.5, -np.inf, 3.0], np.float32)
    oa[1] = np.nan                                                # an empty side's output must not leak, whatever it holds
    out, lse = oracle32.merge_lse(oa, la, ob, lb)
    assert np.array_equal(out[0], oa[0]) and lse[0] == np.float32(0.5)
    assert np.array_equal(out[1], ob[1]) and lse[1] == np.float32(1.5)
    assert np.all(out[2] == 0) and lse[2] == -np.inf
    assert np.allclose(out[3], 0.5 * (oa[3] + ob[3]), atol=1e-6) and abs(lse[3] - (3.0 + math.log(2.0))) < 1e-6
