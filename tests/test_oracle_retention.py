"""Pins for the oracle's prefill token retention: observation-window importance (Sec. 4.1 "Token importance
measurement"), global top-k retention (Sec. 4.1 "Token selection within sentence buckets", App. "Effect of Sentence
Length") and Eq. 1 over the retained tokens.

Independent references: scipy's softmax on a dense float64 logit matrix with the causal mask written out, the
decomposition of an N-token window into N single-query problems on truncated prompts, closed forms (equal keys),
shift invariance of the softmax, numpy lexsort / bincount / cumsum, an O(n^2) sort-free characterisation, hand-worked
cases in tests/golden/retain_cases.txt.
"""
import os

import numpy as np
import pytest
import torch
from scipy.special import softmax

from workload import gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _randn(shape, seed, dtype=torch.float32):
    return torch.randn(*shape, generator=torch.Generator().manual_seed(seed)).to(dtype)


def _dense_alpha(q, K, N):
    """float64: probabilities of the model's causal attention for the last N queries, summed per prefix token."""
    Hq, _, D = q.shape
    H, T, _ = K.shape
    G, Tp = Hq // H, T - N
    alpha = np.zeros(Tp)
    for j in range(Hq):
        logits = q[j] @ K[j // G].T / np.sqrt(D)                 # [N][T]
        for n in range(N):
            logits[n, Tp + n + 1:] = -np.inf                     # query n sits at position Tp + n
        alpha += softmax(logits, axis=1)[:, :Tp].sum(axis=0)
    return alpha


@pytest.mark.parametrize("dtype,Hq,H,N,T", [(torch.float32, 4, 1, 4, 50), (torch.bfloat16, 8, 2, 32, 200),
                                            (torch.float32, 8, 8, 1, 33), (torch.bfloat16, 16, 2, 7, 64)])
def test_importance_equals_dense_causal_softmax(oracle32, oracle64, dtype, Hq, H, N, T):
    q, K = _randn((Hq, N, 128), 1, dtype), _randn((H, T, 128), 2, dtype)
    want = _dense_alpha(q.double().numpy(), K.double().numpy(), N)
    got64 = oracle64.token_importance(gen.to_numpy(q), gen.to_numpy(K))
    got32 = oracle32.token_importance(gen.to_numpy(q), gen.to_numpy(K))
    assert got32.shape == (T - N,)
    assert np.abs(got64 - want).max() <= 1e-6 * want.max()       # float output of a double computation
    assert np.abs(got32 - want).max() <= 2e-5 * want.max()
    assert abs(want.sum() - Hq * N) < Hq * N                     # a real share of the mass lies on the prefix


def test_importance_window_decomposes_into_single_query_problems(oracle32):
    """alpha of an N-token window = sum over n of the alpha of the one-query problem (query n, keys 0..Tp+n):
    pins the causal mask and the position of each window query."""
    Hq, H, N, T = 4, 2, 5, 40
    Tp = T - N
    q, K = _randn((Hq, N, 128), 3), _randn((H, T, 128), 4)
    full = oracle32.token_importance(q.numpy(), K.numpy())
    parts = np.zeros(Tp)
    for n in range(N):
        a = oracle32.token_importance(q[:, n:n + 1].contiguous().numpy(), K[:, :Tp + n + 1].contiguous().numpy())
        assert a.shape == (Tp + n,)
        parts += a[:Tp].astype(np.float64)
    assert np.abs(full - parts).max() <= 1e-5 * parts.max()
    # a key after the last window query's own position does not exist; the last key matters only to the last query
    K2 = K.clone()
    K2[:, T - 1] += 3.0
    q0 = q.clone()
    q0[:, N - 1] = 0.0                                            # last query uniform over its keys either way
    a1, a2 = oracle32.token_importance(q0.numpy(), K.numpy()), oracle32.token_importance(q0.numpy(), K2.numpy())
    assert np.array_equal(a1, a2)


def test_importance_closed_forms(oracle32, oracle64):
    """All keys equal -> every visible key gets 1/(visible): alpha_i = Hq * sum_n 1/(Tp + n + 1)."""
    Hq, H, N, T = 8, 2, 4, 30
    Tp = T - N
    q = _randn((Hq, N, 128), 5)
    K = _randn((1, 1, 128), 6).expand(H, T, 128).contiguous()
    want = Hq * sum(1.0 / (Tp + n + 1) for n in range(N))
    got = oracle64.token_importance(q.numpy(), K.numpy())
    assert np.allclose(got, want, rtol=1e-6)
    # zero queries: the same uniform weights for any keys
    got = oracle32.token_importance(np.zeros((Hq, N, 128), np.float32), _randn((H, T, 128), 7).numpy())
    assert np.allclose(got, want, rtol=1e-5)


def test_importance_is_invariant_to_a_common_key_shift_and_not_to_scaling(oracle64):
    Hq, H, N, T = 4, 1, 3, 25
    q, K = _randn((Hq, N, 128), 8), _randn((H, T, 128), 9)
    a = oracle64.token_importance(q.numpy(), K.numpy())
    shifted = (K + _randn((1, 1, 128), 10)).contiguous()
    b = oracle64.token_importance(q.numpy(), shifted.numpy())
    assert np.abs(a - b).max() <= 1e-4 * a.max()                 # inputs are float32: the shift rounds
    c = oracle64.token_importance((2 * q).numpy(), K.numpy())    # the 1/sqrt(D) scale is really applied
    want = _dense_alpha((2 * q).double().numpy(), K.double().numpy(), N)
    assert np.abs(c - want).max() <= 1e-6 * want.max() and np.abs(c - a).max() > 1e-3 * a.max()


def test_importance_groups_do_not_leak(oracle32):
    """Query head j only sees KV head floor(j/G)."""
    Hq, H, N, T = 4, 2, 2, 20
    q, K = _randn((Hq, N, 128), 11), _randn((H, T, 128), 12)
    base = oracle32.token_importance(q.numpy(), K.numpy())
    q2 = q.clone()
    q2[2:] = 0                                                    # heads of KV head 1 become uniform
    K2 = K.clone()
    K2[1] = _randn((T, 128), 13)                                  # ... so KV head 1's keys no longer matter
    a = oracle32.token_importance(q2.numpy(), K.numpy())
    b = oracle32.token_importance(q2.numpy(), K2.numpy())
    assert np.array_equal(a, b) and not np.array_equal(a, base)


# ----------------------------------------------------------------------------- retention

def _golden():
    out = []
    for line in open(os.path.join(GOLDEN, "retain_cases.txt")):
        line = line.rstrip("\n")
        if not line or line.startswith("#"):
            continue
        a, seg, k, keep, lens = line.split("|")
        out.append((np.array([float(x) for x in a.split(",")], np.float32), np.array([int(x) for x in seg.split(",")], np.int32),
                    int(k), [int(x) for x in keep.split(",")] if keep else [], [int(x) for x in lens.split(",")]))
    return out


@pytest.mark.parametrize("case", _golden(), ids=[f"case{i}" for i in range(len(_golden()))])
def test_retain_hand_worked(oracle32, case):
    alpha, seg, k, keep, lens = case
    S = int(seg.max()) + 1
    got_keep, off, ln = oracle32.retain(alpha, k, seg, S)
    assert got_keep.tolist() == keep
    assert ln.tolist() == lens
    assert off.tolist() == [0] + np.cumsum(lens).tolist()


@pytest.mark.parametrize("seed", range(6))
def test_retain_equals_numpy_lexsort_and_counting_rule(oracle32, seed):
    rng = np.random.default_rng(seed)
    Tp = int(rng.integers(1, 400))
    alpha = rng.choice(np.array([0.0, 0.25, 0.5, 1.0, 3.0], np.float32), size=Tp) if seed % 2 else rng.random(Tp).astype(np.float32)
    if seed == 3:
        alpha[rng.integers(0, Tp, 5)] = np.nan
    lens = gen.sentence_lengths(("uniform", 1, 9), Tp, seed)
    seg = np.repeat(np.arange(len(lens)), lens).astype(np.int32)
    S = len(lens)
    for k in (0, 1, Tp // 3, Tp - 1, Tp, Tp + 5):
        keep, off, ln = oracle32.retain(alpha, k, seg, S)
        key = np.where(np.isnan(alpha), -np.inf, alpha)
        nanlast = np.isnan(alpha)
        order = np.lexsort((np.arange(Tp), -key, nanlast))       # NaN last, higher alpha first, lower position first
        want = np.sort(order[:min(k, Tp)])
        assert np.array_equal(keep, want)
        # sort-free: token i is kept iff fewer than k tokens rank before it
        for i in rng.integers(0, Tp, 20):
            if np.isnan(alpha[i]):
                before = int((~nanlast).sum() + (nanlast[:i]).sum())
            else:
                before = int(((alpha > alpha[i]) & ~nanlast).sum() + ((alpha[:i] == alpha[i])).sum())
            assert (i in keep) == (before < k)
        assert np.array_equal(ln, np.bincount(seg[keep], minlength=S)) and np.array_equal(off, np.concatenate([[0], np.cumsum(ln)]))


def test_buckets_without_retained_tokens_do_not_exist(oracle32):
    """Selection over the retained pool with zero-length buckets kept in the numbering == selection after deleting
    them; their mean key is stored as zeros; the mean of a surviving bucket is over its retained tokens only."""
    rng = np.random.default_rng(5)
    H, D, T = 2, 128, 300
    lens = gen.sentence_lengths(("uniform", 2, 12), T, 5)
    seg = np.repeat(np.arange(len(lens)), lens).astype(np.int32)
    S = len(lens)
    alpha = rng.random(T).astype(np.float32)
    keep, off, ln = oracle32.retain(alpha, 60, seg, S)
    assert (ln == 0).any() and (ln > 0).any()
    K = _randn((1, H, T, D), 6)
    K_ret = K[:, :, torch.from_numpy(keep).long()].contiguous()
    sv = oracle32.semvec(K_ret.numpy(), off)[0]
    assert np.all(sv[:, ln == 0] == 0)
    Kd = K[0].double().numpy()
    for s in np.flatnonzero(ln > 0)[:10]:
        members = keep[seg[keep] == s]
        assert np.allclose(sv[:, s], Kd[:, members].mean(axis=1), atol=1e-5)
    q = _randn((8, D), 7).numpy()
    sc = oracle32.score(q, sv)
    alive = np.flatnonzero(ln > 0)
    for budget in (5, 17, 40, 1000):
        sel, n_sel, tok, n_tok = oracle32.select(sc, off[:-1], ln, budget)
        off2 = np.concatenate([[0], np.cumsum(ln[alive])]).astype(np.int32)
        sel2, n_sel2, tok2, n_tok2 = oracle32.select(np.ascontiguousarray(sc[:, alive]), off2[:-1], ln[alive], budget)
        assert np.array_equal(n_tok, n_tok2) and np.array_equal(n_sel, n_sel2)
        for h in range(H):
            assert np.array_equal(tok[h, :n_tok[h]], tok2[h, :n_tok2[h]])
            assert np.array_equal(sel[h, :n_sel[h]], alive[sel2[h, :n_sel2[h]]])
            assert np.all(ln[sel[h, :n_sel[h]]] > 0)
