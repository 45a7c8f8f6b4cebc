"""Pins for the oracle's sentence query cache (Sec. 4.2 "Sentence-level query aggregation", Eq. 2; Alg. 1
decoding phase).

Independent references: hand-worked runs in tests/golden/query_cache_cases.txt, numpy float64 means over the
slices between terminators (computed from the raw queries, no running state), torch's own float32 -> bfloat16
conversion for the storage rounding, and closed forms (one query, constant queries, 1..n).
"""
import os

import numpy as np
import pytest
import torch

from workload import gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
TERM, OTHER, VOCAB = 7, 3, 64


def _bitmap():
    bm = np.zeros(2, dtype=np.uint32)
    bm[0] = 1 << TERM
    return bm


def _cases():
    out = []
    for line in open(os.path.join(GOLDEN, "query_cache_cases.txt")):
        line = line.rstrip("\n")
        if not line or line.startswith("#"):
            continue
        stream, qs, ns, means = line.split("|")
        out.append((stream, [float(x) for x in qs.split(",")], [int(x) for x in ns.split(",")],
                    [float(x) for x in means.split(",")]))
    return out


@pytest.mark.parametrize("stream,qs,ns,means", _cases(), ids=[c[0] for c in _cases()])
@pytest.mark.parametrize("real", ["f32", "f64"])
def test_hand_worked_runs(oracle32, oracle64, real, stream, qs, ns, means):
    o = oracle32 if real == "f32" else oracle64
    per = 8
    cache = o.query_cache(per, cap=16)
    for c, q, n, m in zip(stream, qs, ns, means):
        before = len(cache)
        qbar, store = cache.step(np.full(per, q, dtype=np.float32), TERM if c == "." else OTHER, _bitmap(), VOCAB)
        assert before + 1 == n                                   # |Q_s| the mean was taken over
        assert np.array_equal(qbar, np.full(per, m, dtype=np.float32)), (c, q, qbar[0], m)   # small dyadic values: exact
        assert np.array_equal(store, qbar)
        assert len(cache) == (0 if c == "." else n)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_mean_equals_float64_slice_mean(oracle32, oracle64, dtype):
    """q-bar at step t = float64 mean of the raw queries since the last boundary (no running state)."""
    per, n_steps = 2 * 128, 60
    q = torch.randn(n_steps, per, generator=torch.Generator().manual_seed(3)).to(dtype)
    rng = np.random.default_rng(4)
    is_term = rng.random(n_steps) < 0.15
    is_term[10] = is_term[11] = True                             # a run of terminators
    qd = q.to(torch.float64).numpy()
    c32, c64 = oracle32.query_cache(per, 64), oracle64.query_cache(per, 64)
    start = 0
    for t in range(n_steps):
        tok = TERM if is_term[t] else OTHER
        m32, _ = c32.step(gen.to_numpy(q[t]), tok, _bitmap(), VOCAB)
        m64, _ = c64.step(gen.to_numpy(q[t]), tok, _bitmap(), VOCAB)
        want = qd[start:t + 1].mean(axis=0)
        n = t + 1 - start
        scale = np.abs(qd[start:t + 1]).sum(axis=0) / n
        assert np.all(np.abs(m64 - want) <= 2.0 ** -23 * np.maximum(np.abs(want), 1e-30) + 1e-30)   # one float rounding
        assert np.all(np.abs(m32 - want) <= (n + 1) * 2.0 ** -24 * scale + 1e-30)                    # n float adds + divide
        if is_term[t]:
            start = t + 1
    assert start > 0                                             # the run did cross sentence boundaries


def test_single_query_is_returned_exactly(oracle32):
    q = torch.randn(4 * 128, generator=torch.Generator().manual_seed(5))
    for dtype in (torch.float32, torch.bfloat16):
        x = gen.to_numpy(q.to(dtype))
        qbar, store = oracle32.query_cache(x.size).step(x, OTHER, _bitmap(), VOCAB)
        assert np.array_equal(store, x)
        assert np.array_equal(qbar, q.to(dtype).float().numpy())


def test_constant_and_arithmetic_sequences(oracle32):
    """n equal queries -> that query exactly; queries 1..n -> (n+1)/2."""
    per = 16
    c = oracle32.query_cache(per, 128)
    for t in range(100):
        qbar, _ = c.step(np.full(per, 0.3, dtype=np.float32), OTHER, _bitmap(), VOCAB)
    assert np.allclose(qbar, 0.3, rtol=1e-5)
    c = oracle32.query_cache(per, 128)
    for t in range(1, 101):
        qbar, _ = c.step(np.full(per, float(t), dtype=np.float32), OTHER, _bitmap(), VOCAB)
        assert np.array_equal(qbar, np.full(per, (t + 1) / 2.0, dtype=np.float32))


def test_bf16_storage_rounding_is_torch_round_to_nearest_even(oracle32):
    """The stored q-bar is the float mean rounded once; compared with torch's float32 -> bfloat16 conversion,
    including exact ties (mean of two neighbouring bf16 values) in both parities."""
    per = 4096
    g = torch.Generator().manual_seed(6)
    a = torch.randn(per, generator=g).to(torch.bfloat16)
    bits = a.view(torch.int16).clone()
    b = (bits + 1).view(torch.bfloat16)                          # the next bf16 pattern: (a + b) / 2 is an exact tie
    c = oracle32.query_cache(per, 4)
    c.step(gen.to_numpy(a), OTHER, _bitmap(), VOCAB)
    qbar, store = c.step(gen.to_numpy(b), OTHER, _bitmap(), VOCAB)
    want = torch.from_numpy(qbar).to(torch.bfloat16)
    assert np.array_equal(store, gen.to_numpy(want))
    finite = np.isfinite(qbar)
    ties = (qbar.view(np.uint32) & 0xffff) == 0x8000
    assert finite.all() and ties.sum() > per // 2                # ties were exercised ...
    low_bit = (store & 1)
    assert np.all(low_bit[ties] == 0)                            # ... and went to the even pattern
    # random (non-tie) means too
    c = oracle32.query_cache(per, 4)
    for s in range(3):
        x = torch.randn(per, generator=g).to(torch.bfloat16)
        qbar, store = c.step(gen.to_numpy(x), OTHER, _bitmap(), VOCAB)
    assert np.array_equal(store, gen.to_numpy(torch.from_numpy(qbar).to(torch.bfloat16)))


def test_ids_outside_the_vocabulary_never_reset_and_full_cache_is_an_error(oracle32):
    c = oracle32.query_cache(4, cap=3)
    for tok in (-1, VOCAB, VOCAB + TERM):
        c.step(np.ones(4, dtype=np.float32), tok, _bitmap(), VOCAB)
    assert len(c) == 3
    with pytest.raises(OverflowError):
        c.step(np.ones(4, dtype=np.float32), OTHER, _bitmap(), VOCAB)
    assert len(c) == 3


def test_mean_query_feeds_the_score_linearly(oracle32):
    """Score of q-bar = mean over the sentence so far of the scores of the individual queries (Eq. 2 into the
    similarity of Sec. 4.2) -- ties the cache to the scoring step it feeds."""
    Hq, H, D, S = 8, 2, 128, 11
    g = torch.Generator().manual_seed(8)
    sv = torch.randn(H, S, D, generator=g).numpy()
    qs = torch.randn(5, Hq, D, generator=g)
    c = oracle32.query_cache(Hq * D, 8)
    for t in range(5):
        qbar, _ = c.step(qs[t].numpy(), OTHER, _bitmap(), VOCAB)
    got = oracle32.score(qbar, sv)
    each = np.stack([oracle32.score(qs[t].numpy(), sv).astype(np.float64) for t in range(5)]).mean(axis=0)
    assert np.allclose(got, each, rtol=0, atol=1e-4 * np.abs(each).max())
