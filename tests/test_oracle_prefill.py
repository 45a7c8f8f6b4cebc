"""Pins for the oracle's prefill steps: sentence segmentation (Sec. 4.1) and mean key vectors (Eq. 1).

None of these checks re-uses the oracle's own loop: they compare against hand-built streams with
written-out answers, numpy's prefix sum, the lengths the generator drew before it built the token
stream, and float64 brute force from the raw keys.
"""
import os

import numpy as np
import pytest
import torch

from workload import gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
VOCAB, TERM = 64, 7          # tiny vocabulary for hand-built streams: id 7 is the only terminator


def _bitmap(vocab, terms):
    w = np.zeros((vocab + 31) // 32, dtype=np.uint32)
    for t in terms:
        w[t // 32] |= np.uint32(1) << np.uint32(t % 32)
    return w


def _stream(text):
    return np.array([TERM if c == "." else 3 for c in text], dtype=np.int32)


def _cases():
    out = []
    for line in open(os.path.join(GOLDEN, "segment_cases.txt")):
        if line.startswith("#") or "|" not in line:
            continue
        text, lens = line.rstrip("\n").split("|")
        out.append((text, [int(x) for x in lens.split(",")] if lens else []))
    return out


@pytest.mark.parametrize("text,lens", _cases())
def test_segment_hand_built_streams(oracle32, text, lens):
    seg_id, off, ln, S = oracle32.segment(_stream(text), _bitmap(VOCAB, [TERM]), VOCAB)
    assert S == len(lens)
    assert ln.tolist() == lens
    starts = [sum(lens[:i]) for i in range(len(lens) + 1)]
    assert off.tolist() == starts
    expect_ids = [s for s, n in enumerate(lens) for _ in range(n)]
    assert seg_id.tolist() == expect_ids


def test_segment_matches_exclusive_prefix_sum_and_invariants(oracle32):
    rng = np.random.default_rng(5)
    bitmap = gen.terminator_bitmap(1000, 20)
    for T in (1, 2, 63, 64, 65, 1000, 4097):
        tok = rng.integers(0, 1000, size=T).astype(np.int32)
        flag = (tok % 20 == 0).astype(np.int64)
        seg_id, off, ln, S = oracle32.segment(tok, bitmap, 1000)
        excl = np.concatenate([[0], np.cumsum(flag)[:-1]])        # textbook exclusive scan
        assert np.array_equal(seg_id, excl)
        assert S == seg_id[-1] + 1
        assert ln.sum() == T and ln.min() >= 1
        assert np.all(np.diff(off) > 0) and off[0] == 0 and off[-1] == T
        assert np.array_equal(np.diff(seg_id), flag[:-1])
        assert np.array_equal(off[1:] - off[:-1], ln)
        # every sentence but possibly the last ends with a terminator and has none inside
        for s in range(S):
            inner = flag[off[s]: off[s + 1] - 1]
            assert inner.sum() == 0
            if s < S - 1:
                assert flag[off[s + 1] - 1] == 1


def test_segment_ignores_ids_outside_vocabulary(oracle32):
    tok = np.array([3, -1, 7, 64, 9999, 7, 2], dtype=np.int32)
    _, off, ln, S = oracle32.segment(tok, _bitmap(VOCAB, [TERM]), VOCAB)
    assert ln.tolist() == [3, 3, 1]


def test_segment_recovers_generator_lengths(oracle32):
    """The generator draws lengths first and only then plants terminators: the segmenter must return them."""
    wl = gen.CFG3.scaled(n_tokens=32768)
    p = gen.prefill_inputs(wl, seed=3, with_keys=False)
    seg_id, off, ln, S = oracle32.segment(p.tok, p.bitmap, wl.vocab)
    assert S == len(p.lengths)
    assert np.array_equal(ln, p.lengths)
    # about 5% of positions are terminators (the contract's probability)
    assert 0.04 < S / wl.n_tokens < 0.06


def test_segment_capacity_overflow_reported(oracle32):
    with pytest.raises(OverflowError):
        oracle32.segment(_stream("a.a.a.a."), _bitmap(VOCAB, [TERM]), VOCAB, cap_sent=3)
    _, off, ln, S = oracle32.segment(_stream("a.a.a.a."), _bitmap(VOCAB, [TERM]), VOCAB, cap_sent=4)
    assert S == 4


# ----------------------------------------------------------------------------- Eq. 1

def _keys(L, H, T, D, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(L, H, T, D, generator=g).to(dtype)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_semvec_equals_float64_brute_force(oracle32, oracle64, dtype):
    lens = np.array([1, 5, 17, 1, 64, 3, 130, 2], dtype=np.int32)
    off = gen.offsets_of(lens)
    K = _keys(2, 3, int(lens.sum()), 128, dtype, 11)
    got = oracle32.semvec(gen.to_numpy(K), off)
    got64 = oracle64.semvec(gen.to_numpy(K), off)
    Kd = K.to(torch.float64).numpy()
    for s in range(len(lens)):
        want = Kd[:, :, off[s]:off[s + 1], :].mean(axis=2)
        assert np.allclose(got[:, :, s, :], want, rtol=1e-6, atol=1e-6)
        assert np.allclose(got64[:, :, s, :], want.astype(np.float32), rtol=0, atol=1e-7)


def test_semvec_special_cases(oracle32):
    D = 128
    # length-1 sentences: the vector is the key itself, bit for bit
    K = _keys(1, 2, 9, D, torch.bfloat16, 2)
    off = np.arange(10, dtype=np.int32)
    sv = oracle32.semvec(gen.to_numpy(K), off)
    assert np.array_equal(sv[0], K[0].to(torch.float32).numpy())
    # constant keys inside a sentence: the mean is that key exactly (sums of n equal floats of
    # few mantissa bits are exact, and x*n/n == x)
    row = torch.randn(D, generator=torch.Generator().manual_seed(4)).to(torch.bfloat16)
    K = row.expand(1, 1, 12, D).contiguous()
    sv = oracle32.semvec(gen.to_numpy(K), np.array([0, 4, 12], dtype=np.int32))
    assert np.array_equal(sv[0, 0, 0], row.to(torch.float32).numpy())
    assert np.array_equal(sv[0, 0, 1], row.to(torch.float32).numpy())
    # a wrong divisor or an off-by-one range would break this: keys 1..n -> mean (n+1)/2
    K = torch.arange(1, 8, dtype=torch.float32).view(1, 1, 7, 1).expand(1, 1, 7, D).contiguous()
    sv = oracle32.semvec(K.numpy(), np.array([0, 3, 7], dtype=np.int32))
    assert np.all(sv[0, 0, 0] == 2.0) and np.all(sv[0, 0, 1] == 5.5)


def test_semvec_tracks_sentence_centres_of_the_synthetic_keys(oracle32):
    """Structure of the workload: key = centre + 0.5*noise, so the mean is within ~4*0.5/sqrt(len) of the centre."""
    lens = gen.sentence_lengths(("uniform", 8, 40), 1024, seed=1)
    K, _ = gen.kv_layer(lens, 2, 128, torch.float32, seed=1, layer=0)
    # regenerate the centres exactly as the generator does (first draw of the layer's stream)
    g = gen._tgen(1, 1000, "cpu")
    centres = torch.randn(2, len(lens), 128, generator=g).numpy()
    sv = oracle32.semvec(K.unsqueeze(0).numpy(), gen.offsets_of(lens))[0]
    bound = 5.0 * 0.5 / np.sqrt(lens.astype(np.float64))
    assert np.all(np.abs(sv - centres).max(axis=2) <= bound[None, :])


# ----------------------------------------------------------------------------- bf16 mean key vectors

def test_bf16_semvec_is_the_float_mean_rounded_once(oracle32):
    """Mixed-precision sentence vectors: the stored bf16 value is torch's float32 -> bfloat16 conversion of the oracle's
    own float mean; scores from the bf16 table equal a float64 dot product with the widened values."""
    import torch
    lens = np.array([3, 1, 40, 7, 25, 12, 2], dtype=np.int32)
    off = gen.offsets_of(lens)
    g = torch.Generator().manual_seed(31)
    K = torch.randn(2, 2, int(lens.sum()), 128, generator=g).to(torch.bfloat16)
    sv32 = oracle32.semvec(gen.to_numpy(K), off)
    sv16 = oracle32.semvec(gen.to_numpy(K), off, sv_dtype="bf16")
    assert sv16.dtype == np.uint16 and sv16.shape == sv32.shape
    assert np.array_equal(sv16, gen.to_numpy(torch.from_numpy(sv32).to(torch.bfloat16)))
    one = lens == 1
    assert np.array_equal(sv16[:, :, one], gen.to_numpy(K)[:, :, off[:-1][one]])          # bf16 keys of length-1 buckets survive exactly
    q = torch.randn(8, 128, generator=g).to(torch.bfloat16)
    got = oracle32.score(gen.to_numpy(q), sv16[0])
    wide = torch.from_numpy(sv16[0].astype(np.int32) << 16).view(torch.float32).double().numpy()
    qd = q.double().numpy()
    want = np.stack([wide[h] @ qd[4 * h:4 * h + 4].sum(axis=0) for h in range(2)])
    assert np.abs(got - want).max() <= 1e-5 * np.abs(want).max()
    # the rounding is really there: the bf16 scores differ from the float-table scores, by about 2^-9 relative per term
    ref = oracle32.score(gen.to_numpy(q), sv32[0])
    d = np.abs(got - ref).max()
    assert 0 < d <= 2.0 ** -7 * np.abs(qd).sum(axis=1).max() * np.abs(sv32).max()


# ----------------------------------------------------------------------------- E4M3 mean key vectors

def _torch_e4m3(x: np.ndarray) -> np.ndarray:
    """torch's float32 -> float8_e4m3fn conversion as codes (nearest, ties to even; NaN beyond the format)."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def test_e4m3_codes_decode_to_the_format_definition(oracle32):
    """All 256 codes against the written-out definition (-1)^s 2^(e-7) (1 + m/8), subnormals m 2^-9, and against torch."""
    import torch
    codes = np.arange(256, dtype=np.uint8)
    got = oracle32.e4m3_decode(codes)
    for c in range(256):
        if (c & 0x7f) == 0x7f:
            continue                                                    # the two NaN codes never occur in a table
        s, e, m = c >> 7, (c >> 3) & 15, c & 7
        want = (m * 2.0 ** -9) if e == 0 else 2.0 ** (e - 7) * (1 + m / 8)
        assert got[c] == (-want if s else want), c
    fin = (codes & 0x7f) != 0x7f
    assert np.array_equal(got[fin], torch.from_numpy(codes).view(torch.float8_e4m3fn).float().numpy()[fin])
    assert got[0x7e] == 448.0 and got[0x01] == 2.0 ** -9


def test_e4m3_rounding_matches_torch_in_range_and_saturates(oracle32):
    rng = np.random.default_rng(5)
    # values over the whole range, every midpoint between neighbouring codes (ties), and values next to the midpoints
    vals = oracle32.e4m3_decode(np.arange(0x7f, dtype=np.uint8)).astype(np.float64)
    mids = (vals[:-1] + vals[1:]) / 2
    x = np.concatenate([rng.normal(0, 1, 20000), rng.normal(0, 60, 20000), rng.uniform(-2.0 ** -6, 2.0 ** -6, 5000), vals, mids,
                        np.nextafter(mids.astype(np.float32), np.float32(0)), np.nextafter(mids.astype(np.float32), np.float32(1e9)),
                        [0.0, -0.0, 448.0, 463.9, 464.0]]).astype(np.float32)
    x = np.concatenate([x, -x])
    x = x[np.abs(x) <= 464.0]                                           # torch turns what lies beyond into NaN
    assert np.array_equal(oracle32.e4m3_encode(x), _torch_e4m3(x))
    # the rule for what does not fit: the largest finite value, sign kept (hand-written cases)
    big = np.array([464.5, 480.0, 1e4, 3e38, -464.5, -1e30], dtype=np.float32)
    assert oracle32.e4m3_encode(big).tolist() == [0x7e, 0x7e, 0x7e, 0x7e, 0xfe, 0xfe]
    # ties go to the even code: 17 -> 16, 19 -> 20, 2^-10 -> 0, 1.5 * 2^-9 -> 2 * 2^-9
    assert oracle32.e4m3_decode(oracle32.e4m3_encode(np.array([17, 19, 2.0 ** -10, 1.5 * 2.0 ** -9], dtype=np.float32))).tolist() == \
        [16.0, 20.0, 0.0, 2.0 ** -8]
    # monotone, idempotent on the format's own values
    xs = np.sort(x)
    assert np.all(np.diff(oracle32.e4m3_decode(oracle32.e4m3_encode(xs))) >= 0)
    assert np.array_equal(oracle32.e4m3_encode(vals.astype(np.float32)), np.arange(0x7f, dtype=np.uint8))


def test_e4m3_semvec_is_the_float_mean_rounded_once(oracle32):
    """The stored code is torch's float32 -> float8_e4m3fn conversion of the oracle's own float mean; scores from the table
    equal a float64 dot product with the decoded values; the rounding is visible in the scores."""
    import torch
    lens = np.array([3, 1, 40, 7, 25, 12, 2], dtype=np.int32)
    off = gen.offsets_of(lens)
    g = torch.Generator().manual_seed(37)
    K = torch.randn(2, 2, int(lens.sum()), 128, generator=g).to(torch.bfloat16)
    sv32 = oracle32.semvec(gen.to_numpy(K), off)
    sv8 = oracle32.semvec(gen.to_numpy(K), off, sv_dtype="fp8")
    assert sv8.dtype == np.uint8 and sv8.shape == sv32.shape
    assert np.array_equal(sv8, _torch_e4m3(sv32))
    q = torch.randn(8, 128, generator=g).to(torch.bfloat16)
    got = oracle32.score(gen.to_numpy(q), sv8[0])
    wide = torch.from_numpy(sv8[0]).view(torch.float8_e4m3fn).double().numpy()
    qd = q.double().numpy()
    want = np.stack([wide[h] @ qd[4 * h:4 * h + 4].sum(axis=0) for h in range(2)])
    assert np.abs(got - want).max() <= 1e-5 * np.abs(want).max()
    ref = oracle32.score(gen.to_numpy(q), sv32[0])
    d = np.abs(got - ref).max()
    assert 0 < d <= 2.0 ** -4 * np.abs(qd).sum(axis=1).max() * np.abs(sv32).max()
