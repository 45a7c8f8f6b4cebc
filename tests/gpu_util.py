"""Helpers for the GPU parity tests: allocate device buffers, call the C ABI through the binding,
bring results back as numpy, and the checks every selection comparison shares.  No arithmetic of the method lives
here: the selection rule itself is always the oracle's."""
from __future__ import annotations

import numpy as np
import torch

import paper_2504_00970_amd as skv
from workload import gen

DEV = "cuda:0"


def i32(a, device=DEV):
    return torch.as_tensor(np.ascontiguousarray(a, dtype=np.int32)).to(device)


def empty_i32(*shape, fill=None):
    t = torch.empty(*shape, dtype=torch.int32, device=DEV)
    if fill is not None:
        t.fill_(fill)
    return t


def make_ctx(wl: gen.Workload, T, S, budget, batch=1, sv_dtype="f32"):
    return skv.Context(skv.Desc(n_layers=wl.n_layers, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                                kv_dtype=skv.dtype_code(wl.torch_dtype), max_tokens=max(T, 1),
                                max_sentences=max(S, 1), max_budget=max(budget, 1), max_batch=batch,
                                semvec_dtype={"f32": skv.SKV_F32, "bf16": skv.SKV_BF16, "fp8": skv.SKV_FP8_E4M3}[sv_dtype]))


def sv_torch_dtype(sv_dtype):
    return {"f32": torch.float32, "bf16": torch.bfloat16, "fp8": torch.uint8}[sv_dtype]


def bf16_table_close(got_bits: np.ndarray, ref_bits: np.ndarray) -> bool:
    """Two bf16 tables that round fp32 means differing in summation order: equal almost everywhere, and where they differ
    the two values are neighbours of the format (one step of 2^-7 relative) or, for means that cancel to almost nothing,
    within the fp32 summation error of values of order one."""
    wide = lambda b: (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    g, r = wide(got_bits), wide(ref_bits)
    same = float((got_bits == ref_bits).mean())
    return bool(np.all(np.abs(g - r) <= 2.0 ** -7 * np.maximum(np.abs(g), np.abs(r)) + 1e-6) and same >= 0.995)


def e4m3_table_close(got: np.ndarray, ref: np.ndarray, decode) -> bool:
    """Two E4M3 tables that round fp32 means differing in summation order: equal almost everywhere, and where they differ
    the two values are neighbours of the format (one step of 2^(e-10) at their magnitude, 2^-9 below 2^-6)."""
    g, r = decode(got).astype(np.float64), decode(ref).astype(np.float64)
    mag = np.maximum(np.abs(g), np.abs(r))
    step = np.where(mag < 2.0 ** -6, 2.0 ** -9, 2.0 ** (np.floor(np.log2(np.maximum(mag, 2.0 ** -6))) - 3))
    same = float((got == ref).mean())
    return bool(np.all(np.abs(g - r) <= step) and same >= 0.99)


def np_of(t: torch.Tensor) -> np.ndarray:
    return gen.to_numpy(t.detach().cpu())


def gpu_segment(ctx, tok: np.ndarray, bitmap: np.ndarray, vocab: int, cap: int):
    T = len(tok)
    d_tok = i32(tok) if T else empty_i32(4)
    d_bm = torch.as_tensor(bitmap.view(np.int32)).to(DEV)
    seg_id = empty_i32(max(T, 4), fill=-7)
    off = empty_i32(cap + 1 + 4, fill=-7)
    ln = empty_i32(cap + 4, fill=-7)
    n = empty_i32(4, fill=-7)
    S = ctx.segment(d_tok, d_bm, vocab, seg_id, off, ln, n, T=T)
    torch.cuda.synchronize()
    return seg_id.cpu().numpy()[:T], off.cpu().numpy(), ln.cpu().numpy(), S, int(n.cpu()[0])


def gpu_decode_chain(ctx, wl, layer, q_dev, K_dev, V_dev, semvec_dev, sent_off, sent_len, budget, pool_in_host=False):
    """score -> select -> gather -> attend through the four C entry points.  Returns numpy results."""
    H, Hq, D = wl.n_kv_heads, wl.n_q_heads, wl.head_dim
    T = K_dev.shape[2]
    S = len(sent_len)
    max_sel = ctx.desc.max_sel
    d_off, d_len = i32(sent_off), i32(sent_len) if S else empty_i32(4)
    score = torch.full((H, max(S, 1)), -777.0, dtype=torch.float32, device=DEV)
    sel = empty_i32(H, max_sel, fill=-1)
    n_sel, n_tok = empty_i32(max(H, 4), fill=-5), empty_i32(max(H, 4), fill=-5)
    tok_idx = empty_i32(H, max(budget, 1), fill=-1)
    K_sel = torch.zeros(H, max(budget, 1), D, dtype=wl.torch_dtype, device=DEV)
    V_sel = torch.zeros_like(K_sel)
    out = torch.full((Hq, D), 555.0, dtype=torch.float32, device=DEV)
    lse = torch.full((max(Hq, 4),), 555.0, dtype=torch.float32, device=DEV)
    ctx.score(layer, q_dev, semvec_dev, S, score)
    ctx.select(score, d_off, d_len, S, budget, sel, n_sel, tok_idx, n_tok)
    ctx.gather(layer, K_dev, V_dev, T, tok_idx, n_tok, budget, K_sel, V_sel, pool_in_host=pool_in_host)
    ctx.attend(q_dev, K_sel, V_sel, n_tok, budget, out, lse)
    torch.cuda.synchronize()
    return dict(score=score.cpu().numpy()[:, :S], sel_sent=sel.cpu().numpy(), n_sel=n_sel.cpu().numpy()[:H],
                tok_idx=tok_idx.cpu().numpy(), n_tok=n_tok.cpu().numpy()[:H], K_sel=np_of(K_sel), V_sel=np_of(V_sel),
                out=out.cpu().numpy(), lse=lse.cpu().numpy()[:Hq])


def score_tolerance(score_ref: np.ndarray) -> np.ndarray:
    """Allowed |gpu - oracle| per score: 1e-5 relative to the larger of |score| and the head's rms score.
    Both sides sum the same G*D = 512..1024 fp32 products in different orders; the rounding error of
    such a sum scales with the magnitude of its partial sums (the rms score of the head, or of all heads
    when that is larger: one bucket per head leaves no other sample), not with a score that happens to
    cancel to near zero."""
    if not score_ref.size:
        return 1e-5 * np.abs(score_ref)
    sq = score_ref.astype(np.float64) ** 2
    rms = np.maximum(np.sqrt(sq.mean(axis=1, keepdims=True)), np.sqrt(sq.mean()))   # a head with a single bucket: all heads
    return 1e-5 * np.maximum(np.abs(score_ref), rms)


def ranking(score: np.ndarray) -> np.ndarray:
    """Bucket ids by (score descending, id ascending); NaN last."""
    key = np.where(np.isnan(score), -np.inf, score.astype(np.float64))
    return np.lexsort((np.arange(len(score)), np.isnan(score), -key))


def documented_tie(score_cpu: np.ndarray, score_gpu: np.ndarray, upto: int, rel=1e-5):
    """Among the first `upto` ranks (the part of the ranking that decides the selection) the two
    rankings first diverge at a pair of buckets; returns (is_tie, a, b, relative gap of the oracle's
    scores of that pair).  A selection difference is acceptable only when that gap is < rel."""
    oc, og = ranking(score_cpu)[:upto], ranking(score_gpu)[:upto]
    neq = np.nonzero(oc != og)[0]
    if len(neq) == 0:
        return True, -1, -1, 0.0
    a, b = int(oc[neq[0]]), int(og[neq[0]])
    gap = abs(float(score_cpu[a]) - float(score_cpu[b])) / max(abs(float(score_cpu[a])), abs(float(score_cpu[b])), 1e-30)
    return gap < rel, a, b, gap


MAX_TIES_PER_TEST = 4      # documented ties a single test case may log before it fails (none occurs on the committed seeds)


def gpu_scores(ctx, layer: int, q_dev, semvec_dev, S_total: int, H: int) -> np.ndarray:
    """skv_score of one sequence's queries over the whole (concatenated) bucket axis: [H][S_total].  A bucket's score
    depends on its vector and the group's queries only, so the slice of a sequence holds the very floats the fused
    step ranks for that sequence."""
    score = torch.full((H, max(S_total, 1)), -777.0, dtype=torch.float32, device=DEV)
    ctx.score(layer, q_dev, semvec_dev, S_total, score)
    torch.cuda.synchronize()
    return score.cpu().numpy()[:, :S_total]


def check_selection(oracle, sc_cpu, sc_gpu, sent_off, sent_len, budget, tok_idx_gpu, n_tok_gpu, what="") -> int:
    """The selection gate of the fused step, for one sequence (all KV heads).
      (i)   the GPU's scores are within the score tolerance of the oracle's;
      (ii)  the oracle's rule applied to the GPU's own scores gives the GPU's n_tok / tok_idx bit for bit (whole
            buckets, a prefix of the ranking, maximal, ascending positions: all implied);
      (iii) where that differs from the oracle's selection on the oracle's scores, the two rankings first diverge,
            inside the deciding prefix, at a pair of buckets whose oracle scores are within 1e-5 relative.
    Returns the number of heads with a documented tie; anything else fails."""
    H = sc_cpu.shape[0]
    assert np.all(np.abs(sc_gpu - sc_cpu) <= score_tolerance(sc_cpu)), what
    sel_g, n_sel_g, tok_g, n_g = oracle.select(sc_gpu, sent_off, sent_len, budget)
    sel_c, n_sel_c, tok_c, n_c = oracle.select(sc_cpu, sent_off, sent_len, budget)
    ties = 0
    for h in range(H):
        assert n_tok_gpu[h] == n_g[h] and n_g[h] <= budget, (what, h, int(n_tok_gpu[h]), int(n_g[h]))
        assert np.array_equal(tok_idx_gpu[h, :n_g[h]], tok_g[h, :n_g[h]]), (what, h)
        if n_g[h] != n_c[h] or not np.array_equal(tok_g[h, :n_g[h]], tok_c[h, :n_c[h]]):
            ok, a, b, gap = documented_tie(sc_cpu[h], sc_gpu[h], upto=int(max(n_sel_c[h], n_sel_g[h])) + 1)
            print(f"  documented tie: {what} head {h} buckets {a},{b} relative gap {gap:.3e}", flush=True)
            assert ok, (what, h, a, b, gap)
            ties += 1
    return ties
