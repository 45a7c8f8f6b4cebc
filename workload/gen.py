"""Seeded synthetic inputs for the SentenceKV decode / prefill hot path.

This module only *draws* inputs: sentence lengths, token streams, terminator
bitmaps, key/value pools and queries.  It contains none of the method's
arithmetic (no segmentation scan, no sentence means, no scores, no selection,
no attention); both the CPU oracle's tests and the GPU path's tests consume the
very same bytes produced here.

Shapes follow Llama-3.1-8B / Llama-3-70B attention geometry; sentence ("bucket")
lengths follow the 25-30 token median bucket size the paper reports for its
corpora (appendix on the chunk-size sensitivity of the fixed-chunk baseline).
The tensors stand in for the paper's LongBench / RULER / NIAH / PG-19 prompts
and the models' real K/V activations, none of which are available here.

Structure of the keys: every (layer, kv head, sentence) gets a centre
c ~ N(0, I_D); a token's key is its sentence's centre plus 0.5 * N(0, I_D)
noise, so that sentence means are well separated (as the paper's motivation
section observes for real sentence embeddings).  Values and queries are N(0, 1).
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Optional, Sequence, Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    """Static description of one synthetic configuration."""
    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str                      # "f32" | "bf16"
    n_tokens: int                   # context length (per sequence for batch == 1)
    len_dist: Tuple                 # ("uniform", lo, hi) | ("lognormal", median, sigma, lo, hi) | ("geometric", p)
    budgets: Tuple[int, ...] = ()
    batch: int = 1
    t_range: Optional[Tuple[int, int]] = None   # ragged batch: T_b ~ U[lo, hi]
    vocab: int = 131072
    term_mod: int = 20              # token id is a terminator iff id % term_mod == 0

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def elt_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five configurations the benchmark contract names.
CFG0 = Workload("cfg0_4k_f32", 1, 32, 8, 128, "f32", 4096, ("uniform", 8, 40), (512,))
CFG1 = Workload("cfg1_32k_bf16", 32, 32, 8, 128, "bf16", 32768, ("lognormal", 20.0, 0.7, 3, 120), (1024, 2048))
CFG2 = Workload("cfg2_128k_bf16", 32, 32, 8, 128, "bf16", 131072, ("lognormal", 20.0, 0.7, 3, 120), (2048,))
CFG3 = Workload("cfg3_prefill_32k", 32, 32, 8, 128, "bf16", 32768, ("geometric", 0.05), ())
CFG4 = Workload("cfg4_ragged_70b", 80, 64, 8, 128, "bf16", 0, ("lognormal", 20.0, 0.7, 3, 120), (2048,),
                batch=16, t_range=(8192, 65536))
CONFIGS = {"cfg0": CFG0, "cfg1": CFG1, "cfg2": CFG2, "cfg3": CFG3, "cfg4": CFG4}


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, stream]))


def _tgen(seed: int, stream: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + stream * 7919 + 12345) & 0x7FFFFFFFFFFFFFFF)
    return g


def sentence_lengths(len_dist: Tuple, n_tokens: int, seed: int, stream: int = 0) -> np.ndarray:
    """Draw sentence lengths until they cover `n_tokens`; the last one is cut to fit.

    Returns int32 [S] with every entry >= 1 and sum == n_tokens (empty for n_tokens == 0).
    """
    if n_tokens <= 0:
        return np.zeros(0, dtype=np.int32)
    rng = _rng(seed, 100 + stream)
    kind = len_dist[0]
    out = []
    total = 0
    while total < n_tokens:
        n = max(64, n_tokens // 8)
        if kind == "uniform":
            draw = rng.integers(len_dist[1], len_dist[2] + 1, size=n)
        elif kind == "lognormal":
            _, median, sigma, lo, hi = len_dist
            draw = np.rint(np.exp(np.log(median) + sigma * rng.standard_normal(n)))
            draw = np.clip(draw, lo, hi).astype(np.int64)
        elif kind == "geometric":
            draw = rng.geometric(len_dist[1], size=n)
        elif kind == "fixed":
            draw = np.full(n, len_dist[1], dtype=np.int64)
        else:
            raise ValueError(f"unknown length distribution {kind!r}")
        out.append(draw.astype(np.int64))
        total += int(draw.sum())
    lens = np.concatenate(out)
    cum = np.cumsum(lens)
    k = int(np.searchsorted(cum, n_tokens))          # first index with cum >= n_tokens
    lens = lens[: k + 1].copy()
    lens[k] -= int(cum[k]) - n_tokens
    assert lens.sum() == n_tokens and lens.min() >= 1
    return lens.astype(np.int32)


def terminator_bitmap(vocab: int, term_mod: int) -> np.ndarray:
    """uint32 [ceil(vocab/32)]: bit (id % 32) of word (id // 32) is set iff id is a terminator."""
    ids = np.arange(0, vocab, term_mod, dtype=np.int64)
    words = np.zeros((vocab + 31) // 32, dtype=np.uint32)
    np.bitwise_or.at(words, ids // 32, (np.uint32(1) << (ids % 32).astype(np.uint32)))
    return words


def token_stream(lengths: np.ndarray, vocab: int, term_mod: int, seed: int,
                 last_open: bool = True, stream: int = 0) -> np.ndarray:
    """int32 token ids [sum(lengths)]: the last token of every sentence is a terminator id
    (id % term_mod == 0) and every other token is not.  With `last_open` the final sentence
    is left without a terminator (a prompt that stops mid-sentence)."""
    rng = _rng(seed, 200 + stream)
    T = int(lengths.sum())
    tok = rng.integers(0, vocab, size=T, dtype=np.int64)
    # push every token off the terminator residue class, then plant terminators at sentence ends
    tok = np.where(tok % term_mod == 0, (tok + 1 + rng.integers(0, term_mod - 1, size=T)) % vocab, tok)
    tok = np.where(tok % term_mod == 0, tok + 1, tok)           # wrap-around landed on 0
    ends = np.cumsum(lengths.astype(np.int64)) - 1
    if last_open and len(ends) > 0:
        ends = ends[:-1]
    n_term_ids = (vocab + term_mod - 1) // term_mod
    tok[ends] = rng.integers(0, n_term_ids, size=len(ends)) * term_mod
    return tok.astype(np.int32)


def _sentence_of_token(lengths: np.ndarray, device) -> torch.Tensor:
    """int64 [T]: which drawn sentence each token position belongs to (generator-side bookkeeping)."""
    return torch.repeat_interleave(torch.arange(len(lengths), dtype=torch.int64),
                                   torch.from_numpy(lengths.astype(np.int64))).to(device)


def kv_layer(lengths: np.ndarray, n_kv_heads: int, head_dim: int, dtype: torch.dtype,
             seed: int, layer: int, device="cpu", noise: float = 0.5,
             out_k: Optional[torch.Tensor] = None, out_v: Optional[torch.Tensor] = None):
    """K, V [Hkv][T][D] for one layer: K = centre(sentence) + noise * N(0,1), V = N(0,1)."""
    T = int(lengths.sum())
    S = len(lengths)
    g = _tgen(seed, 1000 + layer, device)
    sid = _sentence_of_token(lengths, device)
    centres = torch.randn(n_kv_heads, max(S, 1), head_dim, generator=g, device=device, dtype=torch.float32)
    k = torch.randn(n_kv_heads, T, head_dim, generator=g, device=device, dtype=torch.float32)
    k.mul_(noise)
    if T > 0:
        k.add_(centres[:, sid, :])
    v = torch.randn(n_kv_heads, T, head_dim, generator=g, device=device, dtype=torch.float32)
    if out_k is not None:
        out_k.copy_(k)
        out_v.copy_(v)
        return out_k, out_v
    return k.to(dtype), v.to(dtype)


def queries(n: int, n_q_heads: int, head_dim: int, dtype: torch.dtype, seed: int, device="cpu") -> torch.Tensor:
    """q [n][Hq][D] ~ N(0,1): one per layer (or per rotating step)."""
    g = _tgen(seed, 5000, device)
    return torch.randn(n, n_q_heads, head_dim, generator=g, device=device, dtype=torch.float32).to(dtype)


@dataclass
class DecodeInputs:
    wl: Workload
    lengths: np.ndarray             # int32 [S]   (what the generator drew)
    sent_off: np.ndarray            # int32 [S+1] (running start positions of the drawn sentences)
    K: torch.Tensor                 # [L][Hkv][T][D]
    V: torch.Tensor                 # [L][Hkv][T][D]
    q: torch.Tensor                 # [L][Hq][D]


def offsets_of(lengths: np.ndarray) -> np.ndarray:
    off = np.zeros(len(lengths) + 1, dtype=np.int32)
    if len(lengths):
        off[1:] = np.cumsum(lengths.astype(np.int64)).astype(np.int32)
    return off


def decode_inputs(wl: Workload, seed: int = 0, device="cpu", pin_pool: bool = False) -> DecodeInputs:
    """Full-context K/V pool [L][Hkv][T][D], one query per layer, and the sentence structure.

    With `pin_pool` the pool is allocated in pinned host memory (the paper's CPU-offload design)
    and filled layer by layer from the generating device."""
    lengths = sentence_lengths(wl.len_dist, wl.n_tokens, seed)
    L, H, T, D = wl.n_layers, wl.n_kv_heads, wl.n_tokens, wl.head_dim
    if pin_pool:
        K = torch.empty(L, H, T, D, dtype=wl.torch_dtype, pin_memory=True)
        V = torch.empty(L, H, T, D, dtype=wl.torch_dtype, pin_memory=True)
    else:
        K = torch.empty(L, H, T, D, dtype=wl.torch_dtype, device=device)
        V = torch.empty(L, H, T, D, dtype=wl.torch_dtype, device=device)
    for l in range(L):
        kv_layer(lengths, H, D, wl.torch_dtype, seed, l, device, out_k=K[l], out_v=V[l])
    q = queries(L, wl.n_q_heads, D, wl.torch_dtype, seed, device)
    return DecodeInputs(wl, lengths, offsets_of(lengths), K, V, q)


@dataclass
class PrefillInputs:
    wl: Workload
    lengths: np.ndarray             # int32 [S] drawn sentence lengths (ground truth for the segmenter)
    tok: np.ndarray                 # int32 [T]
    bitmap: np.ndarray              # uint32 [ceil(vocab/32)]
    K: Optional[torch.Tensor]       # [L][Hkv][T][D] or None


def prefill_inputs(wl: Workload, seed: int = 0, device="cpu", with_keys: bool = True) -> PrefillInputs:
    """Token-id stream whose positions are sentence terminators with the probability the
    length distribution implies (geometric(p) lengths <=> iid Bernoulli(p) terminator flags),
    the vocabulary's terminator bitmap, and the key pool built on that sentence structure."""
    lengths = sentence_lengths(wl.len_dist, wl.n_tokens, seed)
    tok = token_stream(lengths, wl.vocab, wl.term_mod, seed)
    bitmap = terminator_bitmap(wl.vocab, wl.term_mod)
    K = None
    if with_keys:
        L, H, T, D = wl.n_layers, wl.n_kv_heads, wl.n_tokens, wl.head_dim
        K = torch.empty(L, H, T, D, dtype=wl.torch_dtype, device=device)
        for l in range(L):
            k, _ = kv_layer(lengths, H, D, wl.torch_dtype, seed, l, device)
            K[l].copy_(k)
    return PrefillInputs(wl, lengths, tok, bitmap, K)


@dataclass
class RaggedInputs:
    wl: Workload
    seq_tokens: np.ndarray          # int32 [B]
    lengths: list                   # B arrays of int32 sentence lengths
    cu_tok: np.ndarray              # int32 [B+1]
    cu_sent: np.ndarray             # int32 [B+1]
    sent_off: np.ndarray            # int32 [S_total + B]: per sequence b, S_b+1 local offsets at cu_sent[b]+b
    sent_len: np.ndarray            # int32 [S_total]
    K: torch.Tensor                 # [Lr][Hkv][T_total][D]  (Lr resident layers)
    V: torch.Tensor
    q: torch.Tensor                 # [Lr][B][Hq][D]
    budget: np.ndarray              # int32 [B]


def ragged_inputs(wl: Workload, seed: int = 0, device="cpu", resident_layers: Optional[int] = None,
                  seq_tokens=None, budgets=None) -> RaggedInputs:
    """Ragged batch: B sequences concatenated along the token axis and the sentence axis.  `seq_tokens` fixes the
    context lengths (zero allowed: a sequence without tokens or buckets), `budgets` the per-sequence budgets."""
    rng = _rng(seed, 300)
    B = wl.batch
    lo, hi = wl.t_range
    if seq_tokens is None:
        seq_tokens = rng.integers(lo, hi + 1, size=B).astype(np.int32)
    else:
        seq_tokens = np.asarray(seq_tokens, dtype=np.int32)
        assert seq_tokens.shape == (B,) and seq_tokens.min() >= 0
    lens = [sentence_lengths(wl.len_dist, int(seq_tokens[b]), seed, stream=1 + b) for b in range(B)]
    cu_tok = np.zeros(B + 1, dtype=np.int32)
    cu_tok[1:] = np.cumsum(seq_tokens.astype(np.int64))
    cu_sent = np.zeros(B + 1, dtype=np.int32)
    cu_sent[1:] = np.cumsum([len(x) for x in lens])
    sent_off = np.concatenate([offsets_of(x) for x in lens]).astype(np.int32)
    sent_len = np.concatenate(lens).astype(np.int32)
    all_lengths = sent_len                              # sentence structure of the concatenated stream
    Lr = wl.n_layers if resident_layers is None else resident_layers
    T_total = int(cu_tok[-1])
    K = torch.empty(Lr, wl.n_kv_heads, T_total, wl.head_dim, dtype=wl.torch_dtype, device=device)
    V = torch.empty_like(K)
    for l in range(Lr):
        kv_layer(all_lengths, wl.n_kv_heads, wl.head_dim, wl.torch_dtype, seed, l, device, out_k=K[l], out_v=V[l])
    q = queries(Lr * B, wl.n_q_heads, wl.head_dim, wl.torch_dtype, seed, device).view(Lr, B, wl.n_q_heads, wl.head_dim)
    budget = np.full(B, wl.budgets[0], dtype=np.int32) if budgets is None else np.asarray(budgets, dtype=np.int32)
    assert budget.shape == (B,)
    return RaggedInputs(wl, seq_tokens, lens, cu_tok, cu_sent, sent_off, sent_len, K, V, q, budget)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """View a CPU bf16 tensor as a numpy uint16 array of the same shape (bit pattern, no rounding)."""
    assert t.dtype == torch.bfloat16
    return t.contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def to_numpy(t: torch.Tensor) -> np.ndarray:
    """CPU numpy view of a tensor: float32 stays float32, bf16 becomes its uint16 bit pattern."""
    if t.dtype == torch.bfloat16:
        return bf16_bits(t)
    return t.contiguous().cpu().numpy()
