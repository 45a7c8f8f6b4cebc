"""Thin ctypes binding of libsentencekv (see include/sentencekv.h).

Argument marshalling only: every function here forwards raw device pointers of caller-allocated
torch tensors to the C entry point of the same name and raises on a non-zero status.  Nothing is
computed in Python and there is no fallback: if the HIP library is missing or fails, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

from . import _build

SKV_F32, SKV_BF16, SKV_FP8_E4M3 = 0, 1, 2
SKV_OK, SKV_EINVAL, SKV_ECAPACITY, SKV_EHIP, SKV_ENOMEM = 0, -1, -2, -3, -4


class SkvError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {_lib().skv_strerror(status).decode()} ({status})")


class _Desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("n_layers", "n_q_heads", "n_kv_heads", "head_dim", "kv_dtype",
                                              "max_tokens", "max_sentences", "max_budget", "max_batch", "semvec_dtype")]


_LIB = None
_vp, _i32, _int, _i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int, ctypes.c_int64

_SIGNATURES = {
    "skv_create": (_int, [ctypes.POINTER(_vp), ctypes.POINTER(_Desc), _vp]),
    "skv_destroy": (None, [_vp]),
    "skv_set_stream": (_int, [_vp, _vp]),
    "skv_strerror": (ctypes.c_char_p, [_int]),
    "skv_workspace_bytes": (_i64, [_vp]),
    "skv_set_wait_limit": (_int, [_vp, _i32]),
    "skv_set_single_launch": (_int, [_vp, _i32]),
    "skv_set_budget_hint": (_int, [_vp, _i32]),
    "skv_segment": (_int, [_vp, _vp, _i32, _vp, _i32, _vp, _vp, _vp, _vp, _vp]),
    "skv_build_semvec": (_int, [_vp, _vp, _i32, _vp, _i32, _vp]),
    "skv_build_semvec_layers": (_int, [_vp, _vp, _i32, _vp, _i32, _vp]),
    "skv_token_importance_work_bytes": (_i64, [_vp, _i32, _i32]),
    "skv_token_importance": (_int, [_vp, _vp, _vp, _i32, _i32, _vp, _vp, _i64]),
    "skv_retain": (_int, [_vp, _vp, _i32, _i32, _vp, _i32, _vp, _vp, _vp, _vp]),
    "skv_compact_pool": (_int, [_vp, _vp, _vp, _i32, _vp, _i32, _vp, _vp, _vp]),
    "skv_query_update": (_int, [_vp, _i32, _vp, _vp, _vp, _i32, _vp, _vp, _vp]),
    "skv_score": (_int, [_vp, _i32, _vp, _vp, _i32, _vp]),
    "skv_select": (_int, [_vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp]),
    "skv_gather": (_int, [_vp, _i32, _vp, _vp, _i32, _int, _vp, _vp, _i32, _vp, _vp]),
    "skv_attend": (_int, [_vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp]),
    "skv_merge_lse": (_int, [_vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp]),
    "skv_decode_step": (_int, [_vp, _i32, _i32, _vp, _vp, _vp, _vp, _i32, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp,
                               _vp, _vp, _vp]),
    "skv_decode_step_noalloc": (_int, [ctypes.POINTER(_Desc), _vp, _i32, _i32, _vp, _vp, _vp, _vp, _i32, _vp, _i32, _vp, _vp,
                                       _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
}
EXPORTS = tuple(_SIGNATURES)


def lib_path() -> str:
    return _build.LIB


def _lib():
    """Load the built library; build it first only if no library is there at all."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(_build.LIB):
            _build.build(force=True)
        lib = ctypes.CDLL(_build.LIB)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _LIB = lib
    return _LIB


def _p(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_contiguous(), "tensors handed to libsentencekv must be contiguous"
    return t.data_ptr()


def _check(status: int, what: str) -> None:
    if status != SKV_OK:
        raise SkvError(status, what)


@dataclass
class Desc:
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int = 128
    kv_dtype: int = SKV_BF16
    max_tokens: int = 1
    max_sentences: int = 1
    max_budget: int = 1
    max_batch: int = 1
    semvec_dtype: int = SKV_F32

    @property
    def max_sel(self) -> int:
        return min(self.max_sentences, self.max_budget)


def dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return SKV_F32
    if dt == torch.bfloat16:
        return SKV_BF16
    raise TypeError(f"K/V/q must be float32 or bfloat16, got {dt}")


class Context:
    """Owns one skv_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, desc: Desc, stream: Optional[int] = None):
        lib = _lib()
        self.desc = desc
        d = _Desc(desc.n_layers, desc.n_q_heads, desc.n_kv_heads, desc.head_dim, desc.kv_dtype, desc.max_tokens,
                  desc.max_sentences, desc.max_budget, desc.max_batch, desc.semvec_dtype)
        h = _vp()
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else 0
        _check(lib.skv_create(ctypes.byref(h), ctypes.byref(d), _vp(stream)), "skv_create")
        self._h = h

    def close(self) -> None:
        if getattr(self, "_h", None):
            _lib().skv_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_stream(self, stream: int) -> None:
        _check(_lib().skv_set_stream(self._h, _vp(stream)), "skv_set_stream")

    def workspace_bytes(self) -> int:
        return int(_lib().skv_workspace_bytes(self._h))

    def set_budget_hint(self, budget: int) -> None:
        _check(_lib().skv_set_budget_hint(self._h, budget), "skv_set_budget_hint")

    def set_wait_limit(self, polls: int) -> None:
        _check(_lib().skv_set_wait_limit(self._h, polls), "skv_set_wait_limit")

    def set_single_launch(self, enable: bool) -> None:
        _check(_lib().skv_set_single_launch(self._h, 1 if enable else 0), "skv_set_single_launch")

    # ---- (1) prefill ----------------------------------------------------------------------------
    def segment(self, tok, term_bitmap, vocab: int, seg_id, sent_off, sent_len, n_sent_dev, sync: bool = True,
                T: Optional[int] = None) -> Optional[int]:
        host = ctypes.c_int32(-1)
        T = tok.shape[0] if T is None else T
        rc = _lib().skv_segment(self._h, _p(tok), T, _p(term_bitmap), vocab, _p(seg_id), _p(sent_off),
                                _p(sent_len), _p(n_sent_dev), ctypes.addressof(host) if sync else None)
        _check(rc, "skv_segment")
        return int(host.value) if sync else None

    def build_semvec(self, K_pool, sent_off, S: int, semvec) -> None:
        T = K_pool.shape[2]
        _check(_lib().skv_build_semvec(self._h, _p(K_pool), T, _p(sent_off), S, _p(semvec)), "skv_build_semvec")

    def build_semvec_layers(self, K_pool, sent_off, S: int, semvec) -> None:
        T = K_pool.shape[2]
        _check(_lib().skv_build_semvec_layers(self._h, _p(K_pool), T, _p(sent_off), S, _p(semvec)), "skv_build_semvec_layers")

    # ---- prefill-side token retention (Sec. 4.1) ---------------------------------------------------------
    def token_importance_work_bytes(self, T: int, N: int) -> int:
        return int(_lib().skv_token_importance_work_bytes(self._h, T, N))

    def token_importance(self, q_obs, K_pool, T: int, N: int, alpha, work) -> None:
        _check(_lib().skv_token_importance(self._h, _p(q_obs), _p(K_pool), T, N, _p(alpha), _p(work),
                                           work.numel() * work.element_size()), "skv_token_importance")

    def retain(self, alpha, Tp: int, k: int, seg_id, S: int, keep_idx, n_keep, ret_off, ret_len) -> None:
        _check(_lib().skv_retain(self._h, _p(alpha), Tp, k, _p(seg_id), S, _p(keep_idx), _p(n_keep), _p(ret_off),
                                 _p(ret_len)), "skv_retain")

    def compact_pool(self, K_pool, V_pool, T: int, keep_idx, k: int, n_keep, K_ret, V_ret) -> None:
        _check(_lib().skv_compact_pool(self._h, _p(K_pool), _p(V_pool), T, _p(keep_idx), k, _p(n_keep), _p(K_ret),
                                       _p(V_ret)), "skv_compact_pool")

    # ---- sentence query cache (Eq. 2) ----------------------------------------------------------------
    def query_update(self, B: int, q_t, tok_t, term_bitmap, vocab: int, q_sum, q_cnt, q_bar) -> None:
        _check(_lib().skv_query_update(self._h, B, _p(q_t), _p(tok_t), _p(term_bitmap), vocab, _p(q_sum), _p(q_cnt),
                                       _p(q_bar)), "skv_query_update")

    # ---- (2)-(5) decode, one layer, one sequence ---------------------------------------------------
    def score(self, layer: int, q_score, semvec, S: int, score) -> None:
        _check(_lib().skv_score(self._h, layer, _p(q_score), _p(semvec), S, _p(score)), "skv_score")

    def select(self, score, sent_off, sent_len, S: int, budget: int, sel_sent, n_sel, tok_idx, n_tok) -> None:
        _check(_lib().skv_select(self._h, _p(score), _p(sent_off), _p(sent_len), S, budget, _p(sel_sent), _p(n_sel),
                                 _p(tok_idx), _p(n_tok)), "skv_select")

    def gather(self, layer: int, K_pool, V_pool, T: int, tok_idx, n_tok, budget: int, K_sel, V_sel,
               pool_in_host: bool = False) -> None:
        _check(_lib().skv_gather(self._h, layer, _p(K_pool), _p(V_pool), T, int(pool_in_host), _p(tok_idx), _p(n_tok),
                                 budget, _p(K_sel), _p(V_sel)), "skv_gather")

    def attend(self, q_attn, K_sel, V_sel, n_tok, budget: int, out, lse=None) -> None:
        _check(_lib().skv_attend(self._h, _p(q_attn), _p(K_sel), _p(V_sel), _p(n_tok), budget, _p(out), _p(lse)),
               "skv_attend")

    # ---- fused, ragged batch -----------------------------------------------------------------------
    def decode_step(self, layer: int, B: int, q_score, q_attn, K_pool, V_pool, T_total: int, semvec, S_total: int,
                    cu_tok, cu_sent, sent_off, sent_len, budget, out, lse=None, tok_idx_out=None, n_tok_out=None) -> None:
        _check(_lib().skv_decode_step(self._h, layer, B, _p(q_score), _p(q_attn), _p(K_pool), _p(V_pool), T_total,
                                      _p(semvec), S_total, _p(cu_tok), _p(cu_sent), _p(sent_off), _p(sent_len),
                                      _p(budget), _p(out), _p(lse), _p(tok_idx_out), _p(n_tok_out)), "skv_decode_step")

    def merge_lse(self, n_heads: int, out_a, lse_a, out_b, lse_b, out, lse=None) -> None:
        _check(_lib().skv_merge_lse(self._h, n_heads, _p(out_a), _p(lse_a), _p(out_b), _p(lse_b), _p(out), _p(lse)),
               "skv_merge_lse")


NOALLOC_SCRATCH_BYTES = 8 * 1024 * 1024


def decode_step_noalloc(desc: Desc, layer: int, B: int, q_score, q_attn, K_pool, V_pool, T_total: int, semvec, S_total: int,
                        cu_tok, cu_sent, sent_off, sent_len, budget, out, lse=None, tok_idx_out=None, n_tok_out=None,
                        stream: Optional[int] = None) -> None:
    """skv_decode_step_noalloc: the decode step without a context, on the library's static device scratch."""
    d = _Desc(desc.n_layers, desc.n_q_heads, desc.n_kv_heads, desc.head_dim, desc.kv_dtype, desc.max_tokens,
              desc.max_sentences, desc.max_budget, desc.max_batch, desc.semvec_dtype)
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else 0
    _check(_lib().skv_decode_step_noalloc(ctypes.byref(d), _vp(stream), layer, B, _p(q_score), _p(q_attn), _p(K_pool),
                                          _p(V_pool), T_total, _p(semvec), S_total, _p(cu_tok), _p(cu_sent), _p(sent_off),
                                          _p(sent_len), _p(budget), _p(out), _p(lse), _p(tok_idx_out), _p(n_tok_out)),
           "skv_decode_step_noalloc")
