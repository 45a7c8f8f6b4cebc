"""ctypes loader for the SentenceKV CPU oracle -- TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
The product path (paper_2504_00970_amd) never does.

Two builds of the same C source exist: `f32` (REAL = float, the reference precision of the
parity gates) and `f64` (REAL = double, used by the pins to bound the f32 build's own rounding).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sentencekv_oracle.c")
# SKVO_SANITIZE=1 in the environment selects an AddressSanitizer + UndefinedBehaviorSanitizer build of the same source
# (its own folder; the process must have the ASan runtime preloaded, see tests/test_oracle_sanitized.py)
_SANITIZE = os.environ.get("SKVO_SANITIZE", "") == "1"
_BUILD = os.path.join(_HERE, "_build_san" if _SANITIZE else "_build")

F32, BF16, FP8 = 0, 1, 2


def lib_path(real: str) -> str:
    return os.path.join(_BUILD, f"libskv_oracle_{real}.so")


def build(force: bool = False) -> None:
    """Compile both precision builds with gcc (no fast-math, no FMA contraction)."""
    os.makedirs(_BUILD, exist_ok=True)
    for real, ctype in (("f32", "float"), ("f64", "double")):
        out = lib_path(real)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        opt = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"] if _SANITIZE else ["-O2"]
        cmd = ["gcc", "-std=c99", *opt, "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
               f"-DSKVO_REAL={ctype}", "-shared", "-fPIC", _SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


_i32p = ctypes.POINTER(ctypes.c_int32)
_u32p = ctypes.POINTER(ctypes.c_uint32)
_f32p = ctypes.POINTER(ctypes.c_float)
_vp = ctypes.c_void_p
_i = ctypes.c_int32
_ci = ctypes.c_int


def _ptr(a: np.ndarray, typ):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(typ)


def _dtype_of(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.uint8:
        return FP8
    raise TypeError(f"oracle inputs are float32, bf16-as-uint16 or E4M3-as-uint8, got {a.dtype}")


class Oracle:
    """numpy front end of one precision build of the oracle."""

    def __init__(self, real: str = "f32"):
        build()
        self.real = real
        self.lib = ctypes.CDLL(lib_path(real))
        L = self.lib
        L.skvo_segment.argtypes = [_i32p, _i, _u32p, _i, _i32p, _i32p, _i32p, _i, _i32p]
        L.skvo_segment.restype = _ci
        L.skvo_semvec.argtypes = [_vp, _ci, _i, _i, _i, _i, _i32p, _i, _f32p]
        L.skvo_semvec.restype = None
        L.skvo_semvec_to.argtypes = [_vp, _ci, _i, _i, _i, _i, _i32p, _i, _ci, _vp]
        L.skvo_semvec_to.restype = None
        L.skvo_score_from.argtypes = [_vp, _ci, _i, _i, _i, _vp, _ci, _i, _f32p]
        L.skvo_score_from.restype = None
        L.skvo_e4m3_encode.argtypes = [_f32p, ctypes.c_int64, _vp]
        L.skvo_e4m3_encode.restype = None
        L.skvo_e4m3_decode.argtypes = [_vp, ctypes.c_int64, _f32p]
        L.skvo_e4m3_decode.restype = None
        L.skvo_score.argtypes = [_vp, _ci, _i, _i, _i, _f32p, _i, _f32p]
        L.skvo_score.restype = None
        L.skvo_select.argtypes = [_f32p, _i32p, _i32p, _i, _i, _i, _i32p, _i, _i32p, _i32p, _i, _i32p]
        L.skvo_select.restype = None
        L.skvo_gather.argtypes = [_vp, _ci, _i, _i, _i, _i32p, _i, _i32p, _vp]
        L.skvo_gather.restype = None
        L.skvo_attend.argtypes = [_vp, _vp, _vp, _ci, _i, _i, _i, _i32p, _i, _f32p, _f32p]
        L.skvo_attend.restype = None
        L.skvo_query_cache_step.argtypes = [_vp, _ci, _i, _i, _u32p, _i, _f32p, _i, _i32p, _f32p, _vp]
        L.skvo_query_cache_step.restype = _ci
        L.skvo_token_importance.argtypes = [_vp, _vp, _ci, _i, _i, _i, _i, _i, _f32p]
        L.skvo_token_importance.restype = None
        L.skvo_retain.argtypes = [_f32p, _i, _i, _i32p, _i, _i32p, _i32p, _i32p, _i32p]
        L.skvo_retain.restype = None
        L.skvo_merge_lse.argtypes = [_f32p, _f32p, _f32p, _f32p, _i, _i, _f32p, _f32p]
        L.skvo_merge_lse.restype = None
        L.skvo_real_bytes.restype = _ci
        assert L.skvo_real_bytes() == (4 if real == "f32" else 8)

    # -- prefill ---------------------------------------------------------------------------
    def segment(self, tok: np.ndarray, bitmap: np.ndarray, vocab: int, cap_sent: Optional[int] = None):
        """-> (seg_id[T], sent_off[S+1], sent_len[S], S).  Raises if S exceeds cap_sent."""
        tok = np.ascontiguousarray(tok, dtype=np.int32)
        bitmap = np.ascontiguousarray(bitmap, dtype=np.uint32)
        T = tok.shape[0]
        cap = T if cap_sent is None else cap_sent
        seg_id = np.zeros(T, dtype=np.int32)
        off = np.zeros(cap + 1, dtype=np.int32)
        ln = np.zeros(max(cap, 1), dtype=np.int32)
        n = np.zeros(1, dtype=np.int32)
        rc = self.lib.skvo_segment(_ptr(tok, _i32p), T, _ptr(bitmap, _u32p), vocab, _ptr(seg_id, _i32p),
                                   _ptr(off, _i32p), _ptr(ln, _i32p), cap, _ptr(n, _i32p))
        S = int(n[0])
        if rc != 0:
            raise OverflowError(f"{S} sentences exceed capacity {cap}")
        return seg_id, off[: S + 1].copy(), ln[:S].copy(), S

    def semvec(self, K: np.ndarray, sent_off: np.ndarray, sv_dtype: str = "f32") -> np.ndarray:
        """K [L][Hkv][T][D] (float32 or bf16 bits) -> semvec [L][Hkv][S][D]: float32, bf16 bits (sv_dtype="bf16") or
        E4M3 codes (sv_dtype="fp8")."""
        K = np.ascontiguousarray(K)
        L, H, T, D = K.shape
        sent_off = np.ascontiguousarray(sent_off, dtype=np.int32)
        S = sent_off.shape[0] - 1
        out = np.zeros((L, H, S, D), dtype={"f32": np.float32, "bf16": np.uint16, "fp8": np.uint8}[sv_dtype])
        self.lib.skvo_semvec_to(K.ctypes.data_as(_vp), _dtype_of(K), L, H, T, D, _ptr(sent_off, _i32p), S, _dtype_of(out),
                                out.ctypes.data_as(_vp))
        return out

    def e4m3_encode(self, x: np.ndarray) -> np.ndarray:
        """float32 -> E4M3 codes (nearest, ties to even, saturating at 448)."""
        x = np.ascontiguousarray(x, dtype=np.float32)
        out = np.zeros(x.shape, dtype=np.uint8)
        self.lib.skvo_e4m3_encode(_ptr(x, _f32p), ctypes.c_int64(x.size), out.ctypes.data_as(_vp))
        return out

    def e4m3_decode(self, code: np.ndarray) -> np.ndarray:
        code = np.ascontiguousarray(code, dtype=np.uint8)
        out = np.zeros(code.shape, dtype=np.float32)
        self.lib.skvo_e4m3_decode(code.ctypes.data_as(_vp), ctypes.c_int64(code.size), _ptr(out, _f32p))
        return out

    def token_importance(self, q_obs: np.ndarray, K: np.ndarray) -> np.ndarray:
        """q_obs [Hq][N][D], K [Hkv][T][D] (one layer) -> alpha float32 [T - N]."""
        q_obs, K = np.ascontiguousarray(q_obs), np.ascontiguousarray(K)
        Hq, N, D = q_obs.shape
        H, T, D2 = K.shape
        assert D == D2 and Hq % H == 0 and _dtype_of(q_obs) == _dtype_of(K)
        alpha = np.zeros(max(T - N, 0), dtype=np.float32)
        self.lib.skvo_token_importance(q_obs.ctypes.data_as(_vp), K.ctypes.data_as(_vp), _dtype_of(K), Hq, H, T, N, D,
                                       _ptr(alpha, _f32p))
        return alpha

    def retain(self, alpha: np.ndarray, k: int, seg_id: np.ndarray, S: int):
        """-> (keep_idx[min(k, Tp)] ascending, ret_off[S+1], ret_len[S])."""
        alpha = np.ascontiguousarray(alpha, dtype=np.float32)
        seg_id = np.ascontiguousarray(seg_id, dtype=np.int32)
        Tp = alpha.shape[0]
        assert seg_id.shape[0] >= Tp
        keep = np.zeros(max(min(k, Tp), 1), dtype=np.int32)
        n = np.zeros(1, dtype=np.int32)
        off = np.zeros(S + 1, dtype=np.int32)
        ln = np.zeros(max(S, 1), dtype=np.int32)
        self.lib.skvo_retain(_ptr(alpha, _f32p), Tp, k, _ptr(seg_id, _i32p), S, _ptr(keep, _i32p), _ptr(n, _i32p),
                             _ptr(off, _i32p), _ptr(ln, _i32p))
        return keep[: int(n[0])].copy(), off, ln[:S].copy()

    # -- decode ----------------------------------------------------------------------------
    def query_cache(self, per: int, cap: int = 4096) -> "QueryCache":
        """An empty sentence cache Q_s for one sequence and layer (per = Hq * D elements per token)."""
        return QueryCache(self, per, cap)

    def score(self, q: np.ndarray, semvec: np.ndarray) -> np.ndarray:
        """q [Hq][D], semvec [Hkv][S][D] float32, bf16 bits or E4M3 codes -> score float32 [Hkv][S]."""
        q = np.ascontiguousarray(q)
        semvec = np.ascontiguousarray(semvec)
        Hq, D = q.shape
        H, S, D2 = semvec.shape
        assert D == D2 and Hq % H == 0
        out = np.zeros((H, S), dtype=np.float32)
        self.lib.skvo_score_from(q.ctypes.data_as(_vp), _dtype_of(q), Hq, H, D, semvec.ctypes.data_as(_vp), _dtype_of(semvec), S,
                                 _ptr(out, _f32p))
        return out

    def select(self, score: np.ndarray, sent_off: np.ndarray, sent_len: np.ndarray, budget: int,
               budget_stride: Optional[int] = None, max_sel: Optional[int] = None):
        """-> (sel_sent[Hkv][max_sel], n_sel[Hkv], tok_idx[Hkv][stride], n_tok[Hkv]); unused slots are -1."""
        score = np.ascontiguousarray(score, dtype=np.float32)
        H, S = score.shape
        sent_off = np.ascontiguousarray(sent_off, dtype=np.int32)
        sent_len = np.ascontiguousarray(sent_len, dtype=np.int32)
        stride = max(budget, 1) if budget_stride is None else budget_stride
        assert stride >= budget
        msel = max(min(S, max(budget, 0)), 1) if max_sel is None else max_sel
        sel = np.full((H, msel), -1, dtype=np.int32)
        n_sel = np.zeros(H, dtype=np.int32)
        tok_idx = np.full((H, stride), -1, dtype=np.int32)
        n_tok = np.zeros(H, dtype=np.int32)
        self.lib.skvo_select(_ptr(score, _f32p), _ptr(sent_off, _i32p), _ptr(sent_len, _i32p), S, H, budget,
                             _ptr(sel, _i32p), msel, _ptr(n_sel, _i32p), _ptr(tok_idx, _i32p), stride,
                             _ptr(n_tok, _i32p))
        return sel, n_sel, tok_idx, n_tok

    def gather(self, pool: np.ndarray, tok_idx: np.ndarray, n_tok: np.ndarray) -> np.ndarray:
        """pool [Hkv][T][D] -> [Hkv][stride][D]; rows past n_tok[h] stay zero."""
        pool = np.ascontiguousarray(pool)
        H, T, D = pool.shape
        tok_idx = np.ascontiguousarray(tok_idx, dtype=np.int32)
        n_tok = np.ascontiguousarray(n_tok, dtype=np.int32)
        stride = tok_idx.shape[1]
        out = np.zeros((H, stride, D), dtype=pool.dtype)
        self.lib.skvo_gather(pool.ctypes.data_as(_vp), _dtype_of(pool), H, T, D, _ptr(tok_idx, _i32p), stride,
                             _ptr(n_tok, _i32p), out.ctypes.data_as(_vp))
        return out

    def attend(self, q: np.ndarray, K_sel: np.ndarray, V_sel: np.ndarray, n_tok: np.ndarray):
        """q [Hq][D], K_sel/V_sel [Hkv][stride][D] -> (out float32 [Hq][D], lse float32 [Hq])."""
        q = np.ascontiguousarray(q)
        K_sel = np.ascontiguousarray(K_sel)
        V_sel = np.ascontiguousarray(V_sel)
        n_tok = np.ascontiguousarray(n_tok, dtype=np.int32)
        Hq, D = q.shape
        H, stride, _ = K_sel.shape
        assert _dtype_of(q) == _dtype_of(K_sel) == _dtype_of(V_sel)
        out = np.zeros((Hq, D), dtype=np.float32)
        lse = np.zeros(Hq, dtype=np.float32)
        self.lib.skvo_attend(q.ctypes.data_as(_vp), K_sel.ctypes.data_as(_vp), V_sel.ctypes.data_as(_vp),
                             _dtype_of(q), Hq, H, D, _ptr(n_tok, _i32p), stride, _ptr(out, _f32p), _ptr(lse, _f32p))
        return out, lse

    def merge_lse(self, out_a: np.ndarray, lse_a: np.ndarray, out_b: np.ndarray, lse_b: np.ndarray):
        """Two partial attention results over disjoint token sets -> (out, lse) over their union."""
        out_a, out_b = np.ascontiguousarray(out_a, np.float32), np.ascontiguousarray(out_b, np.float32)
        lse_a, lse_b = np.ascontiguousarray(lse_a, np.float32), np.ascontiguousarray(lse_b, np.float32)
        n, D = out_a.shape
        out, lse = np.zeros((n, D), np.float32), np.zeros(n, np.float32)
        self.lib.skvo_merge_lse(_ptr(out_a, _f32p), _ptr(lse_a, _f32p), _ptr(out_b, _f32p), _ptr(lse_b, _f32p), n, D,
                                _ptr(out, _f32p), _ptr(lse, _f32p))
        return out, lse

    def decode_step(self, q_score, q_attn, K_layer, V_layer, semvec_layer, sent_off, sent_len, budget):
        """The whole decode chain for one layer, one sequence (score -> select -> gather -> attend)."""
        sc = self.score(q_score, semvec_layer)
        sel, n_sel, tok_idx, n_tok = self.select(sc, sent_off, sent_len, budget)
        Ks = self.gather(K_layer, tok_idx, n_tok)
        Vs = self.gather(V_layer, tok_idx, n_tok)
        out, lse = self.attend(q_attn, Ks, Vs, n_tok)
        return dict(score=sc, sel_sent=sel, n_sel=n_sel, tok_idx=tok_idx, n_tok=n_tok, K_sel=Ks, V_sel=Vs,
                    out=out, lse=lse)


class QueryCache:
    """The sentence cache Q_s of Eq. 2 for one sequence: the list of queries since the last boundary."""

    def __init__(self, oracle: Oracle, per: int, cap: int):
        self.o, self.per, self.cap = oracle, per, cap
        self.cache = np.zeros((cap, per), dtype=np.float32)
        self.n = np.zeros(1, dtype=np.int32)

    def __len__(self) -> int:
        return int(self.n[0])

    def step(self, q_t: np.ndarray, tok: int, bitmap: np.ndarray, vocab: int):
        """Append q_t, -> (q-bar float32, q-bar in q_t's storage type); Q_s is emptied if tok is a terminator."""
        q_t = np.ascontiguousarray(q_t)
        assert q_t.size == self.per
        bitmap = np.ascontiguousarray(bitmap, dtype=np.uint32)
        qbar = np.zeros(q_t.shape, dtype=np.float32)
        store = np.zeros(q_t.shape, dtype=q_t.dtype)
        rc = self.o.lib.skvo_query_cache_step(q_t.ctypes.data_as(_vp), _dtype_of(q_t), self.per, int(tok),
                                              _ptr(bitmap, _u32p), vocab, _ptr(self.cache, _f32p), self.cap,
                                              _ptr(self.n, _i32p), _ptr(qbar, _f32p), store.ctypes.data_as(_vp))
        if rc != 0:
            raise OverflowError(f"sentence cache holds {self.cap} queries already")
        return qbar, store


_cache = {}


def get(real: str = "f32") -> Oracle:
    if real not in _cache:
        _cache[real] = Oracle(real)
    return _cache[real]
