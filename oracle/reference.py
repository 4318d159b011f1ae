"""ctypes front end of the UniSparse CPU oracle -- TEST INFRASTRUCTURE ONLY.

Loads ``liboracle.so`` (plain C, built from ``unisparse_oracle.c`` with gcc) and adds
the bookkeeping the paper leaves to the caller: the loop over heads, grouped-query
head mapping, packed variable-length batches (each sequence is an independent
problem) and optional head-level compression (Eq. (2), Alg. 1 "if c_h > 1").

Nothing here may be imported by the product package; the product never falls back
to this code.

Array conventions (host numpy, values exactly representable in bf16):
  Q : float32 [H, T, d]      K, V : float32 [H_kv, T, d]      T = sum of sequence lengths
  cu_seqlens : int sequence, B+1 entries, cu[0] = 0, cu[B] = T
  mask  : uint8  [H, NQ, NK]  NQ = sum_b ceil(L_b / S) (packed query-block rows),
                              NK = max_b ceil(L_b / S); column j = key block j of the row's own sequence
  score : float64 [H, NQ, NK] (0 outside the row's valid set)
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "unisparse_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

TOP_P = 0
TOP_K = 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a second or two). Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c99", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    f32p = ctypes.POINTER(ctypes.c_float)
    f64p = ctypes.POINTER(ctypes.c_double)
    i32p = ctypes.POINTER(ctypes.c_int32)
    u8p = ctypes.POINTER(ctypes.c_uint8)
    i64 = ctypes.c_int64
    ci = ctypes.c_int
    lib.oracle_bf16_round_scalar.argtypes = [ctypes.c_float]
    lib.oracle_bf16_round_scalar.restype = ctypes.c_float
    lib.oracle_avgpool_seq.argtypes = [f32p, i64, ci, ci, f32p]
    lib.oracle_avgpool_seq.restype = None
    lib.oracle_maxpool_seq.argtypes = [f32p, i64, ci, ci, f32p]
    lib.oracle_maxpool_seq.restype = None
    lib.oracle_stochpool_seq.argtypes = [f32p, i64, ci, ci, f32p, f32p, i32p]
    lib.oracle_stochpool_seq.restype = None
    lib.oracle_avgpool_head.argtypes = [f32p, ci, i64, ci, ci, f32p]
    lib.oracle_avgpool_head.restype = None
    lib.oracle_block_scores.argtypes = [f32p, f32p, i64, i64, ci, ci, ci, ci, ci, ctypes.c_double,
                                        i32p, ci, i64, f64p]
    lib.oracle_block_scores.restype = None
    lib.oracle_select_top_p.argtypes = [f64p, ci, ctypes.c_double, u8p]
    lib.oracle_select_top_p.restype = ci
    lib.oracle_select_top_k.argtypes = [f64p, ci, ctypes.c_double, u8p]
    lib.oracle_select_top_k.restype = ci
    lib.oracle_masked_attention.argtypes = [f32p, f32p, f32p, i64, ci, ci, ci, ctypes.c_double,
                                            u8p, i32p, ci, f64p, f64p]
    lib.oracle_masked_attention.restype = None
    _lib = lib
    return lib


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _f32c(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


# --------------------------------------------------------------------------- pooling

def avgpool_seq(x: np.ndarray, c: int) -> np.ndarray:
    """Eq. (1): x [L, d] float32 (one sequence) -> [ceil(L / c), d] composite tokens (bf16-valued float32)."""
    lib = _load()
    x = _f32c(x)
    L, d = x.shape
    out = np.empty((-(-L // c), d), dtype=np.float32)
    lib.oracle_avgpool_seq(_p(x, ctypes.c_float), L, d, c, _p(out, ctypes.c_float))
    return out


def maxpool_seq(x: np.ndarray, c: int) -> np.ndarray:
    """Channel-wise maximum over the windows of Eq. (1) (ablation "Compression Strategy"): x [L, d] -> [ceil(L / c), d]."""
    lib = _load()
    x = _f32c(x)
    L, d = x.shape
    out = np.empty((-(-L // c), d), dtype=np.float32)
    lib.oracle_maxpool_seq(_p(x, ctypes.c_float), L, d, c, _p(out, ctypes.c_float))
    return out


def stochpool_seq(x: np.ndarray, c: int, u: np.ndarray, return_choice: bool = False):
    """Stochastic pooling (ablation "Compression Strategy"): one token per window, drawn by its share of the
    window's L2 norms from the uniform numbers u [ceil(L / c)].  x [L, d] -> [ceil(L / c), d] (, offsets chosen)."""
    lib = _load()
    x = _f32c(x)
    L, d = x.shape
    Lc = -(-L // c)
    u = _f32c(u)
    assert u.shape == (Lc,)
    out = np.empty((Lc, d), dtype=np.float32)
    sel = np.empty(Lc, dtype=np.int32)
    lib.oracle_stochpool_seq(_p(x, ctypes.c_float), L, d, c, _p(u, ctypes.c_float), _p(out, ctypes.c_float),
                             _p(sel, ctypes.c_int32))
    return (out, sel) if return_choice else out


POOL_AVG, POOL_MAX, POOL_STOCHASTIC = 0, 1, 2


def pool_seq(x: np.ndarray, c: int, pool: int = POOL_AVG, u: Optional[np.ndarray] = None) -> np.ndarray:
    if pool == POOL_STOCHASTIC:
        return stochpool_seq(x, c, u)
    return maxpool_seq(x, c) if pool == POOL_MAX else avgpool_seq(x, c)


def avgpool_head(x: np.ndarray, c_h: int) -> np.ndarray:
    """Eq. (2): x [H, Lc, d] -> [H // c_h, Lc, d]."""
    lib = _load()
    x = _f32c(x)
    H, Lc, d = x.shape
    out = np.empty((H // c_h, Lc, d), dtype=np.float32)
    lib.oracle_avgpool_head(_p(x, ctypes.c_float), H, Lc, d, c_h, _p(out, ctypes.c_float))
    return out


# --------------------------------------------------------------------------- scores

def block_scores_head(qt: np.ndarray, kt: np.ndarray, S: int, c_q: int, c_k: int, causal_mode: int,
                      scale: float, rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """Score(i, :) of Eq. (3) for one (compressed) head.

    qt [Lq, d], kt [Lk, d] composite tokens.  Returns float64 [len(rows), N].
    """
    lib = _load()
    qt = _f32c(qt)
    kt = _f32c(kt)
    Lq, d = qt.shape
    Lk = kt.shape[0]
    N = -(-(Lk * c_k) // S)                      # the last block may be a shorter remainder
    if rows is None:
        rows = np.arange(-(-(Lq * c_q) // S), dtype=np.int32)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    out = np.zeros((len(rows), N), dtype=np.float64)
    lib.oracle_block_scores(_p(qt, ctypes.c_float), _p(kt, ctypes.c_float), Lq, Lk, d, S, c_q, c_k,
                            causal_mode, float(scale), _p(rows, ctypes.c_int32), len(rows), N,
                            _p(out, ctypes.c_double))
    return out


def select_row(score_valid: np.ndarray, mode: int, param: float) -> np.ndarray:
    """Select key blocks of one row from the scores of its valid blocks (uint8 0/1)."""
    lib = _load()
    s = np.ascontiguousarray(score_valid, dtype=np.float64)
    sel = np.zeros(len(s), dtype=np.uint8)
    if mode == TOP_P:
        lib.oracle_select_top_p(_p(s, ctypes.c_double), len(s), float(param), _p(sel, ctypes.c_uint8))
    elif mode == TOP_K:
        lib.oracle_select_top_k(_p(s, ctypes.c_double), len(s), float(param), _p(sel, ctypes.c_uint8))
    else:
        raise ValueError("mode")
    return sel


def select_mask(score: np.ndarray, cu_seqlens: Sequence[int], S: int, causal: bool, mode: int,
                param: float, rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """Alg. 1 step 4 on a score tensor [H, NQ, NK] (any float dtype) -> uint8 mask of the same shape.

    Row r (packed query-block index) belongs to sequence b with local index i; its valid set is
    {j <= i} when causal, else {j < N_b}.  Only ``rows`` (default: all) are filled.
    """
    score = np.asarray(score)
    H, NQ, NK = score.shape
    seq_of, loc_of, nb_of = _row_tables(cu_seqlens, S)
    mask = np.zeros((H, NQ, NK), dtype=np.uint8)
    rr = range(NQ) if rows is None else rows
    for h in range(H):
        for r in rr:
            nv = loc_of[r] + 1 if causal else nb_of[r]
            mask[h, r, :nv] = select_row(score[h, r, :nv].astype(np.float64), mode, param)
    return mask


def _row_tables(cu_seqlens, S):
    seq_of, loc_of, nb_of = [], [], []
    for b in range(len(cu_seqlens) - 1):
        Lb = int(cu_seqlens[b + 1]) - int(cu_seqlens[b])
        nb = -(-Lb // S)                         # ceil: a shorter last block when S does not divide L_b
        for i in range(nb):
            seq_of.append(b)
            loc_of.append(i)
            nb_of.append(nb)
    return seq_of, loc_of, nb_of


def composite_offsets(cu_seqlens, c: int):
    """Packed offsets of the composite tokens: sequence b owns ceil(L_b / c) of them."""
    off = [0]
    for b in range(len(cu_seqlens) - 1):
        off.append(off[-1] + -(-(int(cu_seqlens[b + 1]) - int(cu_seqlens[b])) // c))
    return off


def _pool_packed(X: np.ndarray, cu_seqlens, c: int, pool: int = POOL_AVG, u: Optional[np.ndarray] = None) -> np.ndarray:
    """Eq. (1) per sequence (windows never straddle sequences; a last window may be partial), packed again.
    u [heads, packed composite tokens]: the uniform numbers of stochastic pooling, laid out like the result."""
    off = composite_offsets(cu_seqlens, c)
    return np.stack([np.concatenate([pool_seq(X[h, int(cu_seqlens[b]):int(cu_seqlens[b + 1])], c, pool,
                                              None if u is None else u[h, off[b]:off[b + 1]])
                                     for b in range(len(cu_seqlens) - 1)]) for h in range(X.shape[0])])


def composite_tokens(Q: np.ndarray, K: np.ndarray, cu_seqlens, c_q: int, c_k: int, c_h: int = 1,
                     pool: int = POOL_AVG, rand=None):
    """Alg. 1 step 1 for a packed batch.

    Returns (Qt [H', sum_b ceil(L_b/c_q), d], Kt [H', sum_b ceil(L_b/c_k), d]) with H' = H / c_h *query-side*
    compressed heads; the keys are first repeated over the query heads of their group (query head h uses KV
    head h // G), then pooled over heads exactly like the queries, so row h' of Kt pairs with row h' of Qt.
    """
    H, T, d = Q.shape
    Hkv = K.shape[0]
    G = H // Hkv
    rq, rk = rand if rand is not None else (None, None)   # stochastic pooling: uniforms [H, Tq], [Hkv, Tk]
    Qt = _pool_packed(Q, cu_seqlens, c_q, pool, rq)
    Ktkv = _pool_packed(K, cu_seqlens, c_k, pool, rk)
    if c_h == 1:
        Kt = Ktkv[np.arange(H) // G]
        return Qt, Kt
    Qt = avgpool_head(Qt, c_h)
    Kt = avgpool_head(Ktkv[np.arange(H) // G], c_h)
    return Qt, Kt


def block_scores(Q: np.ndarray, K: np.ndarray, cu_seqlens: Sequence[int], S: int, c_q: int, c_k: int,
                 causal: bool, scale: Optional[float] = None, c_h: int = 1,
                 rows: Optional[Sequence[int]] = None, literal_alg1: bool = False, pool: int = POOL_AVG,
                 rand=None) -> np.ndarray:
    """Alg. 1 steps 1-3 for a packed batch.  Returns float64 [H / c_h, NQ, NK]; only ``rows`` are filled."""
    H, T, d = Q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    Qt, Kt = composite_tokens(Q, K, cu_seqlens, c_q, c_k, c_h, pool, rand)
    Hc = Qt.shape[0]
    seq_of, loc_of, nb_of = _row_tables(cu_seqlens, S)
    NQ = len(seq_of)
    NK = max(nb_of)
    score = np.zeros((Hc, NQ, NK), dtype=np.float64)
    want = set(range(NQ)) if rows is None else set(int(r) for r in rows)
    cmode = (2 if literal_alg1 else 1) if causal else 0
    oq, ok = composite_offsets(cu_seqlens, c_q), composite_offsets(cu_seqlens, c_k)
    row0 = 0
    for b in range(len(cu_seqlens) - 1):
        t0, t1 = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        nb = -(-(t1 - t0) // S)
        loc = [i for i in range(nb) if (row0 + i) in want]
        if loc:
            for h in range(Hc):
                sc = block_scores_head(Qt[h, oq[b]:oq[b + 1]], Kt[h, ok[b]:ok[b + 1]], S, c_q, c_k,
                                       cmode, scale, loc)
                if causal:                                   # Alg. 1 step 4, first line: drop j > i
                    for n, i in enumerate(loc):
                        sc[n, i + 1:] = 0.0
                score[h, [row0 + i for i in loc], :nb] = sc
        row0 += nb
    return score


def build_mask(Q: np.ndarray, K: np.ndarray, cu_seqlens: Sequence[int], S: int, c_q: int, c_k: int,
               causal: bool, mode: int, param: float, scale: Optional[float] = None, c_h: int = 1,
               rows: Optional[Sequence[int]] = None, pool: int = POOL_AVG, rand=None):
    """Alg. 1 steps 1-4 (+ head broadcast).  Returns (mask uint8 [H, NQ, NK], score float64 [H/c_h, NQ, NK])."""
    score = block_scores(Q, K, cu_seqlens, S, c_q, c_k, causal, scale, c_h, rows, pool=pool, rand=rand)
    m = select_mask(score, cu_seqlens, S, causal, mode, param, rows)
    if c_h > 1:
        m = np.repeat(m, c_h, axis=0)                        # Broadcast_head
    return m, score


# --------------------------------------------------------------------------- attention

def masked_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, cu_seqlens: Sequence[int], S: int,
                     causal: bool, mask: Optional[np.ndarray], scale: Optional[float] = None,
                     rows: Optional[Sequence[int]] = None, heads: Optional[Sequence[int]] = None):
    """Block-sparse attention by its definition (Sec. 2.2).  mask None = every valid block (dense).

    Returns (O float64 [H, T, d], lse float64 [H, T]); only the tokens of ``rows`` (packed
    query-block rows, default all) of ``heads`` (default all) are filled, the rest is NaN.
    """
    lib = _load()
    Q, K, V = _f32c(Q), _f32c(K), _f32c(V)
    H, T, d = Q.shape
    G = H // K.shape[0]
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    seq_of, loc_of, nb_of = _row_tables(cu_seqlens, S)
    NQ = len(seq_of)
    want = set(range(NQ)) if rows is None else set(int(r) for r in rows)
    O = np.full((H, T, d), np.nan, dtype=np.float64)
    lse = np.full((H, T), np.nan, dtype=np.float64)
    hh = range(H) if heads is None else heads
    row0 = 0
    for b in range(len(cu_seqlens) - 1):
        t0, t1 = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        L = t1 - t0
        nb = -(-L // S)
        loc = np.array([i for i in range(nb) if (row0 + i) in want], dtype=np.int32)
        if len(loc):
            for h in hh:
                if mask is None:
                    mb = np.ones((nb, nb), dtype=np.uint8)
                else:
                    mb = np.ascontiguousarray(mask[h, row0:row0 + nb, :nb], dtype=np.uint8)
                q = np.ascontiguousarray(Q[h, t0:t1])
                k = np.ascontiguousarray(K[h // G, t0:t1])
                v = np.ascontiguousarray(V[h // G, t0:t1])
                o = np.empty((len(loc), S, d), dtype=np.float64)
                ls = np.empty((len(loc), S), dtype=np.float64)
                lib.oracle_masked_attention(_p(q, ctypes.c_float), _p(k, ctypes.c_float),
                                            _p(v, ctypes.c_float), L, d, S, int(causal), float(scale),
                                            _p(mb, ctypes.c_uint8), _p(loc, ctypes.c_int32), len(loc),
                                            _p(o, ctypes.c_double), _p(ls, ctypes.c_double))
                for n, i in enumerate(loc):
                    m = min(S, L - i * S)                    # tokens of the block that exist
                    O[h, t0 + i * S:t0 + i * S + m] = o[n, :m]
                    lse[h, t0 + i * S:t0 + i * S + m] = ls[n, :m]
        row0 += nb
    return O, lse


def sparsity(mask: np.ndarray, cu_seqlens: Sequence[int], S: int, causal: bool) -> float:
    """rho of Sec. 2.2: 1 - selected / valid block pairs (valid = j <= i under causality)."""
    seq_of, loc_of, nb_of = _row_tables(cu_seqlens, S)
    valid = sum((l + 1) if causal else n for l, n in zip(loc_of, nb_of)) * mask.shape[0]
    return 1.0 - float(mask.sum()) / float(valid)
