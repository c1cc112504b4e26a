"""StructKV CPU oracle (fp64, plain C) -- TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It shares no code with the HIP library and imports nothing from
it.  The arithmetic lives in structkv_oracle.c; this file only builds it with
gcc and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "structkv_oracle.c")
# STRUCTKV_ORACLE_SANITIZE=1 (set by tests/test_host_sanitizers.py for its child process) selects a build with
# AddressSanitizer and UndefinedBehaviorSanitizer; the process must then have libasan preloaded.
_SANITIZE = os.environ.get("STRUCTKV_ORACLE_SANITIZE") == "1"
_LIB = os.path.join(_HERE, "libstructkv_oracle_san.so" if _SANITIZE else "libstructkv_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (x86-64-v3 so the binary also runs on the GPU machine's host)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer"] if _SANITIZE else ["-O3"]
        cmd = ["gcc"] + opt + ["-march=x86-64-v3", "-fopenmp", "-shared", "-fPIC", "-std=c11",
                               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32, i64, f64, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.skv_oracle_num_threads.restype = i32
        lib.skv_oracle_score_layer.restype = i32
        lib.skv_oracle_score_layer.argtypes = [i32, vp, vp, i64, i64, i32, i32, i32, i32, i64, i32, f64,
                                               vp, vp, vp, vp]
        lib.skv_oracle_accumulate.restype = None
        lib.skv_oracle_accumulate.argtypes = [vp, vp, i64, f64, f64]
        lib.skv_oracle_centrality_closed.restype = None
        lib.skv_oracle_centrality_closed.argtypes = [vp, i32, i64, f64, vp]
        lib.skv_oracle_select_topk.restype = i32
        lib.skv_oracle_select_topk.argtypes = [vp, i64, i64, i64, vp]
        lib.skv_oracle_gather_rows.restype = None
        lib.skv_oracle_gather_rows.argtypes = [vp, i64, i64, vp, i64, i64, i32, i64, vp, i64, i64, i64]
        lib.skv_oracle_block_scores.restype = None
        lib.skv_oracle_block_scores.argtypes = [vp, i64, i64, vp]
        lib.skv_oracle_pivot_metrics.restype = None
        lib.skv_oracle_pivot_metrics.argtypes = [vp, i32, i32, i64, f64, vp, vp]
        lib.skv_oracle_transition.restype = i32
        lib.skv_oracle_transition.argtypes = [vp, vp, vp, i32, f64, f64, f64, vp]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().skv_oracle_num_threads())


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _as_input(a) -> Tuple[np.ndarray, int]:
    """numpy float32 -> dtype 0; numpy uint16 holding bf16 bit patterns -> dtype 1."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float32:
        return a, 0
    if a.dtype == np.uint16:
        return a, 1
    raise TypeError("oracle inputs must be float32 or uint16 (bf16 bits), got %s" % a.dtype)


def score_layer(q_win, k, n_q_heads: int, n_kv_heads: int, head_dim: int, window: int,
                seq_lens: Sequence[int], causal: bool = False, scale: float = 0.0,
                want_probs: bool = False):
    """q_win [B,Hq,w,d], k [G,total,d] (float32 or bf16-bits uint16).

    Returns (indeg [total] f64, entropy [B] f64, entropy_per_head [B,Hq] f64, probs list or None).
    """
    lib = _load()
    q_win, dq = _as_input(q_win)
    k, dk = _as_input(k)
    assert dq == dk
    B = len(seq_lens)
    Hq, G, d, w = n_q_heads, n_kv_heads, head_dim, window
    total = int(sum(seq_lens))
    assert q_win.shape == (B, Hq, w, d), q_win.shape
    assert k.shape == (G, total, d), k.shape
    indeg = np.zeros(total, dtype=np.float64)
    ent = np.zeros(B, dtype=np.float64)
    ent_h = np.zeros((B, Hq), dtype=np.float64)
    probs: Optional[List[np.ndarray]] = [] if want_probs else None
    esz = k.dtype.itemsize
    off = 0
    for b, n in enumerate(seq_lens):
        n = int(n)
        if n == 0:
            if want_probs:
                probs.append(np.zeros((Hq, w, 0)))
            continue
        p = np.zeros((Hq, w, n), dtype=np.float64) if want_probs else None
        e = ctypes.c_double(0.0)
        kb = ctypes.c_void_p(k.ctypes.data + off * d * esz)
        rc = lib.skv_oracle_score_layer(dq, _ptr(q_win[b]), kb, total * d, d, Hq, G, d, w, n,
                                        int(bool(causal)), float(scale), _ptr(indeg[off:off + n]),
                                        ctypes.byref(e), _ptr(ent_h[b]),
                                        _ptr(p) if want_probs else None)
        if rc != 0:
            raise ValueError("skv_oracle_score_layer failed with code %d" % rc)
        ent[b] = e.value
        if want_probs:
            probs.append(p)
        off += n
    return indeg, ent, ent_h, probs


def accumulate(centrality: np.ndarray, indeg: np.ndarray, lam: float, inv_w: float) -> None:
    """In place: C <- lam*C + inv_w*D."""
    assert centrality.dtype == np.float64 and indeg.dtype == np.float64
    assert centrality.flags.c_contiguous and indeg.flags.c_contiguous and centrality.shape == indeg.shape
    _load().skv_oracle_accumulate(_ptr(centrality), _ptr(indeg), centrality.size, float(lam), float(inv_w))


def centrality_closed_form(S: np.ndarray, lam: float) -> np.ndarray:
    S = np.ascontiguousarray(S, dtype=np.float64)
    L, n = S.shape
    C = np.zeros(n, dtype=np.float64)
    _load().skv_oracle_centrality_closed(_ptr(S), L, n, float(lam), _ptr(C))
    return C


def select_topk(scores, seq_lens: Sequence[int], k_per_seq: Sequence[int], keep_tail: int) -> List[np.ndarray]:
    """Per sequence: ascending int32 indices (sequence-local) of the top-k of the prefix plus the tail."""
    lib = _load()
    scores = np.ascontiguousarray(scores, dtype=np.float64)  # float32 -> float64 is exact
    out = []
    off = 0
    for n, k in zip(seq_lens, k_per_seq):
        n, k = int(n), int(k)
        idx = np.zeros(k + keep_tail, dtype=np.int32)
        seg = np.ascontiguousarray(scores[off:off + n])
        rc = lib.skv_oracle_select_topk(_ptr(seg), n, k, keep_tail, _ptr(idx))
        if rc != 0:
            raise ValueError("skv_oracle_select_topk failed with code %d" % rc)
        out.append(idx)
        off += n
    return out


def gather_kv(src: np.ndarray, idx_per_seq: Sequence[np.ndarray], seq_lens: Sequence[int]) -> np.ndarray:
    """src [G,total,d] (any 2- or 4-byte dtype) -> [G, sum(len(idx_b)), d], exact row copies."""
    lib = _load()
    src = np.ascontiguousarray(src)
    G, total, d = src.shape
    rows = int(sum(len(i) for i in idx_per_seq))
    dst = np.zeros((G, rows, d), dtype=src.dtype)
    rb = d * src.dtype.itemsize
    so = do = 0
    for idx, n in zip(idx_per_seq, seq_lens):
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        if len(idx):
            lib.skv_oracle_gather_rows(_ptr(src), total * rb, rb, _ptr(dst), rows * rb, rb, G, rb,
                                       _ptr(idx), len(idx), so, do)
        so += int(n)
        do += len(idx)
    return dst


def truncate_hidden(h: np.ndarray, positions: Optional[np.ndarray], idx_per_seq: Sequence[np.ndarray],
                    seq_lens: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 11-12: keep hidden states and positions at the structural indices.

    h [total, hidden] (any 2- or 4-byte dtype), positions [total] int64 or None (= 0..n_b-1 per sequence).
    Returns (h' [rows, hidden], positions' [rows] int64), rows = sum(len(idx_b)), exact row copies.
    """
    h = np.ascontiguousarray(h)
    total = h.shape[0]
    if positions is None:
        positions = np.concatenate([np.arange(n, dtype=np.int64) for n in seq_lens]) if len(seq_lens) else \
            np.zeros(0, np.int64)
    positions = np.ascontiguousarray(positions, dtype=np.int64)
    assert positions.shape == (total,)
    h_out = gather_kv(h[None], idx_per_seq, seq_lens)[0]
    p_out = gather_kv(positions.view(np.int32).reshape(1, total, 2), idx_per_seq, seq_lens)[0]
    return h_out, np.ascontiguousarray(p_out).view(np.int64).reshape(-1)


def block_scores(scores: np.ndarray, seq_lens: Sequence[int], block: int) -> List[np.ndarray]:
    """Sec. 4.1 (implementation details): per sequence, the sum of the scores of every cache block of
    `block` tokens (the last block of a sequence may be shorter).  fp64."""
    lib = _load()
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    out, off = [], 0
    for n in seq_lens:
        n = int(n)
        o = np.zeros((n + block - 1) // block, dtype=np.float64)
        if n:
            seg = np.ascontiguousarray(scores[off:off + n])
            lib.skv_oracle_block_scores(_ptr(seg), n, int(block), _ptr(o))
        out.append(o)
        off += n
    return out


def pivot_metrics(probs: Sequence[np.ndarray], top_frac: float = 0.1) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 5-6 per sequence from the attention rows score_layer(want_probs=True) returns ([Hq,w,n_b] each).

    Reading: a head's attention is pooled (mean) over the window rows; sparsity = mass of its ceil(top_frac n)
    largest keys, variance = population variance over the keys; both averaged over the heads.
    Returns (sparsity [B], variance [B]) fp64.
    """
    lib = _load()
    rho = np.zeros(len(probs))
    var = np.zeros(len(probs))
    for b, p in enumerate(probs):
        p = np.ascontiguousarray(p, dtype=np.float64)
        Hq, w, n = p.shape
        if n == 0:
            continue
        r, v = ctypes.c_double(0.0), ctypes.c_double(0.0)
        lib.skv_oracle_pivot_metrics(_ptr(p), Hq, w, n, float(top_frac), ctypes.byref(r), ctypes.byref(v))
        rho[b], var[b] = r.value, v.value
    return rho, var


def transition_scores(entropy: Sequence[float], sparsity: Sequence[float], variance: Sequence[float],
                      weights: Sequence[float] = (0.2, 0.3, 0.5)) -> Tuple[np.ndarray, int]:
    """Eq. 7-9 over the given layers: (T [L] with T[0] = 0, L* = argmax_l T_l + 1)."""
    lib = _load()
    H = np.ascontiguousarray(entropy, dtype=np.float64)
    R = np.ascontiguousarray(sparsity, dtype=np.float64)
    V = np.ascontiguousarray(variance, dtype=np.float64)
    assert H.shape == R.shape == V.shape and H.ndim == 1
    T = np.zeros(len(H))
    ls = lib.skv_oracle_transition(_ptr(H), _ptr(R), _ptr(V), len(H), float(weights[0]), float(weights[1]),
                                   float(weights[2]), _ptr(T))
    return T, int(ls)
