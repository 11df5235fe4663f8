"""ctypes front end of the C oracle (test infrastructure only; never imported by the product path).

Marshals numpy arrays into oracle/libsfi_oracle.so; no arithmetic happens here.
bf16 tensors are ``numpy.uint16`` bit patterns, layouts as in sfi_oracle.c.
"""
from __future__ import annotations

import ctypes as C
import math
import os
from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

from .build import LIB, build_oracle

_lib = None


class _Cfg(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("d", C.c_int32),
        ("n_sink", C.c_int32), ("recent", C.c_int32),
        ("scale", C.c_double),
        ("k_stride_b", C.c_int64), ("k_stride_h", C.c_int64), ("k_stride_t", C.c_int64),
        ("v_stride_b", C.c_int64), ("v_stride_h", C.c_int64), ("v_stride_t", C.c_int64),
        ("mode", C.c_int32), ("nms_radius", C.c_int32),
        ("alpha", C.c_double),
        ("gamma", C.c_double), ("beta", C.c_double), ("p", C.c_double), ("eta", C.c_double),
        ("lambda_clip", C.c_double), ("alpha_soft", C.c_double), ("alpha_cross", C.c_double),
        ("temp", C.c_double), ("eps", C.c_double),
    ]


@dataclass
class SelectorParams:
    """Selector hyper-parameters.  lambda_clip, alpha_soft, alpha_cross, eps are the paper's defaults
    (Sec. 5 "Default SFI configuration", Sec. 3.2); the rest are not given by the paper."""
    mode: int = 0
    alpha: float = 1.0
    gamma: float = 0.5
    beta: float = 1.0
    p: float = 2.0
    eta: float = 0.5
    lambda_clip: float = 0.02
    alpha_soft: float = 0.5
    alpha_cross: float = 0.35
    temp: float = 1.0
    eps: float = 1e-8
    nms_radius: int = 2


def lib() -> C.CDLL:
    """The compiled oracle.  SFI_ORACLE_LIB names another build of sfi_oracle.c to load instead (the mutation
    test runs the pins against deliberately broken copies this way)."""
    global _lib
    if _lib is None:
        path = os.environ.get("SFI_ORACLE_LIB") or LIB
        if path == LIB and not os.path.exists(LIB):
            build_oracle()
        _lib = C.CDLL(path)
        _lib.sfio_num_threads.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(lib().sfio_num_threads())


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _cfg(B, Hq, Hkv, d, n_sink, recent, scale, K=None, V=None, sp: Optional[SelectorParams] = None) -> _Cfg:
    sp = sp or SelectorParams()
    c = _Cfg()
    c.B, c.Hq, c.Hkv, c.d, c.n_sink, c.recent = B, Hq, Hkv, d, n_sink, recent
    c.scale = (1.0 / math.sqrt(d)) if scale is None else float(scale)
    if K is not None:
        assert K.dtype == np.uint16 and K.ndim == 4 and K.strides[3] == 2
        c.k_stride_b, c.k_stride_h, c.k_stride_t = (s // 2 for s in K.strides[:3])
    if V is not None:
        assert V.dtype == np.uint16 and V.ndim == 4 and V.strides[3] == 2
        c.v_stride_b, c.v_stride_h, c.v_stride_t = (s // 2 for s in V.strides[:3])
    c.mode, c.nms_radius = sp.mode, sp.nms_radius
    c.alpha, c.gamma, c.beta, c.p, c.eta = sp.alpha, sp.gamma, sp.beta, sp.p, sp.eta
    c.lambda_clip, c.alpha_soft, c.alpha_cross, c.temp, c.eps = (
        sp.lambda_clip, sp.alpha_soft, sp.alpha_cross, sp.temp, sp.eps)
    return c


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def logits(q: np.ndarray, K: np.ndarray, ctx_len, scale=None) -> np.ndarray:
    """l[b, g, j] = scale * <q[b, g], K[b, g // G, j]>; float64 [B, Hq, max ctx_len], 0 beyond ctx_len."""
    B, Hq, d = q.shape
    Hkv = K.shape[1]
    ctx_len = _i32(ctx_len)
    ld = int(max(1, ctx_len.max()))
    out = np.zeros((B, Hq, ld), dtype=np.float64)
    c = _cfg(B, Hq, Hkv, d, 0, 0, scale, K=K)
    q = np.ascontiguousarray(q)
    rc = lib().sfio_logits(C.byref(c), _p(q), _p(K), _p(ctx_len), _p(out), C.c_int64(ld))
    assert rc == 0
    return out


def dense(q: np.ndarray, K: np.ndarray, V: np.ndarray, ctx_len, scale=None) -> np.ndarray:
    """Dense attention over [0, ctx_len[b]): float64 [B, Hq, d]."""
    B, Hq, d = q.shape
    Hkv = K.shape[1]
    ctx_len = _i32(ctx_len)
    out = np.zeros((B, Hq, d), dtype=np.float64)
    c = _cfg(B, Hq, Hkv, d, 0, 0, scale, K=K, V=V)
    q = np.ascontiguousarray(q)
    rc = lib().sfio_dense(C.byref(c), _p(q), _p(K), _p(V), _p(ctx_len), _p(out))
    assert rc == 0
    return out


def sparse(q, K, V, sel_idx, n_sel, recent_start, ctx_len, n_sink: int, scale=None) -> np.ndarray:
    """Sparse attention over [0, n_sink) U sel_idx[b, h, :n_sel] U [recent_start[b], ctx_len[b])."""
    B, Hq, d = q.shape
    Hkv = K.shape[1]
    ctx_len, recent_start = _i32(ctx_len), _i32(recent_start)
    sel_idx, n_sel = _i32(sel_idx), _i32(n_sel)
    assert sel_idx.ndim == 3 and sel_idx.shape[:2] == (B, Hkv) and n_sel.shape == (B, Hkv)
    out = np.zeros((B, Hq, d), dtype=np.float64)
    c = _cfg(B, Hq, Hkv, d, n_sink, 0, scale, K=K, V=V)
    q = np.ascontiguousarray(q)
    rc = lib().sfio_sparse(C.byref(c), _p(q), _p(K), _p(V), _p(sel_idx), _p(n_sel),
                           C.c_int64(sel_idx.shape[2]), _p(recent_start), _p(ctx_len), _p(out))
    if rc != 0:
        raise ValueError("sel_idx entry outside [0, ctx_len)")
    return out


def reorg(K, V, sel_idx, n_sel, ctx_len, n_sink: int, Kc: np.ndarray, Vc: np.ndarray) -> None:
    """Reorg: fills rows [0, min(n_sink, L)) and [n_sink, n_sink + n_sel) of the uint16 compact buffers
    Kc, Vc [B, Hkv, c_rows, d] in place; every other row keeps its contents."""
    B, Hkv = K.shape[0], K.shape[1]
    d = K.shape[3]
    sel_idx, n_sel, ctx_len = _i32(sel_idx), _i32(n_sel), _i32(ctx_len)
    assert Kc.dtype == np.uint16 and Vc.dtype == np.uint16 and Kc.flags.c_contiguous and Vc.flags.c_contiguous
    assert Kc.shape == Vc.shape and Kc.shape[:2] == (B, Hkv) and Kc.shape[3] == d
    c = _cfg(B, Hkv, Hkv, d, n_sink, 0, None, K=K, V=V)
    rc = lib().sfio_reorg(C.byref(c), _p(K), _p(V), _p(sel_idx), _p(n_sel), C.c_int64(sel_idx.shape[2]), _p(ctx_len),
                          _p(Kc), _p(Vc), C.c_int64(Kc.shape[2]))
    if rc != 0:
        raise ValueError("selected index outside [0, ctx_len) or compact buffer too small")


def trigger_schedule(tokens, trigger_ids, t_max: int) -> np.ndarray:
    """g_t of one request: uint8 [len(tokens)]; tokens[t] is the token generated at step t."""
    x = _i32(tokens)
    trig = _i32(sorted(set(int(i) for i in trigger_ids)))
    g = np.zeros(x.shape[0], dtype=np.uint8)
    lib().sfio_trigger_schedule(_p(x), C.c_int32(x.shape[0]), _p(trig), C.c_int32(trig.shape[0]), C.c_int32(t_max), _p(g))
    return g


def selector_from_logits(lg: np.ndarray, ctx_len, Hkv: int, budget: int, n_sink: int, recent: int,
                         sp: Optional[SelectorParams] = None, knorm: Optional[np.ndarray] = None,
                         debug: bool = False, vis=None):
    """Algorithm 2 on given logits float64 [B, Hq, ld].  Returns (sel_idx, n_sel, z[, dbg dict]).
    vis: optional int32 [B, Hq]: vector (b, g) sees rows [0, vis[b, g]) only (causal mask of a window query)."""
    sp = sp or SelectorParams()
    lg = np.ascontiguousarray(lg, dtype=np.float64)
    B, Hq, ld = lg.shape
    ctx_len = _i32(ctx_len)
    assert int(ctx_len.max()) <= ld
    if sp.mode != 0:
        assert knorm is not None and knorm.shape == (B, Hkv, ld)
        knorm = np.ascontiguousarray(knorm, dtype=np.float64)
    sel = np.full((B, Hkv, max(budget, 1)), -1, dtype=np.int32)
    nsel = np.zeros((B, Hkv), dtype=np.int32)
    z = np.zeros((B, Hkv, ld), dtype=np.float64)
    dbg = {}
    if debug:
        for k in ("f", "r", "s", "zbase", "znms"):
            dbg[k] = np.zeros((B, Hkv, ld), dtype=np.float64)
        dbg["lambda"] = np.zeros((B, Hkv), dtype=np.float64)
    c = _cfg(B, Hq, Hkv, 1, n_sink, recent, 1.0, sp=sp)
    sel_c = np.ascontiguousarray(sel[:, :, :budget]) if budget > 0 else sel
    vis = None if vis is None else _i32(vis).reshape(B, Hq)
    rc = lib().sfio_selector_from_logits(
        C.byref(c), _p(lg), _p(knorm), C.c_int64(ld), _p(vis), _p(ctx_len), C.c_int32(budget), _p(sel_c), _p(nsel),
        _p(z), C.c_int64(ld), _p(dbg.get("f")), _p(dbg.get("r")), _p(dbg.get("s")), _p(dbg.get("zbase")),
        _p(dbg.get("znms")), _p(dbg.get("lambda")))
    assert rc == 0
    if budget > 0:
        sel = sel_c
    return (sel, nsel, z, dbg) if debug else (sel, nsel, z)


def selector(q, K, ctx_len, budget: int, n_sink: int, recent: int, scale=None,
             sp: Optional[SelectorParams] = None, vis=None) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Slow-step Selector from q and K: (sel_idx int32 [B,Hkv,budget], n_sel int32 [B,Hkv], z float64 [B,Hkv,ld]).
    vis: optional int32 [B, Hq]: vector (b, g) sees rows [0, vis[b, g]) only (causal mask of a window query)."""
    sp = sp or SelectorParams()
    B, Hq, d = q.shape
    Hkv = K.shape[1]
    ctx_len = _i32(ctx_len)
    ld = int(max(1, ctx_len.max()))
    sel = np.full((B, Hkv, max(budget, 1)), -1, dtype=np.int32)
    nsel = np.zeros((B, Hkv), dtype=np.int32)
    z = np.zeros((B, Hkv, ld), dtype=np.float64)
    c = _cfg(B, Hq, Hkv, d, n_sink, recent, scale, K=K, sp=sp)
    q = np.ascontiguousarray(q)
    sel_c = np.ascontiguousarray(sel[:, :, :budget]) if budget > 0 else sel
    vis = None if vis is None else _i32(vis).reshape(B, Hq)
    rc = lib().sfio_selector(C.byref(c), _p(q), _p(K), _p(vis), _p(ctx_len), C.c_int32(budget), _p(sel_c), _p(nsel),
                             _p(z), C.c_int64(ld))
    assert rc == 0
    if budget > 0:
        sel = sel_c
    return sel, nsel, z


def advance(ctx_len, recent_start, n_sink: int, recent: int) -> Tuple[np.ndarray, np.ndarray]:
    """State update between two decode steps: returns the new (ctx_len, recent_start), int32 [B]."""
    ctx_len, recent_start = _i32(ctx_len).copy(), _i32(recent_start).copy()
    c = _cfg(ctx_len.shape[0], 1, 1, 1, n_sink, recent, 1.0)
    rc = lib().sfio_advance(C.byref(c), _p(ctx_len), _p(recent_start))
    assert rc == 0
    return ctx_len, recent_start


def decode_loop(q_steps: np.ndarray, K, V, ctx_len, recent_start, g, budget: int, n_sink: int, recent: int,
                sel_idx=None, n_sel=None, scale=None, sp: Optional[SelectorParams] = None) -> dict:
    """Algorithm 1 with a scripted slow/fast indicator g uint8 [n_steps, B] over q_steps uint16 [n_steps, B, Hq, d].
    ctx_len / recent_start: the state before step 0.  sel_idx / n_sel: I_sel before step 0 (default: empty).
    Returns a dict: out float64 [n_steps, B, Hq, d]; sel_hist, nsel_hist (I_sel after each step); ctx_hist, rs_hist
    (the state each step ran on); ctx_len, recent_start, sel_idx, n_sel (the state after the last step)."""
    sp = sp or SelectorParams()
    q_steps = np.ascontiguousarray(q_steps)
    T, B, Hq, d = q_steps.shape
    Hkv = K.shape[1]
    g = np.ascontiguousarray(g, dtype=np.uint8).reshape(T, B)
    ctx_len, recent_start = _i32(ctx_len).copy(), _i32(recent_start).copy()
    bw = max(budget, 1)
    sel = np.full((B, Hkv, bw), -1, np.int32) if sel_idx is None else np.ascontiguousarray(sel_idx, np.int32).copy()
    nsel = np.zeros((B, Hkv), np.int32) if n_sel is None else _i32(n_sel).copy()
    assert sel.shape == (B, Hkv, bw) and budget > 0
    out = np.zeros((T, B, Hq, d), np.float64)
    sel_hist = np.zeros((T, B, Hkv, bw), np.int32)
    nsel_hist = np.zeros((T, B, Hkv), np.int32)
    ctx_hist, rs_hist = np.zeros((T, B), np.int32), np.zeros((T, B), np.int32)
    c = _cfg(B, Hq, Hkv, d, n_sink, recent, scale, K=K, V=V, sp=sp)
    rc = lib().sfio_decode_loop(C.byref(c), _p(q_steps), _p(K), _p(V), C.c_int32(T), _p(g), C.c_int32(budget),
                                _p(ctx_len), _p(recent_start), _p(sel), _p(nsel), _p(out), _p(sel_hist), _p(nsel_hist),
                                _p(ctx_hist), _p(rs_hist))
    if rc != 0:
        raise ValueError("decode loop: a selected index left the context")
    return dict(out=out, sel_hist=sel_hist, nsel_hist=nsel_hist, ctx_hist=ctx_hist, rs_hist=rs_hist, ctx_len=ctx_len,
                recent_start=recent_start, sel_idx=sel, n_sel=nsel)
