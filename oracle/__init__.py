"""ctypes front-end of the fp64 reference oracle (TEST INFRASTRUCTURE ONLY).

Only the test-suite, the smoke check and the benchmark's reported CPU baseline
may import this package; the GPU library and its Python binding never do.
Arrays are numpy: bf16 tensors travel as ``uint16`` bit patterns, fp32 as
``float32``, fp64 as ``float64``.  All arithmetic lives in ``milora_oracle.c``;
this file only marshals arguments.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "milora_oracle.c")
_LIB = os.path.join(_HERE, "_build", "libmilora_oracle.so")

BF16, F32, F64 = 0, 1, 2
POOL_MEAN, POOL_LAST, POOL_MAX, POOL_SELFATTN = 0, 1, 2, 3
ACT_IDENTITY, ACT_TANH, ACT_RELU, ACT_GELU, ACT_RATIONAL = 0, 1, 2, 3, 4
FLAG_RMSNORM = 1
NMOD = 7
SITES = ("q", "k", "v", "o", "gate", "up", "down")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math: sums keep their written order)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        os.makedirs(os.path.dirname(_LIB), exist_ok=True)
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def n_threads() -> int:
    """Threads the OpenMP loops of the oracle will use."""
    omp = ctypes.CDLL("libgomp.so.1")
    return int(omp.omp_get_max_threads())


def dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.float64:
        return F64
    raise TypeError(f"unsupported storage dtype {a.dtype}")


def _p(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _u8(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.uint8))


def site_dims(site: int, d: int, F: int):
    d1, d2 = ctypes.c_int(), ctypes.c_int()
    lib().orc_site_dims(site, d, F, ctypes.byref(d1), ctypes.byref(d2))
    return d1.value, d2.value


def param_counts(d: int, F: int, L: int, r: int):
    out = (ctypes.c_int64 * 3)()
    lib().orc_param_counts(d, F, L, r, out)
    return int(out[0]), int(out[1]), int(out[2])


@dataclass
class Adapters:
    """Per-tenant LoRA stacks of one layer: A[t][site] is [d1, r_t], B[t][site] is [r_t, d2]."""

    A: Sequence[Sequence[np.ndarray]]
    B: Sequence[Sequence[np.ndarray]]
    rank: Sequence[int]

    def tables(self):
        T = len(self.rank)
        A_tab = (ctypes.c_void_p * (T * NMOD))()
        B_tab = (ctypes.c_void_p * (T * NMOD))()
        dt = None
        for t in range(T):
            for m in range(NMOD):
                a, b = self.A[t][m], self.B[t][m]
                assert a.flags["C_CONTIGUOUS"] and b.flags["C_CONTIGUOUS"]
                assert a.shape[1] == self.rank[t] and b.shape[0] == self.rank[t]
                dt = dtype_code(a) if dt is None else dt
                assert dtype_code(a) == dt and dtype_code(b) == dt
                A_tab[t * NMOD + m] = a.ctypes.data
                B_tab[t * NMOD + m] = b.ctypes.data
        return A_tab, B_tab, _i32(self.rank), T, dt


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def pool(H, seq_start, seq_len, pool_kind, w_sa=None, tenant_id=None):
    H = np.ascontiguousarray(H)
    M_tok, d = H.shape
    ss, sl = _i32(seq_start), _i32(seq_len)
    B = len(ss)
    h = np.empty((B, d), dtype=np.float64)
    tid = _i32(tenant_id) if tenant_id is not None else None
    T = 0 if w_sa is None else w_sa.shape[0]
    rc = lib().orc_pool(_p(H), dtype_code(H), ctypes.c_int64(M_tok), d, _p(ss), _p(sl), B, pool_kind,
                        _p(w_sa), _p(tid), T, _p(h))
    _check(rc, "pool")
    return h


def activation(z, act_kind, coef=None):
    z = np.array(z, dtype=np.float64, copy=True, order="C")
    c = None if coef is None else np.ascontiguousarray(np.asarray(coef, dtype=np.float64))
    assert c is None or c.size == 12
    _check(lib().orc_activation(_p(z), ctypes.c_int64(z.size), act_kind, _p(c)), "activation")
    return z


def router_logits(z, Wr, tenant_id):
    z = np.ascontiguousarray(np.asarray(z, dtype=np.float64))
    B, d = z.shape
    Wr = np.ascontiguousarray(Wr)
    T = Wr.shape[0]
    assert Wr.shape == (T, NMOD, d)
    tid = _i32(tenant_id)
    out = np.empty((B, NMOD), dtype=np.float64)
    _check(lib().orc_router_logits(_p(z), B, d, _p(Wr), dtype_code(Wr), _p(tid), T, _p(out)), "router_logits")
    return out


def softmax7(logit):
    l = np.ascontiguousarray(np.asarray(logit, dtype=np.float64))
    assert l.shape == (NMOD,)
    out = np.empty(NMOD, dtype=np.float64)
    lib().orc_softmax7(_p(l), _p(out))
    return out


def select(logits):
    l = np.ascontiguousarray(np.asarray(logits, dtype=np.float64))
    B = l.shape[0]
    route = np.empty(B, dtype=np.uint8)
    gap = np.empty(B, dtype=np.float64)
    lib().orc_select(_p(l), B, _p(route), _p(gap))
    return route, gap


def select_topk(logits, k):
    """Route bytes and the k-th/(k+1)-th logit gaps for top-k selection (k = 1: site index; k > 1: 0x80 | mask)."""
    l = np.ascontiguousarray(np.asarray(logits, dtype=np.float64))
    B = l.shape[0]
    route = np.empty(B, dtype=np.uint8)
    gap = np.empty(B, dtype=np.float64)
    _check(lib().orc_select_topk(_p(l), B, int(k), _p(route), _p(gap)), "select_topk")
    return route, gap


def route_has(route_byte: int, site: int) -> bool:
    return bool(lib().orc_route_has(ctypes.c_uint8(int(route_byte)), int(site)))


@dataclass
class RouteResult:
    route: np.ndarray  # uint8 [B]
    logits: np.ndarray  # float64 [B, 7]
    gap: np.ndarray  # float64 [B], top-1 minus top-2 logit
    h: np.ndarray  # float64 [B, d], pooled state before the activation


def route(H, seq_start, seq_len, tenant_id, Wr, pool_kind=POOL_MEAN, act_kind=ACT_IDENTITY, w_sa=None,
          act_coef=None, top_k=1) -> RouteResult:
    H = np.ascontiguousarray(H)
    Wr = np.ascontiguousarray(Wr)
    M_tok, d = H.shape
    T = Wr.shape[0]
    assert Wr.shape == (T, NMOD, d) and dtype_code(Wr) == dtype_code(H)
    ss, sl, tid = _i32(seq_start), _i32(seq_len), _i32(tenant_id)
    B = len(ss)
    r = np.empty(B, dtype=np.uint8)
    logits = np.empty((B, NMOD), dtype=np.float64)
    gap = np.empty(B, dtype=np.float64)
    h = np.empty((B, d), dtype=np.float64)
    c = None if act_coef is None else np.ascontiguousarray(np.asarray(act_coef, dtype=np.float64))
    if w_sa is not None:
        w_sa = np.ascontiguousarray(w_sa)
        assert w_sa.shape == (T, d) and dtype_code(w_sa) == dtype_code(H)
    rc = lib().orc_route(_p(H), dtype_code(H), ctypes.c_int64(M_tok), d, _p(ss), _p(sl), _p(tid), B, T, _p(Wr),
                         pool_kind, act_kind, _p(w_sa), _p(c), _p(r), _p(logits), _p(gap), _p(h))
    _check(rc, "route")
    if top_k != 1:
        r, gap = select_topk(logits, top_k)
    return RouteResult(r, logits, gap, h)


def routed_linear(X, W, adapters: Adapters, site, tenant_id, route, row_to_req=None, bias=None, rows=None):
    """y = x W + bias + [route == site] (x A) B for every row, or only for ``rows``."""
    X, W = np.ascontiguousarray(X), np.ascontiguousarray(W)
    M, d1 = X.shape
    d2 = W.shape[0]
    assert W.shape == (d2, d1)
    A_tab, B_tab, rank, T, adt = adapters.tables()
    assert adt == dtype_code(W)
    tid, rt = _i32(tenant_id), _u8(route)
    B = len(tid)
    r2r = _i32(row_to_req) if row_to_req is not None else None
    rws = np.ascontiguousarray(np.asarray(rows, dtype=np.int64)) if rows is not None else None
    n = M if rws is None else len(rws)
    Y = np.empty((n, d2), dtype=np.float64)
    if bias is not None:
        bias = np.ascontiguousarray(bias)
        assert dtype_code(bias) == dtype_code(W)
    rc = lib().orc_routed_linear(_p(X), dtype_code(X), ctypes.c_int64(M), d1, d2, _p(r2r), _p(W), _p(bias),
                                 dtype_code(W), A_tab, B_tab, _p(rank), T, site, _p(tid), _p(rt), B, _p(rws),
                                 ctypes.c_int64(n), _p(Y))
    _check(rc, "routed_linear")
    return Y


def routed_linear_dense(X, W, adapters: Adapters, site, tenant_id, gate, row_to_req=None, bias=None):
    """Dense mixture form: the LoRA branch of every request, scaled by gate[b, site]."""
    X, W = np.ascontiguousarray(X), np.ascontiguousarray(W)
    M, d1 = X.shape
    d2 = W.shape[0]
    A_tab, B_tab, rank, T, adt = adapters.tables()
    assert adt == dtype_code(W)
    tid = _i32(tenant_id)
    B = len(tid)
    gate = np.ascontiguousarray(np.asarray(gate, dtype=np.float64))
    assert gate.shape == (B, NMOD)
    r2r = _i32(row_to_req) if row_to_req is not None else None
    Y = np.empty((M, d2), dtype=np.float64)
    if bias is not None:
        bias = np.ascontiguousarray(bias)
    rc = lib().orc_routed_linear_dense(_p(X), dtype_code(X), ctypes.c_int64(M), d1, d2, _p(r2r), _p(W), _p(bias),
                                       dtype_code(W), A_tab, B_tab, _p(rank), T, site, _p(tid), _p(gate), B,
                                       _p(Y))
    _check(rc, "routed_linear_dense")
    return Y


def layer_decode(x, W7, adapters: Adapters, tenant_id, route, F, flags=0, attn_out=None):
    """One decode step through the seven routed linears; returns (y [B,d], qkv [B,3d]) in fp64."""
    x = np.ascontiguousarray(x)
    B, d = x.shape
    W7 = [np.ascontiguousarray(w) for w in W7]
    assert len(W7) == NMOD
    wdt = dtype_code(W7[0])
    Wp = (ctypes.c_void_p * NMOD)()
    for m, w in enumerate(W7):
        d1, d2 = site_dims(m, d, F)
        assert w.shape == (d2, d1) and dtype_code(w) == wdt
        Wp[m] = w.ctypes.data
    A_tab, B_tab, rank, T, adt = adapters.tables()
    assert adt == wdt
    tid, rt = _i32(tenant_id), _u8(route)
    assert len(tid) == B and len(rt) == B
    y = np.empty((B, d), dtype=np.float64)
    qkv = np.empty((B, 3 * d), dtype=np.float64)
    if attn_out is not None:
        attn_out = np.ascontiguousarray(attn_out)
        assert attn_out.shape == (B, d) and dtype_code(attn_out) == dtype_code(x)
    rc = lib().orc_layer_decode(_p(x), dtype_code(x), B, d, F, Wp, wdt, A_tab, B_tab, _p(rank), T, _p(tid),
                                _p(rt), flags, _p(attn_out), _p(y), _p(qkv))
    _check(rc, "layer_decode")
    return y, qkv
