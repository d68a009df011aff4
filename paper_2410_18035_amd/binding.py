"""Python face of the C-ABI library: same entry points, torch tensors in, argument marshalling only.

Every step of the path runs in the HIP library; this module converts tensors to
raw device pointers, sizes workspaces and raises on a non-zero status.  There is
no CPU fallback: if ``libmilora.so`` has not been built, or no GPU is present
when a compute call is made, the call raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "_lib", "libmilora.so")

NUM_SITES = 7
BF16, F32 = 0, 1
POOL = {"mean": 0, "last": 1, "max": 2, "selfattn": 3}
ACT = {"identity": 0, "tanh": 1, "relu": 2, "gelu": 3, "rational": 4}
W_ROWMAJOR, W_PACKED = 0, 1
LAYER_RMSNORM = 1
ROUTE_NONE = 255
ROUTE_SET = 0x80
MAX_RANK = 256
MAX_DECODE_BATCH = 128

EXPORTS = (
    "milora_version", "milora_status_string", "milora_last_hip_error",
    "milora_route_workspace_bytes", "milora_route",
    "milora_routed_linear_workspace_bytes", "milora_routed_linear_kernel", "milora_routed_linear",
    "milora_layer_decode_workspace_bytes", "milora_layer_decode", "milora_layer_decode_noalloc",
    "milora_layer_decode_profile", "milora_layer_decode_trace_bytes", "milora_layer_decode_trace",
    "milora_pack_weight", "milora_packed_workspace_status", "milora_set_wait_limit",
    "milora_measure_workspace_bytes", "milora_measure_matrix_rate", "milora_measure_read_rate",
)


class MiloraError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: status {status} ({status_string(status)}), hip error {last_hip_error()}")


class _Adapters(ctypes.Structure):
    _fields_ = [("n_tenants", ctypes.c_int32), ("r_max", ctypes.c_int32), ("rank", ctypes.c_void_p),
                ("A", ctypes.c_void_p), ("B", ctypes.c_void_p)]


class _LayerWeights(ctypes.Structure):
    _fields_ = [("W", ctypes.c_void_p * NUM_SITES), ("layout", ctypes.c_int32)]


_lib = None


def lib() -> ctypes.CDLL:
    """Load the HIP library (built in-tree by ``paper_2410_18035_amd.build``); raise if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -m paper_2410_18035_amd.build` (there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
        L.milora_version.restype = ctypes.c_char_p
        L.milora_status_string.restype = ctypes.c_char_p
        L.milora_status_string.argtypes = [i32]
        L.milora_last_hip_error.restype = i32
        L.milora_route_workspace_bytes.restype = sz
        L.milora_route_workspace_bytes.argtypes = [i32, i32, i64]
        L.milora_route.restype = i32
        L.milora_route.argtypes = [vp, i64, i32, i32, vp, vp, vp, i32, i32, vp, i32, i32, vp, ctypes.POINTER(ctypes.c_float),
                                   i32, vp, vp, vp, sz, vp]
        L.milora_routed_linear_workspace_bytes.restype = sz
        L.milora_routed_linear_workspace_bytes.argtypes = [i64, i32, i32, i32]
        L.milora_routed_linear_kernel.restype = i32
        L.milora_routed_linear_kernel.argtypes = [i64, i32, i32, i32, i32]
        L.milora_routed_linear.restype = i32
        L.milora_routed_linear.argtypes = [vp, i64, i32, i32, i32, vp, vp, i32, vp, ctypes.POINTER(_Adapters), i32,
                                           vp, vp, i32, vp, vp, sz, vp]
        L.milora_layer_decode_workspace_bytes.restype = sz
        L.milora_layer_decode_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.milora_layer_decode.restype = i32
        L.milora_layer_decode.argtypes = [vp, i32, i32, i32, i32, ctypes.POINTER(_LayerWeights),
                                          ctypes.POINTER(_Adapters), vp, vp, ctypes.c_uint32, vp, vp, vp, vp, sz, vp]
        L.milora_layer_decode_noalloc.restype = i32
        L.milora_layer_decode_noalloc.argtypes = L.milora_layer_decode.argtypes[:13] + [vp]
        L.milora_layer_decode_profile.restype = i32
        L.milora_layer_decode_profile.argtypes = L.milora_layer_decode.argtypes + [i32, ctypes.POINTER(ctypes.c_float)]
        L.milora_layer_decode_trace_bytes.restype = sz
        L.milora_layer_decode_trace_bytes.argtypes = []
        L.milora_layer_decode_trace.restype = i32
        L.milora_layer_decode_trace.argtypes = L.milora_layer_decode.argtypes + [vp, sz, ctypes.POINTER(ctypes.c_int32)]
        L.milora_pack_weight.restype = i32
        L.milora_pack_weight.argtypes = [vp, vp, i32, i32, vp]
        L.milora_packed_workspace_status.restype = i32
        L.milora_packed_workspace_status.argtypes = [vp, ctypes.POINTER(ctypes.c_int), vp]
        L.milora_set_wait_limit.restype = i32
        L.milora_set_wait_limit.argtypes = [i32]
        L.milora_measure_workspace_bytes.restype = sz
        L.milora_measure_workspace_bytes.argtypes = []
        L.milora_measure_matrix_rate.restype = i32
        L.milora_measure_matrix_rate.argtypes = [i32, i32, vp, sz, ctypes.POINTER(ctypes.c_double), vp]
        L.milora_measure_read_rate.restype = i32
        L.milora_measure_read_rate.argtypes = [vp, sz, i32, vp, sz, ctypes.POINTER(ctypes.c_double), vp]
        _lib = L
    return _lib


def version() -> str:
    return lib().milora_version().decode()


def status_string(status: int) -> str:
    return lib().milora_status_string(status).decode()


def last_hip_error() -> int:
    return int(lib().milora_last_hip_error())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dev(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("the library works on device memory only: pass CUDA/HIP tensors")
    if not t.is_contiguous():
        raise ValueError("tensors must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.zeros(max(int(nbytes), 256), dtype=torch.uint8, device=device)


@dataclass
class AdapterTable:
    """Device-side pointer tables of one layer's per-tenant LoRA stacks (keeps the matrices alive)."""

    rank: torch.Tensor  # int32 [T] device
    A_ptrs: torch.Tensor  # int64 [T*7] device
    B_ptrs: torch.Tensor  # int64 [T*7] device
    r_max: int
    n_tenants: int
    keep: tuple

    @staticmethod
    def from_tensors(A: Sequence[Sequence[torch.Tensor]], B: Sequence[Sequence[torch.Tensor]],
                     rank: Sequence[int], r_max: Optional[int] = None) -> "AdapterTable":
        T = len(rank)
        dev = A[0][0].device
        a_ptrs, b_ptrs = [], []
        for t in range(T):
            for m in range(NUM_SITES):
                a, b = A[t][m], B[t][m]
                if not (a.is_cuda and b.is_cuda and a.is_contiguous() and b.is_contiguous()):
                    raise ValueError("adapter matrices must be contiguous device tensors")
                if a.shape[1] != rank[t] or b.shape[0] != rank[t]:
                    raise ValueError("A must be [d1, r_t] and B must be [r_t, d2]")
                a_ptrs.append(a.data_ptr())
                b_ptrs.append(b.data_ptr())
        return AdapterTable(torch.tensor(list(rank), dtype=torch.int32, device=dev),
                            torch.tensor(a_ptrs, dtype=torch.int64, device=dev),
                            torch.tensor(b_ptrs, dtype=torch.int64, device=dev),
                            int(r_max if r_max is not None else max(rank)), T, (A, B))

    def c_struct(self) -> _Adapters:
        return _Adapters(self.n_tenants, self.r_max, self.rank.data_ptr(), self.A_ptrs.data_ptr(),
                         self.B_ptrs.data_ptr())


def route_workspace_bytes(B: int, d: int, M_tok: int) -> int:
    return int(lib().milora_route_workspace_bytes(B, d, M_tok))


def milora_route(H: torch.Tensor, seq_start: torch.Tensor, seq_len: torch.Tensor, tenant_id: torch.Tensor,
                 Wr: torch.Tensor, pool: str = "mean", act: str = "identity",
                 route_out: Optional[torch.Tensor] = None, want_logits: bool = True,
                 workspace: Optional[torch.Tensor] = None, w_sa: Optional[torch.Tensor] = None,
                 act_coef: Optional[Sequence[float]] = None, top_k: int = 1):
    """Prompt-aware router of one layer; returns (route uint8 [B], logits float32 [B,7] or None).

    pool "selfattn" needs w_sa [T, d]; act "rational" needs the 12 coefficients a_0..a_6, b_1..b_5."""
    M_tok, d = H.shape
    B = tenant_id.numel()
    T = Wr.shape[0]
    if Wr.shape != (T, NUM_SITES, d) or Wr.dtype != H.dtype:
        raise ValueError("Wr must be [T, 7, d] in the dtype of H")
    if route_out is None:
        route_out = torch.empty(B, dtype=torch.uint8, device=H.device)
    logits = torch.empty(B, NUM_SITES, dtype=torch.float32, device=H.device) if want_logits else None
    if workspace is None:
        workspace = _workspace(route_workspace_bytes(B, d, M_tok), H.device)
    if w_sa is not None and (w_sa.shape != (T, d) or w_sa.dtype != H.dtype):
        raise ValueError("w_sa must be [T, d] in the dtype of H")
    coef = None
    if act_coef is not None:
        if len(act_coef) != 12:
            raise ValueError("act_coef holds a_0..a_6 and b_1..b_5")
        coef = (ctypes.c_float * 12)(*[float(c) for c in act_coef])
    rc = lib().milora_route(_dev(H), M_tok, d, _dtype_code(H), _dev(seq_start, torch.int32),
                            _dev(seq_len, torch.int32), _dev(tenant_id, torch.int32), B, T, _dev(Wr), POOL[pool],
                            ACT[act], _dev(w_sa), coef, top_k, _dev(route_out, torch.uint8), _dev(logits), _dev(workspace),
                            workspace.numel(), _stream())
    if rc != 0:
        raise MiloraError(rc, "milora_route")
    return route_out, logits


def routed_linear_workspace_bytes(M: int, d1: int, d2: int, r_max: int) -> int:
    return int(lib().milora_routed_linear_workspace_bytes(M, d1, d2, r_max))


KERNEL_GENERIC, KERNEL_STREAM, KERNEL_TILES = 0, 1, 2


def milora_routed_linear_kernel(M: int, d1: int, d2: int, dtype: torch.dtype, w_layout: int = W_ROWMAJOR) -> int:
    code = {torch.bfloat16: 0, torch.float32: 1}[dtype] if not isinstance(dtype, int) else dtype
    return int(lib().milora_routed_linear_kernel(M, d1, d2, code, w_layout))


def milora_routed_linear(X: torch.Tensor, W: torch.Tensor, adapters: AdapterTable, site: int,
                         tenant_id: torch.Tensor, route: torch.Tensor, row_to_req: Optional[torch.Tensor] = None,
                         bias: Optional[torch.Tensor] = None, w_layout: int = W_ROWMAJOR,
                         d2: Optional[int] = None, out: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Y = X W + bias + [route == site] (X A) B.  W is [d2, d1] row-major, or packed (then pass d2)."""
    M, d1 = X.shape
    if w_layout == W_ROWMAJOR:
        d2 = W.shape[0]
        if W.shape != (d2, d1):
            raise ValueError("W must be [d2, d1]")
    elif d2 is None or W.numel() != d1 * d2:
        raise ValueError("a packed W needs d2 and d1*d2 elements")
    if W.dtype != X.dtype:
        raise TypeError("W and X must share a dtype")
    B = tenant_id.numel()
    if out is None:
        out = torch.empty(M, d2, dtype=X.dtype, device=X.device)
    if workspace is None:
        workspace = _workspace(routed_linear_workspace_bytes(M, d1, d2, adapters.r_max), X.device)
    ad = adapters.c_struct()
    rc = lib().milora_routed_linear(_dev(X), M, d1, d2, _dtype_code(X), _dev(row_to_req, torch.int32), _dev(W),
                                    w_layout, _dev(bias, X.dtype), ctypes.byref(ad), site,
                                    _dev(tenant_id, torch.int32), _dev(route, torch.uint8), B, _dev(out),
                                    _dev(workspace), workspace.numel(), _stream())
    if rc != 0:
        raise MiloraError(rc, "milora_routed_linear")
    return out


def layer_decode_workspace_bytes(B: int, d: int, F: int, r_max: int) -> int:
    return int(lib().milora_layer_decode_workspace_bytes(B, d, F, r_max))


PROFILE_SLOTS = 8


def milora_layer_decode(x: torch.Tensor, weights: Sequence[torch.Tensor], adapters: AdapterTable,
                        tenant_id: torch.Tensor, route: torch.Tensor, F: int, w_layout: int = W_ROWMAJOR,
                        rmsnorm: bool = False, attn_out: Optional[torch.Tensor] = None,
                        y: Optional[torch.Tensor] = None, qkv_out: Optional[torch.Tensor] = None,
                        want_qkv: bool = True, workspace: Optional[torch.Tensor] = None, profile_reps: int = 0):
    """One decode step through the seven routed linears of a layer; returns (y [B,d], qkv [B,3d] or None).

    With profile_reps > 0 the call goes to milora_layer_decode_profile and returns (y, qkv, slot_ms)."""
    B, d = x.shape
    if len(weights) != NUM_SITES:
        raise ValueError("seven base weights expected")
    lw = _LayerWeights()
    for m, w in enumerate(weights):
        if w.dtype != x.dtype:
            raise TypeError("weights and x must share a dtype")
        lw.W[m] = _dev(w)
    lw.layout = w_layout
    if y is None:
        y = torch.empty_like(x)
    if qkv_out is None and want_qkv:
        qkv_out = torch.empty(B, 3 * d, dtype=x.dtype, device=x.device)
    if workspace is None:
        workspace = _workspace(layer_decode_workspace_bytes(B, d, F, adapters.r_max), x.device)
    ad = adapters.c_struct()
    args = (_dev(x), B, d, F, _dtype_code(x), ctypes.byref(lw), ctypes.byref(ad), _dev(tenant_id, torch.int32),
            _dev(route, torch.uint8), LAYER_RMSNORM if rmsnorm else 0, _dev(attn_out, x.dtype), _dev(y),
            _dev(qkv_out), _dev(workspace), workspace.numel(), _stream())
    if profile_reps > 0:
        slots = (ctypes.c_float * PROFILE_SLOTS)()
        rc = lib().milora_layer_decode_profile(*args, profile_reps, slots)
        if rc != 0:
            raise MiloraError(rc, "milora_layer_decode_profile")
        return y, qkv_out, [float(v) for v in slots]
    rc = lib().milora_layer_decode(*args)
    if rc != 0:
        raise MiloraError(rc, "milora_layer_decode")
    return y, qkv_out


def milora_layer_decode_trace(x: torch.Tensor, weights: Sequence[torch.Tensor], adapters: AdapterTable,
                              tenant_id: torch.Tensor, route: torch.Tensor, F: int, y: torch.Tensor,
                              qkv_out: Optional[torch.Tensor], workspace: torch.Tensor, rmsnorm: bool = False,
                              attn_out: Optional[torch.Tensor] = None):
    """One traced decode step on packed weights; returns (stamps int64 [G, stages, waves, slots] on the host in
    units of 10 ns, 0 = not written)."""
    B, d = x.shape
    lw = _LayerWeights()
    for m, w in enumerate(weights):
        lw.W[m] = _dev(w, x.dtype)
    lw.layout = W_PACKED
    ad = adapters.c_struct()
    nbytes = int(lib().milora_layer_decode_trace_bytes())
    stamps = torch.empty(nbytes // 8, dtype=torch.int64, device=x.device)
    dims = (ctypes.c_int32 * 5)()
    rc = lib().milora_layer_decode_trace(_dev(x), B, d, F, _dtype_code(x), ctypes.byref(lw), ctypes.byref(ad),
                                         _dev(tenant_id, torch.int32), _dev(route, torch.uint8),
                                         LAYER_RMSNORM if rmsnorm else 0, _dev(attn_out, x.dtype), _dev(y), _dev(qkv_out),
                                         _dev(workspace), workspace.numel(), _stream(), _dev(stamps), nbytes, dims)
    if rc != 0:
        raise MiloraError(rc, "milora_layer_decode_trace")
    G, stages, smax, waves, slots = (int(v) for v in dims)
    return stamps.cpu().view(-1, smax, waves, slots)[:G, :stages]


def milora_layer_decode_noalloc(x: torch.Tensor, weights: Sequence[torch.Tensor], adapters: AdapterTable,
                                tenant_id: torch.Tensor, route: torch.Tensor, F: int, y: torch.Tensor,
                                qkv_out: Optional[torch.Tensor] = None, rmsnorm: bool = False,
                                attn_out: Optional[torch.Tensor] = None) -> None:
    """milora_layer_decode on the library's own scratch array (packed bf16 weights, B <= 32): the caller passes
    every buffer, nothing is allocated here or in the library."""
    B, d = x.shape
    lw = _LayerWeights()
    for m, w in enumerate(weights):
        lw.W[m] = _dev(w, x.dtype)
    lw.layout = W_PACKED
    ad = adapters.c_struct()
    rc = lib().milora_layer_decode_noalloc(_dev(x), B, d, F, _dtype_code(x), ctypes.byref(lw), ctypes.byref(ad),
                                           _dev(tenant_id, torch.int32), _dev(route, torch.uint8),
                                           LAYER_RMSNORM if rmsnorm else 0, _dev(attn_out, x.dtype), _dev(y),
                                           _dev(qkv_out), _stream())
    if rc != 0:
        raise MiloraError(rc, "milora_layer_decode_noalloc")


def milora_pack_weight(W: torch.Tensor) -> torch.Tensor:
    """One-time re-ordering of a row-major bf16 [d2, d1] weight into the packed decode layout."""
    d2, d1 = W.shape
    out = torch.empty(d1 * d2, dtype=W.dtype, device=W.device)
    rc = lib().milora_pack_weight(_dev(W, torch.bfloat16), _dev(out), d1, d2, _stream())
    if rc != 0:
        raise MiloraError(rc, "milora_pack_weight")
    return out


MFMA_16X16X32, MFMA_32X32X16 = 0, 1
MFMA_MIXED_OPERANDS = 2  # added to a shape: operands that use every mantissa bit


def milora_measure_matrix_rate(iters: int = 4000, device="cuda:0", shape: int = MFMA_16X16X32) -> float:
    """Sustained bf16 matrix-core rate of the GPU in TFLOP/s (a kernel of nothing but matrix instructions of
    the given shape)."""
    ws = torch.empty(lib().milora_measure_workspace_bytes(), dtype=torch.uint8, device=device)
    out = ctypes.c_double(0.0)
    rc = lib().milora_measure_matrix_rate(shape, iters, _dev(ws), ws.numel(), ctypes.byref(out), _stream())
    if rc:
        raise MiloraError(rc, "milora_measure_matrix_rate")
    return out.value


def milora_measure_read_rate(buf: torch.Tensor, reps: int = 5) -> float:
    """Rate in GB/s at which one pass of 16-byte loads reads `buf` (make it much larger than the caches)."""
    ws = torch.empty(lib().milora_measure_workspace_bytes(), dtype=torch.uint8, device=buf.device)
    out = ctypes.c_double(0.0)
    nbytes = buf.numel() * buf.element_size()
    rc = lib().milora_measure_read_rate(_dev(buf), nbytes, reps, _dev(ws), ws.numel(), ctypes.byref(out), _stream())
    if rc:
        raise MiloraError(rc, "milora_measure_read_rate")
    return out.value


def milora_set_wait_limit(polls: int) -> int:
    """Polls after which a bounded wait inside a packed-weight launch gives up (<= 0: the default); returns the old value."""
    return int(lib().milora_set_wait_limit(int(polls)))


def milora_packed_workspace_status(workspace: Optional[torch.Tensor]) -> int:
    """0 unless a bounded wait inside a packed-weight launch on this workspace ran out (waits for the stream).
    None: the scratch array of milora_layer_decode_noalloc on the current GPU."""
    out = ctypes.c_int(-1)
    rc = lib().milora_packed_workspace_status(_dev(workspace), ctypes.byref(out), _stream())
    if rc:
        raise MiloraError(rc, "milora_packed_workspace_status")
    return out.value
