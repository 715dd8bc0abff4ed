"""ctypes binding of libsste.so: argument marshalling only."""
import ctypes
import os
from typing import Optional, Tuple

import torch

BF16 = 0
F8E4M3 = 1
F32 = 2
F8E5M2 = 3         # e5m2 output gradients against e4m3 operands: backward calls only

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsste.so")
_lib = None

_STATUS = {0: "OK", 1: "ERR_NULL", 2: "ERR_SHAPE", 3: "ERR_ALIGN", 4: "ERR_DTYPE", 5: "ERR_VALUE",
           6: "ERR_WORKSPACE", 7: "ERR_UNSUPPORTED", 8: "ERR_HIP"}


class SsteError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"sste status {status} ({_STATUS.get(status, '?')}): {message}")
        self.status = status


def library() -> ctypes.CDLL:
    """Loads libsste.so (building it first only if it has never been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build
        build.build_library(verbose=False)
    lib = ctypes.CDLL(_LIB_PATH)
    i64, f32, vp, ci, u64, sz = ctypes.c_int64, ctypes.c_float, ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_size_t
    lib.sste_version.restype = ci
    lib.sste_last_error.restype = ctypes.c_char_p
    lib.sste_project_pack.argtypes = [vp, i64, i64, i64, f32, ci, f32, vp, vp, vp, vp]
    lib.sste_project_pack_gamma.argtypes = [vp, i64, i64, i64, f32, f32, ci, f32, vp, vp, vp, vp]
    lib.sste_project_pack_gamma.restype = ci
    lib.sste_compute_beta_ex.argtypes = [vp, i64, i64, i64, ci, f32, vp, vp, sz, vp]
    lib.sste_compute_beta_ex.restype = ci
    lib.sste_sgd_project_pack.argtypes = [vp, ci, i64, i64, i64, vp, i64, f32, f32, ci, f32, vp, vp, vp]
    lib.sste_sgd_project_pack_batch_prepare.argtypes = [vp, ci, ci, ci, vp, ctypes.POINTER(i64)]
    lib.sste_sgd_project_pack_batch.argtypes = [vp, ci, i64, ci, ci, f32, vp]
    lib.sste_project_pack_batch_prepare.argtypes = [vp, ci, ci, vp, ctypes.POINTER(i64)]
    lib.sste_project_pack_batch.argtypes = [vp, ci, i64, ci, vp]
    lib.sste_linear_fwd.argtypes = [vp, i64, i64, i64, ci, f32, vp, vp, i64, f32, vp, i64, vp]
    lib.sste_linear_fwd_ex.argtypes = [vp, i64, i64, i64, ci, f32, vp, vp, i64, f32, vp, i64, ci, f32, vp, vp]
    lib.sste_linear_fwd_ex.restype = ci
    lib.sste_linear_fwd_act.argtypes = [vp, i64, i64, i64, ci, f32, vp, vp, i64, f32, ci, vp, i64, vp, i64, ci, f32, vp, vp]
    lib.sste_linear_fwd_act.restype = ci
    lib.sste_linear_dgrad_act.argtypes = [vp, i64, i64, i64, ci, f32, vp, vp, i64, f32, ci, vp, i64, vp, i64, vp]
    lib.sste_linear_dgrad_act.restype = ci
    lib.sste_amax_history_init.argtypes = [vp, ci]
    lib.sste_amax_history_init.restype = None
    lib.sste_amax_history_push.argtypes = [vp, f32, f32]
    lib.sste_amax_history_push.restype = f32
    lib.sste_linear_dgrad.argtypes = [vp, i64, i64, i64, ci, f32, vp, vp, i64, f32, vp, i64, vp]
    lib.sste_linear_wgrad.argtypes = [vp, i64, i64, i64, ci, f32, vp, i64, i64, f32, u64, u64, vp, i64, ci, vp, sz, vp]
    lib.sste_linear_wgrad_noalloc.argtypes = [vp, i64, i64, i64, ci, f32, vp, i64, i64, f32, u64, u64, vp, i64, ci, vp]
    lib.sste_linear_wgrad_noalloc.restype = ci
    lib.sste_wgrad_plan_override.argtypes = [ci, ci, ci]
    lib.sste_wgrad_plan_override.restype = ci
    lib.sste_wgrad_workspace_bytes.argtypes = [i64, i64, i64, ci]
    lib.sste_wgrad_workspace_bytes.restype = sz
    lib.sste_mvue_materialize.argtypes = [vp, i64, i64, i64, ci, u64, u64, vp, vp, vp]
    lib.sste_mvue_materialize_at.argtypes = [vp, i64, i64, i64, ci, u64, u64, i64, vp, vp, vp]
    lib.sste_mvue_materialize_at.restype = ci
    lib.sste_linear_wgrad_at.argtypes = [vp, i64, i64, i64, ci, f32, vp, i64, i64, f32, u64, u64, i64, vp, i64, ci, vp, sz, vp]
    lib.sste_linear_wgrad_at.restype = ci
    lib.sste_compute_beta.argtypes = [vp, i64, i64, i64, vp, vp, sz, vp]
    lib.sste_beta_workspace_bytes.argtypes = [i64, i64]
    lib.sste_beta_workspace_bytes.restype = sz
    lib.sste_cast_fp8.argtypes = [vp, i64, i64, i64, ci, f32, vp, i64, vp, vp]
    lib.sste_flip_count.argtypes = [vp, vp, i64, i64, vp, vp]
    lib.sste_timing_begin.argtypes = [ci]
    lib.sste_timing_begin.restype = ci
    lib.sste_timing_end.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ci)]
    lib.sste_timing_end.restype = ci
    for name in ("sste_project_pack", "sste_sgd_project_pack", "sste_sgd_project_pack_batch_prepare", "sste_sgd_project_pack_batch", "sste_project_pack_batch_prepare", "sste_project_pack_batch", "sste_linear_fwd", "sste_linear_dgrad",
                 "sste_linear_wgrad", "sste_mvue_materialize", "sste_compute_beta", "sste_flip_count", "sste_cast_fp8"):
        getattr(lib, name).restype = ci
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != 0:
        raise SsteError(status, library().sste_last_error().decode())


def _stream(t: torch.Tensor) -> int:
    return torch.cuda.current_stream(t.device).cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    return t.data_ptr() if t.numel() > 0 else None


def _matrix(t: torch.Tensor, itemsize: int, name: str) -> Tuple[int, int, int]:
    """(rows, cols, leading dimension in elements) of a 2-D device tensor with unit inner stride."""
    if t.dim() != 2:
        raise ValueError(f"{name} must be 2-D")
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if t.element_size() != itemsize:
        raise ValueError(f"{name} must have {itemsize}-byte elements")
    if t.shape[1] > 1 and t.stride(1) != 1:
        raise ValueError(f"{name} must have unit stride along its last axis")
    ld = t.stride(0) if t.shape[0] > 1 else max(t.shape[1], t.stride(0) if t.shape[0] == 1 else t.shape[1])
    return t.shape[0], t.shape[1], max(ld, t.shape[1])


def _esize(dtype: int) -> int:
    return 1 if dtype in (F8E4M3, F8E5M2) else 2


def packed_buffers(R: int, K: int, dtype: int, device):
    """Uninitialised device buffers for a packed 2:4 operand with R rows and K dense columns: the blocked
    layout pads the rows to a multiple of 16."""
    rows = (R + 15) // 16 * 16
    vals = torch.empty((rows, K // 2), dtype=torch.uint8 if dtype in (F8E4M3, F8E5M2) else torch.int16, device=device)
    meta = torch.empty((rows, K // 8), dtype=torch.uint8, device=device)
    return vals, meta


def project_pack(W: torch.Tensor, beta: float, val_dtype: int = BF16, val_scale: float = 1.0,
                 vals: Optional[torch.Tensor] = None, meta: Optional[torch.Tensor] = None,
                 amax_out: Optional[torch.Tensor] = None, gamma: float = 0.0):
    """sste_project_pack(_gamma): beta * S_soft(W) packed 2:4.  Returns (vals, meta)."""
    O, I, ldw = _matrix(W, 2, "W")
    if vals is None or meta is None:
        v, m = packed_buffers(O, I, val_dtype, W.device)
        vals = v if vals is None else vals
        meta = m if meta is None else meta
    if gamma == 0.0:
        _check(library().sste_project_pack(_ptr(W), O, I, ldw, beta, val_dtype, val_scale, _ptr(vals), _ptr(meta),
                                           _ptr(amax_out), _stream(W)))
    else:
        _check(library().sste_project_pack_gamma(_ptr(W), O, I, ldw, beta, gamma, val_dtype, val_scale, _ptr(vals), _ptr(meta),
                                                 _ptr(amax_out), _stream(W)))
    return vals, meta


def sgd_project_pack(W: torch.Tensor, G: torch.Tensor, alpha: float, beta: float, val_dtype: int = BF16,
                     val_scale: float = 1.0, vals: Optional[torch.Tensor] = None, meta: Optional[torch.Tensor] = None):
    """sste_sgd_project_pack: W <- W - alpha * G in place (W bf16 or float32), then beta * S_soft(W)
    packed 2:4.  Returns (vals, meta)."""
    w_f32 = W.dtype == torch.float32
    O, I, ldw = _matrix(W, 4 if w_f32 else 2, "W")
    Og, Ig, ldg = _matrix(G, 4, "G")
    if (Og, Ig) != (O, I) or G.dtype != torch.float32:
        raise ValueError("G must be a float32 matrix of W's shape")
    if vals is None or meta is None:
        v, m = packed_buffers(O, I, val_dtype, W.device)
        vals = v if vals is None else vals
        meta = m if meta is None else meta
    _check(library().sste_sgd_project_pack(_ptr(W), F32 if w_f32 else BF16, O, I, ldw, _ptr(G), ldg, alpha, beta,
                                           val_dtype, val_scale, _ptr(vals), _ptr(meta), _stream(W)))
    return vals, meta


class _PackItem(ctypes.Structure):
    """sste_pack_item of include/sste.h."""
    _fields_ = [("W", ctypes.c_void_p), ("vals", ctypes.c_void_p), ("meta", ctypes.c_void_p),
                ("O", ctypes.c_int64), ("I", ctypes.c_int64), ("ldw", ctypes.c_int64),
                ("beta", ctypes.c_float), ("val_scale", ctypes.c_float)]


PACK_TABLE_ITEM_BYTES = 64


class PackBatch:
    """A prepared sste_project_pack_batch: the device table plus the tensors it points to.  `launch()`
    re-projects and re-packs every tensor in one kernel; call it again whenever the weights changed."""

    def __init__(self, Ws, betas, val_dtype: int = BF16, val_scales=None, vals=None, metas=None):
        n = len(Ws)
        if len(betas) != n:
            raise ValueError("one beta per tensor")
        val_scales = [1.0] * n if val_scales is None else list(val_scales)
        self.Ws, self.val_dtype = list(Ws), val_dtype
        self.vals, self.metas = [], []
        items = (_PackItem * max(n, 1))()
        for k, W in enumerate(self.Ws):
            O, I, ldw = _matrix(W, 2, "W")
            v, m = (vals[k], metas[k]) if vals is not None and metas is not None else packed_buffers(O, I, val_dtype, W.device)
            self.vals.append(v)
            self.metas.append(m)
            items[k] = _PackItem(_ptr(W), _ptr(v), _ptr(m), O, I, ldw, float(betas[k]), float(val_scales[k]))
        table_host = torch.zeros(max(n, 1) * PACK_TABLE_ITEM_BYTES, dtype=torch.uint8)
        total = ctypes.c_int64(0)
        _check(library().sste_project_pack_batch_prepare(ctypes.cast(items, ctypes.c_void_p), n, val_dtype,
                                                         ctypes.c_void_p(table_host.data_ptr()), ctypes.byref(total)))
        self.n, self.total_blocks = n, int(total.value)
        self.device = self.Ws[0].device if n else torch.device("cuda")
        self.table = table_host.to(self.device)

    def launch(self):
        """sste_project_pack_batch on the current stream of the tensors' device."""
        _check(library().sste_project_pack_batch(_ptr(self.table), self.n, self.total_blocks, self.val_dtype,
                                                 _stream(self.table)))
        return self.vals, self.metas


class _UpdateItem(ctypes.Structure):
    """sste_update_item of include/sste.h."""
    _fields_ = [("W", ctypes.c_void_p), ("G", ctypes.c_void_p), ("vals", ctypes.c_void_p), ("meta", ctypes.c_void_p),
                ("O", ctypes.c_int64), ("I", ctypes.c_int64), ("ldw", ctypes.c_int64), ("ldg", ctypes.c_int64),
                ("beta", ctypes.c_float), ("val_scale", ctypes.c_float)]


UPDATE_TABLE_ITEM_BYTES = 80


class UpdateBatch:
    """A prepared sste_sgd_project_pack_batch: `launch(alpha)` applies W <- W - alpha * G to every
    tensor in place and re-projects and re-packs it, in one kernel."""

    def __init__(self, Ws, Gs, betas, val_dtype: int = BF16, val_scales=None, vals=None, metas=None):
        n = len(Ws)
        if len(betas) != n or len(Gs) != n:
            raise ValueError("one gradient and one beta per tensor")
        val_scales = [1.0] * n if val_scales is None else list(val_scales)
        self.Ws, self.Gs, self.val_dtype = list(Ws), list(Gs), val_dtype
        w_f32 = n > 0 and self.Ws[0].dtype == torch.float32
        self.w_dtype = F32 if w_f32 else BF16
        self.vals, self.metas = [], []
        items = (_UpdateItem * max(n, 1))()
        for k, (W, G) in enumerate(zip(self.Ws, self.Gs)):
            if (W.dtype == torch.float32) != w_f32:
                raise ValueError("all dense weights of one table have the same type")
            O, I, ldw = _matrix(W, 4 if w_f32 else 2, "W")
            Og, Ig, ldg = _matrix(G, 4, "G")
            if (Og, Ig) != (O, I) or G.dtype != torch.float32:
                raise ValueError("G must be a float32 matrix of W's shape")
            v, m = (vals[k], metas[k]) if vals is not None and metas is not None else packed_buffers(O, I, val_dtype, W.device)
            self.vals.append(v)
            self.metas.append(m)
            items[k] = _UpdateItem(_ptr(W), _ptr(G), _ptr(v), _ptr(m), O, I, ldw, ldg, float(betas[k]), float(val_scales[k]))
        table_host = torch.zeros(max(n, 1) * UPDATE_TABLE_ITEM_BYTES, dtype=torch.uint8)
        total = ctypes.c_int64(0)
        _check(library().sste_sgd_project_pack_batch_prepare(ctypes.cast(items, ctypes.c_void_p), n, self.w_dtype, val_dtype,
                                                             ctypes.c_void_p(table_host.data_ptr()), ctypes.byref(total)))
        self.n, self.total_blocks = n, int(total.value)
        self.device = self.Ws[0].device if n else torch.device("cuda")
        self.table = table_host.to(self.device)

    def launch(self, alpha: float):
        """sste_sgd_project_pack_batch on the current stream of the tensors' device."""
        _check(library().sste_sgd_project_pack_batch(_ptr(self.table), self.n, self.total_blocks, self.w_dtype,
                                                     self.val_dtype, alpha, _stream(self.table)))
        return self.vals, self.metas


def linear_fwd(X: torch.Tensor, vals: torch.Tensor, meta: torch.Tensor, O: int, dtype: int = BF16, x_scale: float = 1.0,
               w_scale: float = 1.0, Z: Optional[torch.Tensor] = None) -> torch.Tensor:
    """sste_linear_fwd: Z = (x_scale * w_scale) * X decode(vals, meta)^T, bf16 output.  O = rows of the
    packed operand (the buffers themselves are padded to a multiple of 16 rows)."""
    T, I, ldx = _matrix(X, _esize(dtype), "X")
    if Z is None:
        Z = torch.empty((T, O), dtype=torch.bfloat16, device=X.device)
    _, _, ldz = _matrix(Z, 2, "Z")
    _check(library().sste_linear_fwd(_ptr(X), T, I, ldx, dtype, x_scale, _ptr(vals), _ptr(meta), O, w_scale, _ptr(Z), ldz,
                                     _stream(X)))
    return Z


def linear_fwd_ex(X: torch.Tensor, vals: torch.Tensor, meta: torch.Tensor, O: int, dtype: int = BF16, x_scale: float = 1.0,
                  w_scale: float = 1.0, z_dtype: int = BF16, z_scale: float = 1.0, Z: Optional[torch.Tensor] = None,
                  amax_out: Optional[torch.Tensor] = None):
    """sste_linear_fwd_ex: the forward product with a bf16 or e4m3 output and the output's largest magnitude.
    Returns (Z, amax_out)."""
    T, I, ldx = _matrix(X, _esize(dtype), "X")
    if Z is None:
        Z = torch.empty((T, O), dtype=torch.uint8 if z_dtype == F8E4M3 else torch.bfloat16, device=X.device)
    if amax_out is None and z_dtype == F8E4M3:
        amax_out = torch.empty(1, dtype=torch.float32, device=X.device)
    _, _, ldz = _matrix(Z, _esize(z_dtype), "Z")
    _check(library().sste_linear_fwd_ex(_ptr(X), T, I, ldx, dtype, x_scale, _ptr(vals), _ptr(meta), O, w_scale, _ptr(Z), ldz,
                                        z_dtype, z_scale, _ptr(amax_out), _stream(X)))
    return Z, amax_out


ACT_NONE, ACT_GELU_TANH = 0, 1


def linear_fwd_act(X: torch.Tensor, vals: torch.Tensor, meta: torch.Tensor, O: int, dtype: int = BF16, x_scale: float = 1.0,
                   w_scale: float = 1.0, act: int = ACT_GELU_TANH, a_dtype: int = BF16, a_scale: float = 1.0,
                   H: Optional[torch.Tensor] = None, A: Optional[torch.Tensor] = None, amax_out: Optional[torch.Tensor] = None,
                   store_pre: bool = True):
    """sste_linear_fwd_act: the forward product with the activation in its epilogue.  Returns (H or None, A, amax_out)."""
    T, I, ldx = _matrix(X, _esize(dtype), "X")
    if H is None and store_pre:
        H = torch.empty((T, O), dtype=torch.bfloat16, device=X.device)
    if A is None:
        A = torch.empty((T, O), dtype=torch.uint8 if a_dtype == F8E4M3 else torch.bfloat16, device=X.device)
    if amax_out is None and a_dtype == F8E4M3:
        amax_out = torch.empty(1, dtype=torch.float32, device=X.device)
    ldh = _matrix(H, 2, "H")[2] if H is not None else 0
    _, _, lda = _matrix(A, _esize(a_dtype), "A")
    _check(library().sste_linear_fwd_act(_ptr(X), T, I, ldx, dtype, x_scale, _ptr(vals), _ptr(meta), O, w_scale, act, _ptr(H), ldh,
                                         _ptr(A), lda, a_dtype, a_scale, _ptr(amax_out), _stream(X)))
    return H, A, amax_out


def linear_dgrad_act(dY: torch.Tensor, vals: torch.Tensor, meta: torch.Tensor, I: int, H: torch.Tensor, dtype: int = BF16,
                     dy_scale: float = 1.0, w_scale: float = 1.0, act: int = ACT_GELU_TANH, dX: Optional[torch.Tensor] = None):
    """sste_linear_dgrad_act: dX = (dY decode(vals, meta)) * act'(H), bf16 output."""
    T, O, lddy = _matrix(dY, _esize(dtype), "dY")
    if dX is None:
        dX = torch.empty((T, I), dtype=torch.bfloat16, device=dY.device)
    _, _, lddx = _matrix(dX, 2, "dX")
    _, _, ldh = _matrix(H, 2, "H")
    _check(library().sste_linear_dgrad_act(_ptr(dY), T, O, lddy, dtype, dy_scale, _ptr(vals), _ptr(meta), I, w_scale, act, _ptr(H),
                                           ldh, _ptr(dX), lddx, _stream(dY)))
    return dX


class AmaxHistory:
    """sste_amax_history: window of the last `length` largest magnitudes of one tensor (host side)."""

    class _Struct(ctypes.Structure):
        _fields_ = [("window", ctypes.c_float * 64), ("length", ctypes.c_int), ("next", ctypes.c_int)]

    def __init__(self, length: int):
        self._h = AmaxHistory._Struct()
        library().sste_amax_history_init(ctypes.byref(self._h), length)

    def push(self, amax: float, format_max: float) -> float:
        """Records amax and returns the scale to use next."""
        return float(library().sste_amax_history_push(ctypes.byref(self._h), amax, format_max))


def linear_dgrad(dY: torch.Tensor, vals: torch.Tensor, meta: torch.Tensor, I: int, dtype: int = BF16, dy_scale: float = 1.0,
                 w_scale: float = 1.0, dX: Optional[torch.Tensor] = None) -> torch.Tensor:
    """sste_linear_dgrad: dX = (dy_scale * w_scale) * dY decode(vals, meta), bf16 output.  I = dense columns of
    the packed operand."""
    T, O, lddy = _matrix(dY, _esize(dtype), "dY")
    if dX is None:
        dX = torch.empty((T, I), dtype=torch.bfloat16, device=dY.device)
    _, _, lddx = _matrix(dX, 2, "dX")
    _check(library().sste_linear_dgrad(_ptr(dY), T, O, lddy, dtype, dy_scale, _ptr(vals), _ptr(meta), I, w_scale, _ptr(dX),
                                       lddx, _stream(dY)))
    return dX


def wgrad_plan_override(mi: int = 0, ni: int = 0, splits: int = 0) -> None:
    """sste_wgrad_plan_override: fix the tile / split choice of the large-problem weight gradient (0 = automatic)."""
    _check(library().sste_wgrad_plan_override(mi, ni, splits))


def wgrad_workspace_bytes(T: int, O: int, I: int, dtype: int = BF16) -> int:
    return int(library().sste_wgrad_workspace_bytes(T, O, I, dtype))


def linear_wgrad(dY: torch.Tensor, X: torch.Tensor, seed: int, offset: int, dtype: int = BF16, dy_scale: float = 1.0,
                 x_scale: float = 1.0, dW: Optional[torch.Tensor] = None, accumulate: bool = False,
                 workspace: Optional[torch.Tensor] = None, first_token: int = 0) -> torch.Tensor:
    """sste_linear_wgrad(_at): dW (+)= scale * MVUE(dY^T; seed, offset) X, float32 output.  first_token: global
    index of the first token row when dY and X are a shard of the token axis."""
    T, O, lddy = _matrix(dY, _esize(dtype), "dY")
    T2, I, ldx = _matrix(X, _esize(dtype), "X")
    if T2 != T:
        raise ValueError("dY and X must have the same number of rows (tokens)")
    if dW is None:
        if accumulate:
            raise ValueError("accumulate needs an existing dW")
        dW = torch.empty((O, I), dtype=torch.float32, device=X.device)
    _, _, lddw = _matrix(dW, 4, "dW")
    need = wgrad_workspace_bytes(T, O, I, dtype)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(library().sste_linear_wgrad_at(_ptr(dY), T, O, lddy, dtype, dy_scale, _ptr(X), I, ldx, x_scale, seed, offset,
                                          first_token, _ptr(dW), lddw, int(bool(accumulate)), _ptr(workspace), ws_bytes, _stream(X)))
    return dW


NOALLOC_SCRATCH_BYTES = 64 << 20


def linear_wgrad_noalloc(dY: torch.Tensor, X: torch.Tensor, seed: int, offset: int, dW: torch.Tensor, dtype: int = BF16,
                         dy_scale: float = 1.0, x_scale: float = 1.0, accumulate: bool = False) -> torch.Tensor:
    """sste_linear_wgrad_noalloc: the weight gradient into a caller-owned dW with the library's built-in
    scratch; nothing is allocated on the way (not by this wrapper either)."""
    T, O, lddy = _matrix(dY, _esize(dtype), "dY")
    T2, I, ldx = _matrix(X, _esize(dtype), "X")
    if T2 != T:
        raise ValueError("dY and X must have the same number of rows (tokens)")
    _, _, lddw = _matrix(dW, 4, "dW")
    _check(library().sste_linear_wgrad_noalloc(_ptr(dY), T, O, lddy, dtype, dy_scale, _ptr(X), I, ldx, x_scale, seed, offset,
                                               _ptr(dW), lddw, int(bool(accumulate)), _stream(X)))
    return dW


def cast_fp8(X: torch.Tensor, scale: float, out_dtype: int = F8E4M3, Q: Optional[torch.Tensor] = None,
             amax_out: Optional[torch.Tensor] = None, store: bool = True):
    """sste_cast_fp8: Q = RNE(clamp(X / scale)) as e4m3 / e5m2 codes, amax_out = max |X|.  store=False asks
    for the largest magnitude only.  Returns (Q or None, amax_out)."""
    R, C, ldx = _matrix(X, 2, "X")
    if amax_out is None:
        amax_out = torch.empty(1, dtype=torch.float32, device=X.device)
    ldq = C
    if store:
        if Q is None:
            Q = torch.empty((R, C), dtype=torch.uint8, device=X.device)
        _, _, ldq = _matrix(Q, 1, "Q")
    _check(library().sste_cast_fp8(_ptr(X), R, C, ldx, out_dtype, scale, _ptr(Q) if store else None, ldq, _ptr(amax_out),
                                   _stream(X)))
    return (Q if store else None), amax_out


def mvue_materialize(dY: torch.Tensor, seed: int, offset: int, dtype: int = BF16, first_token: int = 0):
    """sste_mvue_materialize(_at): MVUE(dY^T) as a packed 2:4 operand.  Returns (vals (O, T/2), meta (O, T/8))."""
    T, O, lddy = _matrix(dY, _esize(dtype), "dY")
    vals, meta = packed_buffers(O, T, dtype, dY.device)
    vals.zero_()
    meta.zero_()
    _check(library().sste_mvue_materialize_at(_ptr(dY), T, O, lddy, dtype, seed, offset, first_token, _ptr(vals), _ptr(meta),
                                              _stream(dY)))
    return vals, meta


BETA_MSE, BETA_L1 = 0, 1


def compute_beta(W: torch.Tensor, kind: int = BETA_MSE, gamma: float = 0.0) -> torch.Tensor:
    """sste_compute_beta(_ex): the MSE-optimal (or L1-preserving) scale as a 1-element float32 device tensor."""
    O, I, ldw = _matrix(W, 2, "W")
    need = int(library().sste_beta_workspace_bytes(O, I))
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=W.device)
    out = torch.empty(1, dtype=torch.float32, device=W.device)
    if kind == BETA_MSE and gamma == 0.0:
        _check(library().sste_compute_beta(_ptr(W), O, I, ldw, _ptr(out), _ptr(ws), ws.numel(), _stream(W)))
    else:
        _check(library().sste_compute_beta_ex(_ptr(W), O, I, ldw, kind, gamma, _ptr(out), _ptr(ws), ws.numel(), _stream(W)))
    return out


def flip_count(meta_a: torch.Tensor, meta_b: torch.Tensor, O: int) -> torch.Tensor:
    """sste_flip_count: number of positions whose recorded state differs (1-element int64 device tensor)."""
    rows, I8, _ = _matrix(meta_a, 1, "meta_a")
    if tuple(meta_b.shape) != tuple(meta_a.shape) or not meta_a.is_contiguous() or not meta_b.is_contiguous():
        raise ValueError("metadata arrays must be contiguous and of equal shape")
    out = torch.empty(1, dtype=torch.int64, device=meta_a.device)
    _check(library().sste_flip_count(_ptr(meta_a), _ptr(meta_b), O, I8 * 8, _ptr(out), _stream(meta_a)))
    return out


KERNEL_NAMES = ("project_pack", "fwd", "wgrad", "wgrad_reduce", "mvue_pack", "dgrad", "sgd_project_pack", "cast")


def timing_begin(max_launches: int = 4096) -> None:
    """sste_timing_begin: bracket every following hot-path kernel launch with its own HIP event pair."""
    _check(library().sste_timing_begin(max_launches))


def timing_end():
    """sste_timing_end: {kernel name: (total milliseconds, launches)} since timing_begin."""
    ms = (ctypes.c_double * len(KERNEL_NAMES))()
    n = (ctypes.c_int * len(KERNEL_NAMES))()
    _check(library().sste_timing_end(ms, n))
    return {name: (float(ms[i]), int(n[i])) for i, name in enumerate(KERNEL_NAMES)}
