"""ctypes binding of ``libbigcn.so`` (see ``include/bigcn.h``).

Argument marshalling only: every step of the forward path runs in the HIP kernels of the
library.  PyTorch is used for device memory (``torch.empty``) and for the current stream.
There is no CPU fallback: if the library has not been built, or no GPU is present, calls
raise.
"""

from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIBRARY = os.path.join(HERE, "libbigcn.so")

BIGCN_OK = 0
BIGCN_EINVAL = -1
BIGCN_ENULL = -2
BIGCN_ESHAPE = -3
BIGCN_EWORKSPACE = -4
BIGCN_EGRAPH = -5
BIGCN_EHIP = -6
MAX_K_BITS = 8192
GEMM_AUTO, GEMM_VALU, GEMM_MFMA, GEMM_FP4 = 0, 1, 2, 3
MAX_FORWARD_D_OUT = 512
VALIDATE_NONE, VALIDATE_GCN, VALIDATE_NEIGHBOURS = 0, 1, 2

EXPORTS = (
    "bigcn_status_string", "bigcn_version", "bigcn_pack", "bigcn_binary_gemm",
    "bigcn_binary_gemm_variant", "bigcn_gcn_norm",
    "bigcn_plan_create", "bigcn_plan_destroy", "bigcn_plan_rows", "bigcn_plan_nnz", "bigcn_spmm",
    "bigcn_forward_workspace_bytes", "bigcn_forward_row_bytes", "bigcn_forward", "bigcn_profile_create",
    "bigcn_profile_destroy", "bigcn_forward_profiled", "bigcn_profile_read",
    "bigcn_mean_norm", "bigcn_sage_forward_workspace_bytes", "bigcn_sage_forward",
    "bigcn_sage_forward_profiled", "bigcn_forward_packed", "bigcn_column_stats_workspace_bytes",
    "bigcn_column_stats", "bigcn_predict", "bigcn_layer_backward_workspace_bytes",
    "bigcn_layer_backward", "bigcn_entropy_workspace_bytes", "bigcn_entropy",
    "bigcn_gat_layer_workspace_bytes", "bigcn_gat_layer", "bigcn_forward_static",
    "bigcn_probe_fp4_multiply_rate", "bigcn_probe_fp4_expand_multiply_rate", "bigcn_probe_stream_read",
    "bigcn_forward_gemm_path",
    "bigcn_forward_row_layout", "bigcn_forward_workspace_map",
)


class BigcnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class LayerDesc(ctypes.Structure):
    """Mirror of ``bigcn_layer``."""
    _fields_ = [
        ("w_bits", ctypes.c_void_p), ("alpha", ctypes.c_void_p),
        ("d_in", ctypes.c_int64), ("d_out", ctypes.c_int64), ("ld_words", ctypes.c_int64),
        ("bn_shift", ctypes.c_void_p), ("bn_mul", ctypes.c_void_p),
    ]


class SageLayerDesc(ctypes.Structure):
    """Mirror of ``bigcn_sage_layer``."""
    _fields_ = [
        ("w_self_bits", ctypes.c_void_p), ("alpha_self", ctypes.c_void_p),
        ("w_nbr_bits", ctypes.c_void_p), ("alpha_nbr", ctypes.c_void_p),
        ("d_in", ctypes.c_int64), ("d_out", ctypes.c_int64), ("ld_words", ctypes.c_int64),
        ("bn_shift", ctypes.c_void_p), ("bn_mul", ctypes.c_void_p),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIBRARY):
            raise RuntimeError(
                f"{LIBRARY} is missing: build it with `python -m paper_2210_13149_amd.build` "
                "(or __graft_entry__.build()); there is no CPU fallback")
        L = ctypes.CDLL(LIBRARY)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.bigcn_status_string.restype = ctypes.c_char_p
        L.bigcn_status_string.argtypes = [i32]
        L.bigcn_version.restype = i32
        L.bigcn_version.argtypes = []
        L.bigcn_pack.restype = i32
        L.bigcn_pack.argtypes = [vp, i64, i64, i64, i64, vp, vp, vp, i64, vp, vp]
        L.bigcn_binary_gemm.restype = i32
        L.bigcn_binary_gemm.argtypes = [vp, vp, i64, i64, vp, vp, i64, i64, i64, vp, i64, vp, i64, vp]
        L.bigcn_binary_gemm_variant.restype = i32
        L.bigcn_binary_gemm_variant.argtypes = [vp, vp, i64, i64, vp, vp, i64, i64, i64, vp, i64, vp, i64,
                                                i32, vp]
        L.bigcn_gcn_norm.restype = i32
        L.bigcn_gcn_norm.argtypes = [vp, vp, i64, vp, vp, vp]
        L.bigcn_plan_create.restype = i32
        L.bigcn_plan_create.argtypes = [vp, vp, i64, i32, ctypes.POINTER(vp), vp]
        L.bigcn_plan_destroy.restype = None
        L.bigcn_plan_destroy.argtypes = [vp]
        L.bigcn_plan_rows.restype = i64
        L.bigcn_plan_rows.argtypes = [vp]
        L.bigcn_plan_nnz.restype = i64
        L.bigcn_plan_nnz.argtypes = [vp]
        L.bigcn_spmm.restype = i32
        L.bigcn_spmm.argtypes = [vp, vp, vp, vp, i64, vp, i64, i64, vp, i64, vp]
        L.bigcn_forward_workspace_bytes.restype = ctypes.c_size_t
        L.bigcn_forward_workspace_bytes.argtypes = [i64, ctypes.POINTER(LayerDesc), i32]
        L.bigcn_forward_row_bytes.restype = i64
        L.bigcn_forward_row_bytes.argtypes = [i64, i64, ctypes.POINTER(i32)]
        L.bigcn_forward_gemm_path.restype = i32
        L.bigcn_forward_gemm_path.argtypes = [i64, i64, i64]
        L.bigcn_forward_row_layout.restype = i32
        L.bigcn_forward_row_layout.argtypes = [i64, i64, ctypes.POINTER(i32)]
        L.bigcn_forward_workspace_map.restype = i32
        L.bigcn_forward_workspace_map.argtypes = [i64, ctypes.POINTER(LayerDesc), i32, ctypes.POINTER(ctypes.c_size_t)]
        L.bigcn_forward.restype = i32
        L.bigcn_forward.argtypes = [vp, vp, vp, vp, i64, vp, i64, ctypes.POINTER(LayerDesc), i32, vp,
                                    i64, vp, ctypes.c_size_t, vp]
        L.bigcn_forward_static.restype = i32
        L.bigcn_forward_static.argtypes = [vp, vp, vp, vp, i64, vp, i64, ctypes.POINTER(LayerDesc), i32, vp,
                                           i64, vp]
        L.bigcn_probe_fp4_multiply_rate.restype = i32
        L.bigcn_probe_fp4_multiply_rate.argtypes = [i32, vp, i64, ctypes.POINTER(i64), vp]
        L.bigcn_probe_stream_read.restype = i32
        L.bigcn_probe_stream_read.argtypes = [vp, i64, vp, i64, vp]
        L.bigcn_probe_fp4_expand_multiply_rate.restype = i32
        L.bigcn_probe_fp4_expand_multiply_rate.argtypes = [i32, vp, i64, ctypes.POINTER(i64), vp]
        L.bigcn_profile_create.restype = i32
        L.bigcn_profile_create.argtypes = [i32, i32, ctypes.POINTER(vp)]
        L.bigcn_profile_destroy.restype = None
        L.bigcn_profile_destroy.argtypes = [vp]
        L.bigcn_forward_profiled.restype = i32
        L.bigcn_forward_profiled.argtypes = L.bigcn_forward.argtypes + [vp]
        L.bigcn_profile_read.restype = i32
        L.bigcn_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32)]
        L.bigcn_forward_packed.restype = i32
        L.bigcn_forward_packed.argtypes = [vp, vp, vp, vp, i64, vp, i64, vp, ctypes.POINTER(LayerDesc), i32,
                                           vp, i64, vp, ctypes.c_size_t, vp]
        L.bigcn_column_stats_workspace_bytes.restype = ctypes.c_size_t
        L.bigcn_column_stats_workspace_bytes.argtypes = [i64, i64]
        L.bigcn_column_stats.restype = i32
        L.bigcn_column_stats.argtypes = [vp, i64, i64, i64, ctypes.c_double, vp, vp, vp, ctypes.c_size_t, vp]
        L.bigcn_predict.restype = i32
        L.bigcn_predict.argtypes = [vp, i64, i64, i64, vp, vp, i64, vp]
        L.bigcn_layer_backward_workspace_bytes.restype = ctypes.c_size_t
        L.bigcn_layer_backward_workspace_bytes.argtypes = [i64, i64, i64]
        L.bigcn_layer_backward.restype = i32
        L.bigcn_layer_backward.argtypes = [vp, vp, vp, vp, i64, vp, i64, vp, i64, vp, vp, i64, i64, i64, vp,
                                           vp, i64, vp, i64, vp, ctypes.c_size_t, vp]
        L.bigcn_entropy_workspace_bytes.restype = ctypes.c_size_t
        L.bigcn_entropy_workspace_bytes.argtypes = [i64, i32]
        L.bigcn_entropy.restype = i32
        L.bigcn_entropy.argtypes = [vp, i64, i64, i64, i32, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.bigcn_gat_layer_workspace_bytes.restype = ctypes.c_size_t
        L.bigcn_gat_layer_workspace_bytes.argtypes = [i64, i64, i64, i32]
        L.bigcn_gat_layer.restype = i32
        L.bigcn_gat_layer.argtypes = [vp, vp, vp, i64, vp, i64, vp, vp, vp, vp, i64, i64, i64, i32, vp, vp,
                                      ctypes.c_float, vp, i64, vp, ctypes.c_size_t, vp]
        L.bigcn_mean_norm.restype = i32
        L.bigcn_mean_norm.argtypes = [vp, i64, vp, vp]
        L.bigcn_sage_forward_workspace_bytes.restype = ctypes.c_size_t
        L.bigcn_sage_forward_workspace_bytes.argtypes = [i64, ctypes.POINTER(SageLayerDesc), i32]
        L.bigcn_sage_forward.restype = i32
        L.bigcn_sage_forward.argtypes = [vp, vp, vp, vp, i64, vp, i64, ctypes.POINTER(SageLayerDesc), i32,
                                         vp, i64, vp, ctypes.c_size_t, vp]
        L.bigcn_sage_forward_profiled.restype = i32
        L.bigcn_sage_forward_profiled.argtypes = L.bigcn_sage_forward.argtypes + [vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().bigcn_status_string(int(status)).decode()


def version() -> int:
    return int(lib().bigcn_version())


def _check(status: int, where: str) -> None:
    if status != BIGCN_OK:
        raise BigcnError(status, where)


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA (HIP) tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    return t


def n_words(k_bits: int) -> int:
    return (int(k_bits) + 63) // 64


# ------------------------------------------------------------------------------------------
# kernel 1
# ------------------------------------------------------------------------------------------
def bigcn_pack(x: torch.Tensor, shift: Optional[torch.Tensor] = None,
               mul: Optional[torch.Tensor] = None, ld_words: Optional[int] = None
               ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Binarise + pack the rows of a 2-D fp32 tensor (any strides, e.g. ``W.t()``).
    Returns ``(bits int64 (rows, ld_words) holding the uint64 words, scale fp32 (rows,))``."""
    _dev(x, torch.float32, "x")
    if x.dim() != 2:
        raise ValueError("x must be a matrix")
    rows, cols = x.shape
    words = n_words(cols)
    ld = words if ld_words is None else int(ld_words)
    bits = torch.zeros((rows, max(ld, 1)), dtype=torch.int64, device=x.device)
    scale = torch.empty((rows,), dtype=torch.float32, device=x.device)
    for p, name in ((shift, "shift"), (mul, "mul")):
        if p is not None:
            _dev(p, torch.float32, name)
            if p.shape != (cols,) or not p.is_contiguous():
                raise ValueError(f"{name} must be a contiguous vector of length cols")
    _check(lib().bigcn_pack(_ptr(x), rows, cols, x.stride(0), x.stride(1), _ptr(shift), _ptr(mul),
                            _ptr(bits), ld, _ptr(scale), _stream()), "bigcn_pack")
    return bits, scale


def pack_weight(w: torch.Tensor) -> Tuple[torch.Tensor, torch.Tensor]:
    """Packed signs of the columns of W (d_in, d_out) and their scales alpha (d_out,)."""
    return bigcn_pack(w.t())


# ------------------------------------------------------------------------------------------
# kernel 2
# ------------------------------------------------------------------------------------------
def bigcn_binary_gemm(a_bits: torch.Tensor, a_scale: Optional[torch.Tensor], b_bits: torch.Tensor,
                      b_scale: Optional[torch.Tensor], k_bits: int, want_acc: bool = True,
                      want_out: bool = True, variant: int = 0
                      ) -> Tuple[Optional[torch.Tensor], Optional[torch.Tensor]]:
    """``acc = K - 2 popcount(a xor b)`` (int32) and / or ``out = a_scale_i b_scale_j acc``.
    ``variant``: GEMM_AUTO (per shape), GEMM_VALU (XOR + bit count), GEMM_MFMA (int8 matrix
    cores) or GEMM_FP4 (FP4 codes of +-1 on the block-scaled matrix cores)."""
    _dev(a_bits, torch.int64, "a_bits")
    _dev(b_bits, torch.int64, "b_bits")
    m, n = a_bits.shape[0], b_bits.shape[0]
    acc = torch.empty((m, n), dtype=torch.int32, device=a_bits.device) if want_acc else None
    out = torch.empty((m, n), dtype=torch.float32, device=a_bits.device) if want_out else None
    if want_out:
        _dev(a_scale, torch.float32, "a_scale")
        _dev(b_scale, torch.float32, "b_scale")
    args = (_ptr(a_bits), _ptr(a_scale), m, a_bits.stride(0), _ptr(b_bits), _ptr(b_scale), n,
            b_bits.stride(0), int(k_bits), _ptr(acc), n, _ptr(out), n)
    if variant == GEMM_AUTO:
        _check(lib().bigcn_binary_gemm(*args, _stream()), "bigcn_binary_gemm")
    else:
        _check(lib().bigcn_binary_gemm_variant(*args, int(variant), _stream()), "bigcn_binary_gemm_variant")
    return acc, out


# ------------------------------------------------------------------------------------------
# graph helpers and kernel 3
# ------------------------------------------------------------------------------------------
def bigcn_gcn_norm(row_ptr: torch.Tensor, col_idx: torch.Tensor, want_vals: bool = False
                   ) -> Tuple[torch.Tensor, Optional[torch.Tensor]]:
    _dev(row_ptr, torch.int64, "row_ptr")
    _dev(col_idx, torch.int32, "col_idx")
    n = row_ptr.numel() - 1
    dinv = torch.empty((n,), dtype=torch.float32, device=row_ptr.device)
    vals = torch.empty((col_idx.numel(),), dtype=torch.float32, device=row_ptr.device) if want_vals else None
    _check(lib().bigcn_gcn_norm(_ptr(row_ptr), _ptr(col_idx), n, _ptr(dinv), _ptr(vals), _stream()),
           "bigcn_gcn_norm")
    return dinv, vals


class Plan:
    """Owner of a ``bigcn_plan`` (destroyed with the object)."""

    def __init__(self, row_ptr: torch.Tensor, col_idx: torch.Tensor, validate=True):
        """``validate``: False / True (pattern of A + I) or one of the ``VALIDATE_*`` values."""
        _dev(row_ptr, torch.int64, "row_ptr")
        _dev(col_idx, torch.int32, "col_idx")
        self.n = row_ptr.numel() - 1
        handle = ctypes.c_void_p()
        self._handle = None
        _check(lib().bigcn_plan_create(_ptr(row_ptr), _ptr(col_idx), self.n, int(validate),
                                       ctypes.byref(handle), _stream()), "bigcn_plan_create")
        self._handle = handle

    @property
    def handle(self) -> ctypes.c_void_p:
        if self._handle is None:
            raise RuntimeError("plan was destroyed")
        return self._handle

    @property
    def nnz(self) -> int:
        return int(lib().bigcn_plan_nnz(self.handle))

    def destroy(self) -> None:
        if self._handle is not None:
            lib().bigcn_plan_destroy(self._handle)
            self._handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def bigcn_spmm(plan: Plan, row_ptr: torch.Tensor, col_idx: torch.Tensor,
               vals: Optional[torch.Tensor], z: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """``out = sum_p vals[p] * z[col_idx[p], :]`` per CSR row (vals None = ones)."""
    _dev(z, torch.float32, "z")
    if z.dim() != 2 or (z.shape[1] > 1 and z.stride(1) != 1):
        raise ValueError("z must be a row-major matrix")
    if vals is not None:
        _dev(vals, torch.float32, "vals")
    n, d = z.shape
    if out is None:
        out = torch.empty((n, d), dtype=torch.float32, device=z.device)
    else:
        _dev(out, torch.float32, "out")
        if out.shape != z.shape or (d > 1 and out.stride(1) != 1):
            raise ValueError("out must be a row-major matrix of z's shape")
    _check(lib().bigcn_spmm(plan.handle, _ptr(row_ptr), _ptr(col_idx), _ptr(vals), n, _ptr(z), d,
                            z.stride(0), _ptr(out), out.stride(0), _stream()), "bigcn_spmm")
    return out


# ------------------------------------------------------------------------------------------
# fused forward
# ------------------------------------------------------------------------------------------
class Layer:
    """Device-resident parameters of one binarised layer."""

    def __init__(self, w_bits: torch.Tensor, alpha: torch.Tensor, d_in: int, d_out: int,
                 bn_shift: Optional[torch.Tensor] = None, bn_mul: Optional[torch.Tensor] = None):
        self.w_bits = _dev(w_bits, torch.int64, "w_bits")
        self.alpha = _dev(alpha, torch.float32, "alpha")
        self.d_in, self.d_out = int(d_in), int(d_out)
        self.bn_shift = None if bn_shift is None else _dev(bn_shift, torch.float32, "bn_shift").contiguous()
        self.bn_mul = None if bn_mul is None else _dev(bn_mul, torch.float32, "bn_mul").contiguous()

    @classmethod
    def from_weight(cls, w: torch.Tensor, bn_shift=None, bn_mul=None) -> "Layer":
        bits, alpha = pack_weight(w)
        return cls(bits, alpha, w.shape[0], w.shape[1], bn_shift, bn_mul)

    def desc(self) -> LayerDesc:
        return LayerDesc(_ptr(self.w_bits), _ptr(self.alpha), self.d_in, self.d_out,
                         self.w_bits.stride(0), _ptr(self.bn_shift), _ptr(self.bn_mul))


def _descs(layers: Sequence[Layer]):
    arr = (LayerDesc * len(layers))(*[l.desc() for l in layers])
    return arr


def bigcn_forward_row_bytes(d_in: int, d_out: int) -> Tuple[int, bool]:
    """(bytes of the per-node product row of such a layer, whether the source scale is inside)."""
    flag = ctypes.c_int(0)
    size = int(lib().bigcn_forward_row_bytes(int(d_in), int(d_out), ctypes.byref(flag)))
    return size, bool(flag.value)


ROW_LAYOUT_FIELDS = ("groups", "vec", "kind", "k_eff", "fold_last", "scale_place", "escape", "alt_kind")


def bigcn_forward_row_layout(d_in: int, d_out: int) -> dict:
    """The compact product-row layout of a layer as a dict of ``ROW_LAYOUT_FIELDS``."""
    fields = (ctypes.c_int32 * 8)()
    _check(lib().bigcn_forward_row_layout(d_in, d_out, fields), "bigcn_forward_row_layout")
    return dict(zip(ROW_LAYOUT_FIELDS, (int(v) for v in fields)))


def bigcn_forward_workspace_map(n: int, layers: Sequence["Layer"]) -> dict:
    """Byte offsets of the workspace regions of ``bigcn_forward`` (see the header)."""
    off = (ctypes.c_size_t * 6)()
    _check(lib().bigcn_forward_workspace_map(n, _descs(layers), len(layers), off), "bigcn_forward_workspace_map")
    return dict(zip(("bits", "scale0", "scale1", "rows", "alt_rows", "total"), (int(v) for v in off)))


def bigcn_forward_gemm_path(n: int, d_in: int, d_out: int) -> int:
    """GEMM_FP4 or GEMM_VALU: the evaluation path the fused forward uses for such a layer."""
    path = lib().bigcn_forward_gemm_path(n, d_in, d_out)
    _check(min(path, 0), "bigcn_forward_gemm_path")
    return path


def bigcn_forward_workspace_bytes(n: int, layers: Sequence[Layer]) -> int:
    return int(lib().bigcn_forward_workspace_bytes(int(n), _descs(layers), len(layers)))


class Profile:
    """Owner of a ``bigcn_profile``: per-launch HIP-event timing of forward calls."""

    def __init__(self, n_layers: int, max_calls: int):
        self.n_layers = int(n_layers)
        handle = ctypes.c_void_p()
        self._handle = None
        _check(lib().bigcn_profile_create(self.n_layers, int(max_calls), ctypes.byref(handle)),
               "bigcn_profile_create")
        self._handle = handle

    @property
    def handle(self):
        if self._handle is None:
            raise RuntimeError("profile was destroyed")
        return self._handle

    def read(self) -> Tuple[List[float], int]:
        """Mean milliseconds per launch slot over the calls since the last read, and that count."""
        ms = (ctypes.c_float * (1 + 2 * self.n_layers))()
        calls = ctypes.c_int(0)
        _check(lib().bigcn_profile_read(self.handle, ms, ctypes.byref(calls)), "bigcn_profile_read")
        return [float(v) for v in ms], int(calls.value)

    def destroy(self) -> None:
        if self._handle is not None:
            lib().bigcn_profile_destroy(self._handle)
            self._handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def bigcn_forward(plan: Plan, row_ptr: torch.Tensor, col_idx: torch.Tensor, dinv_sqrt: torch.Tensor,
                  x: torch.Tensor, layers: Sequence[Layer], workspace: Optional[torch.Tensor] = None,
                  logits: Optional[torch.Tensor] = None, profile: Optional[Profile] = None
                  ) -> torch.Tensor:
    """L-layer fused forward; returns fp32 logits (n, d_out of the last layer).  With
    ``profile`` the call goes through ``bigcn_forward_profiled``."""
    _dev(x, torch.float32, "x")
    if x.dim() != 2 or (x.shape[1] > 1 and x.stride(1) != 1):
        raise ValueError("x must be a row-major matrix")
    n = x.shape[0]
    descs = _descs(layers)
    if workspace is None:
        need = bigcn_forward_workspace_bytes(n, layers)
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=x.device)
    if logits is None:
        logits = torch.empty((n, layers[-1].d_out), dtype=torch.float32, device=x.device)
    args = (plan.handle, _ptr(row_ptr), _ptr(col_idx), _ptr(dinv_sqrt), n, _ptr(x), x.stride(0), descs,
            len(layers), _ptr(logits), logits.stride(0), _ptr(workspace), workspace.numel(), _stream())
    if profile is None:
        _check(lib().bigcn_forward(*args), "bigcn_forward")
    else:
        _check(lib().bigcn_forward_profiled(*args, profile.handle), "bigcn_forward_profiled")
    return logits


def bigcn_probe_fp4_multiply_rate(iterations: int, sink: Optional[torch.Tensor] = None) -> int:
    """Launch the multiply-only kernel (measurement aid); returns the multiply-accumulates it performs."""
    if sink is None:
        sink = torch.empty((256 * 1024,), dtype=torch.float32, device="cuda")
    _dev(sink, torch.float32, "sink")
    macs = ctypes.c_int64(0)
    _check(lib().bigcn_probe_fp4_multiply_rate(int(iterations), _ptr(sink), sink.numel(), ctypes.byref(macs), _stream()),
           "bigcn_probe_fp4_multiply_rate")
    return int(macs.value)


def bigcn_probe_fp4_expand_multiply_rate(iterations: int, sink: Optional[torch.Tensor] = None) -> int:
    """Launch the expand-and-multiply kernel (measurement aid); returns the multiply-accumulates it performs."""
    if sink is None:
        sink = torch.empty((256 * 1024,), dtype=torch.float32, device="cuda")
    _dev(sink, torch.float32, "sink")
    macs = ctypes.c_int64(0)
    _check(lib().bigcn_probe_fp4_expand_multiply_rate(int(iterations), _ptr(sink), sink.numel(), ctypes.byref(macs),
                                                      _stream()), "bigcn_probe_fp4_expand_multiply_rate")
    return int(macs.value)


def bigcn_probe_stream_read(src: torch.Tensor, sink: Optional[torch.Tensor] = None) -> int:
    """Launch the read-only kernel over `src` (measurement aid); returns the bytes it reads."""
    if not src.is_cuda or not src.is_contiguous():
        raise TypeError("src must be a contiguous device tensor")
    if sink is None:
        sink = torch.empty((8192 * 1024,), dtype=torch.float32, device="cuda")
    _dev(sink, torch.float32, "sink")
    nbytes = src.numel() * src.element_size()
    _check(lib().bigcn_probe_stream_read(_ptr(src), nbytes, _ptr(sink), sink.numel(), _stream()), "bigcn_probe_stream_read")
    return nbytes // 16 * 16


STATIC_WORKSPACE_BYTES = 32 << 20   # BIGCN_STATIC_WORKSPACE_BYTES of the header


def bigcn_forward_static(plan: Plan, row_ptr: torch.Tensor, col_idx: torch.Tensor, dinv_sqrt: torch.Tensor,
                         x: torch.Tensor, layers: Sequence[Layer], logits: torch.Tensor) -> torch.Tensor:
    """``bigcn_forward`` with the workspace in the library's own per-GPU array: the call allocates
    nothing, so the caller provides ``logits``."""
    _dev(x, torch.float32, "x")
    _dev(logits, torch.float32, "logits")
    if x.dim() != 2 or (x.shape[1] > 1 and x.stride(1) != 1):
        raise ValueError("x must be a row-major matrix")
    _check(lib().bigcn_forward_static(plan.handle, _ptr(row_ptr), _ptr(col_idx), _ptr(dinv_sqrt), x.shape[0],
                                      _ptr(x), x.stride(0), _descs(layers), len(layers), _ptr(logits),
                                      logits.stride(0), _stream()), "bigcn_forward_static")
    return logits


def bigcn_forward_packed(plan: Plan, row_ptr: torch.Tensor, col_idx: torch.Tensor,
                         dinv_sqrt: torch.Tensor, x_bits: torch.Tensor, x_beta: torch.Tensor,
                         layers: Sequence[Layer], workspace: Optional[torch.Tensor] = None,
                         logits: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The fused forward from packed input signs and row scales (outputs of ``bigcn_pack``)."""
    _dev(x_bits, torch.int64, "x_bits")
    _dev(x_beta, torch.float32, "x_beta")
    if x_bits.dim() != 2 or (x_bits.shape[1] > 1 and x_bits.stride(1) != 1):
        raise ValueError("x_bits must be a row-major matrix of words")
    n = x_bits.shape[0]
    if x_beta.numel() != n:
        raise ValueError("x_beta must hold one scale per row of x_bits")
    descs = _descs(layers)
    if workspace is None:
        need = bigcn_forward_workspace_bytes(n, layers)
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=x_bits.device)
    if logits is None:
        logits = torch.empty((n, layers[-1].d_out), dtype=torch.float32, device=x_bits.device)
    _check(lib().bigcn_forward_packed(plan.handle, _ptr(row_ptr), _ptr(col_idx), _ptr(dinv_sqrt), n,
                                      _ptr(x_bits), x_bits.stride(0), _ptr(x_beta), descs, len(layers),
                                      _ptr(logits), logits.stride(0), _ptr(workspace), workspace.numel(),
                                      _stream()), "bigcn_forward_packed")
    return logits


def bigcn_column_stats(x: torch.Tensor, eps: float = 1e-5) -> Tuple[torch.Tensor, torch.Tensor]:
    """Per-column ``(mean, 1/sqrt(var + eps))`` of an fp32 device matrix, as fp32 vectors."""
    _dev(x, torch.float32, "x")
    if x.dim() != 2 or (x.shape[1] > 1 and x.stride(1) != 1):
        raise ValueError("x must be a row-major matrix")
    rows, cols = x.shape
    need = int(lib().bigcn_column_stats_workspace_bytes(rows, cols))
    workspace = torch.empty((max(need, 8) // 8,), dtype=torch.float64, device=x.device)
    shift = torch.empty((cols,), dtype=torch.float32, device=x.device)
    mul = torch.empty((cols,), dtype=torch.float32, device=x.device)
    _check(lib().bigcn_column_stats(_ptr(x), rows, cols, x.stride(0), float(eps), _ptr(shift), _ptr(mul),
                                    _ptr(workspace), workspace.numel() * 8, _stream()), "bigcn_column_stats")
    return shift, mul


def bigcn_predict(logits: torch.Tensor, want_probs: bool = False
                  ) -> Tuple[torch.Tensor, Optional[torch.Tensor]]:
    """``(labels int32 (n,), softmax probabilities (n, d) or None)`` of a row-major fp32 matrix."""
    _dev(logits, torch.float32, "logits")
    if logits.dim() != 2 or (logits.shape[1] > 1 and logits.stride(1) != 1):
        raise ValueError("logits must be a row-major matrix")
    n, d = logits.shape
    labels = torch.empty((n,), dtype=torch.int32, device=logits.device)
    probs = torch.empty((n, d), dtype=torch.float32, device=logits.device) if want_probs else None
    _check(lib().bigcn_predict(_ptr(logits), n, d, logits.stride(0), _ptr(labels), _ptr(probs), d, _stream()),
           "bigcn_predict")
    return labels, probs


def bigcn_layer_backward(plan: Plan, row_ptr: torch.Tensor, col_idx: torch.Tensor, vals: torch.Tensor,
                         g_out: torch.Tensor, f_bits: torch.Tensor, beta: torch.Tensor, w: torch.Tensor,
                         bn_mul: Optional[torch.Tensor] = None, want_input_grad: bool = True,
                         workspace: Optional[torch.Tensor] = None
                         ) -> Tuple[torch.Tensor, Optional[torch.Tensor]]:
    """Back propagation through one binarised layer: returns ``(g_w (d_in, d_out), g_in (n, d_in)
    or None)`` from ``g_out (n, d_out)``, the layer's packed input ``(f_bits, beta)`` and its
    fp32 weights ``w (d_in, d_out)``."""
    for t, name in ((g_out, "g_out"), (beta, "beta"), (w, "w"), (vals, "vals")):
        _dev(t, torch.float32, name)
    _dev(f_bits, torch.int64, "f_bits")
    if g_out.dim() != 2 or w.dim() != 2 or g_out.stride(1) != 1 or w.stride(1) != 1:
        raise ValueError("g_out and w must be row-major matrices")
    n, d_out = g_out.shape
    d_in = w.shape[0]
    if w.shape[1] != d_out or f_bits.shape[0] != n or beta.numel() != n:
        raise ValueError("shape mismatch")
    need = int(lib().bigcn_layer_backward_workspace_bytes(n, d_in, d_out))
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=g_out.device)
    g_w = torch.empty((d_in, d_out), dtype=torch.float32, device=g_out.device)
    g_in = torch.empty((n, d_in), dtype=torch.float32, device=g_out.device) if want_input_grad else None
    _check(lib().bigcn_layer_backward(plan.handle, _ptr(row_ptr), _ptr(col_idx), _ptr(vals), n, _ptr(g_out),
                                      g_out.stride(0), _ptr(f_bits), f_bits.stride(0), _ptr(beta), _ptr(w),
                                      w.stride(0), d_in, d_out, _ptr(bn_mul), _ptr(g_w), g_w.stride(0),
                                      _ptr(g_in), d_in, _ptr(workspace), workspace.numel(), _stream()),
           "bigcn_layer_backward")
    return g_w, g_in


def bigcn_entropy(h: torch.Tensor, bins: int, want_counts: bool = False
                  ) -> Tuple[torch.Tensor, torch.Tensor, Optional[torch.Tensor]]:
    """Binning estimate of the entropy of a hidden layer: ``(per-neuron entropies in bits (fp64),
    their sum (fp64 scalar tensor), counts (cols, bins) int32 or None)``."""
    _dev(h, torch.float32, "h")
    if h.dim() != 2 or (h.shape[1] > 1 and h.stride(1) != 1):
        raise ValueError("h must be a row-major matrix")
    rows, cols = h.shape
    need = int(lib().bigcn_entropy_workspace_bytes(cols, int(bins)))
    workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=h.device)
    per = torch.empty((cols,), dtype=torch.float64, device=h.device)
    total = torch.empty((1,), dtype=torch.float64, device=h.device)
    counts = torch.empty((cols, int(bins)), dtype=torch.int32, device=h.device) if want_counts else None
    _check(lib().bigcn_entropy(_ptr(h), rows, cols, h.stride(0), int(bins), _ptr(per), _ptr(total), _ptr(counts),
                               _ptr(workspace), workspace.numel(), _stream()), "bigcn_entropy")
    return per, total[0], counts


def bigcn_gat_layer(plan: Plan, row_ptr: torch.Tensor, col_idx: torch.Tensor, x: torch.Tensor,
                    layer: "Layer", a_src: torch.Tensor, a_dst: torch.Tensor, heads: int = 1,
                    negative_slope: float = 0.2) -> torch.Tensor:
    """One Bi-GAT layer: ``layer`` holds the packed weights (and optional standardisation), ``a_src`` /
    ``a_dst`` the attention vectors, shape (heads, d_out / heads).  Returns fp32 (n, d_out)."""
    _dev(x, torch.float32, "x")
    a_src = _dev(a_src, torch.float32, "a_src").contiguous()
    a_dst = _dev(a_dst, torch.float32, "a_dst").contiguous()
    if x.dim() != 2 or (x.shape[1] > 1 and x.stride(1) != 1):
        raise ValueError("x must be a row-major matrix")
    if a_src.numel() != layer.d_out or a_dst.numel() != layer.d_out:
        raise ValueError("attention vectors must hold d_out entries each")
    n = x.shape[0]
    need = int(lib().bigcn_gat_layer_workspace_bytes(n, layer.d_in, layer.d_out, int(heads)))
    workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=x.device)
    out = torch.empty((n, layer.d_out), dtype=torch.float32, device=x.device)
    _check(lib().bigcn_gat_layer(plan.handle, _ptr(row_ptr), _ptr(col_idx), n, _ptr(x), x.stride(0),
                                 _ptr(layer.bn_shift), _ptr(layer.bn_mul), _ptr(layer.w_bits), _ptr(layer.alpha),
                                 layer.w_bits.stride(0), layer.d_in, layer.d_out, int(heads), _ptr(a_src),
                                 _ptr(a_dst), float(negative_slope), _ptr(out), out.stride(0), _ptr(workspace),
                                 workspace.numel(), _stream()), "bigcn_gat_layer")
    return out


class BiGCN:
    """Graph + packed layers + workspace, ready for repeated forward passes."""

    def __init__(self, row_ptr: torch.Tensor, col_idx: torch.Tensor, weights: Sequence[torch.Tensor],
                 bn: Optional[Sequence[Optional[Tuple[torch.Tensor, torch.Tensor]]]] = None,
                 validate: bool = True):
        self.row_ptr, self.col_idx = row_ptr, col_idx
        self.n = row_ptr.numel() - 1
        self.plan = Plan(row_ptr, col_idx, validate=validate)
        self.dinv_sqrt, _ = bigcn_gcn_norm(row_ptr, col_idx)
        bn = list(bn) if bn is not None else [None] * len(weights)
        self.layers: List[Layer] = []
        for w, p in zip(weights, bn):
            shift, mul = p if p is not None else (None, None)
            self.layers.append(Layer.from_weight(w, shift, mul))
        need = bigcn_forward_workspace_bytes(self.n, self.layers)
        self.workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=row_ptr.device)
        self.logits = torch.empty((self.n, self.layers[-1].d_out), dtype=torch.float32,
                                  device=row_ptr.device)

    def forward(self, x: torch.Tensor, profile: Optional[Profile] = None) -> torch.Tensor:
        return bigcn_forward(self.plan, self.row_ptr, self.col_idx, self.dinv_sqrt, x, self.layers,
                             self.workspace, self.logits, profile)


# ------------------------------------------------------------------------------------------
# Bi-GraphSAGE (mean aggregator)
# ------------------------------------------------------------------------------------------
def bigcn_mean_norm(row_ptr: torch.Tensor) -> torch.Tensor:
    """``1/|N_i|`` per CSR row (0 for an empty row)."""
    _dev(row_ptr, torch.int64, "row_ptr")
    n = row_ptr.numel() - 1
    inv_deg = torch.empty((n,), dtype=torch.float32, device=row_ptr.device)
    _check(lib().bigcn_mean_norm(_ptr(row_ptr), n, _ptr(inv_deg), _stream()), "bigcn_mean_norm")
    return inv_deg


class SageLayer:
    """Device-resident parameters of one binarised mean-aggregator layer."""

    def __init__(self, w_self_bits: torch.Tensor, alpha_self: torch.Tensor, w_nbr_bits: torch.Tensor,
                 alpha_nbr: torch.Tensor, d_in: int, d_out: int,
                 bn_shift: Optional[torch.Tensor] = None, bn_mul: Optional[torch.Tensor] = None):
        self.w_self_bits = _dev(w_self_bits, torch.int64, "w_self_bits")
        self.alpha_self = _dev(alpha_self, torch.float32, "alpha_self")
        self.w_nbr_bits = _dev(w_nbr_bits, torch.int64, "w_nbr_bits")
        self.alpha_nbr = _dev(alpha_nbr, torch.float32, "alpha_nbr")
        if self.w_self_bits.stride(0) != self.w_nbr_bits.stride(0):
            raise ValueError("both packed weight matrices must share one row stride")
        self.d_in, self.d_out = int(d_in), int(d_out)
        self.bn_shift = None if bn_shift is None else _dev(bn_shift, torch.float32, "bn_shift").contiguous()
        self.bn_mul = None if bn_mul is None else _dev(bn_mul, torch.float32, "bn_mul").contiguous()

    @classmethod
    def from_weights(cls, w_self: torch.Tensor, w_nbr: torch.Tensor, bn_shift=None, bn_mul=None
                     ) -> "SageLayer":
        if w_self.shape != w_nbr.shape:
            raise ValueError("W_theta and W_n must have the same shape")
        bits_s, alpha_s = pack_weight(w_self)
        bits_n, alpha_n = pack_weight(w_nbr)
        return cls(bits_s, alpha_s, bits_n, alpha_n, w_self.shape[0], w_self.shape[1], bn_shift, bn_mul)

    def desc(self) -> SageLayerDesc:
        return SageLayerDesc(_ptr(self.w_self_bits), _ptr(self.alpha_self), _ptr(self.w_nbr_bits),
                             _ptr(self.alpha_nbr), self.d_in, self.d_out, self.w_nbr_bits.stride(0),
                             _ptr(self.bn_shift), _ptr(self.bn_mul))


def _sage_descs(layers: Sequence[SageLayer]):
    return (SageLayerDesc * len(layers))(*[l.desc() for l in layers])


def bigcn_sage_forward_workspace_bytes(n: int, layers: Sequence[SageLayer]) -> int:
    return int(lib().bigcn_sage_forward_workspace_bytes(int(n), _sage_descs(layers), len(layers)))


def bigcn_sage_forward(plan: Plan, row_ptr: torch.Tensor, col_idx: torch.Tensor, inv_deg: torch.Tensor,
                       x: torch.Tensor, layers: Sequence[SageLayer],
                       workspace: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                       profile: Optional[Profile] = None) -> torch.Tensor:
    """L-layer fused Bi-GraphSAGE forward; returns fp32 h^(L) (n, d_out of the last layer)."""
    _dev(x, torch.float32, "x")
    if x.dim() != 2 or (x.shape[1] > 1 and x.stride(1) != 1):
        raise ValueError("x must be a row-major matrix")
    n = x.shape[0]
    descs = _sage_descs(layers)
    if workspace is None:
        need = bigcn_sage_forward_workspace_bytes(n, layers)
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=x.device)
    if out is None:
        out = torch.empty((n, layers[-1].d_out), dtype=torch.float32, device=x.device)
    args = (plan.handle, _ptr(row_ptr), _ptr(col_idx), _ptr(inv_deg), n, _ptr(x), x.stride(0), descs,
            len(layers), _ptr(out), out.stride(0), _ptr(workspace), workspace.numel(), _stream())
    if profile is None:
        _check(lib().bigcn_sage_forward(*args), "bigcn_sage_forward")
    else:
        _check(lib().bigcn_sage_forward_profiled(*args, profile.handle), "bigcn_sage_forward_profiled")
    return out


class BiGraphSAGE:
    """Neighbour-list graph + packed layer pairs + workspace, ready for repeated forward passes."""

    def __init__(self, row_ptr: torch.Tensor, col_idx: torch.Tensor,
                 weights: Sequence[Tuple[torch.Tensor, torch.Tensor]],
                 bn: Optional[Sequence[Optional[Tuple[torch.Tensor, torch.Tensor]]]] = None,
                 validate: bool = True):
        self.row_ptr, self.col_idx = row_ptr, col_idx
        self.n = row_ptr.numel() - 1
        self.plan = Plan(row_ptr, col_idx, validate=VALIDATE_NEIGHBOURS if validate else VALIDATE_NONE)
        self.inv_deg = bigcn_mean_norm(row_ptr)
        bn = list(bn) if bn is not None else [None] * len(weights)
        self.layers: List[SageLayer] = []
        for (w_self, w_nbr), p in zip(weights, bn):
            shift, mul = p if p is not None else (None, None)
            self.layers.append(SageLayer.from_weights(w_self, w_nbr, shift, mul))
        need = bigcn_sage_forward_workspace_bytes(self.n, self.layers)
        self.workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=row_ptr.device)
        self.out = torch.empty((self.n, self.layers[-1].d_out), dtype=torch.float32,
                               device=row_ptr.device)

    def forward(self, x: torch.Tensor, profile: Optional[Profile] = None) -> torch.Tensor:
        return bigcn_sage_forward(self.plan, self.row_ptr, self.col_idx, self.inv_deg, x, self.layers,
                                  self.workspace, self.out, profile)
