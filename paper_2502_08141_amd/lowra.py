"""Thin Python binding of the C-ABI HIP library (include/lowra.h): argument marshalling only.

Functions carry the names of the C entry points.  Tensors are torch CUDA (ROCm) tensors used as
device memory; every step of the path runs in the library's kernels on torch's current stream.
There is no CPU fallback: a missing library or a failing call raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblowra_hip.so")
_lib = None

OK, INVALID_ARG, UNSUPPORTED, MISALIGNED, WORKSPACE_TOO_SMALL, HIP_ERROR, OUT_OF_MEMORY = range(7)
STATIC_SCRATCH_BYTES = 4 << 20
OP_LINEAR_FWD, OP_LINEAR_BWD_INPUT, OP_ADAPTER_GRADS, OP_LOFTQ_INIT = 0, 1, 2, 3
OUT_BF16, OUT_FP32 = 0, 1
PATH_AUTO, PATH_GEMV, PATH_GEMM, PATH_GEMV_GENERAL = 0, 1, 2, 3
SCALE_FP32, SCALE_BF16 = 0, 1

SYMBOLS = [
    "lowra_status_string", "lowra_plan_rows", "lowra_layout_create", "lowra_layout_destroy", "lowra_layout_set_scale_dtype",
    "lowra_packed_bytes", "lowra_workspace_bytes", "lowra_quantize", "lowra_quantize_batch", "lowra_dequantize",
    "lowra_linear_fwd", "lowra_linear_fwd_static", "lowra_linear_bwd_input", "lowra_set_linear_path", "lowra_set_fwd_tiling", "lowra_plan_fwd_tiling", "lowra_set_kernel_timer",
    "lowra_learn_tables", "lowra_average_thresholds", "lowra_channel_mse", "lowra_assign_precisions",
    "lowra_adapter_grads", "lowra_linear_side_product", "lowra_adapter_grads_from_side", "lowra_loftq_init",
    "lowra_fwd_batch_workspace_bytes", "lowra_fwd_batch_create", "lowra_fwd_batch_run", "lowra_fwd_batch_destroy",
    "lowra_bwd_batch_workspace_bytes", "lowra_bwd_batch_create", "lowra_bwd_batch_run", "lowra_bwd_batch_destroy",
    "lowra_measure_copy", "lowra_measure_read", "lowra_measure_mfma", "lowra_measure_mfma_random",
]


class FwdItem(C.Structure):
    """lowra_fwd_item: one matrix of a batched small-token forward (device pointers)."""
    _fields_ = [("layout", C.c_void_p), ("packed", C.c_void_p), ("absmax", C.c_void_p), ("x", C.c_void_p),
                ("A", C.c_void_p), ("B", C.c_void_p), ("y", C.c_void_p)]


class LowraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def lib() -> C.CDLL:
    """Load liblowra_hip.so (built by paper_2502_08141_amd.build); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2502_08141_amd.build` first")
        L = C.CDLL(LIB_PATH)
        vp, u8p, f32p, u16p = C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p
        L.lowra_status_string.restype = C.c_char_p
        L.lowra_status_string.argtypes = [C.c_int]
        L.lowra_plan_rows.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.lowra_layout_create.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int,
                                          C.c_void_p, C.POINTER(C.c_void_p)]
        L.lowra_layout_destroy.restype = None
        L.lowra_layout_destroy.argtypes = [vp]
        L.lowra_packed_bytes.restype = C.c_size_t
        L.lowra_packed_bytes.argtypes = [vp]
        L.lowra_workspace_bytes.restype = C.c_size_t
        L.lowra_workspace_bytes.argtypes = [vp, C.c_int, C.c_int, C.c_int]
        L.lowra_layout_set_scale_dtype.argtypes = [vp, C.c_int]
        L.lowra_quantize.argtypes = [vp, f32p, f32p, u8p, f32p, vp]
        L.lowra_quantize_batch.argtypes = [C.c_int, vp, vp, vp, vp, vp, vp]
        L.lowra_dequantize.argtypes = [vp, u8p, f32p, f32p, C.c_int, vp, vp]
        lin = [vp, u8p, f32p, f32p, u16p, C.c_int, u16p, u16p, C.c_int, C.c_float, u16p, vp, C.c_size_t, vp]
        L.lowra_linear_fwd.argtypes = lin
        L.lowra_linear_bwd_input.argtypes = lin
        L.lowra_linear_fwd_static.argtypes = lin[:11] + [vp]
        L.lowra_learn_tables.argtypes = [vp, f32p, f32p, f32p, C.c_int, f32p, f32p, f32p, vp]
        L.lowra_average_thresholds.argtypes = [vp, f32p, vp]
        L.lowra_adapter_grads.argtypes = [vp, u16p, u16p, C.c_int, u16p, u16p, C.c_int, C.c_float, f32p, f32p, vp, C.c_size_t, vp]
        L.lowra_linear_side_product.argtypes = [vp, C.c_int, C.c_int, C.c_int, vp]
        L.lowra_linear_side_product.restype = C.c_void_p
        L.lowra_adapter_grads_from_side.argtypes = [vp, u16p, u16p, C.c_int, C.c_int, u16p, u16p, f32p, f32p, vp, C.c_size_t, vp]
        L.lowra_loftq_init.argtypes = [vp, f32p, f32p, f32p, C.c_int, C.c_int, C.c_int, u16p, u8p, f32p, u16p, u16p, vp, C.c_size_t, vp]
        L.lowra_fwd_batch_workspace_bytes.restype = C.c_size_t
        L.lowra_fwd_batch_workspace_bytes.argtypes = [C.c_int, C.c_void_p, C.c_int]
        L.lowra_fwd_batch_create.argtypes = [C.c_int, C.c_void_p, f32p, C.c_int, C.c_int, C.c_float, vp, C.c_size_t, C.c_void_p]
        L.lowra_fwd_batch_run.argtypes = [vp, vp]
        L.lowra_fwd_batch_destroy.restype = None
        L.lowra_fwd_batch_destroy.argtypes = [vp]
        L.lowra_bwd_batch_workspace_bytes.restype = C.c_size_t
        L.lowra_bwd_batch_workspace_bytes.argtypes = [C.c_int, C.c_void_p, C.c_int, C.c_int]
        L.lowra_bwd_batch_create.argtypes = [C.c_int, C.c_void_p, f32p, C.c_int, C.c_int, C.c_float, vp, C.c_size_t, C.c_void_p]
        L.lowra_bwd_batch_run.argtypes = [vp, vp]
        L.lowra_bwd_batch_destroy.restype = None
        L.lowra_bwd_batch_destroy.argtypes = [vp]
        L.lowra_channel_mse.argtypes = [C.c_int, C.c_int, f32p, f32p, f32p, f32p, vp]
        L.lowra_assign_precisions.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_double, C.c_void_p]
        L.lowra_measure_copy.argtypes = [vp, vp, C.c_size_t, vp]
        L.lowra_measure_read.argtypes = [vp, C.c_size_t, vp, vp]
        L.lowra_measure_mfma.argtypes = [C.c_int, C.c_int, vp, C.POINTER(C.c_double), vp]
        L.lowra_measure_mfma_random.argtypes = [C.c_int, C.c_int, vp, C.POINTER(C.c_double), vp]
        L.lowra_set_linear_path.argtypes = [C.c_int]
        L.lowra_set_fwd_tiling.argtypes = [C.c_int, C.c_int, C.c_int]
        L.lowra_plan_fwd_tiling.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int), C.POINTER(C.c_int)]
        L.lowra_set_kernel_timer.argtypes = [vp, vp]
        _lib = L
    return _lib


def status_string(st: int) -> str:
    return lib().lowra_status_string(int(st)).decode()


def _check(st: int, where: str):
    if st != OK:
        raise LowraError(st, where)


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _dev(t: torch.Tensor, dtype, name: str):
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError(f"{name}: need a contiguous {dtype} device tensor")
    return t


def lowra_plan_rows(K: int, bits) -> np.ndarray:
    """Host only: byte offset of every channel's row in the packed buffer, int64 [N+1]."""
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    off = np.zeros(bits.size + 1, dtype=np.int64)
    _check(lib().lowra_plan_rows(bits.size, int(K), 64, bits.ctypes.data, off.ctypes.data), "lowra_plan_rows")
    return off


class Layout:
    """Owner of a lowra_layout handle (lowra_layout_create / lowra_layout_destroy)."""

    def __init__(self, K: int, bits, codebook_id, codebook_bits, group: int = 64):
        self.bits = np.ascontiguousarray(bits, dtype=np.uint8)
        self.cb = np.ascontiguousarray(codebook_id, dtype=np.int32)
        self.cb_bits = np.ascontiguousarray(codebook_bits, dtype=np.uint8)
        if self.cb.shape != self.bits.shape:
            raise ValueError("bits and codebook_id must have the same length")
        self.N, self.K, self.C = int(self.bits.size), int(K), int(self.cb_bits.size)
        h = C.c_void_p()
        st = lib().lowra_layout_create(self.N, self.K, int(group), self.bits.ctypes.data, self.cb.ctypes.data,
                                       self.C, self.cb_bits.ctypes.data, C.byref(h))
        _check(st, "lowra_layout_create")
        self.handle = h

        self.scale_dtype = torch.float32

    def set_scale_dtype(self, dtype):
        """torch.float32 (default) or torch.bfloat16: the type of the stored group scales (lowra_layout_set_scale_dtype)."""
        code = {torch.float32: SCALE_FP32, torch.bfloat16: SCALE_BF16}[dtype]
        _check(lib().lowra_layout_set_scale_dtype(self.handle, code), "lowra_layout_set_scale_dtype")
        self.scale_dtype = dtype
        return self

    @property
    def packed_bytes(self) -> int:
        return int(lib().lowra_packed_bytes(self.handle))

    def workspace_bytes(self, op: int, M: int, r: int) -> int:
        return int(lib().lowra_workspace_bytes(self.handle, int(op), int(M), int(r)))

    def close(self):
        if getattr(self, "handle", None):
            lib().lowra_layout_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


lowra_layout_create = Layout


def lowra_quantize(layout: Layout, W, thresholds, packed=None, absmax=None):
    """W [N,K] fp32, thresholds [C,16] fp32 -> (packed uint8 [packed_bytes], absmax fp32 [N,K/64])."""
    _dev(W, torch.float32, "W"); _dev(thresholds, torch.float32, "thresholds")
    if tuple(W.shape) != (layout.N, layout.K) or tuple(thresholds.shape) != (layout.C, 16):
        raise ValueError("shape mismatch")
    if packed is None:
        packed = torch.empty(layout.packed_bytes, dtype=torch.uint8, device=W.device)
    if absmax is None:
        absmax = torch.empty((layout.N, layout.K // 64), dtype=layout.scale_dtype, device=W.device)
    _dev(packed, torch.uint8, "packed"); _dev(absmax, layout.scale_dtype, "absmax")
    if packed.numel() != layout.packed_bytes or absmax.numel() != layout.N * (layout.K // 64):
        raise ValueError("output size mismatch")
    _check(lib().lowra_quantize(layout.handle, _ptr(W), _ptr(thresholds), _ptr(packed), _ptr(absmax), _stream()),
           "lowra_quantize")
    return packed, absmax


def lowra_quantize_batch(layouts, Ws, thresholds, packed=None, absmax=None):
    """The matrices of a list in as few launches as possible: lists of what lowra_quantize takes -> (list of packed, list of absmax)."""
    n = len(layouts)
    if len(Ws) != n or len(thresholds) != n:
        raise ValueError("list lengths differ")
    packed = [None] * n if packed is None else list(packed)
    absmax = [None] * n if absmax is None else list(absmax)
    if len(packed) != n or len(absmax) != n:
        raise ValueError("list lengths differ")
    for i, (lay, W, thr) in enumerate(zip(layouts, Ws, thresholds)):
        _dev(W, torch.float32, "W"); _dev(thr, torch.float32, "thresholds")
        if tuple(W.shape) != (lay.N, lay.K) or tuple(thr.shape) != (lay.C, 16):
            raise ValueError("shape mismatch")
        if packed[i] is None:
            packed[i] = torch.empty(lay.packed_bytes, dtype=torch.uint8, device=W.device)
        if absmax[i] is None:
            absmax[i] = torch.empty((lay.N, lay.K // 64), dtype=lay.scale_dtype, device=W.device)
        _dev(packed[i], torch.uint8, "packed"); _dev(absmax[i], lay.scale_dtype, "absmax")
        if packed[i].numel() != lay.packed_bytes or absmax[i].numel() != lay.N * (lay.K // 64):
            raise ValueError("output size mismatch")
    arr = lambda values: (C.c_void_p * n)(*values)
    _check(lib().lowra_quantize_batch(n, arr([lay.handle for lay in layouts]), arr([_ptr(W) for W in Ws]),
                                      arr([_ptr(t) for t in thresholds]), arr([_ptr(p) for p in packed]),
                                      arr([_ptr(a) for a in absmax]), _stream()), "lowra_quantize_batch")
    return packed, absmax


def _state(layout, packed, absmax, mappings):
    _dev(packed, torch.uint8, "packed"); _dev(absmax, layout.scale_dtype, "absmax"); _dev(mappings, torch.float32, "mappings")
    if packed.numel() != layout.packed_bytes or absmax.numel() != layout.N * (layout.K // 64) or \
            tuple(mappings.shape) != (layout.C, 16):
        raise ValueError("quantized state does not match the layout")


def lowra_dequantize(layout: Layout, packed, absmax, mappings, out_dtype=torch.bfloat16, out=None):
    """-> What [N,K] in bf16 (default) or fp32."""
    _state(layout, packed, absmax, mappings)
    code = {torch.bfloat16: OUT_BF16, torch.float32: OUT_FP32}[out_dtype]
    if out is None:
        out = torch.empty((layout.N, layout.K), dtype=out_dtype, device=packed.device)
    _dev(out, out_dtype, "out")
    if out.numel() != layout.N * layout.K:
        raise ValueError("output size mismatch")
    _check(lib().lowra_dequantize(layout.handle, _ptr(packed), _ptr(absmax), _ptr(mappings), code, _ptr(out), _stream()),
           "lowra_dequantize")
    return out


def _linear(fn, name, op, layout, packed, absmax, mappings, act, act_cols, out_cols, A, B, s, out, workspace):
    _state(layout, packed, absmax, mappings)
    _dev(act, torch.bfloat16, "activation")
    if act.dim() != 2 or act.shape[1] != act_cols:
        raise ValueError("activation shape mismatch")
    M = int(act.shape[0])
    r = 0
    if A is not None and B is not None and A.shape[0] > 0:
        _dev(A, torch.bfloat16, "A"); _dev(B, torch.bfloat16, "B")
        r = int(A.shape[0])
        if tuple(A.shape) != (r, layout.K) or tuple(B.shape) != (layout.N, r):
            raise ValueError("LoRA operand shape mismatch")
    else:
        A = B = None
    if out is None:
        out = torch.empty((M, out_cols), dtype=torch.bfloat16, device=act.device)
    _dev(out, torch.bfloat16, "out")
    if tuple(out.shape) != (M, out_cols):
        raise ValueError("output shape mismatch")
    need = layout.workspace_bytes(op, M, r)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=act.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(fn(layout.handle, _ptr(packed), _ptr(absmax), _ptr(mappings), _ptr(act), M, _ptr(A), _ptr(B), r,
              C.c_float(s), _ptr(out), _ptr(workspace), C.c_size_t(ws_bytes), _stream()), name)
    return out


def lowra_linear_fwd(layout: Layout, packed, absmax, mappings, x, A, B, s, y=None, workspace=None):
    """y [M,N] bf16 = x What^T + s (x A^T) B^T."""
    return _linear(lib().lowra_linear_fwd, "lowra_linear_fwd", OP_LINEAR_FWD, layout, packed, absmax, mappings,
                   x, layout.K, layout.N, A, B, s, y, workspace)


def lowra_linear_fwd_static(layout: Layout, packed, absmax, mappings, x, A, B, s, y):
    """lowra_linear_fwd without a workspace argument (the library's static scratch); `y` [M,N] bf16 is the
    caller's: nothing is allocated here or in the library."""
    _state(layout, packed, absmax, mappings)
    _dev(x, torch.bfloat16, "x"); _dev(y, torch.bfloat16, "y")
    M = int(x.shape[0])
    if tuple(x.shape) != (M, layout.K) or tuple(y.shape) != (M, layout.N):
        raise ValueError("shape mismatch")
    r = 0
    if A is not None and B is not None and A.shape[0] > 0:
        _dev(A, torch.bfloat16, "A"); _dev(B, torch.bfloat16, "B")
        r = int(A.shape[0])
        if tuple(A.shape) != (r, layout.K) or tuple(B.shape) != (layout.N, r):
            raise ValueError("LoRA operand shape mismatch")
    else:
        A = B = None
    _check(lib().lowra_linear_fwd_static(layout.handle, _ptr(packed), _ptr(absmax), _ptr(mappings), _ptr(x), M, _ptr(A),
                                         _ptr(B), r, C.c_float(s), _ptr(y), _stream()), "lowra_linear_fwd_static")
    return y


def lowra_linear_bwd_input(layout: Layout, packed, absmax, mappings, dY, A, B, s, dX=None, workspace=None):
    """dX [M,K] bf16 = dY What + s (dY B) A."""
    return _linear(lib().lowra_linear_bwd_input, "lowra_linear_bwd_input", OP_LINEAR_BWD_INPUT, layout, packed,
                   absmax, mappings, dY, layout.N, layout.K, A, B, s, dX, workspace)


def lowra_learn_tables(layout: Layout, W, init_thresholds, init_mappings, iterations: int = 2):
    """W [N,K] fp32, init tables [C,16] fp32 -> (thresholds [N,16], mappings [N,16], mse [N,iterations+1]), all fp32."""
    _dev(W, torch.float32, "W"); _dev(init_thresholds, torch.float32, "init_thresholds"); _dev(init_mappings, torch.float32, "init_mappings")
    if tuple(W.shape) != (layout.N, layout.K) or tuple(init_thresholds.shape) != (layout.C, 16) or \
            tuple(init_mappings.shape) != (layout.C, 16):
        raise ValueError("shape mismatch")
    thr = torch.empty((layout.N, 16), dtype=torch.float32, device=W.device)
    mp = torch.empty((layout.N, 16), dtype=torch.float32, device=W.device)
    mse = torch.empty((layout.N, int(iterations) + 1), dtype=torch.float32, device=W.device)
    _check(lib().lowra_learn_tables(layout.handle, _ptr(W), _ptr(init_thresholds), _ptr(init_mappings), int(iterations),
                                    _ptr(thr), _ptr(mp), _ptr(mse), _stream()), "lowra_learn_tables")
    return thr, mp, mse


def lowra_average_thresholds(layout: Layout, thresholds):
    """In place on thresholds [N,16] fp32: per width, the mean over the channels of that width."""
    _dev(thresholds, torch.float32, "thresholds")
    if tuple(thresholds.shape) != (layout.N, 16):
        raise ValueError("shape mismatch")
    _check(lib().lowra_average_thresholds(layout.handle, _ptr(thresholds), _stream()), "lowra_average_thresholds")
    return thresholds


def lowra_adapter_grads(layout: Layout, x, dY, A, B, s, workspace=None):
    """x [M,K], dY [M,N], A [r,K], B [N,r] bf16 -> (dA fp32 [r,K], dB fp32 [N,r])."""
    for t, nme in ((x, "x"), (dY, "dY"), (A, "A"), (B, "B")):
        _dev(t, torch.bfloat16, nme)
    M, r = int(x.shape[0]), int(A.shape[0])
    if tuple(x.shape) != (M, layout.K) or tuple(dY.shape) != (M, layout.N) or tuple(A.shape) != (r, layout.K) or \
            tuple(B.shape) != (layout.N, r):
        raise ValueError("shape mismatch")
    need = layout.workspace_bytes(OP_ADAPTER_GRADS, M, r)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    dA = torch.empty((r, layout.K), dtype=torch.float32, device=x.device)
    dB = torch.empty((layout.N, r), dtype=torch.float32, device=x.device)
    _check(lib().lowra_adapter_grads(layout.handle, _ptr(x), _ptr(dY), M, _ptr(A), _ptr(B), r, float(s), _ptr(dA), _ptr(dB),
                                     _ptr(workspace), workspace.numel(), _stream()), "lowra_adapter_grads")
    return dA, dB


def lowra_linear_side_product(layout: Layout, op: int, M: int, r: int, workspace):
    """The rank-r intermediate a finished linear call left in `workspace`: a bf16 [M,64] view of it, or None."""
    _dev(workspace, torch.uint8, "workspace")
    p = lib().lowra_linear_side_product(layout.handle, int(op), int(M), int(r), _ptr(workspace))
    if not p:
        return None
    off = int(p) - workspace.data_ptr()
    return workspace[off:off + M * 64 * 2].view(torch.bfloat16).view(M, 64)


def lowra_adapter_grads_from_side(layout: Layout, x, dY, r, st, su, workspace=None):
    """x [M,K], dY [M,N], st = s x A^T, su = s dY B (bf16 [M,64], from lowra_linear_side_product) -> (dA fp32 [r,K], dB fp32 [N,r])."""
    for t, nme in ((x, "x"), (dY, "dY"), (st, "st"), (su, "su")):
        _dev(t, torch.bfloat16, nme)
    M, r = int(x.shape[0]), int(r)
    if tuple(x.shape) != (M, layout.K) or tuple(dY.shape) != (M, layout.N) or tuple(st.shape) != (M, 64) or tuple(su.shape) != (M, 64):
        raise ValueError("shape mismatch")
    need = layout.workspace_bytes(OP_ADAPTER_GRADS, M, r)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    dA = torch.empty((r, layout.K), dtype=torch.float32, device=x.device)
    dB = torch.empty((layout.N, r), dtype=torch.float32, device=x.device)
    _check(lib().lowra_adapter_grads_from_side(layout.handle, _ptr(x), _ptr(dY), M, r, _ptr(st), _ptr(su), _ptr(dA), _ptr(dB),
                                               _ptr(workspace), workspace.numel(), _stream()), "lowra_adapter_grads_from_side")
    return dA, dB


def lowra_loftq_init(layout: Layout, W, thresholds, mappings, r, omega, steps=5, power_iterations=16, workspace=None):
    """W fp32 [N,K], omega bf16 [r,K] (random start) -> (packed, absmax, A bf16 [r,K], B bf16 [N,r])."""
    _dev(W, torch.float32, "W"); _dev(thresholds, torch.float32, "thresholds"); _dev(mappings, torch.float32, "mappings")
    if tuple(W.shape) != (layout.N, layout.K):
        raise ValueError("W shape mismatch")
    r = int(r)
    if r > 0:
        _dev(omega, torch.bfloat16, "omega")
        if tuple(omega.shape) != (r, layout.K):
            raise ValueError("omega shape mismatch")
    need = layout.workspace_bytes(OP_LOFTQ_INIT, 0, r) if r > 0 else 0
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=W.device)
    packed = torch.empty(max(layout.packed_bytes, 1), dtype=torch.uint8, device=W.device)[:layout.packed_bytes]
    absmax = torch.empty((layout.N, layout.K // 64), dtype=torch.float32, device=W.device)
    A = torch.empty((r, layout.K), dtype=torch.bfloat16, device=W.device)
    B = torch.empty((layout.N, r), dtype=torch.bfloat16, device=W.device)
    _check(lib().lowra_loftq_init(layout.handle, _ptr(W), _ptr(thresholds), _ptr(mappings), r, int(steps), int(power_iterations),
                                  _ptr(omega) if r > 0 else C.c_void_p(0), _ptr(packed), _ptr(absmax), _ptr(A), _ptr(B),
                                  _ptr(workspace), workspace.numel(), _stream()), "lowra_loftq_init")
    return packed, absmax, A, B


class FwdBatch:
    """Several small-token forwards (M <= 16) as one run.  `items`: list of (layout, packed, absmax, x, A, B)
    with A = B = None when r == 0; the outputs y[i] ([M, N_i] bf16) are allocated here.  Every tensor is kept
    alive by the object: the library holds their addresses."""

    def __init__(self, items, mappings, s, workspace=None):
        if not items:
            raise ValueError("empty batch")
        _dev(mappings, torch.float32, "mappings")
        M = int(items[0][3].shape[0])
        r = 0 if items[0][4] is None else int(items[0][4].shape[0])
        self.y, self._keep = [], [mappings]
        arr = (FwdItem * len(items))()
        for i, (layout, packed, absmax, x, A, B) in enumerate(items):
            _dev(packed, torch.uint8, "packed"); _dev(absmax, layout.scale_dtype, "absmax"); _dev(x, torch.bfloat16, "x")
            if tuple(x.shape) != (M, layout.K) or packed.numel() != layout.packed_bytes or absmax.numel() != layout.N * (layout.K // 64):
                raise ValueError(f"item {i}: shape mismatch")
            if r:
                _dev(A, torch.bfloat16, "A"); _dev(B, torch.bfloat16, "B")
                if tuple(A.shape) != (r, layout.K) or tuple(B.shape) != (layout.N, r):
                    raise ValueError(f"item {i}: LoRA shape mismatch")
            y = torch.empty((M, layout.N), dtype=torch.bfloat16, device=x.device)
            arr[i] = FwdItem(layout.handle.value if isinstance(layout.handle, C.c_void_p) else layout.handle,
                             packed.data_ptr(), absmax.data_ptr(), x.data_ptr(),
                             A.data_ptr() if r else 0, B.data_ptr() if r else 0, y.data_ptr())
            self.y.append(y)
            self._keep += [layout, packed, absmax, x, A, B]
        need = int(lib().lowra_fwd_batch_workspace_bytes(len(items), C.addressof(arr), r))
        if workspace is None:
            workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=mappings.device)
        self._keep.append(workspace)
        self.handle = C.c_void_p()
        _check(lib().lowra_fwd_batch_create(len(items), C.addressof(arr), _ptr(mappings), M, r, float(s), _ptr(workspace),
                                            workspace.numel(), C.addressof(self.handle)), "lowra_fwd_batch_create")

    def run(self):
        _check(lib().lowra_fwd_batch_run(self.handle, _stream()), "lowra_fwd_batch_run")
        return self.y

    def close(self):
        if self.handle:
            lib().lowra_fwd_batch_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class BwdBatch:
    """Several small-token input gradients (M <= 16) as one run.  `items`: list of (layout, packed, absmax, dY, A, B)
    with A = B = None when r == 0; the outputs dX[i] ([M, K_i] bf16) are allocated here.  Every tensor is kept
    alive by the object: the library holds their addresses."""

    def __init__(self, items, mappings, s, workspace=None):
        if not items:
            raise ValueError("empty batch")
        _dev(mappings, torch.float32, "mappings")
        M = int(items[0][3].shape[0])
        r = 0 if items[0][4] is None else int(items[0][4].shape[0])
        self.dX, self._keep = [], [mappings]
        arr = (FwdItem * len(items))()          # same record: layout, packed, absmax, activations in, A, B, out
        for i, (layout, packed, absmax, dY, A, B) in enumerate(items):
            _dev(packed, torch.uint8, "packed"); _dev(absmax, layout.scale_dtype, "absmax"); _dev(dY, torch.bfloat16, "dY")
            if tuple(dY.shape) != (M, layout.N) or packed.numel() != layout.packed_bytes or absmax.numel() != layout.N * (layout.K // 64):
                raise ValueError(f"item {i}: shape mismatch")
            if r:
                _dev(A, torch.bfloat16, "A"); _dev(B, torch.bfloat16, "B")
                if tuple(A.shape) != (r, layout.K) or tuple(B.shape) != (layout.N, r):
                    raise ValueError(f"item {i}: LoRA shape mismatch")
            dX = torch.empty((M, layout.K), dtype=torch.bfloat16, device=dY.device)
            arr[i] = FwdItem(layout.handle.value if isinstance(layout.handle, C.c_void_p) else layout.handle,
                             packed.data_ptr(), absmax.data_ptr(), dY.data_ptr(),
                             A.data_ptr() if r else 0, B.data_ptr() if r else 0, dX.data_ptr())
            self.dX.append(dX)
            self._keep += [layout, packed, absmax, dY, A, B]
        need = int(lib().lowra_bwd_batch_workspace_bytes(len(items), C.addressof(arr), M, r))
        if workspace is None:
            workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=mappings.device)
        self._keep.append(workspace)
        self.handle = C.c_void_p()
        _check(lib().lowra_bwd_batch_create(len(items), C.addressof(arr), _ptr(mappings), M, r, float(s), _ptr(workspace),
                                            workspace.numel(), C.addressof(self.handle)), "lowra_bwd_batch_create")

    def run(self):
        _check(lib().lowra_bwd_batch_run(self.handle, _stream()), "lowra_bwd_batch_run")
        return self.dX

    def close(self):
        if self.handle:
            lib().lowra_bwd_batch_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def lowra_channel_mse(W, thresholds3, mappings3):
    """W [N,K] fp32, tables [3,16] fp32 (rows: 1, 2, 4 bits) -> mse fp32 [N,3]."""
    _dev(W, torch.float32, "W"); _dev(thresholds3, torch.float32, "thresholds3"); _dev(mappings3, torch.float32, "mappings3")
    if W.dim() != 2 or tuple(thresholds3.shape) != (3, 16) or tuple(mappings3.shape) != (3, 16):
        raise ValueError("shape mismatch")
    N, K = W.shape
    mse = torch.empty((N, 3), dtype=torch.float32, device=W.device)
    _check(lib().lowra_channel_mse(int(N), int(K), _ptr(W), _ptr(thresholds3), _ptr(mappings3), _ptr(mse), _stream()),
           "lowra_channel_mse")
    return mse


def lowra_assign_precisions(channel_params, mse, budget_bits_per_param: float) -> np.ndarray:
    """Host only: greedy budgeted assignment. channel_params int64 [N], mse fp32 [N,3] -> bits uint8 [N]."""
    params = np.ascontiguousarray(channel_params, dtype=np.int64)
    mse = np.ascontiguousarray(mse, dtype=np.float32)
    if mse.shape != (params.size, 3):
        raise ValueError("shape mismatch")
    bits = np.zeros(params.size, dtype=np.uint8)
    _check(lib().lowra_assign_precisions(int(params.size), params.ctypes.data, mse.ctypes.data, float(budget_bits_per_param),
                                         bits.ctypes.data), "lowra_assign_precisions")
    return bits


def lowra_set_linear_path(path: int):
    _check(lib().lowra_set_linear_path(int(path)), "lowra_set_linear_path")


def lowra_plan_fwd_tiling(N: int, M: int, compute_units: int = 256):
    """(rows_a, rows_b, cols_a) the forward GEMM's planner picks (host only)."""
    ra, rb, ca = C.c_int(), C.c_int(), C.c_int()
    _check(lib().lowra_plan_fwd_tiling(int(N), int(M), int(compute_units), C.byref(ra), C.byref(rb), C.byref(ca)), "lowra_plan_fwd_tiling")
    return ra.value, rb.value, ca.value


def lowra_set_fwd_tiling(rows_a: int = 0, rows_b: int = 0, cols_a: int = 0):
    _check(lib().lowra_set_fwd_tiling(int(rows_a), int(rows_b), int(cols_a)), "lowra_set_fwd_tiling")


def lowra_set_kernel_timer(start_event=None, stop_event=None):
    """Measurement hook: raw hipEvent_t handles (ints) recorded around the dominant kernel of linear calls."""
    _check(lib().lowra_set_kernel_timer(C.c_void_p(start_event or 0), C.c_void_p(stop_event or 0)),
           "lowra_set_kernel_timer")


def lowra_measure_copy(dst, src):
    """Measurement kernel: dst = src (uint8 device tensors of equal size, a multiple of 16 bytes)."""
    _check(lib().lowra_measure_copy(_ptr(dst), _ptr(src), C.c_size_t(src.numel() * src.element_size()), _stream()), "lowra_measure_copy")


def lowra_measure_read(src, out4):
    """Measurement kernel: stream src once."""
    _check(lib().lowra_measure_read(_ptr(src), C.c_size_t(src.numel() * src.element_size()), _ptr(out4), _stream()), "lowra_measure_read")


def lowra_measure_mfma(workgroups: int, iterations: int, out4, random_operands: bool = False) -> float:
    """Measurement kernel: a loop of independent bf16 MFMAs on registers (constant operands, or pseudo-random ones
    that change with every instruction); returns its flop count."""
    fl = C.c_double(0.0)
    fn = lib().lowra_measure_mfma_random if random_operands else lib().lowra_measure_mfma
    _check(fn(int(workgroups), int(iterations), _ptr(out4), C.byref(fl), _stream()), "lowra_measure_mfma")
    return float(fl.value)
