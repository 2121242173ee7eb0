"""ctypes face of the CPU oracle (oracle/lowra_oracle.c) -- test infrastructure.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this.
It takes and returns numpy arrays; bf16 tensors travel as uint16 bit patterns.
Every function names the step of the paper it runs (see the C file's header).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lowra_oracle.c")
_LIB = os.path.join(_HERE, "liblowra_oracle.so")
_lib = None

ERRORS = {1: "bad argument", 2: "bits not in {1,2,4}", 3: "bad table / table index",
          4: "non-finite weight", 5: "out of memory"}


def build() -> str:
    """Compile the oracle with gcc; FMA contraction and fast-math stay off so fp32 steps are IEEE."""
    cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-shared",
           "-fPIC", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
            build()
        _lib = C.CDLL(_LIB)
    return _lib


def _p(a, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def _chk(rc):
    if rc:
        raise ValueError(f"oracle: {ERRORS.get(rc, rc)}")


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def num_threads() -> int:
    return int(_load().lowra_oracle_num_threads())


def bf16_rne(f32: np.ndarray) -> np.ndarray:
    """D2 on an array: fp32 -> bf16 bit patterns, round to nearest even."""
    flat = _c(f32, np.float32).ravel()
    out = np.zeros(flat.size, dtype=np.uint16)
    _load().lowra_oracle_bf16_rne_array(C.c_size_t(flat.size), _p(flat, C.c_float), _p(out, C.c_uint16))
    return out.reshape(np.shape(f32))


def row_offsets(K: int, bits: np.ndarray) -> np.ndarray:
    """Q5 offsets: exclusive prefix sum of K*bits[n]/8 in channel order, int64 [N+1]."""
    bits = _c(bits, np.uint8)
    off = np.zeros(bits.size + 1, dtype=np.int64)
    _chk(_load().lowra_oracle_row_offsets(C.c_int(bits.size), C.c_int(K), _p(bits, C.c_uint8), _p(off, C.c_int64)))
    return off


def _scale_flag(scale_dtype):
    return {"fp32": 0, "bf16": 1}[scale_dtype]


def quantize_codes(W, bits, cb, thresholds, scale_dtype="fp32"):
    """Q1-Q4: returns (codes uint8 [N,K], absmax fp32 [N,K/64]).  scale_dtype "bf16": the scale is rounded to bf16
    after Q1 and used that way; the returned floats are then exactly representable in bf16."""
    W = _c(W, np.float32); bits = _c(bits, np.uint8); cb = _c(cb, np.int32)
    thresholds = _c(thresholds, np.float32)
    N, K = W.shape
    codes = np.zeros((N, K), dtype=np.uint8)
    absmax = np.zeros((N, K // 64), dtype=np.float32)
    _chk(_load().lowra_oracle_quantize_codes_s(C.c_int(N), C.c_int(K), _p(W, C.c_float), _p(bits, C.c_uint8),
                                               _p(cb, C.c_int32), C.c_int(thresholds.shape[0]),
                                               _p(thresholds, C.c_float), C.c_int(_scale_flag(scale_dtype)),
                                               _p(codes, C.c_uint8), _p(absmax, C.c_float)))
    return codes, absmax


def pack(codes, bits):
    """Q5: codes uint8 [N,K] -> packed uint8 [sum K*b/8]."""
    codes = _c(codes, np.uint8); bits = _c(bits, np.uint8)
    N, K = codes.shape
    packed = np.zeros(int(row_offsets(K, bits)[-1]), dtype=np.uint8)
    _chk(_load().lowra_oracle_pack(C.c_int(N), C.c_int(K), _p(bits, C.c_uint8), _p(codes, C.c_uint8), _p(packed, C.c_uint8)))
    return packed


def unpack(packed, bits, K):
    """Inverse of Q5: packed -> codes uint8 [N,K]."""
    packed = _c(packed, np.uint8); bits = _c(bits, np.uint8)
    N = bits.size
    assert packed.size == int(row_offsets(K, bits)[-1])
    codes = np.zeros((N, K), dtype=np.uint8)
    _chk(_load().lowra_oracle_unpack(C.c_int(N), C.c_int(K), _p(bits, C.c_uint8), _p(packed, C.c_uint8), _p(codes, C.c_uint8)))
    return codes


def quantize(W, bits, cb, thresholds, scale_dtype="fp32"):
    """Q1-Q5 (App. A.1): returns (packed uint8, absmax fp32 [N,K/64]); scale_dtype as in quantize_codes."""
    W = _c(W, np.float32); bits = _c(bits, np.uint8); cb = _c(cb, np.int32)
    thresholds = _c(thresholds, np.float32)
    N, K = W.shape
    packed = np.zeros(int(row_offsets(K, bits)[-1]), dtype=np.uint8)
    absmax = np.zeros((N, K // 64), dtype=np.float32)
    _chk(_load().lowra_oracle_quantize_s(C.c_int(N), C.c_int(K), _p(W, C.c_float), _p(bits, C.c_uint8),
                                         _p(cb, C.c_int32), C.c_int(thresholds.shape[0]), _p(thresholds, C.c_float),
                                         C.c_int(_scale_flag(scale_dtype)), _p(packed, C.c_uint8), _p(absmax, C.c_float)))
    return packed, absmax


def dequantize(packed, absmax, bits, cb, mappings, K, out_dtype="bf16"):
    """D1-D2 (App. A.2): returns uint16 bf16 bit patterns [N,K] (or fp32 when out_dtype='fp32')."""
    packed = _c(packed, np.uint8); absmax = _c(absmax, np.float32); bits = _c(bits, np.uint8)
    cb = _c(cb, np.int32); mappings = _c(mappings, np.float32)
    N = bits.size
    assert absmax.shape == (N, K // 64)
    assert packed.size == int(row_offsets(K, bits)[-1])
    code = {"bf16": 0, "fp32": 1}[out_dtype]
    out = np.zeros((N, K), dtype=np.uint16 if code == 0 else np.float32)
    _chk(_load().lowra_oracle_dequantize(C.c_int(N), C.c_int(K), _p(packed, C.c_uint8), _p(absmax, C.c_float),
                                         _p(bits, C.c_uint8), _p(cb, C.c_int32), C.c_int(mappings.shape[0]),
                                         _p(mappings, C.c_float), C.c_int(code), out.ctypes.data_as(C.c_void_p)))
    return out


def _lora(A, B, K, N):
    if A is None or B is None:
        return 0, np.zeros(1, np.uint16), np.zeros(1, np.uint16)
    A = _c(A, np.uint16); B = _c(B, np.uint16)
    r = A.shape[0]
    assert A.shape == (r, K) and B.shape == (N, r)
    return r, A, B


def linear_fwd(packed, absmax, bits, cb, mappings, x, A, B, s):
    """L1: y = x What^T + s (x A^T) B^T in fp64.  x, A, B: uint16 bf16 bit patterns."""
    x = _c(x, np.uint16)
    M, K = x.shape
    bits = _c(bits, np.uint8); N = bits.size
    packed = _c(packed, np.uint8); absmax = _c(absmax, np.float32)
    cb = _c(cb, np.int32); mappings = _c(mappings, np.float32)
    r, A, B = _lora(A, B, K, N)
    y = np.zeros((M, N), dtype=np.float64)
    _chk(_load().lowra_oracle_linear_fwd(C.c_int(N), C.c_int(K), _p(packed, C.c_uint8), _p(absmax, C.c_float),
                                         _p(bits, C.c_uint8), _p(cb, C.c_int32), C.c_int(mappings.shape[0]),
                                         _p(mappings, C.c_float), C.c_int(M), _p(x, C.c_uint16), C.c_int(r),
                                         _p(A, C.c_uint16), _p(B, C.c_uint16), C.c_float(s), _p(y, C.c_double)))
    return y


def linear_bwd_input(packed, absmax, bits, cb, mappings, dY, A, B, s, K):
    """L2: dX = dY What + s (dY B) A in fp64.  dY, A, B: uint16 bf16 bit patterns."""
    dY = _c(dY, np.uint16)
    M, N = dY.shape
    bits = _c(bits, np.uint8)
    assert bits.size == N
    packed = _c(packed, np.uint8); absmax = _c(absmax, np.float32)
    cb = _c(cb, np.int32); mappings = _c(mappings, np.float32)
    r, A, B = _lora(A, B, K, N)
    dX = np.zeros((M, K), dtype=np.float64)
    _chk(_load().lowra_oracle_linear_bwd_input(C.c_int(N), C.c_int(K), _p(packed, C.c_uint8), _p(absmax, C.c_float),
                                               _p(bits, C.c_uint8), _p(cb, C.c_int32), C.c_int(mappings.shape[0]),
                                               _p(mappings, C.c_float), C.c_int(M), _p(dY, C.c_uint16), C.c_int(r),
                                               _p(A, C.c_uint16), _p(B, C.c_uint16), C.c_float(s), _p(dX, C.c_double)))
    return dX


def learn_tables(W, bits, cb, init_thresholds, init_mappings, iters=2):
    """Mapping/threshold learner (Sec. 5, App. G): weighted Lloyd-Max per channel.
    Returns (thresholds fp32 [N,16], mappings fp32 [N,16], mse fp64 [N,iters+1], iters_done int32 [N])."""
    W = _c(W, np.float32); bits = _c(bits, np.uint8); cb = _c(cb, np.int32)
    it = _c(init_thresholds, np.float32); im = _c(init_mappings, np.float32)
    N, K = W.shape
    assert it.shape == im.shape and it.shape[1] == 16
    thr = np.zeros((N, 16), dtype=np.float32); mp = np.zeros((N, 16), dtype=np.float32)
    mse = np.zeros((N, iters + 1), dtype=np.float64); done = np.zeros(N, dtype=np.int32)
    _chk(_load().lowra_oracle_learn_tables(C.c_int(N), C.c_int(K), _p(W, C.c_float), _p(bits, C.c_uint8),
                                           _p(cb, C.c_int32), C.c_int(it.shape[0]), _p(it, C.c_float), _p(im, C.c_float),
                                           C.c_int(iters), _p(thr, C.c_float), _p(mp, C.c_float), _p(mse, C.c_double),
                                           _p(done, C.c_int32)))
    return thr, mp, mse, done


def average_thresholds(bits, thresholds):
    """Threshold averaging (Sec. 5): per width, the mean over the channels of that width.  Returns a new array."""
    bits = _c(bits, np.uint8)
    thr = np.array(thresholds, dtype=np.float32, order="C", copy=True)
    assert thr.shape == (bits.size, 16)
    _chk(_load().lowra_oracle_average_thresholds(C.c_int(bits.size), _p(bits, C.c_uint8), _p(thr, C.c_float)))
    return thr


def channel_mse(W, thresholds3, mappings3):
    """Per-channel error table (Sec. 6.1): mse fp64 [N,3] for 1, 2 and 4 bits with tables [3,16] fp32."""
    W = _c(W, np.float32); t = _c(thresholds3, np.float32); m = _c(mappings3, np.float32)
    assert t.shape == (3, 16) and m.shape == (3, 16)
    N, K = W.shape
    out = np.zeros((N, 3), dtype=np.float64)
    _chk(_load().lowra_oracle_channel_mse(C.c_int(N), C.c_int(K), _p(W, C.c_float), _p(t, C.c_float), _p(m, C.c_float),
                                          _p(out, C.c_double)))
    return out


def assign_greedy(params, mse, budget_bpp):
    """Greedy budgeted precision assignment (stand-in for the ILP of Sec. 6): bits uint8 [N]."""
    params = _c(params, np.int64); mse = _c(mse, np.float32)
    N = params.size
    assert mse.shape == (N, 3)
    bits = np.zeros(N, dtype=np.uint8)
    _chk(_load().lowra_oracle_assign_greedy(C.c_int(N), _p(params, C.c_int64), _p(mse, C.c_float), C.c_double(budget_bpp),
                                            _p(bits, C.c_uint8)))
    return bits


def adapter_grads(x, dY, A, B, s):
    """G1, G2: (dA fp64 [r,K], dB fp64 [N,r]) of y = x What^T + s (x A^T) B^T given dY.  bf16 bit patterns in."""
    x = _c(x, np.uint16); dY = _c(dY, np.uint16); A = _c(A, np.uint16); B = _c(B, np.uint16)
    M, K = x.shape
    N = dY.shape[1]
    r = A.shape[0]
    assert dY.shape == (M, N) and A.shape == (r, K) and B.shape == (N, r)
    dA = np.zeros((r, K), dtype=np.float64); dB = np.zeros((N, r), dtype=np.float64)
    _chk(_load().lowra_oracle_adapter_grads(C.c_int(N), C.c_int(K), C.c_int(M), C.c_int(r), _p(x, C.c_uint16),
                                            _p(dY, C.c_uint16), _p(A, C.c_uint16), _p(B, C.c_uint16), C.c_float(s),
                                            _p(dA, C.c_double), _p(dB, C.c_double)))
    return dA, dB


def best_rank_r(E, r):
    """I2: the best rank-r approximation of E in the Frobenius norm, from numpy's SVD (a library
    primitive used as one step): E ~ B A with A = the first r right singular vectors as rows
    (orthonormal) and B = E A^T = U_r S_r.  The paper fixes only the product (App. D speaks of "a
    low-rank approximation"); this split is a reading, and only B A enters what follows."""
    E = np.asarray(E, dtype=np.float64)
    _, _, Vt = np.linalg.svd(E, full_matrices=False)
    A = Vt[:r].copy()
    return E @ A.T, A


def loftq_init(W, bits, cb, thresholds, mappings, r, steps=5):
    """I1-I3, the alternating low-rank initialisation the paper adopts (Sec. 4.1, "Using LoftQ as
    low-rank initializer"; App. D; five alternating steps): start from B A = 0; in every step
      I1  quantize the residual W - B A with the layer's widths and tables (Q1-Q5; the residual is
          rounded to fp32, the quantizer's input type), decode it in fp32 (D1-D2): What;
      I2  take the best rank-r approximation of what the quantized weights miss: B A ~ W - What.
    Quantization comes first, so step 1 quantizes W itself (App. D: the order that tells this
    scheme from the SVD-first one).  Returns the last step's (packed, absmax), A [r,K] and B [N,r]
    in fp64, and the objective |W - What_t - B_t A_t|_F after every step."""
    W = _c(W, np.float32)
    N, K = W.shape
    W64 = W.astype(np.float64)
    A = np.zeros((r, K)); B = np.zeros((N, r))
    objective = []
    packed = absmax = None
    for _ in range(steps):
        R = (W64 - B @ A).astype(np.float32)
        packed, absmax = quantize(R, bits, cb, thresholds)
        What = dequantize(packed, absmax, bits, cb, mappings, K, "fp32").astype(np.float64)
        E = W64 - What
        B, A = best_rank_r(E, r)
        objective.append(float(np.linalg.norm(E - B @ A)))
    return packed, absmax, A, B, np.array(objective)
