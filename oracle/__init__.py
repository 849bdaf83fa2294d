"""CPU oracle for the quantized fully-connected layer: ctypes front end.

TEST INFRASTRUCTURE ONLY.  Only tests, the smoke check and the CPU-baseline leg
of the benchmark may import this package; the product path never does.  The
arithmetic of the layer lives in ``qfc_oracle.c`` (plain C, fp64 / fp32 as stated
there) and this file only marshals numpy arrays; the element-wise operators fused
with the layer are plain numpy in ``elementwise.py``.  It imports nothing from the GPU package.

Passages followed (section 3.7 for the two stages, section 4.2 for the weight
formats and FP16 activations) are cited function by function in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from .elementwise import GELU_TANH, SILU, add_residual, embedding, gated_input, gated_input_f32, gated_output, gelu_tanh, norm_weighted_input, rms_scale, rmsnorm, silu  # noqa: F401
from .attention import attention, rope, rope_qkv_layout, rope_qkv_layout_exact  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qfc_oracle.c")
_LIB = os.path.join(_HERE, "libqfc_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (about a second)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fno-fast-math", "-ffp-contract=off", "-fopenmp",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.qfc_oracle_threads.restype = ctypes.c_int
        _lib.qfc_oracle_f16_to_f64.restype = ctypes.c_double
        _lib.qfc_oracle_f16_to_f64.argtypes = [ctypes.c_uint16]
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _i64(v):
    return ctypes.c_int64(int(v))


def threads() -> int:
    return int(_load().qfc_oracle_threads())


def f16_bits_to_f64(bits: int) -> float:
    return float(_load().qfc_oracle_f16_to_f64(ctypes.c_uint16(bits)))


def _as_f16_bits(x) -> np.ndarray:
    x = np.ascontiguousarray(x)
    if x.dtype == np.float16:
        return x.view(np.uint16)
    if x.dtype == np.uint16:
        return x
    raise TypeError("binary16 data must be float16 or uint16 bit patterns")


def dequantize(wq, scales, group_size: int = 0) -> np.ndarray:
    """Explicit dequantized weight matrix in fp64, [N, K].

    group_size 0: ``scales`` is fp32 [N] (one per output channel);
    group_size g: ``scales`` is binary16 [N, K/g].
    """
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    N, K = wq.shape
    what = np.empty((N, K), dtype=np.float64)
    lib = _load()
    if group_size == 0:
        s = np.ascontiguousarray(scales, dtype=np.float32)
        assert s.shape == (N,)
        lib.qfc_oracle_dequant_per_channel(_p(wq), _p(s), _i64(N), _i64(K), _p(what))
    else:
        assert K % group_size == 0
        s = _as_f16_bits(scales)
        assert s.shape == (N, K // group_size)
        lib.qfc_oracle_dequant_group(_p(wq), _p(s), _i64(N), _i64(K), _i64(group_size), _p(what))
    return what


def fc_weight_only(x_f16, wq, scales, group_size: int = 0) -> np.ndarray:
    """y = x . dequant(Wq)^T in fp64 (weight-only path), [M, N]."""
    xb = _as_f16_bits(x_f16)
    M, K = xb.shape
    what = dequantize(wq, scales, group_size)
    N = what.shape[0]
    assert what.shape[1] == K
    y = np.empty((M, N), dtype=np.float64)
    _load().qfc_oracle_fc_f64(_p(xb), _p(what), _i64(M), _i64(N), _i64(K), _p(y))
    return y


def quantize_activations(x_f16):
    """Per-token symmetric int8 quantization; returns (xq int8 [M,K], sx fp32 [M])."""
    xb = _as_f16_bits(x_f16)
    M, K = xb.shape
    xq = np.empty((M, K), dtype=np.int8)
    sx = np.empty((M,), dtype=np.float32)
    _load().qfc_oracle_quantize_activations(_p(xb), _i64(M), _i64(K), _p(xq), _p(sx))
    return xq, sx


def int_contract(xq, wq) -> np.ndarray:
    """acc[m,n] = sum_k xq[m,k] * Wq[n,k], exact, int64."""
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    M, K = xq.shape
    N = wq.shape[0]
    assert wq.shape[1] == K
    acc = np.empty((M, N), dtype=np.int64)
    _load().qfc_oracle_int_contract(_p(xq), _p(wq), _i64(M), _i64(N), _i64(K), _p(acc))
    return acc


def rescale(acc, sx, sw) -> np.ndarray:
    acc = np.ascontiguousarray(acc, dtype=np.int64)
    sx = np.ascontiguousarray(sx, dtype=np.float32)
    sw = np.ascontiguousarray(sw, dtype=np.float32)
    M, N = acc.shape
    y = np.empty((M, N), dtype=np.float64)
    _load().qfc_oracle_rescale(_p(acc), _p(sx), _p(sw), _i64(M), _i64(N), _p(y))
    return y


def fc_int8_act(x_f16, wq, sw):
    """Prefill path, step by step: quantize x, integer contraction, rescale.

    Returns (xq, sx, acc, y) so that every intermediate can be compared.
    """
    xq, sx = quantize_activations(x_f16)
    acc = int_contract(xq, wq)
    y = rescale(acc, sx, sw)
    return xq, sx, acc, y


def _row_floor(y_ref: np.ndarray):
    """rho_m: root mean square of row m of the reference; of the whole output when a row has fewer
    than 32 entries (too few terms for a scale of its own: at N = 1 it would be |y| itself)."""
    if y_ref.ndim == 2 and y_ref.shape[1] < 32:
        return np.sqrt(np.mean(y_ref * y_ref))
    return np.sqrt(np.mean(y_ref * y_ref, axis=1, keepdims=True))


def floored_denominator(y_ref) -> np.ndarray:
    """max(|y_ref[m,n]|, rho_m) element by element: the denominator of the acceptance metric."""
    y_ref = np.asarray(y_ref, dtype=np.float64)
    den = np.maximum(np.abs(y_ref), _row_floor(y_ref))
    return np.where(den == 0.0, 1.0, den)


def floored_rel_error(y_gpu, y_ref) -> float:
    """Acceptance metric of the floating-point paths.

    E = max_{m,n} |y_gpu - y_ref| / max(|y_ref[m,n]|, rho_m), with rho_m the
    root-mean-square of row m of the reference (of the whole output when a
    row has fewer than 32 entries).  The floor keeps outputs that
    cancel to almost zero from dominating; the bound is 2e-3.
    """
    y_ref = np.asarray(y_ref, dtype=np.float64)
    y_gpu = np.asarray(y_gpu, dtype=np.float64)
    den = np.maximum(np.abs(y_ref), _row_floor(y_ref))
    den = np.where(den == 0.0, 1.0, den)
    return float(np.max(np.abs(y_gpu - y_ref) / den)) if y_ref.size else 0.0


def plain_rel_error_above_floor(y_gpu, y_ref) -> float:
    """max |y_gpu - y_ref| / |y_ref| over the entries with |y_ref| >= rho_m (0 if there are none):
    the plain relative error where it is meaningful, i.e. away from sums that cancel.  It can
    never exceed floored_rel_error; it is reported and asserted beside it so that the bound is
    also checked in the form "maximum relative error"."""
    y_ref = np.asarray(y_ref, dtype=np.float64)
    y_gpu = np.asarray(y_gpu, dtype=np.float64)
    if not y_ref.size:
        return 0.0
    keep = (np.abs(y_ref) >= _row_floor(y_ref)) & (y_ref != 0.0)
    if not np.any(keep):
        return 0.0
    return float(np.max(np.abs(y_gpu - y_ref)[keep] / np.abs(y_ref)[keep]))
