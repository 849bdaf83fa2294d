"""CPU oracle, element-wise operators fused with the fully connected operator.

TEST INFRASTRUCTURE ONLY (same rule as the package: tests, the smoke check and
the CPU-baseline leg of the benchmark may import it; the product path never
does).  Plain numpy in fp64, one function per operator, nothing blocked or
reordered.  It imports nothing from the GPU package.

The paper (operator fusion, section 3.6 and its figure) merges element-wise
operators of two branches into a fully connected operator and residual
connections into the neighbouring operator; it prints no formulas for them.
The two branches in the models it evaluates are the gated feed-forward network:
Llama multiplies SiLU(gate) with the other branch, Gemma the tanh form of GELU.
"""
from __future__ import annotations

import numpy as np

SILU = 0
GELU_TANH = 1


def silu(g) -> np.ndarray:
    """g * sigmoid(g) = g / (1 + exp(-g)), fp64."""
    g = np.asarray(g, dtype=np.float64)
    return g / (1.0 + np.exp(-g))


def gelu_tanh(g) -> np.ndarray:
    """0.5 g (1 + tanh(sqrt(2/pi) (g + 0.044715 g^3))), fp64."""
    g = np.asarray(g, dtype=np.float64)
    return 0.5 * g * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (g + 0.044715 * g * g * g)))


def gated_input(gate_f16, up_f16, activation: int) -> np.ndarray:
    """The FC input of the fused operator: act(gate) * up, rounded once to binary16.

    That is the tensor an unfused element-wise operator would have written with
    FP16 activations (section 4.2).  Returns float16 [M, K].
    """
    g = np.asarray(gate_f16, dtype=np.float16).astype(np.float64)
    u = np.asarray(up_f16, dtype=np.float16).astype(np.float64)
    if activation == SILU:
        a = silu(g)
    elif activation == GELU_TANH:
        a = gelu_tanh(g)
    else:
        raise ValueError("unknown activation")
    return (a * u).astype(np.float16)  # fp64 -> binary16, round to nearest even


def gated_input_f32(gate_f16, up_f16, activation: int) -> np.ndarray:
    """gated_input with every step taken in binary32, the precision the kernels evaluate the gate
    in: t = g (c1 + c3 g^2), a = g / (1 + exp(-t)), fp16(a * up), each operation rounded to binary32
    (the multiply-add c3 g^2 + c1 rounded once).  For the path where the rounded value goes on to
    decide an 8-bit code (the row maximum and every code depend on its last bit), so that both
    sides of a comparison take that decision in the same precision; elsewhere gated_input (fp64)
    is the reference.  The two agree except where the real value lies within a few binary32 units
    of a binary16 rounding boundary (pinned in the CPU tests).  Returns float16 [M, K]."""
    f32 = np.float32
    g = np.asarray(gate_f16, dtype=np.float16).astype(f32)
    u = np.asarray(up_f16, dtype=np.float16).astype(f32)
    if activation == SILU:
        c1, c3 = f32(1.0), f32(0.0)
    elif activation == GELU_TANH:
        c1 = f32(1.5957691216)                      # 2 sqrt(2 / pi)
        c3 = f32(f32(1.5957691216) * f32(0.044715))
    else:
        raise ValueError("unknown activation")
    gg = (g * g).astype(f32)
    inner = (c3.astype(np.float64) * gg.astype(np.float64) + np.float64(c1)).astype(f32)  # one rounding, like an fma
    t = (g * inner).astype(f32)
    e = np.exp((-t).astype(f32)).astype(f32)
    a = (g / (f32(1.0) + e).astype(f32)).astype(f32)
    return (a * u).astype(f32).astype(np.float16)


def add_residual(y, residual_f16) -> np.ndarray:
    """y + residual in fp64 (the caller's comparison applies the final binary16 rounding)."""
    return np.asarray(y, dtype=np.float64) + np.asarray(residual_f16, dtype=np.float16).astype(np.float64)


def gated_output(y, activation: int) -> np.ndarray:
    """A layer that produces both branches: act(y[:, :N/2]) * y[:, N/2:] in fp64 on the unrounded
    outputs (the fused operator keeps them in registers; nothing is rounded in between)."""
    y = np.asarray(y, dtype=np.float64)
    half = y.shape[1] // 2
    assert y.shape[1] == 2 * half
    f = silu if activation == SILU else gelu_tanh if activation == GELU_TANH else None
    if f is None:
        raise ValueError("unknown activation")
    return f(y[:, :half]) * y[:, half:]


def rmsnorm(x_f16, gamma_f16, eps: float, gamma_offset: float = 0.0, residual_f16=None):
    """Root-mean-square normalization with the residual connection merged in (section 3.6, figure).

    h = x + residual, rounded once to binary16 (the residual stream as it is stored with FP16
    activations; h = x when there is no residual); per token row
    y[k] = h[k] / sqrt(mean_k(h^2) + eps) * (gamma_offset + gamma[k]) in fp64 on the stored h.
    gamma_offset is 0 for Llama and 1 for Gemma.  Returns (h float16 [M, K], y float64 [M, K]).
    """
    x = np.asarray(x_f16, dtype=np.float16)
    h = x if residual_f16 is None else (x.astype(np.float64) + np.asarray(residual_f16, dtype=np.float16).astype(np.float64)).astype(np.float16)
    hd = h.astype(np.float64)
    ms = np.mean(hd * hd, axis=1, keepdims=True)
    w = gamma_offset + np.asarray(gamma_f16, dtype=np.float16).astype(np.float64)
    return h, hd / np.sqrt(ms + eps) * w[None, :]


def rms_scale(x_f16, eps: float) -> np.ndarray:
    """rs[m] = 1 / sqrt(mean_k x[m, k]^2 + eps), fp64 [M]."""
    x = np.asarray(x_f16, dtype=np.float16).astype(np.float64)
    return 1.0 / np.sqrt(np.mean(x * x, axis=1) + eps)


def norm_weighted_input(x_f16, gamma_f16, gamma_offset: float = 0.0) -> np.ndarray:
    """x[m, k] * (gamma_offset + gamma[k]), rounded once to binary16: the input of a layer that has
    the RMS normalization merged into it.  Normalizing scales a row by one number, which commutes
    with the layer: rmsnorm(x) W^T = rs * ((x * weight) W^T), so the merged operator feeds the
    weighted row to the layer and multiplies its output by rs (rms_scale)."""
    x = np.asarray(x_f16, dtype=np.float16).astype(np.float64)
    w = gamma_offset + np.asarray(gamma_f16, dtype=np.float16).astype(np.float64)
    return (x * w[None, :]).astype(np.float16)


def embedding(ids, wq, scales, group_size: int = 0) -> np.ndarray:
    """Rows ``ids`` of the quantized table as binary16, [M, K] (section 4.2 of the paper: the
    embedding table is quantized like the layers): fp16(s * q) with the product taken in fp32, the
    precision the lookup computes in (exact for binary16 group scales; one rounding to fp32 before
    the rounding to binary16 for fp32 channel scales).  An id outside [0, N) gives zeros."""
    wq = np.asarray(wq, dtype=np.int8)
    ids = np.asarray(ids, dtype=np.int64)
    N, K = wq.shape
    ok = (ids >= 0) & (ids < N)
    safe = np.where(ok, ids, 0)
    q = wq[safe].astype(np.float32)
    if group_size == 0:
        s = np.asarray(scales, dtype=np.float32)[safe][:, None]
    else:
        s = np.repeat(np.asarray(scales, dtype=np.float16)[safe].astype(np.float32), group_size, axis=1)
    out = (s * q).astype(np.float16)
    out[~ok] = np.float16(0)
    return out
