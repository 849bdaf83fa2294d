"""Seeded synthetic workloads with the FC shapes of the paper's LLM benchmarks.

The paper measures on Gemma2 2B and Llama 3.1 8B checkpoints (section 4.2);
those weights are not available, so random layers with the same FC shapes stand
in.  This module only draws random tensors and lists shapes.  It holds none of
the method's arithmetic (no quantization, no dequantization, no matmul) and is
the one module both the CPU oracle's tests and the GPU path's tests consume.

Formats: "w8c" = int8 weights with one fp32 scale per output channel;
"w4g32" = int4 weights (one value per int8, range [-8, 7]) with one binary16
scale per 32 consecutive k of a row, scales [N, K/32];
"w4c" = int4 weights with one fp32 scale per output channel (the paper's
per-channel 4-bit scheme).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

KIND_X, KIND_W, KIND_S = 0, 1, 2


@dataclass(frozen=True)
class FC:
    name: str
    K: int
    N: int
    fmt: str  # "w8c" | "w4g32" | "w4c"


# Llama-3.1-8B: hidden 4096, 32 q heads + 2 x 8 kv heads of 128, FFN 14336.
LLAMA_FCS_W4 = (FC("qkv", 4096, 6144, "w4g32"), FC("o", 4096, 4096, "w4g32"),
                FC("gate_up", 4096, 28672, "w4g32"), FC("down", 14336, 4096, "w4g32"))
LLAMA_FCS_W8 = tuple(FC(f.name, f.K, f.N, "w8c") for f in LLAMA_FCS_W4)
LLAMA_FCS_W4C = tuple(FC(f.name, f.K, f.N, "w4c") for f in LLAMA_FCS_W4)
LLAMA_LM_HEAD = FC("lm_head", 4096, 128256, "w8c")
LLAMA_LAYERS = 32
# Gemma2-2B: hidden 2304, 8 q heads + 2 x 4 kv heads of 256, FFN 9216.
GEMMA_FCS_W4 = (FC("qkv", 2304, 4096, "w4g32"), FC("o", 2048, 2304, "w4g32"),
                FC("gate_up", 2304, 18432, "w4g32"), FC("down", 9216, 2304, "w4g32"))
GEMMA_FCS_W4C = tuple(FC(f.name, f.K, f.N, "w4c") for f in GEMMA_FCS_W4)
GEMMA_LM_HEAD = FC("lm_head", 2304, 256000, "w8c")
CFG1_FC = FC("fc", 512, 1024, "w8c")


def _rng(cfg_seed: int, layer: int, fc_id: int, kind: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([cfg_seed, layer, fc_id, kind]))


def activations(cfg_seed: int, layer: int, fc_id: int, M: int, K: int) -> np.ndarray:
    """fp16 activations ~ N(0, 1), [M, K]."""
    return _rng(cfg_seed, layer, fc_id, KIND_X).standard_normal((M, K), dtype=np.float32).astype(np.float16)


def weights(cfg_seed: int, layer: int, fc_id: int, fc: FC):
    """(Wq int8 [N, K], scales) for one FC.

    w8c: Wq uniform in [-127, 127], scales fp32 log-uniform in [1e-3, 1e-1].
    w4g32: Wq uniform in [-8, 7], scales binary16 log-uniform in [2e-3, 2e-2].
    w4c: Wq uniform in [-8, 7], scales fp32 log-uniform in [2e-3, 2e-2].
    """
    rw = _rng(cfg_seed, layer, fc_id, KIND_W)
    rs = _rng(cfg_seed, layer, fc_id, KIND_S)
    if fc.fmt == "w8c":
        wq = rw.integers(-127, 128, size=(fc.N, fc.K), dtype=np.int8)
        s = np.exp(rs.uniform(np.log(1e-3), np.log(1e-1), size=fc.N)).astype(np.float32)
    elif fc.fmt == "w4g32":
        wq = rw.integers(-8, 8, size=(fc.N, fc.K), dtype=np.int8)
        s = np.exp(rs.uniform(np.log(2e-3), np.log(2e-2), size=(fc.N, fc.K // 32))).astype(np.float16)
    elif fc.fmt == "w4c":
        wq = rw.integers(-8, 8, size=(fc.N, fc.K), dtype=np.int8)
        s = np.exp(rs.uniform(np.log(2e-3), np.log(2e-2), size=fc.N)).astype(np.float32)
    else:
        raise ValueError(fc.fmt)
    return wq, s


def algorithmic_bytes(fc: FC, M: int) -> int:
    """Bytes one decode FC must move: packed weights once, scales, x and y."""
    if fc.fmt == "w8c":
        w = fc.N * fc.K + 4 * fc.N
    elif fc.fmt == "w4c":
        w = fc.N * fc.K // 2 + 4 * fc.N
    else:
        w = fc.N * fc.K // 2 + 2 * fc.N * (fc.K // 32)
    return w + 2 * M * fc.K + 2 * M * fc.N


def algorithmic_ops(fc: FC, M: int) -> int:
    """Multiply-adds x 2 of one prefill FC."""
    return 2 * M * fc.N * fc.K
