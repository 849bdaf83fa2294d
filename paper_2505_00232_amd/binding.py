"""Thin ctypes binding of libqfc.so: same names as include/qfc.h, argument
marshalling only.  PyTorch supplies device memory and the stream; every step of
the path runs in the library's HIP kernels.  There is no fallback: if the
library is missing or a call fails, an exception is raised."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqfc.so")

QFC_OK = 0
QFC_ERR_INVALID_ARG, QFC_ERR_UNSUPPORTED, QFC_ERR_BUFFER_TOO_SMALL, QFC_ERR_ALIGNMENT, QFC_ERR_HIP = 1, 2, 3, 4, 5
QFC_ERR_SCRATCH_LIMIT = 6
QFC_STATIC_SCRATCH_BYTES = 16 << 20
QFC_SCALE_F32, QFC_SCALE_F16 = 0, 1
QFC_COMPUTE_FP16_DEQUANT, QFC_COMPUTE_INT8_ACT, QFC_COMPUTE_INT8_ACT_DECODE = 0, 1, 2
QFC_ACT_SILU, QFC_ACT_GELU_TANH = 0, 1
QFC_PACK_GATED_PAIRS = 1

EXPORTS = ["qfc_packed_size", "qfc_pack_weights", "qfc_unpack_weights", "qfc_workspace_size",
           "qfc_bind_workspace", "qfc_quantize_activations", "qfc_forward", "qfc_forward_fused", "qfc_forward_static", "qfc_rmsnorm", "qfc_rope_qkv", "qfc_rope_table", "qfc_forward_qkv_rope", "qfc_attention_workspace_size", "qfc_attention", "qfc_forward_q8",
           "qfc_forward_acc_i32", "qfc_embedding", "qfc_forward_batch", "qfc_destroy", "qfc_status_string"]


class Desc(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int32), ("K", ctypes.c_int32), ("wbits", ctypes.c_int32),
                ("group_size", ctypes.c_int32), ("scale_dtype", ctypes.c_int32),
                ("compute_mode", ctypes.c_int32), ("flags", ctypes.c_int32)]


class Fusion(ctypes.Structure):
    """qfc_fusion_t: element-wise parts fused with the layer (null = absent)."""
    _fields_ = [("gate", ctypes.c_void_p), ("activation", ctypes.c_int32), ("residual", ctypes.c_void_p),
                ("gated_output", ctypes.c_int32), ("norm_gamma", ctypes.c_void_p), ("norm_eps", ctypes.c_float),
                ("norm_offset", ctypes.c_float)]


class RmsNorm(ctypes.Structure):
    """qfc_rmsnorm_t."""
    _fields_ = [("x", ctypes.c_void_p), ("residual", ctypes.c_void_p), ("gamma", ctypes.c_void_p),
                ("eps", ctypes.c_float), ("gamma_offset", ctypes.c_float), ("h_out", ctypes.c_void_p),
                ("y", ctypes.c_void_p), ("xq", ctypes.c_void_p), ("sx", ctypes.c_void_p),
                ("consumer", ctypes.c_void_p)]


class AttnShape(ctypes.Structure):
    """qfc_attn_shape_t."""
    _fields_ = [("batch", ctypes.c_int32), ("h_q", ctypes.c_int32), ("h_kv", ctypes.c_int32),
                ("d_head", ctypes.c_int32), ("cache_size", ctypes.c_int32)]


class QfcError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} (status {code})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; built beforehand by paper_2505_00232_amd.build."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2505_00232_amd.build` first")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        L.qfc_packed_size.argtypes = [ctypes.POINTER(Desc), ctypes.POINTER(sz)]
        L.qfc_pack_weights.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, sz, vp, ctypes.POINTER(vp)]
        L.qfc_unpack_weights.argtypes = [vp, vp, vp, vp]
        L.qfc_workspace_size.argtypes = [vp, i32, ctypes.POINTER(sz)]
        L.qfc_bind_workspace.argtypes = [vp, vp, sz]
        L.qfc_quantize_activations.argtypes = [vp, i32, i32, vp, vp, vp]
        L.qfc_forward.argtypes = [vp, vp, i32, vp, vp]
        L.qfc_forward_static.argtypes = [vp, vp, i32, vp, vp]
        L.qfc_forward_fused.argtypes = [vp, vp, i32, vp, ctypes.POINTER(Fusion), vp]
        L.qfc_rmsnorm.argtypes = [ctypes.POINTER(RmsNorm), i32, i32, vp]
        L.qfc_rope_qkv.argtypes = [vp, i32, i32, ctypes.POINTER(AttnShape), ctypes.c_float, vp, vp, vp, vp]
        L.qfc_attention_workspace_size.argtypes = [ctypes.POINTER(AttnShape), i32, ctypes.POINTER(sz)]
        L.qfc_attention.argtypes = [vp, vp, vp, i32, i32, ctypes.POINTER(AttnShape), vp, sz, vp, vp]
        L.qfc_rope_table.argtypes = [ctypes.POINTER(AttnShape), ctypes.c_float, i32, vp, vp]
        L.qfc_forward_qkv_rope.argtypes = [vp, vp, ctypes.POINTER(Fusion), ctypes.POINTER(AttnShape), i32, vp, i32, vp, vp, vp, vp]
        L.qfc_forward_q8.argtypes = [vp, vp, vp, i32, vp, vp]
        L.qfc_forward_acc_i32.argtypes = [vp, vp, i32, vp, vp]
        L.qfc_embedding.argtypes = [vp, vp, i32, vp, vp]
        L.qfc_forward_batch.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(vp), i32, ctypes.POINTER(vp), i32, vp]
        L.qfc_destroy.argtypes = [vp]
        L.qfc_status_string.argtypes = [ctypes.c_int]
        L.qfc_status_string.restype = ctypes.c_char_p
        L.qfc_tune.argtypes = [i32, i32]
        L.qfc_tune.restype = None
        L.qfc_probe_mfma.argtypes = [i32, i32, i32, i32, vp, vp]
        L.qfc_probe_mfma.restype = ctypes.c_int
        for name in EXPORTS:
            if name != "qfc_status_string":
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(code: int) -> str:
    return lib().qfc_status_string(int(code)).decode()


def _check(code: int, where: str):
    if code != QFC_OK:
        raise QfcError(code, where)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr() if t is not None else 0)


def _want(t: torch.Tensor, dtype, shape, what: str):
    """The C ABI sees pointers and sizes only: dtype, device, contiguity and the dimensions a
    kernel derives its addresses from are checked here, before anything is launched."""
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise ValueError(f"{what}: a CUDA tensor is required")
    if t.dtype != dtype:
        raise ValueError(f"{what}: dtype {t.dtype}, expected {dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{what}: must be contiguous (row-major, no strides)")
    if shape is not None:
        if t.dim() != len(shape) or any(w is not None and int(d) != int(w) for d, w in zip(t.shape, shape)):
            raise ValueError(f"{what}: shape {tuple(t.shape)}, expected {tuple('*' if w is None else w for w in shape)}")


_dims: dict[int, tuple[int, int]] = {}  # handle value -> (N, K), kept from qfc_pack_weights to qfc_destroy


def _nk(h):
    try:
        return _dims[h.value]
    except KeyError:
        raise ValueError("unknown handle (not created by qfc_pack_weights of this binding, or destroyed)") from None


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_desc(N: int, K: int, fmt: str, compute_mode: int | None = None, gated_pairs: bool = False) -> Desc:
    flags = QFC_PACK_GATED_PAIRS if gated_pairs else 0
    if fmt == "w8c":
        mode = QFC_COMPUTE_INT8_ACT if compute_mode is None else compute_mode
        return Desc(N, K, 8, 0, QFC_SCALE_F32, mode, flags)
    if fmt == "w4g32":
        mode = QFC_COMPUTE_FP16_DEQUANT if compute_mode is None else compute_mode
        return Desc(N, K, 4, 32, QFC_SCALE_F16, mode, flags)
    if fmt == "w4c":
        mode = QFC_COMPUTE_FP16_DEQUANT if compute_mode is None else compute_mode
        return Desc(N, K, 4, 0, QFC_SCALE_F32, mode, flags)
    raise ValueError(fmt)


def qfc_packed_size(desc: Desc) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().qfc_packed_size(ctypes.byref(desc), ctypes.byref(out)), "qfc_packed_size")
    return out.value


def qfc_pack_weights(desc: Desc, wq_logical: torch.Tensor, scales: torch.Tensor, packed: torch.Tensor):
    _want(wq_logical, torch.int8, (desc.N, desc.K), "wq_logical")
    if desc.group_size:
        _want(scales, torch.float16, (desc.N, desc.K // desc.group_size), "scales")
    else:
        _want(scales, torch.float32, (desc.N,), "scales")
    _want(packed, torch.uint8, None, "packed")
    h = ctypes.c_void_p(0)
    _check(lib().qfc_pack_weights(ctypes.byref(desc), _ptr(wq_logical), _ptr(scales), _ptr(packed),
                                  packed.numel() * packed.element_size(), _stream(), ctypes.byref(h)),
           "qfc_pack_weights")
    _dims[h.value] = (int(desc.N), int(desc.K))
    return h


def qfc_unpack_weights(h, wq_logical: torch.Tensor, scales: torch.Tensor):
    N, K = _nk(h)
    _want(wq_logical, torch.int8, (N, K), "wq_logical")
    if scales.dtype == torch.float16:
        _want(scales, torch.float16, (N, None), "scales")
    else:
        _want(scales, torch.float32, (N,), "scales")
    _check(lib().qfc_unpack_weights(h, _ptr(wq_logical), _ptr(scales), _stream()), "qfc_unpack_weights")


def qfc_workspace_size(h, M: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().qfc_workspace_size(h, M, ctypes.byref(out)), "qfc_workspace_size")
    return out.value


def qfc_bind_workspace(h, ws: torch.Tensor):
    _check(lib().qfc_bind_workspace(h, _ptr(ws), ws.numel() * ws.element_size()), "qfc_bind_workspace")


def qfc_quantize_activations(x: torch.Tensor, xq: torch.Tensor, sx: torch.Tensor):
    _want(x, torch.float16, (None, None), "x")
    M, K = x.shape
    _want(xq, torch.int8, (M, K), "xq")
    _want(sx, torch.float32, (M,), "sx")
    _check(lib().qfc_quantize_activations(_ptr(x), M, K, _ptr(xq), _ptr(sx), _stream()), "qfc_quantize_activations")


def qfc_forward(h, x: torch.Tensor, y: torch.Tensor):
    N, K = _nk(h)
    _want(x, torch.float16, (None, K), "x")
    _want(y, torch.float16, (x.shape[0], N), "y")
    _check(lib().qfc_forward(h, _ptr(x), x.shape[0], _ptr(y), _stream()), "qfc_forward")


def qfc_forward_static(h, x: torch.Tensor, y: torch.Tensor):
    N, K = _nk(h)
    _want(x, torch.float16, (None, K), "x")
    _want(y, torch.float16, (x.shape[0], N), "y")
    _check(lib().qfc_forward_static(h, _ptr(x), x.shape[0], _ptr(y), _stream()), "qfc_forward_static")


def qfc_forward_fused(h, x: torch.Tensor, y: torch.Tensor, gate: torch.Tensor | None = None,
                      activation: int = QFC_ACT_SILU, residual: torch.Tensor | None = None,
                      gated_output: bool = False, norm_gamma: torch.Tensor | None = None, norm_eps: float = 0.0,
                      norm_offset: float = 0.0):
    N, K = _nk(h)
    _want(x, torch.float16, (None, K), "x")
    M = x.shape[0]
    _want(y, torch.float16, (M, N // 2 if gated_output else N), "y")
    if gate is not None:
        _want(gate, torch.float16, (M, K), "gate")
    if residual is not None and not gated_output:  # (the library rejects that combination itself)
        _want(residual, torch.float16, (M, N), "residual")
    if norm_gamma is not None:
        _want(norm_gamma, torch.float16, (K,), "norm_gamma")
    f = Fusion(gate.data_ptr() if gate is not None else None, activation,
               residual.data_ptr() if residual is not None else None, 1 if gated_output else 0,
               norm_gamma.data_ptr() if norm_gamma is not None else None, norm_eps, norm_offset)
    _check(lib().qfc_forward_fused(h, _ptr(x), x.shape[0], _ptr(y), ctypes.byref(f), _stream()), "qfc_forward_fused")


def qfc_rmsnorm(x: torch.Tensor, gamma: torch.Tensor, eps: float, gamma_offset: float = 0.0, residual=None,
                h_out=None, y=None, xq=None, sx=None, consumer=None):
    def p(t):
        return t.data_ptr() if t is not None else None
    _want(x, torch.float16, (None, None), "x")
    M, K = x.shape
    _want(gamma, torch.float16, (K,), "gamma")
    for t, name in ((residual, "residual"), (h_out, "h_out"), (y, "y")):
        if t is not None:
            _want(t, torch.float16, (M, K), name)
    if xq is not None:
        _want(xq, torch.int8, (M, K), "xq")
    if sx is not None:
        _want(sx, torch.float32, (M,), "sx")
    if consumer is not None and _nk(consumer)[1] != K:
        raise ValueError("consumer: K of the layer differs from the normalized width")
    a = RmsNorm(p(x), p(residual), p(gamma), eps, gamma_offset, p(h_out), p(y), p(xq), p(sx),
                consumer.value if consumer is not None else None)
    _check(lib().qfc_rmsnorm(ctypes.byref(a), M, K, _stream()), "qfc_rmsnorm")


def qfc_rope_qkv(qkv: torch.Tensor, pos0: int, shape: AttnShape, rope_base: float, q_out: torch.Tensor,
                 kcache: torch.Tensor, vcache: torch.Tensor):
    S = qkv.shape[1]
    _check(lib().qfc_rope_qkv(_ptr(qkv), S, pos0, ctypes.byref(shape), rope_base, _ptr(q_out), _ptr(kcache),
                              _ptr(vcache), _stream()), "qfc_rope_qkv")


def qfc_rope_table(shape: AttnShape, rope_base: float, positions: int, device="cuda") -> torch.Tensor:
    """cos and sin of the rotary angles of the first `positions` positions: float32 [positions, d_head / 2, 2]."""
    table = torch.empty((positions, shape.d_head // 2, 2), dtype=torch.float32, device=device)
    _check(lib().qfc_rope_table(ctypes.byref(shape), rope_base, positions, _ptr(table), _stream()), "qfc_rope_table")
    return table


def qfc_forward_qkv_rope(h, x: torch.Tensor, pos0: int, shape: AttnShape, rope_table: torch.Tensor, q_out: torch.Tensor,
                         kcache: torch.Tensor, vcache: torch.Tensor, norm_gamma: torch.Tensor | None = None,
                         norm_eps: float = 0.0, norm_offset: float = 0.0):
    """Decode step of the QKV layer with rotary embedding, layout transformation and cache append merged in."""
    N, K = _nk(h)
    g = shape.h_q // max(shape.h_kv, 1)
    G = shape.batch * shape.h_kv
    _want(x, torch.float16, (shape.batch, K), "x")
    _want(rope_table, torch.float32, (None, shape.d_head // 2, 2), "rope_table")
    _want(q_out, torch.float16, (G, g, shape.d_head), "q_out")
    _want(kcache, torch.float16, (G, shape.cache_size, shape.d_head), "kcache")
    _want(vcache, torch.float16, (G, shape.cache_size // 64, shape.d_head, 64), "vcache")
    f = None
    if norm_gamma is not None:
        _want(norm_gamma, torch.float16, (K,), "norm_gamma")
        f = Fusion(None, 0, None, 0, norm_gamma.data_ptr(), norm_eps, norm_offset)
    _check(lib().qfc_forward_qkv_rope(h, _ptr(x), ctypes.byref(f) if f is not None else None, ctypes.byref(shape), pos0,
                                      _ptr(rope_table), rope_table.shape[0], _ptr(q_out), _ptr(kcache), _ptr(vcache),
                                      _stream()), "qfc_forward_qkv_rope")


def vcache_physical(v_logical: torch.Tensor) -> torch.Tensor:
    """[G, d_head, cache] -> the library's V cache layout [G, cache / 64, d_head, 64] (a copy)."""
    G, d, C = v_logical.shape
    return v_logical.reshape(G, d, C // 64, 64).permute(0, 2, 1, 3).contiguous()


def vcache_logical(v_physical: torch.Tensor) -> torch.Tensor:
    """Inverse of vcache_physical."""
    G, nb, d, _ = v_physical.shape
    return v_physical.permute(0, 2, 1, 3).reshape(G, d, nb * 64).contiguous()


def qfc_attention_workspace_size(shape: AttnShape, S: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().qfc_attention_workspace_size(ctypes.byref(shape), S, ctypes.byref(out)), "qfc_attention_workspace_size")
    return out.value


def qfc_attention(q: torch.Tensor, kcache: torch.Tensor, vcache: torch.Tensor, S: int, n_ctx: int, shape: AttnShape,
                  workspace: torch.Tensor, out: torch.Tensor):
    _check(lib().qfc_attention(_ptr(q), _ptr(kcache), _ptr(vcache), S, n_ctx, ctypes.byref(shape), _ptr(workspace),
                               workspace.numel() * workspace.element_size(), _ptr(out), _stream()), "qfc_attention")


def qfc_forward_q8(h, xq: torch.Tensor | None, sx: torch.Tensor | None, y: torch.Tensor):
    """xq = sx = None: the activations a preceding qfc_rmsnorm(..., consumer=h) left in h's workspace."""
    N, K = _nk(h)
    if xq is None and sx is None:
        _want(y, torch.float16, (None, N), "y")
        _check(lib().qfc_forward_q8(h, None, None, y.shape[0], _ptr(y), _stream()), "qfc_forward_q8")
        return
    _want(xq, torch.int8, (None, K), "xq")
    _want(sx, torch.float32, (xq.shape[0],), "sx")
    _want(y, torch.float16, (xq.shape[0], N), "y")
    _check(lib().qfc_forward_q8(h, _ptr(xq), _ptr(sx), xq.shape[0], _ptr(y), _stream()), "qfc_forward_q8")


def qfc_forward_acc_i32(h, xq: torch.Tensor, acc: torch.Tensor):
    N, K = _nk(h)
    _want(xq, torch.int8, (None, K), "xq")
    _want(acc, torch.int32, (xq.shape[0], N), "acc")
    _check(lib().qfc_forward_acc_i32(h, _ptr(xq), xq.shape[0], _ptr(acc), _stream()), "qfc_forward_acc_i32")


def qfc_embedding(h, ids: torch.Tensor, y: torch.Tensor):
    N, K = _nk(h)
    _want(ids, torch.int32, (None,), "ids")
    _want(y, torch.float16, (ids.shape[0], K), "y")
    _check(lib().qfc_embedding(h, _ptr(ids), ids.shape[0], _ptr(y), _stream()), "qfc_embedding")


class ForwardBatch:
    """Pre-marshalled argument arrays for qfc_forward_batch."""

    def __init__(self, handles, xs, ys, M: int):
        n = len(handles)
        if len(xs) != n or len(ys) != n:
            raise ValueError("handles, xs and ys must have one entry per layer")
        for h, x, y in zip(handles, xs, ys):
            N, K = _nk(h)
            _want(x, torch.float16, (M, K), "x")
            _want(y, torch.float16, (M, N), "y")
        arr = ctypes.c_void_p * n
        self.h = arr(*[h.value for h in handles])
        self.x = arr(*[x.data_ptr() for x in xs])
        self.y = arr(*[y.data_ptr() for y in ys])
        self.n, self.M = n, M
        self._keep = (list(xs), list(ys))

    def run(self):
        _check(lib().qfc_forward_batch(self.h, self.x, self.M, self.y, self.n, _stream()), "qfc_forward_batch")


def qfc_destroy(h):
    _check(lib().qfc_destroy(h), "qfc_destroy")
    _dims.pop(h.value, None)


def qfc_tune(key: int, value: int):
    lib().qfc_tune(key, value)


def qfc_probe_mfma(kind: int, random_operands: bool, iters: int, workgroups: int, ticks):
    """Measurement probe of qfc_experimental.h: ticks = int64 device tensor [workgroups, 2]."""
    _want(ticks, torch.int64, (workgroups, 2), "ticks")
    _check(lib().qfc_probe_mfma(kind, int(bool(random_operands)), iters, workgroups, _ptr(ticks), _stream()),
           "qfc_probe_mfma")


class QuantLinear:
    """Convenience owner of one packed layer: device buffers + handle."""

    def __init__(self, wq, scales, fmt: str, compute_mode: int | None = None, device="cuda", max_m: int = 8,
                 workspace: torch.Tensor | None = None, gated_pairs: bool = False):
        wq_d = torch.as_tensor(wq).to(device).contiguous()
        s_d = torch.as_tensor(scales).to(device).contiguous()
        N, K = wq_d.shape
        self.N, self.K, self.fmt = N, K, fmt
        self.desc = make_desc(N, K, fmt, compute_mode, gated_pairs)
        self.packed = torch.empty(qfc_packed_size(self.desc), dtype=torch.uint8, device=device)
        self.handle = qfc_pack_weights(self.desc, wq_d, s_d, self.packed)
        need = max(qfc_workspace_size(self.handle, m) for m in sorted({1, min(max_m, 8), max_m}))
        if workspace is None or workspace.numel() < need:
            workspace = torch.empty(need, dtype=torch.uint8, device=device)
        self.workspace = workspace
        qfc_bind_workspace(self.handle, self.workspace)
        torch.cuda.current_stream().synchronize()  # inputs of the conversion may now be freed

    def forward(self, x: torch.Tensor, y: torch.Tensor | None = None) -> torch.Tensor:
        if y is None:
            y = torch.empty((x.shape[0], self.N), dtype=torch.float16, device=x.device)
        qfc_forward(self.handle, x, y)
        return y

    def close(self):
        if self.handle is not None:
            qfc_destroy(self.handle)
            self.handle = None
