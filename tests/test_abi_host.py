"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before touching a
device."""
import ctypes
import os
import re
import subprocess

import pytest

from paper_2505_00232_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.lib()


def _declared(header_name):
    header = open(os.path.join(ROOT, "include", header_name)).read()
    return set(re.findall(r"\b(qfc_[a-z0-9_]+)\s*\(", header))


def test_header_symbols_are_exported(L):
    """qfc.h declares exactly the binding's entry points, and the library's dynamic symbol table
    holds no qfc_* function beyond what the two headers declare (qfc_experimental.h: the
    tunables of tests and sweeps, which are not part of the interface)."""
    declared = _declared("qfc.h")
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name
    experimental = _declared("qfc_experimental.h")
    assert experimental == {"qfc_tune", "qfc_probe_mfma"}
    nm = subprocess.run(["nm", "-D", "--defined-only", binding.LIB_PATH], capture_output=True, text=True, check=True)
    exported = {ln.split()[-1] for ln in nm.stdout.splitlines() if len(ln.split()) >= 3 and ln.split()[-2] in "TW"}
    assert {e for e in exported if e.startswith("qfc_")} == declared | experimental


def test_status_strings(L):
    seen = {binding.status_string(c) for c in range(7)}
    assert len(seen) == 7 and binding.status_string(0) == "ok"
    assert binding.status_string(99) == "unknown status"


def test_packed_size_and_descriptor_checks(L):
    d = binding.make_desc(1024, 512, "w8c")
    # 1024 x 512 codes + 1024 fp32 scales, no padding needed
    assert binding.qfc_packed_size(d) == 1024 * 512 + 4 * 1024
    d = binding.make_desc(4096, 2304, "w4g32")
    # per 16 rows: 18 KiB tiles of 128 k plus 3 scale tiles
    assert binding.qfc_packed_size(d) == (4096 // 16) * (18 + 3) * 1024
    d = binding.make_desc(1, 32, "w4g32")
    assert binding.qfc_packed_size(d) == 16 * 2 * 1024  # padded to 256 rows x 128 k, one scale tile each
    d = binding.make_desc(4096, 2304, "w4c")
    # per 16 rows: 18 KiB tiles of 128 k, no scale tiles; 4096 fp32 scales follow
    assert binding.qfc_packed_size(d) == (4096 // 16) * 18 * 1024 + 4 * 4096
    out = ctypes.c_size_t(0)
    bad = [binding.Desc(0, 512, 8, 0, 0, 1), binding.Desc(8, 48, 8, 0, 0, 1), binding.Desc(8, 64, 3, 0, 0, 1),
           binding.Desc(8, 64, 8, -1, 0, 1), binding.Desc(8, 64, 8, 0, 7, 1), binding.Desc(8, 64, 8, 0, 0, 5)]
    assert binding.qfc_packed_size(binding.Desc(8, 64, 4, 0, 0, 2)) > 0  # int8-activation decode, per-channel int4
    for d in bad:
        assert L.qfc_packed_size(ctypes.byref(d), ctypes.byref(out)) == 1
    assert binding.qfc_packed_size(binding.Desc(8, 64, 4, 0, 0, 1)) > 0  # int8-activation prefill, per-channel int4 ("8/4/4")
    unsupported = [binding.Desc(8, 64, 8, 32, 0, 1), binding.Desc(8, 64, 4, 32, 1, 1),
                   binding.Desc(8, 64, 4, 0, 1, 0), binding.Desc(8, 64, 8, 0, 1, 1),
                   binding.Desc(8, 64, 4, 32, 1, 2)]
    for d in unsupported:
        assert L.qfc_packed_size(ctypes.byref(d), ctypes.byref(out)) == 2
    assert L.qfc_packed_size(None, ctypes.byref(out)) == 1
    assert L.qfc_packed_size(ctypes.byref(binding.make_desc(8, 64, "w8c")), None) == 1


def test_argument_errors_before_any_launch(L):
    d = binding.make_desc(64, 64, "w8c")
    h = ctypes.c_void_p(0)
    a = ctypes.c_void_p(0x1000)   # never dereferenced: checks fail first
    odd = ctypes.c_void_p(0x1008)
    s = ctypes.c_void_p(0)
    assert L.qfc_pack_weights(ctypes.byref(d), None, a, a, 1 << 20, s, ctypes.byref(h)) == 1
    assert L.qfc_pack_weights(ctypes.byref(d), a, a, a, 1 << 20, s, None) == 1
    assert L.qfc_pack_weights(ctypes.byref(d), odd, a, a, 1 << 20, s, ctypes.byref(h)) == 4
    assert L.qfc_pack_weights(ctypes.byref(d), a, a, a, 16, s, ctypes.byref(h)) == 3
    assert h.value is None
    for fn, args in [(L.qfc_forward, (None, a, 1, a, s)), (L.qfc_forward_static, (None, a, 1, a, s)), (L.qfc_unpack_weights, (None, a, a, s)),
                     (L.qfc_bind_workspace, (None, a, 1024)), (L.qfc_forward_q8, (None, a, a, 1, a, s)),
                     (L.qfc_forward_acc_i32, (None, a, 1, a, s)), (L.qfc_embedding, (None, a, 1, a, s)),
                     (L.qfc_destroy, (None,))]:
        assert fn(*args) == 1
    out = ctypes.c_size_t(0)
    assert L.qfc_workspace_size(None, 1, ctypes.byref(out)) == 1
    assert L.qfc_quantize_activations(a, 0, 64, a, a, s) == 1
    assert L.qfc_quantize_activations(a, 4, 40, a, a, s) == 1
    assert L.qfc_quantize_activations(odd, 4, 64, a, a, s) == 4
    assert L.qfc_quantize_activations(None, 4, 64, a, a, s) == 1
    assert L.qfc_forward_batch(None, None, 1, None, 0, s) == 1
    assert L.qfc_forward_fused(None, a, 1, a, None, s) == 1
    # RMS normalization: argument checks come before any launch
    R = binding.RmsNorm
    A, ODD = 0x1000, 0x1008
    assert L.qfc_rmsnorm(None, 1, 64, s) == 1
    assert L.qfc_rmsnorm(ctypes.byref(R(A, None, A, 1e-5, 0.0, None, None, None, None)), 1, 64, s) == 1   # no output
    assert L.qfc_rmsnorm(ctypes.byref(R(A, None, A, 1e-5, 0.0, None, A, A, None)), 1, 64, s) == 1        # xq without sx
    assert L.qfc_rmsnorm(ctypes.byref(R(A, None, A, 1e-5, 0.0, None, A, None, None)), 1, 40, s) == 1      # K % 32
    assert L.qfc_rmsnorm(ctypes.byref(R(A, None, A, -1.0, 0.0, None, A, None, None)), 1, 64, s) == 1      # eps < 0
    assert L.qfc_rmsnorm(ctypes.byref(R(A, None, A, 1e-5, 0.0, None, A, None, None)), 1, 14368, s) == 2   # row too long
    assert L.qfc_rmsnorm(ctypes.byref(R(A, ODD, A, 1e-5, 0.0, None, A, None, None)), 1, 64, s) == 4
    assert L.qfc_rmsnorm(ctypes.byref(R(None, None, A, 1e-5, 0.0, None, A, None, None)), 1, 64, s) == 1
    # attention-side operators
    S8 = binding.AttnShape
    A = ctypes.c_void_p(0x1000)
    out = ctypes.c_size_t(0)
    assert L.qfc_attention_workspace_size(ctypes.byref(S8(1, 32, 8, 128, 4096)), 1, ctypes.byref(out)) == 0
    assert out.value == 8 * 64 * 4 * 130 * 4
    assert L.qfc_attention_workspace_size(ctypes.byref(S8(1, 32, 8, 96, 4096)), 1, ctypes.byref(out)) == 2    # head size
    assert L.qfc_attention_workspace_size(ctypes.byref(S8(1, 32, 8, 128, 4128)), 1, ctypes.byref(out)) == 1   # cache % 64
    assert L.qfc_attention_workspace_size(ctypes.byref(S8(1, 32, 6, 128, 4096)), 1, ctypes.byref(out)) == 1   # h_q % h_kv
    assert L.qfc_attention_workspace_size(ctypes.byref(S8(1, 32, 8, 128, 4096)), 5, ctypes.byref(out)) == 0   # prefill path
    assert out.value == 256
    sh = S8(1, 32, 8, 128, 4096)
    assert L.qfc_attention(A, A, A, 1, 0, ctypes.byref(sh), A, 1 << 30, A, s) == 1        # n_ctx < S
    assert L.qfc_attention(A, A, A, 1, 5000, ctypes.byref(sh), A, 1 << 30, A, s) == 1     # n_ctx > cache
    assert L.qfc_attention(A, A, A, 1, 100, ctypes.byref(sh), A, 1024, A, s) == 3         # workspace too small
    assert L.qfc_attention(A, A, ctypes.c_void_p(0x1008), 1, 100, ctypes.byref(sh), A, 1 << 30, A, s) == 4
    assert L.qfc_rope_qkv(A, 1, 4096, ctypes.byref(sh), 10000.0, A, A, A, s) == 1           # position past the cache
    assert L.qfc_rope_qkv(A, 1, 0, ctypes.byref(sh), 1.0, A, A, A, s) == 1                  # base must exceed 1
    assert L.qfc_rope_qkv(None, 1, 0, ctypes.byref(sh), 10000.0, A, A, A, s) == 1


def test_build_refuses_spills_in_kernels_with_hand_placed_loads():
    """The build parses the compiler's resource-usage remarks of the kernels whose operand loads are
    asynchronous assembly (a spilled destination register would be saved before its load lands)."""
    from paper_2505_00232_amd import build
    pre = "gemm_i8.hip:527:1: remark: "
    suf = " [-Rpass-analysis=kernel-resource-usage]"
    def remarks(name, scratch, vspill):
        return [pre + f"Function Name: {name}" + suf, pre + "    VGPRs: 220" + suf,
                pre + f"    ScratchSize [bytes/lane]: {scratch}" + suf, pre + "    SGPRs Spill: 0" + suf,
                pre + f"    VGPRs Spill: {vspill}" + suf]
    clean = remarks("_ZN3qfc18gemm_i8_dw4_kernelILi4ELi2ELi4ELi0EEEv", 0, 0)
    other = remarks("_ZN3qfc14gemm_i8_kernelILi128ELi128EEEv", 76, 18)   # not one of the guarded kernels
    bad = remarks("_ZN3qfc17gemm_i8_dw_kernelILi9ELi4ELi4ELi0ELb1EEEv", 76, 18)
    frag = build.NO_SPILL["gemm_i8.hip"]
    assert build._spilling_kernels(clean + other, frag) == []
    assert build._spilling_kernels(clean + bad + other, frag) == ["_ZN3qfc17gemm_i8_dw_kernelILi9ELi4ELi4ELi0ELb1EEEv"]
