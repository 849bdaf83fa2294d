"""The entry point that allocates nothing (qfc_forward_static) against qfc_forward, through the
C ABI: two calls in a row on the same GPU, the second with a smaller input, so that whatever the
first call left in the library's static scratch array lies under the second one."""
import numpy as np
import pytest
import torch

from paper_2505_00232_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _bits(t):
    return t.cpu().numpy().view(np.uint16)


def test_static_scratch_entry_point_matches_qfc_forward():
    fc = synth.FC("t", 2304, 1000, "w8c")
    wq, sw = synth.weights(9100, 0, 0, fc)
    layer = binding.QuantLinear(wq, sw, "w8c", compute_mode=binding.QFC_COMPUTE_INT8_ACT, max_m=300)
    mem0 = torch.cuda.memory_allocated()
    for M in (300, 100, 8, 300):  # int8 prefill twice (larger, then smaller), a decode call, prefill again
        print(f"static scratch M={M}", flush=True)
        x = torch.from_numpy(synth.activations(9100, M, 1, M, fc.K)).to(DEV)
        y_ref = torch.empty((M, fc.N), dtype=torch.float16, device=DEV)
        y = torch.full((M, fc.N), 123.0, dtype=torch.float16, device=DEV)
        binding.qfc_forward(layer.handle, x, y_ref)
        binding.qfc_forward_static(layer.handle, x, y)
        torch.cuda.synchronize()
        # same kernels on the same inputs: the bound of the floating-point path holds with zero error
        assert np.array_equal(_bits(y), _bits(y_ref)), M
        del x, y, y_ref
    assert torch.cuda.memory_allocated() == mem0

    # a handle with no usable workspace bound: qfc_forward refuses, the static entry point does not care
    tiny = torch.zeros(256, dtype=torch.uint8, device=DEV)
    binding.qfc_bind_workspace(layer.handle, tiny)
    x = torch.from_numpy(synth.activations(9100, 64, 2, 64, fc.K)).to(DEV)
    y = torch.empty((64, fc.N), dtype=torch.float16, device=DEV)
    with pytest.raises(binding.QfcError) as e:
        binding.qfc_forward(layer.handle, x, y)
    assert e.value.code == binding.QFC_ERR_BUFFER_TOO_SMALL
    binding.qfc_forward_static(layer.handle, x, y)
    binding.qfc_bind_workspace(layer.handle, layer.workspace)
    y_ref = torch.empty_like(y)
    binding.qfc_forward(layer.handle, x, y_ref)
    torch.cuda.synchronize()
    assert np.array_equal(_bits(y), _bits(y_ref))
    layer.close()

    # the other formats use no scratch: same bits as qfc_forward, decode and fp16 prefill
    fc4 = synth.FC("t", 512, 264, "w4g32")
    wq, s = synth.weights(9101, 0, 0, fc4)
    l4 = binding.QuantLinear(wq, s, "w4g32", max_m=64)
    for M in (64, 3):
        x = torch.from_numpy(synth.activations(9101, M, 1, M, fc4.K)).to(DEV)
        y, y_ref = (torch.empty((M, fc4.N), dtype=torch.float16, device=DEV) for _ in range(2))
        binding.qfc_forward(l4.handle, x, y_ref)
        binding.qfc_forward_static(l4.handle, x, y)
        torch.cuda.synchronize()
        assert np.array_equal(_bits(y), _bits(y_ref)), M
    l4.close()


def test_static_scratch_limit_is_an_error_before_any_launch():
    fc = synth.FC("t", 14336, 64, "w8c")
    wq, sw = synth.weights(9102, 0, 0, fc)
    layer = binding.QuantLinear(wq, sw, "w8c", compute_mode=binding.QFC_COMPUTE_INT8_ACT, max_m=16)
    M = 1280  # 1280 x 14336 bytes of codes exceed the 16 MiB array
    assert binding.qfc_workspace_size(layer.handle, M) > binding.QFC_STATIC_SCRATCH_BYTES
    assert binding.qfc_workspace_size(layer.handle, 1024) <= binding.QFC_STATIC_SCRATCH_BYTES
    x = torch.zeros((M, fc.K), dtype=torch.float16, device=DEV)
    y = torch.full((M, fc.N), 5.0, dtype=torch.float16, device=DEV)
    with pytest.raises(binding.QfcError) as e:
        binding.qfc_forward_static(layer.handle, x, y)
    assert e.value.code == binding.QFC_ERR_SCRATCH_LIMIT
    torch.cuda.synchronize()
    assert bool((y == 5.0).all())  # nothing was launched
    layer.close()
