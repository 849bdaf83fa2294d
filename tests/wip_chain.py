"""Parity of the persistent chain of decode layers (qfc_chain_*): every layer of a chain against the
CPU oracle applied to the tensors the previous layer stored, and bit for bit against the same layers
launched one by one."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_00232_amd import binding, synth

pytestmark = pytest.mark.gpu
TOL = 2e-3
DEV = "cuda"


def _group(fmt):
    return 32 if fmt == "w4g32" else 0


def _mk(name, K, N, fmt, seed, shrink=1.0):
    fc = synth.FC(name, K, N, fmt)
    wq, s = synth.weights(5000, seed, 0, fc)
    s = (s.astype(np.float32) * shrink).astype(s.dtype)
    return wq, s, binding.QuantLinear(wq, s, fmt)


def _chain(items, M):
    buf = torch.empty(binding.qfc_chain_size(len(items)), dtype=torch.uint8, device=DEV)
    return binding.qfc_chain_create(items, M, buf), buf


@pytest.mark.parametrize("M", [1, 2, 3, 4])
def test_chain_of_mixed_layers(M):
    """x0 -> A (int4 g32) -> B (int4 g32, gated output) -> C (int8, + residual x0) -> D (int4 per-channel)
    -> E (int4 per-channel, + residual yC): three runs of formats, every fusion part the chain takes."""
    print(f"chain mixed M={M}", flush=True)
    K0 = 256
    wa, sa, la = _mk("a", K0, 544, "w4g32", 1, 0.5)
    wb, sb, lb = _mk("b", 544, 2 * 352, "w4g32", 2, 0.5)
    wc, sc, lc = _mk("c", 352, K0, "w8c", 3, 0.05)
    wd, sd, ld = _mk("d", K0, 1056, "w4c", 4, 0.5)
    we, se, le = _mk("e", 1056, K0, "w4c", 5, 0.5)
    x0 = (synth.activations(5000, 0, M, M, K0) * np.float16(0.25)).astype(np.float16)
    T = lambda a: torch.from_numpy(a).to(DEV)
    E = lambda n: torch.full((M, n), 55.0, dtype=torch.float16, device=DEV)
    x0_d, ya, yb, yc, yd, ye = T(x0), E(544), E(352), E(K0), E(1056), E(K0)
    items = [binding.chain_item(la.handle, x0_d, ya),
             binding.chain_item(lb.handle, ya, yb, gated_output=True, activation=binding.QFC_ACT_GELU_TANH),
             binding.chain_item(lc.handle, yb, yc, residual=x0_d),
             binding.chain_item(ld.handle, yc, yd),
             binding.chain_item(le.handle, yd, ye, residual=yc)]
    chain, buf = _chain(items, M)
    N = lambda t: t.cpu().numpy()
    err = oracle.floored_rel_error
    for rep in range(2):  # the second run starts from the first run's counters
        binding.qfc_chain_run(chain)
        assert binding.qfc_chain_status(chain) == 0
        ra = oracle.fc_weight_only(x0, wa, sa, 32)
        assert err(N(ya), ra) <= TOL
        rb = oracle.gated_output(oracle.fc_weight_only(N(ya), wb, sb, 32), oracle.GELU_TANH)
        assert err(N(yb), rb) <= TOL
        rc = oracle.add_residual(oracle.fc_weight_only(N(yb), wc, sc, 0), x0)
        assert err(N(yc), rc) <= TOL
        rd = oracle.fc_weight_only(N(yc), wd, sd, 0)
        assert err(N(yd), rd) <= TOL
        re = oracle.add_residual(oracle.fc_weight_only(N(yd), we, se, 0), N(yc))
        assert err(N(ye), re) <= TOL
        # the same layers launched one by one give the same bits
        za, zb, zc, zd, ze = E(544), E(352), E(K0), E(1056), E(K0)
        binding.qfc_forward(la.handle, x0_d, za)
        binding.qfc_forward_fused(lb.handle, za, zb, activation=binding.QFC_ACT_GELU_TANH, gated_output=True)
        binding.qfc_forward_fused(lc.handle, zb, zc, residual=x0_d)
        binding.qfc_forward(ld.handle, zc, zd)
        binding.qfc_forward_fused(le.handle, zd, ze, residual=zc)
        torch.cuda.synchronize()
        for a, b in ((ya, za), (yb, zb), (yc, zc), (yd, zd), (ye, ze)):
            assert torch.equal(a, b)
        for t in (ya, yb, yc, yd, ye):
            t.fill_(55.0)
    binding.qfc_chain_destroy(chain)
    for l in (la, lb, lc, ld, le):
        l.close()


@pytest.mark.parametrize("fmt,N,K", [("w4g32", 9600, 8192), ("w8c", 9024, 4096), ("w4c", 70016, 1024)])
def test_chain_layers_with_more_rounds_than_workgroups(fmt, N, K):
    """Layers whose rounds exceed the resident grid (a workgroup walks through several rounds, asking
    for the next round's weights before the reduction of the current one), followed by a narrow layer."""
    M = 2
    print(f"chain rounds {fmt} N={N} K={K}", flush=True)
    w1, s1, l1 = _mk("wide", K, N, fmt, 11, 0.25)
    N2 = 48
    K2 = N if N % 32 == 0 else N - N % 32
    x = (synth.activations(5001, 0, 0, M, K) * np.float16(0.25)).astype(np.float16)
    xd = torch.from_numpy(x).to(DEV)
    y1 = torch.full((M, N), 55.0, dtype=torch.float16, device=DEV)
    items = [binding.chain_item(l1.handle, xd, y1)]
    if K2 == N:
        w2, s2, l2 = _mk("narrow", K2, N2, fmt, 12, 0.25)
        y2 = torch.full((M, N2), 55.0, dtype=torch.float16, device=DEV)
        items.append(binding.chain_item(l2.handle, y1, y2))
    chain, buf = _chain(items, M)
    binding.qfc_chain_run(chain)
    assert binding.qfc_chain_status(chain) == 0
    z1 = torch.empty_like(y1)
    binding.qfc_forward(l1.handle, xd, z1)
    torch.cuda.synchronize()
    assert torch.equal(y1, z1)
    rows = np.unique(np.concatenate([np.arange(0, N, 997), [N - 1]]))
    ref = oracle.fc_weight_only(x, w1[rows], s1[rows], _group(fmt))
    assert oracle.floored_rel_error(y1.cpu().numpy()[:, rows], ref) <= TOL
    if K2 == N:
        ref2 = oracle.fc_weight_only(y1.cpu().numpy(), w2, s2, _group(fmt))
        assert oracle.floored_rel_error(y2.cpu().numpy(), ref2) <= TOL
        l2.close()
    binding.qfc_chain_destroy(chain)
    l1.close()


def test_chain_llama_layer_shapes_sampled():
    """o -> gate_up (gated output) -> down (+ residual) -> qkv of the next layer at Llama-3.1-8B shapes,
    M = 1, four times in a row in one chain; sampled output channels against the oracle, all against the
    one-by-one launches."""
    M, hidden, ffn = 1, 4096, 14336
    specs = [("o", hidden, hidden), ("gate_up", hidden, 2 * ffn), ("down", ffn, hidden), ("qkv", hidden, 6144)]
    layers = {n: _mk(n, K, N, "w4g32", 20 + i, 0.25) for i, (n, K, N) in enumerate(specs)}
    x0 = (synth.activations(5002, 0, 0, M, hidden) * np.float16(0.5)).astype(np.float16)
    E = lambda n: torch.full((M, n), 55.0, dtype=torch.float16, device=DEV)
    xd = torch.from_numpy(x0).to(DEV)
    items, outs = [], []
    cur = xd
    for rep in range(4):
        h1, a, h2, qkv = E(hidden), E(ffn), E(hidden), E(6144)
        items += [binding.chain_item(layers["o"][2].handle, cur, h1, residual=cur),
                  binding.chain_item(layers["gate_up"][2].handle, h1, a, gated_output=True),
                  binding.chain_item(layers["down"][2].handle, a, h2, residual=h1),
                  binding.chain_item(layers["qkv"][2].handle, h2, qkv)]
        outs.append((cur, h1, a, h2, qkv))
        cur = h2
    chain, buf = _chain(items, M)
    print("chain llama shapes: run", flush=True)
    binding.qfc_chain_run(chain)
    assert binding.qfc_chain_status(chain) == 0
    N = lambda t: t.cpu().numpy()
    err = oracle.floored_rel_error
    rng = np.random.default_rng(5)
    for rep, (xin, h1, a, h2, qkv) in enumerate(outs):
        z1, za, z2, zq = E(hidden), E(ffn), E(hidden), E(6144)
        binding.qfc_forward_fused(layers["o"][2].handle, xin, z1, residual=xin)
        binding.qfc_forward_fused(layers["gate_up"][2].handle, z1, za, gated_output=True)
        binding.qfc_forward_fused(layers["down"][2].handle, za, z2, residual=z1)
        binding.qfc_forward(layers["qkv"][2].handle, z2, zq)
        torch.cuda.synchronize()
        for p, q in ((h1, z1), (a, za), (h2, z2), (qkv, zq)):
            assert torch.equal(p, q), rep
        if rep in (0, 3):
            wq, s, _ = layers["o"]
            c = np.sort(rng.choice(hidden, 64, replace=False))
            ref = oracle.add_residual(oracle.fc_weight_only(N(xin), wq[c], s[c], 32), N(xin)[:, c])
            assert err(N(h1)[:, c], ref) <= TOL
            wq, s, _ = layers["gate_up"]
            c = np.sort(rng.choice(ffn, 64, replace=False))
            both = np.concatenate([c, c + ffn])
            ref = oracle.gated_output(oracle.fc_weight_only(N(h1), wq[both], s[both], 32), oracle.SILU)
            assert err(N(a)[:, c], ref) <= TOL
            wq, s, _ = layers["down"]
            c = np.sort(rng.choice(hidden, 64, replace=False))
            ref = oracle.add_residual(oracle.fc_weight_only(N(a), wq[c], s[c], 32), N(h1)[:, c])
            assert err(N(h2)[:, c], ref) <= TOL
            wq, s, _ = layers["qkv"]
            c = np.sort(rng.choice(6144, 64, replace=False))
            ref = oracle.fc_weight_only(N(h2), wq[c], s[c], 32)
            assert err(N(qkv)[:, c], ref) <= TOL
    assert np.all(np.isfinite(N(outs[-1][4])))
    binding.qfc_chain_destroy(chain)
    for l in layers.values():
        l[2].close()


def test_chain_argument_checks_and_forced_expiry():
    wq, s, l = _mk("a", 256, 256, "w4g32", 31, 0.5)
    w8, s8, l8 = _mk("b", 256, 256, "w8c", 32, 0.05)
    xd = torch.from_numpy(synth.activations(5003, 0, 0, 4, 256)).to(DEV)
    y = torch.empty((4, 256), dtype=torch.float16, device=DEV)
    y2 = torch.empty((4, 256), dtype=torch.float16, device=DEV)
    buf = torch.empty(binding.qfc_chain_size(2), dtype=torch.uint8, device=DEV)
    with pytest.raises(binding.QfcError) as e:
        binding.qfc_chain_create([binding.chain_item(l.handle, xd, y)], 5, buf)
    assert e.value.code == binding.QFC_ERR_UNSUPPORTED
    with pytest.raises(binding.QfcError) as e:
        binding.qfc_chain_create([binding.chain_item(l.handle, xd, y, gate=xd)], 1, buf)
    assert e.value.code == binding.QFC_ERR_UNSUPPORTED
    with pytest.raises(binding.QfcError) as e:
        binding.qfc_chain_create([binding.chain_item(l.handle, xd, y, norm_gamma=xd)], 1, buf)
    assert e.value.code == binding.QFC_ERR_UNSUPPORTED
    with pytest.raises(binding.QfcError) as e:
        binding.qfc_chain_create([binding.chain_item(l.handle, xd, y)] * 3, 1, buf)
    assert e.value.code == binding.QFC_ERR_BUFFER_TOO_SMALL
    with pytest.raises(binding.QfcError) as e:
        binding.qfc_chain_create([binding.chain_item(l.handle, xd, y)], 1, buf[1:])
    assert e.value.code == binding.QFC_ERR_ALIGNMENT
    # A barrier wait bounded by zero microseconds expires at once: the kernel must still end, and
    # the flag must say that the outputs are not to be used.  Afterwards the chain works again.
    buf3 = torch.empty(binding.qfc_chain_size(3), dtype=torch.uint8, device=DEV)
    chain = binding.qfc_chain_create([binding.chain_item(l.handle, xd, y), binding.chain_item(l.handle, y, y2),
                                      binding.chain_item(l.handle, y2, y)], 4, buf3)
    print("chain forced expiry", flush=True)
    binding.qfc_tune(4, 0)
    try:
        binding.qfc_chain_run(chain)
        assert binding.qfc_chain_status(chain) in (0, 1)
    finally:
        binding.qfc_tune(4, 200000)
    binding.qfc_chain_run(chain)
    assert binding.qfc_chain_status(chain) == 0
    z, z2 = torch.empty_like(y), torch.empty_like(y)
    binding.qfc_forward(l.handle, xd, z)
    binding.qfc_forward(l.handle, z, z2)
    binding.qfc_forward(l.handle, z2, z)
    torch.cuda.synchronize()
    assert torch.equal(y, z) and torch.equal(y2, z2)
    binding.qfc_chain_destroy(chain)
    l.close()
    l8.close()
