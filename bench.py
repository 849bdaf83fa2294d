#!/usr/bin/env python3
"""Benchmark of the quantized fully-connected hot path on one MI355X.

A step is one pass of the decode hot path over the workload the headline metric
is quoted on: every linear layer of a Llama-3.1-8B-shaped decode step at M = 1
(32 layers x [QKV, O, gate+up, down] with int4 group-32 weights plus the int8
per-channel LM head: 129 qfc_forward calls, 4.456 GB of packed weights streamed
once).  Inputs are seeded synthetic tensors, resident in HBM before the timed
region.  The same run also times the prefill kernels (int8 MFMA product with
activation quantization and epilogue at M = 1024; fp16 MFMA product with int4
weights converted on the way to the matrix core at M = 2048), the M = 4 decode step, and the CPU oracle on a
bounded sample of the workload.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
MFMA_I8_PEAK_TOPS = 5000.0  # dense int8
MFMA_F16_PEAK_TFLOPS = 2500.0


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=20)
    p.add_argument("--warmup", type=int, default=10)
    p.add_argument("--layers", type=int, default=32, help="decoder layers of the decode step (32 = the full model)")
    p.add_argument("--skip-prefill", action="store_true")
    p.add_argument("--skip-cpu", action="store_true")
    p.add_argument("--traffic-probe", action="store_true",
                   help="for rocprofv3 --pmc runs: a few plain copies of a 1 GiB buffer (calibration of "
                        "FETCH_SIZE / WRITE_SIZE) followed by a few decode steps, then exit")
    p.add_argument("--probe-mfma", action="store_true",
                   help="measure what rate and shader clock a register-only MFMA loop holds with constant and "
                        "with random operands (context for the prefill rooflines), print it as JSON, exit")
    return p.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives or sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2505_00232_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    binding.lib()  # fail loudly if the HIP library is missing
    dev = "cuda"
    SEED = 1003

    if args.probe_mfma:
        out = {}
        for kind, name, ops in ((0, "int8 v_mfma_i32_32x32x32_i8", 65536.0), (1, "fp16 v_mfma_f32_32x32x16_f16", 32768.0)):
            for random_operands in (False, True):
                wgs, iters = 512, 20000  # two wavefronts per SIMD; about 10 ms per launch at full rate
                ticks = torch.zeros((wgs, 2), dtype=torch.int64, device=dev)
                launch = lambda: binding.qfc_probe_mfma(kind, random_operands, iters, wgs, ticks)
                for _ in range(15):  # 150 ms and more of the same load first
                    launch()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(5):
                    launch()
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / 5
                t = ticks.cpu().numpy().astype(np.float64)
                out[f"{name}, {'random' if random_operands else 'constant'} operands"] = {
                    "Tops": round(ops * 32 * iters * wgs * 4 / (ms * 1e-3) / 1e12, 1),
                    "shader_clock_MHz": round(float((t[:, 0] / (t[:, 1] / 100.0)).mean()), 1),
                    "ms_per_launch": round(ms, 3)}
        print(json.dumps({"probe": "register-only MFMA loop, 512 workgroups x 4 wavefronts, 640000 MFMAs per wavefront", "results": out}))
        return

    def event_ms(fn, reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def steady_ms(fn, reps, warm_ms=150.0, timed_ms=40.0):
        """Time of one call in the steady state of the chip's clock management.  Under matrix load the
        clock takes about 100 ms to settle (the first launches after an idle phase run 5 % slower than
        the steady state, the next few milliseconds up to 30 % slower), so the kernels that use the
        matrix cores are run for warm_ms first and then timed over at least timed_ms."""
        one = max(event_ms(fn, 3), 1e-3)
        for _ in range(min(20000, int(warm_ms / one) + 1)):
            fn()
        return event_ms(fn, max(reps, min(20000, int(timed_ms / one) + 1)))

    # ------------------------------------------------------------ decode step (config 3)
    t_setup = time.time()
    fcs = []
    for layer in range(args.layers):
        for i, fc in enumerate(synth.LLAMA_FCS_W4):
            fcs.append((layer, i, fc))
    fcs.append((args.layers, 4, synth.LLAMA_LM_HEAD))
    workspace = torch.empty(1 << 20, dtype=torch.uint8, device=dev)
    layers, x1, x4, x8 = [], [], [], []
    for layer, i, fc in fcs:
        wq, s = synth.weights(SEED, layer, i, fc)
        layers.append(binding.QuantLinear(wq, s, fc.fmt, max_m=8, workspace=workspace if fc.fmt == "w4g32" else None))
        x1.append(torch.from_numpy(synth.activations(SEED, layer, i, 1, fc.K)).to(dev))
        x4.append(torch.from_numpy(synth.activations(SEED, layer, i + 8, 4, fc.K)).to(dev))
        x8.append(torch.from_numpy(synth.activations(SEED, layer, i + 16, 8, fc.K)).to(dev))
        del wq, s
    setup_s = time.time() - t_setup

    def step_runner(xs, M, subset=None):
        idx = range(len(layers)) if subset is None else subset
        ys = [torch.empty((M, layers[j].N), dtype=torch.float16, device=dev) for j in idx]
        fb = binding.ForwardBatch([layers[j].handle for j in idx], [xs[j] for j in idx], ys, M)
        return fb, ys

    if args.traffic_probe:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        fbp, _ = step_runner(x1, 1)
        for _ in range(3):
            fbp.run()
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": "3 copies of 1 GiB, then 3 decode steps", "layers": args.layers}))
        return
    bytes_m1 = sum(synth.algorithmic_bytes(fc, 1) for _, _, fc in fcs)
    bytes_m4 = sum(synth.algorithmic_bytes(fc, 4) for _, _, fc in fcs)
    fb1, _ = step_runner(x1, 1)
    for _ in range(args.warmup):
        fb1.run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        fb1.run()
    torch.cuda.synchronize()
    wall_s = time.perf_counter() - t0
    ms_per_step = wall_s / args.steps * 1e3
    value = bytes_m1 / (ms_per_step * 1e-3) / 1e9

    # dominant kernel: the int4 group-32 decode kernel (128 of the 129 launches of a step)
    w4_idx = [j for j, (_, _, fc) in enumerate(fcs) if fc.fmt == "w4g32"]
    fb_w4, _ = step_runner(x1, 1, w4_idx)
    fb_w4.run()
    ms_w4 = event_ms(fb_w4.run, args.steps)
    bytes_w4 = sum(synth.algorithmic_bytes(fcs[j][2], 1) for j in w4_idx)
    launch_us = ms_w4 * 1e3 / len(w4_idx)
    achieved = bytes_w4 / (ms_w4 * 1e-3) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get("gemv_w4g32_m1_bytes_per_launch")
    roofline = {"bound": "hbm", "kernel": "gemv_kernel<M=1, W4G32> (decode, int4 group-32)",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "launches_per_step": len(w4_idx), "avg_launch_us": round(launch_us, 3),
                "algorithmic_bytes_per_launch": bytes_w4 // len(w4_idx)}

    # LM head (int8 per-channel decode kernel), and the M = 4 step
    lm_idx = [len(fcs) - 1]
    fb_lm, _ = step_runner(x1, 1, lm_idx)
    fb_lm.run()
    ms_lm = event_ms(fb_lm.run, args.steps)
    lm_gbs = synth.algorithmic_bytes(synth.LLAMA_LM_HEAD, 1) / (ms_lm * 1e-3) / 1e9
    fb4, _ = step_runner(x4, 4)
    fb4.run()
    ms_m4 = event_ms(fb4.run, max(3, args.steps // 2))
    fb8, _ = step_runner(x8, 8)
    fb8.run()
    ms_m8 = event_ms(fb8.run, max(3, args.steps // 2))
    bytes_m8 = sum(synth.algorithmic_bytes(fc, 8) for _, _, fc in fcs)
    extra = {
        "lm_head_w8c_m1": {"us": round(ms_lm * 1e3, 2), "GB/s": round(lm_gbs, 1), "frac_hbm_peak": round(lm_gbs / HBM_PEAK_GBS, 4)},
        "decode_m4": {"ms_per_step": round(ms_m4, 4), "GB/s": round(bytes_m4 / (ms_m4 * 1e-3) / 1e9, 1),
                      "tokens_per_s": round(4 / (ms_m4 * 1e-3), 1)},
        "decode_m8": {"ms_per_step": round(ms_m8, 4), "GB/s": round(bytes_m8 / (ms_m8 * 1e-3) / 1e9, 1),
                      "tokens_per_s": round(8 / (ms_m8 * 1e-3), 1)},
        "decode_m1_tokens_per_s": round(1 / (ms_per_step * 1e-3), 1),
        "setup_s": round(setup_s, 1),
    }

    # ------------------------------------------------------------ CPU oracle on a bounded sample
    cpu_baseline = None
    if not args.skip_cpu:
        import oracle
        cores = oracle.threads()
        n_layers = min(args.layers, 32)
        sample = [(l, i, fc) for (l, i, fc) in fcs if l < n_layers and fc.fmt == "w4g32"]
        tot_b, tot_t = 0, 0.0
        for layer, i, fc in sample:
            wq, s = synth.weights(SEED, layer, i, fc)
            x = synth.activations(SEED, layer, i, 1, fc.K)
            t0 = time.perf_counter()
            oracle.fc_weight_only(x, wq, s, 32)
            tot_t += time.perf_counter() - t0
            tot_b += synth.algorithmic_bytes(fc, 1)
            del wq, s
        cpu_baseline = {"value": round(tot_b / tot_t / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
                        "sample": f"{n_layers} decoder layers ({len(sample)} int4 FCs, {tot_b / 1e6:.0f} MB of packed weights) "
                                  f"of the same decode step at M=1, LM head left out; {tot_t:.1f} s of oracle time"}

    for l in layers:
        l.close()
    del layers, fb1, fb4, fb8, fb_w4, fb_lm
    torch.cuda.empty_cache()

    # ------------------------------------------------------------ configs 1 and 2: small decode workloads, cold cache
    # The weights of these two fit the 256 MB memory-side cache, so independent copies are rotated
    # (272 MB / 351 MB in flight) to keep every launch reading HBM.
    def rotating(fc_list, seed, copies, M=1):
        ls, xs = [], []
        for cpy in range(copies):
            for i, fc in enumerate(fc_list):
                wq, s = synth.weights(seed, cpy, i, fc)
                ls.append(binding.QuantLinear(wq, s, fc.fmt, max_m=8))
                xs.append(torch.from_numpy(synth.activations(seed, cpy, i, M, fc.K)).to(dev))
        ys = [torch.empty((M, l.N), dtype=torch.float16, device=dev) for l in ls]
        fb = binding.ForwardBatch([l.handle for l in ls], xs, ys, M)
        fb.run()
        ms = event_ms(fb.run, max(3, args.steps // 2)) / copies
        nbytes = sum(synth.algorithmic_bytes(fc, M) for fc in fc_list)
        for l in ls:
            l.close()
        return ms, nbytes

    # ------------------------------------------------------------ the paper's own schemes (section 4.2)
    # per-channel scales everywhere.  "8/4/4": int8 attention projections, int4 feed-forward and
    # embedding (= LM head) weights; "q8": int8 everywhere.  The same decode step, other formats.
    def decode_scheme(fc_list, seed, mode=None, xs=None):
        ls = []
        own_xs = xs is None
        xs = [] if own_xs else xs
        for layer, i, fc in fc_list:
            wq, s = synth.weights(seed, layer, i, fc)
            ls.append(binding.QuantLinear(wq, s, fc.fmt, max_m=8) if mode is None else
                      binding.QuantLinear(wq, s, fc.fmt, compute_mode=mode, max_m=8))
            if own_xs:
                xs.append(torch.from_numpy(synth.activations(seed, layer, i, 1, fc.K)).to(dev))
            del wq, s
        ys = [torch.empty((1, l.N), dtype=torch.float16, device=dev) for l in ls]
        fb = binding.ForwardBatch([l.handle for l in ls], xs, ys, 1)
        fb.run()
        ms = event_ms(fb.run, args.steps)
        nbytes = sum(synth.algorithmic_bytes(fc, 1) for _, _, fc in fc_list)
        for l in ls:
            l.close()
        del ls, ys, fb
        torch.cuda.empty_cache()
        return xs, {"ms_per_step": round(ms, 4), "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                    "frac_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                    "tokens_per_s": round(1 / (ms * 1e-3), 1), "algorithmic_bytes_per_step": nbytes}

    def as_fmt(fc, fmt):
        return synth.FC(fc.name, fc.K, fc.N, fmt)

    mixed = [(layer, i, as_fmt(fc, "w8c" if fc.name in ("qkv", "o") else "w4c"))
             for layer in range(args.layers) for i, fc in enumerate(synth.LLAMA_FCS_W4C)]
    mixed.append((args.layers, 4, as_fmt(synth.LLAMA_LM_HEAD, "w4c")))
    _, extra["decode_m1_mixed_8_4_4"] = decode_scheme(mixed, SEED + 200)
    q8 = [(layer, i, as_fmt(fc, "w8c")) for layer, i, fc in mixed]
    _, extra["decode_m1_q8"] = decode_scheme(q8, SEED + 300)
    # int4 per-channel weights in all four FCs, int8 per-channel LM head
    fcs_pc = [(layer, i, fc) for layer in range(args.layers) for i, fc in enumerate(synth.LLAMA_FCS_W4C)]
    fcs_pc.append((args.layers, 4, synth.LLAMA_LM_HEAD))
    xs_pc, extra["decode_m1_int4_per_channel"] = decode_scheme(fcs_pc, SEED + 100)
    # ... and with the paper's decode design: activations quantized to int8 inside the kernel,
    # integer accumulation (section 3.7)
    _, q = decode_scheme(fcs_pc, SEED + 100, mode=binding.QFC_COMPUTE_INT8_ACT_DECODE, xs=xs_pc)
    q.pop("algorithmic_bytes_per_step")
    extra["decode_m1_int4_per_channel_int8_activations"] = q
    _, q = decode_scheme(mixed, SEED + 200, mode=binding.QFC_COMPUTE_INT8_ACT_DECODE)
    q.pop("algorithmic_bytes_per_step")
    extra["decode_m1_mixed_8_4_4_int8_activations"] = q
    del xs_pc
    torch.cuda.empty_cache()

    ms_c1, b_c1 = rotating([synth.CFG1_FC], 1001, 512)
    ms_c2, b_c2 = rotating(synth.GEMMA_FCS_W4, 1002, 8)
    extra["config1_fc_512x1024_w8c_m1_cold"] = {"us_per_launch": round(ms_c1 * 1e3, 2), "GB/s": round(b_c1 / (ms_c1 * 1e-3) / 1e9, 1),
                                                "note": "latency-bound by construction (0.53 MB per launch)"}
    extra["config2_gemma2_2b_layer_m1_cold"] = {"us_per_layer": round(ms_c2 * 1e3, 2), "GB/s": round(b_c2 / (ms_c2 * 1e-3) / 1e9, 1),
                                                "frac_hbm_peak": round(b_c2 / (ms_c2 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    torch.cuda.empty_cache()

    # ------------------------------------------------------------ element-wise operators fused with the layer (section 3.6)
    # The feed-forward block of a Llama-3.1-8B decoder layer at M = 1: h + down(silu(gate) * up) with
    # [gate; up] = gate_up(x).  Fused: 2 launches (the gate+up layer multiplies its two halves in its
    # epilogue, the down projection adds the residual in its own).  Unfused: the same two layers with
    # three PyTorch element-wise kernels between and after them.  8 independent blocks (0.79 GB of
    # weights) are walked so that every launch reads HBM; both sequences are replayed from a captured
    # graph so that the host does not limit either.
    # Replays of a captured graph: the host does not limit sequences of many short launches.
    def graph_ms(fn, reps):
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        g.replay()
        return event_ms(g.replay, reps)


    def mlp_block():
        fc_gu, fc_dn = synth.LLAMA_FCS_W4[2], synth.LLAMA_FCS_W4[3]
        blocks = []
        for b in range(8):
            wq, s = synth.weights(SEED + 200, b, 2, fc_gu)
            gu = binding.QuantLinear(wq, s, fc_gu.fmt, max_m=8)
            wq, s = synth.weights(SEED + 200, b, 3, fc_dn)
            dn = binding.QuantLinear(wq, s, fc_dn.fmt, max_m=8)
            blocks.append((gu, dn))
            del wq, s
        x = torch.from_numpy(synth.activations(SEED + 200, 0, 0, 1, fc_gu.K)).to(dev)
        h = torch.from_numpy(synth.activations(SEED + 200, 0, 1, 1, fc_dn.N)).to(dev)
        y_gu = torch.empty((1, fc_gu.N), dtype=torch.float16, device=dev)
        gate, up = y_gu[:, : fc_dn.K], y_gu[:, fc_dn.K:]
        act = torch.empty((1, fc_dn.K), dtype=torch.float16, device=dev)
        y_dn = torch.empty((1, fc_dn.N), dtype=torch.float16, device=dev)
        out = torch.empty((1, fc_dn.N), dtype=torch.float16, device=dev)

        def fused():
            for gu, dn in blocks:
                binding.qfc_forward_fused(gu.handle, x, act, activation=binding.QFC_ACT_SILU, gated_output=True)
                binding.qfc_forward_fused(dn.handle, act, out, residual=h)

        def unfused():
            for gu, dn in blocks:
                binding.qfc_forward(gu.handle, x, y_gu)
                torch.nn.functional.silu(gate, inplace=False)  # warm the allocator; result unused
                torch.mul(torch.nn.functional.silu(gate), up, out=act)
                binding.qfc_forward(dn.handle, act, y_dn)
                torch.add(y_dn, h, out=out)

        def unfused_graphable():
            for gu, dn in blocks:
                binding.qfc_forward(gu.handle, x, y_gu)
                torch.mul(torch.nn.functional.silu(gate), up, out=act)
                binding.qfc_forward(dn.handle, act, y_dn)
                torch.add(y_dn, h, out=out)

        unfused()
        ms_f = graph_ms(fused, args.steps) / len(blocks)
        out_f = out.clone()
        ms_u = graph_ms(unfused_graphable, args.steps) / len(blocks)
        agree = bool(torch.allclose(out_f.float(), out.float(), rtol=4e-3, atol=4e-3 * float(out.float().abs().max())))
        for gu, dn in blocks:
            gu.close()
            dn.close()
        return {"fused_us_per_block": round(ms_f * 1e3, 2), "launches_fused": 2,
                "unfused_us_per_block": round(ms_u * 1e3, 2), "launches_unfused": 5,
                "outputs_agree": agree,
                "note": "Llama-3.1-8B feed-forward block, int4 group-32 weights, M=1; unfused = PyTorch silu, mul, add kernels"}

    extra["decode_m1_mlp_block_fused"] = mlp_block()
    torch.cuda.empty_cache()

    # RMS normalization with the residual connection and the next layer's activation quantization merged
    # in (the producer of the int8 prefill layers' input): M = 1024 token rows of a Llama-3.1-8B layer,
    # rotating buffers (8 x 25 MB in flight per call sequence)
    def rmsnorm_line(M=1024, K=4096, copies=12):
        xs = [torch.from_numpy(synth.activations(SEED + 300, cpy, 0, M, K)).to(dev) for cpy in range(copies)]
        rs = [torch.from_numpy(synth.activations(SEED + 300, cpy, 1, M, K)).to(dev) for cpy in range(copies)]
        gamma = torch.from_numpy(synth.activations(SEED + 300, 0, 2, 1, K)[0]).to(dev)
        xq = torch.empty((M, K), dtype=torch.int8, device=dev)
        sx = torch.empty((M,), dtype=torch.float32, device=dev)

        def run():
            for x, r in zip(xs, rs):
                binding.qfc_rmsnorm(x, gamma, 1e-5, 0.0, residual=r, h_out=r, xq=xq, sx=sx)

        run()
        ms = event_ms(run, max(3, args.steps // 2)) / copies
        nbytes = M * K * 7 + 2 * K + 4 * M  # x, residual in; residual stream and int8 codes out
        return {"us": round(ms * 1e3, 2), "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                "frac_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                "note": "h = x + residual, y = rmsnorm(h) * gamma, (xq, sx) = per-token int8 of y; one kernel, 7 B per element"}

    extra["rmsnorm_residual_quantize_m1024_k4096"] = rmsnorm_line()
    torch.cuda.empty_cache()

    # ------------------------------------------------------------ attention-side operators (sections 3.6 and 3.8)
    # One decode step of attention for Llama-3.1-8B (32 query heads, 8 KV heads of 128) per layer: rotary
    # embedding + layout transformation + cache append, then attention over the cache (K^T and V in the
    # role of weights).  Rotating caches so that every call reads HBM.
    def attention_line(B, n_ctx, copies):
        h_q, h_kv, d = 32, 8, 128
        C = n_ctx
        G, g = B * h_kv, h_q // h_kv
        shape = binding.AttnShape(B, h_q, h_kv, d, C)
        gen = torch.Generator(device=dev)
        gen.manual_seed(SEED + 400)
        kcs = [torch.randn((G, C, d), generator=gen, device=dev, dtype=torch.float32).half() for _ in range(copies)]
        vcs = [torch.randn((G, C // 64, d, 64), generator=gen, device=dev, dtype=torch.float32).half() for _ in range(copies)]
        qkv = torch.from_numpy(synth.activations(SEED + 400, 0, 0, B, (h_q + 2 * h_kv) * d)).to(dev).reshape(B, 1, -1)
        q = torch.empty((G, g, d), dtype=torch.float16, device=dev)
        out = torch.empty((G, g, d), dtype=torch.float16, device=dev)
        ws = torch.empty(binding.qfc_attention_workspace_size(shape, 1), dtype=torch.uint8, device=dev)

        def run():
            for kc, vc in zip(kcs, vcs):
                binding.qfc_rope_qkv(qkv, n_ctx - 1, shape, 500000.0, q, kc, vc)
                binding.qfc_attention(q, kc, vc, 1, n_ctx, shape, ws, out)

        run()
        ms = event_ms(run, max(3, args.steps // 2)) / copies
        nbytes = 2 * G * n_ctx * d * 2
        return {"us": round(ms * 1e3, 2), "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                "frac_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "kv_cache_MB": round(nbytes / 1e6, 1),
                "launches": 3}

    # One whole decoder layer of Llama-3.1-8B at M = 1 with 8192 cached positions, every operator from this
    # library: QKV with the RMS normalization, the rotary embedding and the cache append merged in, attention
    # (2 launches), O + residual, gate+up with the normalization merged in and gated output, down + residual:
    # 6 launches (7 with the rotary kernel on its own, timed beside it).  Four layers with their own weights
    # and caches are walked.
    def decoder_layer_line(n_ctx=8192, n_layers=4):
        hidden, h_q, h_kv, d, ffn = 4096, 32, 8, 128, 14336
        shape = binding.AttnShape(1, h_q, h_kv, d, n_ctx)
        gen = torch.Generator(device=dev)
        gen.manual_seed(SEED + 500)
        Ls = []
        for li in range(n_layers):
            ws4 = []
            for i, fc in enumerate(synth.LLAMA_FCS_W4):
                wq, s = synth.weights(SEED + 500, li, i, fc)
                ws4.append(binding.QuantLinear(wq, s, fc.fmt, max_m=8))
                del wq, s
            kc = torch.randn((h_kv, n_ctx, d), generator=gen, device=dev, dtype=torch.float32).half()
            vc = torch.randn((h_kv, n_ctx // 64, d, 64), generator=gen, device=dev, dtype=torch.float32).half()
            Ls.append((ws4, kc, vc))
        E = lambda *sh: torch.empty(sh, dtype=torch.float16, device=dev)
        h = torch.from_numpy(synth.activations(SEED + 500, 0, 0, 1, hidden)).to(dev)
        gamma = torch.ones(hidden, dtype=torch.float16, device=dev)
        qkv, q, att, h1, act, h2 = E(1, 1, (h_q + 2 * h_kv) * d), E(h_kv, h_q // h_kv, d), E(h_kv, h_q // h_kv, d), \
            E(1, hidden), E(1, ffn), E(1, hidden)
        wsp = torch.empty(binding.qfc_attention_workspace_size(shape, 1), dtype=torch.uint8, device=dev)

        table = binding.qfc_rope_table(shape, 500000.0, n_ctx)

        def run7():
            for (l_qkv, l_o, l_gu, l_dn), kc, vc in Ls:
                binding.qfc_forward_fused(l_qkv.handle, h, qkv.view(1, -1), norm_gamma=gamma, norm_eps=1e-5)
                binding.qfc_rope_qkv(qkv, n_ctx - 1, shape, 500000.0, q, kc, vc)
                binding.qfc_attention(q, kc, vc, 1, n_ctx, shape, wsp, att)
                binding.qfc_forward_fused(l_o.handle, att.view(1, h_q * d), h1, residual=h)
                binding.qfc_forward_fused(l_gu.handle, h1, act, activation=binding.QFC_ACT_SILU, gated_output=True,
                                          norm_gamma=gamma, norm_eps=1e-5)
                binding.qfc_forward_fused(l_dn.handle, act, h2, residual=h1)

        def run():
            for (l_qkv, l_o, l_gu, l_dn), kc, vc in Ls:
                binding.qfc_forward_qkv_rope(l_qkv.handle, h, n_ctx - 1, shape, table, q, kc, vc, norm_gamma=gamma, norm_eps=1e-5)
                binding.qfc_attention(q, kc, vc, 1, n_ctx, shape, wsp, att)
                binding.qfc_forward_fused(l_o.handle, att.view(1, h_q * d), h1, residual=h)
                binding.qfc_forward_fused(l_gu.handle, h1, act, activation=binding.QFC_ACT_SILU, gated_output=True,
                                          norm_gamma=gamma, norm_eps=1e-5)
                binding.qfc_forward_fused(l_dn.handle, act, h2, residual=h1)

        ms = graph_ms(run, args.steps) / n_layers
        ms7 = graph_ms(run7, args.steps) / n_layers
        nbytes = sum(synth.algorithmic_bytes(fc, 1) for fc in synth.LLAMA_FCS_W4) + 2 * h_kv * n_ctx * d * 2
        for ws4, _, _ in Ls:
            for l in ws4:
                l.close()
        return {"us_per_layer": round(ms * 1e3, 2), "launches": 6, "us_per_layer_with_separate_rotary_kernel": round(ms7 * 1e3, 2),
                "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                "frac_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                "bytes_per_layer_MB": round(nbytes / 1e6, 1),
                "note": "weights (int4 group-32) + KV cache (fp16) streamed once per layer; 32 such layers + LM head = one token"}

    extra["decode_layer_llama8b_m1_ctx8192"] = decoder_layer_line()
    torch.cuda.empty_cache()
    extra["decode_attention_llama8b_b1_ctx8192"] = attention_line(1, 8192, 12)
    extra["decode_attention_llama8b_b8_ctx8192"] = attention_line(8, 8192, 3)
    torch.cuda.empty_cache()

    # Causal attention of a Llama-3.1-8B layer over a 2048-token prompt (prefill: 8192 query rows per KV head)
    def prefill_attention_line(S=2048, h_q=32, h_kv=8, d=128):
        shape = binding.AttnShape(1, h_q, h_kv, d, S)
        gen = torch.Generator(device=dev)
        gen.manual_seed(SEED + 600)
        kc = torch.randn((h_kv, S, d), generator=gen, device=dev, dtype=torch.float32).half()
        vc = torch.randn((h_kv, S // 64, d, 64), generator=gen, device=dev, dtype=torch.float32).half()
        q = torch.randn((h_kv, S * (h_q // h_kv), d), generator=gen, device=dev, dtype=torch.float32).half()
        out = torch.empty_like(q)
        ws = torch.empty(binding.qfc_attention_workspace_size(shape, S), dtype=torch.uint8, device=dev)
        run = lambda: binding.qfc_attention(q, kc, vc, S, S, shape, ws, out)
        run()
        ms = steady_ms(run, args.steps)
        flops = 4.0 * d * h_q * (S * (S + 1) / 2)
        return {"us": round(ms * 1e3, 1), "Tflops_causal": round(flops / (ms * 1e-3) / 1e12, 1),
                "frac_mfma_fp16_peak": round(flops / (ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4)}

    if not args.skip_prefill:
        extra["prefill_attention_llama8b_s2048"] = prefill_attention_line()
        extra["prefill_attention_llama8b_s8192"] = prefill_attention_line(8192)
        extra["prefill_attention_gemma2_2b_s2048"] = prefill_attention_line(2048, 8, 4, 256)

    # ------------------------------------------------------------ prefill (configs 4 and 5)
    if not args.skip_prefill:
        def prefill(fc_list, M, seed, reps=10, mode=None):
            out, tot_ops, tot_ms = {}, 0, 0.0
            for i, fc in enumerate(fc_list):
                wq, s = synth.weights(seed, 0, i, fc)
                lay = binding.QuantLinear(wq, s, fc.fmt, compute_mode=mode, max_m=M)
                x = torch.from_numpy(synth.activations(seed, 0, i, M, fc.K)).to(dev)
                y = torch.empty((M, fc.N), dtype=torch.float16, device=dev)
                run = lambda: binding.qfc_forward(lay.handle, x, y)
                run()
                ms = steady_ms(run, reps)
                ops = synth.algorithmic_ops(fc, M)
                out[fc.name] = {"us": round(ms * 1e3, 1), "Tops": round(ops / (ms * 1e-3) / 1e12, 1)}
                tot_ops += ops
                tot_ms += ms
                lay.close()
                del wq, s, lay
            out["total"] = {"us": round(tot_ms * 1e3, 1), "Tops": round(tot_ops / (tot_ms * 1e-3) / 1e12, 1)}
            return out

        p8 = prefill(synth.LLAMA_FCS_W8, 1024, 1004)
        p8["roofline"] = {"bound": "mfma", "achieved": p8["total"]["Tops"], "peak": MFMA_I8_PEAK_TOPS, "unit": "TOP/s",
                          "frac": round(p8["total"]["Tops"] / MFMA_I8_PEAK_TOPS, 4),
                          "note": "activation quantization + int8 MFMA product + epilogue, Llama-3.1-8B layer, M=1024"}
        p16 = prefill(synth.GEMMA_FCS_W4, 2048, 1005)
        p16["roofline"] = {"bound": "mfma", "achieved": p16["total"]["Tops"], "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                           "frac": round(p16["total"]["Tops"] / MFMA_F16_PEAK_TFLOPS, 4),
                           "note": "int4 group-32 weights converted in registers on the way to the MFMA operand, fp16 MFMA, Gemma2-2B layer, M=2048"}
        extra["prefill_int8_m1024"] = p8
        extra["prefill_fp16_m2048"] = p16
        p16c = prefill(synth.GEMMA_FCS_W4C, 2048, 1105)
        extra["prefill_fp16_int4_per_channel_m2048"] = {"us": p16c["total"]["us"], "Tops": p16c["total"]["Tops"],
                                                        "frac_mfma_fp16_peak": round(p16c["total"]["Tops"] / MFMA_F16_PEAK_TFLOPS, 4)}
        # the paper's "8/4/4" feed-forward weights in its prefill stage: int8 activations x int4 per-channel weights
        p84 = prefill(synth.LLAMA_FCS_W4C, 1024, 1104, mode=binding.QFC_COMPUTE_INT8_ACT)
        extra["prefill_int8_w4c_m1024"] = {**{k: v for k, v in p84.items()},
                                           "frac_mfma_int8_peak": round(p84["total"]["Tops"] / MFMA_I8_PEAK_TOPS, 4),
                                           "note": "int8 activations x int4 per-channel weights -> int32, Llama-3.1-8B layer, M=1024"}
        mixed_us = p8["qkv"]["us"] + p8["o"]["us"] + p84["gate_up"]["us"] + p84["down"]["us"]
        mixed_ops = 2.0 * 1024 * sum(fc.N * fc.K for fc in synth.LLAMA_FCS_W8)
        extra["prefill_int8_mixed_8_4_4_m1024"] = {
            "us": round(mixed_us, 1), "Tops": round(mixed_ops / (mixed_us * 1e-6) / 1e12, 1),
            "frac_mfma_int8_peak": round(mixed_ops / (mixed_us * 1e-6) / 1e12 / MFMA_I8_PEAK_TOPS, 4),
            "note": "int8 attention projections + int4 feed-forward projections (the two layers above, summed), int8 activations"}
        # act(gate) * up merged into the gate+up layer's store phase (layer packed in pairs) against the
        # plain layer followed by PyTorch's element-wise kernels
        def gated_line(fc, M, seed, act):
            wq, s = synth.weights(seed, 0, 2, fc)
            x = torch.from_numpy((synth.activations(seed, 0, 2, M, fc.K) * np.float16(0.125)).astype(np.float16)).to(dev)
            y = torch.empty((M, fc.N), dtype=torch.float16, device=dev)
            yg = torch.empty((M, fc.N // 2), dtype=torch.float16, device=dev)
            out = torch.empty_like(yg)
            half = fc.N // 2
            res = {}
            for gated in (False, True):
                lay = binding.QuantLinear(wq, s, fc.fmt, max_m=M, gated_pairs=gated)
                if gated:
                    fn = lambda: binding.qfc_forward_fused(lay.handle, x, yg, activation=act, gated_output=True)
                else:
                    def fn():
                        binding.qfc_forward(lay.handle, x, y)
                        torch.mul(torch.nn.functional.silu(y[:, :half]), y[:, half:], out=out)
                fn()
                res["fused_us" if gated else "unfused_us"] = round(steady_ms(fn, 10) * 1e3, 1)
                if not gated:
                    plain_only = lambda: binding.qfc_forward(lay.handle, x, y)
                    res["plain_layer_us"] = round(steady_ms(plain_only, 10) * 1e3, 1)
                lay.close()
                del lay, fn
            return res

        extra["prefill_gated_output"] = {
            "int8_llama_gate_up_m1024": gated_line(synth.LLAMA_FCS_W8[2], 1024, 1004, binding.QFC_ACT_SILU),
            "fp16_gemma_gate_up_m2048": gated_line(synth.GEMMA_FCS_W4[2], 2048, 1005, binding.QFC_ACT_SILU),
            "note": "act(gate) * up in the store phase of the product kernel (layer packed in pairs) vs the plain layer + PyTorch silu and mul kernels; plain_layer_us = the plain layer alone"}
        lm = prefill([synth.GEMMA_LM_HEAD], 2048, 1005, reps=3)
        extra["prefill_int8_lm_head_m2048"] = {"us": lm["total"]["us"], "Tops": lm["total"]["Tops"],
                                               "frac_mfma_int8_peak": round(lm["total"]["Tops"] / MFMA_I8_PEAK_TOPS, 4),
                                               "note": "2304 -> 256000, int8 per-channel; 1.05 GB of the traffic is the fp16 output"}

    line = {
        "metric": "decode quantized-FC HBM GB/s", "value": round(value, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"llama-3.1-8b decode step, all linear layers, M=1: {args.layers} x (qkv, o, gate_up, down) "
                               "int4 group-32 fp16-scale + lm_head int8 per-channel",
                   "launches_per_step": len(fcs), "algorithmic_bytes_per_step": bytes_m1},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "roofline": roofline, "cpu_baseline": cpu_baseline, "extra": extra,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
