#!/usr/bin/env python3
"""Benchmark of the QZO hot path on one MI355X.

A step is one full iteration of Algorithm 1 (two perturbed forwards, SPSA
scalar + clipping, scale update) on the Llama-2-7B-shaped synthetic model
(32 layers, d 4096, FFN 11008, vocab 32000, int4 group-128 RTN weights with
bf16 scales, batch 16 x seq 512 uniform tokens).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA = 2.5e15     # MI355X dense bf16, flop/s
PROF_STRIDE = 5
PEAK_HBM = 8.0e12           # bytes/s


def cpu_baseline(shape, tokens_sample=1536):
    """The oracle on the host cores, on a bounded sample of the same workload:
    `tokens_sample` tokens through ONE decoder layer's four perturbed linears and
    the lm_head at the real widths, and the update of one layer's scales;
    extrapolated to n_layers and two passes.  Attention, norms and the other
    elementwise work are left out (they are under 3 % of the flops)."""
    import numpy as np
    from oracle import oracle as O
    from paper_2505_13430_amd import synth
    rng = np.random.default_rng(0)
    d, V, L = shape["d_model"], shape["vocab"], shape["n_layers"]
    t_lin = 0.0
    t_upd = 0.0
    row = 0
    for name, N, K in synth.quantized_linears(shape):
        x, qp, s = synth.linear_case(tokens_sample, N, K, seed=N + K)
        t0 = time.perf_counter()
        se = O.effective_scales(s, row, 1, np.float32(1e-3))
        O.qlinear(x, qp, se)
        t_lin += time.perf_counter() - t0

        class Seg:
            pass
        sg = Seg()
        sg.name, sg.offset, sg.rows, sg.G, sg.row_base = name, 0, N, K // 128, row
        m = O.Model(shape={}, tensors=[], names=[], scales=s.reshape(-1), segments=[sg])
        t0 = time.perf_counter()
        O.update_scales(m, 1, 1e-5, 10.0)
        t_upd += time.perf_counter() - t0
        row += N
    hx = rng.standard_normal((tokens_sample, d))
    lm = synth.bf16_exact(rng.standard_normal((V, d)).astype(np.float32) * 0.02)
    t0 = time.perf_counter()
    O.linear(hx, lm)
    t_lm = time.perf_counter() - t0
    step_s = 2 * (L * t_lin + t_lm) + L * t_upd
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": tokens_sample / step_s, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{tokens_sample} tokens through one decoder layer's 4 perturbed linears + lm_head "
                      f"at full width and one layer's scale update, measured {t_lin + t_lm + t_upd:.1f} s, "
                      f"extrapolated x{L} layers x2 passes; attention/norms omitted"}


def measured_traffic(key):
    """HBM bytes per launch from the committed rocprofv3 counter summary, or None."""
    path = os.path.join(ROOT, "profiles", "w4a16_gemm_and_update_hbm_traffic.md")
    try:
        for line in open(path):
            if line.startswith(key + ":"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def other_config_memory(torch, qb, synth, DeviceModel, tok_seed=5678):
    """Total device memory of the Llama-2-13B-shaped workload (batch 8 x 512), both quantizer variants:
    two full QZO steps each, outside any timed region; peak bytes torch's allocator handed out
    (weights, scales, workspace, tokens)."""
    out = {}
    shape = dict(synth.SHAPES["llama-2-13b"])
    tok = torch.from_numpy(synth.tokens(shape, tok_seed)).cuda()
    for name in ("int4_g128", "codebook_16bit_per_8"):
        torch.cuda.empty_cache()
        torch.cuda.reset_peak_memory_stats()
        base = torch.cuda.memory_allocated()
        dm = (DeviceModel.synthetic_codebook(shape, seed=1234, device="cuda:0") if name.startswith("codebook")
              else DeviceModel.synthetic(shape, seed=1234, device="cuda:0"))
        resident = torch.cuda.memory_allocated() - base
        t0 = time.perf_counter()
        for i in range(2):
            dm.step(tok, 1 + i, 1e-3, 1e-7, 100.0)
        torch.cuda.synchronize()
        res = qb.read_step_result(dm.result)
        out[name] = {"peak_GiB": torch.cuda.max_memory_allocated() / 2 ** 30,
                     "model_GiB": resident / 2 ** 30, "ms_per_step_untimed": (time.perf_counter() - t0) / 2 * 1e3,
                     "loss_plus": res["loss_plus"], "status": res["status"]}
        dm.close()
        del dm
    return out


def fused_leg(torch, qb, dm, tok, steps, n_lin, eps, eta, clip):
    """The same workload with every int4 linear on the fused dequantizing GEMM (int4 unpack and scale
    perturbation inside the LDS-staged weight tile): a short timed leg of its own."""
    dm.set_int4_path(1)
    dm.step(tok, 50, eps, eta, clip)
    torch.cuda.synchronize()
    qb.qzo_profile_stride(PROF_STRIDE)
    qb.qzo_profile_begin(steps * (n_lin + 64))
    t0 = time.perf_counter()
    for i in range(steps):
        dm.step(tok, 60 + i, eps, eta, clip)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    g = qb.qzo_profile_collect(qb.PROFILE_KINDS["w4a16_gemm"])
    rate = g["work"] / (g["total_ms"] * 1e-3)
    dm.set_int4_path(0)
    return {"bound": "mfma", "kernel": "gemm_kernel<0,false,4,2> (fused perturbed W4A16 GEMM)",
            "achieved": rate / 1e12, "peak": PEAK_BF16_MFMA / 1e12, "unit": "TFLOP/s", "frac": rate / PEAK_BF16_MFMA,
            "traffic": measured_traffic("traffic_bytes_per_launch_gemm_qkv_fused"),
            "launches": g["launches"], "avg_launch_ms": g["total_ms"] / max(g["launches"], 1),
            "steps": steps, "ms_per_step": dt / steps * 1e3}


def mfma_ceiling(torch, qb, iters=60000):
    """bf16 MFMA rate the board sustains with nothing but MFMAs in flight (TFLOP/s), with
    all-zero and with pseudo-random register operands; timed with events on the current stream."""
    sink = torch.empty(512 * 512, dtype=torch.float32, device="cuda:0")
    out = {}
    for name, rnd in (("zero_operands", False), ("random_operands", True)):
        qb.qzo_debug_mfma_rate(2000, rnd, sink)           # warm-up
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        wgs = qb.qzo_debug_mfma_rate(iters, rnd, sink)
        e1.record()
        torch.cuda.synchronize()
        out[name] = wgs * 8 * 16 * 32768.0 * iters / (e0.elapsed_time(e1) * 1e-3) / 1e12
    return out


def probe(torch, qb):
    """Launches for rocprofv3 counter runs: a plain copy of known size (256 MiB read +
    256 MiB written) that calibrates the HBM counters, the perturbed linear at the Llama-2-7B
    qkv shape (M 8192, N 12288, K 4096) three ways (the fused dequantizing GEMM; the expansion
    of the perturbed weights to bf16; the plain bf16 GEMM on them), the scale update over 50,593,792 scales, and the
    matrix-pipe rate probe with zero and with random operands (engine-clock comparison)."""
    dev = "cuda:0"
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    src = torch.randint(0, 256, (256 << 20,), generator=g, device=dev, dtype=torch.uint8)
    dst = torch.empty_like(src)
    M, N, K = 8192, 12288, 4096
    x = torch.randn(M, K, generator=g, device=dev).to(torch.bfloat16)
    q = torch.randint(0, 256, (N, K // 2), generator=g, device=dev, dtype=torch.uint8)
    s = (torch.rand(N, K // 128, generator=g, device=dev) * 0.015 + 0.005).to(torch.bfloat16)
    y = torch.empty(M, N, dtype=torch.bfloat16, device=dev)
    arena = (torch.rand(1581056, 32, generator=g, device=dev) * 0.01 + 0.003).to(torch.bfloat16)
    se = torch.empty(N, K // 128, dtype=torch.float32, device=dev)
    wexp = torch.empty(N, K, dtype=torch.bfloat16, device=dev)
    torch.cuda.synchronize()
    for _ in range(3):
        dst.copy_(src)
        torch.cuda.synchronize()
        qb.qzo_dequant_gemm(x, q, s, 0, 7, 1e-3, 1, y)
        torch.cuda.synchronize()
        qb.qzo_int4_expand(q, s, None, 0, 7, 1e-3, 1, se, wexp)
        torch.cuda.synchronize()
        qb.qzo_debug_bf16_gemm(x, wexp, y, 2)
        torch.cuda.synchronize()
        qb.qzo_apply_update(arena, 0, 7, 1e-7, 10.0)
        torch.cuda.synchronize()
    sink = torch.empty(512 * 512, dtype=torch.float32, device=dev)
    for rnd in (False, True):
        for _ in range(3):
            qb.qzo_debug_mfma_rate(20000, rnd, sink)
            torch.cuda.synchronize()
    print(json.dumps({"probe": "copy 2x268435456 B, fused gemm / expansion / plain gemm 8192x12288x4096, update 50593792 scales, "
                               "mfma rate 20000 iters x 16 MFMAs per wavefront (zero, then random operands)"}))


def probe_few(torch, qb):
    """Launches for rocprofv3 counter runs of the few-token kernel: the perturbed linear at the
    Llama-2-7B qkv shape with 16 tokens (M 16, N 12288, K 4096), six times."""
    dev = "cuda:0"
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    M, N, K = 16, 12288, 4096
    x = torch.randn(M, K, generator=g, device=dev).to(torch.bfloat16)
    q = torch.randint(0, 256, (N, K // 2), generator=g, device=dev, dtype=torch.uint8)
    s = (torch.rand(N, K // 128, generator=g, device=dev) * 0.015 + 0.005).to(torch.bfloat16)
    y = torch.empty(M, N, dtype=torch.bfloat16, device=dev)
    for _ in range(6):
        qb.qzo_dequant_gemm(x, q, s, 0, 7, 1e-3, 1, y)
        torch.cuda.synchronize()
    print(json.dumps({"probe": "few-token perturbed linear 16x12288x4096, 6 launches"}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="llama-2-7b")
    ap.add_argument("--variant", default="int4", choices=["int4", "int4-zp", "nf4", "codebook"],
                    help="int4 group-128 scales (the metric's configuration), the same with per-group "
                         "zero-points, NormalFloat-4 blocks of 64, or the codebook variant with per-channel "
                         "scales (no cpu_baseline leg)")
    ap.add_argument("--fused", action="store_true",
                    help="int4 variants: always the fused dequantizing GEMM (default: expand-then-multiply "
                         "for linears with enough tokens per pass, about 2700-4300 at the 7B widths)")
    ap.add_argument("--expanded", action="store_true",
                    help="int4 variants: always expand-then-multiply, whatever the token count")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time its replays (every replay repeats the "
                         "same seed; no per-kernel events, so the roofline fields are null)")
    ap.add_argument("--joint", action="store_true",
                    help="joint mode: the un-quantized parameters are perturbed and updated too (SPSA)")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size")
    ap.add_argument("--seq", type=int, default=0, help="override the workload's sequence length")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-other", action="store_true",
                    help="skip the untimed Llama-2-13B-shaped memory report (two variants, two steps each)")
    ap.add_argument("--probe-few", action="store_true",
                    help="counter probe: the few-token W4A16 kernel at 16 x 12288 x 4096, six launches")
    ap.add_argument("--probe", action="store_true",
                    help="counter probe: a plain 256 MiB copy, the qkv-shaped W4A16 GEMM and the "
                         "7B-sized scale update, three launches each (for rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2505_13430_amd import binding as qb
    from paper_2505_13430_amd import synth
    from paper_2505_13430_amd.model import DeviceModel

    if args.probe_few:
        probe_few(torch, qb)
        return
    if args.probe:
        probe(torch, qb)
        return
    shape = dict(synth.SHAPES[args.workload])
    if args.batch:
        shape["batch"] = args.batch
    if args.seq:
        shape["seq"] = args.seq
    B, S = shape["batch"], shape["seq"]
    torch.cuda.set_device(0)
    codebook = args.variant == "codebook"
    # the counters were read on this one
    main_cfg = (args.workload == "llama-2-7b" and args.variant == "int4" and not args.joint
                and not args.batch and not args.seq)
    few_tokens = B * S <= 64 and args.variant in ("int4", "int4-zp")   # the weight-streaming path
    if codebook:
        dm = DeviceModel.synthetic_codebook(shape, seed=1234, device="cuda:0")
    else:
        dm = DeviceModel.synthetic(shape, seed=1234, device="cuda:0", asym=args.variant == "int4-zp",
                                   nf4=args.variant == "nf4")
    tok = torch.from_numpy(synth.tokens(shape, 5678)).cuda()
    eps, eta, clip = 1e-3, 1e-7, 100.0
    stream = torch.cuda.current_stream()
    if not codebook and args.variant != "nf4":
        dm.set_int4_path(1 if args.fused else (2 if args.expanded else 0))
    if args.joint:
        dm.enable_joint()
        plain_step = dm.step_joint
        dm.step = lambda tok, seed, eps, eta, clip: plain_step(tok, seed, eps, eta, eta, clip)

    for i in range(args.warmup):
        dm.step(tok, 1 + i, eps, eta, clip)
    torch.cuda.synchronize()

    n_lin = 4 * shape["n_layers"] * 2
    if args.graph:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            dm.step(tok, 100, eps, eta, clip)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        out = {"metric": "qzo_step_tokens_per_s", "value": B * S * args.steps / dt, "unit": "tokens/s",
               "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
               "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
               "data": "synthetic",
               "config": {"workload": f"{args.workload}-shaped decoder, {args.variant}, full QZO step replayed "
                                      f"from a captured HIP graph (same seed every replay)",
                          "batch": B, "seq_len": S, "eps": eps, "eta": eta, "clip": clip},
               "last_step": qb.read_step_result(dm.result), "roofline": None, "cpu_baseline": None}
        dm.close()
        print(json.dumps(out))
        return
    # every PROF_STRIDE-th launch of each kernel class is bracketed by HIP events on the step's stream
    # (odd, so that the four linears of a layer are sampled in turn); bracketing every launch costs
    # about 3 % of the step
    qb.qzo_profile_stride(PROF_STRIDE)
    qb.qzo_profile_begin(args.steps * (2 * n_lin + 2 * shape["n_layers"] + 16))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        dm.step(tok, 100 + i, eps, eta, clip)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = {k: qb.qzo_profile_collect(v) for k, v in qb.PROFILE_KINDS.items()}
    res = qb.read_step_result(dm.result)
    peak_bytes = torch.cuda.max_memory_allocated()
    # outside the timed region: one more step, to report how many stored scales it moved
    # (16-bit storage rounds most of the paper-sized updates away)
    before = dm.scales.clone()
    dm.step(tok, 10_000, eps, eta, clip)
    torch.cuda.synchronize()
    changed = float((dm.scales.view(torch.int16) != before.view(torch.int16)).float().mean().item())
    # ... and by the largest update the clipping of Eq. 6 admits (d' = C), applied directly
    before.copy_(dm.scales)
    dm.apply_update(10_001, eta, clip)
    torch.cuda.synchronize()
    changed_clip = float((dm.scales.view(torch.int16) != before.view(torch.int16)).float().mean().item())
    del before

    # whether the linears were written out as perturbed bf16 matrices first (most of them, when mixed)
    expanded = prof["expand"]["launches"] * 2 > prof["w4a16_gemm"]["launches"]
    ms_per_step = dt / args.steps * 1e3
    steps_per_s = args.steps / dt
    g = prof["w4a16_gemm"]
    gemm_flops_s = g["work"] / (g["total_ms"] * 1e-3)
    # the W4A16 linear as a whole: the matrix kernel plus, on the expanded route, the passes that write the
    # perturbed scales and the perturbed weights out
    linear_flops_s = g["work"] / ((g["total_ms"] + prof["expand"]["total_ms"]) * 1e-3)
    u = prof["scale_update"]
    upd_bytes_s = u["work"] / (u["total_ms"] * 1e-3) if u["total_ms"] > 0 else 0.0
    out = {
        "metric": "qzo_step_tokens_per_s",
        "value": B * S * steps_per_s,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}-shaped decoder, "
                               f"{'16-bit codes per 8 weights + fp16 channel scales' if codebook else 'int4 g128 RTN'}"
                               f"{' with zero-points' if args.variant == 'int4-zp' else ''}"
                               f"{' -> NormalFloat-4 blocks of 64 instead' if args.variant == 'nf4' else ''}"
                               f", full QZO step "
                               f"(2 perturbed forwards + DDC + scale update"
                               f"{'; un-quantized parameters perturbed and updated jointly' if args.joint else ''})",
                   "batch": B, "seq_len": S, "eps": eps, "eta": eta, "clip": clip},
        "steps_per_s": steps_per_s,
        "forward_tokens_per_s": 2 * B * S * steps_per_s,
        "last_step": res,
        "scales_changed_frac": changed,
        "scales_changed_frac_at_clip": changed_clip,
        "roofline": {"bound": "mfma",
                     "kernel": "wide_gemm_kernel (qkv, o, down) and gemm_kernel<1,false,4,3> (gate/up with SwiGLU): plain bf16 GEMM on the expanded perturbed weights"
                     if expanded
                     else ("gemm_kernel<2,...> (codebook GEMM, perturbed channel scales)" if codebook
                           else "gemm_kernel<0,false,4,2> (fused perturbed W4A16 GEMM)"),
                     "achieved": linear_flops_s / 1e12, "peak": PEAK_BF16_MFMA / 1e12,
                     "unit": "TFLOP/s", "frac": linear_flops_s / PEAK_BF16_MFMA,
                     "achieved_note": "2MNK of the perturbed linears over the time of their matrix kernel PLUS "
                                      "the expansion passes (perturbed scales, perturbed bf16 weights) they depend on",
                     "matrix_kernel_alone_TFLOPs": gemm_flops_s / 1e12,
                     "traffic": measured_traffic("traffic_bytes_per_launch_gemm_qkv" if expanded else
                                                 "traffic_bytes_per_launch_gemm_qkv_fused")
                     if args.workload == "llama-2-7b" and args.variant == "int4" and not args.batch and not args.seq
                     else None,
                     "traffic_note": "bytes of one qkv-shaped launch (8192x12288x4096), FETCH_SIZE + WRITE_SIZE "
                                     "scaled by a plain copy; algorithmic " + ("3.69e8" if expanded else "2.94e8"),
                     "launches": g["launches"], "avg_launch_ms": g["total_ms"] / max(g["launches"], 1),
                     "flops_per_launch_avg": g["work"] / max(g["launches"], 1),
                     "mfma_only_measured_TFLOPs": mfma_ceiling(torch, qb)},
        "kernels": {
            k: {"total_ms_per_step": v["total_ms"] * PROF_STRIDE / args.steps,
                "launches_per_step": v["launches"] * PROF_STRIDE / args.steps, "bracketed_launches": v["launches"]}
            for k, v in prof.items()},
        "kernels_note": f"every {PROF_STRIDE}th launch of a class is timed; per-step totals are scaled up by that",
        "scale_update": {"bound": "hbm", "achieved": upd_bytes_s / 1e9, "peak": PEAK_HBM / 1e9,
                         "unit": "GB/s", "frac": upd_bytes_s / PEAK_HBM,
                         "avg_launch_ms": u["total_ms"] / max(u["launches"], 1),
                         "bytes_per_launch": u["work"] / max(u["launches"], 1),
                         "traffic": measured_traffic("traffic_bytes_per_launch_scale_update")
                         if main_cfg else None},
        "device_memory_GiB": peak_bytes / 2 ** 30,
    }
    if args.joint:
        out["dense_parameters"] = int(dm.dense_master.numel())
    if few_tokens:
        # every int4 weight and scale is read once per launch: the roof is HBM
        wbytes = sum(N * K // 2 + N * K // 64 for _, N, K in synth.quantized_linears(shape))
        per_launch = wbytes / 4.0
        out["roofline"] = {"bound": "hbm", "kernel": "skinny_gemm_kernel + skinny_reduce_kernel (few-token W4A16 linear)",
                           "achieved": per_launch / (g["total_ms"] / max(g["launches"], 1) * 1e-3) / 1e9,
                           "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                           "frac": per_launch / (g["total_ms"] / max(g["launches"], 1) * 1e-3) / PEAK_HBM,
                           "traffic": None, "launches": g["launches"],
                           "avg_launch_ms": g["total_ms"] / max(g["launches"], 1),
                           "bytes_per_launch_avg": per_launch}
    if main_cfg and not args.fused and not args.expanded:
        out["roofline_fused_kernel"] = fused_leg(torch, qb, dm, tok, max(2, args.steps // 4), n_lin, eps, eta, clip)
    dm.close()
    del dm
    if main_cfg and not args.no_other:
        out["llama_2_13b_shape_memory"] = other_config_memory(torch, qb, synth, DeviceModel)
    if not args.no_cpu and not codebook and main_cfg:
        out["cpu_baseline"] = cpu_baseline(shape)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
