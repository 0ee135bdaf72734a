#!/usr/bin/env python3
"""Benchmark of the fused dequantise-and-multiply GEMM on one MI355X.

Workload (benchmark configs[1]): the four weight matrices of an OPT-175B decoder layer
(QKV 12288x36864, out-proj 12288x12288, FC1 12288x49152, FC2 49152x12288), int4 codes with one
fp16 scale per 128 rows, fp16 activations, decode-sized M = 1 and M = 8.  One "step" is one
pass over all eight products.  The metric is the weight-stream rate: bytes of packed codes and
scales that the step must read, divided by the step time, with everything resident in HBM
before the timed region.  Weights are synthetic (N(0, 0.02) with 0.1 % of entries x20) and are
quantised on the GPU by fq_quantize before timing; the four matrices total 0.93 GB, far more
than the 256 MB last-level cache, so consecutive products evict each other's weights.

Prints ONE JSON line (see the keys below).  Usage: python bench.py [--gpus 1] [--steps K] [--warmup W]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = 2500.0      # dense fp16 / bf16, published
BITS = 4
GROUP = 128
DECODE_M = (1, 8)


def make_weight(torch, K, N, seed):
    """N(0, 0.02) with a Bernoulli(0.001) mask of entries multiplied by 20, as fp16 on the GPU."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    w = torch.randn((K, N), generator=gen, device="cuda", dtype=torch.float32) * 0.02
    mask = torch.rand((K, N), generator=gen, device="cuda", dtype=torch.float32) < 1e-3
    w = torch.where(mask, w * 20.0, w)
    return w.to(torch.float16)


def cpu_baseline(seconds_target=12.0):
    """The CPU oracle timed on the host cores on a bounded sample of the same workload:
    out-proj-shaped slab (K = 12288, 2048 columns), int4 g = 128, M = 1 and M = 8."""
    import numpy as np

    import oracle
    from paper_2308_09723_amd import workloads

    K, N = 12288, 2048
    W = workloads.weights_gaussian(K, N, seed=7, outlier_prob=1e-3)
    q, s = oracle.quantize(W, BITS, GROUP)          # not timed: quantisation is offline
    acts = [workloads.activations(M, K, "f16", 11 + M) for M in DECODE_M]
    wbytes = K * N * BITS // 8 + (K // GROUP) * N * 2
    t0 = time.perf_counter()
    passes = 0
    while True:
        for A in acts:
            oracle.gemm_ref(A, q, s)
        passes += 1
        el = time.perf_counter() - t0
        if el >= seconds_target or passes >= 2000:
            break
    rate = passes * len(acts) * wbytes / el / 1e12
    return {
        "value": rate,
        "unit": "TB/s",
        "cores": len(os.sched_getaffinity(0)),
        "kind": "oracle",
        "sample": f"K=12288 x N=2048 slab of the out-proj layer, int4 g=128, M in {list(DECODE_M)}, "
                  f"{passes} passes in {el:.1f} s (fp64 dequantise + matmul; quantisation not timed)",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--settle", type=float, default=1.0,
                    help="seconds of untimed steps before the warm-up: after idling, the device runs about 10 %% "
                         "slower for the first ~0.1-0.5 s of sustained load (clock ramp); 0 disables")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--large-m", action="store_true", help="also time the M >= 256 products (reported under 'extra')")
    ap.add_argument("--no-large-m", action="store_true",
                    help="leave out the short M >= 256 / mid-M block of the default line ('roofline_large_m', 'mid_m')")
    ap.add_argument("--all-configs", action="store_true",
                    help="also time the other BASELINE configurations (reported under 'extra'): prefill and mid-M "
                         "products (configs[2]), the grouped expert products (configs[3]) and the heavy-tailed "
                         "stress layer (configs[4])")
    ap.add_argument("--profile", choices=["decode", "prefill", "prefill-int8", "copy", "moe", "midm", "quantize", "w4a8", "w4a8-prefill"], default=None,
                    help="short untimed run of one case for rocprofv3 (no JSON line): 'decode' = the benchmark "
                         "step, 'prefill' = QKV-shaped product at M = 2048 (bf16, then fp16; 'prefill-int8': the same with "
                         "8-bit codes, one group per column), 'copy' = a 1 GiB device copy "
                         "whose FETCH_SIZE / WRITE_SIZE calibrate the counters, 'moe' = the grouped expert products of "
                         "configs[3], 'midm' = the QKV-shaped product at M = 32 and M = 128 (bf16), 'quantize' = the offline "
                         "steps (fq_quantize, fq_choose_group, fq_quant_error) on the FC1-shaped matrix")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build targets one GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2308_09723_amd import fq, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    fq.load(build_if_missing=False)
    torch.cuda.set_device(0)
    if args.profile == "copy":
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").zero_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        return
    if args.profile == "prefill":
        profile_prefill(torch, fq, workloads, args.steps, args.settle)
        return
    if args.profile == "prefill-int8":
        profile_prefill(torch, fq, workloads, args.steps, args.settle, bits=8, group=0)
        return
    if args.profile == "moe":
        moe_section(torch, fq, workloads)
        return
    if args.profile == "quantize":
        quantize_section(torch, fq, workloads)
        return
    if args.profile == "w4a8":
        print(json.dumps(w4a8_section(torch, fq, workloads, layers=("qkv",))), file=sys.stderr)
        return
    if args.profile == "w4a8-prefill":
        print(json.dumps(w4a8_section(torch, fq, workloads, layers=("qkv",), Ms=(2048,))), file=sys.stderr)
        return
    if args.profile == "midm":
        K, N = workloads.OPT175B_LAYERS["qkv"]
        codes, scales = fq.quantize(make_weight(torch, K, N, 100), BITS, GROUP)
        large_m_section(torch, fq, [("qkv", K, N, codes, scales)], (32, 128))
        return

    layers = []
    for i, (name, (K, N)) in enumerate(workloads.OPT175B_LAYERS.items()):
        W = make_weight(torch, K, N, 100 + i)
        codes, scales = fq.quantize(W, BITS, GROUP)
        del W
        layers.append((name, K, N, codes, scales))
    torch.cuda.synchronize()
    torch.cuda.empty_cache()

    calls = []   # (name, M, A, codes, scales, C, workspace, weight_bytes, algorithmic_bytes)
    # Order: every layer at M = 1, then every layer at M = 8.  Between two uses of one layer's weights the
    # other three layers (>= 620 MB) stream through, more than twice the 256 MB Infinity Cache, so no
    # product finds its weights cache-resident.
    for M in DECODE_M:
        for name, K, N, codes, scales in layers:
            gen = torch.Generator(device="cuda")
            gen.manual_seed(1000 + M)
            A = torch.randn((M, K), generator=gen, device="cuda", dtype=torch.float32).to(torch.float16)
            C = torch.empty((M, N), device="cuda", dtype=torch.float16)
            need = fq.gemm_workspace_bytes(M, N, K, BITS, GROUP)
            ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
            wbytes = codes.numel() + scales.numel() * 2
            abytes = wbytes + 2 * M * K + 2 * M * N
            calls.append((name, M, A, codes, scales, C, ws, wbytes, abytes))
    stream = torch.cuda.current_stream().cuda_stream

    def step(events=None):
        for i, (name, M, A, codes, scales, C, ws, _, _) in enumerate(calls):
            if events is not None:
                events[i][0].record()
            st = fq.gemm_raw(A.data_ptr(), fq.FQ_F16, M, C.shape[1], A.shape[1], codes.data_ptr(), scales.data_ptr(),
                             BITS, GROUP, C.data_ptr(), ws.data_ptr(), ws.numel(), stream)
            if st != fq.FQ_OK:
                raise fq.FqError(st, "fq_gemm")
            if events is not None:
                events[i][1].record()

    if args.settle > 0:
        t_end = time.perf_counter() + args.settle
        while time.perf_counter() < t_end:
            for _ in range(50):
                step()
            torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.profile == "decode":
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        return
    # timed region: exactly `steps` steps.  HIP events are recorded on the launch stream: in every
    # EVENT_STRIDE-th step one pair brackets the whole step (its eight launches run back to back, so the
    # pair measures the sum of their durations: this is what the roofline uses), and half a stride later
    # a pair brackets each product (the per-product breakdown; each of these carries the ~1.5 us that an
    # event record between two kernels costs, so their sum is larger than the step figure).
    EVENT_STRIDE = 8
    ev_step = {k: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for k in range(0, args.steps, EVENT_STRIDE)}
    ev = {k: [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in calls]
          for k in range(EVENT_STRIDE // 2, args.steps, EVENT_STRIDE)}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        pair = ev_step.get(k)
        if pair is not None:
            pair[0].record()
        step(ev.get(k))
        if pair is not None:
            pair[1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    ms_per_step = elapsed * 1e3 / args.steps
    weight_bytes_step = sum(c[7] for c in calls)
    value = weight_bytes_step / (elapsed / args.steps) / 1e12
    step_us = [a.elapsed_time(b) * 1e3 for a, b in ev_step.values()]
    kernel_us = sum(step_us) / len(step_us)
    algo_bytes = sum(c[8] for c in calls)
    achieved = algo_bytes / (kernel_us * 1e-6) / 1e9
    per_call_us = []
    for i in range(len(calls)):
        ts = [ev[k][i][0].elapsed_time(ev[k][i][1]) * 1e3 for k in ev]
        per_call_us.append(sum(ts) / len(ts) if ts else float("nan"))
    per_layer = {f"{c[0]}_M{c[1]}": {"us": round(t, 2), "weight_TBps": round(c[7] / t / 1e6, 3),
                                    "frac_of_hbm_peak": round(c[7] / t / 1e3 / HBM_PEAK_GBS, 4),
                                    "plan": fq.gemm_describe(c[1], c[5].shape[1], c[2].shape[1], BITS, GROUP)}
                 for c, t in zip(calls, per_call_us)}
    traffic, traffic_note = profiled_traffic([v["plan"] for v in per_layer.values()])

    out = {
        "metric": "W4A16 GEMM weight-stream rate, OPT-175B decode layers (M=1 and M=8)",
        "value": round(value, 4),
        "unit": "TB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_seconds": args.settle,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {
            "workload": "BASELINE configs[1]: OPT-175B-shaped QKV/out-proj/FC1/FC2, fp16 activations M in {1, 8}, "
                        "int4 weights, group_size 128, N(0,0.02) weights with 0.1% x20 outliers",
            "products_per_step": len(calls),
            "weight_bytes_per_step": weight_bytes_step,
            "frac_of_hbm_peak": round(value * 1e3 / HBM_PEAK_GBS, 4),
        },
        "roofline": {
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            # HBM bytes per step from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes recorded in
            # profiles/ (counter-calibrated with a 1 GiB copy); null when that record was taken with other
            # kernel plans than the ones this run used
            "traffic": traffic,
            "traffic_source": traffic_note,
            "kernel": "fq_gemm_skinny_kernel (8 products per step, plus fq_reduce_kernel for the one that splits K "
                      "over the grid; algorithmic bytes of the step / mean HIP-event duration of its back-to-back "
                      "launches)",
            "algorithmic_bytes_per_step": algo_bytes,
            "kernel_us_per_step": round(kernel_us, 2),
        },
        "per_product": per_layer,
    }
    out["stream_ceiling"] = stream_ceiling(torch, fq)
    if not args.no_large_m:
        out.update(default_large_m(torch, fq, layers))
        w8 = w4a8_section(torch, fq, workloads, layers=("qkv",), Ms=(8, 2048), time_quantizers=False)
        out["roofline_w4a8"] = {
            "bound": "mfma", "unit": "TOP/s", "peak": INT8_PEAK_TOPS, "achieved": w8["qkv_M2048"]["TOPs"],
            "frac": w8["qkv_M2048"]["frac_of_int8_peak"],
            "kernel": "fq_gemm_w4a8_kernel (v_mfma_i32_16x16x64_i8; M = 8: fq_w4a8_skinny_kernel), the integer path: int8 "
                      "activations x int4 weights with integer group scales; the product alone, activations quantised "
                      "beforehand",
            "workload": "QKV 12288 x 36864, g=128, M = 2048 (and M = 8 against the HBM peak)",
            "cases": w8,
            "mfma_ceiling": mfma_ceiling(torch, fq, int8=True),
        }
    if args.large_m or args.all_configs:
        out["extra"] = large_m_section(torch, fq, layers, (32, 128, 512, 2048) if args.all_configs else (256, 2048))
    if args.all_configs:
        del layers, calls
        torch.cuda.empty_cache()
        out["extra_moe"] = moe_section(torch, fq, workloads)
        out["extra_stress"] = stress_section(torch, fq, workloads)
        out["extra_quantize"] = quantize_section(torch, fq, workloads)
        out["extra_bf16_scales"] = bf16_scales_section(torch, fq, workloads)
        out["extra_int3"] = int3_section(torch, fq, workloads)
        out["extra_w4a8"] = w4a8_section(torch, fq, workloads)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out))


TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "fq_gemm_skinny_kernel_opt175b_decode.md")


def profiled_traffic(plans):
    """HBM bytes per decode step as the rocprofv3 counter passes recorded them.  The profile summary carries
    one line `bench-traffic: bytes_per_step=<float> commit=<hash> plans=<the eight plan descriptions joined by
    ';'>`; the figure is used only if this run's plans are the recorded ones, so that it cannot outlive the
    kernels it was measured on unnoticed."""
    try:
        with open(TRAFFIC_PROFILE) as f:
            lines = [ln.strip() for ln in f if ln.strip().startswith("bench-traffic:")]
    except OSError:
        return None, "no profile summary found"
    if not lines:
        return None, "profile summary carries no bench-traffic line"
    fields = dict(kv.split("=", 1) for kv in lines[-1][len("bench-traffic:"):].strip().split(" ", 2))
    if fields.get("plans", "") != ";".join(plans):
        return None, (f"profiles/{os.path.basename(TRAFFIC_PROFILE)} (commit {fields.get('commit')}) was taken with "
                      "other kernel plans; re-profile")
    return float(fields["bytes_per_step"]), (f"rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, profiles/"
                                             f"{os.path.basename(TRAFFIC_PROFILE)}, commit {fields.get('commit')}")


def default_large_m(torch, fq, layers):
    """The M >= 256 half of the metric in the default line, kept to a few seconds: the QKV-shaped product at
    M = 2048 with bf16 and with fp16 activations (for bf16 the rewrite of the activation rows that precedes
    the product is inside the timed bracket), as TFLOP/s against the dense fp16 / bf16 MFMA peak; and the
    transition regime, QKV at M = 32 (against the HBM peak) and M = 128 (against the MFMA peak), bf16, cycling
    through copies of the weights."""
    qkv = [l for l in layers if l[0] == "qkv"]
    big = large_m_section(torch, fq, qkv, (2048,), settle=0.4, reps=10)
    mid = large_m_section(torch, fq, qkv, (32, 128), dtypes=("bf16",), settle=0.25, reps=20)
    best = max(big.values(), key=lambda r: r["TFLOPs"])
    res = {
        "roofline_large_m": {
            "bound": "mfma", "unit": "TFLOP/s", "peak": MFMA_PEAK_TFLOPS,
            "achieved": best["TFLOPs"], "frac": best["frac_of_mfma_peak"],
            "kernel": "fq_gemm_mma_kernel, 128-row x 384-column blocks (bf16 activations: fq_rows_to_f16_kernel + the "
                      "product on the fp16 matrix path, both inside the timed bracket); flops = 2 M N K / mean HIP-event "
                      "time of 10 back-to-back calls",
            "workload": "BASELINE configs[2] shape: QKV 12288 x 36864, int4 g=128, M = 2048",
            "cases": big,
            "mfma_ceiling": mfma_ceiling(torch, fq),
        },
        "mid_m": {
            "workload": "BASELINE configs[2] shape: QKV 12288 x 36864, int4 g=128, bf16, weights cycled through "
                        "copies so that none is cache-resident",
            "M32": dict(mid["qkv_M32_bf16"], bound="hbm",
                        frac=round(mid["qkv_M32_bf16"]["weight_TBps"] * 1e3 / HBM_PEAK_GBS, 4)),
            "M128": dict(mid["qkv_M128_bf16"], bound="mfma", frac=mid["qkv_M128_bf16"]["frac_of_mfma_peak"]),
        },
    }
    return res


def stream_ceiling(torch, fq):
    """What this machine's memory system delivers to a kernel that only reads (fq_stream_read_probe over a 2 GiB
    buffer, eight times the Infinity Cache, in the launch shape of the small-M kernel), next to the vendor
    peak the roofline uses."""
    n = 1 << 31
    buf = torch.empty(n, dtype=torch.uint8, device="cuda").zero_()
    sink = torch.empty(8192, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream

    def run():
        st = fq.stream_read_probe_raw(buf.data_ptr(), n, sink.data_ptr(), stream)
        if st != fq.FQ_OK:
            raise fq.FqError(st, "fq_stream_read_probe")
    ms = _timed(torch, run, settle=0.2, reps=20)
    return {"kind": "read-only kernel over a 2 GiB buffer", "GBps": round(n / ms / 1e6, 1),
            "frac_of_hbm_peak": round(n / ms / 1e6 / HBM_PEAK_GBS, 4)}


def mfma_ceiling(torch, fq, int8=False):
    """What this box's matrix pipes deliver to a loop of nothing but MFMAs on operands distributed like the
    product's (fq_mfma_rate_probe: N(0,1) activations and N(0,0.02) weights in binary16, or, for the integer
    path, int8 activations quantised from N(0,1) rows and codes times multipliers), with and without the
    product's LDS fragment reads, and on all-zero operands: the clock under load follows the switching activity of
    the operands, so the vendor's peak is reached on zeros only."""
    nb = fq.mfma_rate_probe_operand_bytes()
    sb = fq.mfma_rate_probe_sink_bytes()
    if int8:
        # activations: rne(x * 127 / max|x|) of N(0,1) rows (max ~ 4.5 sigma over 12288 values); weights: code x multiplier
        ops = torch.clamp(torch.round(torch.randn(nb, device="cuda") * (127.0 / 4.5)), -127, 127).to(torch.int8)
        wq = torch.clamp(torch.round(torch.randn(512 * 3 * 16, device="cuda") * 2.3), -7, 7)
        wz = torch.randint(8, 17, (512 * 3 * 16,), device="cuda").float()
        ops[nb - 512 * 3 * 16:] = (wq * wz).to(torch.int8)
        zeros = torch.zeros(nb, device="cuda", dtype=torch.int8)
        kind = "v_mfma_i32_16x16x64_i8"
        peak = INT8_PEAK_TOPS
    else:
        n16 = nb // 2
        ops = torch.randn(n16, device="cuda", dtype=torch.float32).to(torch.float16)
        ops[n16 - 512 * 3 * 8:] *= 0.02                      # the tail holds the weight-like operands
        zeros = torch.zeros(n16, device="cuda", dtype=torch.float16)
        kind = "v_mfma_f32_16x16x32_f16"
        peak = MFMA_PEAK_TFLOPS
    sink = torch.empty(sb, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    iters = 200
    flops = fq.mfma_rate_probe_flops(iters, int(int8))
    out = {"kind": f"fq_mfma_rate_probe: the 128-row shape's MFMA loop ({kind}) without loads, conversions or "
                   f"barriers; {'TOP/s' if int8 else 'TFLOP/s'}"}
    for key, buf, lds in (("random_operands_with_lds_reads", ops, 1), ("random_operands_registers_only", ops, 0),
                          ("zero_operands_registers_only", zeros, 0)):
        def run():
            st = fq.mfma_rate_probe_raw(buf.data_ptr(), nb, sink.data_ptr(), sb, iters, lds, int(int8), stream)
            if st != fq.FQ_OK:
                raise fq.FqError(st, "fq_mfma_rate_probe")
        ms = _timed(torch, run, settle=0.3, reps=10)
        out[key] = round(flops / ms / 1e9, 1)
    out["frac_of_peak"] = round(out["random_operands_with_lds_reads"] / peak, 4)
    return out


def profile_prefill(torch, fq, workloads, reps, settle, bits=BITS, group=GROUP):
    """QKV-shaped product at M = 2048, first with bf16 and then with fp16 activations: `settle` seconds of
    launches each, then `reps` more (for rocprofv3; the last records of each kernel in the trace are the
    settled ones)."""
    K, N = workloads.OPT175B_LAYERS["qkv"]
    M = 2048
    W = make_weight(torch, K, N, 100)
    codes, scales = fq.quantize(W, bits, group)
    del W
    need = fq.gemm_workspace_bytes(M, N, K, bits, group)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    for act, dt in ((fq.FQ_BF16, torch.bfloat16), (fq.FQ_F16, torch.float16)):
        A = torch.randn((M, K), device="cuda", dtype=torch.float32).to(dt)
        C = torch.empty((M, N), device="cuda", dtype=dt)

        def run():
            st = fq.gemm_raw(A.data_ptr(), act, M, N, K, codes.data_ptr(), scales.data_ptr(), bits, group,
                             C.data_ptr(), ws.data_ptr(), ws.numel(), stream)
            if st != fq.FQ_OK:
                raise fq.FqError(st, "fq_gemm")
        t_end = time.perf_counter() + settle
        while time.perf_counter() < t_end:
            for _ in range(4):
                run()
            torch.cuda.synchronize()
        for _ in range(max(1, min(reps, 20))):
            run()
        torch.cuda.synchronize()


# Bytes of distinct weights that must pass between two uses of the same buffer in the weight-stream-bound
# measurements: three times the 256 MB Infinity Cache, so that no call finds its weights cached.
ROTATE_BYTES = 768e6


def rotating(codes, scales, M):
    """Copies of (codes, scales) to cycle through when the product is bound by the weight stream (M <= 128) and
    one copy would fit the Infinity Cache; a single entry otherwise.  Returns (list, next_index function)."""
    wbytes = codes.numel() * codes.element_size() + scales.numel() * scales.element_size()
    n = 1 if M > 128 else max(1, int(-(-ROTATE_BYTES // wbytes)) + 1)
    bufs = [(codes, scales)] + [(codes.clone(), scales.clone()) for _ in range(n - 1)]
    state = {"i": 0}

    def nxt():
        state["i"] = (state["i"] + 1) % n
        return bufs[state["i"]]
    return bufs, nxt


def _timed(torch, run, settle=0.3, reps=20):
    """Mean milliseconds per call of run(), after `settle` seconds of the same call."""
    run()
    torch.cuda.synchronize()
    t_end = time.perf_counter() + settle
    while time.perf_counter() < t_end:
        for _ in range(4):
            run()
        torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def moe_section(torch, fq, workloads):
    """BASELINE configs[3]: 64 experts, d_model 4096, d_ff 16384, int4 g = 64, fp16; 2048 tokens routed top-2
    with Zipf(1.1) popularity.  FC1 and FC2 timed separately.  Both rooflines are reported: the weights of
    the experts that received rows must be read once (HBM), and 2 * rows * K * N flops must be done (MFMA)."""
    import numpy as np
    E = workloads.MOE["experts"]
    dm, dff = workloads.MOE["d_model"], workloads.MOE["d_ff"]
    offsets, _ = workloads.zipf_routing(2048, E, 2, 1.1, seed=5)
    counts = np.diff(offsets)
    rows = int(offsets[-1])
    hit = int((counts > 0).sum())
    stream = torch.cuda.current_stream().cuda_stream
    res = {"rows_per_expert": counts.tolist()}
    for K, N, tag in ((dm, dff, "fc1"), (dff, dm, "fc2")):
        codes_l, scales_l = [], []
        for e in range(E):
            c, s = fq.quantize(make_weight(torch, K, N, 500 + e), 4, 64)
            codes_l.append(c)
            scales_l.append(s.reshape(-1))
        codes = torch.cat(codes_l)
        scales = torch.cat(scales_l)
        del codes_l, scales_l
        A = torch.randn((rows, K), device="cuda", dtype=torch.float32).to(torch.float16)
        C = torch.empty((rows, N), device="cuda", dtype=torch.float16)
        offs = offsets.tolist()

        def run():
            st = fq.gemm_grouped_raw(A.data_ptr(), fq.FQ_F16, offs, N, K, codes.data_ptr(), scales.data_ptr(), 4, 64,
                                     C.data_ptr(), None, 0, stream)
            if st != fq.FQ_OK:
                raise fq.FqError(st, "fq_gemm_grouped")
        ms = _timed(torch, run, settle=0.5, reps=10)
        wbytes = hit * (K * N // 2 + (K // 64) * N * 2)
        flops = 2.0 * rows * K * N
        res[tag] = {"ms": round(ms, 4), "weight_TBps": round(wbytes / ms / 1e9, 3),
                    "frac_of_hbm_peak": round(wbytes / ms / 1e6 / HBM_PEAK_GBS, 4),
                    "TFLOPs": round(flops / ms / 1e9, 1), "frac_of_mfma_peak": round(flops / ms / 1e9 / MFMA_PEAK_TFLOPS, 4),
                    "experts_hit": hit, "weight_bytes": wbytes}
        del codes, scales, A, C
        torch.cuda.empty_cache()
    return res


def quantize_section(torch, fq, workloads):
    """The offline steps on the FC1-shaped matrix (1.21 GB of fp16 weights): fq_quantize (scales, codes,
    packing), fq_choose_group and fq_quant_error.  Rates count the weights read once plus the outputs."""
    K, N = workloads.OPT175B_LAYERS["fc1"]
    W = make_weight(torch, K, N, 321)
    stream = torch.cuda.current_stream().cuda_stream
    res = {}
    for bits, g in ((4, 128), (4, 32), (8, 0)):
        codes = torch.empty(fq.codes_bytes(K, N, bits), dtype=torch.uint8, device="cuda")
        scales = torch.empty(fq.scales_bytes(K, N, g) // 2, dtype=torch.float16, device="cuda")

        def run():
            st = fq.quantize_raw(W.data_ptr(), K, N, bits, g, codes.data_ptr(), scales.data_ptr(), stream)
            if st != fq.FQ_OK:
                raise fq.FqError(st, "fq_quantize")
        ms = _timed(torch, run, settle=0.1, reps=10)
        nbytes = K * N * 2 + codes.numel() + scales.numel() * 2
        res[f"quantize_int{bits}_g{g or K}"] = {"ms": round(ms, 4), "TBps": round(nbytes / ms / 1e9, 3)}
        if (bits, g) == (4, 128):
            t0 = time.perf_counter()
            sse, mx = fq.quant_error(W, codes, scales, bits, g)
            res["quant_error_int4_g128"] = {"ms": round((time.perf_counter() - t0) * 1e3, 4), "mse": sse / (K * N),
                                            "max_abs": mx}
    fq.choose_group(W, 0, 32, 0.9)
    t0 = time.perf_counter()
    gsel = fq.choose_group(W, 0, 32, 0.9)
    res["choose_group_alpha0.9"] = {"ms": round((time.perf_counter() - t0) * 1e3, 4), "group_size": gsel}
    return res


def bf16_scales_section(torch, fq, workloads):
    """The bfloat16 scale format (scales of the activation's type) on the QKV-shaped int4 matrix with bf16
    activations, next to the binary16 format: quantiser time and products at M = 8, 32 and 2048."""
    K, N = workloads.OPT175B_LAYERS["qkv"]
    W = make_weight(torch, K, N, 100)
    stream = torch.cuda.current_stream().cuda_stream
    res = {}
    for tag, sf in (("f16_scales", fq.FQ_SCALE_F16), ("bf16_scales", fq.FQ_SCALE_BF16)):
        codes = torch.empty(fq.codes_bytes(K, N, BITS), dtype=torch.uint8, device="cuda")
        scales = torch.empty((K // GROUP, N), dtype=torch.bfloat16 if sf else torch.float16, device="cuda")

        def quant():
            st = fq.quantize_sf_raw(W.data_ptr(), K, N, BITS, GROUP, sf, codes.data_ptr(), scales.data_ptr(), stream)
            if st != fq.FQ_OK:
                raise fq.FqError(st, "fq_quantize_sf")
        res[f"quantize_{tag}"] = {"ms": round(_timed(torch, quant), 4)}
        sse, mx = fq.quant_error(W, codes, scales, BITS, GROUP)
        res[f"quantize_{tag}"]["mse"] = sse / (K * N)
        for M in (8, 32, 2048):
            A = torch.randn((M, K), device="cuda", dtype=torch.float32).to(torch.bfloat16)
            C = torch.empty((M, N), device="cuda", dtype=torch.bfloat16)
            need = fq.gemm_workspace_bytes(M, N, K, BITS, GROUP)
            ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")

            bufs, nxt = rotating(codes, scales, M)

            def run():
                c, s_ = nxt()
                st = fq.gemm_sf_raw(A.data_ptr(), fq.FQ_BF16, M, N, K, c.data_ptr(), s_.data_ptr(), sf, BITS,
                                    GROUP, C.data_ptr(), ws.data_ptr(), ws.numel(), stream)
                if st != fq.FQ_OK:
                    raise fq.FqError(st, "fq_gemm_sf")
            ms = _timed(torch, run)
            del bufs
            wbytes = codes.numel() + scales.numel() * 2
            res[f"M{M}_{tag}"] = {"us": round(ms * 1e3, 2), "weight_TBps": round(wbytes / ms / 1e9, 3),
                                  "TFLOPs": round(2.0 * M * N * K / ms / 1e9, 1)}
    return res


def int3_section(torch, fq, workloads):
    """3-bit codes (group 128) on the four OPT-175B shapes: decode products at M = 1 and 8 (fp16), and the
    QKV-shaped prefill product at M = 2048 (bf16)."""
    stream = torch.cuda.current_stream().cuda_stream
    res = {}
    for name, (K, N) in workloads.OPT175B_LAYERS.items():
        W = make_weight(torch, K, N, 100)
        codes, scales = fq.quantize(W, 3, GROUP)
        del W
        wbytes = codes.numel() + scales.numel() * 2
        cases = [(1, torch.float16, fq.FQ_F16), (8, torch.float16, fq.FQ_F16)]
        if name == "qkv":
            cases.append((2048, torch.bfloat16, fq.FQ_BF16))
        for M, dt, act in cases:
            A = torch.randn((M, K), device="cuda", dtype=torch.float32).to(dt)
            C = torch.empty((M, N), device="cuda", dtype=dt)
            need = fq.gemm_workspace_bytes(M, N, K, 3, GROUP)
            ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")

            bufs, nxt = rotating(codes, scales, M)

            def run():
                c, s_ = nxt()
                st = fq.gemm_raw(A.data_ptr(), act, M, N, K, c.data_ptr(), s_.data_ptr(), 3, GROUP,
                                 C.data_ptr(), ws.data_ptr(), ws.numel(), stream)
                if st != fq.FQ_OK:
                    raise fq.FqError(st, "fq_gemm")
            ms = _timed(torch, run)
            del bufs
            res[f"{name}_M{M}"] = {"us": round(ms * 1e3, 2), "weight_TBps": round(wbytes / ms / 1e9, 3),
                                   "TFLOPs": round(2.0 * M * N * K / ms / 1e9, 1),
                                   "plan": fq.gemm_describe(M, N, K, 3, GROUP)}
        del codes, scales
    return res


INT8_PEAK_TOPS = 5000.0        # dense int8 MFMA, published


def w4a8_section(torch, fq, workloads, layers=("qkv", "out_proj", "fc1", "fc2"), Ms=(1, 8, 32, 128, 512, 2048),
                 time_quantizers=True):
    """The integer path (int8 activations x int4 weights with integer group scales, g = 128) on the OPT-175B
    shapes: the product alone (activations quantised beforehand) at M = 1, 8, 32, 128, 512, 2048, against the HBM
    peak (weight stream) and the dense int8 MFMA peak; plus the two quantisers' times."""
    res = {}
    stream = torch.cuda.current_stream().cuda_stream
    for name in layers:
        K, N = workloads.OPT175B_LAYERS[name]
        W = make_weight(torch, K, N, 100)
        codes, z, t = fq.quantize_w4a8(W, GROUP)

        def quant():
            st = fq.quantize_w4a8_raw(W.data_ptr(), K, N, GROUP, codes.data_ptr(), z.data_ptr(), t.data_ptr(), stream)
            if st != fq.FQ_OK:
                raise fq.FqError(st, "fq_quantize_w4a8")
        if name == "qkv" and time_quantizers:
            res["quantize_w4a8_qkv_ms"] = round(_timed(torch, quant, settle=0.1, reps=5), 3)
        del W
        wbytes = codes.numel() + z.numel() + t.numel() * 2
        for M in Ms:
            A = torch.randn((M, K), device="cuda", dtype=torch.float32).to(torch.bfloat16)
            Aq, alpha = fq.quantize_act_i8(A)
            C = torch.empty((M, N), device="cuda", dtype=torch.bfloat16)
            need = fq.gemm_w4a8_workspace_bytes(M, N, K, GROUP)
            ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
            n = 1 if M > 128 else max(1, int(-(-ROTATE_BYTES // wbytes)) + 1)
            bufs = [(codes, z)] + [(codes.clone(), z.clone()) for _ in range(n - 1)]
            state = {"i": 0}

            def run():
                state["i"] = (state["i"] + 1) % n
                c, zz = bufs[state["i"]]
                st = fq.gemm_w4a8_raw(Aq.data_ptr(), alpha.data_ptr(), M, N, K, c.data_ptr(), zz.data_ptr(), t.data_ptr(),
                                      GROUP, C.data_ptr(), fq.FQ_BF16, ws.data_ptr(), ws.numel(), stream)
                if st != fq.FQ_OK:
                    raise fq.FqError(st, "fq_gemm_w4a8")
            ms = _timed(torch, run, settle=0.2, reps=20)
            del bufs
            tops = 2.0 * M * N * K / ms / 1e9
            res[f"{name}_M{M}"] = {"us": round(ms * 1e3, 2), "weight_TBps": round(wbytes / ms / 1e9, 3),
                                   "frac_of_hbm_peak": round(wbytes / ms / 1e6 / HBM_PEAK_GBS, 4),
                                   "TOPs": round(tops, 1), "frac_of_int8_peak": round(tops / INT8_PEAK_TOPS, 4)}
            if name == "qkv" and M == 2048 and time_quantizers:
                def aq():
                    st = fq.quantize_act_i8_raw(A.data_ptr(), fq.FQ_BF16, M, K, Aq.data_ptr(), alpha.data_ptr(), stream)
                    if st != fq.FQ_OK:
                        raise fq.FqError(st, "fq_quantize_act_i8")
                res["quantize_act_M2048_K12288_us"] = round(_timed(torch, aq, settle=0.05, reps=20) * 1e3, 2)
        del codes, z, t
    return res


def stress_section(torch, fq, workloads):
    """BASELINE configs[4]: K = 8192, N = 28672, 0.02 * Student-t(3) weights with 1 % of the columns x50,
    bf16 activations and output, M in {1, 16, 256}, int4 and int8 at g in {32, 128, K}."""
    K, N = workloads.STRESS_LAYER
    gen = torch.Generator(device="cuda")
    gen.manual_seed(900)
    # Student-t(3) = normal / sqrt(chi2_3 / 3)
    z = torch.randn((K, N), generator=gen, device="cuda")
    chi = (torch.randn((3, K, N), generator=gen, device="cuda") ** 2).sum(0)
    W = 0.02 * z / torch.sqrt(chi / 3.0)
    del z, chi
    cols = torch.rand((N,), generator=gen, device="cuda") < 0.01
    W = torch.where(cols[None, :], W * 50.0, W).clamp_(-65504.0, 65504.0).to(torch.float16)
    stream = torch.cuda.current_stream().cuda_stream
    res = {}
    for bits in (4, 8):
        for g in (32, 128, 0):
            codes, scales = fq.quantize(W, bits, g)
            wbytes = codes.numel() + scales.numel() * 2
            for M in (1, 16, 256):
                A = torch.randn((M, K), device="cuda", dtype=torch.float32).to(torch.bfloat16)
                C = torch.empty((M, N), device="cuda", dtype=torch.bfloat16)
                need = fq.gemm_workspace_bytes(M, N, K, bits, g)
                ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")

                bufs, nxt = rotating(codes, scales, M)

                def run():
                    c, s_ = nxt()
                    st = fq.gemm_raw(A.data_ptr(), fq.FQ_BF16, M, N, K, c.data_ptr(), s_.data_ptr(), bits, g,
                                     C.data_ptr(), ws.data_ptr(), ws.numel(), stream)
                    if st != fq.FQ_OK:
                        raise fq.FqError(st, "fq_gemm")
                ms = _timed(torch, run, settle=0.15, reps=20)
                del bufs
                res[f"int{bits}_g{g or K}_M{M}"] = {
                    "us": round(ms * 1e3, 2), "weight_TBps": round(wbytes / ms / 1e9, 3),
                    "TFLOPs": round(2.0 * M * N * K / ms / 1e9, 1), "plan": fq.gemm_describe(M, N, K, bits, g)}
            del codes, scales
    return res


def large_m_section(torch, fq, layers, Ms=(256, 2048), dtypes=("bf16", "f16"), settle=0.3, reps=20):
    """Prefill-sized and mid-M products on the same int4 weights: TFLOP/s and fraction of the dense MFMA peak,
    and the weight-stream rate.  Up to M = 128 the calls cycle through copies of the weights (see `rotating`),
    so that the rate is not that of the Infinity Cache."""
    res = {}
    stream = torch.cuda.current_stream().cuda_stream
    for name, K, N, codes, scales in layers:
        for M in Ms:
            for tag, act, dt in (("bf16", fq.FQ_BF16, torch.bfloat16), ("f16", fq.FQ_F16, torch.float16)):
                if tag not in dtypes:
                    continue
                A = torch.randn((M, K), device="cuda", dtype=torch.float32).to(dt)
                C = torch.empty((M, N), device="cuda", dtype=dt)
                need = fq.gemm_workspace_bytes(M, N, K, BITS, GROUP)
                ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")

                bufs, nxt = rotating(codes, scales, M)

                def run():
                    c, s_ = nxt()
                    st = fq.gemm_raw(A.data_ptr(), act, M, N, K, c.data_ptr(), s_.data_ptr(), BITS, GROUP,
                                     C.data_ptr(), ws.data_ptr(), ws.numel(), stream)
                    if st != fq.FQ_OK:
                        raise fq.FqError(st, "fq_gemm")
                # untimed: about 0.3 s of the same product, so that the clocks have settled
                run()
                torch.cuda.synchronize()
                t_end = time.perf_counter() + settle
                while time.perf_counter() < t_end:
                    for _ in range(4):
                        run()
                    torch.cuda.synchronize()
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    run()
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / reps
                tflops = 2.0 * M * N * K / (ms * 1e-3) / 1e12
                wbytes = codes.numel() + scales.numel() * 2
                res[f"{name}_M{M}_{tag}"] = {"ms": round(ms, 4), "TFLOPs": round(tflops, 1),
                                             "frac_of_mfma_peak": round(tflops / MFMA_PEAK_TFLOPS, 4),
                                             "weight_TBps": round(wbytes / ms / 1e9, 3),
                                             "plan": fq.gemm_describe(M, N, K, BITS, GROUP)}
    return res


if __name__ == "__main__":
    main()
