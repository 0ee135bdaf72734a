"""Quantisation-quality report on synthetic weights, computed by the GPU library.

Two tables, after section 3.2 / figure 2 of the FineQuant paper:
  * mean squared round-trip error against the group size (the MSE axis of figure 2a), from
    fq_quantize + fq_quant_error, for 4- and 8-bit codes;
  * the group size the adaptive heuristic of section 3.3 picks against its threshold alpha, and the
    storage that choice costs (bits per weight = b + 16 / g: one half-precision scale per group).
No checkpoint is available, so the matrices are the seeded synthetic stand-ins of the benchmark
configurations (Gaussian with sparse outliers; heavy-tailed with a few amplified columns); the numbers
therefore show the mechanism, not the paper's model-level results.

Usage: python -m paper_2308_09723_amd.report [--layer out_proj|qkv|fc1|fc2|stress] [--json]
"""
import argparse
import json
import sys


def _weights(torch, layer, seed):
    from . import workloads

    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    if layer == "stress":
        K, N = workloads.STRESS_LAYER
        z = torch.randn((K, N), generator=gen, device="cuda")
        chi = (torch.randn((3, K, N), generator=gen, device="cuda") ** 2).sum(0)
        W = 0.02 * z / torch.sqrt(chi / 3.0)
        cols = torch.rand((N,), generator=gen, device="cuda") < 0.01
        W = torch.where(cols[None, :], W * 50.0, W).clamp_(-65504.0, 65504.0)
    else:
        K, N = workloads.OPT175B_LAYERS[layer]
        W = torch.randn((K, N), generator=gen, device="cuda") * 0.02
        mask = torch.rand((K, N), generator=gen, device="cuda") < 1e-3
        W = torch.where(mask, W * 20.0, W)
    return W.to(torch.float16)


def run(layer="out_proj", seed=100):
    import torch

    from . import fq

    fq.load(build_if_missing=False)
    W = _weights(torch, layer, seed)
    K, N = W.shape
    sizes = [g for g in (K, 2048, 1024, 512, 256, 128, 64, 32) if g <= K and K % g == 0]
    sizes = sorted(set(sizes), reverse=True)
    mse = []
    for bits in (4, 8):
        for g in sizes:
            codes, scales = fq.quantize(W, bits, g)
            sse, mx = fq.quant_error(W, codes, scales, bits, g)
            mse.append({"bits": bits, "group_size": g, "mse": sse / (K * N), "max_abs_err": mx,
                        "bits_per_weight": bits + 16.0 / g})
            del codes, scales
    heur = []
    for alpha in (0.0, 0.1, 0.25, 0.5, 0.75, 0.9, 0.95, 0.99, 1.0):
        g = fq.choose_group(W, 0, 32, alpha)
        heur.append({"alpha": alpha, "group_size": g, "int4_bits_per_weight": 4 + 16.0 / g,
                     "int8_bits_per_weight": 8 + 16.0 / g})
    return {"layer": layer, "K": K, "N": N, "mse_vs_group_size": mse, "heuristic_vs_alpha": heur}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--layer", default="out_proj", choices=["out_proj", "qkv", "fc1", "fc2", "stress"])
    ap.add_argument("--json", action="store_true")
    args = ap.parse_args()
    res = run(args.layer)
    if args.json:
        print(json.dumps(res))
        return
    print(f"layer {res['layer']}: K = {res['K']}, N = {res['N']} (synthetic)")
    print("| bits | group size | bits / weight | MSE | max abs error |")
    print("|---|---|---|---|---|")
    for r in res["mse_vs_group_size"]:
        print(f"| {r['bits']} | {r['group_size']} | {r['bits_per_weight']:.4f} | {r['mse']:.4e} | {r['max_abs_err']:.4e} |")
    print()
    print("| alpha | chosen group size | int4 bits / weight | int8 bits / weight |")
    print("|---|---|---|---|")
    for r in res["heuristic_vs_alpha"]:
        print(f"| {r['alpha']} | {r['group_size']} | {r['int4_bits_per_weight']:.4f} | {r['int8_bits_per_weight']:.4f} |")


if __name__ == "__main__":
    sys.exit(main())
