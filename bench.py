#!/usr/bin/env python3
"""Benchmark of the ARMOR per-layer factorization hot path on one MI355X.

One "step" is one pass of the whole hot path over one synthetic layer: Gram of the calibration
activations (armor_gram + armor_gram_diag), then armor_factorize_layer (normalise, initialise,
n_iters BCD iterations, final loss) and armor_pack_nm, with W and X already resident in HBM.
Workload (default): the Llama-7B-shaped attention projection of the baseline configs:
W 4096x4096 bf16, X 262144x4096 bf16, H fp32, 2:4 along d_in, d_block 128, 50 BCD iterations.

Prints ONE JSON line.  `value` = BCD iterations per second over the whole step.
`roofline` is for the chain kernel family that takes the most time, from HIP events the library
records around each of its launches during the timed steps.  `cpu_baseline` times the CPU oracle
(test infrastructure, never tuned) on a bounded sample of the same layer.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

WORKLOADS = {
    # name: (d_out, d_in, n_tokens, d_block, N, M, n_iters, w_bf16, x_bf16, act_outlier_frac, act_outlier_scale)
    "llama7b_attn_4096x4096_b128_2:4_50it": (4096, 4096, 262144, 128, 2, 4, 50, True, True, 0.005, 20.0),
    "small_256x256_b32_2:4_20it": (256, 256, 512, 32, 2, 4, 20, False, False, 0.0, 1.0),
    # one square layer at d_block 256 (the hidden size of the 70B-shaped stress workload): short enough for counter runs
    "llama70b_attn_8192x8192_b256_2:4_10it": (8192, 8192, 32768, 256, 2, 4, 10, True, True, 0.005, 20.0),
}
DEFAULT = "llama7b_attn_4096x4096_b128_2:4_50it"

# Multi-matrix workloads (the other baseline configs; not the default bench line).  Each input site
# gets one Gram; every matrix is factorized from its site's diagonal.  One step = all Grams + all
# factorizations + packing.  sites: name -> (d_in, generator); matrices: (name, d_out, site).
BLOCK_WORKLOADS = {
    "llama7b_mlp_b128_2:4_50it": dict(
        tokens=262144, d_block=128, patterns=[(2, 4, 0)], n_iters=50, hidden=4096,
        sites={"mlp_in": 4096, "down_in": 11008},
        matrices=[("gate", 11008, "mlp_in"), ("up", 11008, "mlp_in"), ("down", 4096, "down_in")]),
    "llama3_8b_block_b128_2:4_50it": dict(
        tokens=262144, d_block=128, patterns=[(2, 4, 0)], n_iters=50, hidden=4096,
        sites={"qkv_in": 4096, "o_in": 4096, "mlp_in": 4096, "down_in": 14336},
        matrices=[("q", 4096, "qkv_in"), ("k", 1024, "qkv_in"), ("v", 1024, "qkv_in"), ("o", 4096, "o_in"),
                  ("gate", 14336, "mlp_in"), ("up", 14336, "mlp_in"), ("down", 4096, "down_in")]),
    "llama3_70b_mlp_b256_2:4_4:8_unstructured_30it": dict(
        tokens=131072, d_block=256, patterns=[(2, 4, 0), (4, 8, 0), (2, 4, 1)], n_iters=30, hidden=8192,
        sites={"mlp_in": 8192, "down_in": 28672},
        matrices=[("gate", 28672, "mlp_in"), ("up", 28672, "mlp_in"), ("down", 8192, "down_in")]),
}

# The factorized layer applied to a batch of activations (the batched product of Sec. 4.4, on the
# gate_proj shape of a 14B model): (d_out, d_in, n_tokens, d_block).  Not the default bench line.
APPLY_WORKLOADS = {
    "qwen14b_gate_apply_8192tok_b128_2:4": (13824, 5120, 8192, 128),
    "llama7b_attn_apply_8192tok_b128_2:4": (4096, 4096, 8192, 128),
    "llama70b_gate_apply_8192tok_b256_2:4": (28672, 8192, 8192, 256),
}

# The layer-wise objective against the whole Gram matrix, tr(R H R^T), for a given factorization (evaluation
# only; not part of the method's loop and not the default bench line): (d_out, d_in, d_block).
FULL_GRAM_WORKLOADS = {
    "llama7b_attn_full_gram_loss_4096x4096_b128": (4096, 4096, 128),
    "llama3_8b_gate_full_gram_loss_14336x4096_b128": (14336, 4096, 128),
    "llama70b_attn_full_gram_loss_8192x8192_b256": (8192, 8192, 256),
}

FP32_MFMA_PEAK = 157.3e12  # MI355X dense fp32 matrix peak, FLOP/s
BF16_MFMA_PEAK = 2.5e15    # MI355X dense bf16 matrix peak, FLOP/s

# HBM traffic per launch is not measured by this program: it comes from two rocprofv3 --pmc runs of it
# (FETCH_SIZE, then WRITE_SIZE, each scaled by what the counter reads for a plain 256 MiB device copy), whose
# summary is tracked here.  The file names the commands; the table is read at run time so that the figure
# and its source travel together.  Workloads without such a summary report null.
TRAFFIC_PROFILES = {"llama7b_attn_4096x4096_b128_2:4_50it": "profiles/chain_kernels_llama7b_attn_pmc.txt"}
TRAFFIC_KERNEL_ROWS = {"phase_A": "phase_A_stream_kernel", "phase_B": "phase_B_stream_kernel",
                       "phase_WS": "phase_WS_stream_kernel<true>", "phase_FB": "phase_FB_stream_kernel",
                       "phase_GS": "phase_GS_stream_kernel"}


def measured_traffic(workload, kind):
    """(bytes per launch, source) from the tracked counter summary, or (None, reason)."""
    rel = TRAFFIC_PROFILES.get(workload)
    if rel is None or kind not in TRAFFIC_KERNEL_ROWS:
        return None, "no tracked rocprofv3 --pmc summary for this workload / kernel"
    path = os.path.join(ROOT, rel)
    try:
        header, rows = None, {}
        for line in open(path):
            if line.startswith("#") or not line.strip():
                continue
            cols = line.split()
            if cols[0] == "kernel":
                header = line
                continue
            # kernel name (may contain spaces inside <...>), then 7 numeric columns
            name, vals = " ".join(cols[:-7]), cols[-7:]
            rows[name] = vals
        for name, vals in rows.items():
            if TRAFFIC_KERNEL_ROWS[kind] in name:
                fetch_mib, write_mib = float(vals[3]), float(vals[4])
                return (fetch_mib + write_mib) * 2 ** 20, rel
    except (OSError, ValueError, IndexError):
        pass
    return None, "could not read %s" % rel



def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def chain_algorithmic_flops(kind, d_out, d_in, b, N, M):
    """Algorithmic flops of one launch of a chain kernel: 2*P*b per dense b-deep block product,
    N/M of that where the N:M core itself is an operand, half for the symmetric Gram-type product."""
    P = d_out * d_in
    unit = 2.0 * P * b
    sparse = unit * N / M
    if kind in ("phase_A", "phase_B"):
        return sparse + unit + unit + 0.5 * unit
    if kind == "phase_GS":  # S' = A C (core operand), What, U, G
        return sparse + 3 * unit
    if kind == "phase_WS" and b <= 128:
        # What, U, G, V = (G.M) K (N:M-sparse operand), Z = (A^T A) V; S' = A C comes from the B step
        return 3 * unit + sparse + unit
    # phase_WS at d_block 256: S' = A C (core operand) is formed here as well
    # phase_FB: S = C B (core operand), What, grad_A, T, C^T T (core operand), T B^T
    return sparse + 3 * unit + sparse + unit


def run_block_workload(args, armor, synth, torch, dev, workload=None, steps=None, warmup=None):
    """Whole-block wall time for a multi-matrix workload; returns the result as a dict."""
    workload = workload or args.workload
    steps = steps or args.steps
    warmup = args.warmup if warmup is None else warmup
    cfg = BLOCK_WORKLOADS[workload]
    n_tok = args.tokens or cfg["tokens"]
    b, n_iters, hidden = cfg["d_block"], cfg["n_iters"], cfg["hidden"]
    # inputs: one hidden-width activation matrix per hidden-width site; the MLP down site is SiLU(gate)*up of it
    weights = {name: synth.torch_weight(d_out, cfg["sites"][site], 100 + k, dev)
               for k, (name, d_out, site) in enumerate(cfg["matrices"])}
    X = {}
    for k, (site, width) in enumerate(cfg["sites"].items()):
        if width == hidden:
            X[site] = synth.torch_calibration(n_tok, width, 10 + k, dev, outlier_frac=0.005, outlier_scale=20.0)
    for site, width in cfg["sites"].items():
        if width != hidden:  # scale the projections so that the activations are O(1) at the 0.02 init scale
            X[site] = synth.torch_mlp_down_inputs(X["mlp_in"], weights["gate"] * 8.0, weights["up"] * 8.0)
    H = {site: torch.empty((w, w), device=dev, dtype=torch.float32) for site, w in cfg["sites"].items()}
    gws_bytes = max(armor.gram_workspace_bytes(n_tok, w, True) for w in cfg["sites"].values())
    gws = torch.empty(max(gws_bytes, 256), device=dev, dtype=torch.uint8)
    ws_bytes = 0
    for (name, d_out, site) in cfg["matrices"]:
        for (N, M, sp) in cfg["patterns"]:
            ws_bytes = max(ws_bytes, armor.factorize_workspace_bytes(d_out, cfg["sites"][site], b, N, M, sparsity=sp))
    ws = torch.empty(ws_bytes, device=dev, dtype=torch.uint8)
    torch.cuda.synchronize()

    def step(timings=None):
        D = {}
        for site in cfg["sites"]:
            armor.gram(X[site], H=H[site], ws=gws)
            D[site] = armor.gram_diag(H[site])
        last = None
        for (name, d_out, site) in cfg["matrices"]:
            d_in = cfg["sites"][site]
            for (N, M, sp) in cfg["patterns"]:
                if timings is not None:
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                out = armor.factorize_layer(weights[name], D[site], b, N, M, n_iters, seed=0, sparsity=sp,
                                            unstructured_keep=(d_out * d_in) // 2 if sp else 0, ws=ws)
                if not sp:
                    armor.pack_nm(out["S"], out["mask_bits"], N, M, bf16=True)
                if timings is not None:
                    torch.cuda.synchronize()
                    tag = "%s_%dx%d_%s" % (name, d_out, d_in, "unstructured" if sp else "%d:%d" % (N, M))
                    timings[tag] = timings.get(tag, 0.0) + (time.perf_counter() - t0)
                last = out
        return last

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        out = step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    per = {}
    step(per)  # one extra, untimed-in-aggregate pass with a sync per matrix for the breakdown
    ms_per_step = (t1 - t0) * 1e3 / steps
    total_iters = n_iters * len(cfg["matrices"]) * len(cfg["patterns"])
    tr = out["loss_trace"].cpu().numpy()
    return ({
        "metric": "BCD iterations/sec per layer", "value": total_iters / (ms_per_step * 1e-3), "unit": "iterations/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": workload + ("_tokens%d" % n_tok if args.tokens else ""), "n_tokens": n_tok,
                   "d_block": b, "n_iters": n_iters, "matrices": len(cfg["matrices"]), "grams": len(cfg["sites"]),
                   "step": "all Grams + every factorize_layer (+ pack_nm) of the block"},
        "whole_block_wall_s": ms_per_step * 1e-3,
        "per_matrix": {k: {"s": v, "iterations_per_s": n_iters / v} for k, v in per.items()},
        "last_loss_first_last": [float(tr[0]), float(tr[-1])],
    })


def run_apply_workload(args, armor, synth, torch, dev):
    """One step = one armor_apply_packed call (Y = A(S(BX)) for the whole batch), factors and
    activations resident in HBM.  Factors are synthetic (random 2:4 core, near-identity wrappers):
    the product's cost does not depend on their values."""
    import numpy as np
    d_out, d_in, n_tok, b = APPLY_WORKLOADS[args.workload]
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    S = torch.randn((d_out, d_in), device=dev, generator=g) * 0.02
    scores = torch.rand((d_out, d_in // 4, 4), device=dev, generator=g)
    keep = scores.argsort(dim=-1, descending=True)[..., :2]
    mask = torch.zeros((d_out, d_in // 4, 4), device=dev, dtype=torch.uint8).scatter_(-1, keep, 1)
    S = S * mask.reshape(d_out, d_in)
    bits = (mask.to(torch.int32) << torch.arange(4, device=dev, dtype=torch.int32)).sum(-1).to(torch.uint8)
    A = torch.eye(b, device=dev).repeat(d_out // b, 1, 1) + 0.02 * torch.randn((d_out // b, b, b), device=dev, generator=g)
    Bw = torch.eye(b, device=dev).repeat(d_in // b, 1, 1) + 0.02 * torch.randn((d_in // b, b, b), device=dev, generator=g)
    X = torch.randn((n_tok, d_in), device=dev, generator=g).to(torch.bfloat16)
    vals, meta = armor.pack_nm(S.contiguous(), bits.contiguous(), 2, 4, bf16=True)
    Ab, Bb = armor.to_bf16(A.contiguous()), armor.to_bf16(Bw.contiguous())
    Y = torch.empty((n_tok, d_out), device=dev, dtype=torch.bfloat16)
    ws = torch.empty(armor.apply_workspace_bytes(n_tok, d_in), device=dev, dtype=torch.uint8)
    prepared = armor.apply_prepare(vals, meta, 2, 4)   # once per layer, outside the timed region
    torch.cuda.synchronize()

    def step():
        armor.apply_packed(X, Ab, prepared, Bb, 2, 4, Y=Y, ws=ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    armor.profile_enable(True)
    armor.profile_read()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = armor.profile_read()
    armor.profile_enable(False)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kernels = {k: {"launches": int(c), "avg_ms": ms / c} for k, (ms, c) in prof.items() if c > 0}
    P = d_out * d_in
    flops_main = 2.0 * n_tok * (P / 2 + d_out * b)          # 2:4 core product (kept entries only) + A wrapper
    flops_pre = 2.0 * n_tok * d_in * b
    main_ms = kernels["apply_main"]["avg_ms"]
    achieved = flops_main / (main_ms * 1e-3) / 1e12
    kernels["apply_main"]["tflops_algorithmic"] = achieved
    kernels["apply_main"]["tflops_dense_equivalent"] = 2.0 * n_tok * (P + d_out * b) / (main_ms * 1e-3) / 1e12
    pre_bytes = 2 * 2 * n_tok * d_in                           # X in, U out
    kernels["apply_pre"]["hbm_GBps"] = pre_bytes / (kernels["apply_pre"]["avg_ms"] * 1e-3) / 1e9
    kernels["apply_pre"]["tflops_algorithmic"] = flops_pre / (kernels["apply_pre"]["avg_ms"] * 1e-3) / 1e12
    result = {
        "metric": "tokens/s through one factorized layer (batched y = A(S(Bx)))", "value": n_tok / (ms_per_step * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "d_out": d_out, "d_in": d_in, "n_tokens": n_tok, "d_block": b,
                   "pattern": "2:4", "step": "armor_apply_packed (pre-product + core product with wrapper epilogue)"},
        "roofline": {"bound": "mfma", "kernel": "apply_main", "achieved": achieved, "peak": BF16_MFMA_PEAK / 1e12,
                     "unit": "TFLOP/s", "frac": achieved / (BF16_MFMA_PEAK / 1e12), "traffic": None,
                     "algorithmic_flops_per_launch": flops_main, "avg_launch_ms": main_ms},
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        # about 10-20 s of single-thread oracle time (44 tokens/s on the 13824 x 5120 layer)
        sample = 2048 if d_out * d_in <= 1 << 24 else (512 if d_out * d_in <= 1 << 27 else 128)
        ev = vals[:, :].float().cpu().numpy()
        idx = armor.unpack_meta(meta.cpu().numpy(), d_in, 2, 4)
        c0 = time.perf_counter()
        ref = oracle.apply_packed(X[:sample].float().cpu().numpy(), Ab.float().cpu().numpy(), ev, idx,
                                  Bb.float().cpu().numpy(), 2, 4, round_bf16=True)
        c1 = time.perf_counter()
        got = Y[:sample].float().cpu().numpy().astype(np.float64)
        result["cpu_baseline"] = {"value": sample / (c1 - c0), "unit": "tokens/s", "cores": 1, "kind": "oracle",
                                  "sample": "%d of the %d tokens through the same layer; %.1f s wall" % (sample, n_tok, c1 - c0),
                                  "rel_fro_err_vs_gpu": float(np.linalg.norm(got - ref) / np.linalg.norm(ref))}
    print(json.dumps(result))


def run_full_gram_workload(args, armor, synth, torch, dev):
    """One step = one armor_proxy_loss_full_h call: the forward chain that leaves R = Wbar - A S B, then <R, R H>."""
    import numpy as np
    d_out, d_in, b = FULL_GRAM_WORKLOADS[args.workload]
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    W = synth.torch_weight(d_out, d_in, 0, dev, bf16=False).float().contiguous()
    X = synth.torch_calibration(8192, d_in, 0, dev, outlier_frac=0.005, outlier_scale=20.0, dtype=torch.float32)
    H = (X.T @ X).contiguous()
    S = (W * (torch.rand((d_out, d_in), device=dev, generator=g) > 0.5)).contiguous()
    A = (torch.eye(b, device=dev).repeat(d_out // b, 1, 1) + 0.02 * torch.randn((d_out // b, b, b), device=dev, generator=g)).contiguous()
    Bw = (torch.eye(b, device=dev).repeat(d_in // b, 1, 1) + 0.02 * torch.randn((d_in // b, b, b), device=dev, generator=g)).contiguous()
    ws = torch.empty(armor.load_library().armor_proxy_loss_full_h_workspace_bytes(d_out, d_in, b), device=dev, dtype=torch.uint8)
    for _ in range(args.warmup):
        out = armor.proxy_loss_full_h(W, A, S, Bw, H, ws=ws)
    torch.cuda.synchronize()
    armor.profile_enable(True)
    armor.profile_read()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out = armor.proxy_loss_full_h(W, A, S, Bw, H, ws=ws)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = armor.profile_read()
    armor.profile_enable(False)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kernels = {k: {"launches": int(cn), "avg_ms": ms / cn} for k, (ms, cn) in prof.items() if cn > 0}
    flops = 2.0 * d_out * d_in * d_in                       # R H; the reduction <R, R H> rides in its epilogue
    k_ms = kernels["full_gram_loss"]["avg_ms"]
    split = d_out % 128 == 0 and d_in % 128 == 0            # 128-wide tiles: six bf16 partial products per fp32 product
    achieved = (6.0 if split else 1.0) * flops / (k_ms * 1e-3) / 1e12
    peak = (BF16_MFMA_PEAK if split else FP32_MFMA_PEAK) / 1e12
    result = {
        "metric": "full-Gram loss evaluations/s", "value": 1e3 / ms_per_step, "unit": "evaluations/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "d_out": d_out, "d_in": d_in, "d_block": b,
                   "step": "armor_proxy_loss_full_h (forward chain leaving R, then <R, R H>)"},
        "loss": float(out.item()),
        "roofline": {"bound": "mfma", "kernel": "full_h_loss_kernel", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": None,
                     "flops_counted": "executed bf16 flops per launch (6 partial products per fp32 product)" if split else "fp32 flops",
                     "algorithmic_flops_per_launch": flops, "avg_launch_ms": k_ms,
                     "fp32_equivalent": {"achieved": flops / (k_ms * 1e-3) / 1e12, "peak": FP32_MFMA_PEAK / 1e12,
                                         "frac": flops / (k_ms * 1e-3) / FP32_MFMA_PEAK}},
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        rows = 256                                              # the oracle on a slice of rows (the value is a sum over rows)
        c0 = time.perf_counter()
        ref = oracle.proxy_loss_full_h(W[:rows].cpu().numpy(), A[:rows // b].cpu().numpy(), S[:rows].cpu().numpy(),
                                       Bw.cpu().numpy(), H.cpu().numpy())
        c1 = time.perf_counter()
        got = armor.proxy_loss_full_h(W[:rows].contiguous(), A[:rows // b].contiguous(), S[:rows].contiguous(), Bw, H).item()
        result["cpu_baseline"] = {"value": rows / d_out / (c1 - c0), "unit": "evaluations/s", "cores": os.cpu_count(), "kind": "oracle",
                                  "sample": "the first %d of %d rows (the value is a sum over rows), scaled; %.1f s wall" % (rows, d_out, c1 - c0),
                                  "rel_err_vs_gpu_on_the_sample": abs(got - ref) / abs(ref)}
    print(json.dumps(result))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default 3; 100 for the ~1 ms apply workloads)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps first (default 1; 20 for the apply workloads)")
    ap.add_argument("--workload", default=DEFAULT, choices=sorted(WORKLOADS) + sorted(BLOCK_WORKLOADS) + sorted(APPLY_WORKLOADS) + sorted(FULL_GRAM_WORKLOADS))
    ap.add_argument("--variant", default="gd", choices=["gd", "adam"],
                    help="continuous step: sequential 1/beta gradient steps (default; the monotone variant) or the "
                         "joint Adam step the authors run in practice (lr 1e-4)")
    ap.add_argument("--pattern", default="", help="N:M override for the single-layer workloads, e.g. 4:8, 5:8, 6:8")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-block", action="store_true",
                    help="default workload only: skip the extra Llama-3-8B decoder-block timing (key llama3_8b_block)")
    ap.add_argument("--cpu-iters", type=int, default=2)
    ap.add_argument("--tokens", type=int, default=0,
                    help="override the number of calibration tokens (profiling runs only; the reported "
                         "workload name gets a suffix)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain device copy of known size (256 MiB read + 256 MiB written, 3 times) "
                         "so that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings can be scaled")
    args = ap.parse_args()
    short = args.workload in APPLY_WORKLOADS or args.workload in FULL_GRAM_WORKLOADS  # a step of ~1 ms: a few of them would time the clock ramp
    if args.steps is None:
        args.steps = 100 if short else 3
    if args.warmup is None:
        args.warmup = 20 if short else 1
    if args.copy_calibration:
        import torch
        src = torch.ones(64 * 1024 * 1024, device="cuda:0", dtype=torch.float32)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4,
                                               "copies": 3}}))
        return
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every box has one GPU); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2510_05528_amd as armor
    from paper_2510_05528_amd import synth

    armor.load_library()
    dev = torch.device("cuda:0")
    if args.workload in BLOCK_WORKLOADS:
        print(json.dumps(run_block_workload(args, armor, synth, torch, dev)))
        return
    if args.workload in APPLY_WORKLOADS:
        run_apply_workload(args, armor, synth, torch, dev)
        return
    if args.workload in FULL_GRAM_WORKLOADS:
        run_full_gram_workload(args, armor, synth, torch, dev)
        return
    d_out, d_in, n_tok, b, N, M, n_iters, w_bf16, x_bf16, ofrac, oscale = WORKLOADS[args.workload]
    workload_name = args.workload + ("_adam" if args.variant == "adam" else "")
    if args.pattern:
        N, M = (int(v) for v in args.pattern.split(":"))
        workload_name = workload_name.replace("2:4", args.pattern)
    variant = 1 if args.variant == "adam" else 0
    if args.tokens > 0:
        n_tok = args.tokens
        workload_name += "_tokens%d" % n_tok

    # ---- synthetic inputs, resident in HBM before any timed region ----
    W = synth.torch_weight(d_out, d_in, 0, dev, bf16=w_bf16)
    X = synth.torch_calibration(n_tok, d_in, 0, dev, outlier_frac=ofrac, outlier_scale=oscale,
                                dtype=torch.bfloat16 if x_bf16 else torch.float32)
    H = torch.empty((d_in, d_in), device=dev, dtype=torch.float32)
    ws = torch.empty(armor.factorize_workspace_bytes(d_out, d_in, b, N, M, variant=variant), device=dev, dtype=torch.uint8)
    gws = torch.empty(max(armor.gram_workspace_bytes(n_tok, d_in, x_bf16), 256), device=dev, dtype=torch.uint8)
    torch.cuda.synchronize()

    def step():
        armor.gram(X, H=H, ws=gws)
        D = armor.gram_diag(H)
        out = armor.factorize_layer(W, D, b, N, M, n_iters, seed=0, ws=ws, variant=variant)
        vals, meta = armor.pack_nm(out["S"], out["mask_bits"], N, M, bf16=True)
        return out, D, vals, meta

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    armor.profile_enable(True)
    armor.profile_read()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out, D, vals, meta = step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = armor.profile_read()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = n_iters / (ms_per_step * 1e-3)
    # context, outside the timed step: the weights of Eq. 2 straight from X (all the method itself needs
    # of the calibration data), one HBM-bound pass instead of the full Gram
    for _ in range(3):
        armor.gram_diag_x(X)
    torch.cuda.synchronize()
    diag_x = armor.profile_read().get("gram_diag_x", (0.0, 0))
    armor.profile_enable(False)

    # ---- roofline of the dominant chain kernel, from the library's HIP events ----
    kernels = {}
    for k, (ms, cnt) in prof.items():
        if cnt > 0:
            kernels[k] = {"launches": int(cnt), "avg_ms": ms / cnt, "total_ms_per_step": ms / args.steps}
    chain = {k: v for k, v in kernels.items() if k.startswith("phase_")}
    dom = max(chain, key=lambda k: chain[k]["total_ms_per_step"])
    flops = chain_algorithmic_flops(dom, d_out, d_in, b, N, M)
    achieved = flops / (chain[dom]["avg_ms"] * 1e-3) / 1e12
    traffic, traffic_source = measured_traffic(args.workload if not args.pattern and not args.tokens else "", dom)
    roofline = {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": FP32_MFMA_PEAK / 1e12,
                "unit": "TFLOP/s", "frac": achieved / (FP32_MFMA_PEAK / 1e12),
                "traffic": traffic, "traffic_source": traffic_source,
                "algorithmic_flops_per_launch": flops, "avg_launch_ms": chain[dom]["avg_ms"]}
    if b >= 128:
        # At d_block 128 and 256 the fp32 products run on the bf16 matrix instruction: every operand is cut exactly
        # into three bf16 pieces and a product takes six partial products (fp32 accumulation).  The kernel is priced
        # against the peak of the instruction it issues: achieved = the bf16 flops it executes (6 x the dense fp32
        # products it forms: the N:M core is multiplied as a dense operand, a symmetric product forms 10 of its
        # 16 tiles at b = 128 and 3 of 4 sub-tiles at b = 256).  The delivered fp32 contraction, which is what
        # the figure meant before the switch of instruction, stays beside it as `fp32_equivalent`.
        sym = 0.625 if b == 128 else 0.75
        executed_dense = {"phase_A": 2 * (3 + sym), "phase_B": 2 * (3 + sym), "phase_WS": 10.0, "phase_GS": 8.0,
                          "phase_FB": 12.0}.get(dom)
        if executed_dense:
            ex = 6.0 * executed_dense * d_out * d_in * b
            roofline["fp32_equivalent"] = {"achieved": achieved, "peak": FP32_MFMA_PEAK / 1e12,
                                           "frac": achieved / (FP32_MFMA_PEAK / 1e12),
                                           "note": "algorithmic fp32 flops over the same duration, against the fp32 matrix peak"}
            roofline["matrix_instruction"] = "v_mfma_f32_32x32x16_bf16, 6 partial products per fp32 product"
            roofline["flops_counted"] = "executed bf16 flops per launch"
            roofline["executed_flops_per_launch"] = ex
            roofline["achieved"] = ex / (chain[dom]["avg_ms"] * 1e-3) / 1e12
            roofline["peak"] = BF16_MFMA_PEAK / 1e12
            roofline["frac"] = roofline["achieved"] / roofline["peak"]
    for k in chain:
        kernels[k]["tflops_algorithmic"] = chain_algorithmic_flops(k, d_out, d_in, b, N, M) / (chain[k]["avg_ms"] * 1e-3) / 1e12
    # HBM-bound kernels: algorithmic bytes (each operand read or written once) over the measured duration
    P, wb = d_out * d_in, (2 if w_bf16 else 4)
    hbm_bytes = {
        "sparse_step": 4 * P,                                   # one pass over the core gradient
        "normalize": 2 * wb * P + 4 * P,                        # W for the column norms, W again for rows + scaling, Wbar out
        "init": 4 * P + 4 * P + P // M,                         # Wbar in, core out, one mask byte per group
        "pack_nm": 4 * P + P // M + 2 * (P * N // M) + P * N // M // 4,  # core + mask in, bf16 values + 2-bit indices out
    }
    for k, nbytes in hbm_bytes.items():
        if k in kernels:
            kernels[k]["algorithmic_bytes"] = nbytes
            kernels[k]["hbm_GBps"] = nbytes / (kernels[k]["avg_ms"] * 1e-3) / 1e9
            kernels[k]["hbm_frac_of_8TBps"] = kernels[k]["hbm_GBps"] / 8000.0
    if diag_x[1] > 0:
        nbytes = n_tok * d_in * (2 if x_bf16 else 4)
        kernels["gram_diag_x_not_in_step"] = {"launches": int(diag_x[1]), "avg_ms": diag_x[0] / diag_x[1], "algorithmic_bytes": nbytes,
                                              "hbm_GBps": nbytes / (diag_x[0] / diag_x[1] * 1e-3) / 1e9}
    if "gram" in kernels:
        kernels["gram"]["tflops_algorithmic"] = n_tok * d_in * (d_in + 1) / (kernels["gram"]["avg_ms"] * 1e-3) / 1e12

    trace = out["loss_trace"].cpu().numpy()
    result = {
        "metric": "BCD iterations/sec per layer", "value": value, "unit": "iterations/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": workload_name, "d_out": d_out, "d_in": d_in, "n_tokens": n_tok, "d_block": b,
                   "pattern": "%d:%d" % (N, M), "n_iters": n_iters,
                   "step": "gram + gram_diag + factorize_layer + pack_nm"},
        "s_per_layer": ms_per_step * 1e-3,
        "loss_first_last": [float(trace[0]), float(trace[-1])],
        "roofline": roofline,
        "kernels": kernels,
    }

    # ---- CPU oracle on a bounded sample of the same layer (reported baseline, not the target) ----
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        Wh = W.float().cpu().numpy()
        Dh = D.cpu().numpy()
        cpu_iters = args.cpu_iters if d_out * d_in > 1 << 20 else n_iters
        c0 = time.perf_counter()
        if variant == 1:
            ref = oracle.factorize_layer_adam(Wh, Dh, b, N, M, cpu_iters, seed=0)
        else:
            ref = oracle.factorize_layer(Wh, Dh, b, N, M, cpu_iters, seed=0)
        c1 = time.perf_counter()
        cores = int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)
        result["cpu_baseline"] = {
            "value": cpu_iters / (c1 - c0), "unit": "iterations/s", "cores": cores, "kind": "oracle",
            "sample": "%d of %d BCD iterations of the same %dx%d layer (normalise + init + iterations + per-iteration "
                      "loss; Gram excluded, D taken from the GPU Gram); %.1f s wall" % (cpu_iters, n_iters, d_out, d_in, c1 - c0),
            "cpu_model": cpu_model(),
        }
        # the same oracle on one thread, on a row slice (its cost is linear in d_out): one iteration
        if d_out * d_in > 1 << 20 and variant == 0:
            rows = max(b, (d_out // 8) // b * b)
            oracle.set_threads(1)
            s0 = time.perf_counter()
            oracle.factorize_layer(Wh[:rows], Dh, b, N, M, 1, seed=0)
            s1 = time.perf_counter()
            oracle.set_threads(cores)
            result["cpu_baseline"]["single_thread"] = {
                "value": 1.0 / ((s1 - s0) * d_out / rows), "unit": "iterations/s", "cores": 1,
                "sample": "1 BCD iteration of the first %d of %d rows of the same layer, %.1f s wall, scaled by "
                          "%d/%d (the oracle's cost is linear in the row count)" % (rows, d_out, s1 - s0, d_out, rows)}
        # cheap cross-check of the timed run against the oracle's first iterations
        result["cpu_baseline"]["loss_trace_rel_err_first_iters"] = float(
            np.max(np.abs(trace[:cpu_iters + 1] - ref["loss_trace"]) / ref["loss_trace"]))
    if args.workload == DEFAULT and variant == 0 and not args.pattern and not args.tokens and not args.no_block:
        # the Llama-3-8B-shaped decoder block of the baseline configs (7 matrices, 4 Grams, 50 iterations each):
        # whole-block wall time and per-matrix breakdown, one warm-up pass and one timed pass
        del W, X, H, ws, gws, out, vals, meta
        torch.cuda.empty_cache()
        blk = run_block_workload(args, armor, synth, torch, dev, workload="llama3_8b_block_b128_2:4_50it", steps=1, warmup=1)
        result["llama3_8b_block"] = {k: blk[k] for k in ("whole_block_wall_s", "value", "unit", "per_matrix", "config")}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
