"""PRAC hot-path benchmark on one MI355X.

One "step" is what Alg. 1 + Alg. 2 do for one linear layer at training step t:
refresh the basis when t mod T == 0 (T = 500, the paper's pre-training interval),
compress the saved activation (C = X P) and form the weight gradient
(dW = P_s (C^T dY)).  Workload: the LLaMA-1B attention-projection shape
(N = 32768 tokens, d = m = 2048, k = r = 128, bf16), synthetic activations with
a power-law spectrum and outlier channels, rotated over four independent input
sets so that no step finds its inputs in the 256 MB last-level cache.

Prints ONE JSON line: metric, value (tokens/s), roofline of the dominant kernel, the oracle timed on the host.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

WORKLOAD = dict(name="llama1b_attn_proj", N=32768, d=2048, m=2048, k=128, r=128, alpha=0.8,
                n_out=8, out_scale=30.0, dy_std=1e-3, refresh_every=500, n_sets=4, layer_seed=3000,
                warm_iters=2, warm_oversample=-1, row_stride=1)
# The other layer shapes of the configurations (same protocol; `--workload NAME`).  The headline
# above is what the driver's plain `python bench.py` measures.
OTHER_WORKLOADS = {
    "llama1b_up_gate": dict(WORKLOAD, name="llama1b_up_gate", m=5461),
    "llama1b_down": dict(WORKLOAD, name="llama1b_down", d=5461, m=2048, n_sets=2),
    "llama130m_attn_proj": dict(WORKLOAD, name="llama130m_attn_proj", d=768, m=768, k=64, r=64, alpha=1.0, n_out=4,
                                out_scale=20.0, layer_seed=2000),
    "llama130m_down": dict(WORKLOAD, name="llama130m_down", d=2048, m=768, k=64, r=64, alpha=1.0, n_out=4,
                           out_scale=20.0, layer_seed=2001),
    "rank_sweep_0_256": dict(WORKLOAD, name="rank_sweep_0_256", k=0, r=256, n_out=0, layer_seed=4000),
    "rank_sweep_512_512": dict(WORKLOAD, name="rank_sweep_512_512", k=512, r=512, n_out=0, layer_seed=4001),
    # basis refitted on every step from the Gram matrix of a 4096-token subsample
    "llama7b_up_gate": dict(WORKLOAD, name="llama7b_up_gate", N=16384, d=4096, m=11008, k=256, r=256, n_out=16,
                            out_scale=50.0, refresh_every=1, row_stride=4, n_sets=2, layer_seed=5000),
}
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def algorithmic_bytes(kind: str, w: dict) -> float:
    """Bytes the method must move per launch of a kernel (bf16 data, fp32 T)."""
    N, d, m, c = w["N"], w["d"], w["m"], w["k"] + w["r"]
    if kind == "compress":
        return 2.0 * (N * d + d * c + N * c)
    if kind == "ct_dy":
        return 2.0 * (N * c + N * m) + 4.0 * c * m
    if kind == "t_reduce":
        return 4.0 * c * m + 2.0 * c * m
    if kind == "p_t":
        return 2.0 * (d * c + c * m + d * m)
    raise KeyError(kind)


def algorithmic_flops(kind: str, w: dict) -> float:
    N, d, m, c = w["N"], w["d"], w["m"], w["k"] + w["r"]
    return {"compress": 2.0 * N * d * c, "ct_dy": 2.0 * N * c * m, "t_reduce": float(c * m),
            "p_t": 2.0 * d * c * m}[kind]


def read_traffic(kind: str, workload: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, or None."""
    path = os.path.join(ROOT, "profiles", "pmc_traffic.md")
    if not os.path.exists(path):
        return None
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 4 and cells[0] == kind and cells[1] == workload:
            try:
                return float(cells[2]) + float(cells[3])
            except ValueError:
                return None
    return None


def cpu_baseline(X, dY, k, r, refresh_every):
    """The fp64 oracle timed on the host cores: one basis fit (Gram, eigendecomposition,
    complement draw and QR) plus compress + weight gradient over the whole batch, combined
    as the GPU path combines them: one fit per `refresh_every` steps."""
    import numpy as np

    import synth_inputs as si
    from oracle import prac_oracle as orc

    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    X64, dY64 = si.as_f64(X), si.as_f64(dY)
    t0 = time.perf_counter()
    P64, s = orc.fit_basis(X64, k, r, seed=1234, draw=0)
    t_fit = time.perf_counter() - t0
    t_cw = float("inf")
    for _ in range(2):
        t0 = time.perf_counter()
        C = orc.compress(X64, P64)
        dW = orc.weight_grad(C, dY64, P64, k, s)
        t_cw = min(t_cw, time.perf_counter() - t0)
    assert np.isfinite(dW).all()
    n = X64.shape[0]
    return dict(value=n / (t_cw + t_fit / refresh_every), unit="tokens/s", cores=int(cores), kind="oracle",
                sample=f"all {n} tokens of one batch in fp64 numpy: fit {t_fit:.2f} s (once per {refresh_every} "
                       f"steps), compress + weight-grad {t_cw:.2f} s (best of 2)")


BLOCK_WORKLOAD = "llama1b_block"


def run_block(args):
    """All seven linear layers of one LLaMA-1B transformer block with subspace sharing (Section 5.1):
    q/k/v share the compressed attention input, up/gate the compressed MLP input; o and down have
    their own.  4 compressions + 7 weight gradients per step, each of the 4 bases refreshed (tracking
    refit on the step's batch) every 500 steps."""
    import torch

    import synth_inputs as si
    from paper_2602_23111_amd.prac import C_PACKED, Prac

    N, k, r, refresh_every, n_sets = 32768, 128, 128, 500, 2
    c = k + r
    groups = [("attn_in:q,k,v", 2048, [2048, 2048, 2048]), ("attn_out:o", 2048, [2048]),
              ("mlp_in:up,gate", 2048, [5461, 5461]), ("mlp_down:down", 5461, [2048])]
    ld8 = lambda n: (n + 7) // 8 * 8
    dev = torch.device("cuda:0")
    torch.cuda.set_device(0)
    ctx = Prac(0)
    G = []
    for gi, (name, d, ms) in enumerate(groups):
        seed = 3000 + 10 * gi
        g = dict(name=name, d=d, ms=ms, P=torch.zeros((d, c), dtype=torch.float32, device=dev), lp=None, scale=0.0,
                 X=[si.activation_torch(N, d, 0.8, seed, 8, 30.0, torch.bfloat16, dev, ld=ld8(d), batch=i)
                    for i in range(n_sets)],
                 dY=[[si.grad_output_torch(N, m, 1e-3, seed + 100 + 10 * i + j, torch.bfloat16, dev, ld=ld8(m))
                      for j, m in enumerate(ms)] for i in range(n_sets)],
                 C=[torch.empty(ctx.compressed_bytes(N, c) // 2, dtype=torch.bfloat16, device=dev) for _ in range(n_sets)],
                 dW=[torch.empty((d, ld8(m)), dtype=torch.bfloat16, device=dev)[:, :m] for m in ms])
        G.append(g)
    fits = [0]

    def layer_compress(g, i):
        ctx.compress(g["X"][i], g["P"], P_lp=g["lp"], out=g["C"][i], layout=C_PACKED)

    def layer_wgrad(g, i):
        if len(g["ms"]) == 1:
            ctx.weight_grad(g["C"][i], g["dY"][i][0], g["P"], k, r, g["scale"], P_lp=g["lp"], out=g["dW"][0],
                            layout=C_PACKED)
        else:
            ctx.weight_grad_shared(g["C"][i], g["dY"][i], g["P"], k, r, g["scale"], P_lp=g["lp"], outs=g["dW"],
                                   layout=C_PACKED)

    def step(t):
        i = t % n_sets
        for g in G:
            if t % refresh_every == 0:
                warm = g["lp"] is not None
                _, g["lp"], g["scale"] = ctx.fit_basis(g["X"][i], k, r, seed=1234, draw=t // refresh_every, P=g["P"],
                                                       warm_start=warm, iters=WORKLOAD["warm_iters"] if warm else 0,
                                                       oversample=WORKLOAD["warm_oversample"] if warm else 0)
                fits[0] += 1
            layer_compress(g, i)
            layer_wgrad(g, i)

    for t in range(max(min(args.warmup, 5), 1)):
        step(t)
    torch.cuda.synchronize()

    def wall(fn, reps=20):
        for t in range(2):
            fn(t % n_sets)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(reps):
            fn(t % n_sets)
        torch.cuda.synchronize()
        return 1e6 * (time.perf_counter() - t0) / reps

    layers_us = {}
    for g in G:
        layers_us[g["name"]] = {"compress": wall(lambda i: layer_compress(g, i)), "weight_grad": wall(lambda i: layer_wgrad(g, i))}
    fits[0] = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(args.steps):
        step(t)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ctx.sync_status()
    ms_per_step = 1e3 * elapsed / args.steps
    # algorithmic bytes of the block: every X, dY, C (written and read once per gradient launch), P and dW once
    by = 0.0
    for _, d, ms in groups:
        by += 2.0 * (N * d + d * c + N * c) + 2.0 * (N * c + sum(N * m + d * m for m in ms) + d * c)
    out = {
        "metric": "PRAC compress+weight-grad tokens/s at LLaMA-1B shape",
        "value": N / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{BLOCK_WORKLOAD}: the 7 linear layers of one LLaMA-1B block, N={N} k={k} r={r} bf16, dW bf16, "
                               f"q/k/v and up/gate share their compressed input (4 compressions, 7 weight gradients per "
                               f"step), 4 bases refreshed every {refresh_every} steps ({fits[0]} refits in the timed region), "
                               f"{n_sets} rotating input sets"},
        "roofline": {"kernel": "whole step", "bound": "hbm", "achieved": by / (ms_per_step * 1e-3) / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": by / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "traffic": None},
        "cpu_baseline": None,
        "layers_us": layers_us,
    }
    print(json.dumps(out))
    ctx.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--cpu-sample", type=int, default=1, help="0: skip the oracle's timed run on the host")
    ap.add_argument("--workload", default=WORKLOAD["name"], choices=[WORKLOAD["name"], BLOCK_WORKLOAD] + sorted(OTHER_WORKLOADS),
                    help="layer shape to run (default: the headline attention projection of the LLaMA-1B configuration)")
    ap.add_argument("--others", type=int, default=1,
                    help="0: skip timing the fused forward and the reconstruction (outside the timed region)")
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="after the timed region, also run three plain device copies of this many MB "
                         "(a kernel of known traffic, for scaling rocprofv3 --pmc byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import synth_inputs as si
    from paper_2602_23111_amd.prac import C_PACKED, KERNEL_KINDS, Prac

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.workload == BLOCK_WORKLOAD:
        return run_block(args)
    w = WORKLOAD if args.workload == WORKLOAD["name"] else OTHER_WORKLOADS[args.workload]
    if w is not WORKLOAD:
        args.others = 0          # the extra entry points are timed at the headline shape only
        args.cpu_sample = 0      # ... and so is the oracle on the host (an eigendecomposition of d x d)
        if w["refresh_every"] == 1 and args.steps == 500:
            args.steps = 50      # a refit per step: keep the default run short
    N, d, m, k, r = w["N"], w["d"], w["m"], w["k"], w["r"]
    ld8 = lambda n: (n + 7) // 8 * 8
    c = k + r
    dev = torch.device("cuda:0")
    torch.cuda.set_device(0)
    ctx = Prac(0)

    Xs, dYs, Cs = [], [], []
    for i in range(w["n_sets"]):
        # batches of one layer: same spectrum and principal subspace, fresh tokens
        Xs.append(si.activation_torch(N, d, w["alpha"], w["layer_seed"], w["n_out"], w["out_scale"], torch.bfloat16,
                                      dev, ld=ld8(d), batch=i))
        dYs.append(si.grad_output_torch(N, m, w["dy_std"], w["layer_seed"] + 100 + i, torch.bfloat16, dev, ld=ld8(m)))
        Cs.append(torch.empty(ctx.compressed_bytes(N, c) // 2, dtype=torch.bfloat16, device=dev))
    dW = torch.empty((d, ld8(m)), dtype=torch.bfloat16, device=dev)[:, :m]
    P = torch.zeros((d, c), dtype=torch.float32, device=dev)
    state = dict(lp=None, scale=0.0, fits=0)

    def step(t: int):
        i = t % w["n_sets"]
        if t % w["refresh_every"] == 0:
            # every refresh after the first starts the subspace iteration from the previous Q1
            warm = state["lp"] is not None
            _, state["lp"], state["scale"] = ctx.fit_basis(Xs[i], k, r, seed=1234, draw=t // w["refresh_every"], P=P,
                                                           warm_start=warm, iters=w["warm_iters"] if warm else 0,
                                                           oversample=w["warm_oversample"] if warm else 0,
                                                           row_stride=w["row_stride"])
            state["fits"] += 1
        ctx.compress(Xs[i], P, P_lp=state["lp"], out=Cs[i], layout=C_PACKED)
        ctx.weight_grad(Cs[i], dYs[i], P, k, r, state["scale"], P_lp=state["lp"], out=dW, layout=C_PACKED)

    # warm-up (includes the first fit so that scratch is allocated), then find the dominant kernel
    for t in range(max(args.warmup, 1)):
        step(t)
    torch.cuda.synchronize()
    per_kernel_us = {}
    for kind in ("compress", "ct_dy", "t_reduce", "p_t"):
        ctx.profile_select(KERNEL_KINDS[kind])
        for t in range(1, 9):
            step(t)
        ms, n = ctx.profile_read()
        per_kernel_us[kind] = 1e3 * ms / max(n, 1)
    dominant = max(per_kernel_us, key=per_kernel_us.get)
    ctx.profile_select(KERNEL_KINDS[dominant])
    ctx.profile_read()

    # fit alone, for the record (not part of `value` beyond its share of the timed steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ctx.fit_basis(Xs[0], k, r, seed=1234, draw=0, P=P, warm_start=True, iters=w["warm_iters"],
                  oversample=w["warm_oversample"], row_stride=w["row_stride"])
    torch.cuda.synchronize()
    fit_ms = 1e3 * (time.perf_counter() - t0)

    # the other entry points of the path at the same shape, outside the timed region: forward
    # fused with the compression (W stored m x d, the layout of Section 5.2) and the reconstruction
    other_us = {}
    if args.others:
        g = torch.Generator(device=dev)
        g.manual_seed(3200)
        W = (torch.randn((m, d), generator=g, device=dev) * 0.02).to(torch.bfloat16)
        Y = torch.empty((N, m), dtype=torch.bfloat16, device=dev)
        for kind, fn in (("fused_fwd", lambda i: ctx.compress_fused_fwd(Xs[i], W, P, w_layout=1, P_lp=state["lp"], Y=Y,
                                                                        out=Cs[i], layout=C_PACKED)),
                         ("reconstruct", lambda i: ctx.reconstruct(Cs[i], P, k, r, state["scale"], N=N, out=Y,
                                                                   layout=C_PACKED))):
            fn(0)
            ctx.profile_select(KERNEL_KINDS[kind])
            for t in range(8):
                fn(t % w["n_sets"])
            ms, n = ctx.profile_read()
            other_us[kind] = 1e3 * ms / max(n, 1)
        # for scale: the vendor library's forward alone (torch.matmul, hipBLASLt); unfused = this + compress
        for _ in range(3):
            torch.matmul(Xs[0], W.t(), out=Y)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for t in range(8):
            torch.matmul(Xs[t % w["n_sets"]], W.t(), out=Y)
        e1.record()
        torch.cuda.synchronize()
        other_us["fwd_vendor_gemm"] = 1e3 * e0.elapsed_time(e1) / 8
        del W, Y
        # query / key / value gradients from the one compressed activation they share (Section 5.1):
        # one call for the three against three calls, wall clock over 8 repetitions each
        dY3 = [dYs[0], dYs[1], dYs[2]]
        dW3 = [torch.empty((d, m), dtype=torch.bfloat16, device=dev) for _ in range(3)]
        ctx.profile_select(0)

        def wall(fn, reps=8):
            fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return 1e6 * (time.perf_counter() - t0) / reps

        other_us["wgrad_qkv_shared"] = wall(lambda: ctx.weight_grad_shared(
            Cs[0], dY3, P, k, r, state["scale"], P_lp=state["lp"], outs=dW3, layout=C_PACKED))
        other_us["wgrad_qkv_three_calls"] = wall(lambda: [ctx.weight_grad(
            Cs[0], y, P, k, r, state["scale"], P_lp=state["lp"], out=o, layout=C_PACKED) for y, o in zip(dY3, dW3)])
        del dW3
        ctx.profile_select(KERNEL_KINDS[dominant])
        ctx.profile_read()
        for i in range(w["n_sets"]):  # C was overwritten by the fused launches with the same values
            ctx.compress(Xs[i], P, P_lp=state["lp"], out=Cs[i], layout=C_PACKED)

    state["fits"] = 0
    # an event pair costs about 4 us of stream time: every 8th launch of the dominant kernel carries one
    sample_every = 8 if args.steps >= 64 else 1
    ctx.set_tuning(2, sample_every)
    ctx.profile_select(KERNEL_KINDS[dominant])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(args.steps):
        step(t)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    dom_each = ctx.profile_read_each()
    ctx.set_tuning(2, 1)
    dom_ms, dom_n = sum(dom_each), len(dom_each)
    ctx.profile_select(0)
    ctx.sync_status()

    ms_per_step = 1e3 * elapsed / args.steps
    dom_us = 1e3 * dom_ms / max(dom_n, 1)
    ach_gbs = algorithmic_bytes(dominant, w) / (dom_us * 1e-6) / 1e9
    ach_tf = algorithmic_flops(dominant, w) / (dom_us * 1e-6) / 1e12
    # the resource whose roofline time is the longer one bounds the kernel
    hbm_bound = ach_gbs / HBM_PEAK_GBS >= ach_tf / MFMA_BF16_PEAK_TFLOPS
    roofline = dict(kernel=dominant, bound="hbm" if hbm_bound else "mfma",
                    achieved=ach_gbs if hbm_bound else ach_tf,
                    peak=HBM_PEAK_GBS if hbm_bound else MFMA_BF16_PEAK_TFLOPS,
                    unit="GB/s" if hbm_bound else "TFLOP/s",
                    frac=ach_gbs / HBM_PEAK_GBS if hbm_bound else ach_tf / MFMA_BF16_PEAK_TFLOPS,
                    traffic=read_traffic(dominant, w["name"]),
                    avg_us=dom_us, median_us=1e3 * sorted(dom_each)[len(dom_each) // 2] if dom_each else None,
                    min_us=1e3 * min(dom_each) if dom_each else None, launches=dom_n, sampled_every=sample_every, hbm_gbs=ach_gbs, hbm_frac=ach_gbs / HBM_PEAK_GBS,
                    mfma_tflops=ach_tf, mfma_frac=ach_tf / MFMA_BF16_PEAK_TFLOPS)

    cpu = None
    if args.calib_copy_mb > 0:
        src = torch.empty(args.calib_copy_mb << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    if args.cpu_sample > 0:
        cpu = cpu_baseline(Xs[0].cpu(), dYs[0].cpu(), k, r, w["refresh_every"])

    out = {
        "metric": "PRAC compress+weight-grad tokens/s at LLaMA-1B shape",
        "value": N / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{w['name']}: N={N} d={d} m={m} k={k} r={r} bf16, dW bf16, "
                               f"basis refresh every {w['refresh_every']} steps ({state['fits']} in the timed region, warm-started"
                               + (f", Gram over every {w['row_stride']}th token" if w["row_stride"] > 1 else "") + "), "
                               f"{w['n_sets']} rotating input sets"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels_us": per_kernel_us,
        "other_entry_points_us": other_us,
        "fit_basis_ms": fit_ms,
    }
    print(json.dumps(out))
    ctx.close()


if __name__ == "__main__":
    main()
