#!/usr/bin/env python3
"""Benchmark of the local-update step on one MI355X.

A step is one lp_local_step over one synthetic minibatch: forward through every layer, every
auxiliary head's loss and in-window backward pass, and every optimizer update.  Inputs are
pre-staged in HBM; the timed region holds only the K step calls between two device
synchronisations.  One JSON line goes to stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3       # MI355X fp32 vector
PEAK_HBM_GBS = 8000.0



def measured_traffic(cfg_name, kernel):
    """HBM-side traffic of one kernel instance in this workload, bytes per launch, from the committed rocprofv3
    counter summary profiles/<cfg>_step_hbm_traffic_pmc.md (FETCH_SIZE and WRITE_SIZE of two separate runs of this
    file, scaled by the same counters' readings for the plain copy kernel of --copy-calibration).  Counters cannot
    be read from inside this process; the summary holds one machine-readable line per kernel:
      traffic: kernel="<name>" fetch_bytes_per_launch=<x> write_bytes_per_launch=<y>
    Returns (bytes per launch or None, note)."""
    import re
    path = os.path.join(ROOT, "profiles", f"{cfg_name}_step_hbm_traffic_pmc.md")
    if not os.path.exists(path):
        return None, f"no counter summary for {cfg_name} under profiles/"
    pat = re.compile(r'traffic: kernel="([^"]+)" fetch_bytes_per_launch=([0-9.eE+-]+) write_bytes_per_launch=([0-9.eE+-]+)')
    for line in open(path):
        m = pat.search(line)
        if m and m.group(1) == kernel:
            return float(m.group(2)) + float(m.group(3)), f"profiles/{os.path.basename(path)}"
    return None, f"profiles/{os.path.basename(path)} has no line for {kernel}"


def gemm_flops_per_step(cfg):
    """Algorithmic FLOPs of the dense contractions of one step (2*M*N*K each): forward once per
    layer; per head, its own forward + dgrad + wgrad and the dgrad of every layer in its window; the
    wgrad of every covered layer once (appendix A.2 counts a whole backward pass per (head, layer);
    the weight-gradient half of it is shared between the heads that cover a layer)."""
    import lp_inputs as LI
    B = cfg.batch
    kind = cfg.layers[0].kind

    def layer_fwd(l):
        if kind == "decoder":
            T = B * l.seq_len
            return 2.0 * T * l.width * (3 * l.width + l.width + 2 * l.hidden)
        if kind == "resmlp":
            f = 2.0 * B * l.width * l.hidden * 2
            if l.in_dim != l.width:
                f += 2.0 * B * l.in_dim * l.width
            return f
        # resnet stage
        f = 0.0
        hw_out = l.in_hw // l.stride
        if l.has_stem:
            f += 2.0 * B * l.in_hw * l.in_hw * l.out_ch * 9 * l.in_ch
        for b in range(l.n_basic_blocks):
            first = (b == 0 and not l.has_stem)
            cin = l.in_ch if first else l.out_ch
            f += 2.0 * B * hw_out * hw_out * l.out_ch * 9 * cin
            f += 2.0 * B * hw_out * hw_out * l.out_ch * 9 * l.out_ch
            if first and (l.stride != 1 or cin != l.out_ch):
                f += 2.0 * B * hw_out * hw_out * l.out_ch * cin
        return f

    def head_fwd(h):
        l = cfg.layers[h.after_layer - 1]
        rows = B * l.seq_len if kind == "decoder" else B
        return 2.0 * rows * h.in_dim * h.n_classes

    total = sum(layer_fwd(l) for l in cfg.layers)
    covered = set()
    for h, (s, e) in zip(cfg.heads, LI.head_windows(cfg)):
        total += 3.0 * head_fwd(h)
        for li in range(s + 1, e + 1):
            total += layer_fwd(cfg.layers[li - 1])          # the input-gradient products, once per (head, layer)
            covered.add(li)
    # the weight-gradient products once per covered layer: a layer inside several windows takes ONE parameter pass,
    # driven by the sum of the heads' gradients at its output (the parameter gradient is linear in it)
    total += sum(layer_fwd(cfg.layers[li - 1]) for li in covered)
    return total


def attention_flops_per_step(cfg):
    """Causal attention: forward 2*B*H*S^2*dh (two matmuls, half masked), backward twice that."""
    import lp_inputs as LI
    if cfg.layers[0].kind != "decoder":
        return 0.0, 0.0
    B = cfg.batch
    fwd = 0.0
    bwd = 0.0
    per = [2.0 * B * l.n_heads * l.seq_len ** 2 * (l.width // l.n_heads) for l in cfg.layers]
    fwd = sum(per)
    for (s, e) in LI.head_windows(cfg):
        for li in range(s + 1, e + 1):
            bwd += 2.0 * per[li - 1]
    return fwd, bwd


def optimizer_bytes_per_step(cfg):
    """Adam 30 B/param (read p, g, m, v; write p, m, v in fp32 + the bf16 copy), SGD-momentum 22,
    SGD 12 (+2 with a bf16 copy); only parameters covered by a window are updated."""
    import numpy as np
    import lp_inputs as LI
    per = {"sgd": 12, "sgdm": 20, "adam": 28}[cfg.opt.kind] + (2 if cfg.dtype == "bf16" else 0)
    covered = set()
    for (s, e) in LI.head_windows(cfg):
        covered |= set(range(s + 1, e + 1))
    n = 0
    for name, shape in LI.param_shapes(cfg).items():
        if name.startswith("H") or int(name.split(".")[0][1:]) in covered:
            n += int(np.prod(shape))
    return n * per, n


def cpu_baseline(cfg, budget_s=30.0):
    """The CPU oracle (float32 mode, numpy/BLAS on the host cores) timed on a bounded sample of the
    same workload and scaled to whole-step samples/s."""
    import numpy as np
    import lp_inputs as LI
    import oracle
    from oracle import local as OL
    cores = os.cpu_count() or 1
    try:
        import threadpoolctl
        info = threadpoolctl.threadpool_info()
        threads = max([i.get("num_threads", 1) for i in info] or [1])
    except Exception:
        threads = cores
    P = LI.init_params(cfg)
    x, y = LI.make_batch(cfg, 0)
    kind = cfg.layers[0].kind
    if kind == "decoder":
        # the first blocks of the step, one after another (a block's input is the stored output of the layer its
        # window starts after), until about ten seconds of CPU work are spent
        import dataclasses
        wins = LI.head_windows(cfg)
        outs, done, dt, sample_flops = {0: x}, [], 0.0, 0.0
        for hi, (s, e) in enumerate(wins, start=1):
            if s not in outs or (done and dt > 10.0):
                break
            names = [k for k in P if k.startswith(f"H{hi}.") or (k[0] == "L" and s < int(k.split(".")[0][1:]) <= e)]
            st = oracle.new_state(cfg, {k: P[k] for k in names}, np.float32)
            t0 = time.perf_counter()
            loss, grads, out = oracle.block_gradients(cfg, P, hi, outs[s], y, dtype=np.float32)
            for k in grads:
                OL.optimizer_update(cfg.opt, P[k], grads[k].astype(np.float32), st, k, 1)
            dt += time.perf_counter() - t0
            outs[e] = out
            done.append(hi)
            sub = dataclasses.replace(cfg, layers=cfg.layers[s:e], heads=(dataclasses.replace(cfg.heads[hi - 1], after_layer=e - s, window=e - s),))
            sample_flops += gemm_flops_per_step(sub) + sum(attention_flops_per_step(sub))
        total_flops = gemm_flops_per_step(cfg) + sum(attention_flops_per_step(cfg))
        scale = total_flops / sample_flops
        step_s = dt * scale
        sample = (f"blocks {done[0]}..{done[-1]} of {len(cfg.heads)} (their layers + aux heads + optimizer), float32, "
                  f"{dt:.1f} s, scaled by the step's FLOP ratio x{scale:.2f}")
    else:
        st = oracle.new_state(cfg, P, np.float32)
        oracle.local_step(cfg, P, st, x, y, dtype=np.float32)     # warm-up
        reps = 0
        t0 = time.perf_counter()
        while True:
            oracle.local_step(cfg, P, st, x, y, dtype=np.float32)
            reps += 1
            if time.perf_counter() - t0 > min(budget_s, 10.0) or reps >= 3:
                break
        step_s = (time.perf_counter() - t0) / reps
        sample = f"{reps} whole step(s), float32"
    return {"value": cfg.batch / step_s, "unit": "samples/s", "cores": threads, "kind": "oracle",
            "sample": sample, "host_cpus": cores}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="cfg5",
                    help="cfg1..cfg5; the default is the largest single-GPU configuration (24 layers, 6 chunks)")
    ap.add_argument("--streams", type=int, default=-1,
                    help="side streams for the heads' chains (0 = one stream); default: 2 for the decoders, 3 for the "
                         "residual MLP, and one per stage (at most 4) for the ResNet configurations, whose four "
                         "chains are short enough to run side by side (each the fastest measured)")
    ap.add_argument("--overlap-steps", action="store_true",
                    help="lp_overlap_steps: consecutive steps are not joined into the caller's stream, so the next "
                         "step's first layers run beside the last blocks of the current one (same results, weaker "
                         "buffer contract; see include/lp.h)")
    ap.add_argument("--schedule", default="sync", choices=["sync", "pipelined", "pipelined_grouped"],
                    help="sync: every block works on the call's minibatch (the headline metric); pipelined: block j "
                         "works on block j-1's output of the previous call (steady state after warm-up)")
    ap.add_argument("--graph", action="store_true",
                    help="replay the step through a HIP graph (lp_step_graph; SGD-type optimizers only): each step "
                         "copies its batch into one pair of device buffers and launches the captured graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true", help="skip the HIP-event pass (used under rocprofv3)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run the plain copy kernel (5 x 1 GiB): the known traffic that scales rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (local parallelism is measured on a single MI355X); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import lp_inputs as LI
    import paper_2012_03837_amd as lp

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    if args.copy_calibration:
        from paper_2012_03837_amd import kernels as LK
        n = 1 << 30
        src = torch.full((n,), 7, device="cuda", dtype=torch.uint8)
        dst = torch.zeros_like(src)
        for _ in range(5):
            LK.lpk_copy(src, dst, n)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"kernel": "k_copy16", "launches": 5, "bytes_read_per_launch": n,
                                               "bytes_written_per_launch": n}}))
        return
    cfg = LI.make_config(args.config)
    if args.streams < 0:
        args.streams = lp.default_side_streams(cfg)
    tr = lp.LocalTrainer(cfg, n_streams=args.streams, schedule=args.schedule)
    K, W = args.steps, args.warmup
    if args.schedule != "sync":
        # steady state only: block j first runs in call j, so the warm-up has to cover the ramp-up of the pipeline
        W = max(W, len(cfg.heads) + 2)
    n_stage = min(K + W, 8)
    staged = [tr.stage(*LI.make_batch(cfg, i)) for i in range(n_stage)]
    torch.cuda.synchronize()

    if args.overlap_steps:
        tr.overlap_steps(True)
    if args.graph:
        tr.step_graph(True)
        xb, yb = staged[0][0].clone(), staged[0][1].clone()

    def run(n, first):
        for i in range(n):
            xd, yd = staged[(first + i) % n_stage]
            if args.graph:
                xb.copy_(xd)
                yb.copy_(yd)
                tr.step(xb, yb)
            else:
                tr.step(xd, yd)

    run(W, 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(K, W)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sec = t1 - t0
    ms_per_step = sec / K * 1e3
    value = cfg.batch * K / sec
    losses = tr.losses.cpu().numpy().tolist()

    # second pass over the same K steps with HIP events around every op, for the per-kernel figures
    phases = {}
    roofline = None
    if not args.no_profile:
        lp.lp_profile_enable(tr.ctx, True)
        for i in range(K):
            xd, yd = staged[(W + i) % n_stage]
            tr.step(xd, yd)
            lp.lp_profile_read(tr.ctx, 0)
        for kc, name in enumerate(lp.KERNEL_CLASSES):
            ms, n, fl = lp.lp_profile_read(tr.ctx, kc)
            if n:
                phases[name] = {"ms_per_step": ms / K, "ops_per_step": n / K, "flops_launched_per_step": fl / K}
        shapes = lp.lp_profile_gemm_shapes(tr.ctx)
        lp.lp_profile_enable(tr.ctx, False)
        gf = gemm_flops_per_step(cfg)
        af, ab = attention_flops_per_step(cfg)
        ob, npar = optimizer_bytes_per_step(cfg)
        key = "gemm" if "gemm" in phases and cfg.layers[0].kind != "resnet_stage" else "conv"
        # the class's ops: GEMMs run k_gemm_dma / k_mfma_tiles (+ k_splitk_reduce), convolutions the
        # same tile kernel through gather loaders; the fp32 path runs k_gemm_plain
        kernel_names = {"gemm": "k_gemm_dma+k_mfma_tiles+k_splitk_reduce" if cfg.dtype == "bf16" else "k_gemm_plain",
                        "conv": "k_mfma_tiles<Conv*>+k_gemm_plain(stem)+k_splitk_reduce"}
        if key in phases:
            p = phases[key]
            peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_F32_TFLOPS
            ach = gf / (p["ms_per_step"] * 1e-3) / 1e12
            cls = {"kernels": kernel_names[key], "achieved": ach, "frac": ach / peak, "algorithmic_flops_per_step": gf,
                   "ops_per_step": p["ops_per_step"], "ms_per_step": p["ms_per_step"]}
            kern = lp.lp_profile_gemm_kernels(tr.ctx)
            if key == "conv":
                kern = [r for r in kern if "Conv" in r["name"]]
            if kern:
                # the single time-dominant kernel instance of this run: algorithmic FLOPs of its launches over the
                # summed duration of exactly those launches (an event pair around each, on the launch stream)
                dom = max(kern, key=lambda r: r["ms"])
                d_ach = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
                traffic, note = measured_traffic(cfg.name, dom["name"])
                roofline = {"bound": "mfma", "kernel": dom["name"], "achieved": d_ach, "peak": peak, "unit": "TFLOP/s",
                            "frac": d_ach / peak, "traffic": traffic, "traffic_source": note,
                            "launches_per_step": dom["launches"] / K,
                            "avg_launch_us": dom["ms"] / dom["launches"] * 1e3,
                            "flops_per_launch": dom["flops"] / dom["launches"],
                            "share_of_gemm_time": dom["ms"] / sum(r["ms"] for r in kern),
                            ("gemm_class" if key == "gemm" else "conv_class"): cls,
                            "by_kernel": [{"kernel": r["name"], "launches_per_step": r["launches"] / K,
                                           "avg_launch_us": r["ms"] / r["launches"] * 1e3,
                                           "tflops": r["flops"] / (r["ms"] * 1e-3) / 1e12}
                                          for r in sorted(kern, key=lambda r: -r["ms"])]}
            else:
                roofline = {"bound": "mfma" if cfg.dtype == "bf16" else "alu", "kernel": kernel_names[key],
                            "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak, "traffic": None,
                            "traffic_source": "not measured for this workload",
                            "algorithmic_flops_per_step": gf, "launches_per_step": p["ops_per_step"],
                            "avg_launch_ms": p["ms_per_step"] / p["ops_per_step"]}
        if "gemm" in phases:
            phases["gemm"]["algorithmic_tflops"] = gf / 1e12
            phases["gemm"]["by_shape"] = [
                {"M": r["M"], "N": r["N"], "K": r["K"], "layout": f"{r['a_kc']}{r['b_kc']}", "per_step": r["count"] / K,
                 "avg_us": r["ms"] / r["count"] * 1e3,
                 "tflops": 2.0 * r["M"] * r["N"] * r["K"] * r["count"] / (r["ms"] * 1e-3) / 1e12}
                for r in sorted(shapes, key=lambda r: -r["ms"])[:16]]
        if "attn_fwd" in phases:
            phases["attn_fwd"]["achieved_tflops"] = af / (phases["attn_fwd"]["ms_per_step"] * 1e-3) / 1e12
        if "attn_bwd" in phases:
            phases["attn_bwd"]["achieved_tflops"] = ab / (phases["attn_bwd"]["ms_per_step"] * 1e-3) / 1e12
        if "optimizer" in phases:
            phases["optimizer"]["achieved_GBs"] = ob / (phases["optimizer"]["ms_per_step"] * 1e-3) / 1e9
            phases["optimizer"]["frac_of_hbm_peak"] = phases["optimizer"]["achieved_GBs"] / PEAK_HBM_GBS
            phases["optimizer"]["bytes_per_step"] = ob

    out = {
        "metric": "samples/sec per local-update step", "value": value, "unit": "samples/s", "n_gpus": 1,
        "steps": K, "warmup": W, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "batch": cfg.batch, "n_layers": cfg.n_layers, "n_heads_aux": len(cfg.heads),
                   "windows": LI.head_windows(cfg)[:3] + (["..."] if len(cfg.heads) > 3 else []),
                   "optimizer": cfg.opt.kind, "combine": cfg.combine, "side_streams": args.streams,
                   "schedule": args.schedule, "graph": bool(args.graph), "overlap_steps": bool(args.overlap_steps)},
        "roofline": roofline,
        "phases": phases,
        "final_losses": losses[:4],
    }
    # the paper's hardware-independent axes for this configuration (appendix A): total and sequential FLOPs
    # of one step, from the matmul / convolution / attention FLOPs counted above (backward = 2 x forward)
    try:
        import numpy as np
        sub1 = __import__("dataclasses").replace(cfg, heads=cfg.heads[:0])
        fwd_total = gemm_flops_per_step(sub1) + attention_flops_per_step(sub1)[0]
        l0 = cfg.layers[cfg.heads[0].after_layer - 1]
        rows = cfg.batch * (l0.seq_len if l0.kind == "decoder" else 1)
        aux = 2.0 * rows * cfg.heads[0].in_dim * cfg.heads[0].n_classes / cfg.batch
        npar = float(sum(int(np.prod(sh)) for sh in LI.param_shapes(cfg).values()))
        wins = LI.head_windows(cfg)
        widths = {e - s_ for (s_, e) in wins}
        if len(wins) == 1:
            method, Kc = "backprop", 1
        elif len(wins) == cfg.n_layers and widths == {1}:
            method, Kc = "greedy", 1
        elif len(wins) == cfg.n_layers:
            method, Kc = "overlap", 1
        else:
            method, Kc = "chunk", len(wins)
        cpe, cost, tm, par = lp.lp_cost_model(fwd_total / cfg.batch / cfg.n_layers, aux, 2.0, cfg.n_layers, npar, method,
                                             1.0, float(cfg.batch), Kc)
        out["cost_model"] = {"method": method, "chunks": Kc, "forward_flops_per_layer_per_example": fwd_total / cfg.batch / cfg.n_layers,
                             "aux_flops_per_example": aux, "backward_multiplier": 2.0, "parameters": npar,
                             "total_flops_per_step": cost, "sequential_flops_per_step": tm, "parallelism": par}
    except Exception as ex:      # the cost model is an annotation; it never fails the benchmark
        out["cost_model"] = {"error": str(ex)}
    if cfg.layers[0].kind == "decoder":
        out["tokens_per_s"] = value * cfg.layers[0].seq_len
        out["config"].update(seq_len=cfg.layers[0].seq_len, d_model=cfg.layers[0].width, vocab=cfg.vocab)
    tr.close()
    del tr
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
