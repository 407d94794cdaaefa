"""Throughput of the delayed-gradient training step on one MI355X.

`python bench.py --gpus 1 --steps K --warmup W` runs the whole hot path (forward of the K
modules, their backward, the delayed SGD/Adam updates of Eq. 8-9) on synthetic Zipfian
tokens that are already resident in HBM and prints ONE JSON line.

Headline workload: cfg4 (24 layers, d=1024, vocab 50257, 8 x 1024 tokens, K=8), the largest
of the configurations that fit one GPU.  After priming the staleness rings (K+2 untimed
iterations, so that every update applies a real stale gradient) it runs W warm-up steps and
then times `--windows` windows of exactly K steps each, every window bracketed by device
synchronisations; `value` is the median window.  A further pass of the same steps on one stream
brackets every launch of the main kernel families with HIP events: the bf16 MFMA contraction
(`roofline`), the fused attention kernels, the delayed-update kernel, LayerNorm and the
cross-entropy row pass (`kernels`).  The other configurations (cfg2, cfg3, cfg5) are run the
same way, shorter, and reported under `other_configs`.  The CPU oracle is timed on a bounded
sample of the headline workload (`cpu_baseline`).
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
KIND_CONTRACTION, KIND_UPDATE, KIND_ATTENTION, KIND_LAYERNORM, KIND_CE_ROWS = range(5)


def step_flops(c):
    """Algorithmic flops of one step: 3 x forward; a matmul of P parameters costs 2P per
    token; causal attention counts visible (query, key) pairs only, 4*d per pair (6*d with
    the relative-position term); recomputation, padding and masked work count zero."""
    d, F, L, V, T, M, B = c["d_model"], c["d_ff"], c["n_layer"], c["vocab"], c["seq_len"], c["mem_len"], c["batch"]
    if c["rel_pos"]:
        per_layer = 2 * d * d + (2 * d * d) * (T + M) / T + 2 * d * F   # q,o + k,v over memory too + FFN
        vis = M + (T + 1) / 2
        attn = 6 * d * vis
    else:
        per_layer = 4 * d * d + 2 * d * F
        attn = 4 * d * (T + 1) / 2
    fwd = 2 * (L * per_layer + V * d) + L * attn
    flops = 3.0 * B * T * fwd
    if c["rel_pos"]:
        flops -= B * T * L * 2 * (2 * d * d) * M / T    # the memory rows are constants: no input gradient for them
    return flops


def hbm_traffic_per_launch(config):
    """HBM-side bytes per contraction launch from the rocprofv3 counter summary of this workload
    under profiles/ (FETCH_SIZE and WRITE_SIZE runs of this script, scaled by the plain copy of
    `--copy-probe`); None when no summary has been committed for the configuration."""
    path = os.path.join(ROOT, "profiles", f"{config}_gemm_hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch"):
                    return float(line.split("=")[1])
    except OSError:
        pass
    return None


def describe(name, c):
    return (f"{name}: {c['n_layer']}-layer d={c['d_model']} H={c['n_head']} F={c['d_ff']} V={c['vocab']} T={c['seq_len']} "
            f"M={c['mem_len']} B={c['batch']} K={c['n_module']} {'Adam' if c['optimizer'] else 'SGD'}, Zipf({c['zipf_s']}) tokens")


def run_config(name, steps, warmup, windows, args, kernel_timing=True):
    """Primes, warms up, times `windows` windows of `steps` steps, then (optionally) the per-launch pass."""
    import torch

    import paper_1909_06695_amd as P
    import synth_inputs as S

    c = dict(S.CONFIGS[name])
    c["schedule"] = args.schedule
    c["dropout"] = args.dropout
    K = c["n_module"]
    blobs = S.init_params(c, seed=0)
    distinct = 16                                            # token batches cycle; all resident in HBM
    tok, tgt = S.token_batches(c["vocab"], c["batch"], c["seq_len"], distinct, c["zipf_s"], c["seed"],
                               contiguous=bool(c["mem_len"]))
    m = P.create_model(device="cuda:0", **c)
    for g in range(K + 1):
        m.set_params(g, blobs[g])
    dtok = torch.from_numpy(tok).cuda()
    dtgt = torch.from_numpy(tgt).cuda()
    lr = c["lr"]
    if args.serial:
        m.set_overlap(False)
    it = 0

    def run(n, want_last=False):
        nonlocal it
        loss = None
        for i in range(n):
            loss = m.step(dtok[it % distinct], dtgt[it % distinct], lr, want_loss=(want_last and i == n - 1))
            it += 1
        return loss

    prime = K + 2                                            # rings full: every update uses a real gradient
    run(prime)
    loss = run(warmup, want_last=True) if warmup > 0 else m.get_loss()
    torch.cuda.synchronize()
    win_ms = []
    for _ in range(windows):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(steps)                                           # no host sync inside the window
        torch.cuda.synchronize()
        win_ms.append((time.perf_counter() - t0) / steps * 1e3)
    loss_end = m.get_loss()
    ms = statistics.median(win_ms)
    tokens = c["batch"] * c["seq_len"]
    F = step_flops(c)
    res = {"workload": describe(name, c), "tokens_per_step": tokens, "tokens_per_s": round(tokens / (ms * 1e-3), 1),
           "ms_per_step": round(ms, 3), "ms_per_step_windows": [round(x, 3) for x in win_ms],
           "ms_per_step_min": round(min(win_ms), 3), "ms_per_step_max": round(max(win_ms), 3),
           "mfu_bf16": round(F / (ms * 1e-3) / (PEAK_BF16_TFLOPS * 1e12), 4), "step_tflop": round(F / 1e12, 3),
           "prime_steps": prime, "loss_first_timed": loss, "loss_last": loss_end, "kernels": None}
    if kernel_timing:
        # one more pass of `steps` steps with per-launch HIP events on the library's stream; one
        # stream, so that each bracket (like a profiler's kernel duration) holds that launch alone
        m.set_overlap(False)
        m.timing_enable(True)
        run(steps)
        reads = {k: m.timing_read(k) for k in range(5)}
        m.timing_enable(False)
        # A bracket holds the kernel plus the event-marker cost of the bracket itself; that cost
        # is measured here with empty brackets and subtracted, which makes the average
        # comparable with a profiler's kernel durations.
        ovh_us = m.timing_overhead(200) * 1e3
        kern = {"timed": "one more pass of the timed steps on one stream, HIP events around every launch, "
                         "empty-bracket cost subtracted", "bracket_overhead_us": round(ovh_us, 2)}

        def entry(kind, kernel, bound, unit, peak, scale):
            tms, n, work = reads[kind]
            if not n:
                return None
            raw_us = tms * 1e3 / n
            us = max(raw_us - ovh_us, 1e-3)
            ach = work / n / (us * 1e-6) / scale
            return {"bound": bound, "kernel": kernel, "achieved": round(ach, 2), "peak": peak, "unit": unit,
                    "frac": round(ach / peak, 4), "launches_per_step": n // steps, "avg_launch_us": round(us, 2),
                    "avg_bracket_us": round(raw_us, 2), "work_per_launch_avg": work / n,
                    "kernel_ms_per_step": round(us * n / steps * 1e-3, 3)}

        kern["contraction"] = entry(KIND_CONTRACTION, "bf16 MFMA contraction, all launches (2MNK flops each)",
                                    "mfma", "TFLOP/s", PEAK_BF16_TFLOPS, 1e12)
        if kern["contraction"]:
            kern["contraction"]["traffic"] = hbm_traffic_per_launch(name)
        kern["attention"] = entry(KIND_ATTENTION, "fused attention forward + backward launches (visible-pair flops; "
                                  "a backward launch counts twice its forward)", "mfma", "TFLOP/s", PEAK_BF16_TFLOPS, 1e12)
        kern["update"] = entry(KIND_UPDATE, "update_kernel (delayed SGD/Adam step, Eq. 8-9)", "hbm", "GB/s", PEAK_HBM_GBS, 1e9)
        kern["layernorm"] = entry(KIND_LAYERNORM, "LayerNorm forward and input-gradient launches", "hbm", "GB/s", PEAK_HBM_GBS, 1e9)
        kern["ce_rows"] = entry(KIND_CE_ROWS, "softmax cross-entropy row pass", "hbm", "GB/s", PEAK_HBM_GBS, 1e9)
        res["kernels"] = kern
    m.close()
    del m, dtok, dtgt
    torch.cuda.empty_cache()
    return res, c, blobs


def copy_probe(nbytes, iters):
    """A plain device copy of nbytes (read nbytes, write nbytes per dispatch): the known-size kernel
    that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters."""
    import torch
    a = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
    b = torch.empty_like(a)
    for _ in range(iters):
        b.copy_(a)
    torch.cuda.synchronize()
    print(json.dumps({"copy_probe_bytes": nbytes, "dispatches": iters}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--windows", type=int, default=5, help="timed windows of --steps steps each (median reported)")
    ap.add_argument("--config", default="cfg4", help="headline workload")
    ap.add_argument("--others", default="cfg2,cfg3,cfg5",
                    help="comma-separated configurations reported under other_configs ('' = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-batch", type=int, default=1, help="streams in the CPU oracle sample")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--serial", action="store_true",
                    help="run every kernel on one stream in the timed steps too (the mode the per-launch pass and "
                         "the committed kernel traces use; the default overlaps independent kernels on extra streams)")
    ap.add_argument("--schedule", type=int, default=0, choices=[0, 1],
                    help="0: gradient rings, Eq. 8 to the letter (the headline workload); 1: stored module inputs "
                         "and recomputation (the paper's memory-saving schedule; one more forward pass per module below K)")
    ap.add_argument("--dropout", type=float, default=0.0,
                    help="repeatable dropout rate (0 in the headline workload)")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="BYTES",
                    help="only run plain device copies of BYTES (counter scale for the profiles) and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs the K modules back to back on ONE GPU; --gpus N with N > 1 is not "
              "supported (no collectives, no sharding)", file=sys.stderr)
        sys.exit(2)
    if args.copy_probe:
        copy_probe(args.copy_probe, 5)
        return

    import synth_inputs as S

    head, c, blobs = run_config(args.config, args.steps, args.warmup, args.windows, args, not args.no_kernel_timing)
    others = {}
    for name in [x for x in args.others.split(",") if x and x != args.config]:
        r, _, _ = run_config(name, max(5, args.steps // 2), args.warmup, min(args.windows, 3), args, not args.no_kernel_timing)
        k = r.pop("kernels") or {}
        r["contraction_tflops"] = (k.get("contraction") or {}).get("achieved")
        r["contraction_frac"] = (k.get("contraction") or {}).get("frac")
        r["attention_tflops"] = (k.get("attention") or {}).get("achieved")
        r["attention_frac"] = (k.get("attention") or {}).get("frac")
        r["update_gbs"] = (k.get("update") or {}).get("achieved")
        r["update_frac"] = (k.get("update") or {}).get("frac")
        r["layernorm_gbs"] = (k.get("layernorm") or {}).get("achieved")
        r["ce_rows_gbs"] = (k.get("ce_rows") or {}).get("achieved")
        for drop in ("loss_first_timed", "loss_last", "prime_steps"):
            r.pop(drop, None)
        others[name] = r

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ouro_oracle as O
        try:
            from threadpoolctl import threadpool_info
            threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
        except Exception:
            threads = os.cpu_count()
        sb = min(c["batch"], args.cpu_batch)                 # same per-token shapes, fewer streams
        cs = dict(c, batch=sb)
        orc = O.Oracle(O.Config(**cs), blobs, keep_history=False)
        stok, stgt = S.token_batches(c["vocab"], sb, c["seq_len"], 1, c["zipf_s"], c["seed"], bool(c["mem_len"]))
        t0 = time.perf_counter()
        orc.step(stok[0], stgt[0], c["lr"])
        cdt = time.perf_counter() - t0
        cpu = {"value": round(sb * c["seq_len"] / cdt, 2), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
               "sample": f"{args.config} with {sb} of its {c['batch']} streams (same per-token shapes), one full "
                         f"iteration of the fp64 numpy oracle, {cdt:.1f} s"}

    kern = head.pop("kernels") or {}
    roof = kern.get("contraction")
    if roof:
        roof = dict(roof)
        roof["timed"] = kern["timed"]
    out = {
        "metric": "training tokens/sec on 1 MI355X", "value": head["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if c["dtype"] == 1 else "f32", "data": "synthetic",
        "config": {"workload": head["workload"], "tokens_per_step": head["tokens_per_step"], "modules": c["n_module"]},
        "windows": args.windows, "ms_per_step_windows": head["ms_per_step_windows"],
        "ms_per_step_spread": [head["ms_per_step_min"], head["ms_per_step_max"]],
        "prime_steps": head["prime_steps"],
        "mfu_bf16": head["mfu_bf16"], "step_tflop": head["step_tflop"],
        "streams": "serial" if args.serial else "overlapped",
        "schedule": "stored inputs + recompute" if args.schedule else "gradient rings (Eq. 8)",
        "dropout": args.dropout,
        "loss_first_timed": head["loss_first_timed"], "loss_last": head["loss_last"],
        "roofline": roof,
        "kernels": {k: v for k, v in kern.items() if k not in ("contraction",)} or None,
        "update_kernel": kern.get("update"),
        "other_configs": others or None,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
