#!/usr/bin/env python3
"""Benchmark of the DP-SGD clipped-gradient hot path on one MI355X.

A "step" is one pass of the whole path over one micro-batch of synthetic BERT-Large-shaped input that
is already resident in HBM: zero the norm buffer, pass 1 (per-example squared norms of every layer),
pass 2 (clip-weighted sums of every layer into the fp32 sum buffer), and the noise + AdamW update over
all parameters.  Prints ONE JSON line with the throughput (examples/s), the roofline of the dominant
kernel (the clip-weighted MFMA GEMM) measured with HIP events inside the timed region, and the CPU oracle
timed on a bounded sample of the same workload on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="C3", choices=["C2", "C3", "C4", "C5"],
                    help="C3 is the workload the metric is quoted on; C4 = mega-batch step (64 micro-batches of 1024 "
                         "examples accumulated, one update; the micro-batch buffers are reused), others for comparison")
    ap.add_argument("--path", default="auto", choices=["auto", "gram", "materialise"],
                    help="force the dense-layer norm path of pass 1 (comparison runs; auto is what the metric uses)")
    ap.add_argument("--share-qkv", action="store_true",
                    help="comparison run: the query, key and value layers of a block are given ONE input tensor, as in a "
                         "real attention block (the metric's workload keeps an input tensor per layer)")
    ap.add_argument("--tied-pred", type=int, default=0,
                    help="comparison run: the token table (padded to 30,528 rows) is also the output projection of this many "
                         "prediction slots per example (tied weights); the metric's workload has none")
    ap.add_argument("--full-embeddings", action="store_true",
                    help="comparison run: the embedding stage in full (token-type table with 2 rows and the LayerNorm after the "
                         "sum of the three lookups, which share one output gradient): 334,092,288 parameters")
    ap.add_argument("--batch", type=int, default=0, help="override the micro-batch size (parity/debug only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-examples", type=int, default=0, help="examples in the oracle sample (0 = auto)")
    ap.add_argument("--cpu-update-elems", type=int, default=0,
                    help="parameters in the oracle's update sample (0 = all of them: about 12 s on the GPU box's host)")
    ap.add_argument("--no-calibration", action="store_true",
                    help="skip the register-only MFMA loop and the separately timed 28 B/param update")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy before the timed region (reference for "
                         "scaling the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    return ap.parse_args()


def vendor_tn_gemm(layers):
    """Calibration only: the vendor GEMM library, through torch.matmul, on the contraction A^T G of every dense layer of
    the workload (token rows are the slow index of both operands, as for the clip-weighted GEMM)."""
    import torch

    dense = [l for l in layers if l["kind"] == "dense" and l["A"].dtype == torch.bfloat16]
    if not dense:
        return None
    ops, flops = [], 0.0
    for l in dense:
        K = l["A"].shape[0] * l["A"].shape[1]
        ops.append((l["A"].view(K, -1).t(), l["G"].view(K, -1)))
        flops += 2.0 * K * l["A"].shape[-1] * l["G"].shape[-1]
    outs = {}
    for a, g in ops:
        outs.setdefault((a.shape[0], g.shape[1]), torch.empty(a.shape[0], g.shape[1], dtype=torch.bfloat16, device=a.device))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for rep in range(3):  # the first sweep warms the library up
        if rep == 1:
            e0.record()
        for a, g in ops:
            torch.matmul(a, g, out=outs[(a.shape[0], g.shape[1])])
    e1.record()
    torch.cuda.synchronize()
    return 2 * flops / (e0.elapsed_time(e1) * 1e-3) / 1e12


def cpu_baseline(layers, cfg, n_examples, upd, n_update_elems, P):
    """Time the oracle, as it stands, on a bounded sample of the workload: norms + clip + sum of the first n_examples
    examples over the full manifest, and the noise + Adam update on the first n_update_elems flat parameters."""
    import numpy as np

    import dp_synth as syn
    from oracle import dp_oracle as orc

    try:
        from threadpoolctl import threadpool_info

        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    try:
        allowed = len(os.sched_getaffinity(0))
    except Exception:
        allowed = os.cpu_count() or 1
    host = syn.host_layer_slice(layers, range(n_examples))
    t0 = time.perf_counter()
    sums, sq, c = orc.microbatch_clip_sum(host, cfg["C"])
    dt = time.perf_counter() - t0
    # update leg: the oracle's noise + Adam step over a leading slice of the flat parameter space, in chunks
    rng = np.random.default_rng(7)
    chunk = 1 << 22
    t_upd, done = 0.0, 0
    while done < n_update_elems:
        n = min(chunk, n_update_elems - done)
        th = (rng.standard_normal(n, dtype=np.float32) * np.float32(0.02))
        S = rng.standard_normal(n, dtype=np.float32)
        t1 = time.perf_counter()
        orc.noise_adamw(th, np.zeros(n), np.zeros(n), S, elem_offset=done, sigma=upd["sigma"], C=cfg["C"],
                        seed=upd["noise_seed"], step=1, batch_size=cfg["B"], lr=upd["lr"], beta1=upd["beta1"],
                        beta2=upd["beta2"], eps=1e-11, weight_decay=upd["weight_decay"])
        t_upd += time.perf_counter() - t1
        done += n
    return dict(value=n_examples / dt, unit="examples/s", cores=int(threads), kind="oracle",
                cores_allowed=int(allowed), blas_threads=int(threads),
                update_params_per_s=n_update_elems / t_upd, update_s_per_step_extrapolated=P / (n_update_elems / t_upd),
                sample=f"first {n_examples} examples of the workload, full layer manifest, norms + clip + sum "
                       f"(numpy fp64, {dt:.1f} s); update: noise + Adam on the first {n_update_elems} of {P} parameters "
                       f"(numpy fp64, single thread, {t_upd:.1f} s)"), sq


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no collectives, no sharding here)",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import dp_synth as syn
    import paper_2108_01624_amd as pkg

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU path", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    cfg = syn.CONFIGS[args.workload]
    B = args.batch or cfg["B"]
    T = cfg["T"]
    manifest = cfg["manifest"]()
    if args.tied_pred:
        if args.workload == "C2":
            raise SystemExit("--tied-pred needs a workload with a token table (C3, C4, C5)")
        manifest = syn.bert_manifest(24, 1024, 4096, 30528, 512, tied_pred=args.tied_pred)
    if args.full_embeddings:
        if args.workload == "C2" or args.tied_pred:
            raise SystemExit("--full-embeddings needs a workload with embedding tables (C3, C4, C5) and no --tied-pred")
        manifest = syn.bert_manifest(24, 1024, 4096, 30522, 512, type_vocab=2)
    upd = syn.CONFIGS["C4"]  # update hyper-parameters of the mega-batch workload
    t_gen = time.perf_counter()
    layers = syn.device_layer_inputs(manifest, B, T, dtype=cfg["dtype"], act_std=cfg["act_std"],
                                     grad_std=cfg["grad_std"], data_seed=cfg["data_seed"], device=dev)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen
    if args.share_qkv:
        by_name = {l["name"]: l for l in layers}
        for name, l in by_name.items():
            if name.endswith(".k") or name.endswith(".v"):
                l["A"] = by_name[name[:-2] + ".q"]["A"]
        torch.cuda.empty_cache()
    seen, in_bytes = set(), 0
    for l in layers:
        for k, t in l.items():
            if k in ("A", "G", "X", "ids", "H", "dL") and t.data_ptr() not in seen:
                seen.add(t.data_ptr())
                in_bytes += t.numel() * t.element_size()

    ctx = pkg.Context()
    run = pkg.StepRunner(ctx, manifest, B, device=dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg["data_seed"] + 1)
    run.theta.copy_(torch.randn(run.P, generator=gen, device=dev) * 0.02)

    n_micro = cfg.get("micro_batches", 1) if not args.batch else 1
    path = {"auto": pkg.DP_PATH_AUTO, "gram": pkg.DP_PATH_GRAM, "materialise": pkg.DP_PATH_MATERIALISE}[args.path]

    def step(t):
        for _ in range(n_micro):
            run.pass1(layers, path)
            run.pass2(layers, cfg["C"])
        run.update(sigma=upd["sigma"], C=cfg["C"], seed=upd["noise_seed"], step=t, batch_size=B * n_micro, lr=upd["lr"],
                   beta1=upd["beta1"], beta2=upd["beta2"], weight_decay=upd["weight_decay"], zero_sum=True)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)  # 1 GiB read + 1 GiB written
        torch.cuda.synchronize()
        del src, dst
    for w in range(args.warmup):
        step(w + 1)
    ctx.sync()
    torch.cuda.synchronize()
    ctx.profile_enable(True)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        t = args.warmup + k + 1
        ev = evs[k]
        if n_micro == 1:
            ev[0].record()
            run.pass1(layers, path)
            ev[1].record()
            run.pass2(layers, cfg["C"])
            ev[2].record()
            run.update(sigma=upd["sigma"], C=cfg["C"], seed=upd["noise_seed"], step=t, batch_size=B, lr=upd["lr"],
                       beta1=upd["beta1"], beta2=upd["beta2"], weight_decay=upd["weight_decay"], zero_sum=True)
            ev[3].record()
        else:  # mega-batch: the passes alternate, so only the whole step is bracketed
            for e in ev[:3]:
                e.record()
            step(t)
            ev[3].record()
    ctx.sync()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    phase_ms = [sum(ev[j].elapsed_time(ev[j + 1]) for ev in evs) for j in range(3)]
    ms_per_step = dt * 1e3 / args.steps
    g_ms, g_n, g_flops = ctx.profile_read(pkg.DP_PROF_WGEMM)
    n_ms, n_n, n_bytes = ctx.profile_read(pkg.DP_PROF_GRAM)
    a_ms, a_n, a_bytes = ctx.profile_read(pkg.DP_PROF_ADAMW)
    # Outside the timed region: (a) the update WITHOUT the fused clearing of the sum buffer - 28 bytes per parameter
    # (16 read, 12 written), the definition the update's HBM target is stated on; the step itself uses the fused
    # form (32 bytes per parameter); (b) what a register-only loop of the GEMM's matrix instructions sustains on
    # this card, right after the workload (same thermal state).
    a28_ms = a28_n = a28_bytes = 0
    mfma_ceiling = None
    vendor_tn = None
    if not args.no_calibration:
        for k in range(5):
            run.update(sigma=upd["sigma"], C=cfg["C"], seed=upd["noise_seed"], step=args.warmup + args.steps + 1 + k,
                       batch_size=B * n_micro, lr=upd["lr"], beta1=upd["beta1"], beta2=upd["beta2"],
                       weight_decay=upd["weight_decay"], zero_sum=False)
        a28_ms, a28_n, a28_bytes = ctx.profile_read(pkg.DP_PROF_ADAMW)
        ctx.profile_enable(False)
        mfma_ceiling = ctx.profile_mfma_ceiling(8192, 8)
        vendor_tn = vendor_tn_gemm(layers)
    ctx.profile_enable(False)

    achieved = g_flops / (g_ms * 1e-3) / 1e12 if g_ms > 0 else 0.0
    # HBM bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary of this same
    # command (FETCH_SIZE and WRITE_SIZE runs, scaled as described there); null if no summary is present
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"bench_{args.workload.lower()}_hbm_traffic.json")
    if not args.batch and os.path.exists(tpath):
        try:
            k = json.load(open(tpath))["kernels"]["wgemm_dma16_kernel"]
            traffic = k["hbm_read_bytes_per_launch"] + k["hbm_write_bytes_per_launch"]
        except Exception:
            traffic = None
    out = {
        "metric": "clipped per-example grads/sec (examples/s), BERT-Large seq128; MFMA util %",
        "value": B * n_micro / (ms_per_step * 1e-3),
        "unit": "examples/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if cfg["dtype"] == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: " + (f"mega-batch of {n_micro} micro-batches accumulated, then one update; "
                                                        if n_micro > 1 else "") + "BERT-Large-shaped full parameter set "
                               f"(24 blocks, hidden 1024, FFN 4096, token emb 30522x1024 Zipf(1.1), pos emb 512x1024), "
                               f"micro-batch B={B}, seq T={T}, bf16 inputs / fp32 accumulation, C={cfg['C']}; "
                               f"one step = norms + clip-accumulate over all layers + noise/AdamW over all params"
                               if args.workload != "C2" else f"C2: BERT-Base-shaped stack, B={B}, T={T}",
                   "params": int(run.P), "micro_batch": B, "micro_batches_per_step": n_micro, "seq_len": T, "norm_path": args.path, "shared_qkv_input": bool(args.share_qkv), "tied_prediction_slots": int(args.tied_pred), "full_embedding_stage": bool(args.full_embeddings),
                   "input_bytes": int(in_bytes)},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic,
                     "traffic_unit": "HBM bytes per launch (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, profiles/)",
                     "kernel": "wgemm_dma16_kernel (clip-weighted A^T diag(c) G, up to 32 same-shaped layers per launch)",
                     "avg_launch_ms": g_ms / max(1, g_n), "launches": int(g_n),
                     "sustained_mfma_only": mfma_ceiling,
                     "sustained_mfma_only_note": "TFLOP/s of a register-only loop of the same bf16 16x16x32 matrix "
                                                 "instructions (random operands, 8 waves per CU), measured in this run "
                                                 "after the timed region: the card's power limit, not the nominal peak",
                     "frac_of_sustained": (achieved / mfma_ceiling) if mfma_ceiling else None,
                     "vendor_tn_gemm": vendor_tn,
                     "vendor_tn_gemm_note": "TFLOP/s of the vendor GEMM library (torch.matmul) on the same contractions A^T G "
                                            "of this run's dense layers - same operands and layout, bf16 result, no clip "
                                            "factors, no accumulation into an fp32 sum - timed after the timed region: a "
                                            "reference for the kernel, not part of the path"},
        "kernels": {
            "gram_sqnorms": {"bound": "hbm", "achieved_GBps": n_bytes / (n_ms * 1e-3) / 1e9 if n_ms else 0.0,
                             "frac": n_bytes / (n_ms * 1e-3) / 1e9 / PEAK_HBM_GBS if n_ms else 0.0,
                             "avg_launch_ms": n_ms / max(1, n_n), "launches": int(n_n)},
            "noise_adamw": {"bound": "hbm", "bytes_per_param": 32,
                            "what": "the update as the step runs it: also clears the sum buffer (16 B read, 16 B written per parameter)",
                            "achieved_GBps": a_bytes / (a_ms * 1e-3) / 1e9 if a_ms else 0.0,
                            "frac": a_bytes / (a_ms * 1e-3) / 1e9 / PEAK_HBM_GBS if a_ms else 0.0,
                            "avg_launch_ms": a_ms / max(1, a_n), "launches": int(a_n)},
            "noise_adamw_28B": {"bound": "hbm", "bytes_per_param": 28,
                                "what": "the same kernel without the clearing (16 B read, 12 B written per parameter), "
                                        "timed separately after the timed region",
                                "achieved_GBps": a28_bytes / (a28_ms * 1e-3) / 1e9 if a28_ms else None,
                                "frac": a28_bytes / (a28_ms * 1e-3) / 1e9 / PEAK_HBM_GBS if a28_ms else None,
                                "avg_launch_ms": a28_ms / max(1, a28_n) if a28_ms else None, "launches": int(a28_n)},
        },
        "phase_ms": ({"pass1_norms": phase_ms[0] / args.steps, "pass2_clip_accumulate": phase_ms[1] / args.steps,
                      "noise_adamw": phase_ms[2] / args.steps, "input_gen_s": t_gen} if n_micro == 1 else
                     {"whole_step": phase_ms[2] / args.steps, "input_gen_s": t_gen}),
    }
    if n_micro == 1:
        # whole-phase rates against the same peaks: pass 1 moves every input byte once, pass 2 is priced at the
        # dense layers' 2*B*T*d_in*d_out flops only, the update at 28 bytes per parameter
        p1, p2, p3 = (phase_ms[j] / args.steps * 1e-3 for j in range(3))
        dense_flops = sum(2.0 * B * T * sp.d_in * sp.d_out for sp in manifest if sp.kind == "dense")
        out["phase_rates"] = {"pass1_GBps": in_bytes / p1 / 1e9, "pass1_frac_of_hbm_peak": in_bytes / p1 / 1e9 / PEAK_HBM_GBS,
                              "pass2_TFLOPs": dense_flops / p2 / 1e12,
                              "pass2_frac_of_mfma_peak": dense_flops / p2 / 1e12 / PEAK_BF16_TFLOPS,
                              "noise_adamw_phase_GBps_at_32B_per_param": 32.0 * run.P / p3 / 1e9,
                              "noise_adamw_note": "the step's update also clears the sum buffer for the next step: 32 B "
                                                  "per parameter are moved (kernels.noise_adamw); the 28 B/param form "
                                                  "is timed separately (kernels.noise_adamw_28B)"}
    if not args.no_cpu_baseline:
        # ~155 GFLOP of fp64 work per BERT-Large example at T=128: a few dozen examples are 10-30 s of host time
        n_ex = args.cpu_examples or max(1, min(B, 32 * 128 // T))
        base, _ = cpu_baseline(layers, cfg, n_ex, upd, min(args.cpu_update_elems or int(run.P), int(run.P)), int(run.P))
        out["cpu_baseline"] = base
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
