#!/usr/bin/env python3
"""Benchmark: ZO steps of the MP-LoRA hot path on one MI355X, on seeded synthetic inputs.

One step = mpz_regen_noise + mpz_forward_perturbed + mpz_zo_update (all stages of Algorithm 1 for
q queries x 2 signs in one batched pass).  Prints ONE JSON line (see the fields below).

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2_opt125m] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0       # MI355X dense bf16 MFMA
PEAK_FP64_VECTOR_TFLOPS = 78.6  # fp32-storage models accumulate in fp64 on the vector ALUs
PEAK_HBM_GBPS = 8000.0          # MI355X HBM3E
# HBM bytes per GEMM launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see profiles/); None = not measured
# (the counters see what the XCD-private L2s fetch from the fabric: Infinity Cache or HBM)
GEMM_TRAFFIC = {"c2_opt125m": 102.5e6, "c3_opt1p3b": 1861.7e6, "c4_llama1p1b": 3150.5e6,
                "c5_llama7b": 1483.0e6}   # bytes per launch, profiles/hbm_traffic_gemm_<workload>.md


def gemm_flops_per_step(w, rows_per_copy=None):
    """Algorithmic FLOPs of the base-weight GEMMs (+ LM head where the loss needs the whole vocabulary).
    rows_per_copy: rows a copy occupies in the stacked pass (E*S unless the batch is packed)."""
    T = 2 * w.q * (w.E * w.S if rows_per_copy is None else rows_per_copy)
    d, f = w.d_model, w.d_ffn
    per_tok = d * (d + 2 * w.d_kv) + d * d + d * f * (2 if w.act == "swiglu" else 1) + f * d
    fl = 2.0 * T * w.n_layers * per_tok
    if w.loss_mode == "next_token_all_pos":
        fl += 2.0 * T * d * w.vocab
    elif w.loss_mode == "last_pos_full_vocab":
        fl += 2.0 * 2 * w.q * w.E * d * w.vocab
    return fl


def cpu_baseline(w, frozen, masters, tokens, labels, seed):
    """The oracle as it stands, timed on the host: as many queries (both signs each) of one step as fit into
    about 10-30 s of CPU work - the whole step where that is short enough - with the noise and the update."""
    import numpy as np
    import workloads as W
    from oracle import zo
    from oracle.precision import Precision
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    lay = W.lora_layout(w)
    prec = Precision(w.dtype)
    def timed(nq):
        m = masters.copy()
        t0 = time.perf_counter()
        losses = zo.perturbed_losses(w, lay, frozen, m, tokens, labels, seed, 0, prec, q=nq)
        g = zo.projected_grads(losses, w.eps)
        zo.zo_update(m, g, lay, seed, 0, w.lr, w.perturb_A, prec)
        return time.perf_counter() - t0
    nq, dt = 1, timed(1)
    if w.q > 1 and dt < 10.0:                       # a longer sample: the whole step if that stays under ~30 s
        nq = w.q if dt * w.q <= 30.0 else max(2, min(w.q, int(20.0 / dt)))
        dt = timed(nq)
    toks = 2 * nq * w.E * w.S
    return {"value": toks / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{nq} of {w.q} queries ({2 * nq} of {2 * w.q} copies, {toks} perturbed-copy tokens) of one step "
                      f"incl. noise and update, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2_opt125m")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mode", default="batched", choices=["batched", "inner", "outer", "sequential", "stateful"],
                    help="batched: all 2q copies in one pass (inner + outer loop parallel); inner: one query per pass, "
                         "both signs together (inner-loop parallelisation only); outer: all q queries per pass, the + "
                         "and the - copies in two passes (outer-loop parallelisation only); sequential: one pass per copy "
                         "(MeZO-style); stateful: batched pass, then update + re-perturbation in one kernel from the "
                         "stored pairs (Algorithm 2) instead of regenerate + replay")
    ap.add_argument("--q", type=int, default=None, help="override the workload's number of queries")
    ap.add_argument("--lora-targets", default=None, help="override the adapted projections, e.g. q,v or o")
    ap.add_argument("--lora-rank", type=int, default=None, help="override the LoRA rank")
    ap.add_argument("--E", type=int, default=None, help="override the sequences per copy")
    ap.add_argument("--S", type=int, default=None, help="override the sequence length")
    ap.add_argument("--device-init", action="store_true",
                    help="draw the frozen weights on the GPU (large workloads; implies --no-cpu-baseline)")
    ap.add_argument("--pad-fraction", type=float, default=None,
                    help="right-padded batch of unequal lengths (seeded; about this fraction of the E*S slots is padding): "
                         "the loss runs over real tokens only (mpz_forward_perturbed_varlen)")
    ap.add_argument("--tile-config", type=int, default=0,
                    help="measurement: force one GEMM block-tile configuration (mpz_debug_set_tile_config) instead of the "
                         "choice by shape")
    ap.add_argument("--packed", action="store_true",
                    help="with --pad-fraction: run the same batch without its padding (mpz_forward_perturbed_packed: the "
                         "sequences back to back, every kernel over real tokens only)")
    ap.add_argument("--weight-quant", default=None, choices=["none", "int8", "nf4"],
                    help="weight-only quantisation of the block linears (int8 codes + per-channel scales)")
    ap.add_argument("--one-stream", action="store_true",
                    help="issue the whole pass on one stream also for small models (per-kernel counters and traces then "
                         "see the full-batch kernels only)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 256 MiB device-to-device copies first (a kernel of known traffic, to "
                         "scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (copies would shard across GPUs with one all-gather "
                 "of q floats and every GPU replaying the same noise streams); run with --gpus 1")

    import numpy as np
    import torch
    import workloads as W
    import paper_2409_15520_amd as M

    if args.calibrate_copy:
        a = torch.empty(256 * 1024 * 1024 // 4, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    w = W.get_workload(args.workload)
    over = {k: v for k, v in (("q", args.q), ("E", args.E), ("S", args.S), ("weight_quant", args.weight_quant),
                              ("lora_rank", args.lora_rank),
                              ("lora_targets", tuple(args.lora_targets.split(",")) if args.lora_targets else None))
            if v is not None}
    if over:
        w = w.with_(**over)
    seeds = {"weights": 1234, "lora": 99, "tokens": 2345, "noise": 3456}
    if args.device_init:
        args.no_cpu_baseline = True
        frozen = M.device_random_weights(w, seeds["weights"])
    else:
        frozen = W.make_frozen_weights(w, seeds["weights"])
    masters = W.make_lora_masters(w, seeds["lora"])
    tokens, labels = W.make_tokens(w, seeds["tokens"]), W.make_labels(w, seeds["tokens"])
    m = M.ZoModel(w, frozen, masters, device="cuda:0")
    if args.one_stream:
        M.mpz_debug_set_two_halves(m.handle, False)
    if args.tile_config:
        M.mpz_debug_set_tile_config(m.handle, args.tile_config)
    tok = torch.from_numpy(tokens).cuda()
    lab = torch.from_numpy(labels).cuda()
    lengths = None
    if args.pad_fraction is not None:
        if args.mode not in ("batched", "stateful"):
            sys.exit("bench.py: --pad-fraction needs --mode batched or stateful")
        lengths_host = W.make_lengths(w, seeds["tokens"], pad_fraction=args.pad_fraction)
        lengths = torch.from_numpy(lengths_host).cuda()
    if args.packed and lengths is None:
        sys.exit("bench.py: --packed needs --pad-fraction")
    packed_batch = m.pack_batch(tok, lengths) if args.packed else None      # packed once, outside the timed steps

    def forward():
        if packed_batch is not None:
            m.forward_packed(packed_batch, lab)
        else:
            m.forward_perturbed(tok, lab, lengths)

    group = {"batched": 2 * w.q, "inner": 2, "outer": w.q, "sequential": 1, "stateful": 2 * w.q}[args.mode]
    if args.mode == "stateful":
        m.regen_noise(seeds["noise"], 0)          # the only stand-alone noise pass of the run

    def zo_step(step):
        if args.mode == "stateful":
            forward()
            m.zo_update_regen(step + 1)
            return
        m.regen_noise(seeds["noise"], step)
        if args.mode == "batched":
            forward()
        elif args.mode == "outer":
            m.forward_outer_only(tok, lab)
        else:
            m.forward_sequential(tok, lab, group=group)
        m.zo_update()

    step = 0
    for _ in range(args.warmup):
        zo_step(step)
        step += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        zo_step(step)
        step += 1
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps
    tokens_per_step = 2 * w.q * w.E * w.S

    # second pass over the same number of steps with HIP events around every kernel launch (the events add
    # overhead, so they are kept out of the wall-clock region above)
    M.mpz_profile_begin(m.handle)
    for _ in range(args.steps):
        zo_step(step)
        step += 1
    prof = M.mpz_profile_end(m.handle)
    losses = m.losses[:2 * w.q].cpu().numpy()
    assert np.all(np.isfinite(losses)), losses
    gemm = prof["gemm"]
    achieved = gemm["flops"] / (gemm["ms"] * 1e-3) / 1e12 if gemm["ms"] > 0 else 0.0
    alg = gemm_flops_per_step(w, packed_batch[0].numel() if packed_batch is not None else None)
    assert abs(gemm["flops"] / args.steps - alg) <= 1e-6 * alg, (gemm["flops"] / args.steps, alg)
    bf16 = w.dtype == "bf16"
    peak = PEAK_BF16_TFLOPS if bf16 else PEAK_FP64_VECTOR_TFLOPS
    kernels = {}
    for name, e in prof.items():
        if e["launches"] == 0:
            continue
        sec = e["ms"] * 1e-3
        k = {"ms_per_step": e["ms"] / args.steps, "launches_per_step": e["launches"] / args.steps}
        if e["flops"] > 0:
            k["tflops"] = e["flops"] / sec / 1e12
        if e["bytes"] > 0:
            k["gbps"] = e["bytes"] / sec / 1e9
            k["frac_hbm_peak"] = k["gbps"] / PEAK_HBM_GBPS
        kernels[name] = k
    # noise kernels: normals per second against the generator's own arithmetic ceiling (a kernel that makes the same
    # Philox + Box-Muller calls and moves no data), next to their GB/s against HBM
    n_groups = masters.size // 4
    n_normals = masters.size * w.q                      # per pass over the factors (perturb, and again in the update)
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    st_ptr = torch.cuda.current_stream().cuda_stream
    for _ in range(2):
        M.mpz_debug_noise_alu_probe(n_groups, w.q, sink.data_ptr(), st_ptr)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 20
    e0.record()
    for _ in range(reps):
        M.mpz_debug_noise_alu_probe(n_groups, w.q, sink.data_ptr(), st_ptr)
    e1.record()
    torch.cuda.synchronize()
    ceiling = n_normals / (e0.elapsed_time(e1) * 1e-3 / reps)
    for name in ("noise", "update"):
        if name in kernels and prof[name]["ms"] > 0:
            rate = n_normals * prof[name]["launches"] / (prof[name]["ms"] * 1e-3)
            kernels[name]["normals_per_s"] = rate
            kernels[name]["alu_ceiling_normals_per_s"] = ceiling
            kernels[name]["frac_alu_ceiling"] = rate / ceiling
    out = {
        "metric": "perturbed-copy tokens/sec", "value": tokens_per_step / (ms_per_step * 1e-3), "unit": "tokens/s",
        "zo_steps_per_sec": 1e3 / ms_per_step, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f64", "data": "synthetic",
        "config": {"workload": w.name, "mode": args.mode, "q": w.q, "copies": 2 * w.q, "E": w.E, "S": w.S,
                   "stacked_tokens": tokens_per_step, "layers": w.n_layers, "d_model": w.d_model,
                   "lora_rank": w.lora_rank, "eps": w.eps, "seeds": seeds, "weight_quant": w.weight_quant, "tile_config": args.tile_config,
                   "schedule": "one stream" if args.one_stream else "two halves on two streams where the model is small",
                   "real_tokens_per_copy": int(lengths_host.sum()) if lengths is not None else w.E * w.S,
                   "batch_layout": "packed" if args.packed else ("right-padded" if lengths is not None else "full length")},
        "roofline": {"bound": "mfma" if bf16 else "alu", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": GEMM_TRAFFIC.get(w.name),
                     "kernel": "base-weight GEMMs (all launches of a step)",
                     "launches_per_step": gemm["launches"] / args.steps, "gemm_ms_per_step": gemm["ms"] / args.steps,
                     "algorithmic_flops_per_step": alg},
        "mfma_util_pct": 100.0 * achieved / peak if bf16 else None,
        # device memory of the step: frozen parameters (shared by all copies), fp32 LoRA masters, and the one
        # workspace (perturbed factors of all copies, activations of the stacked batch, staging)
        "memory": {"frozen_bytes": m.frozen_bytes, "lora_master_bytes": int(m.masters.numel()) * 4,
                   "workspace_bytes": m.workspace_bytes},
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, frozen, masters, tokens, labels, seeds["noise"])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
