#!/usr/bin/env python3
"""Benchmark: ZO steps of the MP-LoRA hot path on one MI355X, on seeded synthetic inputs.

One step = mpz_regen_noise + mpz_forward_perturbed + mpz_zo_update (all stages of Algorithm 1 for
q queries x 2 signs in one batched pass).  Prints ONE JSON line.  The headline is the Llama-2-7B-shaped
workload (8192 stacked perturbed-copy tokens through a 7B shape: the work of the paper's inner-loop ablation cell
"batch 16, sequence 256"); the same line carries, under `per_workload`, the same measurement for the other four
workloads, so that one run covers all five.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5_llama7b] [--no-per-workload] [--no-cpu-baseline]

The K timed steps run as blocks (5 when K allows), each bracketed by a device synchronisation; `ms_per_step` is the
median over the blocks, `ms_per_step_mean` the plain mean over all K steps.
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

PEAK_BF16_TFLOPS = 2500.0       # MI355X dense bf16 MFMA
PEAK_FP64_VECTOR_TFLOPS = 78.6  # fp32-storage models accumulate in fp64 on the vector ALUs
PEAK_HBM_GBPS = 8000.0          # MI355X HBM3E
HEADLINE = "c5_llama7b"
ALL_WORKLOADS = ("c1_tiny_fp32", "c2_opt125m", "c3_opt1p3b", "c4_llama1p1b", "c5_llama7b")
# Bytes the XCD-private L2s fetch from / write to the fabric per GEMM launch, measured with rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE on the workload's default configuration (file under profiles/ that holds the run).  Reported only when
# the run has that configuration; None otherwise.
GEMM_TRAFFIC = {"c2_opt125m": (102.4e6, "profiles/hbm_traffic_gemm_c2_opt125m.md"),
                "c3_opt1p3b": (1862.3e6, "profiles/hbm_traffic_gemm_c3_opt1p3b.md"),
                "c4_llama1p1b": (3150.0e6, "profiles/hbm_traffic_gemm_c4_llama1p1b.md"),
                "c5_llama7b": (1481.7e6, "profiles/hbm_traffic_gemm_c5_llama7b.md")}
SEEDS = {"weights": 1234, "lora": 99, "tokens": 2345, "noise": 3456}


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


def host_cores():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1]))
    except Exception:
        return int(os.cpu_count() or 1)


def cpu_baseline_full(w, frozen, masters, tokens, labels, seed):
    """The oracle as it stands, timed on the host: as many queries (both signs each) of one step as fit into
    about 10-30 s of CPU work - the whole step where that is short enough - with the noise and the update."""
    import workloads as W
    from oracle import zo
    from oracle.precision import Precision
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
    return {"value": toks / dt, "unit": "tokens/s", "cores": host_cores(), "kind": "oracle",
            "sample": f"{nq} of {w.q} queries ({2 * nq} of {2 * w.q} copies, {toks} perturbed-copy tokens) of one step "
                      f"incl. noise and update, {dt:.1f} s"}


def _host_array(t, transpose=False):
    import numpy as np
    if t is None:
        return None
    a = t.float().cpu().numpy()
    return np.ascontiguousarray(a.T) if transpose else a


def host_block_from_device(lw):
    """One block of device-drawn weights as the host arrays the oracle reads ([k_in, k_out] float32)."""
    return {k: _host_array(v, transpose=k.startswith("w_")) for k, v in lw.items() if not k.startswith("s_")}


def host_ends_from_device(frozen_dev):
    """Embeddings, final norm and head of device-drawn weights as host arrays (no blocks)."""
    out = {"emb": _host_array(frozen_dev["emb"]), "pos_emb": _host_array(frozen_dev["pos_emb"]), "layers": [],
           "lnf_g": _host_array(frozen_dev["lnf_g"]), "lnf_b": _host_array(frozen_dev["lnf_b"])}
    out["lm_head"] = out["emb"] if frozen_dev["lm_head"] is frozen_dev["emb"] else _host_array(frozen_dev["lm_head"])
    return out


def cpu_baseline_extrapolated(w, frozen_dev, masters, tokens, labels, seed, budget_s=12.0, max_blocks=8):
    """Large workloads: the oracle's stages timed one by one on the host for ONE perturbed copy at the workload's
    full width, on the device-drawn weights of the first blocks (as many as fit into about budget_s seconds of CPU
    work, at most max_blocks; copying a block's weights to the host is not part of the sample), and put together as
    q x (noise + 2 x (embedding + L x block + head and loss) + update term).  Says so in `sample`."""
    import numpy as np
    import workloads as W
    from oracle import zo
    from oracle.model import embed, decoder_layer, head_loss
    from oracle.precision import Precision
    lay = W.lora_layout(w)
    prec = Precision(w.dtype)
    frozen = host_ends_from_device(frozen_dev)
    t_start = time.perf_counter()
    z = zo.draw_z(lay, seed, 0, 0, masters.size, w.perturb_A)
    theta = zo.perturb(masters, z, +1, w.eps, prec)
    zo.perturb(masters, z, -1, w.eps, prec)
    t_noise = time.perf_counter() - t_start                  # one query: its noise and both perturbed copies
    t0 = time.perf_counter()
    zo.zo_update(masters.copy(), np.array([0.1]), lay, seed, 0, w.lr, w.perturb_A, prec)   # one query's share of the update
    t_update = time.perf_counter() - t0
    lora = zo.split_factors(lay, theta)
    t0 = time.perf_counter()
    h = embed(w, frozen, tokens, prec)
    t_embed = time.perf_counter() - t0
    layer_times = []
    spent = time.perf_counter() - t_start
    for li in range(min(w.n_layers, max_blocks)):
        if li > 0 and spent + 1.1 * layer_times[0] > budget_s:
            break                                    # another block would overrun the sample
        lw = host_block_from_device(frozen_dev["layers"][li])
        t0 = time.perf_counter()
        h = decoder_layer(w, lw, li, h, lora, prec)
        layer_times.append(time.perf_counter() - t0)
        spent += layer_times[-1]
        del lw
    t_layer = sum(layer_times) / len(layer_times)
    t0 = time.perf_counter()
    head_loss(w, frozen, h, tokens, labels, prec)
    t_head = time.perf_counter() - t0
    spent += t_head
    t_step = w.q * (t_noise + 2.0 * (t_embed + w.n_layers * t_layer + t_head) + t_update)
    toks = 2 * w.q * w.E * w.S
    return {"value": toks / t_step, "unit": "tokens/s", "cores": host_cores(), "kind": "oracle",
            "seconds_per_step_extrapolated": t_step,
            "sample": f"extrapolated: one perturbed copy ({w.E * w.S} tokens) at full width through "
                      f"{len(layer_times)} of {w.n_layers} blocks + embedding + head/loss, one query's noise and update, "
                      f"{spent:.1f} s of CPU work; step = q x (noise {t_noise:.2f} s + 2 x (embed {t_embed:.2f} s + "
                      f"{w.n_layers} x block {t_layer:.2f} s + head {t_head:.2f} s) + update {t_update:.2f} s)"}


def noise_alu_ceiling(M, torch, n_groups, q):
    """Normals per second of a kernel that makes the noise kernels' Philox + Box-Muller calls and moves no data."""
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    st_ptr = torch.cuda.current_stream().cuda_stream
    for _ in range(2):
        M.mpz_debug_noise_alu_probe(n_groups, q, sink.data_ptr(), st_ptr)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 20
    e0.record()
    for _ in range(reps):
        M.mpz_debug_noise_alu_probe(n_groups, q, sink.data_ptr(), st_ptr)
    e1.record()
    torch.cuda.synchronize()
    return 4.0 * n_groups * q / (e0.elapsed_time(e1) * 1e-3 / reps)


def run_workload(w, args, steps, warmup, device_init, want_cpu_baseline, overridden):
    """Build the model of workload w, time `steps` ZO steps, then the same number again with per-launch HIP events.
    Returns the result dict (the fields of the JSON line that belong to one workload)."""
    import numpy as np
    import torch
    import workloads as W
    import paper_2409_15520_amd as M

    if device_init:
        frozen = M.device_random_weights(w, SEEDS["weights"])
    else:
        frozen = W.make_frozen_weights(w, SEEDS["weights"])
    masters = W.make_lora_masters(w, SEEDS["lora"])
    tokens, labels = W.make_tokens(w, SEEDS["tokens"]), W.make_labels(w, SEEDS["tokens"])
    m = M.ZoModel(w, frozen, masters, device="cuda:0")
    if args.one_stream:
        M.mpz_debug_set_two_halves(m.handle, False)
    if args.tile_config:
        M.mpz_debug_set_tile_config(m.handle, args.tile_config)
    tok = torch.from_numpy(tokens).cuda()
    lab = torch.from_numpy(labels).cuda()
    lengths, lengths_host = None, None
    if args.pad_fraction is not None:
        lengths_host = W.make_lengths(w, SEEDS["tokens"], pad_fraction=args.pad_fraction)
        lengths = torch.from_numpy(lengths_host).cuda()
    packed_batch = m.pack_batch(tok, lengths) if args.packed else None      # packed once, outside the timed steps

    def forward():
        if packed_batch is not None:
            m.forward_packed(packed_batch, lab)
        else:
            m.forward_perturbed(tok, lab, lengths)

    group = {"batched": 2 * w.q, "inner": 2, "outer": w.q, "sequential": 1, "stateful": 2 * w.q}[args.mode]
    if args.mode == "stateful":
        m.regen_noise(SEEDS["noise"], 0)          # the only stand-alone noise pass of the run

    def zo_step(step):
        if args.mode == "stateful":
            forward()
            m.zo_update_regen(step + 1)
            return
        m.regen_noise(SEEDS["noise"], step)
        if args.mode == "batched":
            forward()
        elif args.mode == "outer":
            m.forward_outer_only(tok, lab)
        else:
            m.forward_sequential(tok, lab, group=group)
        m.zo_update()

    step = 0
    for _ in range(warmup):
        zo_step(step)
        step += 1
    timed_streams = M.mpz_debug_last_pass_streams(m.handle)
    # exactly `steps` timed steps, as blocks with a synchronisation on both sides of each
    n_blocks = 5 if steps >= 5 else 1
    sizes = [steps // n_blocks + (1 if i < steps % n_blocks else 0) for i in range(n_blocks)]
    block_ms = []
    torch.cuda.synchronize()
    t_all = time.perf_counter()
    for nb in sizes:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(nb):
            zo_step(step)
            step += 1
        torch.cuda.synchronize()
        block_ms.append(1e3 * (time.perf_counter() - t0) / nb)
    ms_mean = 1e3 * (time.perf_counter() - t_all) / steps
    ms_per_step = statistics.median(block_ms)
    tokens_per_step = 2 * w.q * w.E * w.S

    # second pass over the same number of steps with HIP events around every kernel launch on the stream the kernels
    # run on (the events add overhead, so they are kept out of the wall-clock region above; the pass is issued on one
    # stream, also for the small models whose timed steps overlap two halves on two streams)
    M.mpz_profile_begin(m.handle)
    for _ in range(steps):
        zo_step(step)
        step += 1
    prof = M.mpz_profile_end(m.handle)
    losses = m.losses[:2 * w.q].cpu().numpy()
    assert np.all(np.isfinite(losses)), losses
    gemm = prof["gemm"]
    achieved = gemm["flops"] / (gemm["ms"] * 1e-3) / 1e12 if gemm["ms"] > 0 else 0.0
    alg = gemm_flops_per_step(w, packed_batch[0].numel() if packed_batch is not None else None)
    assert abs(gemm["flops"] / steps - alg) <= 1e-6 * alg, (gemm["flops"] / steps, alg)
    bf16 = w.dtype == "bf16"
    peak = PEAK_BF16_TFLOPS if bf16 else PEAK_FP64_VECTOR_TFLOPS
    kernels = {}
    for name, e in prof.items():
        if e["launches"] == 0:
            continue
        sec = e["ms"] * 1e-3
        k = {"ms_per_step": e["ms"] / steps, "launches_per_step": e["launches"] / steps}
        if e["flops"] > 0:
            k["tflops"] = e["flops"] / sec / 1e12
        if e["bytes"] > 0:
            k["gbps"] = e["bytes"] / sec / 1e9
            k["frac_hbm_peak"] = k["gbps"] / PEAK_HBM_GBPS
        kernels[name] = k
    # which roofline bounds each of the small kernels, and the fraction of THAT bound.  Noise and update: q normals
    # per factor element and pass (a Philox call, two logarithms, two sine/cosine pairs and two square roots per four)
    # against 4 + 8q (perturb) or 8 (update) bytes: the generator's arithmetic, not HBM, once q >= 2; the ceiling is
    # measured live with a kernel that makes the same calls and moves no data.
    n_groups = masters.size // 4
    n_normals = masters.size * w.q
    ceiling = noise_alu_ceiling(M, torch, n_groups, w.q)
    for name in ("noise", "update"):
        if name in kernels and prof[name]["ms"] > 0:
            rate = n_normals * prof[name]["launches"] / (prof[name]["ms"] * 1e-3)
            kernels[name].update({"bound": "alu", "normals_per_s": rate, "alu_ceiling_normals_per_s": ceiling,
                                  "frac_of_bound": rate / ceiling})
    for name in ("pack", "lora_down", "norm", "embed"):
        if name in kernels and "frac_hbm_peak" in kernels[name]:
            kernels[name].update({"bound": "hbm", "frac_of_bound": kernels[name]["frac_hbm_peak"]})
    if "gemm" in kernels:
        kernels["gemm"].update({"bound": "mfma" if bf16 else "alu", "frac_of_bound": achieved / peak})
    # attention: the causal-useful FLOPs of Q K^T and P V against the same contraction peak (its two passes over the
    # keys and the exponentials are overhead of the kernel, not work of the problem); the loss kernels read their
    # logits or partial sums once
    if "attention" in kernels and "tflops" in kernels["attention"]:
        kernels["attention"].update({"bound": "mfma" if bf16 else "alu",
                                     "frac_of_bound": kernels["attention"]["tflops"] / peak})
    if "loss" in kernels and "frac_hbm_peak" in kernels["loss"]:
        kernels["loss"].update({"bound": "hbm", "frac_of_bound": kernels["loss"]["frac_hbm_peak"]})
    two_halves = timed_streams == 2
    traffic = GEMM_TRAFFIC.get(w.name) if (not overridden and args.mode == "batched" and not args.tile_config) else None
    out = {
        "value": tokens_per_step / (ms_per_step * 1e-3), "zo_steps_per_sec": 1e3 / ms_per_step,
        "ms_per_step": ms_per_step, "ms_per_step_mean": ms_mean, "ms_per_step_blocks": block_ms,
        "steps": steps, "warmup": warmup, "dtype": "bf16" if bf16 else "f64",
        "config": {"workload": w.name, "mode": args.mode, "q": w.q, "copies": 2 * w.q, "E": w.E, "S": w.S,
                   "stacked_tokens": tokens_per_step, "layers": w.n_layers, "d_model": w.d_model,
                   "lora_rank": w.lora_rank, "lora_targets": list(w.lora_targets), "eps": w.eps, "seeds": SEEDS,
                   "weights": "drawn on the device" if device_init else "drawn on the host",
                   "weight_quant": w.weight_quant, "tile_config": args.tile_config,
                   "schedule": "two halves of q copies on two streams" if two_halves else "one stream",
                   "real_tokens_per_copy": int(lengths_host.sum()) if lengths_host is not None else w.E * w.S,
                   "batch_layout": "packed" if args.packed else ("right-padded" if lengths is not None else "full length")},
        "roofline": {"bound": "mfma" if bf16 else "alu", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak,
                     "traffic": traffic[0] if traffic else None, "traffic_source": traffic[1] if traffic else None,
                     "kernel": "base-weight GEMMs (all launches of a step)",
                     "launches_per_step": gemm["launches"] / steps, "gemm_ms_per_step": gemm["ms"] / steps,
                     "avg_launch_us": 1e3 * gemm["ms"] / max(gemm["launches"], 1),
                     "algorithmic_flops_per_step": alg,
                     "measured": "HIP events around every launch on the kernels' stream, second pass of the same "
                                 "steps, one stream"},
        "mfma_util_pct": 100.0 * achieved / peak if bf16 else None,
        # device memory of the step: frozen parameters (shared by all copies), fp32 LoRA masters, and the one
        # workspace (perturbed factors of all copies, activations of the stacked batch, staging)
        "memory": {"frozen_bytes": m.frozen_bytes, "lora_master_bytes": int(m.masters.numel()) * 4,
                   "workspace_bytes": m.workspace_bytes},
        "kernels": kernels,
    }
    if want_cpu_baseline and device_init and w.weight_quant != "none":
        out["cpu_baseline"] = None                # device-drawn quantised weights are not copied back for the oracle
    elif want_cpu_baseline:
        if device_init:
            out["cpu_baseline"] = cpu_baseline_extrapolated(w, frozen, masters, tokens, labels, SEEDS["noise"])
        else:
            out["cpu_baseline"] = cpu_baseline_full(w, frozen, masters, tokens, labels, SEEDS["noise"])
    m.close()
    del m, frozen, tok, lab
    torch.cuda.empty_cache()
    return out


def probe(args):
    """--probe: stand-alone rates of the bf16 MFMA path (context for the roofline fractions; plain text lines).  The
    matrix cores alone - zero and random operand bits, with and without the main loop's LDS fragment reads - and the GEMM
    kernel on given shapes MxNxK (out[M, N] = x[M, K] w[N, K]^T), tile configurations and weight distributions;
    --probe-rotate R cycles through R operand sets so that nothing is warm in the caches."""
    import torch
    import paper_2409_15520_amd as M
    stream = torch.cuda.current_stream().cuda_stream

    def timed(fn, reps):
        for _ in range(3):
            fn(0)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(reps):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps      # ms

    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    out = torch.empty(256 * 512, dtype=torch.float32, device="cuda")
    ops = {"zeros": torch.zeros(12288, dtype=torch.bfloat16, device="cuda"),
           "random N(0,1)": torch.randn(12288, generator=g, device="cuda").to(torch.bfloat16)}
    iters = 20000
    modes = {0: "registers only", 1: "6 LDS fragment reads per 8 MFMAs"}
    for name, t in ops.items():
        for mode, what in modes.items():
            ms = timed(lambda i: M.mpz_debug_mfma_probe(t.data_ptr(), 256, iters, mode, out.data_ptr(), stream), 5)
            print(f"MFMA loop, operands {name}, {what}: {256 * 8 * iters * 8 * 32768.0 / ms / 1e9:.0f} TFLOP/s", flush=True)
    ms = timed(lambda i: M.mpz_debug_mfma_probe(ops["zeros"].data_ptr(), 256, iters, 2, out.data_ptr(), stream), 5)
    print(f"LDS fragment reads alone (ds_read_b128, 8 waves per CU): {256 * 8 * iters * 6 * 1024.0 / ms / 1e6:.0f} GB/s "
          f"= {8 * iters * 6 * 1024.0 / (ms * 1e-3) / 2.4e9:.1f} bytes per CU and cycle at 2.4 GHz", flush=True)
    # what the memory system gives a read-only kernel: the ceiling of the few-token (split-K) GEMMs, which stream every
    # weight once.  100.7 MB = the Q|K|V weight of the 7B shape, eight buffers in rotation (nothing warm in a cache) and
    # one buffer (resident in the Infinity Cache)
    rows, row_bytes = 12288, 8192
    bufs = [torch.randint(0, 2 ** 31 - 1, (rows * row_bytes // 4,), dtype=torch.int32, device="cuda", generator=g)
            for _ in range(8)]
    sums = torch.zeros(1 << 16, dtype=torch.int32, device="cuda")
    for what, rr, rb, seg, ks, lds, mode in (
            ("2048 sequential streams of 48 KB", 2048, 1, 16384, 1, 0, 0),
            ("weight tiles of 128 rows x 128 B (the 128 x 64 bf16 tile), 4 K-splits = 384 blocks", rows, 128, 128, 4, 73728, 0),
            ("the same with the activation tile fetched beside every weight tile", rows, 128, 128, 4, 73728, 1),
            ("the same with both tiles staged through LDS behind block barriers", rows, 128, 128, 4, 73728, 3)):
        rbytes = rows * row_bytes // rr
        res = []
        for nrot in (8, 1):
            ms = timed(lambda i: M.mpz_debug_hbm_read_probe(bufs[i % nrot].data_ptr(), rr, rbytes, rb, seg, ks, lds, mode,
                                                            sums.data_ptr(), stream), 20)
            res.append(f"{ms * 1e3:.1f} us = {rows * row_bytes / ms / 1e9:.2f} TB/s")
        print(f"HBM read of 100.7 MB, {what}: cold {res[0]}; resident in the Infinity Cache {res[1]}", flush=True)
    del bufs
    g.manual_seed(2)
    rot = args.probe_rotate
    for shape in args.probe_shapes.split(","):
        m, n, k = (int(v) for v in shape.split("x"))
        for wd in args.probe_weights.split(","):
            xs = [torch.randn(m, k, generator=g, device="cuda").to(torch.bfloat16) for _ in range(rot)]
            if wd == "zeros":
                ws = [torch.zeros(n, k, dtype=torch.bfloat16, device="cuda") for _ in range(rot)]
            else:
                ws = [(torch.randn(n, k, generator=g, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(rot)]
            outs = [torch.empty(m, n, dtype=torch.bfloat16, device="cuda") for _ in range(rot)]
            for cfg in (int(c) for c in args.probe_cfgs.split(",")):
                def fn(i):
                    j = i % rot
                    M.mpz_debug_gemm_bf16(m, n, k, xs[j].data_ptr(), ws[j].data_ptr(), None, -1, outs[j].data_ptr(), False,
                                          stream, cfg)
                ms = timed(fn, 30)
                print(f"GEMM {m}x{n}x{k}, tile configuration {cfg}, weights {wd}, {rot} operand set(s): "
                      f"{ms * 1e3:.1f} us, {2.0 * m * n * k / ms / 1e9:.0f} TFLOP/s", flush=True)
            del xs, ws, outs


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=HEADLINE, choices=list(ALL_WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-workload", action="store_true",
                    help="measure --workload only (by default the line also carries the other four workloads)")
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
                    help="draw the frozen weights on the GPU also for the two small workloads (the three large ones "
                         "always do: drawing and uploading host arrays would take minutes)")
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
    ap.add_argument("--probe", action="store_true", help="stand-alone MFMA and GEMM rates instead of the ZO-step benchmark "
                    "(text lines, see probe())")
    ap.add_argument("--probe-shapes", default="8192x4096x4096,8192x12288x4096,8192x4096x11008,32768x8192x2048")
    ap.add_argument("--probe-cfgs", default="0", help="tile configurations (0 = chosen by shape)")
    ap.add_argument("--probe-weights", default="normal,zeros")
    ap.add_argument("--probe-rotate", type=int, default=1)
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (copies would shard across GPUs with one all-gather "
                 "of q floats and every GPU replaying the same noise streams); run with --gpus 1")
    if args.pad_fraction is not None and args.mode not in ("batched", "stateful"):
        sys.exit("bench.py: --pad-fraction needs --mode batched or stateful")
    if args.packed and args.pad_fraction is None:
        sys.exit("bench.py: --packed needs --pad-fraction")

    import torch
    import workloads as W

    if args.probe:
        probe(args)
        return
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
    plain = not over and args.pad_fraction is None
    large = ("c3_opt1p3b", "c4_llama1p1b", "c5_llama7b")
    head = run_workload(w, args, args.steps, args.warmup, args.device_init or w.name in large,
                        not args.no_cpu_baseline, bool(over))
    out = {"metric": "perturbed-copy tokens/sec", "value": head.pop("value"), "unit": "tokens/s",
           "zo_steps_per_sec": head.pop("zo_steps_per_sec"), "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": head.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": head.pop("dtype"), "data": "synthetic"}
    head.pop("steps"); head.pop("warmup")
    out.update(head)
    if plain and args.mode == "batched" and not args.no_per_workload and not args.tile_config:
        # the other workloads, same measurement, fewer steps for the long ones so that the whole run stays short
        out["per_workload"] = []
        for name in ALL_WORKLOADS:
            if name == w.name:
                continue
            wo = W.get_workload(name)
            st = args.steps if name in ("c1_tiny_fp32", "c2_opt125m") else min(args.steps, 10)
            r = run_workload(wo, args, st, min(args.warmup, 3), args.device_init or name in large, False, False)
            r["metric"], r["unit"] = "perturbed-copy tokens/sec", "tokens/s"
            out["per_workload"].append(r)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
