#!/usr/bin/env python3
"""Benchmark of the federated-round hot path on one MI355X.

Workload: the 1.3B-shaped bf16 round (24 blocks, d = 2048, 16 heads, d_ff = 8192,
vocab 50368, sequence 2048; micro-batch 4 accumulated to 32 sequences = 65,536 tokens per
optimizer step; K = 4 clients run one after another; weighted FedAvg with Dirichlet(1)
client weights).  One "step" is one local optimizer step (8 micro-batches forward + backward
+ fused AdamW); the timed region also contains everything else a round needs: each client's
start from the broadcast model, its pseudo-gradient export, and the aggregation + server step
after the last client.  Inputs (synthetic Zipf tokens, N(0, 0.02) weights) are resident in
HBM before the clock starts.

Prints ONE JSON line: whole-job tokens/s, the roofline figures of the dominant kernel class
(bf16 MFMA GEMMs) and of the bandwidth-bound kernels (AdamW, aggregation), measured live with
HIP events around every launch, and the CPU oracle timed on the host cores on a bounded sample.
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E


def cpu_baseline(cfg, seconds_hint: float = 30.0) -> dict:
    """The float64 oracle, as it stands, on one micro-batch of a reduced-depth copy of the
    workload's model (same widths, vocabulary and sequence length)."""
    import numpy as np

    from oracle import photon_oracle as O
    from paper_2411_02908_amd import configs, synth

    small = configs.reduced_depth(cfg, 1, 1)
    ms = small.model
    sh = O.Shape(ms.n_layers, ms.d_model, ms.n_heads, ms.d_ff, ms.vocab, ms.seq_len, ms.ln_eps)
    theta = synth.init_params(synth.MASTER_SEED, ms.n_layers, ms.d_model, ms.d_ff, ms.vocab).astype(np.float64)
    max_seqs = 16
    toks = synth.client_token_batches(synth.MASTER_SEED, 0, 1, max_seqs, 1, ms.seq_len, ms.vocab, cfg.zipf_s,
                                      cfg.perm_top)[0]
    # whole sequences until about seconds_hint / 2 of CPU work has been done (at least one)
    t0 = time.perf_counter()
    n_seqs, loss = 0, 0.0
    while n_seqs < max_seqs:
        l, _ = O.loss_and_grad(theta, toks[n_seqs], sh)
        loss += l
        n_seqs += 1
        if time.perf_counter() - t0 >= seconds_hint / 2:
            break
    dt = time.perf_counter() - t0
    loss /= n_seqs
    sample_tps = n_seqs * ms.seq_len / dt
    # same FLOP/s on the full-depth model
    full_tps = sample_tps * ms.flops_per_token() / cfg.model.flops_per_token()
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    threads = int(os.environ.get("OMP_NUM_THREADS", cores))
    # beside it: the tiny fp32 round end to end, and the oracle's aggregation at the 125M vector size
    tiny = configs.TINY
    tms = tiny.model
    tsh = O.Shape(tms.n_layers, tms.d_model, tms.n_heads, tms.d_ff, tms.vocab, tms.seq_len, tms.ln_eps)
    tb = [synth.client_token_batches(synth.MASTER_SEED, k, tiny.local_steps, tiny.n_micro, tiny.micro_batch,
                                     tms.seq_len, tms.vocab, tiny.zipf_s, tiny.perm_top) for k in range(tiny.clients)]
    tt = synth.init_params(synth.MASTER_SEED, tms.n_layers, tms.d_model, tms.d_ff, tms.vocab).astype(np.float64)
    t1 = time.perf_counter()
    O.federated_round(tt, tb, configs.lr_array(tiny, tiny.local_steps),
                      O.AdamWHP(tiny.beta1, tiny.beta2, tiny.adam_eps, tiny.weight_decay), tsh,
                      [float(b.size) for b in tb], None, tiny.eta_s, tiny.mu_s, tiny.nesterov)
    tiny_s = time.perf_counter() - t1
    n_agg, k_agg = configs.M125.model.n_params, 4
    rng = np.random.default_rng(1)
    th = rng.standard_normal(n_agg).astype(np.float32)
    ds = [(rng.standard_normal(n_agg) * 1e-3).astype(np.float32).astype(np.float64) for _ in range(k_agg)]
    t2 = time.perf_counter()
    O.aggregate_deltas(th, ds, [1.0] * k_agg, np.zeros(n_agg), 1.0, 0.9, True)
    agg_s = time.perf_counter() - t2
    extra = {"tiny_round_s": tiny_s, "tiny_round_tokens_per_s": tiny.clients * tiny.local_steps * tiny.tokens_per_step / tiny_s,
             "aggregate_125M_K4_nesterov_GBps": (2 * k_agg + 16) * n_agg / agg_s / 1e9}
    return {"value": full_tps, "unit": "tokens/s", "cores": min(cores, threads), "kind": "oracle", **extra,
            "sample": (f"float64 numpy oracle, loss+gradient of {n_seqs} micro-batches of 1 x {ms.seq_len} tokens on the "
                       f"1-block copy of the model (d={ms.d_model}, vocab={ms.vocab}): {dt:.1f} s = "
                       f"{sample_tps:.1f} tokens/s, scaled by the FLOPs/token ratio "
                       f"{ms.flops_per_token() / cfg.model.flops_per_token():.4f} to the 24-block model; "
                       f"mean oracle loss {loss:.4f}")}


# Every n-th launch of the GEMM and of the attention class carries a HIP event pair in the timed region (a pair
# on each of the ~3500 launches per step costs about 2 % of the step it measures).  n is odd and not a multiple
# of 13 -- the number of GEMMs in a block's forward + backward -- so that every shape is sampled evenly, and it
# grows with the number of steps so that about 7000 launches are timed whatever the length of the run.
def event_stride(steps: int) -> int:
    n = max(4, steps // 2) | 1
    while n % 13 == 0:
        n += 2
    return n


# HBM bytes per GEMM launch (rocprofv3 FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000, the factors read off
# kernels of known size in the same counter runs; launch-count weighted over the default run's GEMMs).
# Valid for the kernel source the counters were taken on and for the default workload only.
GEMM_TRAFFIC = {"source_sha256_16": "01fba67ddf86c93b", "bytes_per_launch": 1940.7e6}


def gemm_traffic(args, cfg):
    import hashlib

    if args.layers or args.micro or args.micro_fuse >= 0 or args.config != "1.3B-bf16":
        return None
    src = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2411_02908_amd", "csrc", "gemm_mfma.hip")
    try:
        with open(src, "rb") as f:
            digest = hashlib.sha256(f.read()).hexdigest()[:16]
    except OSError:
        return None
    return GEMM_TRAFFIC["bytes_per_launch"] if digest == GEMM_TRAFFIC["source_sha256_16"] else None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64,
                    help="local optimizer steps in the timed round, all clients together (64 = the 4 x 16 of the workload)")
    ap.add_argument("--warmup", type=int, default=1, help="untimed optimizer steps before the clock starts")
    ap.add_argument("--config", default="1.3B-bf16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--micro-fuse", type=int, default=-1,
                    help="micro-batches of a step the library processes as one pass (default: the workload's setting)")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="leave the per-kernel HIP events out of the timed region (the roofline entries are then empty)")
    ap.add_argument("--layers", type=int, default=0,
                    help="counter runs only: keep this many blocks of the model (same kernel shapes, far fewer "
                         "launches); the line it prints is marked and is not the headline figure")
    ap.add_argument("--micro", type=int, default=0, help="counter runs only: micro-batches per step")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the K clients of a round run one after another on it and nothing "
              "in this path uses a second GPU; run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2411_02908_amd import binding as B
    from paper_2411_02908_amd import configs, synth

    cfg = configs.ALL[args.config]
    reduced = args.layers > 0 or args.micro > 0
    if reduced:
        import dataclasses
        cfg = dataclasses.replace(configs.reduced_depth(cfg, args.layers or cfg.model.n_layers, cfg.micro_batch),
                                  n_micro=args.micro or cfg.n_micro, name=cfg.name + " (reduced for counters)")
    ms = cfg.model
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    B.load()
    stream = torch.cuda.current_stream(dev).cuda_stream
    fuse = cfg.micro_fuse if args.micro_fuse < 0 else max(1, args.micro_fuse)
    ctx = B.photon_create(B.model_cfg(ms, cfg.dtype, cfg.recompute, fuse), cfg.micro_batch, stream)
    n = ms.n_params
    K = cfg.clients
    steps = max(args.steps, 1)
    per_client = [steps // K + (1 if k < steps % K else 0) for k in range(K)]
    active = [k for k in range(K) if per_client[k] > 0]

    # ---- inputs, resident before timing
    gen = torch.Generator(device=dev).manual_seed(synth.MASTER_SEED)
    theta = torch.randn(n, device=dev, generator=gen) * 0.02
    gains, _ = synth.ln_gain_slices(ms.n_layers, ms.d_model, ms.d_ff, ms.vocab)
    for lo, hi in gains:
        theta[lo:hi] = 1.0
    client = torch.empty_like(theta)
    m = torch.empty_like(theta)
    v = torch.empty_like(theta)
    ddt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    dcode = B.BF16 if cfg.dtype == "bf16" else B.FP32
    deltas = [torch.empty(n, dtype=ddt, device=dev) for _ in active]
    mom = torch.zeros_like(theta) if cfg.mu_s != 0.0 else None
    tokens = [torch.from_numpy(synth.client_token_batches(synth.MASTER_SEED, k, max(per_client[k], 1), cfg.n_micro,
                                                          cfg.micro_batch, ms.seq_len, ms.vocab,
                                                          cfg.client_zipf_s(synth.MASTER_SEED, k),
                                                          cfg.perm_top)).to(dev) for k in range(K)]
    if cfg.weights == "dirichlet":
        weights = list(synth.dirichlet_weights(synth.stream_key(synth.MASTER_SEED, "weights"), K))
    else:
        weights = [float(per_client[k] * cfg.tokens_per_step) or 1.0 for k in range(K)]
    hp = B.AdamWHP(cfg.beta1, cfg.beta2, cfg.adam_eps, cfg.weight_decay)
    lrs_all = configs.lr_array(cfg, max(per_client))

    # ---- warm-up (untimed): local steps on a scratch client, one export, one aggregation
    st = B.OptState(m.data_ptr(), v.data_ptr(), 0)
    B.photon_client_init(ctx, theta, client, st)
    if args.warmup > 0:
        wtok = tokens[0][:1].expand(args.warmup, -1, -1, -1).contiguous()
        B.photon_client_local_steps(ctx, client, st, wtok, args.warmup, cfg.n_micro, [cfg.lr] * args.warmup, hp)
        B.photon_export_delta(ctx, theta, client, deltas[0], dcode)
        scratch = theta.clone()
        smom = None if mom is None else torch.zeros_like(theta)
        B.photon_aggregate(ctx, scratch, [deltas[0]], B.CLIENT_DELTAS, dcode, [1.0],
                           B.OuterOpt(cfg.eta_s, cfg.mu_s, int(cfg.nesterov), B._ptr(smom), 0))
        del scratch, smom
    torch.cuda.synchronize(dev)
    print("bench: inputs resident, warm-up done", file=sys.stderr, flush=True)

    # ---- timed round
    if not args.no_kernel_events:
        B.photon_profile_begin_sampled(ctx, event_stride(steps))
    losses = []
    torch.cuda.synchronize(dev)
    t0 = time.perf_counter()
    for i, k in enumerate(active):
        print(f"bench: client {k}: {per_client[k]} local steps", file=sys.stderr, flush=True)
        st = B.OptState(m.data_ptr(), v.data_ptr(), 0)
        B.photon_client_init(ctx, theta, client, st)
        losses.append(B.photon_client_local_steps(ctx, client, st, tokens[k], per_client[k], cfg.n_micro,
                                                  lrs_all[:per_client[k]], hp))
        B.photon_export_delta(ctx, theta, client, deltas[i], dcode)
    oo = B.OuterOpt(cfg.eta_s, cfg.mu_s, int(cfg.nesterov), B._ptr(mom), 0)
    metrics = B.photon_aggregate(ctx, theta, deltas, B.CLIENT_DELTAS, dcode, [weights[k] for k in active], oo)
    torch.cuda.synchronize(dev)
    elapsed = time.perf_counter() - t0
    prof = B.photon_profile_end(ctx)

    tokens_done = steps * cfg.tokens_per_step
    tps = tokens_done / elapsed
    gemm_tflops = prof["gemm_flops"] / (prof["gemm_ms"] * 1e-3) / 1e12 if prof["gemm_ms"] > 0 else 0.0
    attn_tflops = prof["attn_flops"] / (prof["attn_ms"] * 1e-3) / 1e12 if prof["attn_ms"] > 0 else 0.0
    adamw_gbps = prof["adamw_bytes"] / (prof["adamw_ms"] * 1e-3) / 1e9 if prof["adamw_ms"] > 0 else 0.0
    agg_gbps = prof["agg_bytes"] / (prof["agg_ms"] * 1e-3) / 1e9 if prof["agg_ms"] > 0 else 0.0
    delta_gbps = prof["delta_bytes"] / (prof["delta_ms"] * 1e-3) / 1e9 if prof["delta_ms"] > 0 else 0.0
    # class totals: the timed launches' time scaled to all launches of the class
    gemm_total_ms = prof["gemm_ms"] * prof["gemm_launches_total"] / max(1, prof["gemm_launches"])
    attn_total_ms = prof["attn_ms"] * prof["attn_launches_total"] / max(1, prof["attn_launches"])
    other_ms = elapsed * 1e3 - gemm_total_ms - attn_total_ms - prof["adamw_ms"] - prof["agg_ms"] - prof["delta_ms"]

    out = {
        "metric": "local_train_tokens_per_s",
        "value": tps,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed * 1e3 / steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {ms.n_layers} blocks d={ms.d_model} heads={ms.n_heads} d_ff={ms.d_ff} "
                               f"vocab={ms.vocab} seq={ms.seq_len}; micro-batch {cfg.micro_batch} x {cfg.n_micro} "
                               f"accumulation = {cfg.tokens_per_step} tokens/step ({fuse} micro-batches per pass); K={len(active)} clients x "
                               f"{per_client} local AdamW steps, bf16 pseudo-gradients, weighted FedAvg "
                               f"(eta_s={cfg.eta_s}, mu_s={cfg.mu_s})",
                   "params": n, "tokens_per_step": cfg.tokens_per_step, "clients": len(active),
                   "seed": synth.MASTER_SEED},
        "roofline": {"bound": "mfma", "achieved": gemm_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": gemm_tflops / PEAK_BF16_TFLOPS, "traffic": gemm_traffic(args, cfg),
                     "kernel": "gemm_mfma_kernel (all operand/epilogue variants)",
                     "launches": prof["gemm_launches_total"], "launches_timed": prof["gemm_launches"],
                     "avg_launch_ms": prof["gemm_ms"] / max(1, prof["gemm_launches"]),
                     "flops_per_launch": prof["gemm_flops"] / max(1, prof["gemm_launches"])},
        "cpu_baseline": None,
        "model_flops_utilisation": {
            "causal": tps * ms.flops_per_token(True) / (PEAK_BF16_TFLOPS * 1e12),
            "full_attention_convention": tps * ms.flops_per_token(False) / (PEAK_BF16_TFLOPS * 1e12),
            "peak_TFLOPs": PEAK_BF16_TFLOPS},
        "aggregate": {"GBps": agg_gbps, "frac_of_hbm_peak": agg_gbps / PEAK_HBM_GBPS, "ms": prof["agg_ms"],
                      "bytes": prof["agg_bytes"], "peak_GBps": PEAK_HBM_GBPS,
                      "delta_norm2": metrics["delta_norm2"]},
        "adamw": {"GBps": adamw_gbps, "frac_of_hbm_peak": adamw_gbps / PEAK_HBM_GBPS,
                  "ms_per_launch": prof["adamw_ms"] / max(1, prof["adamw_launches"])},
        "delta_export": {"GBps": delta_gbps, "frac_of_hbm_peak": delta_gbps / PEAK_HBM_GBPS},
        "attention": {"TFLOPs_causal": attn_tflops, "frac_of_mfma_peak": attn_tflops / PEAK_BF16_TFLOPS},
        "time_split_ms": {"gemm": gemm_total_ms, "attention": attn_total_ms, "adamw": prof["adamw_ms"],
                          "aggregate": prof["agg_ms"], "delta_export": prof["delta_ms"], "other": other_ms},
        "first_last_loss": [losses[0][0], losses[-1][-1]],
        "workspace_GB": ctx.workspace_bytes / 1e9,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
