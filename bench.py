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
GEMM_TRAFFIC = {"source_sha256_16": "b1764a41bb1e88cf", "bytes_per_launch": 1926.0e6}


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


def measure(cfg, steps: int, warmup: int, fuse: int, kernel_events: bool, log, trained_clients: int | None = None):
    """One timed round of `cfg` on cuda:0: `steps` local optimizer steps spread over the clients
    that are trained (all K, or the first `trained_clients` of them), each followed by its
    pseudo-gradient export, then the aggregation over K buffers.  With trained_clients given the
    round is run in two phases so that the largest configurations fit: the training buffers and
    the model workspace are released before the K pseudo-gradient buffers of the aggregation are
    completed (those of clients that were not trained are copies of the first one: the kernel's
    time does not depend on the values), and only the training phase counts towards tokens/s."""
    import numpy as np
    import torch

    from paper_2411_02908_amd import binding as B
    from paper_2411_02908_amd import configs, synth

    ms = cfg.model
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream(dev).cuda_stream
    ctx = B.photon_create(B.model_cfg(ms, cfg.dtype, cfg.recompute, fuse), cfg.micro_batch, stream)
    n = ms.n_params
    K = cfg.clients
    two_phase = trained_clients is not None
    kt = K if not two_phase else max(1, min(K, trained_clients))
    per_client = [steps // kt + (1 if k < steps % kt else 0) if k < kt else 0 for k in range(K)]
    active = [k for k in range(K) if per_client[k] > 0]

    # ---- inputs, resident before timing
    gen = torch.Generator(device=dev).manual_seed(synth.MASTER_SEED)
    theta = torch.empty(n, device=dev)
    for lo in range(0, n, 1 << 30):           # in slices: no second full-size temporary
        hi = min(n, lo + (1 << 30))
        theta[lo:hi] = torch.randn(hi - lo, device=dev, generator=gen) * 0.02
    gains, _ = synth.ln_gain_slices(ms.n_layers, ms.d_model, ms.d_ff, ms.vocab)
    for lo, hi in gains:
        theta[lo:hi] = 1.0
    client = torch.empty_like(theta)
    m = torch.empty_like(theta)
    v = torch.empty_like(theta)
    ddt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    dcode = B.BF16 if cfg.dtype == "bf16" else B.FP32
    deltas = [torch.empty(n, dtype=ddt, device=dev) for _ in active]
    mom = torch.zeros_like(theta) if (cfg.mu_s != 0.0 and not two_phase) else None
    tokens = {k: torch.from_numpy(synth.client_token_batches(synth.MASTER_SEED, k, per_client[k], cfg.n_micro,
                                                             cfg.micro_batch, ms.seq_len, ms.vocab,
                                                             cfg.client_zipf_s(synth.MASTER_SEED, k),
                                                             cfg.perm_top)).to(dev) for k in active}
    if cfg.weights == "dirichlet":
        weights = list(synth.dirichlet_weights(synth.stream_key(synth.MASTER_SEED, "weights"), K))
    else:
        weights = [1.0] * K
    hp = B.AdamWHP(cfg.beta1, cfg.beta2, cfg.adam_eps, cfg.weight_decay)
    lrs_all = configs.lr_array(cfg, max(per_client))

    # ---- warm-up (untimed): local steps on a scratch client, one export, one aggregation
    st = B.OptState(m.data_ptr(), v.data_ptr(), 0)
    B.photon_client_init(ctx, theta, client, st)
    if warmup > 0:
        wtok = tokens[active[0]][:1].expand(warmup, -1, -1, -1).contiguous()
        B.photon_client_local_steps(ctx, client, st, wtok, warmup, cfg.n_micro, [cfg.lr] * warmup, hp)
        B.photon_export_delta(ctx, theta, client, deltas[0], dcode)
        if not two_phase:
            scratch = theta.clone()
            smom = None if mom is None else torch.zeros_like(theta)
            B.photon_aggregate(ctx, scratch, [deltas[0]], B.CLIENT_DELTAS, dcode, [1.0],
                               B.OuterOpt(cfg.eta_s, cfg.mu_s, int(cfg.nesterov), B._ptr(smom), 0))
            del scratch, smom
    torch.cuda.synchronize(dev)
    log(f"bench: {cfg.name}: inputs resident, warm-up done")

    # ---- timed round
    if kernel_events:
        B.photon_profile_begin_sampled(ctx, event_stride(steps))
    losses = []
    torch.cuda.synchronize(dev)
    t0 = time.perf_counter()
    for i, k in enumerate(active):
        log(f"bench: {cfg.name}: client {k}: {per_client[k]} local steps")
        st = B.OptState(m.data_ptr(), v.data_ptr(), 0)
        B.photon_client_init(ctx, theta, client, st)
        losses.append(B.photon_client_local_steps(ctx, client, st, tokens[k], per_client[k], cfg.n_micro,
                                                  lrs_all[:per_client[k]], hp))
        B.photon_export_delta(ctx, theta, client, deltas[i], dcode)
    metrics = None
    if not two_phase:
        oo = B.OuterOpt(cfg.eta_s, cfg.mu_s, int(cfg.nesterov), B._ptr(mom), 0)
        metrics = B.photon_aggregate(ctx, theta, deltas, B.CLIENT_DELTAS, dcode, [weights[k] for k in active], oo)
    torch.cuda.synchronize(dev)
    elapsed = time.perf_counter() - t0
    prof = B.photon_profile_end(ctx) if kernel_events else None
    workspace = ctx.workspace_bytes
    agg_clients = len(active)
    if two_phase:
        # second phase: the aggregation at the configuration's K, after the training buffers are gone
        ctx.close()
        del client, m, v, tokens
        torch.cuda.empty_cache()
        while len(deltas) < K:
            d = torch.empty(n, dtype=ddt, device=dev)
            d.copy_(deltas[0])
            deltas.append(d)
        mom = torch.zeros_like(theta) if cfg.mu_s != 0.0 else None
        fctx = B.photon_create_flat(n, stream)
        oo = B.OuterOpt(cfg.eta_s, cfg.mu_s, int(cfg.nesterov), B._ptr(mom), 0)
        B.photon_aggregate(fctx, theta, deltas, B.CLIENT_DELTAS, dcode, weights, oo)      # warm-up, and a first
        torch.cuda.synchronize(dev)                                                       # round of momentum
        B.photon_profile_begin(fctx)
        metrics = B.photon_aggregate(fctx, theta, deltas, B.CLIENT_DELTAS, dcode, weights, oo)
        aprof = B.photon_profile_end(fctx)
        fctx.close()
        agg_clients = K
        if prof is not None:
            prof["agg_ms"], prof["agg_bytes"] = aprof["agg_ms"], aprof["agg_bytes"]
    else:
        ctx.close()
    del theta, deltas, mom
    torch.cuda.empty_cache()
    return {"cfg": cfg, "elapsed": elapsed, "steps": steps, "per_client": per_client, "active": active, "prof": prof,
            "losses": losses, "metrics": metrics, "workspace": workspace, "fuse": fuse, "agg_clients": agg_clients,
            "two_phase": two_phase}


def rates(r) -> dict:
    """Throughput and per-class rates of one measured round."""
    cfg, prof, elapsed, steps = r["cfg"], r["prof"], r["elapsed"], r["steps"]
    ms = cfg.model
    tps = steps * cfg.tokens_per_step / elapsed
    out = {"tokens_per_s": tps, "ms_per_step": elapsed * 1e3 / steps,
           "mfu_causal": tps * ms.flops_per_token(True) / (PEAK_BF16_TFLOPS * 1e12)}
    if prof is None:
        return out

    def rate(work, ms_):
        return prof[work] / (prof[ms_] * 1e-3) if prof[ms_] > 0 else 0.0
    out.update({
        "gemm_TFLOPs": rate("gemm_flops", "gemm_ms") / 1e12, "attn_TFLOPs_causal": rate("attn_flops", "attn_ms") / 1e12,
        "adamw_GBps": rate("adamw_bytes", "adamw_ms") / 1e9, "agg_GBps": rate("agg_bytes", "agg_ms") / 1e9,
        "delta_GBps": rate("delta_bytes", "delta_ms") / 1e9,
        # class totals: the timed launches' time scaled to all launches of the class
        "gemm_total_ms": prof["gemm_ms"] * prof["gemm_launches_total"] / max(1, prof["gemm_launches"]),
        "attn_total_ms": prof["attn_ms"] * prof["attn_launches_total"] / max(1, prof["attn_launches"])})
    return out


def hbm_ceiling(n: int) -> dict:
    """What plain streaming kernels reach on this GPU for vectors of n float32, per read : write
    mix, and the library's own bandwidth-bound kernels at the same length beside them."""
    import torch

    from paper_2411_02908_amd import binding as B

    dev = torch.device("cuda:0")
    B.load()
    ctx = B.photon_create_flat(n, torch.cuda.current_stream(dev).cuda_stream)
    src = torch.randn(4 * n, device=dev)
    dst = torch.empty(4 * n, device=dev)
    rows = []
    for r, w in ((1, 0), (2, 0), (4, 0), (0, 1), (0, 3), (1, 1), (2, 1), (3, 1), (4, 1), (1, 3), (4, 3), (4, 4)):
        ms = B.photon_stream_probe(ctx, r, w, src, dst, n, 10)
        rows.append({"kernel": f"plain stream {r} read : {w} write", "GBps": 4.0 * n * (r + w) / ms / 1e6,
                     "frac_of_hbm_peak": 4.0 * n * (r + w) / ms / 1e6 / PEAK_HBM_GBPS})
    # the library's kernels on the same vectors (event-timed by the library)
    p, m, v, g = (src[i * n:(i + 1) * n] for i in range(4))
    w16 = dst[:n // 2 + 8].view(torch.bfloat16)[:n]
    hp = B.AdamWHP(0.9, 0.95, 1e-8, 0.1)
    st = B.OptState(m.data_ptr(), v.data_ptr(), 0)
    v.abs_()
    deltas = [dst[(k * n) // 2 + 16 * k:][:n // 2 + 8].view(torch.bfloat16)[:n] for k in range(8)]
    for d in deltas:
        d.normal_(0, 1e-3)
    B.photon_profile_begin(ctx)
    for _ in range(5):
        B.photon_adamw_step(ctx, p, st, g, 1e-4, hp, None)
    prof = B.photon_profile_end(ctx)
    rows.append({"kernel": "AdamW (4 read : 3 write, no bf16 copy)", "GBps": prof["adamw_bytes"] / prof["adamw_ms"] / 1e6})
    mom = src[3 * n:4 * n]
    for K, mu in ((4, 0.0), (8, 0.0), (4, 0.9), (8, 0.9)):
        B.photon_profile_begin(ctx)
        for _ in range(5):
            B.photon_aggregate(ctx, p, deltas[:K], B.CLIENT_DELTAS, B.BF16, [1.0] * K,
                               B.OuterOpt(1.0, mu, int(mu != 0), B._ptr(mom) if mu else 0, 0), want_metrics=False)
        prof = B.photon_profile_end(ctx)
        rows.append({"kernel": f"aggregate K={K} bf16 pseudo-gradients, momentum {'on' if mu else 'off'}",
                     "GBps": prof["agg_bytes"] / prof["agg_ms"] / 1e6})
    B.photon_profile_begin(ctx)
    for _ in range(5):
        B.photon_export_delta(ctx, p, m, deltas[0], B.BF16)
    prof = B.photon_profile_end(ctx)
    rows.append({"kernel": "pseudo-gradient export (2 read : 0.5 write)", "GBps": prof["delta_bytes"] / prof["delta_ms"] / 1e6})
    for row in rows:
        row["frac_of_hbm_peak"] = row["GBps"] / PEAK_HBM_GBPS
    ctx.close()
    return {"hbm_streaming_ceiling": rows, "n": n, "peak_GBps": PEAK_HBM_GBPS}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64,
                    help="local optimizer steps in the timed round, all clients together (64 = the 4 x 16 of the workload)")
    ap.add_argument("--warmup", type=int, default=1, help="untimed optimizer steps before the clock starts")
    ap.add_argument("--config", default="1.3B-bf16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="leave out the short runs of the other model sizes (125M, 3B, 7B) reported beside the headline")
    ap.add_argument("--micro-fuse", type=int, default=-1,
                    help="micro-batches of a step the library processes as one pass (default: the workload's setting)")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="leave the per-kernel HIP events out of the timed region (the roofline entries are then empty)")
    ap.add_argument("--layers", type=int, default=0,
                    help="counter runs only: keep this many blocks of the model (same kernel shapes, far fewer "
                         "launches); the line it prints is marked and is not the headline figure")
    ap.add_argument("--micro", type=int, default=0, help="counter runs only: micro-batches per step")
    ap.add_argument("--trained-clients", type=int, default=0,
                    help="train only this many of the K clients and run the aggregation as a second phase "
                         "(what the 7B configuration needs to fit; default: all K in one phase)")
    ap.add_argument("--hbm-ceiling", action="store_true",
                    help="instead of the round: streaming bandwidth of plain kernels per read : write mix and of the "
                         "library's bandwidth-bound kernels, on vectors of the 1.3B model's length")
    args = ap.parse_args()
    if args.hbm_ceiling and args.gpus == 1:
        from paper_2411_02908_amd import configs
        print(json.dumps(hbm_ceiling(configs.B1_3.model.n_params)))
        return 0
    if args.gpus != 1:
        print("bench.py measures one GPU: the K clients of a round run one after another on it and nothing "
              "in this path uses a second GPU; run with --gpus 1", file=sys.stderr)
        return 2

    import torch

    from paper_2411_02908_amd import binding as B
    from paper_2411_02908_amd import configs, synth

    def log(msg):
        print(msg, file=sys.stderr, flush=True)

    cfg = configs.ALL[args.config]
    reduced = args.layers > 0 or args.micro > 0
    if reduced:
        import dataclasses
        cfg = dataclasses.replace(configs.reduced_depth(cfg, args.layers or cfg.model.n_layers, cfg.micro_batch),
                                  n_micro=args.micro or cfg.n_micro, name=cfg.name + " (reduced for counters)")
    ms = cfg.model
    torch.cuda.set_device(torch.device("cuda:0"))
    B.load()
    fuse = cfg.micro_fuse if args.micro_fuse < 0 else max(1, args.micro_fuse)
    steps = max(args.steps, 1)
    trained = args.trained_clients if args.trained_clients > 0 else (2 if cfg.name.startswith("7B") else None)
    r = measure(cfg, steps, args.warmup, fuse, not args.no_kernel_events, log, trained)
    q = rates(r)
    prof = r["prof"] or {k: 0 for k in ("gemm_ms", "gemm_flops", "gemm_launches", "gemm_launches_total", "adamw_ms",
                                        "adamw_launches", "agg_ms", "agg_bytes", "delta_ms")}
    elapsed, per_client, active = r["elapsed"], r["per_client"], r["active"]
    tps = q["tokens_per_s"]
    gemm_tflops = q.get("gemm_TFLOPs", 0.0)
    other_ms = elapsed * 1e3 - q.get("gemm_total_ms", 0.0) - q.get("attn_total_ms", 0.0) - prof["adamw_ms"] - \
        (0.0 if r["two_phase"] else prof["agg_ms"]) - prof["delta_ms"]

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
                               f"{[p for p in per_client if p]} local AdamW steps, bf16 pseudo-gradients, weighted FedAvg "
                               f"over {r['agg_clients']} buffers (eta_s={cfg.eta_s}, mu_s={cfg.mu_s})"
                               + ("; aggregation timed as a second phase, outside the tokens/s region" if r["two_phase"] else ""),
                   "params": ms.n_params, "tokens_per_step": cfg.tokens_per_step, "clients": len(active),
                   "seed": synth.MASTER_SEED},
        "roofline": {"bound": "mfma", "achieved": gemm_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": gemm_tflops / PEAK_BF16_TFLOPS, "traffic": gemm_traffic(args, cfg),
                     "traffic_source": "stored figure from rocprofv3 counter runs on this kernel source (profiles/), "
                                       "not measured in this run; null when the source has changed since",
                     "kernel": "gemm_mfma_kernel (all operand/epilogue variants)",
                     "launches": prof["gemm_launches_total"], "launches_timed": prof["gemm_launches"],
                     "avg_launch_ms": prof["gemm_ms"] / max(1, prof["gemm_launches"]),
                     "flops_per_launch": prof["gemm_flops"] / max(1, prof["gemm_launches"])},
        "cpu_baseline": None,
        "model_flops_utilisation": {
            "causal": q["mfu_causal"],
            "full_attention_convention_context_only": tps * ms.flops_per_token(False) / (PEAK_BF16_TFLOPS * 1e12),
            "peak_TFLOPs": PEAK_BF16_TFLOPS},
        "aggregate": {"GBps": q.get("agg_GBps", 0.0), "frac_of_hbm_peak": q.get("agg_GBps", 0.0) / PEAK_HBM_GBPS,
                      "ms": prof["agg_ms"], "bytes": prof["agg_bytes"], "peak_GBps": PEAK_HBM_GBPS,
                      "clients": r["agg_clients"], "delta_norm2": r["metrics"]["delta_norm2"]},
        "adamw": {"GBps": q.get("adamw_GBps", 0.0), "frac_of_hbm_peak": q.get("adamw_GBps", 0.0) / PEAK_HBM_GBPS,
                  "ms_per_launch": prof["adamw_ms"] / max(1, prof["adamw_launches"])},
        "delta_export": {"GBps": q.get("delta_GBps", 0.0), "frac_of_hbm_peak": q.get("delta_GBps", 0.0) / PEAK_HBM_GBPS},
        "attention": {"TFLOPs_causal": q.get("attn_TFLOPs_causal", 0.0),
                      "frac_of_mfma_peak": q.get("attn_TFLOPs_causal", 0.0) / PEAK_BF16_TFLOPS},
        "time_split_ms": {"gemm": q.get("gemm_total_ms", 0.0), "attention": q.get("attn_total_ms", 0.0),
                          "adamw": prof["adamw_ms"], "aggregate": prof["agg_ms"], "delta_export": prof["delta_ms"],
                          "other": other_ms},
        "first_last_loss": [r["losses"][0][0], r["losses"][-1][-1]],
        "workspace_GB": r["workspace"] / 1e9,
    }
    # ---- the other model sizes of the paper's shape table, a few steps each, beside the headline
    if not args.no_other_configs and not reduced and args.config == "1.3B-bf16":
        others = {}
        for name, osteps in (("125M-bf16", 8), ("3B-bf16", 4), ("7B-bf16", 4)):
            oc = configs.ALL[name]
            ro = measure(oc, osteps, 1, oc.micro_fuse, not args.no_kernel_events, log, 2)
            qo = rates(ro)
            others[name] = {
                "tokens_per_s": qo["tokens_per_s"], "ms_per_step": qo["ms_per_step"],
                "tokens_per_step": oc.tokens_per_step, "steps": osteps, "recompute": oc.recompute,
                "model_flops_utilisation_causal": qo["mfu_causal"],
                "gemm_TFLOPs": qo.get("gemm_TFLOPs"), "attention_TFLOPs_causal": qo.get("attn_TFLOPs_causal"),
                "adamw_GBps": qo.get("adamw_GBps"), "delta_export_GBps": qo.get("delta_GBps"),
                "aggregate_GBps": qo.get("agg_GBps"), "aggregate_clients": ro["agg_clients"],
                "aggregate_momentum": oc.mu_s != 0.0, "params": oc.model.n_params,
                "workspace_GB": ro["workspace"] / 1e9,
                "note": "2 of the K clients trained (1 untimed warm-up step, then the timed steps and exports); "
                        "aggregation over K buffers timed as a second phase"}
        out["other_configs"] = others
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
