"""Workload configurations: model shapes from Table 4 of the paper plus the
round structure (clients K, local steps, micro-batching, server optimizer)
each measured workload uses.  Plain data; no arithmetic of the method."""

from __future__ import annotations

from dataclasses import dataclass, field, replace


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    d_ff: int
    vocab: int
    seq_len: int
    ln_eps: float = 1e-5

    @property
    def head_dim(self) -> int:
        return self.d_model // self.n_heads

    @property
    def n_params(self) -> int:
        d, f = self.d_model, self.d_ff
        return self.vocab * d + self.n_layers * (2 * d + 4 * d * d + 2 * d * f) + d

    @property
    def matmul_params(self) -> int:
        d, f = self.d_model, self.d_ff
        return self.vocab * d + self.n_layers * (4 * d * d + 2 * d * f)

    def flops_per_token(self, causal: bool = True) -> float:
        """Model FLOPs per trained token: 6 per matmul parameter plus the attention
        score/value products (halved when only the causal triangle is counted)."""
        attn = 12 * self.n_layers * self.seq_len * self.d_model
        return 6.0 * self.matmul_params + (attn / 2 if causal else attn)


@dataclass(frozen=True)
class RoundConfig:
    name: str
    model: ModelShape
    dtype: str               # "fp32" or "bf16"
    micro_batch: int
    n_micro: int             # micro-batches accumulated per optimizer step
    clients: int             # K
    local_steps: int         # tau
    lr: float
    lr_schedule: str         # "constant" or "cosine"
    weight_decay: float = 0.1
    beta1: float = 0.9
    beta2: float = 0.95
    adam_eps: float = 1e-8
    eta_s: float = 1.0
    mu_s: float = 0.0
    nesterov: bool = False
    weights: str = "uniform"  # "uniform" | "tokens" | "dirichlet"
    zipf_s: float = 1.1
    zipf_s_range: tuple | None = None   # (lo, hi): every client draws its own exponent from its seed
    perm_top: float | None = 0.10
    recompute: int = 0
    micro_fuse: int = 1       # micro-batches the library may process as one pass (memory permitting)

    @property
    def tokens_per_step(self) -> int:
        return self.micro_batch * self.n_micro * self.model.seq_len

    def client_zipf_s(self, seed: int, client: int) -> float:
        """Zipf exponent of one client's token stream."""
        if self.zipf_s_range is None:
            return self.zipf_s
        from . import synth
        return synth.client_zipf_exponent(seed, client, *self.zipf_s_range)


TINY = RoundConfig(
    name="tiny-fp32", dtype="fp32",
    model=ModelShape(2, 64, 4, 256, 256, 32),
    micro_batch=4, n_micro=1, clients=2, local_steps=4, lr=1e-3, lr_schedule="constant",
    weights="tokens", perm_top=None)

M125 = RoundConfig(
    name="125M-bf16", dtype="bf16",
    model=ModelShape(12, 768, 12, 3072, 50368, 2048),
    micro_batch=8, n_micro=1, clients=4, local_steps=32, lr=6e-3, lr_schedule="cosine",
    mu_s=0.9, nesterov=True)

# the two remaining shapes of Table 4, as extra workloads (the 75M model has 56-wide heads, which
# the MFMA attention kernels do not cover: its attention runs on the plain kernels)
M75 = RoundConfig(
    name="75M-bf16", dtype="bf16",
    model=ModelShape(3, 896, 16, 3584, 50368, 1024),
    micro_batch=16, n_micro=1, clients=4, local_steps=32, lr=6e-3, lr_schedule="cosine",
    mu_s=0.9, nesterov=True)

M350 = RoundConfig(
    name="350M-bf16", dtype="bf16",
    model=ModelShape(24, 1024, 16, 4096, 50368, 2048),
    micro_batch=8, n_micro=2, clients=4, local_steps=16, lr=3e-3, lr_schedule="cosine",
    micro_fuse=2)

B1_3 = RoundConfig(
    name="1.3B-bf16", dtype="bf16",
    model=ModelShape(24, 2048, 16, 8192, 50368, 2048),
    micro_batch=4, n_micro=8, clients=4, local_steps=16, lr=4e-3, lr_schedule="constant",
    weights="dirichlet", micro_fuse=4)

B3 = RoundConfig(
    name="3B-bf16", dtype="bf16",
    model=ModelShape(32, 2560, 20, 10240, 50368, 2048),
    micro_batch=2, n_micro=1, clients=8, local_steps=8, lr=2e-3, lr_schedule="constant",
    recompute=1, zipf_s_range=(1.0, 1.3))

B7 = RoundConfig(
    name="7B-bf16", dtype="bf16",
    model=ModelShape(32, 4096, 32, 16384, 50368, 2048),
    micro_batch=1, n_micro=1, clients=8, local_steps=4, lr=1.2e-3, lr_schedule="constant",
    mu_s=0.9, nesterov=True, recompute=1)  # "full" recomputation = every block re-run, only block inputs kept

ALL = {c.name: c for c in (TINY, M75, M125, M350, B1_3, B3, B7)}


def reduced_depth(cfg: RoundConfig, n_layers: int, micro_batch: int = 1) -> RoundConfig:
    """Same kernel shapes (d, heads, d_ff, vocab, seq) with fewer blocks and a
    smaller micro-batch: the sizes at which the CPU oracle can still be run."""
    return replace(cfg, name=f"{cfg.name}-L{n_layers}", model=replace(cfg.model, n_layers=n_layers),
                   micro_batch=micro_batch, n_micro=1)


def lr_array(cfg: RoundConfig, n_steps: int, start: int = 0, period: int | None = None,
             warmup: int = 0) -> list[float]:
    """Per-step learning rates handed to the library (it never derives a schedule
    itself).  Cosine with linear warm-up and eta_min = 0.1 * eta_max, counted over
    sequential steps across rounds (Sec. 5 and the hyper-parameter table)."""
    import math
    out = []
    period = period if period is not None else n_steps
    for s in range(start, start + n_steps):
        if cfg.lr_schedule == "constant":
            out.append(cfg.lr)
        elif s < warmup:
            out.append(cfg.lr * (s + 1) / warmup)
        else:
            frac = min(1.0, (s - warmup) / max(1, period - warmup))
            lo = 0.1 * cfg.lr
            out.append(lo + 0.5 * (cfg.lr - lo) * (1.0 + math.cos(math.pi * frac)))
    return out
