"""Seeded synthetic inputs for the federated-round hot path.

This module only produces *inputs*: random streams, token batches, vocabulary
permutations, client weights and initial parameter vectors.  It contains none
of the method's arithmetic (no model, no optimizer, no averaging), so both the
CPU oracle's tests and the HIP path's tests can draw the same inputs from it.

The public corpora the paper trains on (C4 shards, Sec. 5; The Pile subsets for
the heterogeneity study) are replaced by i.i.d. Zipf token streams: throughput
depends on shapes only, and the skewed unigram law exercises cross-entropy
with unbalanced targets.  Per-client heterogeneity comes from a seeded
permutation of the most frequent ranks.

Random numbers come from one counter-based generator, SplitMix64 (Steele,
Lea, Flood 2014): word i of a stream with key k is mix(k + (i+1)*GOLDEN).
Every draw is therefore reproducible from (seed, purpose, index) alone.
"""

from __future__ import annotations

import math

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
MASTER_SEED = 0x5EED


def _mix64(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def stream_key(seed: int, purpose: str, index: int = 0) -> np.uint64:
    """Key of an independent stream: FNV-1a of the purpose, mixed with seed and index."""
    h = 0xCBF29CE484222325
    for byte in purpose.encode():
        h = ((h ^ byte) * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    with np.errstate(over="ignore"):
        k = _mix64(np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + _GOLDEN * np.uint64(h))
        k = _mix64(k ^ (_GOLDEN * np.uint64(index + 1)))
    return np.uint64(k)


def u64(key: np.uint64, n: int, offset: int = 0) -> np.ndarray:
    """Words offset .. offset+n-1 of the stream."""
    ctr = np.arange(offset + 1, offset + n + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix64(np.uint64(key) + ctr * _GOLDEN)


def uniform(key: np.uint64, n: int, offset: int = 0) -> np.ndarray:
    """float64 uniforms in [0, 1) with 53 random bits."""
    return (u64(key, n, offset) >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)


def normal(key: np.uint64, n: int, std: float = 1.0, chunk: int = 1 << 22) -> np.ndarray:
    """float32 N(0, std^2) by Box-Muller, two uniforms per value."""
    out = np.empty(n, dtype=np.float32)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        w = u64(key, 2 * (hi - lo), 2 * lo)
        u1 = ((w[0::2] >> np.uint64(11)).astype(np.float64) + 1.0) * (2.0 ** -53)  # (0, 1]
        u2 = (w[1::2] >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)
        out[lo:hi] = (std * np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)).astype(np.float32)
    return out


# ----------------------------------------------------------------------------
# tokens

def zipf_cdf(vocab: int, s: float) -> np.ndarray:
    """Cumulative table of p(r) proportional to r^-s over ranks r = 1..vocab (float64)."""
    p = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(p)
    return c / c[-1]


def vocab_permutation(key: np.uint64, vocab: int, top: int | None = None) -> np.ndarray:
    """Seeded permutation of the `top` most frequent ranks (all of them if None);
    identity elsewhere.  Maps rank-1 -> token id."""
    top = vocab if top is None else min(top, vocab)
    perm = np.arange(vocab, dtype=np.int64)
    order = np.argsort(u64(key, top), kind="stable")
    perm[:top] = order
    return perm


def zipf_tokens(key: np.uint64, shape, vocab: int, s: float = 1.1,
                perm: np.ndarray | None = None) -> np.ndarray:
    """i.i.d. Zipf(s) token ids of the given shape (int32), optionally permuted."""
    n = int(np.prod(shape))
    cdf = zipf_cdf(vocab, s)
    ranks0 = np.searchsorted(cdf, uniform(key, n), side="right")
    ranks0 = np.minimum(ranks0, vocab - 1)
    ids = ranks0 if perm is None else perm[ranks0]
    return ids.astype(np.int32).reshape(shape)


def client_token_batches(seed: int, client: int, n_steps: int, n_micro: int, micro_batch: int,
                         seq_len: int, vocab: int, s: float = 1.1,
                         perm_top: float | None = None) -> np.ndarray:
    """int32 [n_steps, n_micro, micro_batch, seq_len + 1] for one client.

    perm_top = None permutes the whole vocabulary per client, a fraction permutes
    only that share of the most frequent ranks."""
    top = None if perm_top is None else max(1, int(vocab * perm_top))
    perm = vocab_permutation(stream_key(seed, "perm", client), vocab, top)
    return zipf_tokens(stream_key(seed, "tokens", client),
                       (n_steps, n_micro, micro_batch, seq_len + 1), vocab, s, perm)


def client_zipf_exponent(seed: int, client: int, lo: float, hi: float) -> float:
    """Per-client Zipf exponent, uniform in [lo, hi) from the client's own stream: clients whose
    token streams differ in skew (heterogeneous data silos)."""
    return float(lo + (hi - lo) * uniform(stream_key(seed, "zipf_s", client), 1)[0])


def zipf_entropy(vocab: int, s: float) -> float:
    """Entropy (nats) of the unigram law: the floor of the loss on i.i.d. tokens."""
    p = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
    p /= p.sum()
    return float(-(p * np.log(p)).sum())


# ----------------------------------------------------------------------------
# client weights

def dirichlet_weights(key: np.uint64, k: int) -> np.ndarray:
    """Dirichlet(alpha = 1) sample: normalised exponentials, float64."""
    e = -np.log1p(-uniform(key, k))
    return e / e.sum()


# ----------------------------------------------------------------------------
# initial parameters

def ln_gain_slices(n_layers: int, d: int, d_ff: int, vocab: int):
    """(start, stop) of every LayerNorm gain inside the flat parameter vector
    [E | per block: g1, Wqkv, Wo, g2, W1, W2 | gf]."""
    out = []
    pos = vocab * d
    for _ in range(n_layers):
        out.append((pos, pos + d))
        pos += d + 3 * d * d + d * d
        out.append((pos, pos + d))
        pos += d + 2 * d * d_ff
    out.append((pos, pos + d))
    return out, pos + d


def init_params(seed: int, n_layers: int, d: int, d_ff: int, vocab: int,
                std: float = 0.02, generator: str = "splitmix") -> np.ndarray:
    """Flat float32 parameter vector: N(0, std^2) everywhere, LayerNorm gains = 1.

    generator = "splitmix": this module's counter streams (Box-Muller), about 10 M values/s;
    "philox": numpy's counter-based Philox bit generator keyed by the same stream key, about ten
    times faster -- for the vectors of a billion parameters that full-depth cases need."""
    gains, n = ln_gain_slices(n_layers, d, d_ff, vocab)
    key = stream_key(seed, "init")
    if generator == "philox":
        rng = np.random.Generator(np.random.Philox(key=int(key)))
        theta = rng.standard_normal(n, dtype=np.float32)
        theta *= np.float32(std)
    else:
        theta = normal(key, n, std)
    for lo, hi in gains:
        theta[lo:hi] = 1.0
    return theta


def gaussian_vector(seed: int, purpose: str, n: int, std: float = 1.0, index: int = 0) -> np.ndarray:
    """A plain float32 Gaussian vector (for optimizer / aggregation unit inputs)."""
    return normal(stream_key(seed, purpose, index), n, std)
