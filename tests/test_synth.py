"""Host logic of the seeded synthetic-input generators."""

import numpy as np

from paper_2411_02908_amd import configs, synth


def test_streams_are_reproducible_and_distinct():
    k0, k1 = synth.stream_key(7, "tokens", 0), synth.stream_key(7, "tokens", 1)
    assert k0 != k1 and k0 == synth.stream_key(7, "tokens", 0)
    a = synth.u64(k0, 100)
    assert np.array_equal(a[10:20], synth.u64(k0, 10, offset=10))     # counter-based
    assert not np.array_equal(a, synth.u64(k1, 100))
    # SplitMix64 reference vector: seed 0 gives 0xE220A8397B1DCDAF as its first word
    assert synth.u64(np.uint64(0), 1)[0] == np.uint64(0xE220A8397B1DCDAF)


def test_normal_moments_and_chunking():
    x = synth.normal(synth.stream_key(1, "n"), 200000, 0.02)
    assert abs(x.mean()) < 2e-4 and abs(x.std() / 0.02 - 1) < 0.01
    assert np.array_equal(x[:1000], synth.normal(synth.stream_key(1, "n"), 200000, 0.02, chunk=777)[:1000])


def test_zipf_frequencies_and_permutation():
    v = 256
    t = synth.zipf_tokens(synth.stream_key(2, "z"), (200000,), v, 1.1)
    assert t.min() >= 0 and t.max() < v and t.dtype == np.int32
    p = np.arange(1, v + 1) ** -1.1
    p /= p.sum()
    freq = np.bincount(t, minlength=v) / t.size
    assert np.abs(freq[:8] - p[:8]).max() < 5e-3
    perm = synth.vocab_permutation(synth.stream_key(2, "perm", 3), v, top=25)
    assert sorted(perm[:25]) == list(range(25)) and np.array_equal(perm[25:], np.arange(25, v))
    full = synth.vocab_permutation(synth.stream_key(2, "perm", 3), v)
    assert sorted(full) == list(range(v))


def test_client_batches_shape_and_heterogeneity():
    a = synth.client_token_batches(5, 0, 2, 3, 4, 32, 256, perm_top=None)
    b = synth.client_token_batches(5, 1, 2, 3, 4, 32, 256, perm_top=None)
    assert a.shape == (2, 3, 4, 33) and not np.array_equal(a, b)
    assert np.bincount(a.ravel()).argmax() != np.bincount(b.ravel()).argmax()


def test_dirichlet_weights_and_init():
    w = synth.dirichlet_weights(synth.stream_key(9, "weights"), 4)
    assert np.isclose(w.sum(), 1.0) and np.all(w > 0)
    th = synth.init_params(1, 2, 64, 256, 256)
    assert th.size == configs.TINY.model.n_params == 115008
    gains, n = synth.ln_gain_slices(2, 64, 256, 256)
    assert len(gains) == 5 and all(np.all(th[lo:hi] == 1.0) for lo, hi in gains)


def test_config_shapes_and_flops():
    assert configs.B1_3.model.n_params == 1311213568
    assert configs.B1_3.tokens_per_step == 65536
    assert abs(configs.B1_3.model.flops_per_token() / 8.47e9 - 1) < 0.01
    lrs = configs.lr_array(configs.M125, 32)
    assert abs(lrs[0] - 6e-3) < 1e-12 and lrs[-1] < 1.1e-3 and all(x >= y for x, y in zip(lrs, lrs[1:]))


def test_client_zipf_exponents_are_seeded_distinct_and_shape_the_stream():
    """Heterogeneous token streams: every client draws its exponent in [lo, hi) from its own
    stream; a larger exponent gives a more skewed unigram law (rank 1 more frequent, the share of
    the closed form 1 / sum r^-s)."""
    from paper_2411_02908_amd import configs
    cfg = configs.B3
    exps = [cfg.client_zipf_s(synth.MASTER_SEED, k) for k in range(cfg.clients)]
    assert exps == [cfg.client_zipf_s(synth.MASTER_SEED, k) for k in range(cfg.clients)]
    assert len(set(exps)) == cfg.clients and all(1.0 <= e < 1.3 for e in exps)
    assert exps != [cfg.client_zipf_s(synth.MASTER_SEED + 1, k) for k in range(cfg.clients)]
    assert configs.B1_3.client_zipf_s(synth.MASTER_SEED, 3) == 1.1            # homogeneous configurations
    vocab = 5000
    for k in (int(np.argmin(exps)), int(np.argmax(exps))):
        tok = synth.zipf_tokens(synth.stream_key(1, "t", k), (200_000,), vocab, exps[k])
        top = float(np.mean(tok == 0))
        expect = 1.0 / float(np.sum(np.arange(1, vocab + 1, dtype=np.float64) ** -exps[k]))
        assert abs(top - expect) < 4 * np.sqrt(expect * (1 - expect) / tok.size)
