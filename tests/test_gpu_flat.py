"""GPU parity of the flat-vector kernels (pseudo-gradient export, weighted FedAvg + server
optimizer, AdamW) against the CPU oracle, through the C ABI."""

import numpy as np
import pytest
import torch

from helpers import bf16_round, rel_l2
from oracle import photon_oracle as O
from paper_2411_02908_amd import configs, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
# spans more than one grid sweep of 2048 x 256 x 8 elements and leaves a ragged tail of 3
N_RAGGED = 2048 * 256 * 8 + 70003


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


def _vec(purpose, n, std=1.0, index=0):
    return synth.gaussian_vector(7, purpose, n, std, index)


@pytest.mark.parametrize("n", [5, 8, 1000, N_RAGGED])
def test_export_delta_fp32_exact_and_bf16_rne(lib, n):
    g, c = _vec("g", n), _vec("c", n, 1.0, 1)
    ctx = lib.photon_create_flat(n)
    out32 = torch.empty(n, dtype=torch.float32, device=DEV)
    out16 = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    lib.photon_export_delta(ctx, _dev(g), _dev(c), out32, lib.FP32)
    lib.photon_export_delta(ctx, _dev(g), _dev(c), out16, lib.BF16)
    ref = O.pseudo_gradient(g, c)                       # float64 difference of float32 values
    got32 = out32.cpu().numpy()
    assert np.array_equal(got32, ref.astype(np.float32))            # one IEEE subtraction: bit-exact
    assert np.array_equal(out16.float().cpu().numpy(), bf16_round(ref.astype(np.float32)))


@pytest.mark.parametrize("K,kind,dtype,mu,nesterov,n", [
    (1, "params", "fp32", 0.0, False, 1000),
    (2, "params", "fp32", 0.0, False, N_RAGGED),
    (4, "deltas", "bf16", 0.0, False, N_RAGGED),
    (4, "deltas", "bf16", 0.9, True, N_RAGGED),
    (3, "deltas", "fp32", 0.5, False, 70001),
    (8, "deltas", "bf16", 0.9, True, 262147),
    (11, "deltas", "bf16", 0.9, True, 70003),
    (11, "params", "fp32", 0.0, False, 4099),
])
def test_aggregate_matches_oracle_and_is_bit_reproducible(lib, K, kind, dtype, mu, nesterov, n):
    theta = _vec("theta", n)
    clients = [theta + _vec("d", n, 0.01, k) for k in range(K)]
    weights = list(synth.dirichlet_weights(synth.stream_key(3, "w"), K) * 17.0)   # unnormalised
    mom0 = _vec("mom", n, 0.01) if mu else None
    eta = 0.7
    ctx = lib.photon_create_flat(n)
    if kind == "params":
        bufs = [_dev(c) for c in clients]
        ref_deltas = [O.pseudo_gradient(theta, c.astype(np.float32)) for c in clients]
        k_, d_ = lib.CLIENT_PARAMS, lib.FP32
    else:
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        bufs = []
        for c in clients:
            d = torch.empty(n, dtype=tdt, device=DEV)
            lib.photon_export_delta(ctx, _dev(theta), _dev(c), d, lib.BF16 if dtype == "bf16" else lib.FP32)
            bufs.append(d)
        # the oracle reads the exported values themselves (each exactly representable in float64)
        ref_deltas = [b.float().cpu().numpy().astype(np.float64) for b in bufs]
        k_, d_ = lib.CLIENT_DELTAS, lib.BF16 if dtype == "bf16" else lib.FP32

    results = []
    for rep in range(2):
        th = _dev(theta)
        mom = _dev(mom0) if mu else None
        oo = lib.OuterOpt(eta, mu, int(nesterov), 0 if mom is None else mom.data_ptr(), 0)
        met = lib.photon_aggregate(ctx, th, bufs, k_, d_, weights, oo)
        assert oo.round == 1
        results.append((th.cpu().numpy(), None if mom is None else mom.cpu().numpy(), met))
    a, b = results
    assert np.array_equal(a[0], b[0])                                    # bit-identical reruns
    assert mu == 0 or np.array_equal(a[1], b[1])
    assert a[2] == b[2]

    ref_theta, ref_b, ref_met = O.aggregate_deltas(theta, ref_deltas, weights, mom0, eta, mu, nesterov)
    err_theta = rel_l2(a[0], ref_theta)
    assert err_theta < 1e-6
    # the applied update: 1e-6 of its own size plus what storing theta in float32 costs
    # (half an ulp of theta for the result, and for PARAMS the float32 difference theta - theta_k)
    upd = theta - ref_theta
    tol_u = 1e-6 + 2.0 ** -23 * np.linalg.norm(theta) / np.linalg.norm(upd)
    err_u = rel_l2(theta.astype(np.float64) - a[0], upd)
    assert err_u < tol_u
    if mu:
        assert rel_l2(a[1], ref_b) < 1e-6
    assert abs(a[2]["delta_norm2"] / ref_met["delta_norm2"] - 1) < 1e-5
    # per-client norms for every K and kind: taken against the model as it was before the step
    assert np.allclose(a[2]["client_norm2"], ref_met["client_norm2"], rtol=1e-5)


def test_fedavg_identities_on_gpu(lib):
    n = 100003
    theta, tk = _vec("theta", n), _vec("tk", n, 1.0, 1)
    ctx = lib.photon_create_flat(n)
    # K identical clients, any weights -> that client; K = 1 -> that client
    for K, w in ((3, [0.2, 0.5, 0.3]), (1, [5.0])):
        th = _dev(theta)
        lib.photon_aggregate(ctx, th, [_dev(tk) for _ in range(K)], lib.CLIENT_PARAMS, lib.FP32, w,
                             lib.OuterOpt(1.0, 0.0, 0, 0, 0))
        assert rel_l2(th.cpu().numpy(), tk) < 1e-6
    # dropping a client = the weighted mean of the survivors
    cl = [_vec("c", n, 1.0, k) for k in range(4)]
    w = [1.0, 4.0, 2.5, 0.5]
    th = _dev(theta)
    lib.photon_aggregate(ctx, th, [_dev(c) for c in (cl[0], cl[1], cl[3])], lib.CLIENT_PARAMS, lib.FP32,
                         [w[0], w[1], w[3]], lib.OuterOpt(1.0, 0.0, 0, 0, 0))
    ref = (w[0] * cl[0].astype(np.float64) + w[1] * cl[1] + w[3] * cl[3]) / (w[0] + w[1] + w[3])
    assert rel_l2(th.cpu().numpy(), ref) < 1e-6


def test_aggregate_rejects_bad_arguments(lib):
    n = 64
    ctx = lib.photon_create_flat(n)
    th, c = _dev(_vec("a", n)), _dev(_vec("b", n))
    oo = lib.OuterOpt(1.0, 0.0, 0, 0, 0)
    for w in ([-1.0], [0.0], [float("nan")], [float("inf")]):
        with pytest.raises(lib.PhotonError):
            lib.photon_aggregate(ctx, th, [c], lib.CLIENT_PARAMS, lib.FP32, w, oo)
    with pytest.raises(lib.PhotonError):                       # momentum missing with mu != 0
        lib.photon_aggregate(ctx, th, [c], lib.CLIENT_PARAMS, lib.FP32, [1.0], lib.OuterOpt(1.0, 0.9, 1, 0, 0))
    with pytest.raises(lib.PhotonError):                       # PARAMS must be fp32
        lib.photon_aggregate(ctx, th, [c], lib.CLIENT_PARAMS, lib.BF16, [1.0], oo)
    with pytest.raises(lib.PhotonError):                       # misaligned pointer
        lib.photon_aggregate(ctx, th, [c[1:]], lib.CLIENT_PARAMS, lib.FP32, [1.0], oo)
    # a client buffer that shares memory with the model or with the momentum buffer, or a momentum
    # buffer that is the model: refused (the kernel rewrites both in place while reading clients)
    mom = torch.zeros(n, device=DEV)
    big = torch.zeros(2 * n, device=DEV)
    for bufs, model, m_ in (([th], th, None), ([mom], th, mom), ([big[n - 8:2 * n - 8]], big[:n], None),
                            ([c], th, th)):
        with pytest.raises(lib.PhotonError):
            lib.photon_aggregate(ctx, model, bufs, lib.CLIENT_PARAMS, lib.FP32, [1.0],
                                 lib.OuterOpt(1.0, 0.5 if m_ is not None else 0.0, 0, lib._ptr(m_), 0))
    assert np.array_equal(th.cpu().numpy(), _vec("a", n))       # nothing was written


@pytest.mark.parametrize("n,with_bf16", [(7, False), (4099, True), (N_RAGGED, True)])
def test_adamw_matches_oracle(lib, n, with_bf16):
    hp_o = O.AdamWHP(0.9, 0.95, 1e-8, 0.1)
    hp = lib.AdamWHP(0.9, 0.95, 1e-8, 0.1)
    theta = _vec("theta", n, 0.02)
    p, m, v = _dev(theta), torch.zeros(n, device=DEV), torch.zeros(n, device=DEV)
    w16 = torch.empty(n, dtype=torch.bfloat16, device=DEV) if with_bf16 else None
    st = lib.OptState(m.data_ptr(), v.data_ptr(), 0)
    ctx = lib.photon_create_flat(n)
    rp, rm, rv, rt = theta.astype(np.float64), np.zeros(n), np.zeros(n), 0
    for s in range(4):
        g = _vec("grad", n, 10.0 ** (s - 3), s)
        lr = 1e-3 * (s + 1)
        lib.photon_adamw_step(ctx, p, st, _dev(g), lr, hp, w16)
        rp, rm, rv, rt = O.adamw_step(rp, rm, rv, g.astype(np.float64), rt, lr, hp_o)
        assert st.step == rt
        assert rel_l2(p.cpu().numpy(), rp) < 1e-6
        assert rel_l2(m.cpu().numpy(), rm) < 1e-6 and rel_l2(v.cpu().numpy(), rv) < 1e-6
        # the step actually taken, not just the parameters
        err_step = rel_l2(p.cpu().numpy().astype(np.float64) - theta, rp - theta)
        assert err_step < 1e-5
        if with_bf16:
            assert np.array_equal(w16.float().cpu().numpy(), bf16_round(p.cpu().numpy()))


def test_clip_delta(lib):
    n = 70003
    d = _vec("d", n, 0.1)
    ctx = lib.photon_create_flat(n)
    ref_norm = float(np.linalg.norm(d.astype(np.float64)))
    for max_norm in (ref_norm * 2, ref_norm / 4):
        t = _dev(d)
        nrm = lib.photon_clip_delta(ctx, t, lib.FP32, max_norm)
        assert abs(nrm / ref_norm - 1) < 1e-6
        assert rel_l2(t.cpu().numpy(), O.clip_update(d.astype(np.float64), max_norm)) < 1e-6


def test_clip_delta_bf16(lib):
    """A bf16 pseudo-gradient is clipped in place: norm of the stored bf16 values; each element
    scaled in float32 and rounded back to bf16 (ties to even), both decided in float32."""
    n = 70003
    d16 = bf16_round(_vec("d", n, 0.1))                      # the values a bf16 buffer holds
    ctx = lib.photon_create_flat(n)
    ref_norm = float(np.linalg.norm(d16.astype(np.float64)))
    for max_norm in (ref_norm * 2, ref_norm / 4):
        t = _dev(d16).to(torch.bfloat16)
        nrm = lib.photon_clip_delta(ctx, t, lib.BF16, max_norm)
        assert abs(nrm / ref_norm - 1) < 1e-6
        got = t.float().cpu().numpy()
        if max_norm > ref_norm:
            assert np.array_equal(got, d16)                   # below the bound: untouched
        else:
            ref = O.clip_update(d16.astype(np.float64), max_norm)
            assert rel_l2(got, ref) < 2.0 ** -8               # bf16 storage: half an ulp = 2^-9 relative per element
            # element-wise: the float32 product with the float32 scale, rounded to bf16
            sc = np.float32(max_norm / nrm)
            assert np.array_equal(got, bf16_round(d16 * sc))


def test_full_size_aggregate_sampled(lib):
    """The 1.3B-parameter vector with K = 4 bf16 deltas, in the launch the benchmark times:
    sampled outputs against the oracle, norms against a float64 library sum."""
    n = 1311213568
    K = 4
    gen = torch.Generator(device=DEV).manual_seed(11)
    theta = torch.randn(n, device=DEV, generator=gen) * 0.02
    deltas = [(torch.randn(n, device=DEV, generator=gen) * 1e-3).to(torch.bfloat16) for _ in range(K)]
    weights = list(synth.dirichlet_weights(synth.stream_key(synth.MASTER_SEED, "weights"), K))
    idx = torch.from_numpy(np.unique(np.concatenate([
        (synth.u64(synth.stream_key(1, "idx"), 200000) % np.uint64(n)).astype(np.int64),
        np.arange(0, 4096), np.arange(n - 4096, n)]))).to(DEV)
    th_s = theta[idx].cpu().numpy()
    d_s = [d[idx].float().cpu().numpy().astype(np.float64) for d in deltas]
    ctx = lib.photon_create_flat(n)
    met = lib.photon_aggregate(ctx, theta, deltas, lib.CLIENT_DELTAS, lib.BF16, weights,
                               lib.OuterOpt(1.0, 0.0, 0, 0, 0))
    ref, _, _ = O.aggregate_deltas(th_s, d_s, weights)
    assert rel_l2(theta[idx].cpu().numpy(), ref) < 1e-6
    for k in range(K):
        exact = float((deltas[k].double() ** 2).sum().item())
        assert abs(met["client_norm2"][k] / exact - 1) < 1e-5


def test_full_size_7b_aggregate_nesterov_sampled(lib):
    """The 7B-shaped configuration's aggregation at its full size: 6.65e9 parameters (indices past
    2^32), K = 8 bf16 deltas streamed in fixed order, server Nesterov momentum, two rounds so that
    the momentum buffer is read as well as written.  Sampled outputs against the oracle."""
    n = configs.B7.model.n_params
    assert n == 6_649_024_512
    K = 8
    gen = torch.Generator(device=DEV).manual_seed(13)
    theta = torch.randn(n, device=DEV, generator=gen) * 0.02
    mom = torch.zeros(n, device=DEV)
    deltas = []
    for _ in range(K):
        d = torch.empty(n, dtype=torch.bfloat16, device=DEV)
        for lo in range(0, n, 1 << 30):        # in slices: no 26 GB float32 temporary per client
            hi = min(n, lo + (1 << 30))
            d[lo:hi] = (torch.randn(hi - lo, device=DEV, generator=gen) * 1e-3).to(torch.bfloat16)
        deltas.append(d)
    weights = [1.0 + 0.25 * k for k in range(K)]
    idx = torch.from_numpy(np.unique(np.concatenate([
        (synth.u64(synth.stream_key(2, "idx"), 200000) % np.uint64(n)).astype(np.int64),
        np.arange(0, 4096), np.arange((1 << 32) - 2048, (1 << 32) + 2048), np.arange(n - 4096, n)]))).to(DEV)
    th_s = theta[idx].cpu().numpy().astype(np.float64)
    d_s = [d[idx].float().cpu().numpy().astype(np.float64) for d in deltas]
    ctx = lib.photon_create_flat(n)
    oo = lib.OuterOpt(0.7, 0.9, 1, mom.data_ptr(), 0)
    print("7B aggregate: inputs resident", flush=True)
    ref_b = None
    for r in range(2):
        met = lib.photon_aggregate(ctx, theta, deltas, lib.CLIENT_DELTAS, lib.BF16, weights, oo)
        th_s, ref_b, _ = O.aggregate_deltas(th_s, d_s, weights, ref_b, 0.7, 0.9, True)
        assert rel_l2(theta[idx].cpu().numpy(), th_s) < 1e-6
        assert rel_l2(mom[idx].cpu().numpy(), ref_b) < 1e-6
    assert oo.round == 2
    exact = float(sum((deltas[0][lo:lo + (1 << 30)].double() ** 2).sum().item() for lo in range(0, n, 1 << 30)))
    assert abs(met["client_norm2"][0] / exact - 1) < 1e-5


def test_stream_probe_moves_what_it_says_and_checks_its_arguments(lib):
    """The measurement aid: with r reads and w writes every destination vector holds the sum of the
    r sources plus the kernel's constant (1, 2, 3, 4 per group of four elements)."""
    n = 4 * 100_003
    ctx = lib.photon_create_flat(n)
    src = torch.arange(3 * n, dtype=torch.float32, device=DEV) * 1e-3
    dst = torch.zeros(2 * n, device=DEV)
    ms = lib.photon_stream_probe(ctx, 3, 2, src, dst, n, 2)
    assert ms > 0
    want = src[:n] + src[n:2 * n] + src[2 * n:] + torch.tensor([1.0, 2.0, 3.0, 4.0], device=DEV).repeat(n // 4)
    assert torch.allclose(dst[:n], want, rtol=1e-6) and torch.equal(dst[:n], dst[n:])
    assert lib.photon_stream_probe(ctx, 2, 0, src, dst, n, 1) > 0          # read-only: dst untouched
    assert torch.equal(dst[:n], dst[n:])
    for bad in ((0, 0, n), (5, 1, n), (1, 5, n), (1, 1, n + 2)):
        with pytest.raises(lib.PhotonError):
            lib.photon_stream_probe(ctx, bad[0], bad[1], src, dst, bad[2], 1)
