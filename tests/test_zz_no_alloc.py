"""photon_aggregate_static -- the aggregation entry point that allocates nothing (its norm slots
live in a device array inside the library) -- against photon_aggregate, through the C ABI:
same kernels, so the model, the momentum and the norms must agree bit for bit.  Two calls in a
row on the same device share the array; the second is smaller in every dimension."""

import numpy as np
import pytest
import torch

from paper_2411_02908_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


def _case(lib, n, K, kind, dtype, mu, nesterov, eta, seed):
    theta = synth.gaussian_vector(seed, "theta", n)
    if kind == lib.CLIENT_DELTAS:
        bufs = [synth.gaussian_vector(seed, "delta", n, 1e-2, k) for k in range(K)]
    else:
        bufs = [(theta + synth.gaussian_vector(seed, "delta", n, 1e-2, k)).astype(np.float32) for k in range(K)]
    tdt = torch.bfloat16 if dtype == lib.BF16 else torch.float32
    dbufs = [_dev(b).to(tdt) for b in bufs]
    weights = [1.0 + 0.5 * k for k in range(K)]
    mom0 = synth.gaussian_vector(seed, "mom", n, 1e-3) if mu != 0.0 else None

    # existing entry point (context with its own workspace)
    ctx = lib.photon_create_flat(n)
    th_a = _dev(theta)
    mom_a = _dev(mom0) if mom0 is not None else None
    oo_a = lib.OuterOpt(eta, mu, int(nesterov), lib._ptr(mom_a), 3)
    met = lib.photon_aggregate(ctx, th_a, dbufs, kind, dtype, weights, oo_a)
    ctx.close()

    # allocation-free entry point: every buffer it touches exists before the call
    th_b = _dev(theta)
    mom_b = _dev(mom0) if mom0 is not None else None
    norms = torch.full((K + 1,), -7.0, dtype=torch.float64, device=DEV)
    oo_b = lib.OuterOpt(eta, mu, int(nesterov), lib._ptr(mom_b), 3)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    lib.photon_aggregate_static(torch.cuda.current_stream().cuda_stream, n, th_b, dbufs, kind, dtype, weights, oo_b, norms)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()

    assert oo_a.round == 4 and oo_b.round == 4
    assert torch.equal(th_a, th_b)
    if mom0 is not None:
        assert torch.equal(mom_a, mom_b)
    got = norms.cpu().numpy()
    assert got[0] == met["delta_norm2"]
    assert list(got[1:]) == met["client_norm2"]
    assert got[0] > 0 and all(g > 0 for g in got[1:])


def test_static_aggregate_matches_context_aggregate_twice_in_a_row(lib):
    # first call: ragged length, K = 4 bf16 pseudo-gradients, Nesterov server momentum
    _case(lib, 1_000_003, 4, lib.CLIENT_DELTAS, lib.BF16, 0.9, True, 0.7, seed=41)
    # second call, smaller in length and unrelated in kind: K = 11 (the run-time-K kernel and the
    # per-client norm passes) client parameter vectors in float32, plain FedAvg
    _case(lib, 70_001, 11, lib.CLIENT_PARAMS, lib.FP32, 0.0, False, 1.0, seed=42)
    # third, smaller again: K = 2 float32 pseudo-gradients with plain server momentum
    _case(lib, 4_099, 2, lib.CLIENT_DELTAS, lib.FP32, 0.5, False, 1.0, seed=43)


def test_static_aggregate_rejects_sizes_beyond_its_scratch(lib):
    n = 1024
    theta = torch.zeros(n, device=DEV)
    K = lib.STATIC_MAX_CLIENTS + 1
    bufs = [torch.zeros(n, device=DEV) for _ in range(K)]
    oo = lib.OuterOpt(1.0, 0.0, 0, None, 0)
    with pytest.raises(lib.PhotonError) as ei:
        lib.photon_aggregate_static(0, n, theta, bufs, lib.CLIENT_DELTAS, lib.FP32, [1.0] * K, oo)
    assert ei.value.status == lib.ELIMIT and oo.round == 0
    with pytest.raises(lib.PhotonError) as ei:     # the ordinary argument checks still apply
        lib.photon_aggregate_static(0, n, theta, [theta], lib.CLIENT_DELTAS, lib.FP32, [1.0], oo)
    assert ei.value.status == lib.EINVAL
