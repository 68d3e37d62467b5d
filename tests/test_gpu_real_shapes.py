"""bf16 parity of TrainClient (Alg. 1; the inner loop of Alg. 3) at the paper's model shapes
(Table 4), as the library actually runs them, against the CPU oracle and through the C ABI:

* several optimizer steps in a row -- teacher-forced (the library restarted from the oracle's
  state at every step) and free-running (one call, the library's own weights carried from step
  to step, which is what shows a stale bf16 working copy);
* the benchmark's launch configuration of the 1.3B workload (16 sequences = 32,768 token rows
  per kernel launch, four LM-head row chunks);
* the 3B- and 7B-shaped blocks at full sequence length and vocabulary under their activation
  recomputation policies;
* the 1.3B-shaped model at its full depth of 24 blocks on one sequence.

Tolerances are the ones stated for bf16 mode: loss 1e-2 relative, gradient 3e-2 relative L2
(whole vector and per parameter group).  Where parameters after an AdamW step are compared, the
bound follows from the update rule: with zero initial moments the first update of every element
is -lr * g / (|g| + eps) -- lr in size, the gradient's sign -- so two gradients that agree to a
few 1e-3 in relative L2 give updates that differ only where |g| is within the noise, by at most
2 lr there.
"""

from dataclasses import replace

import numpy as np
import pytest
import torch

from helpers import group_errors, ohp, oshape, rel_l2
from oracle import photon_oracle as O
from paper_2411_02908_amd import configs, rounds, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


def _check_loss_grad(loss, g, ref_loss, ref_g, ms, label):
    errs = group_errors(g, ref_g, O.param_layout(oshape(ms))[0])
    worst = max(errs, key=errs.get)
    print(f"{label}: loss {loss:.5f} vs oracle {ref_loss:.5f} ({abs(loss - ref_loss) / ref_loss:.2e}); "
          f"gradient rel L2 {rel_l2(g, ref_g):.3e}, worst group {worst} {errs[worst]:.3e}", flush=True)
    assert abs(loss - ref_loss) / ref_loss < 1e-2
    assert rel_l2(g, ref_g) < 3e-2
    assert errs[worst] < 3e-2, errs


def _check_first_update(theta_before, theta_after, ref_after, lr, wd, label):
    """Parameters after one AdamW step from zero moments, against the oracle's: every element
    moved by at most lr from its decayed value, the two sides differ by at most 2 lr, and only
    on a small share of elements (those whose gradient is within the bf16 noise of zero)."""
    decayed = theta_before.astype(np.float64) * (1.0 - lr * wd)
    step = theta_after - decayed
    ref_step = ref_after - decayed
    assert np.abs(step).max() <= lr * (1 + 1e-4)
    differs = np.abs(step - ref_step) > 0.5 * lr
    share = float(differs.mean())
    print(f"{label}: share of parameters whose first update differs by more than lr / 2: {share:.2e}", flush=True)
    assert np.abs(step - ref_step).max() <= 2 * lr * (1 + 1e-4)
    assert share < 2e-2


def test_bf16_three_steps_teacher_forced_and_free_running(lib):
    """1.3B-shaped block (Table 4 widths, vocabulary, sequence length; one block so that the
    oracle finishes in seconds), three AdamW steps at the workload's learning rate on the same
    batch.  Teacher-forced: before every step the library's parameters and moments are those of
    the oracle; loss 1e-2, gradient 3e-2 at every step, and the parameters it writes stay within
    the update rule's bound of the oracle's.  Free-running: one call of three steps from the
    same start; the library's second and third steps run on the weights its own AdamW wrote
    (the bf16 working copy and its transposes), so its losses must follow the oracle's from step
    to step -- the same batch is used for every step, so a stale copy of the weights would
    repeat the first loss, and the oracle's losses are checked to move by far more than the
    tolerance."""
    cfg = configs.reduced_depth(configs.B1_3, 1, 1)
    ms = cfg.model
    sh, hp_o, hp = oshape(ms), ohp(cfg), rounds.make_hp(cfg)
    n_steps, lr = 3, cfg.lr
    theta0 = synth.init_params(synth.MASTER_SEED, ms.n_layers, ms.d_model, ms.d_ff, ms.vocab)
    tok1 = synth.client_token_batches(synth.MASTER_SEED, 0, 1, 1, 1, ms.seq_len, ms.vocab, cfg.zipf_s, cfg.perm_top)
    batches = np.repeat(tok1, n_steps, axis=0)              # [3, 1, 1, S + 1], the same batch
    n = theta0.size
    ctx = lib.photon_create(lib.model_cfg(ms, "bf16"), 1)

    # free-running library run first (one call)
    p, m, v = _dev(theta0), torch.zeros(n, device=DEV), torch.zeros(n, device=DEV)
    st = lib.OptState(m.data_ptr(), v.data_ptr(), 0)
    free = lib.photon_client_local_steps(ctx, p, st, _dev(batches), n_steps, 1, [lr] * n_steps, hp)
    assert st.step == n_steps
    free_theta = p.cpu().numpy()

    # oracle, step by step, with the teacher-forced library steps beside it
    th, mo, vo, t = theta0.astype(np.float64), np.zeros(n), np.zeros(n), 0
    ref_losses = []
    g_dev = torch.empty(n, dtype=torch.float32, device=DEV)
    for s in range(n_steps):
        ref_loss, ref_g = O.step_loss_and_grad(th, batches[s], sh)
        ref_losses.append(ref_loss)
        th32 = th.astype(np.float32)
        loss = lib.photon_client_loss_grad(ctx, _dev(th32), _dev(batches[s, 0]), g_dev)
        _check_loss_grad(loss, g_dev.cpu().numpy(), ref_loss, ref_g, ms, f"teacher-forced step {s}")
        p, m, v = _dev(th32), _dev(mo.astype(np.float32)), _dev(vo.astype(np.float32))
        st = lib.OptState(m.data_ptr(), v.data_ptr(), t)
        tf = lib.photon_client_local_steps(ctx, p, st, _dev(batches[s:s + 1]), 1, 1, [lr], hp)
        assert abs(tf[0] - ref_loss) / ref_loss < 1e-2 and st.step == t + 1
        th_next, mo, vo, t = O.adamw_step(th, mo, vo, ref_g, t, lr, hp_o)
        got = p.cpu().numpy()
        # |m_hat| <= 1.0003 sqrt(v_hat) for the first three steps at betas (0.9, 0.95) (Cauchy-Schwarz on the
        # two weightings of the gradient history), so an update is at most ~lr in size and the two
        # sides can differ by 2 lr, on elements whose gradients are within the bf16 noise only
        diff = np.abs(got - th_next)
        print(f"teacher-forced step {s}: max |theta - oracle| = {diff.max() / lr:.2f} lr, "
              f"share > lr / 2: {(diff > 0.5 * lr).mean():.2e}", flush=True)
        assert diff.max() <= 2.1 * lr and (diff > 0.5 * lr).mean() < 2e-2
        assert rel_l2(m.cpu().numpy(), mo) < 3e-2            # first moment: linear in the gradients
        th = th_next

    rel = [abs(a - b) / b for a, b in zip(free, ref_losses)]
    print("free-running losses", [f"{x:.5f}" for x in free], "oracle", [f"{x:.5f}" for x in ref_losses],
          "relative", [f"{x:.2e}" for x in rel], flush=True)
    moves = [abs(ref_losses[s + 1] - ref_losses[s]) / ref_losses[s] for s in range(n_steps - 1)]
    assert min(moves) > 5e-2, moves                          # the test is sharp: weights that did not move would show
    assert rel[0] < 1e-2
    # later steps run on parameters that differ on a small share of elements (sign-like updates of
    # near-zero gradient entries); the stated bf16 loss tolerance still holds (measured: ~1e-4)
    assert max(rel) < 1e-2
    diff = np.abs(free_theta - th)
    print(f"free-running: max |theta - oracle| = {diff.max() / lr:.2f} lr, share > lr / 2: {(diff > 0.5 * lr).mean():.2e}",
          flush=True)
    assert diff.max() <= 2 * n_steps * lr * (1 + 1e-4)


def test_bf16_benchmark_launch_configuration_against_oracle(lib):
    """What bench.py times, at one block: 16 sequences of the 1.3B-shaped model in one pass
    (4 micro-batches of 4, fused: M = 32,768 token rows per GEMM launch, the LM head in four row
    chunks), against the oracle's mean over the same 16 sequences.  Gradient through the
    single-pass entry point of a 16-sequence context (the same launches), then one optimizer step
    through photon_client_local_steps with micro_fuse = 4 exactly as the benchmark calls it."""
    cfg = replace(configs.reduced_depth(configs.B1_3, 1, configs.B1_3.micro_batch), n_micro=4, micro_fuse=4)
    ms = cfg.model
    sh = oshape(ms)
    theta0 = synth.init_params(synth.MASTER_SEED, ms.n_layers, ms.d_model, ms.d_ff, ms.vocab)
    n = theta0.size
    batches = synth.client_token_batches(synth.MASTER_SEED, 1, 1, cfg.n_micro, cfg.micro_batch, ms.seq_len, ms.vocab,
                                         cfg.zipf_s, cfg.perm_top)            # [1, 4, 4, S + 1]
    seqs = batches.reshape(-1, 1, ms.seq_len + 1)                             # 16 micro-batches of one sequence
    print("oracle: 16 sequences ...", flush=True)
    ref_loss, ref_g = O.step_loss_and_grad(theta0.astype(np.float64), seqs, sh)

    ctx16 = lib.photon_create(lib.model_cfg(ms, "bf16"), 16)
    g = torch.empty(n, dtype=torch.float32, device=DEV)
    loss = lib.photon_client_loss_grad(ctx16, _dev(theta0), _dev(batches.reshape(16, ms.seq_len + 1)), g)
    _check_loss_grad(loss, g.cpu().numpy(), ref_loss, ref_g, ms, "16 sequences, one pass")
    ctx16.close()
    del g
    torch.cuda.empty_cache()

    ctx = lib.photon_create(lib.model_cfg(ms, "bf16", 0, cfg.micro_fuse), cfg.micro_batch)
    p, m, v = _dev(theta0), torch.zeros(n, device=DEV), torch.zeros(n, device=DEV)
    st = lib.OptState(m.data_ptr(), v.data_ptr(), 0)
    losses = lib.photon_client_local_steps(ctx, p, st, _dev(batches), 1, cfg.n_micro, [cfg.lr], rounds.make_hp(cfg))
    print(f"fused step: loss {losses[0]:.5f} vs oracle {ref_loss:.5f}", flush=True)
    assert abs(losses[0] - ref_loss) / ref_loss < 1e-2
    ref_after, _, _, _ = O.adamw_step(theta0.astype(np.float64), np.zeros(n), np.zeros(n), ref_g, 0, cfg.lr, ohp(cfg))
    _check_first_update(theta0, p.cpu().numpy(), ref_after, cfg.lr, cfg.weight_decay, "fused step")
    # first moment after one step = (1 - beta1) g: the gradient of the fused pass itself, 3e-2
    assert rel_l2(m.cpu().numpy(), (1.0 - cfg.beta1) * ref_g) < 3e-2


LARGE = [(configs.B3, "3B-shaped L=1, micro-batch 2, per-block recomputation"),
         (configs.B7, "7B-shaped L=1, micro-batch 1, every block recomputed")]


@pytest.mark.parametrize("full,label", LARGE, ids=["3B", "7B"])
def test_bf16_large_shapes_full_sequence_and_vocabulary(lib, full, label):
    """One block of the 3B- and 7B-shaped models (Table 4) at the workloads' own micro-batch,
    sequence length 2048 and vocabulary 50368, under the workloads' recomputation policies: loss
    and gradient, then one optimizer step."""
    cfg = configs.reduced_depth(full, 1, full.micro_batch)
    ms = cfg.model
    sh = oshape(ms)
    theta0 = synth.init_params(synth.MASTER_SEED, ms.n_layers, ms.d_model, ms.d_ff, ms.vocab, generator="philox")
    n = theta0.size
    batches = synth.client_token_batches(synth.MASTER_SEED, 2, 1, 1, cfg.micro_batch, ms.seq_len, ms.vocab,
                                         cfg.client_zipf_s(synth.MASTER_SEED, 2), cfg.perm_top)   # [1, 1, Bm, S + 1]
    seqs = batches.reshape(-1, 1, ms.seq_len + 1)
    print(f"{label}: N = {n}; oracle ...", flush=True)
    ref_loss, ref_g = O.step_loss_and_grad(theta0.astype(np.float64), seqs, sh)
    ctx = lib.photon_create(lib.model_cfg(ms, "bf16", cfg.recompute), cfg.micro_batch)
    g = torch.empty(n, dtype=torch.float32, device=DEV)
    loss = lib.photon_client_loss_grad(ctx, _dev(theta0), _dev(batches[0, 0]), g)
    _check_loss_grad(loss, g.cpu().numpy(), ref_loss, ref_g, ms, label)
    del g
    p, m, v = _dev(theta0), torch.zeros(n, device=DEV), torch.zeros(n, device=DEV)
    st = lib.OptState(m.data_ptr(), v.data_ptr(), 0)
    losses = lib.photon_client_local_steps(ctx, p, st, _dev(batches), 1, 1, [cfg.lr], rounds.make_hp(cfg))
    assert abs(losses[0] - ref_loss) / ref_loss < 1e-2
    ref_after, _, _, _ = O.adamw_step(theta0.astype(np.float64), np.zeros(n), np.zeros(n), ref_g, 0, cfg.lr, ohp(cfg))
    _check_first_update(theta0, p.cpu().numpy(), ref_after, cfg.lr, cfg.weight_decay, label)


def test_bf16_full_depth_1_3b_one_sequence(lib):
    """The 1.3B-shaped model at its full depth (24 blocks, 1.31e9 parameters) on one sequence of
    2048 tokens: the oracle still runs this (about 1.7e13 float64 operations and 60 GB of host
    memory), so the growth of the bf16 error with depth is measured rather than assumed.  Loss
    1e-2; gradient 3e-2 over the whole vector and for every one of the 146 parameter groups."""
    cfg = configs.reduced_depth(configs.B1_3, configs.B1_3.model.n_layers, 1)
    ms = cfg.model
    sh = oshape(ms)
    print("full depth: parameters ...", flush=True)
    theta0 = synth.init_params(synth.MASTER_SEED, ms.n_layers, ms.d_model, ms.d_ff, ms.vocab, generator="philox")
    n = theta0.size
    assert n == 1_311_213_568
    tok = synth.client_token_batches(synth.MASTER_SEED, 3, 1, 1, 1, ms.seq_len, ms.vocab, cfg.zipf_s, cfg.perm_top)[0, 0]
    ctx = lib.photon_create(lib.model_cfg(ms, "bf16"), 1)
    g = torch.empty(n, dtype=torch.float32, device=DEV)
    loss = lib.photon_client_loss_grad(ctx, _dev(theta0), _dev(tok), g)
    g = g.cpu().numpy()
    ctx.close()
    torch.cuda.empty_cache()
    print(f"full depth: gpu loss {loss:.5f}; oracle ...", flush=True)
    ref_loss, ref_g = O.loss_and_grad(theta0.astype(np.float64), tok, sh)
    layout = O.param_layout(sh)[0]
    errs = group_errors(g, ref_g, layout)
    by_depth = [max(v for k, v in errs.items() if k.endswith(f".{l}")) for l in range(ms.n_layers)]
    print("worst group error per block, first to last:", " ".join(f"{e:.1e}" for e in by_depth), flush=True)
    _check_loss_grad(loss, g, ref_loss, ref_g, ms, "1.3B full depth, 1 x 2048 tokens")
