"""Parity of the HIP library with the CPU oracle, element by element, through the C ABI.

Tolerance (FP32 matrix-core math): max|a-b| / max|b| <= 1e-4 per tensor, applied to the
weights, to every per-step update W_t - W_{t-1}, to the cumulative update, and to every
state buffer; the bases are compared directly (same sign convention) and must be
orthogonal to 1e-5.
"""
import numpy as np
import pytest
import torch

from oracle import br_oracle as oc
from oracle.metrics import orthogonality_defect, rel_err
from paper_2602_03515_amd import synth

pytestmark = pytest.mark.gpu

TOL = 1e-4


@pytest.fixture(scope="module")
def harness():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from tests import gpu_harness
    return gpu_harness


def _storage_floor(W, dW, bf16_params=False):
    """The library keeps weights in FP32 (the master copy for BF16 parameters), so an update read
    back as a difference of stored weights is only known to one FP32 ulp of the weights.  Relative
    to the update that is 2^-23 max|W| / max|dW|; it is added to the tolerance of update
    comparisons (it vanishes when W0 = 0, which a dedicated test uses)."""
    scale = np.abs(dW).max()
    return float(2.0 ** -23 * np.abs(W).max() / scale) if scale > 0 else 0.0


def _run(h, W0s, grads_per_step, freq, lr, tol=TOL, check_q=True, **kw):
    sb = h.SideBySide(W0s, freq=freq, lr=lr, **kw)
    prev_gpu = [sb.gpu_weights(i) for i in range(len(W0s))]
    prev_ref = [w.copy() for w in sb.W_ref]
    w0 = [w.copy() for w in sb.W_ref]
    for t, grads in enumerate(grads_per_step, 1):
        sb.step(grads)
        for i in range(len(W0s)):
            g_now, r_now = sb.gpu_weights(i), sb.W_ref[i]
            e = rel_err(g_now - prev_gpu[i], r_now - prev_ref[i])
            lim = tol + _storage_floor(r_now, r_now - prev_ref[i], kw.get("bf16_params", False))
            assert e <= lim, f"step {t} matrix {i}: update rel err {e:.3e} > {lim:.3e}"
            prev_gpu[i], prev_ref[i] = g_now, r_now.copy()
    for i in range(len(W0s)):
        e = rel_err(sb.gpu_weights(i) - w0[i], sb.W_ref[i] - w0[i])
        lim = tol + _storage_floor(sb.W_ref[i], sb.W_ref[i] - w0[i], kw.get("bf16_params", False))
        assert e <= lim, f"matrix {i}: cumulative update rel err {e:.3e} > {lim:.3e}"
    worst = sb.compare_state(tol, check_q=check_q)
    for i, st in enumerate(sb.states):
        for which, Q in ((sb.B.BR_STATE_QL, st.QL), (sb.B.BR_STATE_QR, st.QR)):
            if Q is not None:
                bar = 1e-5
                assert orthogonality_defect(h.to_np(sb.opt.state(i, which))) < bar
    return sb, worst


def test_config1_256x256_bilateral_20_steps(harness):
    """256 x 256 FP32, bilateral, refresh every 5 steps, 20 steps (delay tau = 3 only renames
    gradient buffers because these gradients do not depend on the weights)."""
    W0, grads = synth.spiked_gradients(seed=0, m=256, n=256, steps=20, noise_std=0.1)
    sb, worst = _run(harness, [W0], [[g] for g in grads], freq=5, lr=1e-3)
    print("config 1 worst rel errs:", {k: f"{v:.2e}" for k, v in worst.items()})
    assert sb.opt.step_count == 20


def test_config1_updates_from_zero_weights(harness):
    """Same gradients as config 1 but W0 = 0: the weights ARE the cumulative update, so the
    1e-4 bar applies to the rotated updates with no storage floor."""
    _, grads = synth.spiked_gradients(seed=0, m=256, n=256, steps=12, noise_std=0.1)
    W0 = np.zeros((256, 256), dtype=np.float32)
    sb = harness.SideBySide([W0], freq=5, lr=1e-3)
    for t, g in enumerate(grads, 1):
        sb.step([g])
        e = rel_err(sb.gpu_weights(0), sb.W_ref[0])
        assert e <= TOL, f"step {t}: {e:.3e}"
    sb.compare_state(TOL)


@pytest.mark.parametrize("math", [0, 2])
@pytest.mark.parametrize("weight_decay", [0.0, 0.1])
def test_every_step_update_read_directly(harness, math, weight_decay):
    """The update of EVERY step read directly, at the bare 1e-4: the weights (the caller's memory) are set to zero
    before each step on both sides, so what the step leaves in them is -lr * Q_L X Q_R^T itself, with nothing of
    the weights' own magnitude in the comparison (no storage floor).  Config 1's gradients, 20 steps, refresh every 5;
    two matrices so that a ragged one runs too.  (Decoupled decay acts on the pre-step weights, here zero, so the result
    must not depend on it.)"""
    _, g0 = synth.spiked_gradients(seed=0, m=256, n=256, steps=20, noise_std=0.1)
    _, g1 = synth.spiked_gradients(seed=1, m=200, n=136, steps=20, noise_std=0.1)
    sb = harness.SideBySide([np.zeros((256, 256), np.float32), np.zeros((200, 136), np.float32)], freq=5, lr=1e-3,
                            math=math, weight_decay=weight_decay)
    worst = 0.0
    for t in range(20):
        for i in range(2):
            sb.params[i].zero_()
            sb.W_ref[i] = np.zeros_like(sb.W_ref[i])
        sb.step([g0[t], g1[t]])
        for i in range(2):
            ref_update = -sb.W_ref[i] / sb.lr                      # the oracle's Q_L X Q_R^T of this step
            assert np.abs(ref_update - sb.states[i].last["dW"]).max() <= 1e-12 * np.abs(ref_update).max()
            e = rel_err(harness.to_np(sb.params[i]), sb.W_ref[i])
            worst = max(worst, e)
            assert e <= TOL, f"step {t + 1} matrix {i}: update rel err {e:.3e}"
    print(f"math {math}: worst per-step update error, read directly: {worst:.2e}")
    sb.compare_state(TOL, check_q=True)


@pytest.mark.parametrize("shape", [(200, 136), (136, 200), (37, 53), (1, 1), (257, 129)])
def test_ragged_shapes_bilateral(harness, shape):
    m, n = shape
    W0, grads = synth.spiked_gradients(seed=7, m=m, n=n, steps=7, noise_std=0.1)
    _run(harness, [W0], [[g] for g in grads], freq=3, lr=1e-3)


@pytest.mark.parametrize("shape", [(1, 40), (40, 1), (130, 3)])
def test_rank_deficient_statistics(harness, shape):
    """When G G^T cannot reach full rank before the refresh, the QR of L Q is rank deficient: the
    basis vectors spanning the null space are not unique (any orthonormal completion is a valid
    QR), so the bases themselves are not compared.  The update at the refresh step is still
    unique, because the rotated first moment vanishes along those vectors.  Refresh on the last
    step; compare every update, M, S, L, R, and require an orthogonal basis."""
    m, n = shape
    W0, grads = synth.spiked_gradients(seed=7, m=m, n=n, steps=5, noise_std=0.1)
    _run(harness, [W0], [[g] for g in grads], freq=5, lr=1e-3, check_q=False)


@pytest.mark.parametrize("shape", [(96, 200), (200, 96), (64, 64)])
def test_unilateral_rotates_smaller_side(harness, shape):
    m, n = shape
    W0, grads = synth.spiked_gradients(seed=8, m=m, n=n, steps=7, noise_std=0.1)
    sb, _ = _run(harness, [W0], [[g] for g in grads], freq=3, lr=1e-3, geometry=1)
    B = sb.B
    assert sb.opt.has_state(0, B.BR_STATE_QL) == (m <= n)
    assert sb.opt.has_state(0, B.BR_STATE_QR) == (m > n)
    assert sb.opt.has_state(0, B.BR_STATE_L) == (m <= n)


def test_batched_mixed_shapes_and_unrotated_tensor(harness):
    shapes = [(160, 160), (160, 288), (288, 160), (160, 160), (160, 288), (500, 64)]
    rotate = [True, True, True, True, True, False]
    rng = np.random.default_rng(3)
    W0s, seqs = [], []
    for k, (m, n) in enumerate(shapes):
        W0, grads = synth.lowrank_gradients(seed=20 + k, m=m, n=n, steps=6, rank=16, sigma=0.01)
        W0s.append(W0)
        seqs.append(grads)
    steps = [[seqs[k][t] for k in range(len(shapes))] for t in range(6)]
    _run(harness, W0s, steps, freq=4, lr=1e-3, rotate=rotate, weight_decay=0.01)


def test_more_matrices_than_one_launch_batch(harness):
    """40 same-shape matrices: three step chunks and two refresh chunks."""
    W0s, seqs = [], []
    for k in range(40):
        W0, grads = synth.spiked_gradients(seed=100 + k, m=48, n=40, steps=3, noise_std=0.1)
        W0s.append(W0)
        seqs.append(grads)
    steps = [[seqs[k][t] for k in range(40)] for t in range(3)]
    _run(harness, W0s, steps, freq=2, lr=1e-3)


def test_fixed_injected_basis_matches_rotated_adam(harness):
    """Fixed-rotation equivalence appendix: overwrite Q_L, Q_R with Haar matrices and never
    refresh; the oracle gets the same bases."""
    m, n = 136, 72
    rng = np.random.default_rng(5)
    A, Bm = synth.haar_orthogonal(rng, m), synth.haar_orthogonal(rng, n)
    W0, grads = synth.spiked_gradients(seed=9, m=m, n=n, steps=5, noise_std=0.1)
    sb = harness.SideBySide([W0], freq=0, lr=1e-2)
    A32, B32 = A.astype(np.float32), Bm.astype(np.float32)
    sb.opt.state(0, sb.B.BR_STATE_QL).copy_(torch.from_numpy(A32))
    sb.opt.state(0, sb.B.BR_STATE_QR).copy_(torch.from_numpy(B32))
    sb.B.br_notify_state_written(sb.opt.ctx)
    sb.states[0].QL, sb.states[0].QR = A32.astype(np.float64), B32.astype(np.float64)
    w0 = sb.W_ref[0].copy()
    for g in grads:
        sb.step([g])
    assert rel_err(sb.gpu_weights(0) - w0, sb.W_ref[0] - w0) <= TOL
    sb.compare_state(TOL)


def test_injected_basis_midway_rebuilds_cached_rotated_moment(harness):
    """Overwrite the bases after a few steps (M is non-zero by then): with the cache on, the
    rotated first moment must be rebuilt from M, not advanced from its stale value."""
    m, n = 72, 136
    rng = np.random.default_rng(6)
    A32 = synth.haar_orthogonal(rng, m).astype(np.float32)
    B32 = synth.haar_orthogonal(rng, n).astype(np.float32)
    W0, grads = synth.spiked_gradients(seed=10, m=m, n=n, steps=6, noise_std=0.1)
    sb = harness.SideBySide([W0], freq=0, lr=1e-2, cache_rotated_moment=1)
    w0 = sb.W_ref[0].copy()
    for t, g in enumerate(grads, 1):
        if t == 4:
            sb.opt.state(0, sb.B.BR_STATE_QL).copy_(torch.from_numpy(A32))
            sb.opt.state(0, sb.B.BR_STATE_QR).copy_(torch.from_numpy(B32))
            sb.B.br_notify_state_written(sb.opt.ctx)
            sb.states[0].QL, sb.states[0].QR = A32.astype(np.float64), B32.astype(np.float64)
        sb.step([g])
    assert rel_err(sb.gpu_weights(0) - w0, sb.W_ref[0] - w0) <= TOL + _storage_floor(sb.W_ref[0], sb.W_ref[0] - w0)
    sb.compare_state(TOL)
    mrot = harness.to_np(sb.opt.state(0, sb.B.BR_STATE_MROT))
    assert rel_err(mrot, sb.states[0].last["M_rot"]) <= TOL


@pytest.mark.parametrize("geometry", [0, 1])
def test_cached_and_recomputed_rotated_moment_agree(harness, geometry):
    """M~ advanced by its own EMA between refreshes (cache on) equals M~ rotated from M every
    step (cache off, Algorithm 1's rotation of M as printed) up to FP32 rounding; both match the oracle."""
    W0, grads = synth.spiked_gradients(seed=15, m=104, n=168, steps=9, noise_std=0.1)
    out = []
    for cache in (0, 1):
        sb, _ = _run(harness, [W0], [[g] for g in grads], freq=4, lr=1e-3, geometry=geometry,
                     cache_rotated_moment=cache)
        assert sb.opt.has_state(0, sb.B.BR_STATE_MROT) == bool(cache)
        out.append(sb.gpu_weights(0))
    w0 = np.asarray(W0, dtype=np.float64)
    assert rel_err(out[0] - w0, out[1] - w0) <= 2e-5 + _storage_floor(out[1], out[1] - w0)


def test_textbook_flags_power_iters_and_stat_beta(harness):
    # two multiplications square the condition number of L Q; 4 x 64 = 256 samples keep the
    # 80 x 80 factor at a condition number of about a dozen, so FP32 resolves the basis to 1e-4
    W0, grads = synth.spiked_gradients(seed=11, m=64, n=80, steps=8, noise_std=0.1)
    _run(harness, [W0], [[g] for g in grads], freq=4, lr=1e-3, bias_correction=1, eps_outside_sqrt=1,
         power_iters=2, stat_beta=0.9, eps=1e-6, beta1=0.8, beta2=0.99)


@pytest.mark.parametrize("math", [0, 2, 1])
@pytest.mark.parametrize("cache", [1, 0])
def test_textbook_flags_on_interior_tiles(harness, math, cache):
    """Bias correction, eps outside the root, weight decay, with and without the cached rotated moment, at a shape
    whose tiles lie partly wholly inside the matrix (300 x 520: the epilogues' paths without bounds tests and the
    general ones side by side), in every math mode."""
    W0, grads = synth.spiked_gradients(seed=13, m=300, n=520, steps=9, noise_std=0.1)
    _run(harness, [W0], [[g] for g in grads], freq=5, lr=1e-3, bias_correction=1, eps_outside_sqrt=1, eps=1e-6,
         weight_decay=0.01, cache_rotated_moment=cache, math=math, tol=2e-2 if math == 1 else TOL, check_q=(math != 1))


@pytest.mark.parametrize("shape", [(48, 200), (200, 48)])
def test_first_moment_source_unilateral(harness, shape):
    """First-order source (Algorithm 2, first-order branch): Power(M M^T, U) with no L/R buffers.  A wide
    noisy M keeps M M^T well conditioned, so the bases are compared directly."""
    m, n = shape
    W0, grads = synth.lowrank_gradients(seed=12, m=m, n=n, steps=6, rank=8, sigma=0.05)
    sb, _ = _run(harness, [W0], [[g] for g in grads], freq=2, lr=1e-3, source=1, geometry=1)
    assert not sb.opt.has_state(0, sb.B.BR_STATE_L) and not sb.opt.has_state(0, sb.B.BR_STATE_R)


def test_first_moment_source_bilateral_square(harness):
    """Square M: cond(M M^T) = cond(M)^2 is large, so the trailing basis vectors are resolved
    only to cond * 2^-24 in FP32 and are not compared; updates, M, S and orthogonality are."""
    W0, grads = synth.lowrank_gradients(seed=12, m=64, n=64, steps=6, rank=64, sigma=0.05)
    _run(harness, [W0], [[g] for g in grads], freq=2, lr=1e-3, source=1, check_q=False)


def test_bf16_params_and_grads_hidden_256_layer(harness):
    """Transformer-layer matrices shrunk to hidden 256 (Q/K/V/O 256^2, gate/up 256 x 704, down
    704 x 256), BF16 parameters and gradients, FP32 master and state, refresh every 10 steps."""
    shapes = [(256, 256)] * 4 + [(256, 704)] * 2 + [(704, 256)]
    W0s, seqs = [], []
    for k, (m, n) in enumerate(shapes):
        W0, grads = synth.lowrank_gradients(seed=2 * 1000 + k, m=m, n=n, steps=12, rank=64, sigma=0.01, bf16=True)
        W0s.append(W0)
        seqs.append(grads)
    steps = [[seqs[k][t] for k in range(len(shapes))] for t in range(12)]
    sb, _ = _run(harness, W0s, steps, freq=10, lr=1e-3, bf16_params=True, bf16_grads=True)
    # the BF16 parameter is the RNE image of the master copy: bit-exact against the GPU's own
    # master, and within one BF16 ulp of the oracle's image
    for i in range(len(shapes)):
        master = sb.opt.state(i, sb.B.BR_STATE_MASTER)
        assert torch.equal(master.to(torch.bfloat16), sb.params[i])
        ref = oc.bf16_round(sb.W_ref[i])
        got = harness.to_np(sb.params[i])
        assert np.abs(got - ref).max() <= 2.0 ** -7 * np.abs(ref).max()
        assert (got != ref).mean() < 0.01


def test_norms_option(harness):
    W0, grads = synth.spiked_gradients(seed=13, m=120, n=88, steps=3, noise_std=0.1)
    sb = harness.SideBySide([W0], freq=2, lr=1e-3, compute_norms=1)
    for g in grads:
        sb.step([g])
    norms = harness.to_np(sb.opt.state(0, sb.B.BR_STATE_NORMS))[0]
    last = sb.states[0].last
    assert abs(norms[0] - np.sum(last["G_rot"] ** 2)) <= 1e-4 * np.sum(last["G_rot"] ** 2)
    assert abs(norms[1] - np.sum(last["X"] ** 2)) <= 1e-4 * np.sum(last["X"] ** 2)
    # rotation preserves the Frobenius norm of the gradient
    assert abs(norms[0] - np.sum(np.asarray(grads[-1], dtype=np.float64) ** 2)) <= 1e-4 * norms[0]


def test_run_to_run_determinism_and_checkpoint_resume(harness):
    W0, grads = synth.spiked_gradients(seed=14, m=96, n=160, steps=8, noise_std=0.1)

    def run(n_steps, resume_from=None):
        sb = harness.SideBySide([W0], freq=3, lr=1e-3)
        if resume_from is not None:
            ws, w, t = resume_from
            sb.opt.workspace[:sb.opt.state_bytes].copy_(ws)
            sb.params[0].copy_(w)
            sb.B.br_set_step_count(sb.opt.ctx, t)
            start = t
        else:
            start = 0
        for g in grads[start:n_steps]:
            sb.opt.step([harness.to_dev(g)])
        torch.cuda.synchronize()
        return sb

    a, b = run(8), run(8)
    assert torch.equal(a.params[0], b.params[0])
    assert torch.equal(a.opt.workspace[:a.opt.state_bytes], b.opt.workspace[:b.opt.state_bytes])
    half = run(4)
    snap = (half.opt.workspace[:half.opt.state_bytes].clone(), half.params[0].clone(), 4)
    c = run(8, resume_from=snap)
    assert torch.equal(a.params[0], c.params[0])
    assert torch.equal(a.opt.workspace[:a.opt.state_bytes], c.opt.workspace[:c.opt.state_bytes])


def test_error_paths_leave_kernels_unlaunched(harness):
    from paper_2602_03515_amd import binding as B
    W = torch.zeros(8, 8, device="cuda")
    from paper_2602_03515_amd.optimizer import BasisRotationAdam
    opt = BasisRotationAdam([W], freq=2)
    g = torch.ones(8, 8, device="cuda")
    with pytest.raises(B.BrError) as e:
        B.br_step(opt.ctx, [W.data_ptr()], [g.data_ptr()], 1e-3)          # no statistics yet
    assert e.value.status == B.BR_ERR_STATE
    with pytest.raises(B.BrError) as e:
        B.br_accumulate_stats(opt.ctx, [g.data_ptr(), g.data_ptr()])      # wrong count
    assert e.value.status == B.BR_ERR_SHAPE
    with pytest.raises(B.BrError) as e:
        B.br_accumulate_stats(opt.ctx, [0])                               # null gradient
    assert e.value.status == B.BR_ERR_INVALID_ARG
    with pytest.raises(B.BrError) as e:
        B.br_accumulate_stats(opt.ctx, [g.data_ptr() + 4])                # misaligned
    assert e.value.status == B.BR_ERR_INVALID_ARG
    B.br_accumulate_stats(opt.ctx, [g.data_ptr()])
    with pytest.raises(B.BrError) as e:
        B.br_accumulate_stats(opt.ctx, [g.data_ptr()])                    # twice
    assert e.value.status == B.BR_ERR_STATE
    with pytest.raises(B.BrError):
        B.br_get_state(opt.ctx, 3, B.BR_STATE_M)
    B.br_step(opt.ctx, [W.data_ptr()], [g.data_ptr()], 1e-3)
    torch.cuda.synchronize()
    assert torch.isfinite(W).all() and opt.step_count == 1


@pytest.mark.parametrize("bf16", [False, True])
def test_global_norm_clipping(harness, bf16):
    """Clipping before the step: norm and factor against the oracle, gradients rescaled in place,
    and the clipped trajectory follows the oracle fed with the oracle's clipped gradients."""
    shapes = [(96, 64), (64, 96), (33, 17), (96, 64)]
    W0s, seqs = [], []
    for k, (m, n) in enumerate(shapes):
        W0, grads = synth.spiked_gradients(seed=300 + k, m=m, n=n, steps=3, noise_std=0.1)
        if bf16:
            W0, grads = synth.to_bf16_f32(W0), [synth.to_bf16_f32(g) for g in grads]
        W0s.append(W0)
        seqs.append(grads)
    sb = harness.SideBySide(W0s, freq=2, lr=1e-3, bf16_params=bf16, bf16_grads=bf16)
    for t in range(3):
        host = [seqs[k][t] for k in range(len(shapes))]
        max_norm = 1.0 if t < 2 else 1e4                       # last step: nothing to clip
        ref, norm, factor = oc.clip_by_global_norm(host, max_norm)
        if bf16:
            ref = [oc.bf16_round(r) for r in ref]
        dev = [harness.to_dev(g, bf16) for g in host]
        sb.opt.clip_gradients(dev, max_norm)
        res = harness.to_np(sb.opt.clip_result())
        assert abs(res[0] - norm) <= 1e-5 * norm and abs(res[1] - factor) <= 1e-5
        for d, r, h0 in zip(dev, ref, host):
            got = harness.to_np(d)
            if t == 2:
                assert np.array_equal(got, np.asarray(h0, dtype=np.float64))   # factor 1: untouched
            elif bf16:
                assert np.abs(got - r).max() <= 2.0 ** -7 * np.abs(r).max() and (got != r).mean() < 0.01
            else:
                assert rel_err(got, r) <= 1e-6
        sb.opt.step(dev, sb.lr)
        torch.cuda.synchronize()
        for i, st in enumerate(sb.states):
            sb.W_ref[i] = oc.optimizer_step(st, sb.W_ref[i], harness.to_np(dev[i]), sb.lr, sb.hp, sb.freq, sb.qr)
    sb.compare_state(TOL)


@pytest.mark.parametrize("geometry", [0, 1])
@pytest.mark.parametrize("shape", [(256, 384), (200, 136), (136, 200), (37, 53)])
def test_bf16x3_math_mode_keeps_the_fp32_bar(harness, shape, geometry):
    """BR_MATH_BF16X3: the step's contractions run on BF16 matrix cores with operands split into
    hi + lo BF16 planes (three products); the 1e-4 bar of the FP32 path applies unchanged."""
    m, n = shape
    W0, grads = synth.spiked_gradients(seed=21, m=m, n=n, steps=7, noise_std=0.1)
    sb, worst = _run(harness, [W0], [[g] for g in grads], freq=3, lr=1e-3, geometry=geometry, math=2)
    print("bf16x3 worst:", {k: f"{v:.2e}" for k, v in worst.items()})


def test_bf16x3_layer_bf16_params_and_cache_off(harness):
    shapes = [(256, 256)] * 2 + [(256, 704), (704, 256)]
    W0s, seqs = [], []
    for k, (m, n) in enumerate(shapes):
        W0, grads = synth.lowrank_gradients(seed=4000 + k, m=m, n=n, steps=6, rank=64, sigma=0.01, bf16=True)
        W0s.append(W0)
        seqs.append(grads)
    steps = [[seqs[k][t] for k in range(len(shapes))] for t in range(6)]
    _run(harness, W0s, steps, freq=4, lr=1e-3, bf16_params=True, bf16_grads=True, math=2, weight_decay=0.01)
    _run(harness, W0s, steps, freq=4, lr=1e-3, bf16_params=True, bf16_grads=True, math=2, cache_rotated_moment=0)


@pytest.mark.parametrize("geometry", [0, 1])
def test_bf16_math_mode_meets_the_2e2_bar(harness, geometry):
    """BR_MATH_BF16: plain BF16 inputs to the matrix cores.  Updates, weights and the moments are
    held to 2e-2; the bases come out of an FP32 QR of statistics that are themselves only BF16
    accurate, so they are checked for orthogonality, not compared entry by entry."""
    W0, grads = synth.spiked_gradients(seed=22, m=192, n=320, steps=8, noise_std=0.1)
    sb, worst = _run(harness, [W0], [[g] for g in grads], freq=4, lr=1e-3, geometry=geometry, math=1, tol=2e-2,
                     check_q=False)
    print("bf16 worst:", {k: f"{v:.2e}" for k, v in worst.items()})


@pytest.mark.parametrize("math", [1, 2])
@pytest.mark.parametrize("shape", [(1, 1), (1, 40), (40, 1), (130, 3)])
def test_degenerate_shapes_in_the_bf16_modes(harness, shape, math):
    """Single rows, single columns and a 1 x 1 matrix through the operand planes (padded to 256 rows and
    64 k): statistics that cannot reach full rank, so the bases are checked for orthogonality only
    (any orthonormal completion of the null space is a valid QR) while every update, the moments and the
    statistics are compared, at the bar of the math mode."""
    m, n = shape
    W0, grads = synth.spiked_gradients(seed=7, m=m, n=n, steps=5, noise_std=0.1)
    _run(harness, [W0], [[g] for g in grads], freq=5, lr=1e-3, check_q=False, math=math, tol=2e-2 if math == 1 else TOL)


def _lapack_qr(P):
    q, r = np.linalg.qr(P)
    d = np.where(np.diag(r) < 0, -1.0, 1.0)
    return q * d[None, :], r * d[:, None]


@pytest.mark.parametrize("math,refresh_math", [(0, 0), (0, 2), (1, 0), (2, 0), (2, 1)])
def test_refresh_alone_on_injected_statistics_several_top_blocks(harness, math, refresh_math):
    """The refresh by itself at orders with three and two ragged top blocks of the QR (1100 and 600
    columns): well-conditioned statistics (Wishart, aspect 3, condition number 14) are written into
    the state, br_refresh_basis runs from Q = I and once more from its own result, and both bases
    are compared entry by entry with the oracle's (float64; LAPACK's QR with the same sign
    convention, pinned against the oracle's own Householder loop in the CPU tests, which would take
    a minute here).  Injecting the statistics keeps the comparison about the refresh: in the BF16
    math mode the statistics themselves are only BF16 accurate, and a young second moment turns
    that into O(1) differences of single update entries on a matrix this large.
    Above order 512 the product A Q and the QR's large updates are either FP32 (refresh_math 1, and the default of
    BR_MATH_F32) or split FP16 products (hi + lo FP16 operands, 22 mantissa bits, FP32 accumulation: refresh_math 2,
    and the default of the BF16 math modes).  Bars: 1e-5 on the entries and on orthogonality for both."""
    m, n = 1100, 600
    rng = np.random.default_rng(77)

    def wishart(k):
        A = rng.standard_normal((k, 3 * k))
        return (A @ A.T / (3 * k)).astype(np.float32)

    L32, R32 = wishart(m), wishart(n)
    W0 = rng.standard_normal((m, n)).astype(np.float32)
    sb = harness.SideBySide([W0], freq=0, lr=1e-3, math=math, refresh_math=refresh_math)
    B, st = sb.B, sb.states[0]
    sb.opt.state(0, B.BR_STATE_L).copy_(torch.from_numpy(L32))
    sb.opt.state(0, B.BR_STATE_R).copy_(torch.from_numpy(R32))
    B.br_notify_state_written(sb.opt.ctx)
    st.L, st.R = L32.astype(np.float64), R32.astype(np.float64)
    bar, orth = 1e-5, 1e-5
    for rep in range(2):
        B.br_refresh_basis(sb.opt.ctx)
        torch.cuda.synchronize()
        oc.refresh(st, sb.hp, _lapack_qr)
        for kind, Q in ((B.BR_STATE_QL, st.QL), (B.BR_STATE_QR, st.QR)):
            q = harness.to_np(sb.opt.state(0, kind))
            e, d = rel_err(q, Q), orthogonality_defect(q)
            print(f"math {math} refresh_math {refresh_math} refresh {rep} order {q.shape[0]}: basis rel err {e:.2e}, "
                  f"orthogonality defect {d:.2e}")
            assert d < orth
            assert e <= bar, f"refresh {rep}, state {kind}: basis rel err {e:.3e} > {bar:.1e}"


@pytest.mark.parametrize("math", [1, 2])
def test_bf16_modes_injected_basis_midway(harness, math):
    """BF16 math modes keep operand planes of the bases between steps; overwriting the bases
    (br_notify_state_written) must rebuild them, and the cached rotated first moment with them."""
    m, n = 200, 328
    rng = np.random.default_rng(16)
    A32 = synth.haar_orthogonal(rng, m).astype(np.float32)
    B32 = synth.haar_orthogonal(rng, n).astype(np.float32)
    W0, grads = synth.spiked_gradients(seed=31, m=m, n=n, steps=6, noise_std=0.1)
    tol = TOL if math == 2 else 2e-2
    sb = harness.SideBySide([W0], freq=0, lr=1e-2, math=math)
    w0 = sb.W_ref[0].copy()
    for t, g in enumerate(grads, 1):
        if t == 4:
            sb.opt.state(0, sb.B.BR_STATE_QL).copy_(torch.from_numpy(A32))
            sb.opt.state(0, sb.B.BR_STATE_QR).copy_(torch.from_numpy(B32))
            sb.B.br_notify_state_written(sb.opt.ctx)
            sb.states[0].QL, sb.states[0].QR = A32.astype(np.float64), B32.astype(np.float64)
        sb.step([g])
    assert rel_err(sb.gpu_weights(0) - w0, sb.W_ref[0] - w0) <= tol + _storage_floor(sb.W_ref[0], sb.W_ref[0] - w0)
    sb.compare_state(tol)


@pytest.mark.parametrize("math", [0, 2, 1])
@pytest.mark.parametrize("shape", [(640, 300), (300, 640)])
def test_unilateral_with_interior_tiles(harness, shape, math):
    """Unilateral rotation (right factor for the tall matrix, left factor for the wide one) at shapes whose 256 x 256
    tiles lie partly wholly inside the matrices, with refreshes, in every math mode."""
    m, n = shape
    W0, grads = synth.spiked_gradients(seed=35, m=m, n=n, steps=8, noise_std=0.1)
    _run(harness, [W0], [[g] for g in grads], freq=4, lr=1e-3, geometry=1, math=math, weight_decay=0.01,
         tol=2e-2 if math == 1 else TOL, check_q=(math != 1))


@pytest.mark.parametrize("math", [1, 2])
def test_bf16_modes_right_factor_only_chain(harness, math):
    """Unilateral rotation of a tall matrix rotates the right side only.  In the BF16 modes that chain
    takes its first contraction transposed (Adam's moments are indexed [col][row] in its epilogue);
    a basis injected midway also forces the cached rotated moment to be rebuilt as M Q_R."""
    m, n = 328, 200
    rng = np.random.default_rng(17)
    B32 = synth.haar_orthogonal(rng, n).astype(np.float32)
    W0, grads = synth.spiked_gradients(seed=34, m=m, n=n, steps=7, noise_std=0.1)
    tol = TOL if math == 2 else 2e-2
    sb = harness.SideBySide([W0], freq=0, lr=1e-2, math=math, geometry=1)
    w0 = sb.W_ref[0].copy()
    for t, g in enumerate(grads, 1):
        if t == 4:
            sb.opt.state(0, sb.B.BR_STATE_QR).copy_(torch.from_numpy(B32))
            sb.B.br_notify_state_written(sb.opt.ctx)
            sb.states[0].QR = B32.astype(np.float64)
        sb.step([g])
    assert rel_err(sb.gpu_weights(0) - w0, sb.W_ref[0] - w0) <= tol + _storage_floor(sb.W_ref[0], sb.W_ref[0] - w0)
    sb.compare_state(tol)
    # and with the refresh running: tall and ragged
    W0, grads = synth.spiked_gradients(seed=35, m=300, n=136, steps=8, noise_std=0.1)
    _run(harness, [W0], [[g] for g in grads], freq=3, lr=1e-3, geometry=1, math=math, tol=tol, check_q=(math == 2))


@pytest.mark.parametrize("math", [2, 0])
@pytest.mark.parametrize("geometry", [0, 1])
def test_bf16x3_fused_and_unfused_chains_agree(harness, geometry, math):
    """With per-matrix norms requested every product is stored in FP32 and Adam's update is a kernel
    of its own (the BF16 modes also split the stored products again); without, Adam runs in the
    epilogue of the contraction that produces the rotated gradient (math = 0: the FP32 kernel stores X
    instead of G~; BF16 modes: products travel as operand planes).  Same result, both against the
    oracle at 1e-4 and against each other."""
    shapes = [(264, 136), (136, 264), (200, 200)]
    W0s, seqs = [], []
    for k, (m, n) in enumerate(shapes):
        W0, grads = synth.spiked_gradients(seed=40 + k, m=m, n=n, steps=7, noise_std=0.1)
        W0s.append(W0)
        seqs.append(grads)
    steps = [[seqs[k][t] for k in range(len(shapes))] for t in range(7)]
    out = []
    for norms in (0, 1):
        sb, _ = _run(harness, W0s, steps, freq=3, lr=1e-3, geometry=geometry, math=math, compute_norms=norms)
        out.append([sb.gpu_weights(i) for i in range(len(shapes))])
    for i, W0 in enumerate(W0s):
        w0 = np.asarray(W0, dtype=np.float64)
        assert rel_err(out[0][i] - w0, out[1][i] - w0) <= 2e-5 + _storage_floor(out[1][i], out[1][i] - w0)


def test_bf16x3_first_moment_source(harness):
    W0, grads = synth.spiked_gradients(seed=33, m=136, n=264, steps=6, noise_std=0.1)
    _run(harness, [W0], [[g] for g in grads], freq=3, lr=1e-3, geometry=1, math=2, source=1)


@pytest.mark.parametrize("bf16", [False, True])
def test_delay_compensation(harness, bf16):
    """G <- G + lambda G.G.(W_now - W_stale) on the device against the oracle, ragged sizes included."""
    shapes = [(96, 64), (33, 17), (5, 3), (257, 129)]
    rng = np.random.default_rng(77)
    W0s = [rng.standard_normal(s) for s in shapes]
    stale = [w + 0.05 * rng.standard_normal(w.shape) for w in W0s]
    grads = [rng.standard_normal(s) for s in shapes]
    if bf16:
        W0s, stale, grads = ([synth.to_bf16_f32(a) for a in x] for x in (W0s, stale, grads))
    sb = harness.SideBySide(W0s, freq=0, lr=1e-3, bf16_params=bf16, bf16_grads=bf16)
    dev_g = [harness.to_dev(g, bf16) for g in grads]
    dev_s = [harness.to_dev(w, bf16) for w in stale]
    lam = 0.5
    sb.opt.delay_compensate(dev_g, dev_s, lam)
    torch.cuda.synchronize()
    for d, g, w, ws in zip(dev_g, grads, W0s, stale):
        ref = oc.delay_compensate(g, w, ws, np.float32(lam))
        got = harness.to_np(d)
        if bf16:
            r = oc.bf16_round(ref)
            assert np.abs(got - r).max() <= 2.0 ** -7 * np.abs(r).max() and (got != r).mean() < 0.01
        else:
            assert rel_err(got, ref) <= 1e-6
    with pytest.raises(Exception):
        sb.opt.delay_compensate(dev_g, dev_s, 1.5)


@pytest.mark.parametrize("math,geometry,cache", [(0, 0, 1), (0, 1, 1), (0, 1, 0), (2, 1, 1), (2, 1, 0)])
def test_statistics_only_on_refresh_steps(harness, math, geometry, cache):
    """Algorithm 2 exactly as Algorithm 1 calls it: L and R are updated inside Eigenbasis-Estimation, i.e. only
    from the gradients of refresh steps (stats_on_refresh_only), against the oracle's flag of the same name.
    Several matrices in two shapes plus an unrotated tensor, refresh every 3 of 8 steps.  At the first refresh the
    statistics hold ONE gradient, so a factor is full rank only on a side no longer than the other: the bilateral
    case takes square matrices, the unilateral one (smaller side) rectangular ones.  The Gram matrix of ONE square
    noisy gradient is ill-conditioned (condition number 1e4 and more), so in the bilateral case the bases are held
    to orthogonality and to what they produce (every update, moments, statistics at the bar), not entry by entry, and
    only the FP32 mode runs it (the split-BF16 modes' bars assume condition numbers of about 100 at most).  Plain
    BF16 inputs are left out: with a first rotation on a two-step-old second moment that mode's 2e-2 does not hold
    (3.6e-2 here at step 3), as its documentation says; the deferred statistics of that mode share every launch
    with BR_MATH_BF16X3."""
    shapes = [(96, 96), (160, 160), (96, 96), (300, 48)] if geometry == 0 else [(136, 200), (200, 136), (136, 200), (300, 48)]
    rotate = [True, True, True, False]
    W0s, seqs = [], []
    for k, (m, n) in enumerate(shapes):
        W0, grads = synth.spiked_gradients(seed=70 + k, m=m, n=n, steps=8, noise_std=0.1)
        W0s.append(W0)
        seqs.append(grads)
    steps = [[seqs[k][t] for k in range(len(shapes))] for t in range(8)]
    tol = 2e-2 if math == 1 else TOL
    sb, _ = _run(harness, W0s, steps, freq=3, lr=1e-3, tol=tol, check_q=(math != 1 and geometry == 1), rotate=rotate,
                 math=math, geometry=geometry, cache_rotated_moment=cache, stats_on_refresh_only=1)
    # the flag did something: the statistics hold exactly two gradients' worth (steps 3 and 6)
    st = sb.states[0]
    b = sb.hp.beta2
    G3, G6 = np.asarray(seqs[0][2], dtype=np.float64), np.asarray(seqs[0][5], dtype=np.float64)
    assert rel_err(st.L, (1 - b) * (G6 @ G6.T) + b * (1 - b) * (G3 @ G3.T)) < 1e-12


def test_statistics_only_on_refresh_steps_bf16_gradients(harness):
    """BF16 gradients: the deferred statistics widen them again at the refresh (unilateral: well conditioned)."""
    shapes = [(136, 200), (200, 136)]
    W0s, seqs = [], []
    for k, (m, n) in enumerate(shapes):
        W0, grads = synth.lowrank_gradients(seed=80 + k, m=m, n=n, steps=7, rank=16, sigma=0.05, bf16=True)
        W0s.append(W0)
        seqs.append(grads)
    steps = [[seqs[k][t] for k in range(len(shapes))] for t in range(7)]
    _run(harness, W0s, steps, freq=3, lr=1e-3, bf16_params=True, bf16_grads=True, geometry=1, stats_on_refresh_only=1)


def test_health_words_qr_wait_given_up_keeps_previous_basis(harness):
    """The failure path of the QR panel clusters, forced from the host: with a wait limit of 0 every exchange
    between the workgroups of a cluster gives up at once (all kernels still end normally).  The left factor of
    a 2000 x 40 matrix (order 2000: panels of two workgroups) must then keep the basis it had before that
    refresh, bit for bit; the right factor (order 40, one workgroup, no exchange) is refreshed as usual; the
    weights stay finite; the health word counts the event and br_check_health reports it.  Statistics are
    injected (well conditioned, full rank) so that every basis is unique and can be checked against the oracle's
    Power step."""
    from paper_2602_03515_amd import binding as B
    from paper_2602_03515_amd.optimizer import BasisRotationAdam
    from tests.tolerances import lapack_qr
    m, n = 2000, 40
    rng = np.random.default_rng(91)

    def spd(k, seed_shift):
        N = np.random.default_rng(910 + seed_shift).standard_normal((k, k))
        return (N + N.T) * (0.3 / (2.0 * np.sqrt(k))) + 2.0 * np.eye(k)

    L1, L2, R1, R2 = spd(m, 1), spd(m, 2), spd(n, 3), spd(n, 4)
    W = harness.to_dev(0.02 * rng.standard_normal((m, n)))
    opt = BasisRotationAdam([W], freq=0, lr=1e-3)

    def inject(L, R):
        opt.state(0, B.BR_STATE_L).copy_(harness.to_dev(L))
        opt.state(0, B.BR_STATE_R).copy_(harness.to_dev(R))
        B.br_notify_state_written(opt.ctx)

    inject(L1, R1)
    opt.refresh_basis()                                     # a normal refresh
    torch.cuda.synchronize()
    assert B.br_check_health(opt.ctx) == [0, 0, 0, 0]
    ql1, qr1 = opt.state(0, B.BR_STATE_QL).clone(), opt.state(0, B.BR_STATE_QR).clone()
    assert rel_err(harness.to_np(ql1), oc.power_qr(L1, np.eye(m), 1, lapack_qr)) <= 1e-5
    inject(L2, R2)
    B.br_set_qr_wait_limit(opt.ctx, 0)
    opt.refresh_basis()                                     # every cluster exchange gives up
    g = harness.to_dev(0.01 * rng.standard_normal((m, n)))
    opt.step([g], 1e-3)                                     # freq = 0: no further refresh
    torch.cuda.synchronize()
    assert torch.equal(opt.state(0, B.BR_STATE_QL), ql1)                   # previous basis kept, bit for bit
    assert rel_err(harness.to_np(opt.state(0, B.BR_STATE_QR)),             # the small factor was refreshed as usual
                   oc.power_qr(R2, harness.to_np(qr1), 1, lapack_qr)) <= 1e-5
    assert bool(torch.isfinite(W).all())
    off = B.br_get_health(opt.ctx) - opt.workspace.data_ptr()
    health = opt.workspace[off:off + 16].view(torch.int32)
    assert int(health[0]) > 0 and int(health[1]) == 0
    with pytest.raises(B.BrError) as e:
        B.br_check_health(opt.ctx)
    assert e.value.status == B.BR_ERR_STATE and "gave up" in str(e.value)
    # back to the default wait: the next refresh works again, from the basis that was kept
    B.br_set_qr_wait_limit(opt.ctx, -1)
    count_before = int(health[0])
    opt.refresh_basis()
    torch.cuda.synchronize()
    L_now = harness.to_np(opt.state(0, B.BR_STATE_L))      # L2 plus the step's gradient (the statistics went on)
    assert rel_err(harness.to_np(opt.state(0, B.BR_STATE_QL)), oc.power_qr(L_now, harness.to_np(ql1), 1, lapack_qr)) <= 1e-5
    assert int(health[0]) == count_before
    opt.close()


@pytest.mark.parametrize("shape", [(72, 40), (512, 256)])
@pytest.mark.parametrize("math", [0, 1])
def test_health_word_counts_non_finite_weights(harness, math, shape):
    """An infinite learning rate (not rejected: only NaN is) makes the stored weights non-finite; the kernels
    that store weights count it, for rotated matrices and for plain-Adam tensors; the second shape has tiles that
    lie wholly inside the matrix (the epilogues' paths without bounds tests)."""
    from paper_2602_03515_amd import binding as B
    from paper_2602_03515_amd.optimizer import BasisRotationAdam
    for rotate in (True, False):
        W = torch.ones(*shape, device="cuda")
        g = torch.ones(*shape, device="cuda")
        opt = BasisRotationAdam([W], freq=0, lr=1e-3, rotate=[rotate], math=math)
        opt.step([g], 1e-3)
        assert B.br_check_health(opt.ctx) == [0, 0, 0, 0]
        opt.step([g], float("inf"))
        with pytest.raises(B.BrError) as e:
            B.br_check_health(opt.ctx)
        assert e.value.status == B.BR_ERR_STATE and "non-finite" in str(e.value)
        assert not bool(torch.isfinite(W).all())
        opt.close()
