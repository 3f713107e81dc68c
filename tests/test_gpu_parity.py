"""GPU parity: the HIP path, called through the C-ABI, against the float64 oracle on the same
seeded inputs.

Error measure (stated with every number): per tensor, max|gpu - ref| / max|ref|.
Tolerances: fp32 mode 1e-4, bf16 mode 2e-2 on the loss, every gradient tensor and the
updated weights.  In bf16 mode the oracle is fed the bf16-rounded weights and features, so the
budget measures the arithmetic, not the input quantisation.
"""
import sys

import numpy as np
import pytest

from oracle import blstm_oracle as orc
from paper_1904_04956_amd import inputs

pytestmark = pytest.mark.gpu

TOL = {0: 1e-4, 1: 2e-2}


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def rel_err(a, ref):
    ref = np.asarray(ref, dtype=np.float64)
    den = np.abs(ref).max()
    num = np.abs(np.asarray(a, dtype=np.float64) - ref).max()
    return num / den if den > 0 else num


def make_problem(dims, mode, seed, theta_scale=1.0):
    dm = orc.Dims(**dims)
    n = orc.param_count(dm)
    bf = mode == 1
    theta = inputs.make_theta(n, seed, bf16=False) * np.float32(theta_scale)
    if bf:
        theta = inputs.round_to_bf16(theta)
    x, labels = inputs.make_batch(dm.T, dm.B, dm.D, dm.V, seed, bf16=bf)
    return dm, theta, x, labels


def check_step(dims, mode, seed, lr=0.1, theta_scale=1.0, tol=None, check_update=True, recurrent_path=0,
               recurrent_sync=None, defer_softmax_wgrad=True):
    """One full training step on the GPU against the oracle; returns the worst relative error."""
    from paper_1904_04956_amd.harness import Learner
    tol = TOL[mode] if tol is None else tol
    dm, theta, x, labels = make_problem(dims, mode, seed, theta_scale)
    say(f"case dims={dims} mode={mode} seed={seed}")
    lrn = Learner(mode=mode, recurrent_path=recurrent_path, recurrent_sync=recurrent_sync, defer_softmax_wgrad=defer_softmax_wgrad, **dims)
    try:
        lrn.set_theta(theta)
        lrn.set_batch(x, labels)
        lrn.calgrad()
        lrn.check_status()
        z_gpu = lrn.z_numpy()
        loss_gpu = lrn.loss_value()
        g_gpu = lrn.grad_numpy()
        lrn.apply(lr)
        th_gpu = lrn.theta_numpy()
        sh_gpu = lrn.shadow.float().cpu().numpy() if mode == 1 else None
    finally:
        lrn.close()
    th64 = theta.astype(np.float64)
    z_ref, _ = orc.blstm_forward(dm, th64, x)
    loss_ref, g_ref = orc.loss_and_grad(dm, th64, x, labels)
    worst = 0.0
    e = rel_err(z_gpu, z_ref); worst = max(worst, e)
    assert e <= tol, f"z: {e}"
    e = abs(loss_gpu - loss_ref) / abs(loss_ref); worst = max(worst, e)
    assert e <= tol, f"loss: gpu {loss_gpu} ref {loss_ref}"
    assert np.all(np.isfinite(g_gpu))
    for name, off, shape in orc.layout(dm):
        k = int(np.prod(shape))
        e = rel_err(g_gpu[off:off + k], g_ref[off:off + k]); worst = max(worst, e)
        assert e <= tol, f"grad {name}: {e}"
    if check_update:
        # the update itself is exact arithmetic on the GPU's own gradient: check it tightly ...
        th_exact = theta.astype(np.float64) - lr * g_gpu.astype(np.float64)
        assert rel_err(th_gpu, th_exact) <= 1e-6
        # ... and the updated weights against the oracle's step within the mode's tolerance
        th_ref, _ = orc.sgd_step(th64, g_ref, lr)
        for name, off, shape in orc.layout(dm):
            k = int(np.prod(shape))
            e = rel_err(th_gpu[off:off + k], th_ref[off:off + k]); worst = max(worst, e)
            assert e <= tol, f"theta {name}: {e}"
        if sh_gpu is not None:
            assert np.array_equal(sh_gpu, inputs.round_to_bf16(th_gpu))
    say(f"  worst relative error {worst:.3e} (tolerance {tol:g})")
    return worst


# ------------------------------------------------------------------ fp32 mode

def test_tiny_workload_fp32():
    w = inputs.WORKLOADS["tiny"]
    check_step(w.dims(), 0, w.seed, lr=w.lr)


@pytest.mark.parametrize("dims", [
    dict(T=1, B=1, D=1, H=1, L=1, P=0, V=2),                # smallest possible
    dict(T=2, B=3, D=5, H=4, L=2, P=3, V=7),                # odd everything: scalar load paths
    dict(T=5, B=37, D=40, H=32, L=2, P=24, V=100),          # M = 185: two row tiles with a ragged tail
    dict(T=3, B=130, D=36, H=96, L=2, P=0, V=300),          # 4H = 384, V = 300: several column tiles, no bottleneck
    dict(T=1, B=16, D=12, H=8, L=1, P=4, V=10),             # a single frame: no recurrent product at all
])
def test_odd_shapes_fp32(dims):
    check_step(dims, 0, seed=77, theta_scale=3.0)


def test_loss_scale_argument_fp32():
    from paper_1904_04956_amd.harness import Learner
    dims = dict(T=4, B=6, D=8, H=8, L=1, P=0, V=9)
    dm, theta, x, labels = make_problem(dims, 0, 5)
    lrn = Learner(mode=0, loss_scale=1.0 / 6, **dims)
    try:
        lrn.set_theta(theta); lrn.set_batch(x, labels); lrn.calgrad()
        loss, g = lrn.loss_value(), lrn.grad_numpy()
    finally:
        lrn.close()
    dmb = orc.Dims(loss_scale=1.0 / 6, **dims)
    lref, gref = orc.loss_and_grad(dmb, theta.astype(np.float64), x, labels)
    assert abs(loss - lref) <= 1e-4 * abs(lref)
    assert rel_err(g, gref) <= 1e-4


# ------------------------------------------------------------------ bf16 mode

@pytest.mark.parametrize("dims", [
    dict(T=21, B=32, D=260, H=128, L=2, P=64, V=1000),      # the paper's feature width, K tail 260 = 4*64 + 4
    dict(T=4, B=19, D=20, H=24, L=2, P=12, V=50),           # nothing a multiple of a tile
    dict(T=3, B=5, D=7, H=6, L=1, P=0, V=11),               # odd leading dimensions: scalar load paths
    dict(T=4, B=32, D=37, H=32, L=2, P=0, V=50),            # M = 4H = 128, odd D: zero-padded copies of x and W_x, unaligned rows
    dict(T=8, B=32, D=200, H=64, L=1, P=16, V=60),          # ... D = 200 padded to 256: two tile columns of dW_x, the second ragged
    dict(T=21, B=128, D=37, H=32, L=1, P=0, V=50),          # ... with a contraction long enough for dW_x to be split along K
])
def test_shapes_bf16(dims):
    check_step(dims, 1, seed=78, theta_scale=2.0)


@pytest.mark.parametrize("V", [8000, 12000, 12004, 40000, 70000])
def test_softmax_row_widths_bf16(V):
    # one softmax row kernel per range of V (256, 512, 1024 threads per row; rows too long or too
    # ragged for the register-resident forms take the three-pass kernel)
    check_step(dict(T=2, B=5, D=8, H=8, L=1, P=8, V=V), 1, seed=80, theta_scale=4.0)


@pytest.mark.parametrize("defer", [False, True])
@pytest.mark.parametrize("dims", [
    dict(T=4, B=64, D=128, H=128, L=2, P=128, V=512),       # whole 256x128 tiles everywhere: dW_s can join the grouped launch
    dict(T=4, B=64, D=40, H=128, L=1, P=128, V=500),        # V not a whole number of tiles: dW_s runs on its own, in the backward pass
])
def test_softmax_weight_gradient_left_to_the_backward_pass(dims, defer):
    # BLSTM_OPT_DEFER_SOFTMAX_WGRAD: dW_s and db_s come out of blstm_backward's grouped launch; both settings against the oracle
    check_step(dims, 1, seed=83, theta_scale=2.0, defer_softmax_wgrad=defer)


def test_deferred_softmax_weight_gradient_call_order():
    # the gradient vector given to blstm_backward must be the one softmax_xent_fwd_bwd left its part to; a forward pass
    # in between drops what was left; the two settings agree to float rounding
    import torch
    from paper_1904_04956_amd import binding as bl
    from paper_1904_04956_amd.harness import Learner
    dims = dict(T=4, B=64, D=128, H=128, L=1, P=128, V=512)
    dm, theta, x, labels = make_problem(dims, 1, 84, 2.0)
    grads = []
    for defer in (False, True):
        lrn = Learner(mode=1, defer_softmax_wgrad=defer, **dims)
        lrn.set_theta(theta); lrn.set_batch(x, labels)
        lrn.calgrad(); lrn.check_status()
        grads.append(lrn.grad_numpy().copy())
        if defer:
            other = torch.zeros_like(lrn.grad)
            bl.blstm_forward(lrn.ctx, lrn.theta_fwd, lrn.x, lrn.z)
            bl.softmax_xent_fwd_bwd(lrn.ctx, lrn.theta_fwd, lrn.z, lrn.labels, lrn.loss, lrn.dz, lrn.grad)
            with pytest.raises(RuntimeError):
                bl.blstm_backward(lrn.ctx, lrn.theta_fwd, lrn.x, lrn.dz, other)
            # a new forward pass drops the pending product: the backward pass then takes any gradient vector and leaves
            # its W_s slice alone
            bl.blstm_forward(lrn.ctx, lrn.theta_fwd, lrn.x, lrn.z)
            bl.blstm_backward(lrn.ctx, lrn.theta_fwd, lrn.x, lrn.dz, other)
            torch.cuda.synchronize()
            off, k = next((o, int(np.prod(sh))) for name, o, sh in orc.layout(dm) if name == "Ws")
            assert float(other[off:off + k].abs().max()) == 0.0
        lrn.close()
    assert rel_err(grads[1], grads[0]) <= 1e-5


@pytest.mark.parametrize("dims", [
    dict(T=4, B=300, D=64, H=512, L=1, P=64, V=200),        # ten batch tiles over eight groups: two tiles per workgroup, some empty
    dict(T=6, B=45, D=32, H=256, L=2, P=0, V=120),          # two wavefronts per workgroup, ragged batch tile
    dict(T=2, B=64, D=16, H=128, L=1, P=16, V=40),          # one wavefront per workgroup
])
@pytest.mark.parametrize("sync", [0, 1])
def test_persistent_recurrent_kernels_bf16(dims, sync):
    check_step(dims, 1, seed=79, theta_scale=2.0, recurrent_sync=sync)


def test_exchange_protocols_agree_bit_for_bit():
    # both protocols order the same arithmetic: any stale or torn read would show as a difference
    from paper_1904_04956_amd.harness import Learner
    dims = dict(T=21, B=96, D=64, H=512, L=2, P=64, V=300)
    dm, theta, x, labels = make_problem(dims, 1, 81, 2.0)
    ref = None
    for sync in (0, 1, 1, 1):
        lrn = Learner(mode=1, recurrent_sync=sync, **dims)
        lrn.set_theta(theta); lrn.set_batch(x, labels)
        for _ in range(5):
            lrn.calgrad(); lrn.check_status()
            out = (lrn.loss_value(), lrn.grad_numpy().copy())
            if ref is None:
                ref = out
            assert out[0] == ref[0] and np.array_equal(out[1], ref[1])
        lrn.close()


def test_abandoned_wait_is_reported_in_band_and_recovered_from():
    # The abort word is raised from the host (test option), so every wait of the persistent kernels returns at
    # once and all kernels run to their end: the step's loss, z and gradient must be NaN (in-band), the status call
    # must report the failure, and the next step must give the bits of a clean run.
    from paper_1904_04956_amd import binding as bl
    from paper_1904_04956_amd.harness import Learner
    dims = dict(T=6, B=64, D=32, H=128, L=2, P=16, V=90)
    dm, theta, x, labels = make_problem(dims, 1, 83, 2.0)
    for sync in (1, 0):
        lrn = Learner(mode=1, recurrent_sync=sync, **dims)
        lrn.set_theta(theta); lrn.set_batch(x, labels)
        lrn.calgrad(); lrn.check_status()
        clean = (lrn.loss_value(), lrn.grad_numpy().copy(), lrn.z_numpy().copy())
        assert np.isfinite(clean[0]) and np.all(np.isfinite(clean[1]))
        bl.blstm_set_option(lrn.ctx, bl.BLSTM_OPT_TEST_ABORT, 1)
        lrn.calgrad()
        with pytest.raises(bl.BlstmError) as e:
            lrn.check_status()
        assert e.value.code == -5 and "abandoned" in str(e.value)
        assert np.isnan(lrn.loss_value()) and np.isnan(lrn.z_numpy()).any() and np.isnan(lrn.grad_numpy()).any()
        lrn.calgrad(); lrn.check_status()                 # recovered: the word is cleared by the next forward pass
        assert lrn.loss_value() == clean[0]
        assert np.array_equal(lrn.grad_numpy(), clean[1]) and np.array_equal(lrn.z_numpy(), clean[2])
        lrn.close()


@pytest.mark.parametrize("V,mode", [(8000, 1), (70000, 1), (300, 0)])
def test_out_of_range_label_gives_nan_loss_and_no_stray_access(V, mode):
    # a label outside [0, V) must never be used as an index: the loss turns NaN, every other frame's row is untouched
    import torch
    from paper_1904_04956_amd.harness import Learner
    dims = dict(T=2, B=5, D=8, H=8, L=1, P=8, V=V)
    dm, theta, x, labels = make_problem(dims, mode, 86, 4.0)
    lrn = Learner(mode=mode, **dims)
    try:
        lrn.set_theta(theta); lrn.set_batch(x, labels)
        lrn.calgrad(); lrn.check_status()
        good_dz = lrn.dz.float().cpu().numpy().copy()
        assert np.isfinite(lrn.loss_value())
        bad = labels.copy(); bad[1, 3] = V + 12345; bad[0, 0] = -7
        lrn.labels.copy_(torch.from_numpy(bad))
        lrn.calgrad(); lrn.check_status()
        assert np.isnan(lrn.loss_value())
        dz = lrn.dz.float().cpu().numpy()
        ok = np.ones((2, 5), dtype=bool); ok[1, 3] = False; ok[0, 0] = False
        assert np.array_equal(dz[ok], good_dz[ok]) and np.all(np.isfinite(dz))
    finally:
        lrn.close()


def test_persistent_and_stepwise_paths_agree():
    from paper_1904_04956_amd.harness import Learner
    dims = dict(T=7, B=70, D=48, H=256, L=2, P=32, V=150)
    dm, theta, x, labels = make_problem(dims, 1, 80, 2.0)
    res = []
    for path in (0, 1):
        lrn = Learner(mode=1, recurrent_path=path, **dims)
        lrn.set_theta(theta); lrn.set_batch(x, labels); lrn.calgrad(); lrn.check_status()
        res.append((lrn.loss_value(), lrn.grad_numpy().copy(), lrn.z_numpy().copy()))
        lrn.close()
    # same arithmetic up to the order of the float sums inside a dot product
    assert abs(res[0][0] - res[1][0]) <= 2e-3 * abs(res[1][0])
    assert rel_err(res[0][2], res[1][2]) <= 2e-2
    assert rel_err(res[0][1], res[1][1]) <= 2e-2


def test_weight_gradients_in_more_than_one_grouped_launch():
    # seven layers: sixteen weight-gradient products with the softmax layer's, more than one grouped launch holds (14); padded first layer among them
    check_step(dict(T=4, B=32, D=130, H=128, L=7, P=128, V=256), 1, seed=84, theta_scale=2.0)
    # shapes the 256x128 tile takes (4H = 2048, M = 256) and a layer count that fills one grouped launch exactly
    check_step(dict(T=8, B=32, D=128, H=512, L=1, P=128, V=384), 1, seed=85, theta_scale=2.0)


def test_kept_weight_copies_change_nothing():
    # the copies derived from the weights (padded W_x of layer 0, transposed U_h), kept across steps and refreshed on
    # blstm_weights_changed, must give the same bits as copies rebuilt in every pass
    from paper_1904_04956_amd.harness import Learner
    dims = dict(T=8, B=64, D=100, H=256, L=3, P=32, V=200)      # D = 100: padded copies; H = 256: persistent kernels
    dm, theta, x, labels = make_problem(dims, 1, 82, 2.0)
    res = []
    for keep in (False, True):
        lrn = Learner(mode=1, keep_weight_copies=keep, **dims)
        lrn.set_theta(theta); lrn.set_batch(x, labels)
        for _ in range(3):
            lrn.train_step(0.05)
        lrn.check_status()
        res.append((lrn.loss_value(), lrn.grad_numpy().copy(), lrn.theta_numpy().copy()))
        lrn.close()
    assert res[0][0] == res[1][0]
    assert np.array_equal(res[0][1], res[1][1]) and np.array_equal(res[0][2], res[1][2])


def test_paper_shaped_workload_bf16_stepwise_path():
    w = inputs.WORKLOADS["paper4x512"]
    d = w.dims(); d["B"] = 64
    check_step(d, 1, w.seed, lr=w.lr, recurrent_path=1)


def test_paper_shaped_workload_bf16_full_size():
    # the configuration the benchmark times, compared in full
    w = inputs.WORKLOADS["paper4x512"]
    check_step(w.dims(), 1, w.seed, lr=w.lr)


def test_paper_shaped_workload_fp32_mode_reduced_batch():
    # same model in fp32 mode for the 1e-4 bar (a quarter of the batch keeps the oracle short)
    w = inputs.WORKLOADS["paper4x512"]
    d = w.dims(); d["B"] = 64
    check_step(d, 0, w.seed, lr=w.lr)


# ------------------------------------------------------------------ update kernels

@pytest.mark.parametrize("n", [1, 3, 4, 1000, 1027, 4099, 1 << 20])
@pytest.mark.parametrize("momentum", [0.0, 0.9])
def test_sgd_step_against_oracle(n, momentum):
    import torch
    from paper_1904_04956_amd import binding as bl
    rng = np.random.default_rng(n)
    th = rng.standard_normal(n).astype(np.float32)
    g = rng.standard_normal(n).astype(np.float32)
    v = rng.standard_normal(n).astype(np.float32)
    dth, dg, dv = (torch.from_numpy(a).cuda() for a in (th, g, v))
    dsh = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    bl.sgd_step(dth, dsh, dg, n, 0.05, momentum, dv if momentum else None)
    ref_t, ref_v = orc.sgd_step(th, g, 0.05, momentum, v)
    out = dth.cpu().numpy()
    assert np.abs(out - ref_t).max() <= 2e-7 * max(1.0, np.abs(ref_t).max())
    if momentum:
        assert np.abs(dv.cpu().numpy() - ref_v).max() <= 2e-7 * np.abs(ref_v).max()
    else:
        assert np.array_equal(dv.cpu().numpy(), v)
    assert np.array_equal(dsh.float().cpu().numpy(), inputs.round_to_bf16(out))
    # lr = 0 is the identity
    before = dth.clone()
    bl.sgd_step(dth, None, dg, n, 0.0, 0.0, None)
    assert torch.equal(before, dth)


@pytest.mark.parametrize("n,R", [(5, 2), (1027, 4), (1 << 18, 16)])
def test_adpsgd_mix_against_oracle(n, R):
    import torch
    from paper_1904_04956_amd import binding as bl
    rng = np.random.default_rng(R)
    th = [rng.standard_normal(n).astype(np.float32) for _ in range(R)]
    dth = [torch.from_numpy(a).cuda() for a in th]
    dsh = [torch.zeros(n, dtype=torch.bfloat16, device="cuda") for _ in range(R)]
    ref = [a.astype(np.float64) for a in th]
    for step in range(6):
        partner = bl.adpsgd_ring_partner(R, step)
        bl.adpsgd_mix(dth, dsh, n, R, partner)
        ref = orc.adpsgd_mix(ref, partner)
        out = [d.cpu().numpy() for d in dth]
        for i in range(R):
            assert np.array_equal(out[i], out[partner[i]])                       # pair members bit-equal
            assert np.abs(out[i] - ref[i]).max() <= 1e-6 * np.abs(ref[i]).max()
            assert np.array_equal(dsh[i].float().cpu().numpy(), inputs.round_to_bf16(out[i]))
    mean0 = np.mean(np.stack([a.astype(np.float64) for a in th]), axis=0)
    mean1 = np.mean(np.stack([d.cpu().numpy().astype(np.float64) for d in dth]), axis=0)
    assert np.abs(mean1 - mean0).max() <= 1e-6 * np.abs(mean0).max()
    # a learner paired with itself is left untouched
    partner = list(range(R))
    snap = [d.clone() for d in dth]
    bl.adpsgd_mix(dth, None, n, R, partner)
    assert all(torch.equal(a, b) for a, b in zip(snap, dth))


def test_adpsgd_mix_full_size_mean_invariant():
    # sixteen replicas of the paper-shaped model resident in HBM, as in the ADPSGD workload
    import torch
    from paper_1904_04956_amd import binding as bl
    n, R = 30_539_264, 16
    gen = torch.Generator(device="cuda").manual_seed(4956)
    dth = [torch.empty(n, dtype=torch.float32, device="cuda").uniform_(-0.1, 0.1, generator=gen) for _ in range(R)]
    dsh = [torch.empty(n, dtype=torch.bfloat16, device="cuda") for _ in range(R)]
    mean0 = torch.stack([d.double() for d in dth]).mean(dim=0)
    before = [d.cpu().numpy() for d in dth[:4]]
    for step in range(2):
        partner = bl.adpsgd_ring_partner(R, step)
        bl.adpsgd_mix(dth, dsh, n, R, partner)
        if step == 0:
            ref = orc.adpsgd_mix(before[:2], [1, 0])
            assert np.abs(dth[0].cpu().numpy() - ref[0]).max() <= 1e-7
            assert torch.equal(dth[0], dth[1]) and torch.equal(dth[2], dth[3])
    mean1 = torch.stack([d.double() for d in dth]).mean(dim=0)
    err = float((mean1 - mean0).abs().max() / mean0.abs().max())
    say(f"replica mean after two mixing steps: relative error {err:.2e}")
    assert err <= 1e-6
    assert torch.equal(dsh[5].float(), dth[5].bfloat16().float())


# ------------------------------------------------------------------ reproducibility, ADPSGD end to end

def test_run_to_run_bit_reproducible():
    from paper_1904_04956_amd.harness import Learner
    dims = dict(T=6, B=40, D=36, H=64, L=2, P=32, V=500)
    dm, theta, x, labels = make_problem(dims, 1, 3)
    outs = []
    for _ in range(3):
        lrn = Learner(mode=1, **dims)
        lrn.set_theta(theta); lrn.set_batch(x, labels); lrn.calgrad()
        outs.append((lrn.loss_value(), lrn.grad_numpy().copy()))
        lrn.close()
    for l, g in outs[1:]:
        assert l == outs[0][0] and np.array_equal(g, outs[0][1])


def test_adpsgd_iterations_reduced_width():
    """Sixteen learners, ten iterations of local step + ring averaging (the ADPSGD workload with the
    model narrowed to H = 64, V = 1000 so that the oracle runs all of it)."""
    from paper_1904_04956_amd import binding as bl
    from paper_1904_04956_amd.harness import Learner, mix
    dims = dict(T=21, B=8, D=260, H=64, L=2, P=32, V=1000)
    R, iters, lr, mode = 16, 10, 0.05, 0
    dm = orc.Dims(**dims)
    n = orc.param_count(dm)
    theta0 = inputs.make_theta(n, 4956)
    learners = [Learner(mode=mode, **dims) for _ in range(R)]
    for l in learners:
        l.set_theta(theta0)
    ref = [theta0.astype(np.float64) for _ in range(R)]
    for it in range(iters):
        for r, l in enumerate(learners):
            x, labels = inputs.make_batch(dm.T, dm.B, dm.D, dm.V, 5000 + 16 * it + r)
            l.set_batch(x, labels)
            l.train_step(lr)
            _, g = orc.loss_and_grad(dm, ref[r], x, labels)
            ref[r], _ = orc.sgd_step(ref[r], g, lr)
        partner = bl.adpsgd_ring_partner(R, it)
        mean_before = np.mean([l.theta_numpy().astype(np.float64) for l in learners], axis=0)
        mix(learners, partner)
        mean_after = np.mean([l.theta_numpy().astype(np.float64) for l in learners], axis=0)
        assert np.abs(mean_after - mean_before).max() <= 1e-6 * np.abs(mean_before).max()
        ref = orc.adpsgd_mix(ref, partner)
    worst = max(rel_err(l.theta_numpy(), ref[r]) for r, l in enumerate(learners))
    say(f"ADPSGD, {iters} iterations, {R} learners: worst relative error of the weights {worst:.2e}")
    assert worst <= 1e-4
    for l in learners:
        l.close()


# ------------------------------------------------------------------ the large workloads at full size
# Every workload is compared with the oracle in full: loss, z, every gradient tensor and the updated master
# weights, element by element.  The oracle's float64 logit matrix of a whole large batch would not fit in
# host memory, so the TEST evaluates the oracle on consecutive chunks of sequences with the whole batch's
# loss scale s = 1/(T*B) and adds the chunks' losses and gradients: sequences of a batch are independent
# (pinned on the CPU by the batch-splitting and loss-scale pins).  As an extra, a property that holds at any
# size: the loss and the gradient of a batch are the means of those of its equal parts.

def oracle_in_chunks(d, theta64, x, labels, chunk):
    """Oracle loss, z and gradient of the whole batch as sums over chunks of `chunk` sequences."""
    B = d["B"]
    s_full = 1.0 / (d["T"] * B)
    loss, grad = 0.0, None
    z = np.empty((d["T"], B, d["P"] if d["P"] > 0 else 2 * d["H"]))
    for b0 in range(0, B, chunk):
        b1 = min(B, b0 + chunk)
        dc = orc.Dims(**dict(d, B=b1 - b0), loss_scale=s_full)
        xc, lc = np.ascontiguousarray(x[:, b0:b1]), np.ascontiguousarray(labels[:, b0:b1])
        zc, cache = orc.blstm_forward(dc, theta64, xc)
        lossc, dz, dWs, dbs, _ = orc.softmax_xent_fwd_bwd(dc, theta64, zc, lc)
        g = orc.blstm_backward(dc, theta64, cache, dz)
        gv = orc.views(g, dc)
        gv["Ws"][...] = dWs
        gv["bs"][...] = dbs
        z[:, b0:b1] = zc
        loss += lossc
        grad = g if grad is None else grad + g
        say(f"  oracle: sequences {b0}..{b1 - 1} of {B} done")
    return loss, z, grad


def elementwise_err(a, ref):
    """max_k |a_k - ref_k| / max(|ref_k|, 1e-3 max|ref|): the element-wise relative error with a floor, reported only."""
    ref = np.asarray(ref, dtype=np.float64)
    floor = 1e-3 * np.abs(ref).max()
    if floor == 0:
        return float(np.abs(a).max())
    return float((np.abs(np.asarray(a, dtype=np.float64) - ref) / np.maximum(np.abs(ref), floor)).max())


def _full_size_check(name, chunk, parts, tol=2e-2):
    from paper_1904_04956_amd.harness import Learner
    w = inputs.WORKLOADS[name]
    d = w.dims()
    bf = w.mode == 1
    dm = orc.Dims(**d)
    say(f"case workload={name} dims={d} mode={w.mode} seed={w.seed}")
    lrn = Learner(mode=w.mode, **d)
    theta = inputs.make_theta(lrn.n, w.seed, bf16=bf)
    x, labels = inputs.make_batch(d["T"], d["B"], d["D"], d["V"], w.seed, bf16=bf)
    lrn.set_theta(theta); lrn.set_batch(x, labels)
    lrn.calgrad(); lrn.check_status()
    z = lrn.z_numpy(); loss = lrn.loss_value(); g = lrn.grad_numpy().copy()
    lrn.apply(w.lr)
    th_gpu = lrn.theta_numpy().copy()
    lrn.close()
    th64 = theta.astype(np.float64)
    loss_ref, z_ref, g_ref = oracle_in_chunks(d, th64, x, labels, chunk)
    th_ref, _ = orc.sgd_step(th64, g_ref, w.lr)
    e = rel_err(z, z_ref)
    say(f"{name}: z relative error {e:.2e} (element-wise with floor {elementwise_err(z, z_ref):.2e})")
    assert e <= tol
    e = abs(loss - loss_ref) / abs(loss_ref)
    say(f"{name}: loss gpu {loss:.6f} oracle {loss_ref:.6f}, relative error {e:.2e}")
    assert e <= tol
    assert abs(loss - np.log(d["V"])) < 0.3              # expected initial loss: ln V plus half the logit variance
    assert np.all(np.isfinite(g))
    worst = worst_el = worst_th = 0.0
    for tname, off, shape in orc.layout(dm):
        k = int(np.prod(shape))
        e = rel_err(g[off:off + k], g_ref[off:off + k])
        ee = elementwise_err(g[off:off + k], g_ref[off:off + k])
        et = rel_err(th_gpu[off:off + k], th_ref[off:off + k])
        worst, worst_el, worst_th = max(worst, e), max(worst_el, ee), max(worst_th, et)
        assert e <= tol, f"grad {tname}: {e}"
        assert et <= tol, f"theta {tname}: {et}"
    say(f"{name}: every gradient tensor against the oracle, worst relative error {worst:.2e} "
        f"(element-wise with floor 1e-3 max|ref|: {worst_el:.2e}); updated weights {worst_th:.2e}; tolerance {tol:g}")
    if parts > 1:
        _parts_property_check(w, d, theta, x, labels, loss, g, parts, tol)


def _parts_property_check(w, d, theta, x, labels, loss, g, parts, tol):
    from paper_1904_04956_amd.harness import Learner
    B = d["B"]; Bp = B // parts
    dp = dict(d); dp["B"] = Bp
    lrn = Learner(mode=w.mode, **dp)
    lrn.set_theta(theta)
    acc = np.zeros_like(g, dtype=np.float64); lsum = 0.0
    for k in range(parts):
        lrn.set_batch(x[:, k * Bp:(k + 1) * Bp], labels[:, k * Bp:(k + 1) * Bp])
        lrn.calgrad(); lrn.check_status()
        acc += lrn.grad_numpy(); lsum += lrn.loss_value()
    lrn.close()
    acc /= parts; lsum /= parts
    assert abs(loss - lsum) <= 1e-3 * abs(lsum)
    dm = orc.Dims(**d)
    worst = 0.0
    for name, off, shape in orc.layout(dm):
        k = int(np.prod(shape))
        e = rel_err(g[off:off + k], acc[off:off + k]); worst = max(worst, e)
        assert e <= tol, f"{name}: {e}"
    say(f"{w.name} B={B}: gradient against the mean of {parts} parts of {Bp}, worst relative difference {worst:.2e}")


def test_large_batch_workload_full_size():
    _full_size_check("largebatch", chunk=128, parts=8)


def test_wide_deep_workload_full_size():
    _full_size_check("wide6x1024", chunk=64, parts=8)


def test_wide_cells_against_oracle_reduced_depth():
    # H = 1024 at a ragged, small shape (one batch tile group, short unroll)
    check_step(dict(T=5, B=96, D=260, H=1024, L=2, P=64, V=1000), 1, seed=4958, lr=0.2)


def test_adpsgd_workload_first_step_full_size():
    # one learner of the ADPSGD workload (batch 128 of the paper-shaped model) against the oracle in full
    w = inputs.WORKLOADS["adpsgd16"]
    check_step(w.dims(), 1, seed=5000, lr=w.lr)


def test_paper_6x512_model_full_size():
    # the model the paper trains and times (section 4.2): six layers of 512 cells per direction, batch 256
    _full_size_check("paper6x512", chunk=128, parts=4)
