"""GPU parity of the strategy rows beyond plain ADPSGD: the fused pair update (Eq. 4 in one pass), the
synchronous R-way average (Fig. 3a), the stale integration order of Fig. 3b and HYBRID (Fig. 3c), through the C-ABI,
against the float64 oracle.  Tolerances: streaming kernels 1e-6 relative (fp32 arithmetic on fp32
data); whole training steps 1e-4 (fp32 mode), per tensor max|gpu - ref| / max|ref|."""
import sys

import numpy as np
import pytest

from oracle import blstm_oracle as orc
from paper_1904_04956_amd import inputs

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def rel_err(a, ref):
    ref = np.asarray(ref, dtype=np.float64)
    den = np.abs(ref).max()
    num = np.abs(np.asarray(a, dtype=np.float64) - ref).max()
    return num / den if den > 0 else num


@pytest.mark.parametrize("n", [1, 3, 6, 1027, 4099, 1 << 20])
@pytest.mark.parametrize("momentum", [0.0, 0.9])
def test_one_sided_pair_update_against_oracle_and_the_two_call_form(n, momentum):
    """sgd_mix_pair without a gradient for replica j: one learner's Eq. 1c followed by Eq. 4's average with a
    neighbour that is taken as it stands (the oracle's pair update with a zero gradient for the neighbour)."""
    import torch
    from paper_1904_04956_amd import binding as bl
    rng = np.random.default_rng(11 * n + 3)
    a, b, ga, va = (rng.standard_normal(n).astype(np.float32) for _ in range(4))
    lr = 0.05
    d = {k: torch.from_numpy(v).cuda() for k, v in dict(a=a, b=b, ga=ga, va=va).items()}
    sa = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    sb = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    e = {k: v.clone() for k, v in d.items()}
    bl.sgd_step(e["a"], None, e["ga"], n, lr, momentum, e["va"] if momentum else None)
    bl.adpsgd_mix([e["a"], e["b"]], None, n, 2, [1, 0])
    bl.sgd_mix_pair(d["a"], d["b"], sa, sb, d["ga"], None, n, lr, momentum, d["va"] if momentum else None, None)
    zero = np.zeros(n, dtype=np.float32)
    ref, rva, _ = orc.sgd_mix_pair(a, b, ga, zero, lr, momentum, va, zero)
    out = d["a"].cpu().numpy()
    assert torch.equal(d["a"], d["b"])
    assert np.abs(out - ref).max() <= 1e-6 * max(1.0, np.abs(ref).max())
    assert torch.equal(d["a"], e["a"]) and torch.equal(d["b"], e["b"])  # same arithmetic as sgd_step + adpsgd_mix
    if momentum:
        assert np.abs(d["va"].cpu().numpy() - rva).max() <= 2e-7 * np.abs(rva).max()
        assert torch.equal(d["va"], e["va"])
    else:
        assert np.array_equal(d["va"].cpu().numpy(), va)
    assert np.array_equal(sa.float().cpu().numpy(), inputs.round_to_bf16(out))
    assert torch.equal(sa, sb)


@pytest.mark.parametrize("n", [1, 3, 6, 1027, 4099, 1 << 20])
@pytest.mark.parametrize("momentum", [0.0, 0.9])
def test_fused_pair_update_against_oracle_and_the_two_call_form(n, momentum):
    import torch
    from paper_1904_04956_amd import binding as bl
    rng = np.random.default_rng(7 * n + 1)
    a, b, ga, gb, va, vb = (rng.standard_normal(n).astype(np.float32) for _ in range(6))
    lr = 0.05
    d = {k: torch.from_numpy(v).cuda() for k, v in dict(a=a, b=b, ga=ga, gb=gb, va=va, vb=vb).items()}
    sa = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    sb = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    # the two-call form on copies: sgd_step on each replica, then adpsgd_mix
    e = {k: v.clone() for k, v in d.items()}
    bl.sgd_step(e["a"], None, e["ga"], n, lr, momentum, e["va"] if momentum else None)
    bl.sgd_step(e["b"], None, e["gb"], n, lr, momentum, e["vb"] if momentum else None)
    bl.adpsgd_mix([e["a"], e["b"]], None, n, 2, [1, 0])
    bl.sgd_mix_pair(d["a"], d["b"], sa, sb, d["ga"], d["gb"], n, lr, momentum,
                    d["va"] if momentum else None, d["vb"] if momentum else None)
    ref, rva, rvb = orc.sgd_mix_pair(a, b, ga, gb, lr, momentum, va, vb)
    out = d["a"].cpu().numpy()
    assert torch.equal(d["a"], d["b"])                                  # both replicas hold the same bits
    assert np.abs(out - ref).max() <= 1e-6 * max(1.0, np.abs(ref).max())
    assert torch.equal(d["a"], e["a"]) and torch.equal(d["b"], e["b"])  # same arithmetic as the two-call form
    if momentum:
        assert np.abs(d["va"].cpu().numpy() - rva).max() <= 2e-7 * np.abs(rva).max()
        assert np.abs(d["vb"].cpu().numpy() - rvb).max() <= 2e-7 * np.abs(rvb).max()
        assert torch.equal(d["va"], e["va"]) and torch.equal(d["vb"], e["vb"])
    else:
        assert np.array_equal(d["va"].cpu().numpy(), va) and np.array_equal(d["vb"].cpu().numpy(), vb)
    assert np.array_equal(sa.float().cpu().numpy(), inputs.round_to_bf16(out))
    assert torch.equal(sa, sb)


@pytest.mark.parametrize("n,R", [(5, 1), (7, 2), (1027, 5), (1 << 18, 16), (4099, 64)])
def test_sync_average_against_oracle(n, R):
    import torch
    from paper_1904_04956_amd import binding as bl
    rng = np.random.default_rng(100 + R)
    th = [rng.standard_normal(n).astype(np.float32) for _ in range(R)]
    dth = [torch.from_numpy(a).cuda() for a in th]
    dsh = [torch.zeros(n, dtype=torch.bfloat16, device="cuda") for _ in range(R)]
    bl.sync_average(dth, dsh, n, R)
    ref = orc.sync_average(th)
    out = [t.cpu().numpy() for t in dth]
    assert all(np.array_equal(out[0], o) for o in out[1:])              # every replica holds the same bits
    assert np.abs(out[0] - ref[0]).max() <= 1e-6 * max(1.0, np.abs(ref[0]).max())
    for s in dsh:
        assert np.array_equal(s.float().cpu().numpy(), inputs.round_to_bf16(out[0]))
    if R == 2:                                                          # two replicas: same value as the pair average
        d2 = [torch.from_numpy(a).cuda() for a in th]
        bl.adpsgd_mix(d2, None, n, 2, [1, 0])
        assert np.abs(d2[0].cpu().numpy() - out[0]).max() <= 1e-7 * max(1.0, np.abs(out[0]).max())
    # averaging again changes nothing beyond the rounding of an R-term float sum (a consensus is a fixed point)
    snap = dth[0].clone()
    bl.sync_average(dth, None, n, R)
    assert np.abs((dth[0] - snap).cpu().numpy()).max() <= 1e-6 * max(1.0, float(snap.abs().max()))


def _learners(dims, R, mode, theta0):
    from paper_1904_04956_amd.harness import Learner
    ls = [Learner(mode=mode, **dims) for _ in range(R)]
    for l in ls:
        l.set_theta(theta0)
    return ls


def test_sync_strategy_is_one_large_batch_step():
    """Fig. 3a on four learners with a quarter of the batch each, the loss normalised over the whole batch:
    after the average every learner holds what one learner gets from the whole batch in one step."""
    from paper_1904_04956_amd.harness import Learner, sync_step
    R, lr = 4, 0.1
    dims = dict(T=7, B=8, D=20, H=32, L=2, P=16, V=120)
    big = dict(dims, B=R * dims["B"])
    dm, dmb = orc.Dims(**dims), orc.Dims(**big)
    theta0 = inputs.make_theta(orc.param_count(dm), 77)
    x, labels = inputs.make_batch(dmb.T, dmb.B, dmb.D, dmb.V, 78)
    ls = _learners(dims, R, 0, theta0)
    for r, l in enumerate(ls):
        l.set_batch(np.ascontiguousarray(x[:, r * dm.B:(r + 1) * dm.B]), np.ascontiguousarray(labels[:, r * dm.B:(r + 1) * dm.B]))
    sync_step(ls, lr)
    _, g = orc.loss_and_grad(dmb, theta0.astype(np.float64), x, labels)
    ref, _ = orc.sgd_step(theta0.astype(np.float64), g, lr)
    errs = [rel_err(l.theta_numpy(), ref) for l in ls]
    say(f"SYNC on {R} learners against one step on the whole batch: worst relative error {max(errs):.2e}")
    assert max(errs) <= 1e-4
    assert all(np.array_equal(ls[0].theta_numpy(), l.theta_numpy()) for l in ls[1:])
    for l in ls:
        l.close()


@pytest.mark.parametrize("order", ["synchronous-fused", "stale"])
def test_adpsgd_orders_against_the_oracle(order):
    """Four learners, six iterations on the alternating ring: Eq. 4 with the fused pair update, and the
    stale order of Fig. 3b (gradient of the own weights applied to the pulled average)."""
    from paper_1904_04956_amd import binding as bl
    from paper_1904_04956_amd.harness import adpsgd_step, stale_adpsgd_step
    R, iters, lr = 4, 6, 0.08
    dims = dict(T=9, B=6, D=24, H=32, L=2, P=16, V=150)
    dm = orc.Dims(**dims)
    theta0 = inputs.make_theta(orc.param_count(dm), 31)
    ls = _learners(dims, R, 0, theta0)
    ref = [theta0.astype(np.float64) + 0.0 for _ in range(R)]
    for it in range(iters):
        partner = bl.adpsgd_ring_partner(R, it)
        grads = []
        for r, l in enumerate(ls):
            x, labels = inputs.make_batch(dm.T, dm.B, dm.D, dm.V, 900 + R * it + r)
            l.set_batch(x, labels)
            grads.append(orc.loss_and_grad(dm, ref[r], x, labels)[1])
        if order == "stale":
            stale_adpsgd_step(ls, lr, partner)
            ref = orc.stale_adpsgd_step(ref, grads, partner, lr)
        else:
            adpsgd_step(ls, lr, partner, fused=True)
            new = [None] * R
            for i, j in enumerate(partner):
                if j > i:
                    m, _, _ = orc.sgd_mix_pair(ref[i], ref[j], grads[i], grads[j], lr)
                    new[i], new[j] = m, m.copy()
            ref = new
    worst = max(rel_err(l.theta_numpy(), ref[r]) for r, l in enumerate(ls))
    say(f"ADPSGD, {order} order, {iters} iterations, {R} learners: worst relative error of the weights {worst:.2e}")
    assert worst <= 1e-4
    if order == "stale":      # after the apply the members of a pair differ again (each used its own gradient)
        assert not np.array_equal(ls[0].theta_numpy(), ls[partner[0]].theta_numpy())
    for l in ls:
        l.close()


def test_hybrid_order_against_the_oracle():
    """Fig. 3c on four learners, six iterations: each gradient is taken on the weights pulled one iteration
    earlier and applied to the mean of what all learners pushed (sync_average), against the oracle's hybrid_step."""
    from paper_1904_04956_amd.harness import hybrid_step
    R, iters, lr = 4, 6, 0.08
    dims = dict(T=9, B=6, D=24, H=32, L=2, P=16, V=150)
    dm = orc.Dims(**dims)
    theta0 = inputs.make_theta(orc.param_count(dm), 33)
    ls = _learners(dims, R, 0, theta0)
    pushed = [theta0.astype(np.float64) + 0.0 for _ in range(R)]
    held = theta0.astype(np.float64)
    for it in range(iters):
        grads = []
        for r, l in enumerate(ls):
            x, labels = inputs.make_batch(dm.T, dm.B, dm.D, dm.V, 1200 + R * it + r)
            l.set_batch(x, labels)
            grads.append(orc.loss_and_grad(dm, held, x, labels)[1])
        hybrid_step(ls, lr)
        pushed, held = orc.hybrid_step(pushed, grads, lr)
        assert all(np.array_equal(ls[0].held.cpu().numpy(), l.held.cpu().numpy()) for l in ls[1:])   # one common pull
        assert rel_err(ls[0].held.cpu().numpy(), held) <= 1e-4
    worst = max(rel_err(l.theta_numpy(), pushed[r]) for r, l in enumerate(ls))
    say(f"HYBRID, {iters} iterations, {R} learners: worst relative error of the pushed weights {worst:.2e}")
    assert worst <= 1e-4
    assert not np.array_equal(ls[0].theta_numpy(), ls[1].theta_numpy())     # each applied its own gradient
    for l in ls:
        l.close()


def test_paper_model_pair_update_full_size():
    """The 6x512 model of section 4.2 (43.1 M parameters, the vector the paper pushes and pulls): fused pair
    update on two replicas at full size, sampled against the oracle and checked against the two-call form."""
    import torch
    from paper_1904_04956_amd import binding as bl
    d = inputs.WORKLOADS["paper6x512"].dims()
    n = orc.param_count(orc.Dims(**d))
    assert n == 43_130_368
    gen = torch.Generator(device="cuda").manual_seed(6512)
    a, b, ga, gb = (torch.empty(n, dtype=torch.float32, device="cuda").uniform_(-0.1, 0.1, generator=gen) for _ in range(4))
    sa = torch.empty(n, dtype=torch.bfloat16, device="cuda"); sb = torch.empty_like(sa)
    ea, eb = a.clone(), b.clone()
    idx = torch.randint(0, n, (4096,), generator=torch.Generator().manual_seed(1)).cuda()
    before = [t[idx].cpu().numpy() for t in (a, b, ga, gb)]
    bl.sgd_mix_pair(a, b, sa, sb, ga, gb, n, 0.1)
    bl.sgd_step(ea, None, ga, n, 0.1); bl.sgd_step(eb, None, gb, n, 0.1); bl.adpsgd_mix([ea, eb], None, n, 2, [1, 0])
    assert torch.equal(a, ea) and torch.equal(b, eb) and torch.equal(a, b)
    ref, _, _ = orc.sgd_mix_pair(*before, 0.1)
    assert np.abs(a[idx].cpu().numpy() - ref).max() <= 1e-7
    assert torch.equal(sa.float(), a.bfloat16().float()) and torch.equal(sa, sb)
    # the one-sided form on the same vectors (replica b enters as it stands): against sgd_step on a + adpsgd_mix, and the oracle
    a2, b2 = ea.clone(), eb.clone()                      # (any two distinct vectors do: the pair above after its update)
    e2a, e2b = a2.clone(), b2.clone()
    before2 = [t[idx].cpu().numpy() for t in (a2, b2, ga)]
    bl.sgd_mix_pair(a2, b2, sa, sb, ga, None, n, 0.1)
    bl.sgd_step(e2a, None, ga, n, 0.1); bl.adpsgd_mix([e2a, e2b], None, n, 2, [1, 0])
    assert torch.equal(a2, e2a) and torch.equal(b2, e2b) and torch.equal(a2, b2)
    ref2, _, _ = orc.sgd_mix_pair(before2[0], before2[1], before2[2], np.zeros_like(before2[2]), 0.1)
    assert np.abs(a2[idx].cpu().numpy() - ref2).max() <= 1e-7
    assert torch.equal(sa.float(), a2.bfloat16().float()) and torch.equal(sa, sb)
