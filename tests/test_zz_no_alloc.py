"""The entry point that allocates nothing (softmax_xent_fwd_bwd_noalloc: scratch in an array of the library's own
code object) against softmax_xent_fwd_bwd on a bound workspace, through the C-ABI.  Same kernels, same plans:
the results must be the same bits.  Two calls in a row, the second on a smaller shape, so that whatever the first
call left in the shared array is seen not to matter."""
import sys

import numpy as np
import pytest

from oracle import blstm_oracle as orc
from paper_1904_04956_amd import inputs

pytestmark = pytest.mark.gpu


def _run_both(dims, mode, seed):
    import torch
    from paper_1904_04956_amd import binding as bl
    from paper_1904_04956_amd.harness import Learner
    dm = orc.Dims(**dims)
    n = orc.param_count(dm)
    bf = mode == 1
    theta = inputs.make_theta(n, seed, bf16=bf)
    rng = np.random.default_rng(seed)
    zdim = dm.zdim
    z = rng.standard_normal((dm.T, dm.B, zdim)).astype(np.float32)
    if bf:
        z = inputs.round_to_bf16(z)
    labels = rng.integers(0, dm.V, size=(dm.T, dm.B)).astype(np.int32)
    print(f"case dims={dims} mode={mode} seed={seed}", flush=True)
    lrn = Learner(mode=mode, defer_softmax_wgrad=False, **dims)     # (softmax_xent_fwd_bwd is called on its own here: it writes dW_s itself)
    try:
        lrn.set_theta(theta)
        lrn.z.copy_(torch.from_numpy(z).to(lrn.act_dtype))
        lrn.labels.copy_(torch.from_numpy(labels))
        th = lrn.theta_fwd
        # the existing entry point, on the bound workspace
        lrn.grad.zero_()
        bl.softmax_xent_fwd_bwd(lrn.ctx, th, lrn.z, lrn.labels, lrn.loss, lrn.dz, lrn.grad)
        ref = (lrn.loss.cpu().numpy().copy(), lrn.dz.float().cpu().numpy().copy(), lrn.grad.cpu().numpy().copy())
        # the entry point that allocates nothing: fresh outputs, nothing allocated between the call and its results
        loss2 = torch.full_like(lrn.loss, -1.0); dz2 = torch.zeros_like(lrn.dz); grad2 = torch.zeros_like(lrn.grad)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        bl.softmax_xent_fwd_bwd_noalloc(lrn.ctx, th, lrn.z, lrn.labels, loss2, dz2, grad2)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        out = (loss2.cpu().numpy(), dz2.float().cpu().numpy(), grad2.cpu().numpy())
    finally:
        lrn.close()
    # against the oracle as well, at the mode's tolerance
    loss_ref, dz_ref, dWs, dbs, _ = orc.softmax_xent_fwd_bwd(dm, theta.astype(np.float64), z, labels)
    tol = 2e-2 if bf else 1e-4
    assert abs(out[0][0] - loss_ref) <= tol * abs(loss_ref)
    assert np.abs(out[1] - dz_ref).max() <= tol * np.abs(dz_ref).max()
    gv = {name: (off, int(np.prod(shape))) for name, off, shape in orc.layout(dm)}
    off, k = gv["Ws"]; assert np.abs(out[2][off:off + k] - dWs.ravel()).max() <= tol * np.abs(dWs).max()
    off, k = gv["bs"]; assert np.abs(out[2][off:off + k] - dbs).max() <= tol * np.abs(dbs).max()
    # and the same bits as the existing entry point
    assert out[0][0] == ref[0][0]
    assert np.array_equal(out[1], ref[1])
    for name in ("Ws", "bs"):
        off, k = gv[name]
        assert np.array_equal(out[2][off:off + k], ref[2][off:off + k])
    return out


def test_noalloc_entry_matches_the_workspace_entry_twice_in_a_row():
    # first call: 336 frames of 12000 classes (8 MB of logits, dz split along K, ragged row tiles) in bf16
    _run_both(dict(T=21, B=16, D=12, H=16, L=1, P=64, V=12000), 1, seed=91)
    # second call, smaller, right after it on the same array; then fp32 mode, smaller again
    _run_both(dict(T=5, B=7, D=12, H=16, L=1, P=24, V=1003), 1, seed=92)
    _run_both(dict(T=3, B=4, D=6, H=8, L=1, P=0, V=50), 0, seed=93)


def test_noalloc_entry_rejects_what_does_not_fit():
    from paper_1904_04956_amd import binding as bl
    import torch
    ctx = bl.blstm_create(21, 64, 8, 8, 1, 16, 32000, 1)     # 86 MB of logits
    t = torch.zeros(1 << 20, dtype=torch.float32, device="cuda")
    try:
        with pytest.raises(bl.BlstmError) as e:
            bl.softmax_xent_fwd_bwd_noalloc(ctx, t, t, t, t, t, t)
        assert e.value.code == -3
    finally:
        bl.blstm_destroy(ctx)
