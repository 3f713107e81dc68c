"""Device-memory plumbing around the C-ABI calls: one learner's buffers and step order.

PyTorch allocates the buffers and provides the stream; every computation is a call
into the library through `binding`.  Used by the GPU tests, the smoke check and the
benchmark.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as bl
from . import inputs


class Learner:
    """Buffers of one learner: master weights, bf16 shadow, gradient, batch, workspace."""

    def __init__(self, T, B, D, H, L, P, V, mode, loss_scale=0.0, device="cuda:0", momentum=0.0, recurrent_path=0, recurrent_sync=None, keep_weight_copies=True,
                 defer_softmax_wgrad=True):
        if not torch.cuda.is_available():
            raise RuntimeError("a GPU is required: the HIP path has no CPU fallback")
        self.dims = dict(T=T, B=B, D=D, H=H, L=L, P=P, V=V)
        self.mode = mode
        self.device = torch.device(device)
        self.ctx = bl.blstm_create(T, B, D, H, L, P, V, mode, loss_scale)
        if recurrent_path:
            bl.blstm_set_option(self.ctx, bl.BLSTM_OPT_RECURRENT_PATH, recurrent_path)
        # the copies the passes derive from the weights are kept across steps: every method below that changes the
        # weights reports it (weights_changed)
        bl.blstm_set_option(self.ctx, bl.BLSTM_OPT_KEEP_WEIGHT_COPIES, int(bool(keep_weight_copies)))
        if recurrent_sync is not None:
            bl.blstm_set_option(self.ctx, bl.BLSTM_OPT_RECURRENT_SYNC, recurrent_sync)
        # calgrad() always runs softmax_xent_fwd_bwd and blstm_backward back to back on the same gradient vector, so the
        # softmax layer's weight gradient may join the backward pass's grouped launch
        bl.blstm_set_option(self.ctx, bl.BLSTM_OPT_DEFER_SOFTMAX_WGRAD, int(bool(defer_softmax_wgrad)))
        self.defer_softmax_wgrad = bool(defer_softmax_wgrad)
        self.n = bl.blstm_param_count(self.ctx)
        self.zdim = P if P > 0 else 2 * H
        self.act_dtype = torch.bfloat16 if mode == 1 else torch.float32
        dev = self.device
        self.workspace = torch.empty(bl.blstm_workspace_bytes(self.ctx), dtype=torch.uint8, device=dev)
        bl.blstm_bind(self.ctx, self.workspace)
        self.theta = torch.zeros(self.n, dtype=torch.float32, device=dev)
        self.shadow = torch.zeros(self.n, dtype=torch.bfloat16, device=dev) if mode == 1 else None
        self.grad = torch.zeros(self.n, dtype=torch.float32, device=dev)
        self.velocity = torch.zeros(self.n, dtype=torch.float32, device=dev) if momentum != 0.0 else None
        self.momentum = momentum
        self.x = torch.zeros((T, B, D), dtype=self.act_dtype, device=dev)
        self.labels = torch.zeros((T, B), dtype=torch.int32, device=dev)
        self.z = torch.zeros((T, B, self.zdim), dtype=self.act_dtype, device=dev)
        self.dz = torch.zeros((T, B, self.zdim), dtype=self.act_dtype, device=dev)
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)
        self.held = None          # HYBRID only: the pulled weights the next gradient is taken on

    def close(self):
        if self.ctx is not None:
            bl.blstm_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- data in ---------------------------------------------------------------------
    def set_theta(self, theta_f32: np.ndarray):
        assert theta_f32.dtype == np.float32 and theta_f32.size == self.n
        self.theta.copy_(torch.from_numpy(theta_f32))
        if self.shadow is not None:
            bl.blstm_shadow_refresh(self.theta, self.shadow, self.n)
        self.weights_changed()

    def weights_changed(self):
        """To be called after anything has written the weights (or the held copy) outside this class."""
        bl.blstm_weights_changed(self.ctx)

    def set_batch(self, x_f32: np.ndarray, labels_i32: np.ndarray):
        self.x.copy_(torch.from_numpy(x_f32).to(self.act_dtype))
        self.labels.copy_(torch.from_numpy(labels_i32.astype(np.int32)))

    @property
    def theta_fwd(self):
        """The weights as the forward and backward passes read them."""
        return self.shadow if self.mode == 1 else self.theta

    # ---- the step ----------------------------------------------------------------------
    def forward(self, stream=None):
        bl.blstm_forward(self.ctx, self.theta_fwd, self.x, self.z, stream)

    def calgrad(self, stream=None, weights=None):
        """g = calGrad(W): forward, softmax cross-entropy, backward (on `weights` if given, in the
        storage type of the mode, else on the learner's own)."""
        th = self.theta_fwd if weights is None else weights
        bl.blstm_forward(self.ctx, th, self.x, self.z, stream)
        bl.softmax_xent_fwd_bwd(self.ctx, th, self.z, self.labels, self.loss, self.dz, self.grad, stream)
        bl.blstm_backward(self.ctx, th, self.x, self.dz, self.grad, stream)

    def apply(self, lr, stream=None):
        """W' = apply(W, g)."""
        bl.sgd_step(self.theta, self.shadow, self.grad, self.n, lr, self.momentum, self.velocity, stream)
        self.weights_changed()

    def hold(self):
        """Keeps a copy of the weights as forward/backward read them now (a device-to-device copy on
        torch's current stream): what pull_weights() returned, for the next iteration's gradient."""
        if self.held is None:
            self.held = torch.empty_like(self.theta_fwd)
        self.held.copy_(self.theta_fwd)
        self.weights_changed()

    def train_step(self, lr, stream=None):
        self.calgrad(stream)
        self.apply(lr, stream)

    def check_status(self, stream=None):
        """Synchronises and raises if a persistent kernel abandoned a wait."""
        bl.blstm_device_status(self.ctx, stream)

    # ---- data out --------------------------------------------------------------------
    def loss_value(self) -> float:
        return float(self.loss.cpu()[0])

    def grad_numpy(self) -> np.ndarray:
        return self.grad.cpu().numpy()

    def theta_numpy(self) -> np.ndarray:
        return self.theta.cpu().numpy()

    def z_numpy(self) -> np.ndarray:
        return self.z.float().cpu().numpy()


def learner_for(workload: inputs.Workload, B=None, device="cuda:0", momentum=0.0) -> Learner:
    d = workload.dims()
    if B is not None:
        d["B"] = B
    return Learner(mode=workload.mode, device=device, momentum=momentum, **d)


def mix(learners, partner, stream=None):
    """One ADPSGD averaging step over the learners' weights (and their bf16 shadows)."""
    masters = [l.theta for l in learners]
    shadows = [l.shadow for l in learners] if learners[0].shadow is not None else None
    bl.adpsgd_mix(masters, shadows, learners[0].n, len(learners), partner, stream)
    for l in learners:
        l.weights_changed()


# ---- the strategies of section 3.2 as orders of the library's calls, R learners in one GPU's memory ----

def adpsgd_step(learners, lr, partner, fused=False, stream=None):
    """Eq. 4 in the synchronous order: g_i = calGrad(W_i), W_i' = apply(W_i, g_i), then the pairs average.
    With fused=True each pair's update and average are one pass over the weights (sgd_mix_pair)."""
    for l in learners:
        l.calgrad(stream)
    if not fused:
        for l in learners:
            l.apply(lr, stream)
        mix(learners, partner, stream)
        return
    for i, j in enumerate(partner):
        a = learners[i]
        if j == i:
            a.apply(lr, stream)
        elif j > i:
            b = learners[j]
            bl.sgd_mix_pair(a.theta, b.theta, a.shadow, b.shadow, a.grad, b.grad, a.n, lr, a.momentum,
                            a.velocity, b.velocity, stream)
            a.weights_changed(); b.weights_changed()


def stale_adpsgd_step(learners, lr, partner, stream=None):
    """The integration order of Fig. 3b: the gradient is computed on the learner's own weights, the
    weights are then replaced by the pair's average (pull) and the gradient is applied to that."""
    for l in learners:
        l.calgrad(stream)
    mix(learners, partner, stream)
    for l in learners:
        l.apply(lr, stream)


def sync_step(learners, lr, stream=None):
    """SYNC of Fig. 3a: every learner applies its own gradient, then all take the mean of the results."""
    for l in learners:
        l.calgrad(stream)
        l.apply(lr, stream)
    masters = [l.theta for l in learners]
    shadows = [l.shadow for l in learners] if learners[0].shadow is not None else None
    bl.sync_average(masters, shadows, learners[0].n, len(learners), stream)
    for l in learners:
        l.weights_changed()


def hybrid_step(learners, lr):
    """HYBRID of Fig. 3c with its push as an average over all learners (section 3.2): the gradient is taken
    on the weights pulled in the iteration before (the common initial weights at first), the pull is the
    mean of what every learner pushed at the end of that iteration (sync_average over the masters), and the
    gradient is applied to the pulled weights.  Runs on the default stream (the held copy is a torch copy)."""
    for l in learners:
        l.calgrad(weights=l.held)
    masters = [l.theta for l in learners]
    shadows = [l.shadow for l in learners] if learners[0].shadow is not None else None
    bl.sync_average(masters, shadows, learners[0].n, len(learners))
    for l in learners:
        l.weights_changed()
        l.hold()
        l.apply(lr)
