"""Float64 CPU oracle for one learner's BLSTM training step and the ADPSGD mixing step.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this module:
only tests/, the smoke check and the benchmark's cpu_baseline leg do.  It shares
no code with the HIP library and imports nothing from it.

What it computes is the plain definition of the method, in numpy float64, with no
blocking, fusion or reordering:

  * model (paper section 4.2): L bidirectional LSTM layers of H cells per direction
    (standard four-gate cell, no peepholes, no recurrent projection, one bias per
    gate; state zero at the first visited frame of every subsequence), the two
    directions concatenated as the next layer's input, a linear bottleneck of P
    units, a softmax over V classes;
  * criterion and gradient (paper Eq. 1a, 1b): E = s * sum over frames of
    -log softmax(u)[label], default s = 1/(T*B); the gradient is back-propagation
    through time over the T-frame unroll, derived by hand below;
  * update (paper Eq. 1c): theta <- theta - alpha * g  (with momentum mu:
    v <- mu*v + g ; theta <- theta - alpha*v);
  * decentralised averaging (paper Eq. 4, second line, and the sender/receiver
    pairing of section 3.2): both members of a pair take (theta_i + theta_j)/2;
  * the orders in which section 3.2's strategies call these (Fig. 3a SYNC, Fig. 3b stale
    ADPSGD, Fig. 3c HYBRID), as functions of the learners' weights and gradients.

Flat parameter layout (row-major, gate blocks in the order i, f, g, o):
  for layer l = 0..L-1, for direction d in (forward, backward):
      W_x [4H, D_l], U_h [4H, H], b [4H]          D_0 = D, D_l = 2H for l > 0
  W_p [P, 2H], b_p [P]                            (absent when P == 0)
  W_s [V, P or 2H], b_s [V]

Parity pins (tests/test_oracle_*.py): closed-form parameter count against the
paper's 165 MB, central finite differences, the stock CPU LSTM of the tensor
library with its autograd, zero-weight closed forms, a scalar hand case,
time-reversal symmetry, batch permutation/splitting, mixing invariants, and the
SYNC identity of section 3.2.  No function here is parity unpinned.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Dims:
    T: int
    B: int
    D: int
    H: int
    L: int
    P: int
    V: int
    loss_scale: float = 0.0   # s; <= 0 means the default 1/(T*B)

    @property
    def s(self) -> float:
        return self.loss_scale if self.loss_scale > 0 else 1.0 / (self.T * self.B)

    def layer_in(self, l: int) -> int:
        return self.D if l == 0 else 2 * self.H

    @property
    def zdim(self) -> int:
        return self.P if self.P > 0 else 2 * self.H


# --------------------------------------------------------------------------- layout

def layout(dm: Dims):
    """List of (name, offset, shape) for every tensor of the flat parameter vector."""
    out = []
    off = 0

    def put(name, shape):
        nonlocal off
        out.append((name, off, shape))
        off += int(np.prod(shape))

    for l in range(dm.L):
        for d in range(2):
            put(f"Wx{l}.{d}", (4 * dm.H, dm.layer_in(l)))
            put(f"Uh{l}.{d}", (4 * dm.H, dm.H))
            put(f"b{l}.{d}", (4 * dm.H,))
    if dm.P > 0:
        put("Wp", (dm.P, 2 * dm.H))
        put("bp", (dm.P,))
    put("Ws", (dm.V, dm.zdim))
    put("bs", (dm.V,))
    return out


def param_count(dm: Dims) -> int:
    name, off, shape = layout(dm)[-1]
    return off + int(np.prod(shape))


def views(flat: np.ndarray, dm: Dims) -> dict:
    """Dictionary of reshaped views into a flat float64 vector."""
    assert flat.dtype == np.float64 and flat.ndim == 1 and flat.size == param_count(dm)
    return {name: flat[off:off + int(np.prod(shape))].reshape(shape) for name, off, shape in layout(dm)}


def sigmoid(a):
    return 1.0 / (1.0 + np.exp(-a))


# --------------------------------------------------------------------------- forward

def visit_order(T: int, d: int):
    """Frames in the order direction d visits them (forward 0..T-1, backward T-1..0)."""
    return list(range(T)) if d == 0 else list(range(T - 1, -1, -1))


def blstm_forward(dm: Dims, theta: np.ndarray, x: np.ndarray):
    """Forward pass of the LSTM stack and the bottleneck.

    x: [T, B, D].  Returns (z [T, B, zdim], cache) where cache keeps every layer's
    input, gate activations and cell states for back-propagation.
    """
    th = views(np.asarray(theta, dtype=np.float64), dm)
    X = np.asarray(x, dtype=np.float64)
    assert X.shape == (dm.T, dm.B, dm.D)
    T, B, H = dm.T, dm.B, dm.H
    cache = {"X": [], "i": [], "f": [], "g": [], "o": [], "c": [], "h": []}
    for l in range(dm.L):
        Y = np.zeros((T, B, 2 * H))
        gi = np.zeros((2, T, B, H)); gf = np.zeros((2, T, B, H))
        gg = np.zeros((2, T, B, H)); go = np.zeros((2, T, B, H))
        cc = np.zeros((2, T, B, H)); hh = np.zeros((2, T, B, H))
        for d in range(2):
            Wx, Uh, b = th[f"Wx{l}.{d}"], th[f"Uh{l}.{d}"], th[f"b{l}.{d}"]
            h_prev = np.zeros((B, H)); c_prev = np.zeros((B, H))
            for t in visit_order(T, d):
                a = X[t] @ Wx.T + h_prev @ Uh.T + b            # [B, 4H]
                i = sigmoid(a[:, 0:H]); f = sigmoid(a[:, H:2 * H])
                g = np.tanh(a[:, 2 * H:3 * H]); o = sigmoid(a[:, 3 * H:4 * H])
                c = f * c_prev + i * g
                h = o * np.tanh(c)
                gi[d, t], gf[d, t], gg[d, t], go[d, t], cc[d, t], hh[d, t] = i, f, g, o, c, h
                Y[t, :, d * H:(d + 1) * H] = h
                h_prev, c_prev = h, c
        cache["X"].append(X)
        for k, v in zip("ifgoch", (gi, gf, gg, go, cc, hh)):
            cache[k].append(v)
        X = Y
    cache["Y"] = X
    if dm.P > 0:
        z = X @ th["Wp"].T + th["bp"]
    else:
        z = X.copy()
    return z, cache


# --------------------------------------------------------------------------- softmax cross-entropy

def softmax_xent_fwd_bwd(dm: Dims, theta: np.ndarray, z: np.ndarray, labels: np.ndarray):
    """Loss E (Eq. 1a with the frame-level cross-entropy) and its gradients.

    Returns (loss, dz [T,B,zdim], dWs [V,zdim], dbs [V], p [T*B, V]).
    """
    th = views(np.asarray(theta, dtype=np.float64), dm)
    M = dm.T * dm.B
    Z = np.asarray(z, dtype=np.float64).reshape(M, dm.zdim)
    lab = np.asarray(labels).reshape(M).astype(np.int64)
    u = Z @ th["Ws"].T + th["bs"]                              # logits [M, V]
    e = np.exp(u - u.max(axis=1, keepdims=True))
    p = e / e.sum(axis=1, keepdims=True)
    loss = dm.s * float(np.sum(-np.log(p[np.arange(M), lab])))
    du = p.copy()
    du[np.arange(M), lab] -= 1.0
    du *= dm.s                                                 # dE/du = s (p - onehot)
    dWs = du.T @ Z
    dbs = du.sum(axis=0)
    dz = du @ th["Ws"]
    return loss, dz.reshape(dm.T, dm.B, dm.zdim), dWs, dbs, p


# --------------------------------------------------------------------------- backward

def blstm_backward(dm: Dims, theta: np.ndarray, cache: dict, dz: np.ndarray, want_dx: bool = False):
    """Back-propagation through the bottleneck and through time in every layer.

    Returns the flat gradient with every slice filled except W_s, b_s (zero there);
    with want_dx also the gradient with respect to the input features.
    """
    th = views(np.asarray(theta, dtype=np.float64), dm)
    T, B, H = dm.T, dm.B, dm.H
    M = T * B
    grad = np.zeros(param_count(dm))
    gv = views(grad, dm)
    dZ = np.asarray(dz, dtype=np.float64).reshape(M, dm.zdim)
    if dm.P > 0:
        Yf = cache["Y"].reshape(M, 2 * H)
        gv["Wp"][...] = dZ.T @ Yf
        gv["bp"][...] = dZ.sum(axis=0)
        dY = (dZ @ th["Wp"]).reshape(T, B, 2 * H)
    else:
        dY = dZ.reshape(T, B, 2 * H).copy()
    for l in range(dm.L - 1, -1, -1):
        X = cache["X"][l]
        dX = np.zeros_like(X)
        for d in range(2):
            Wx, Uh = th[f"Wx{l}.{d}"], th[f"Uh{l}.{d}"]
            gi, gf, gg, go = cache["i"][l][d], cache["f"][l][d], cache["g"][l][d], cache["o"][l][d]
            cc, hh = cache["c"][l][d], cache["h"][l][d]
            order = visit_order(T, d)
            dh_rec = np.zeros((B, H)); dc_rec = np.zeros((B, H))
            for n in range(T - 1, -1, -1):                     # reverse of the visiting order
                t = order[n]
                if n > 0:
                    c_prev, h_prev = cc[order[n - 1]], hh[order[n - 1]]
                else:
                    c_prev, h_prev = np.zeros((B, H)), np.zeros((B, H))
                i, f, g, o, c = gi[t], gf[t], gg[t], go[t], cc[t]
                tc = np.tanh(c)
                dh = dY[t, :, d * H:(d + 1) * H] + dh_rec
                da_o = dh * tc * o * (1.0 - o)
                dc = dh * o * (1.0 - tc * tc) + dc_rec
                da_i = dc * g * i * (1.0 - i)
                da_f = dc * c_prev * f * (1.0 - f)
                da_g = dc * i * (1.0 - g * g)
                da = np.concatenate([da_i, da_f, da_g, da_o], axis=1)   # [B, 4H]
                gv[f"Wx{l}.{d}"] += da.T @ X[t]
                gv[f"Uh{l}.{d}"] += da.T @ h_prev
                gv[f"b{l}.{d}"] += da.sum(axis=0)
                dX[t] += da @ Wx
                dh_rec = da @ Uh
                dc_rec = dc * f
        dY = dX
    return (grad, dY) if want_dx else grad


def loss_and_grad(dm: Dims, theta: np.ndarray, x: np.ndarray, labels: np.ndarray, want_dx: bool = False):
    """g = calGrad(W) of section 3.2: the loss and the full flat gradient."""
    z, cache = blstm_forward(dm, theta, x)
    loss, dz, dWs, dbs, _ = softmax_xent_fwd_bwd(dm, theta, z, labels)
    r = blstm_backward(dm, theta, cache, dz, want_dx=want_dx)
    grad = r[0] if want_dx else r
    gv = views(grad, dm)
    gv["Ws"][...] = dWs
    gv["bs"][...] = dbs
    return (loss, grad, r[1]) if want_dx else (loss, grad)


def loss_only(dm: Dims, theta: np.ndarray, x: np.ndarray, labels: np.ndarray) -> float:
    z, _ = blstm_forward(dm, theta, x)
    return softmax_xent_fwd_bwd(dm, theta, z, labels)[0]


# --------------------------------------------------------------------------- update rules

def sgd_step(theta: np.ndarray, grad: np.ndarray, lr: float, momentum: float = 0.0, velocity=None):
    """W' = apply(W, g): Eq. 1c; with momentum, v <- mu v + g then theta <- theta - alpha v.

    Returns (theta_new, velocity_new); velocity_new is None when momentum == 0.
    """
    th = np.asarray(theta, dtype=np.float64)
    g = np.asarray(grad, dtype=np.float64)
    if momentum == 0.0:
        return th - lr * g, None
    v = momentum * np.asarray(velocity, dtype=np.float64) + g
    return th - lr * v, v


def adpsgd_ring_partner(R: int, step: int):
    """The matching of one iteration on a ring of R learners (R even), section 3.2.

    Learners 0, 2, 4, ... are the senders; on even steps sender i pairs with its
    right neighbour i+1, on odd steps with its left neighbour (i-1) mod R.  The
    result is an involution: partner[partner[i]] == i.
    """
    if R < 2 or R % 2:
        raise ValueError("ring needs an even number of learners")
    partner = [-1] * R
    for i in range(0, R, 2):
        j = (i + 1) % R if step % 2 == 0 else (i - 1) % R
        partner[i] = j
        partner[j] = i
    return partner


def adpsgd_mix(thetas, partner):
    """Second line of Eq. 4 for every pair of the matching; partner[i]==i leaves i untouched."""
    R = len(thetas)
    out = [None] * R
    for i in range(R):
        j = partner[i]
        if partner[j] != i:
            raise ValueError("partner is not an involution")
        a = np.asarray(thetas[i], dtype=np.float64)
        if j == i:
            out[i] = a.copy()
        else:
            out[i] = (a + np.asarray(thetas[j], dtype=np.float64)) / 2.0
    return out


def mixing_matrix(partner):
    """The R x R matrix W with theta(t+1) = W theta'(t) for one matching."""
    R = len(partner)
    W = np.zeros((R, R))
    for i, j in enumerate(partner):
        if i == j:
            W[i, i] = 1.0
        else:
            W[i, i] = 0.5
            W[i, j] = 0.5
    return W


def lr_schedule(epoch: int, base_lr: float, peak_lr: float, warmup_epochs: int = 10, anneal_from: int = 11):
    """Learning rate of a 1-based epoch (section 3.1): linear warm-up from base_lr to
    peak_lr over the first warmup_epochs epochs, then a factor 1/sqrt(2) per epoch from
    epoch anneal_from on.  With base_lr == peak_lr it is the batch-256 recipe."""
    if epoch <= warmup_epochs:
        if warmup_epochs <= 1:
            return peak_lr
        return base_lr + (peak_lr - base_lr) * (epoch - 1) / (warmup_epochs - 1)
    k = max(0, epoch - anneal_from + 1)
    return peak_lr * (2.0 ** (-0.5 * k))


def sgd_mix_pair(theta_i, theta_j, grad_i, grad_j, lr, momentum=0.0, velocity_i=None, velocity_j=None):
    """Both lines of Eq. 4 for one pair: each replica takes its own step of Eq. 1c, then both become
    the average of the two results.  Returns (theta_new, velocity_i_new, velocity_j_new); theta_new is
    the common value of both replicas."""
    ti, vi = sgd_step(theta_i, grad_i, lr, momentum, velocity_i)
    tj, vj = sgd_step(theta_j, grad_j, lr, momentum, velocity_j)
    return (ti + tj) / 2.0, vi, vj


def sync_average(thetas):
    """SYNC of section 3.2 (Fig. 3a): W = allreduce(W') / lambda: every learner ends with the mean of
    all learners' updated weights."""
    m = np.mean(np.stack([np.asarray(t, dtype=np.float64) for t in thetas]), axis=0)
    return [m.copy() for _ in thetas]


def stale_adpsgd_step(thetas, grads, partner, lr):
    """One iteration in the integration order of Fig. 3b: g = calGrad(W) on the learner's own weights,
    W = pull_weights() (the average of what the pair pushed at the end of the previous iteration, which
    is what each learner now holds), W' = apply(W, g), push_weights(W').  grads[i] must have been
    computed on thetas[i]; the gradient is therefore one averaging step stale when it is applied."""
    pulled = adpsgd_mix(thetas, partner)
    return [sgd_step(pulled[i], grads[i], lr)[0] for i in range(len(thetas))]


def hybrid_step(pushed, grads, lr):
    """One iteration of HYBRID in the integration order of Fig. 3c, whose push is an AllReduce over all
    learners (section 3.2): g = calGrad(W) on the weights W the learner pulled in the iteration before,
    W = pull_weights() = the mean of what all learners pushed at the end of that iteration,
    W' = apply(W, g), push_weights(W').  pushed[i] is learner i's W' of the iteration before and grads[i]
    its gradient on the W it pulled then, so the gradient is one iteration stale when applied (Table 1).
    Returns (pushed_new, pulled): the W' the learners push now, and the common W they hold for the next
    gradient.  Before the first iteration every learner holds and has pushed the common initial weights."""
    pulled = np.mean(np.stack([np.asarray(t, dtype=np.float64) for t in pushed]), axis=0)
    return [sgd_step(pulled, grads[i], lr)[0] for i in range(len(pushed))], pulled
