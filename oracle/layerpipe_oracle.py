"""CPU oracle for the LayerPipe delayed-gradient training step.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this file; the HIP
library never does, and this file imports nothing from it.  Everything here is plain numpy in
float64, one function per operator of the paper, written so it can be checked against the paper
by eye: no blocking, no fusion, no reordering.

What the method computes (Sec. II-A, Sec. III-A), in batched row-major form: the paper's
column-vector z = W a becomes Z = A_prev @ W with the stored weight W = (paper's W)^T of shape
[in, out]; delta^l is called dY_l, dE/da^{l-1} is called dA_{l-1}, G^l has the shape of W.

  Eq. 1   Z_l  = A_{l-1} @ W_l              (or 3x3 cross-correlation, stride 1, zero pad 1)
  Eq. 2   A_l  = f(Z_l)                     (then optional 2x2/2 max-pool for conv layers)
  Eq. 4   dA_{l-1} = dY_l @ W_l^T
  Eq. 3   dY_{l-1} = dA_{l-1} (.) f'(Z_{l-1})
  Eq. 5   G_l  = A_{l-1}^T @ dY_l
  Eq. 6   W_l(n) = W_l(n-1) - eta * G_l(n - d_l)   (no update while n - d_l < 1)

Retiming does not change what a data-flow graph computes (Sec. III-A), so the fully pipelined
system equals ordinary back-propagation with d_l delay elements on layer l's gradient->update edge;
that un-retimed graph is what `DelayedGradientTrainer` replays.

Readings where the paper is silent (each also listed in the design notes): no bias terms; the output
layer has identity activation; the loss is softmax cross-entropy averaged over the batch, or the
mean squared error over batch x features; ReLU'(0) = 0; GELU is the exact erf form; the delay
elements start empty, so a layer is not updated while n <= d_l; max-pool ties go to the first
maximum in (row, column) order of the 2x2 window.

Storage rounding: the HIP path keeps working weights, activations and their gradients in bf16 (or
fp32) while G, the master weights and the loss stay fp32.  `storage="bf16"|"f32"` rounds exactly
those stored tensors (round-to-nearest-even) so that discrete decisions (ReLU mask, pool argmax)
are taken on inputs of the same precision on both sides; `storage="f64"` rounds nothing.

Parity status: every function is pinned by tests/test_oracle_*.py (finite differences, an
independent autograd library at zero delay and on a brute-force delayed replay, closed forms).
The numeric trajectories of the five benchmark workloads are "parity unpinned" by the paper itself:
it prints no numeric example of this path.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf

__all__ = [
    "round_bf16", "store", "activation", "activation_derivative", "forward_product", "conv3x3",
    "conv3x3_grad_act", "conv3x3_grad_weight", "maxpool2x2", "maxpool2x2_backward", "softmax_ce",
    "mse", "grad_act", "grad_weight", "act_grad", "delta_prev_unsplit", "delayed_sgd",
    "DelayedGradientTrainer",
]


# --------------------------------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------------------------------
def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bfloat16 (ties to even), returned as float64.  Input goes through fp32."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = ((u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)) << np.uint64(16)
    out = r.astype(np.uint32).view(np.float32)
    out = np.where(np.isnan(f), f, out)
    return out.astype(np.float64).reshape(np.shape(x))


def store(x: np.ndarray, storage: str) -> np.ndarray:
    """Value of `x` after being written to a tensor of the given storage type, as float64."""
    if storage == "f64":
        return np.asarray(x, dtype=np.float64)
    if storage == "f32":
        return np.asarray(x, dtype=np.float32).astype(np.float64)
    if storage == "bf16":
        return round_bf16(x)
    raise ValueError(storage)


# --------------------------------------------------------------------------------------------------
# Eq. 2 and the f' factor of Eq. 3
# --------------------------------------------------------------------------------------------------
def activation(z: np.ndarray, act: str) -> np.ndarray:
    if act == "identity":
        return z.copy()
    if act == "relu":
        return np.where(z > 0.0, z, 0.0)
    if act == "gelu":
        return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))
    if act == "tanh":
        return np.tanh(z)
    if act == "sigmoid":
        return 1.0 / (1.0 + np.exp(-z))
    raise ValueError(act)


def activation_derivative(z: np.ndarray, act: str) -> np.ndarray:
    if act == "identity":
        return np.ones_like(z)
    if act == "relu":
        return np.where(z > 0.0, 1.0, 0.0)
    if act == "gelu":
        cdf = 0.5 * (1.0 + erf(z / np.sqrt(2.0)))
        pdf = np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)
        return cdf + z * pdf
    if act == "tanh":
        return 1.0 - np.tanh(z) ** 2
    if act == "sigmoid":
        s = 1.0 / (1.0 + np.exp(-z))
        return s * (1.0 - s)
    raise ValueError(act)


# --------------------------------------------------------------------------------------------------
# Eq. 1 / 4 / 5 for a fully connected layer and for a 3x3 convolution
# --------------------------------------------------------------------------------------------------
def conv3x3(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """z[b,y,x,o] = sum_{kh,kw,c} xpad[b, y+kh, x+kw, c] * w[kh,kw,c,o]; xpad = x zero-padded by 1."""
    B, H, W, C = x.shape
    xp = np.zeros((B, H + 2, W + 2, C))
    xp[:, 1:H + 1, 1:W + 1, :] = x
    z = np.zeros((B, H, W, w.shape[3]))
    for kh in range(3):
        for kw in range(3):
            z += xp[:, kh:kh + H, kw:kw + W, :] @ w[kh, kw]
    return z


def conv3x3_grad_act(dy: np.ndarray, w: np.ndarray) -> np.ndarray:
    """dE/dx of `conv3x3`: every product term x*w of the forward sum sends dy*w back to its x."""
    B, H, W, O = dy.shape
    dxp = np.zeros((B, H + 2, W + 2, w.shape[2]))
    for kh in range(3):
        for kw in range(3):
            dxp[:, kh:kh + H, kw:kw + W, :] += dy @ w[kh, kw].T
    return dxp[:, 1:H + 1, 1:W + 1, :]


def conv3x3_grad_weight(x: np.ndarray, dy: np.ndarray) -> np.ndarray:
    """G[kh,kw,c,o] = sum_{b,y,x} xpad[b, y+kh, x+kw, c] * dy[b,y,x,o]."""
    B, H, W, C = x.shape
    xp = np.zeros((B, H + 2, W + 2, C))
    xp[:, 1:H + 1, 1:W + 1, :] = x
    g = np.zeros((3, 3, C, dy.shape[3]))
    for kh in range(3):
        for kw in range(3):
            g[kh, kw] = np.tensordot(xp[:, kh:kh + H, kw:kw + W, :], dy, axes=([0, 1, 2], [0, 1, 2]))
    return g


def forward_product(a_prev: np.ndarray, w: np.ndarray) -> np.ndarray:
    """Eq. 1.  2-D weight: Z = A_prev @ W.  4-D weight: 3x3 cross-correlation."""
    return a_prev @ w if w.ndim == 2 else conv3x3(a_prev, w)


def grad_act(dy: np.ndarray, w: np.ndarray, col0: int = 0, col1: int | None = None) -> np.ndarray:
    """Eq. 4: dA_prev = dY @ W^T (or its conv form).

    `[col0, col1)` selects a range of the previous layer's features (input channels): the
    output-channel partition of the delta computation into delta' and delta'' of Sec. III-B.
    """
    if w.ndim == 2:
        col1 = w.shape[0] if col1 is None else col1
        return dy @ w[col0:col1, :].T
    col1 = w.shape[2] if col1 is None else col1
    return conv3x3_grad_act(dy, w[:, :, col0:col1, :])


def grad_weight(a_prev: np.ndarray, dy: np.ndarray) -> np.ndarray:
    """Eq. 5: G = A_prev^T @ dY (sum over the batch), or its conv form."""
    return a_prev.T @ dy if a_prev.ndim == 2 else conv3x3_grad_weight(a_prev, dy)


# --------------------------------------------------------------------------------------------------
# 2x2 stride-2 max-pool
# --------------------------------------------------------------------------------------------------
def maxpool2x2(a: np.ndarray):
    """Returns (pooled, idx); idx in 0..3 = 2*dy+dx of the first maximum of each window."""
    B, H, W, C = a.shape
    win = np.stack([a[:, 0::2, 0::2, :], a[:, 0::2, 1::2, :], a[:, 1::2, 0::2, :], a[:, 1::2, 1::2, :]], axis=0)
    idx = np.argmax(win, axis=0)  # numpy returns the first occurrence of the maximum
    pooled = np.take_along_axis(win, idx[None], axis=0)[0]
    return pooled, idx


def maxpool2x2_backward(dpooled: np.ndarray, idx: np.ndarray) -> np.ndarray:
    B, h, w, C = dpooled.shape
    da = np.zeros((B, 2 * h, 2 * w, C))
    for k in range(4):
        da[:, (k // 2)::2, (k % 2)::2, :] = np.where(idx == k, dpooled, 0.0)
    return da


# --------------------------------------------------------------------------------------------------
# error at the output (the paper only says the error is computed from the ground truth)
# --------------------------------------------------------------------------------------------------
def softmax_ce(z: np.ndarray, labels: np.ndarray):
    """E = -mean_b log softmax(z_b)[y_b];  dY = (softmax(z) - onehot(y)) / B."""
    B = z.shape[0]
    s = z - z.max(axis=1, keepdims=True)
    e = np.exp(s)
    p = e / e.sum(axis=1, keepdims=True)
    logp = s - np.log(e.sum(axis=1, keepdims=True))
    loss = -logp[np.arange(B), labels].mean()
    dy = p.copy()
    dy[np.arange(B), labels] -= 1.0
    return loss, dy / B


def mse(z: np.ndarray, t: np.ndarray):
    """E = mean over batch x features of (z - t)^2;  dY = 2 (z - t) / (B * D)."""
    d = z - t
    return (d * d).mean(), 2.0 * d / d.size


# --------------------------------------------------------------------------------------------------
# Eq. 3: the Hadamard part, in the form that runs where Z_l lives (the previous layer's stage)
# --------------------------------------------------------------------------------------------------
def act_grad(da: np.ndarray, z: np.ndarray, act: str, pool_idx: np.ndarray | None = None) -> np.ndarray:
    """dY_l = dA_l (.) f'(Z_l).  For a pooled conv layer dA_l arrives at pooled resolution and is
    first routed back through the max-pool."""
    if pool_idx is not None:
        da = maxpool2x2_backward(da, pool_idx)
    return da * activation_derivative(z, act)


def delta_prev_unsplit(dy: np.ndarray, w: np.ndarray, z_prev: np.ndarray, act_prev: str) -> np.ndarray:
    """Eq. 3 with Eq. 4 substituted, one loop nest, fully connected layers only: the conventional
    placement of the whole delta computation in one task.  Exists to be compared with the split form
    `act_grad(grad_act(...))`."""
    B, D_prev = z_prev.shape
    out = np.zeros((B, D_prev))
    fprime = activation_derivative(z_prev, act_prev)
    for b in range(B):
        for k in range(D_prev):
            out[b, k] = np.dot(dy[b, :], w[k, :]) * fprime[b, k]
    return out


# --------------------------------------------------------------------------------------------------
# Eq. 6
# --------------------------------------------------------------------------------------------------
def delayed_sgd(w: np.ndarray, g_delayed: np.ndarray | None, eta: float) -> np.ndarray:
    """W(n) = W(n-1) - eta * G(n-M); `None` stands for an empty delay element (no update)."""
    return w.copy() if g_delayed is None else w - eta * g_delayed


# --------------------------------------------------------------------------------------------------
# the whole iteration
# --------------------------------------------------------------------------------------------------
class DelayedGradientTrainer:
    """Replays back-propagation with d_l delay elements between layer l's G and its weight update.

    `layers`: objects with .kind ("linear"|"conv3x3"), .act, .pool; `weights`: list of arrays in
    [in, out] / [3,3,c_in,c_out] layout.  Step numbers n are 1-based as in Eq. 6.
    """

    def __init__(self, layers, weights, delays, lr, loss, storage="f64", split=True):
        assert len(layers) == len(weights) == len(delays)
        assert all(int(d) >= 0 for d in delays)
        self.layers = list(layers)
        self.delays = [int(d) for d in delays]
        self.loss_kind = loss
        self.storage = storage
        self.split = split
        self.master = "f64" if storage == "f64" else "f32"
        self.eta = float(lr) if storage == "f64" else float(np.float32(lr))
        self.W = [store(w, self.master) for w in weights]
        self.G_hist = [dict() for _ in layers]   # step number -> G_l(step)
        self.n = 0
        self.trace = {}

    def _q(self, x):
        return store(x, self.storage)

    def step(self, x, target):
        L = len(self.layers)
        self.n += 1
        n = self.n
        q = self._q
        Wk = [q(w) for w in self.W]                 # working copies: W_l(n-1) for F *and* dX
        A = [q(x)]
        Z, IDX = [], []
        for l, ly in enumerate(self.layers):
            z = q(forward_product(A[l], Wk[l]))     # Eq. 1
            a = q(activation(z, ly.act))            # Eq. 2
            idx = None
            if getattr(ly, "pool", 0) == 2:
                a, idx = maxpool2x2(a)
            if l + 1 < L and self.layers[l + 1].kind == "linear" and a.ndim == 4:
                a = a.reshape(a.shape[0], -1)       # NHWC flatten in front of a fully connected layer
            Z.append(z); IDX.append(idx); A.append(a)

        zL = Z[-1].reshape(Z[-1].shape[0], -1)
        if self.loss_kind == "softmax_ce":
            loss, dyL = softmax_ce(zL, np.asarray(target))
        else:
            loss, dyL = mse(zL, q(np.asarray(target)).reshape(zL.shape))
        dY = [None] * L
        dA = [None] * L
        dY[L - 1] = q(dyL.reshape(Z[-1].shape))     # output layer: identity activation, f' = 1

        G = [None] * L
        for l in range(L - 1, -1, -1):
            ly = self.layers[l]
            G[l] = grad_weight(A[l], dY[l])                                      # Eq. 5
            if l == 0:
                break
            prev = self.layers[l - 1]
            if self.split or prev.kind != "linear" or ly.kind != "linear":
                da = q(grad_act(dY[l], Wk[l]))                                   # Eq. 4, layer l's task
                if IDX[l - 1] is not None:
                    da = da.reshape(IDX[l - 1].shape)
                elif da.shape != Z[l - 1].shape:
                    da = da.reshape(Z[l - 1].shape)
                dA[l - 1] = da
                dY[l - 1] = q(act_grad(da, Z[l - 1], prev.act, IDX[l - 1]))      # Eq. 3, layer l-1's stage
            else:
                # conventional placement; stored-precision rounding of the intermediate is skipped
                dY[l - 1] = q(delta_prev_unsplit(dY[l], Wk[l], Z[l - 1], prev.act))

        for l in range(L):                          # Eq. 6 with M = d_l
            src = n - self.delays[l]
            g_old = None
            if src >= 1:
                g_old = G[l] if src == n else self.G_hist[l].pop(src)
            self.W[l] = store(delayed_sgd(self.W[l], g_old, self.eta), self.master)
            if self.delays[l] > 0:
                self.G_hist[l][n] = G[l]

        self.trace = dict(loss=float(loss), A=A, Z=Z, dA=dA, dY=dY, G=G, IDX=IDX, Wk=Wk)
        return float(loss)
