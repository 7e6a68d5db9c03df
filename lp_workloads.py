"""Seeded synthetic workloads for the LayerPipe hot path (shapes, delay vectors, random inputs).

This module is shared by the CPU oracle's tests and by the HIP path's tests and benchmark.  It holds
*no* arithmetic of the method itself: only network shapes, the per-layer delay rule of Sec. III-A
(the count of delay elements on a layer's gradient->update edge is twice the number of stages that
follow it) and counter-based random draws for weights, inputs and targets.

Random stream: numpy's Philox generator keyed by ``(seed, step, tensor_id)`` so that any tensor of any
step can be regenerated on its own, on either side, in any order.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

# layer kinds / activations / losses / dtypes: plain strings on the Python side
LINEAR, CONV3X3 = "linear", "conv3x3"
IDENTITY, RELU, GELU, TANH, SIGMOID = "identity", "relu", "gelu", "tanh", "sigmoid"
SOFTMAX_CE, MSE = "softmax_ce", "mse"

# tensor ids inside one (seed, step) stream
_T_INPUT, _T_TARGET = 1, 2


@dataclass(frozen=True)
class Layer:
    kind: str          # LINEAR | CONV3X3
    d_in: int          # input features (linear) or input channels (conv)
    d_out: int         # output features (linear) or output channels (conv)
    act: str           # IDENTITY | RELU | GELU
    H: int = 0         # conv only: input height (= output height, stride 1 pad 1)
    W: int = 0         # conv only: input width
    pool: int = 0      # conv only: 0, or 2 for a 2x2 stride-2 max-pool after the activation

    @property
    def fan_in(self) -> int:
        return self.d_in if self.kind == LINEAR else 9 * self.d_in

    @property
    def weight_shape(self) -> Tuple[int, ...]:
        # linear: [in, out]; conv: [kh, kw, c_in, c_out] (reduction index (kh, kw, c_in) is row-major)
        return (self.d_in, self.d_out) if self.kind == LINEAR else (3, 3, self.d_in, self.d_out)

    @property
    def n_params(self) -> int:
        return int(np.prod(self.weight_shape))

    def in_shape(self, batch: int) -> Tuple[int, ...]:
        return (batch, self.d_in) if self.kind == LINEAR else (batch, self.H, self.W, self.d_in)

    def out_shape(self, batch: int) -> Tuple[int, ...]:
        """Shape of the layer's activation output (after the pool, if any)."""
        if self.kind == LINEAR:
            return (batch, self.d_out)
        p = 2 if self.pool == 2 else 1
        return (batch, self.H // p, self.W // p, self.d_out)

    def z_shape(self, batch: int) -> Tuple[int, ...]:
        """Shape of the product z before activation and pool."""
        return (batch, self.d_out) if self.kind == LINEAR else (batch, self.H, self.W, self.d_out)


def delays_for(n_layers: int, stages_after: Optional[List[int]] = None) -> List[int]:
    """Delay count on each layer's gradient->update edge: 2 x (stages after the layer), Sec. III-A.

    With one stage per layer and the last layer feeding the loss directly this is 2*(L-l), l=1..L.
    """
    if stages_after is None:
        stages_after = [n_layers - l for l in range(1, n_layers + 1)]
    return [2 * s for s in stages_after]


@dataclass(frozen=True)
class Workload:
    name: str
    layers: Tuple[Layer, ...]
    batch: int
    dtype: str                 # "f32" | "bf16" (bf16 = bf16 working tensors, fp32 master weights)
    loss: str
    lr: float
    steps: int
    weight_seed: int
    data_seed: int
    delays: Tuple[int, ...] = field(default=())

    @property
    def L(self) -> int:
        return len(self.layers)

    @property
    def n_params(self) -> int:
        return sum(l.n_params for l in self.layers)

    def with_(self, **kw) -> "Workload":
        d = dict(self.__dict__)
        d.update(kw)
        return Workload(**d)

    # ---- per-step algorithmic work, used by the benchmark's roofline arithmetic ----
    def gemm_dims(self, l: int) -> Tuple[int, int, int]:
        """(M, N, K) of layer l's (0-based) forward product seen as a GEMM."""
        ly = self.layers[l]
        if ly.kind == LINEAR:
            return (self.batch, ly.d_out, ly.d_in)
        return (self.batch * ly.H * ly.W, ly.d_out, 9 * ly.d_in)

    def flops_per_step(self) -> Tuple[float, float, float]:
        """Flops of the F, dX and dW products of one step (2*M*N*K each; no dX for layer 1)."""
        f = dx = dw = 0.0
        for l in range(self.L):
            m, n, k = self.gemm_dims(l)
            f += 2.0 * m * n * k
            dw += 2.0 * m * n * k
            if l > 0:
                dx += 2.0 * m * n * k
        return f, dx, dw


def _mlp(widths: List[int], act: str) -> Tuple[Layer, ...]:
    L = len(widths) - 1
    return tuple(Layer(LINEAR, widths[i], widths[i + 1], act if i < L - 1 else IDENTITY) for i in range(L))


def _mk(name, layers, batch, dtype, loss, lr, steps, idx) -> Workload:
    return Workload(name, tuple(layers), batch, dtype, loss, lr, steps,
                    weight_seed=0x4C500000 + idx, data_seed=0xDA7A0000 + idx,
                    delays=tuple(delays_for(len(layers))))


def mlp_small() -> Workload:
    """4-layer ReLU MLP 784-256-128-64-10, fp32, batch 32, 8 steps."""
    return _mk("mlp_small_f32", _mlp([784, 256, 128, 64, 10], RELU), 32, "f32", SOFTMAX_CE, 0.01, 8, 1)


def mlp_4096() -> Workload:
    """8-layer ReLU MLP, widths 4096, 1000 classes, bf16 + fp32 master, batch 256, 50 steps."""
    return _mk("mlp_4096_bf16", _mlp([4096] * 8 + [1000], RELU), 256, "bf16", SOFTMAX_CE, 1e-3, 50, 2)


def vgg_small(batch: int = 128, hw: int = 32, chans=(64, 64, 128, 128, 256, 256)) -> Workload:
    """VGG-style CNN on hw x hw x 3 inputs: three (conv, conv+pool) pairs, then FC -> 10 classes."""
    layers, c_in, s = [], 3, hw
    for i, c in enumerate(chans):
        pool = 2 if i % 2 == 1 else 0
        layers.append(Layer(CONV3X3, c_in, c, RELU, H=s, W=s, pool=pool))
        c_in = c
        if pool:
            s //= 2
    layers.append(Layer(LINEAR, s * s * c_in, 10, IDENTITY))
    return _mk("vgg_small_bf16", layers, batch, "bf16", SOFTMAX_CE, 1e-3, 20, 3)


def ffn_stack(d: int = 4096, hidden: int = 16384, tokens: int = 8192, n_linear: int = 16) -> Workload:
    """Transformer-MLP shaped stack: n_linear/2 x (d -> hidden GELU, hidden -> d identity), MSE loss."""
    layers = []
    for i in range(n_linear):
        layers.append(Layer(LINEAR, d, hidden, GELU) if i % 2 == 0 else Layer(LINEAR, hidden, d, IDENTITY))
    # lr: the configuration names none; 1e-3 diverges under the 2(L-l) delay schedule (in the CPU
    # oracle as well), 1e-5 trains
    return _mk("ffn_stack_bf16", layers, tokens, "bf16", MSE, 1e-5, 10, 4)


def mlp_imbalanced() -> Workload:
    """12-layer ReLU MLP with uneven widths (input width 1024), batch 1024, bf16."""
    outs = [1024, 8192, 2048, 8192, 1024, 4096, 8192, 2048, 4096, 1024, 8192, 1000]
    return _mk("mlp_imbalanced_bf16", _mlp([1024] + outs, RELU), 1024, "bf16", SOFTMAX_CE, 1e-3, 10, 5)


CONFIGS = {
    "mlp_small_f32": mlp_small,
    "mlp_4096_bf16": mlp_4096,
    "vgg_small_bf16": vgg_small,
    "ffn_stack_bf16": ffn_stack,
    "mlp_imbalanced_bf16": mlp_imbalanced,
}


# --------------------------------------------------------------------------------------------------
# random draws
# --------------------------------------------------------------------------------------------------
def _rng(seed: int, step: int, tensor: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, (step << 16) | tensor]))


def init_weights(wl: Workload) -> List[np.ndarray]:
    """He-normal weights (std = sqrt(2 / fan_in)), fp32, one array per layer in `weight_shape` layout."""
    out = []
    for l, ly in enumerate(wl.layers):
        g = _rng(wl.weight_seed, 0, 100 + l)
        w = g.standard_normal(ly.weight_shape, dtype=np.float32)
        w *= np.float32(np.sqrt(2.0 / ly.fan_in))
        out.append(w)
    return out


def batch_input(wl: Workload, step: int) -> np.ndarray:
    """Input minibatch of training step `step` (1-based): N(0,1), fp32."""
    return _rng(wl.data_seed, step, _T_INPUT).standard_normal(wl.layers[0].in_shape(wl.batch), dtype=np.float32)


def batch_target(wl: Workload, step: int) -> np.ndarray:
    """Labels (int32, uniform over classes) for softmax-CE, or N(0,1) fp32 targets for MSE."""
    g = _rng(wl.data_seed, step, _T_TARGET)
    last = wl.layers[-1]
    if wl.loss == SOFTMAX_CE:
        return g.integers(0, last.d_out, size=(wl.batch,), dtype=np.int32)
    return g.standard_normal(last.out_shape(wl.batch), dtype=np.float32)
