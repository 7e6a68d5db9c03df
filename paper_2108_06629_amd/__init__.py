"""Python binding of liblayerpipe.so (include/lp.h): argument marshalling only.

Every arithmetic step of the training path runs in the HIP kernels of the shared library; PyTorch
is used here for device memory (the workspace and the input/target tensors) and for stream handles.
There is no CPU fallback: if the library is missing or was not built, importing succeeds but the
first call raises.

Two layers of API:
  * `lib()` returns the ctypes handle with every `lp_*` function of the header declared; the
    functions of the same names in this module forward to it and raise `LpError` on a non-zero
    status.
  * `Network` owns a context, its workspace tensor and three streams, and converts numpy inputs.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblayerpipe.so")

LP_F32, LP_BF16 = 0, 1
LP_LOSS_SOFTMAX_CE, LP_LOSS_MSE = 0, 1
LP_LINEAR, LP_CONV3X3 = 0, 1
LP_ACT_IDENTITY, LP_ACT_RELU, LP_ACT_GELU, LP_ACT_TANH, LP_ACT_SIGMOID = 0, 1, 2, 3, 4
LP_T_MASTER_W, LP_T_WORK_W, LP_T_A, LP_T_Z, LP_T_DA, LP_T_DY, LP_T_G_LAST = range(7)
LP_TASK_F, LP_TASK_DX, LP_TASK_DW, LP_TASK_HADAMARD, LP_TASK_LOSS, LP_TASK_UPDATE = range(6)
TASK_NAMES = ["F", "dX", "dW", "hadamard", "loss", "update"]
STATUS_NAMES = ["LP_OK", "LP_ERR_NULL", "LP_ERR_SHAPE", "LP_ERR_DTYPE", "LP_ERR_LAYER", "LP_ERR_DELAY",
                "LP_ERR_STATE", "LP_ERR_WORKSPACE", "LP_ERR_HIP"]

EXPORTS = ["lp_create", "lp_destroy", "lp_last_error", "lp_workspace_bytes", "lp_bind_workspace", "lp_set_weights",
           "lp_get_weights", "lp_cast", "lp_forward", "lp_loss_grad", "lp_loss_grad_static", "lp_act_grad", "lp_grad_act", "lp_grad_weight", "lp_update",
           "lp_advance", "lp_step", "lp_step_index", "lp_sync", "lp_tensor", "lp_profile", "lp_profile_read", "lp_profile_read_layer", "lp_partition", "lp_set_delta_split", "lp_set_run_ahead", "lp_set_graphs", "lp_graph_stats", "lp_set_factor_ring", "lp_set_retimed_update", "lp_set_fused_hadamard", "lp_probe_mfma"]


class lp_layer_desc(C.Structure):
    _fields_ = [("kind", C.c_int), ("in_", C.c_int), ("out", C.c_int), ("H", C.c_int), ("W", C.c_int),
                ("act", C.c_int), ("pool", C.c_int), ("delay", C.c_int)]


class LpError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__("%s: %s" % (STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status, msg))
        self.status = status


_lib = None


def load_library():
    """Loads liblayerpipe.so and declares the prototypes of include/lp.h."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("liblayerpipe.so is not built: run `python __graft_entry__.py` (hipcc, gfx950) first")
    L = C.CDLL(LIB_PATH)
    vp, ip, fp = C.c_void_p, C.c_int, C.c_float
    L.lp_create.argtypes = [C.POINTER(lp_layer_desc), ip, ip, ip, ip, fp, C.POINTER(vp)]
    L.lp_destroy.argtypes = [vp]
    L.lp_last_error.argtypes = [vp]
    L.lp_last_error.restype = C.c_char_p
    L.lp_workspace_bytes.argtypes = [vp, C.POINTER(C.c_size_t)]
    L.lp_bind_workspace.argtypes = [vp, vp, C.c_size_t]
    L.lp_set_weights.argtypes = [vp, ip, vp, ip, vp]
    L.lp_get_weights.argtypes = [vp, ip, vp, ip, vp]
    L.lp_cast.argtypes = [vp, vp, vp, C.c_size_t, vp]
    L.lp_forward.argtypes = [vp, ip, vp, vp, vp, vp]
    L.lp_loss_grad.argtypes = [vp, vp, vp, vp, vp, vp]
    L.lp_loss_grad_static.argtypes = [vp, vp, vp, vp, vp, vp]
    L.lp_act_grad.argtypes = [vp, ip, vp, vp, vp, vp]
    L.lp_grad_act.argtypes = [vp, ip, vp, vp, ip, ip, vp]
    L.lp_grad_weight.argtypes = [vp, ip, vp, vp, vp, vp]
    L.lp_update.argtypes = [vp, ip, vp, vp]
    L.lp_advance.argtypes = [vp]
    L.lp_step.argtypes = [vp, vp, vp, C.POINTER(ip), vp, C.POINTER(vp), ip]
    L.lp_step_index.argtypes = [vp, C.POINTER(C.c_long)]
    L.lp_sync.argtypes = [vp]
    L.lp_tensor.argtypes = [vp, ip, ip, C.POINTER(vp), C.POINTER(C.c_size_t)]
    dp = C.POINTER(C.c_double)
    L.lp_partition.argtypes = [dp, dp, ip, ip, C.c_double, C.POINTER(ip), C.POINTER(ip), dp, dp, dp]
    L.lp_set_delta_split.argtypes = [vp, ip, ip]
    L.lp_probe_mfma.argtypes = [vp, C.c_size_t, ip, ip, ip, vp]
    L.lp_set_run_ahead.argtypes = [vp, ip]
    L.lp_set_fused_hadamard.argtypes = [vp, ip]
    L.lp_set_graphs.argtypes = [vp, ip]
    L.lp_set_factor_ring.argtypes = [vp, ip, ip]
    L.lp_set_retimed_update.argtypes = [vp, ip, ip]
    L.lp_graph_stats.argtypes = [vp, C.POINTER(C.c_long), C.POINTER(C.c_long), C.POINTER(C.c_long)]
    L.lp_profile_read_layer.argtypes = [vp, ip, ip, C.POINTER(C.c_double), C.POINTER(C.c_long), ip]
    L.lp_profile.argtypes = [vp, ip]
    L.lp_profile_read.argtypes = [vp, ip, C.POINTER(C.c_double), C.POINTER(C.c_long), ip]
    for name in EXPORTS:
        if name != "lp_last_error":
            getattr(L, name).restype = ip
    _lib = L
    return L


def lib():
    return load_library()


def _check(ctx, status: int):
    if status != 0:
        msg = lib().lp_last_error(ctx)
        raise LpError(status, msg.decode() if msg else "")


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    return s if isinstance(s, int) else s.cuda_stream


_KIND = {"linear": LP_LINEAR, "conv3x3": LP_CONV3X3}
_ACT = {"identity": LP_ACT_IDENTITY, "relu": LP_ACT_RELU, "gelu": LP_ACT_GELU, "tanh": LP_ACT_TANH, "sigmoid": LP_ACT_SIGMOID}
_LOSS = {"softmax_ce": LP_LOSS_SOFTMAX_CE, "mse": LP_LOSS_MSE}
_DTYPE = {"f32": LP_F32, "bf16": LP_BF16}


def make_descs(layers, delays) -> "C.Array[lp_layer_desc]":
    arr = (lp_layer_desc * len(layers))()
    for i, (ly, d) in enumerate(zip(layers, delays)):
        arr[i] = lp_layer_desc(_KIND[ly.kind], ly.d_in, ly.d_out, ly.H, ly.W, _ACT[ly.act], ly.pool, int(d))
    return arr


# ---- functions of the header, same names, status -> exception ---------------------------------------
def lp_create(descs, L: int, batch: int, dtype: int, loss: int, lr: float) -> C.c_void_p:
    ctx = C.c_void_p()
    _check(None, lib().lp_create(descs, L, batch, dtype, loss, lr, C.byref(ctx)))
    return ctx


def lp_destroy(ctx):
    lib().lp_destroy(ctx)


def lp_workspace_bytes(ctx) -> int:
    n = C.c_size_t()
    _check(ctx, lib().lp_workspace_bytes(ctx, C.byref(n)))
    return n.value


def lp_bind_workspace(ctx, dev_ptr, nbytes: int):
    _check(ctx, lib().lp_bind_workspace(ctx, _ptr(dev_ptr), nbytes))


def lp_set_weights(ctx, l: int, W, is_device: bool = False, stream=None):
    _check(ctx, lib().lp_set_weights(ctx, l, _ptr(W), int(is_device), _stream(stream)))


def lp_get_weights(ctx, l: int, dst, is_device: bool = False, stream=None):
    _check(ctx, lib().lp_get_weights(ctx, l, _ptr(dst), int(is_device), _stream(stream)))


def lp_cast(ctx, src, dst, n: int, stream=None):
    _check(ctx, lib().lp_cast(ctx, _ptr(src), _ptr(dst), n, _stream(stream)))


def lp_forward(ctx, l: int, X, Z, A, stream=None):
    _check(ctx, lib().lp_forward(ctx, l, _ptr(X), _ptr(Z), _ptr(A), _stream(stream)))


def lp_loss_grad(ctx, ZL, target, dYL, loss_dev, stream=None):
    _check(ctx, lib().lp_loss_grad(ctx, _ptr(ZL), _ptr(target), _ptr(dYL), _ptr(loss_dev), _stream(stream)))


def lp_loss_grad_static(ctx, ZL, target, dYL, loss_dev, stream=None):
    _check(ctx, lib().lp_loss_grad_static(ctx, _ptr(ZL), _ptr(target), _ptr(dYL), _ptr(loss_dev), _stream(stream)))


def lp_act_grad(ctx, l: int, dA, S, dY, stream=None):
    _check(ctx, lib().lp_act_grad(ctx, l, _ptr(dA), _ptr(S), _ptr(dY), _stream(stream)))


def lp_grad_act(ctx, l: int, dY, dX, col0: int, col1: int, stream=None):
    _check(ctx, lib().lp_grad_act(ctx, l, _ptr(dY), _ptr(dX), col0, col1, _stream(stream)))


def lp_grad_weight(ctx, l: int, X, dY, G, stream=None):
    _check(ctx, lib().lp_grad_weight(ctx, l, _ptr(X), _ptr(dY), _ptr(G), _stream(stream)))


def lp_update(ctx, l: int, G, stream=None):
    _check(ctx, lib().lp_update(ctx, l, _ptr(G), _stream(stream)))


def lp_advance(ctx):
    _check(ctx, lib().lp_advance(ctx))


def lp_step(ctx, X0, target, delay: Optional[Sequence[int]], loss_dev, streams: Sequence):
    d = None if delay is None else (C.c_int * len(delay))(*[int(v) for v in delay])
    ss = (C.c_void_p * len(streams))(*[_stream(s) for s in streams])
    _check(ctx, lib().lp_step(ctx, _ptr(X0), _ptr(target), d, _ptr(loss_dev), ss, len(streams)))


def lp_step_index(ctx) -> int:
    n = C.c_long()
    _check(ctx, lib().lp_step_index(ctx, C.byref(n)))
    return n.value


def lp_sync(ctx):
    _check(ctx, lib().lp_sync(ctx))


def lp_tensor(ctx, l: int, which: int):
    p, n = C.c_void_p(), C.c_size_t()
    _check(ctx, lib().lp_tensor(ctx, l, which, C.byref(p), C.byref(n)))
    return (p.value or 0), n.value


def lp_partition(t_fix, t_flex, n_proc: int, alpha: float = 1.01):
    """Algorithm 1: returns dict(stage_fix, stage_delta_rest, borrowed_frac, stage_time, t_p)."""
    L = len(t_fix)
    arr = C.c_double * L
    st, dr, bf, tt, tp = (C.c_int * L)(), (C.c_int * L)(), arr(), (C.c_double * n_proc)(), C.c_double()
    _check(None, lib().lp_partition(arr(*t_fix), arr(*t_flex), L, n_proc, alpha, st, dr, bf, tt, C.byref(tp)))
    return dict(stage_fix=list(st), stage_delta_rest=list(dr), borrowed_frac=list(bf), stage_time=list(tt), t_p=tp.value)


def lp_set_delta_split(ctx, l: int, cols: int):
    _check(ctx, lib().lp_set_delta_split(ctx, l, cols))


def lp_set_factor_ring(ctx, l: int, enable: bool):
    _check(ctx, lib().lp_set_factor_ring(ctx, l, int(enable)))


def lp_set_retimed_update(ctx, l: int, enable: bool):
    _check(ctx, lib().lp_set_retimed_update(ctx, l, int(enable)))


def lp_set_graphs(ctx, enable: bool):
    _check(ctx, lib().lp_set_graphs(ctx, int(enable)))


def lp_graph_stats(ctx):
    """(captured, replayed, eager) step counts."""
    a, b, c = C.c_long(), C.c_long(), C.c_long()
    _check(ctx, lib().lp_graph_stats(ctx, C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def lp_probe_mfma(out_dev, workgroups: int, iters: int, uniform_values: bool = False, stream=None):
    """out_dev: float32 device tensor of at least workgroups * 512 elements."""
    r = lib().lp_probe_mfma(_ptr(out_dev), out_dev.numel(), int(workgroups), int(iters), int(uniform_values), _stream(stream))
    if r != 0:
        raise LpError(r, "lp_probe_mfma failed with status %d" % r)


def lp_set_fused_hadamard(ctx, enable: bool):
    _check(ctx, lib().lp_set_fused_hadamard(ctx, int(enable)))


def lp_set_run_ahead(ctx, enable: bool):
    _check(ctx, lib().lp_set_run_ahead(ctx, int(enable)))


def lp_profile_read_layer(ctx, task: int, l: int, reset: bool = False):
    ms, n = C.c_double(), C.c_long()
    _check(ctx, lib().lp_profile_read_layer(ctx, task, l, C.byref(ms), C.byref(n), int(reset)))
    return ms.value, n.value


def lp_profile(ctx, enable: bool):
    _check(ctx, lib().lp_profile(ctx, int(enable)))


def lp_profile_read(ctx, task: int, reset: bool = False):
    ms, n = C.c_double(), C.c_long()
    _check(ctx, lib().lp_profile_read(ctx, task, C.byref(ms), C.byref(n), int(reset)))
    return ms.value, n.value


# ---- convenience owner of a context + torch memory --------------------------------------------------
class Network:
    """A context bound to a torch workspace tensor on one GPU.  `layers` are lp_workloads.Layer-like
    objects (kind, d_in, d_out, act, H, W, pool)."""

    def __init__(self, layers, batch: int, dtype: str, loss: str, lr: float, delays, device: str = "cuda:0", n_streams: int = None,
                 run_ahead: bool = False, graphs: bool = False, factor_ring=None, fused_hadamard: bool = True,
                 retimed_update=None):
        import torch
        self.torch = torch
        if n_streams is None:
            n_streams = 4 if run_ahead else 3
        self.layers, self.batch, self.dtype, self.loss = list(layers), batch, dtype, loss
        self.device = torch.device(device)
        self.ctx = lp_create(make_descs(layers, delays), len(layers), batch, _DTYPE[dtype], _LOSS[loss], float(lr))
        self.act_dtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        for l in ([] if factor_ring is None else ([0] if factor_ring is True else list(factor_ring))):
            lp_set_factor_ring(self.ctx, l, True)
        for l in ([] if retimed_update is None else ([0] if retimed_update is True else list(retimed_update))):
            lp_set_retimed_update(self.ctx, l, True)
        if graphs:
            lp_set_graphs(self.ctx, True)
        if not fused_hadamard:
            lp_set_fused_hadamard(self.ctx, False)
        if run_ahead:
            lp_set_run_ahead(self.ctx, True)
            n_streams = max(2, n_streams)
        nbytes = lp_workspace_bytes(self.ctx)
        self.ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        self._ws_off = (-self.ws.data_ptr()) % 256
        lp_bind_workspace(self.ctx, self.ws.data_ptr() + self._ws_off, nbytes)
        with torch.cuda.device(self.device):
            self.streams = [torch.cuda.Stream(device=self.device) for _ in range(max(1, n_streams))]
        if run_ahead and n_streams < 4:
            # roles [critical chain, G tasks, updates, forward]: with 3 streams the updates share the G tasks'
            # stream, with 2 the whole backward pass runs on one stream and the forward chain on the other
            s = self.streams
            self.streams = [s[0], s[1], s[1], s[2]] if n_streams == 3 else [s[0], s[0], s[0], s[1]]
        self.loss_dev = torch.zeros(1, dtype=torch.float32, device=self.device)

    def close(self):
        if self.ctx is not None:
            lp_sync(self.ctx)
            lp_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def L(self) -> int:
        return len(self.layers)

    def set_weights(self, weights: List[np.ndarray]):
        for l, w in enumerate(weights, start=1):
            w = np.ascontiguousarray(w, dtype=np.float32)
            lp_set_weights(self.ctx, l, w, False, self.streams[0])
        self.streams[0].synchronize()

    def get_weights(self, l: int) -> np.ndarray:
        ly = self.layers[l - 1]
        out = np.empty(ly.weight_shape, dtype=np.float32)
        lp_get_weights(self.ctx, l, out, False, self.streams[0])
        return out

    def to_device(self, x: np.ndarray, is_label: bool = False):
        """Host array -> device tensor of the act type (labels: int32).  PyTorch only moves the bytes (float32 or
        int32 as given); the conversion to the act type is the library's (lp_cast on streams[0])."""
        torch = self.torch
        if is_label:
            t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to(self.device)
            torch.cuda.current_stream(self.device).synchronize()
            return t
        src = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(self.device)
        # the upload ran on torch's stream; the library's streams are not ordered after it
        torch.cuda.current_stream(self.device).synchronize()
        out = torch.empty(src.shape, dtype=self.act_dtype, device=self.device)
        lp_cast(self.ctx, src, out, src.numel(), self.streams[0])
        self.streams[0].synchronize()
        return out

    def step_device(self, x_dev, t_dev, delay=None):
        """Enqueues one training step; returns nothing.  `self.loss_dev` holds the loss afterwards."""
        lp_step(self.ctx, x_dev, t_dev, delay, self.loss_dev, self.streams)

    def step(self, x: np.ndarray, target: np.ndarray, delay=None) -> float:
        x_dev = self.to_device(x)
        t_dev = self.to_device(target, is_label=(self.loss == "softmax_ce"))
        self.torch.cuda.synchronize(self.device)
        self.step_device(x_dev, t_dev, delay)
        lp_sync(self.ctx)
        return float(self.loss_dev.item())

    def tensor(self, l: int, which: int):
        """Torch view (no copy) of an internal tensor, or None."""
        p, n = lp_tensor(self.ctx, l, which)
        if not p:
            return None
        off = p - self.ws.data_ptr()
        raw = self.ws[off:off + n]
        if which in (LP_T_MASTER_W, LP_T_G_LAST):
            return raw.view(self.torch.float32)
        return raw.view(self.act_dtype)

    def tensor_np(self, l: int, which: int) -> Optional[np.ndarray]:
        t = self.tensor(l, which)
        return None if t is None else t.to(self.torch.float32).cpu().numpy()
