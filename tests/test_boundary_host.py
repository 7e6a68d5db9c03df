"""Host-side checks of the C-ABI boundary: the shared library loads without a GPU, exports every
function include/lp.h declares, and rejects bad arguments with the documented status codes before
touching any device."""
import ctypes as C
import os
import re

import pytest

import lp_workloads as WL
import paper_2108_06629_amd as lp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not header.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(lp_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 18 and {"lp_forward", "lp_grad_act", "lp_grad_weight", "lp_update", "lp_step"} <= set(names)
    raw = C.CDLL(lp.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), n
    assert sorted(lp.EXPORTS) == names          # the Python binding covers the same set


def descs(wl, delays=None):
    return lp.make_descs(wl.layers, wl.delays if delays is None else delays)


def create_status(d, L, batch, dtype, loss):
    ctx = C.c_void_p()
    st = lp.lib().lp_create(d, L, batch, dtype, loss, 0.01, C.byref(ctx))
    if st == 0:
        lp.lib().lp_destroy(ctx)
    return st


def test_create_rejects_bad_arguments():
    wl = WL.mlp_small()
    ok = descs(wl)
    assert create_status(ok, wl.L, 32, lp.LP_F32, lp.LP_LOSS_SOFTMAX_CE) == 0
    assert create_status(None, wl.L, 32, lp.LP_F32, 0) == 1                      # LP_ERR_NULL
    assert create_status(ok, 0, 32, lp.LP_F32, 0) == 2                           # LP_ERR_SHAPE
    assert create_status(ok, wl.L, 0, lp.LP_F32, 0) == 2
    assert create_status(ok, wl.L, 32, 7, 0) == 3                                # LP_ERR_DTYPE
    assert create_status(ok, wl.L, 32, lp.LP_F32, 9) == 3
    bad = descs(wl); bad[1].in_ = 255
    assert create_status(bad, wl.L, 32, lp.LP_F32, 0) == 4                       # LP_ERR_LAYER (widths do not chain)
    bad = descs(wl); bad[2].delay = -1
    assert create_status(bad, wl.L, 32, lp.LP_F32, 0) == 5                       # LP_ERR_DELAY
    bad = descs(wl); bad[3].act = lp.LP_ACT_RELU
    assert create_status(bad, wl.L, 32, lp.LP_F32, 0) == 3                       # last layer must be identity
    bad = descs(wl); bad[0].kind = 5
    assert create_status(bad, wl.L, 32, lp.LP_F32, 0) == 3
    assert b"layer 1" in lp.lib().lp_last_error(None)
    cnn = WL.vgg_small(batch=2, hw=8, chans=(8, 8))
    assert create_status(descs(cnn), cnn.L, 2, lp.LP_BF16, 0) == 0
    bad = descs(cnn); bad[1].H = 7
    assert create_status(bad, cnn.L, 2, lp.LP_BF16, 0) in (2, 4)
    bad = descs(cnn); bad[2].in_ = 100
    assert create_status(bad, cnn.L, 2, lp.LP_BF16, 0) == 4


def test_create_rejects_what_a_task_launcher_would_refuse():
    """Operand limits of the kernels (32-bit byte offsets) are checked when the context is made, so that a step
    cannot fail on a shape after its first launch."""
    big = (WL.Layer(WL.LINEAR, 32768, 32768, WL.IDENTITY),)                      # 2 GiB of bf16 weights
    assert create_status(lp.make_descs(big, (0,)), 1, 8, lp.LP_BF16, lp.LP_LOSS_MSE) == 2
    assert b"2 GiB" in lp.lib().lp_last_error(None)
    ok = (WL.Layer(WL.LINEAR, 32768, 32760, WL.IDENTITY),)
    assert create_status(lp.make_descs(ok, (0,)), 1, 8, lp.LP_BF16, lp.LP_LOSS_MSE) == 0
    wide = (WL.Layer(WL.LINEAR, 16, 16, WL.IDENTITY),)
    assert create_status(lp.make_descs(wide, (0,)), 1, 1 << 27, lp.LP_BF16, lp.LP_LOSS_MSE) == 2      # batch x width reaches 2 GiB
    assert create_status(lp.make_descs(wide, (0,)), 1, 65535 * 32 + 1, lp.LP_F32, lp.LP_LOSS_MSE) == 2
    img = (WL.Layer(WL.CONV3X3, 8, 64, WL.RELU, H=512, W=512), WL.Layer(WL.LINEAR, 512 * 512 * 64, 8, WL.IDENTITY))
    assert create_status(lp.make_descs(img, (0, 0)), 2, 64, lp.LP_BF16, lp.LP_LOSS_SOFTMAX_CE) == 2   # 64 x 512 x 512 x 64 bf16 = 2 GiB


def test_cast_checks_its_arguments_before_launching():
    wl = WL.mlp_small()
    ctx = lp.lp_create(descs(wl), wl.L, wl.batch, lp.LP_BF16, lp.LP_LOSS_SOFTMAX_CE, 0.01)
    L = lp.lib()
    assert L.lp_cast(None, 0x10000, 0x20000, 8, None) == 1
    assert L.lp_cast(ctx, None, 0x20000, 8, None) == 1 and L.lp_cast(ctx, 0x10000, None, 8, None) == 1
    assert L.lp_cast(ctx, 0x10004, 0x20000, 8, None) == 2 and L.lp_cast(ctx, 0x10000, 0x20008, 8, None) == 2
    assert L.lp_cast(ctx, 0x10000, 0x20000, 0, None) == 0                     # nothing to do, nothing launched
    lp.lp_destroy(ctx)


def test_workspace_size_accounts_for_rings_and_weight_versions():
    wl = WL.mlp_4096()
    ctx = lp.lp_create(descs(wl), wl.L, wl.batch, lp.LP_BF16, lp.LP_LOSS_SOFTMAX_CE, 1e-3)
    n = lp.lp_workspace_bytes(ctx)
    ring = sum((d + 1) * ly.n_params * 4 for d, ly in zip(wl.delays, wl.layers))
    weights = wl.n_params * (4 + 2 + 2)
    assert n % 256 == 0 and ring + weights <= n <= ring + weights + 128 * 2 ** 20
    ctx0 = lp.lp_create(descs(wl, [0] * wl.L), wl.L, wl.batch, lp.LP_BF16, lp.LP_LOSS_SOFTMAX_CE, 1e-3)
    assert lp.lp_workspace_bytes(ctx0) == n - sum(d * ly.n_params * 4 for d, ly in zip(wl.delays, wl.layers))
    lp.lp_destroy(ctx); lp.lp_destroy(ctx0)
    big = WL.ffn_stack()
    ctx = lp.lp_create(descs(big), big.L, big.batch, lp.LP_BF16, lp.LP_LOSS_MSE, 1e-3)
    assert 68.7e9 + 6.4e9 < lp.lp_workspace_bytes(ctx) < 90e9      # fits one 288 GB device
    lp.lp_destroy(ctx)


def test_state_and_argument_errors_before_any_launch():
    wl = WL.mlp_small()
    ctx = lp.lp_create(descs(wl), wl.L, wl.batch, lp.LP_F32, lp.LP_LOSS_SOFTMAX_CE, 0.01)
    L = lp.lib()
    fake = 0x10000        # never dereferenced: every call below must fail in validation
    assert L.lp_forward(ctx, 1, fake, fake, fake, None) == 6                  # LP_ERR_STATE: no workspace
    assert b"workspace" in L.lp_last_error(ctx)
    assert L.lp_bind_workspace(ctx, None, 1 << 30) == 1
    assert L.lp_bind_workspace(ctx, 0x10008, 1 << 30) == 7                    # LP_ERR_WORKSPACE: misaligned
    assert L.lp_bind_workspace(ctx, 0x10000, 16) == 7                         # too small
    assert L.lp_bind_workspace(ctx, 0x10000, 1 << 30) == 0                    # accepted (host bookkeeping only)
    assert L.lp_forward(ctx, 1, fake, fake, fake, None) == 6                  # weights never set
    assert b"weights" in L.lp_last_error(ctx)
    assert L.lp_forward(ctx, 0, fake, fake, fake, None) == 4                  # LP_ERR_LAYER
    assert L.lp_forward(ctx, 5, fake, fake, fake, None) == 4
    assert L.lp_forward(ctx, 1, None, fake, fake, None) == 1
    assert L.lp_forward(ctx, 1, fake, None, None, None) == 1
    assert L.lp_grad_act(ctx, 2, fake, fake, 10, 5, None) == 2                # LP_ERR_SHAPE: empty column range
    assert L.lp_grad_act(ctx, 2, fake, fake, 0, 257, None) == 2
    assert L.lp_grad_weight(ctx, 1, None, fake, None, None) == 1
    assert L.lp_update(ctx, 1, None, None) == 6
    assert L.lp_loss_grad(ctx, None, fake, fake, None, None) == 1
    assert L.lp_act_grad(ctx, 1, None, fake, fake, None) == 1
    streams = (C.c_void_p * 1)(None)
    assert L.lp_step(ctx, fake, fake, None, None, streams, 1) == 6
    assert L.lp_step(ctx, None, fake, None, None, streams, 1) == 1
    assert L.lp_step(ctx, fake, fake, None, None, None, 0) == 1
    n = C.c_long(-1)
    assert L.lp_step_index(ctx, C.byref(n)) == 0 and n.value == 0
    assert L.lp_advance(ctx) == 0 and L.lp_step_index(ctx, C.byref(n)) == 0 and n.value == 1
    assert L.lp_destroy(ctx) == 0
    assert L.lp_destroy(None) == 1
    with pytest.raises(lp.LpError):
        lp.lp_create(descs(wl), wl.L, -3, lp.LP_F32, 0, 0.1)


def test_run_ahead_is_a_layout_decision_made_before_binding():
    wl = WL.mlp_4096()
    ctx = lp.lp_create(descs(wl), wl.L, wl.batch, lp.LP_BF16, lp.LP_LOSS_SOFTMAX_CE, 1e-3)
    L = lp.lib()
    n0 = lp.lp_workspace_bytes(ctx)
    assert L.lp_set_run_ahead(ctx, 1) == 0
    n1 = lp.lp_workspace_bytes(ctx)
    # a second stash per layer: A_l for l < L (ReLU layers stash A only), Z_L for the last layer
    stash = sum(wl.batch * ly.d_out * 2 for ly in wl.layers)
    assert n1 % 256 == 0 and n0 + stash <= n1 <= n0 + stash + 64 * 2 ** 20
    assert L.lp_set_run_ahead(ctx, 0) == 0 and lp.lp_workspace_bytes(ctx) == n0
    assert L.lp_bind_workspace(ctx, 0x10000, 1 << 40) == 0                    # host bookkeeping only
    assert L.lp_set_run_ahead(ctx, 1) == 6                                    # LP_ERR_STATE: workspace already bound
    assert b"lp_bind_workspace" in L.lp_last_error(ctx)
    lp.lp_destroy(ctx)
    small = WL.mlp_small()
    ctx = lp.lp_create(descs(small), small.L, small.batch, lp.LP_F32, lp.LP_LOSS_SOFTMAX_CE, 0.01)
    assert L.lp_set_run_ahead(ctx, 1) == 3                                    # LP_ERR_DTYPE: F32 updates in place
    assert L.lp_set_run_ahead(None, 1) == 1
    lp.lp_destroy(ctx)


def test_graph_replay_is_a_layout_decision_made_before_binding():
    wl = WL.mlp_4096()
    ctx = lp.lp_create(descs(wl), wl.L, wl.batch, lp.LP_BF16, lp.LP_LOSS_SOFTMAX_CE, 1e-3)
    L = lp.lib()
    n0 = lp.lp_workspace_bytes(ctx)
    assert L.lp_set_graphs(ctx, 1) == 0
    # rings of d_l + 1 = 15, 13, 11, 9, 7, 5, 3, 1 slots become 16, 16, 16, 16, 8, 8, 4, 1
    extra = sum((r - (d + 1)) * ly.n_params * 4 for r, d, ly in zip((16, 16, 16, 16, 8, 8, 4, 1), wl.delays, wl.layers))
    assert lp.lp_workspace_bytes(ctx) == n0 + extra
    assert L.lp_set_run_ahead(ctx, 1) == 6                                    # not both
    assert lp.lp_graph_stats(ctx) == (0, 0, 0)
    assert L.lp_set_graphs(ctx, 0) == 0 and lp.lp_workspace_bytes(ctx) == n0
    assert L.lp_set_run_ahead(ctx, 1) == 0 and L.lp_set_graphs(ctx, 1) == 6
    assert L.lp_bind_workspace(ctx, 0x10000, 1 << 40) == 0
    assert L.lp_set_graphs(ctx, 1) == 6                                       # LP_ERR_STATE: workspace already bound
    assert L.lp_set_graphs(None, 1) == 1 and L.lp_graph_stats(None, None, None, None) == 1
    lp.lp_destroy(ctx)


def test_factor_ring_shrinks_the_delay_elements():
    wl = WL.mlp_4096()
    ctx = lp.lp_create(descs(wl), wl.L, wl.batch, lp.LP_BF16, lp.LP_LOSS_SOFTMAX_CE, 1e-3)
    L = lp.lib()
    n0 = lp.lp_workspace_bytes(ctx)
    assert L.lp_set_factor_ring(ctx, 0, 1) == 0
    n1 = lp.lp_workspace_bytes(ctx)
    ring_g = sum((d + 1) * ly.n_params * 4 for d, ly in zip(wl.delays, wl.layers))
    ring_f = sum((d + 1) * wl.batch * (ly.d_in + ly.d_out) * 2 for d, ly in zip(wl.delays, wl.layers))
    assert abs((n0 - n1) - (ring_g - ring_f)) < 2 ** 20 and n1 < n0 / 4
    assert L.lp_set_factor_ring(ctx, 9, 1) == 4 and L.lp_set_factor_ring(ctx, 3, 0) == 0        # LP_ERR_LAYER; one layer back to products
    assert lp.lp_workspace_bytes(ctx) == n1 + (wl.delays[2] + 1) * (wl.layers[2].n_params * 4 - wl.batch * (4096 + 4096) * 2)
    assert L.lp_bind_workspace(ctx, 0x10000, 1 << 40) == 0
    assert L.lp_set_factor_ring(ctx, 0, 1) == 6                                                   # LP_ERR_STATE: already bound
    lp.lp_destroy(ctx)
    small = WL.mlp_small()
    ctx = lp.lp_create(descs(small), small.L, small.batch, lp.LP_F32, lp.LP_LOSS_SOFTMAX_CE, 0.01)
    assert L.lp_set_factor_ring(ctx, 0, 1) == 3                                                   # LP_ERR_DTYPE
    lp.lp_destroy(ctx)
    cnn = WL.vgg_small(batch=2, hw=8, chans=(8, 8))
    ctx = lp.lp_create(descs(cnn), cnn.L, 2, lp.LP_BF16, lp.LP_LOSS_SOFTMAX_CE, 0.01)
    n_cnn = lp.lp_workspace_bytes(ctx)
    # conv: LP_ERR_LAYER; the 128 -> 10 classifier too: its G product runs on the few-outputs kernels, not the tiled GEMM of the fused update
    assert L.lp_set_factor_ring(ctx, 1, 1) == 4 and L.lp_set_factor_ring(ctx, cnn.L, 1) == 4
    assert L.lp_set_factor_ring(ctx, 0, 1) == 0 and lp.lp_workspace_bytes(ctx) == n_cnn             # "every layer": none qualifies
    lp.lp_destroy(ctx)
    # A G product that lp_grad_weight splits over K keeps its product ring: the fused update never splits K, so its
    # bits would differ.  Batch 2048: 512 x 512, 512 x 4096 and 4096 x 16 outputs have fewer than 256 tiles of
    # 128 x 128 and are split; 4096 x 4096 (1024 tiles) is not.
    mixed = WL.mlp_4096().with_(layers=WL._mlp([512, 512, 4096, 4096, 16], WL.RELU), batch=2048, delays=(6, 4, 2, 0))
    ctx = lp.lp_create(descs(mixed), mixed.L, mixed.batch, lp.LP_BF16, lp.LP_LOSS_SOFTMAX_CE, 1e-3)
    n0 = lp.lp_workspace_bytes(ctx)
    for l in (1, 2, 4):
        assert L.lp_set_factor_ring(ctx, l, 1) == 4 and b"split over K" in L.lp_last_error(ctx)
    assert lp.lp_workspace_bytes(ctx) == n0
    assert L.lp_set_factor_ring(ctx, 0, 1) == 0                  # "every linear layer": here that is layer 3 alone
    # layer 3 (d = 2: three slots): a slot of G (4096 x 4096 floats) becomes a slot of factors (2048 x (4096 + 4096) bf16)
    assert n0 - lp.lp_workspace_bytes(ctx) == 3 * (4096 * 4096 * 4 - 2048 * (4096 + 4096) * 2)
    assert L.lp_set_factor_ring(ctx, 3, 0) == 0 and lp.lp_workspace_bytes(ctx) == n0
    lp.lp_destroy(ctx)


def test_retimed_update_trades_the_gradient_ring_for_weight_versions():
    """Host bookkeeping only: a retimed layer holds d + 2 bf16 weight versions in place of d + 1 fp32 gradients and its
    two working copies; which layers qualify; which calls it refuses."""
    wl = WL.mlp_4096()
    L = lp.lib()
    ctx = lp.lp_create(descs(wl), wl.L, wl.batch, lp.LP_BF16, lp.LP_LOSS_SOFTMAX_CE, 1e-3)
    n0 = lp.lp_workspace_bytes(ctx)
    assert L.lp_set_retimed_update(ctx, 0, 1) == 0
    n1 = lp.lp_workspace_bytes(ctx)
    saved = sum((d + 1) * ly.n_params * 4 + 2 * ly.n_params * 2 - (d + 2) * ly.n_params * 2 for d, ly in zip(wl.delays, wl.layers))
    assert abs((n0 - n1) - saved) < 2 ** 16, (n0 - n1, saved)
    assert L.lp_set_retimed_update(ctx, 9, 1) == 4
    assert L.lp_set_factor_ring(ctx, 2, 1) == 4 and b"retimed" in L.lp_last_error(ctx)     # one kind of delay element per layer
    assert L.lp_set_retimed_update(ctx, 2, 0) == 0 and L.lp_set_factor_ring(ctx, 2, 1) == 0
    assert L.lp_set_retimed_update(ctx, 2, 1) == 4                                           # ... either way round
    assert L.lp_set_retimed_update(ctx, 0, 1) == 0                                           # "every layer" leaves layer 2 its factors
    assert L.lp_bind_workspace(ctx, 0x10000, 1 << 40) == 0
    assert L.lp_set_retimed_update(ctx, 0, 1) == 6                                           # LP_ERR_STATE: already bound
    assert not lp.lp_tensor(ctx, 1, lp.LP_T_G_LAST)[0] and not lp.lp_tensor(ctx, wl.L, lp.LP_T_G_LAST)[0]   # no step yet
    # the weights the first step reads are version 0, whatever the delay
    w1, w3 = lp.lp_tensor(ctx, 1, lp.LP_T_WORK_W), lp.lp_tensor(ctx, 3, lp.LP_T_WORK_W)
    assert w1[0] and w1[1] == wl.layers[0].n_params * 2 and w3[0] and w3[0] != w1[0]
    assert L.lp_advance(ctx) == 0
    assert lp.lp_tensor(ctx, 1, lp.LP_T_WORK_W)[0] == w1[0]                                  # d = 14: still version 0 after one step
    lp.lp_destroy(ctx)
    small = WL.mlp_small()
    ctx = lp.lp_create(descs(small), small.L, small.batch, lp.LP_F32, lp.LP_LOSS_SOFTMAX_CE, 0.01)
    assert L.lp_set_retimed_update(ctx, 0, 1) == 3                                           # LP_ERR_DTYPE
    lp.lp_destroy(ctx)
    assert L.lp_set_retimed_update(None, 0, 1) == 1
    cnn = WL.vgg_small(batch=2, hw=8, chans=(8, 8))
    ctx = lp.lp_create(descs(cnn), cnn.L, 2, lp.LP_BF16, lp.LP_LOSS_SOFTMAX_CE, 0.01)
    n_cnn = lp.lp_workspace_bytes(ctx)
    # 2 x 8 x 8 = 128 pixels: the G products of these convolutions are not split over K, so there is no kernel that sums
    # partials for the update to ride in; the 128 -> 10 classifier (few-outputs kernels) qualifies
    assert L.lp_set_retimed_update(ctx, 1, 1) == 4 and b"convolution whose G product is not" in L.lp_last_error(ctx)
    assert L.lp_set_retimed_update(ctx, 0, 1) == 0 and n_cnn - lp.lp_workspace_bytes(ctx) == 128 * 10 * (1 * 4 + 2 * 2 - 2 * 2)
    lp.lp_destroy(ctx)
    # the benchmark's CNN (128 x 32 x 32 pixels): every convolution's G product is split over K, every layer qualifies
    cnn = WL.vgg_small()
    ctx = lp.lp_create(descs(cnn), cnn.L, cnn.batch, lp.LP_BF16, lp.LP_LOSS_SOFTMAX_CE, 0.01)
    n_cnn = lp.lp_workspace_bytes(ctx)
    for l in range(1, cnn.L + 1):
        assert L.lp_set_retimed_update(ctx, l, 1) == 0, l
    saved = sum((d + 1) * ly.n_params * 4 + 2 * ly.n_params * 2 - (d + 2) * ly.n_params * 2 for d, ly in zip(cnn.delays, cnn.layers))
    assert abs((n_cnn - lp.lp_workspace_bytes(ctx)) - saved) < 2 ** 14
    lp.lp_destroy(ctx)
    # batch 2048: the G products of the 512 x 512 and 512 x 4096 layers are split over K (the kernel that adds the partial
    # sums applies the update), the 4096 x 4096 layer runs the tiled GEMM and the 4096 x 16 layer the few-outputs kernel:
    # every linear layer qualifies
    mixed = WL.mlp_4096().with_(layers=WL._mlp([512, 512, 4096, 4096, 16], WL.RELU), batch=2048, delays=(6, 4, 2, 0))
    ctx = lp.lp_create(descs(mixed), mixed.L, mixed.batch, lp.LP_BF16, lp.LP_LOSS_SOFTMAX_CE, 1e-3)
    n0 = lp.lp_workspace_bytes(ctx)
    assert L.lp_set_retimed_update(ctx, 3, 1) == 0
    # layer 3 (d = 2): three gradients and two working copies become four versions
    assert n0 - lp.lp_workspace_bytes(ctx) == 4096 * 4096 * (3 * 4 + 2 * 2 - 4 * 2)
    assert L.lp_set_retimed_update(ctx, 0, 1) == 0
    saved = sum((d + 1) * ly.n_params * 4 + 2 * ly.n_params * 2 - (d + 2) * ly.n_params * 2 for d, ly in zip(mixed.delays, mixed.layers))
    assert n0 - lp.lp_workspace_bytes(ctx) == saved
    lp.lp_destroy(ctx)


def test_mfma_probe_checks_its_arguments_before_launching():
    L = lp.lib()
    assert L.lp_probe_mfma(None, 0, 1, 1, 0, None) == 1          # LP_ERR_NULL
    fake = 4096                                                  # never dereferenced: the checks below fail first
    assert L.lp_probe_mfma(fake, 511, 1, 1, 0, None) == 2        # LP_ERR_SHAPE: one workgroup writes 512 floats
    assert L.lp_probe_mfma(fake, 1 << 20, 0, 1, 0, None) == 2    # no workgroups
    assert L.lp_probe_mfma(fake, 1 << 20, 1, -1, 0, None) == 2   # negative round count


def test_fused_hadamard_switch_decides_whether_dA_is_materialised():
    """Host bookkeeping only: with the Hadamard product of a ReLU layer inside the dX product above it (the default), that
    layer's dA has no address; with the switch off it has one.  An F32 context never fuses."""
    wl = WL.mlp_4096()
    L = lp.lib()
    ctx = lp.lp_create(descs(wl), wl.L, wl.batch, lp.LP_BF16, lp.LP_LOSS_SOFTMAX_CE, 1e-3)
    assert L.lp_bind_workspace(ctx, 0x10000, 1 << 40) == 0
    assert all(not lp.lp_tensor(ctx, l, lp.LP_T_DA)[0] for l in range(1, wl.L))
    assert L.lp_set_fused_hadamard(ctx, 0) == 0
    assert all(lp.lp_tensor(ctx, l, lp.LP_T_DA)[0] for l in range(1, wl.L))
    assert L.lp_set_fused_hadamard(ctx, 1) == 0 and not lp.lp_tensor(ctx, 1, lp.LP_T_DA)[0]
    assert L.lp_set_fused_hadamard(None, 1) == 1
    lp.lp_destroy(ctx)
    small = WL.mlp_small()
    ctx = lp.lp_create(descs(small), small.L, small.batch, lp.LP_F32, lp.LP_LOSS_SOFTMAX_CE, 0.01)
    assert L.lp_bind_workspace(ctx, 0x10000, 1 << 40) == 0
    assert all(lp.lp_tensor(ctx, l, lp.LP_T_DA)[0] for l in range(1, small.L))
    lp.lp_destroy(ctx)


def test_bench_picks_its_streams_from_the_shape_of_the_network():
    """Host logic of bench.py: one stream for a network whose every product fills the chip once the retimed update has
    removed the update tasks, and for one so small that the host's enqueue time bounds its step; three otherwise."""
    import bench
    want = {"mlp_small_f32": 1, "mlp_4096_bf16": 3, "vgg_small_bf16": 3, "ffn_stack_bf16": 1, "mlp_imbalanced_bf16": 3}
    for name, mk in WL.CONFIGS.items():
        assert bench.default_streams(mk(), True) == want[name], name
    assert bench.default_streams(WL.ffn_stack(), False) == 3          # gradient rings: the updates overlap the products
    assert bench.fills_chip(WL.ffn_stack()) and not bench.fills_chip(WL.mlp_4096()) and not bench.fills_chip(WL.vgg_small())
