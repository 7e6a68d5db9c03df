"""The Hadamard product of layer l-1 (Eq. 3, placed by Sec. III-B) applied in the epilogue of the dX product of layer l
(lp_set_fused_hadamard, lp_step's default): dA is rounded to bf16 before the multiplication exactly as if it had been
stored, so losses, weights and every dY must agree bit for bit with the two-kernel form, in every schedule and for every
kernel variant the dX product can take.  The two-kernel form is the one compared with the CPU oracle task by task
(test_gpu_parity.py); the fused form is also compared with the oracle there, through the pair of tasks.  Needs a real MI355X."""
import numpy as np
import pytest
import torch

import lp_workloads as WL
import paper_2108_06629_amd as lp
from test_gpu_parity import DEV

pytestmark = pytest.mark.gpu


def run(wl, W0, steps, splits=None, **kw):
    net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, **kw)
    net.set_weights(W0)
    for l, cols in (splits or {}).items():
        lp.lp_set_delta_split(net.ctx, l, cols)
    xs = [net.to_device(WL.batch_input(wl, n)) for n in range(1, steps + 1)]
    ts = [net.to_device(WL.batch_target(wl, n), is_label=(wl.loss == WL.SOFTMAX_CE)) for n in range(1, steps + 1)]
    losses = torch.zeros(steps, dtype=torch.float32, device=DEV)
    torch.cuda.synchronize()
    for n in range(steps):
        lp.lp_step(net.ctx, xs[n], ts[n], None, losses[n:n + 1], net.streams)
    lp.lp_sync(net.ctx)
    dys = [net.tensor(l, lp.LP_T_DY).view(torch.int16).cpu().numpy().copy() for l in range(1, wl.L + 1)]
    das = [net.tensor(l, lp.LP_T_DA) is not None for l in range(1, wl.L + 1)]
    out = (losses.cpu().numpy().copy(), [net.get_weights(l) for l in range(1, wl.L + 1)], dys, das)
    net.close()
    return out


def assert_same(a, b):
    assert np.array_equal(a[0].view(np.uint32), b[0].view(np.uint32)), (a[0], b[0])
    for l, (wa, wb) in enumerate(zip(a[1], b[1]), start=1):
        assert np.array_equal(wa.view(np.uint32), wb.view(np.uint32)), "master W_%d" % l
    for l, (ya, yb) in enumerate(zip(a[2], b[2]), start=1):
        assert np.array_equal(ya, yb), "dY_%d" % l


def mlp(widths, batch, act=WL.RELU, **kw):
    L = len(widths) - 1
    return WL.mlp_4096().with_(layers=WL._mlp(widths, act), batch=batch, delays=tuple(2 * (L - l) for l in range(1, L + 1)), **kw)


# kernel variants of the dX product: 128 x 128 direct-to-LDS tiles (aligned), the register-staged loop with scalar stores
# (ragged widths), 256 x 256 tiles (a 2304 x 5632 output), K cut into ranges with the epilogue in the reduction kernel
# (batch 256, widths 2048 and 4096: fewer than 256 tiles of 128 x 128, K = 4096), the short-vector kernels of a 10-output classifier
CASES = [([256, 320, 192, 136, 40], 96), ([77, 130, 45, 19, 10], 33), ([512, 5632, 4096, 264, 16], 2304), ([4096, 2048, 4096, 1000], 256),
         ([4096, 4096, 4096, 1000], 256),
         ([264, 2056, 1160, 72], 300), ([256, 320, 72, 10], 96)]


@pytest.mark.parametrize("widths,batch", CASES)
@pytest.mark.parametrize("act", [WL.RELU, WL.GELU])
def test_fused_hadamard_bits_equal_two_kernel_form(widths, batch, act):
    wl = mlp(widths, batch, act)
    W0 = WL.init_weights(wl)
    steps = 2 * (wl.L - 1) + 3
    ref = run(wl, W0, steps, fused_hadamard=False)
    assert np.all(np.isfinite(ref[0]))
    assert all(ref[3][:-1]), "every hidden layer's dA exists in the two-kernel form"
    got = run(wl, W0, steps)
    assert not any(got[3][:-1]), "no hidden layer's dA is stored in the fused form"
    assert_same(ref, got)
    assert_same(ref, run(wl, W0, steps, n_streams=1))


@pytest.mark.parametrize("act", [WL.RELU, WL.GELU])
def test_fused_hadamard_with_delta_split_run_ahead_and_graph_replay(act):
    wl = mlp([256, 320, 192, 136, 40], 96, act)
    W0 = WL.init_weights(wl)
    ref = run(wl, W0, 12, fused_hadamard=False)
    splits = {2: 104, 3: 1, 4: 135}          # delta' | delta'': each range applies the product to its own columns
    assert_same(ref, run(wl, W0, 12, splits=splits))
    assert_same(ref, run(wl, W0, 12, splits=splits, n_streams=1))
    assert_same(ref, run(wl, W0, 12, run_ahead=True))
    assert_same(ref, run(wl, W0, 12, run_ahead=True, splits=splits))
    assert_same(ref, run(wl, W0, 12, factor_ring=True))


@pytest.mark.parametrize("act", [WL.RELU, WL.GELU])
def test_fused_hadamard_in_the_few_outputs_kernels_with_column_ranges(act):
    """A 72 -> 10 classifier: its dX runs on the short-vector kernel, whole (16-byte accesses) and cut at column 52 (a range
    that starts and ends off a multiple of 8: 2-byte accesses, same sums)."""
    wl = mlp([256, 320, 72, 10], 96, act)
    W0 = WL.init_weights(wl)
    ref = run(wl, W0, 8, fused_hadamard=False)
    assert_same(ref, run(wl, W0, 8))
    assert_same(ref, run(wl, W0, 8, splits={3: 20, 2: 8}))
    assert_same(ref, run(wl, W0, 8, splits={3: 20}, fused_hadamard=False))
    assert_same(ref, run(wl, W0, 8, splits={3: 16}, run_ahead=True))


def test_fused_hadamard_under_graph_replay():
    wl = mlp([256, 320, 192, 136, 40], 96, WL.GELU)
    W0 = WL.init_weights(wl)

    def replayed(**kw):
        net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, graphs=True, **kw)
        net.set_weights(W0)
        xs = [net.to_device(WL.batch_input(wl, n)) for n in range(1, 4)]
        ts = [net.to_device(WL.batch_target(wl, n), is_label=True) for n in range(1, 4)]
        losses = torch.zeros(60, dtype=torch.float32, device=DEV)
        loss_slot = torch.zeros(1, dtype=torch.float32, device=DEV)      # one fixed address, as a captured step needs
        torch.cuda.synchronize()
        for n in range(60):      # rings of 8, 4, 2, 1 slots and a pool of 3 inputs: 24 combinations, then replays
            lp.lp_step(net.ctx, xs[n % 3], ts[n % 3], None, loss_slot, net.streams)
            with torch.cuda.stream(net.streams[0]):
                losses[n:n + 1].copy_(loss_slot)
        lp.lp_sync(net.ctx)
        torch.cuda.synchronize()
        stats = lp.lp_graph_stats(net.ctx)
        out = (losses.cpu().numpy().copy(), [net.get_weights(l) for l in range(1, wl.L + 1)])
        net.close()
        return out, stats

    (la, wa), sa = replayed()
    (lb, wb), sb = replayed(fused_hadamard=False)
    assert sa[1] > 0 and sb[1] > 0, "steps were replayed from graphs"
    assert np.array_equal(la.view(np.uint32), lb.view(np.uint32))
    assert all(np.array_equal(a.view(np.uint32), b.view(np.uint32)) for a, b in zip(wa, wb))


def test_which_layers_are_fused():
    """Fused: the dX product (fully connected or convolution) above an element-wise ReLU / GELU layer of a bf16 context.
    Not fused (dA stays in memory): tanh and sigmoid below, a pooled convolution below a fully connected layer, fp32."""
    acts = [WL.RELU, WL.TANH, WL.GELU, WL.SIGMOID, WL.IDENTITY]
    layers = tuple(WL.Layer(WL.LINEAR, 64, 64, a) for a in acts) + (WL.Layer(WL.LINEAR, 64, 8, WL.IDENTITY),)
    for dtype, want in (("bf16", [False, True, False, True]), ("f32", [True, True, True, True])):
        net = lp.Network(layers, 16, dtype, WL.SOFTMAX_CE, 0.01, (0,) * len(layers))
        net.set_weights([np.zeros(l.weight_shape, dtype=np.float32) for l in layers])
        assert [net.tensor(l, lp.LP_T_DA) is not None for l in (1, 2, 3, 4)] == want, dtype
        lp.lp_set_fused_hadamard(net.ctx, False)
        assert all(net.tensor(l, lp.LP_T_DA) is not None for l in (1, 2, 3, 4))
        net.close()
    cnn = (WL.Layer(WL.CONV3X3, 8, 8, WL.RELU, H=8, W=8, pool=0), WL.Layer(WL.CONV3X3, 8, 8, WL.RELU, H=8, W=8, pool=2),
           WL.Layer(WL.LINEAR, 4 * 4 * 8, 16, WL.RELU), WL.Layer(WL.LINEAR, 16, 8, WL.IDENTITY))
    net = lp.Network(cnn, 4, "bf16", WL.SOFTMAX_CE, 0.01, (0, 0, 0, 0))
    net.set_weights([np.zeros(l.weight_shape, dtype=np.float32) for l in cnn])
    assert [net.tensor(l, lp.LP_T_DA) is not None for l in (1, 2, 3)] == [False, True, False]
    net.close()


def test_unpooled_convolution_below_a_fully_connected_layer():
    """The stash of a convolution layer read as [batch, H*W*C] by the dX epilogue of the classifier above it."""
    layers = (WL.Layer(WL.CONV3X3, 8, 16, WL.RELU, H=8, W=8, pool=0), WL.Layer(WL.LINEAR, 8 * 8 * 16, 40, WL.RELU),
              WL.Layer(WL.LINEAR, 40, 10, WL.IDENTITY))
    wl = WL.vgg_small(batch=12, hw=8, chans=(8, 8)).with_(layers=tuple(layers), delays=(4, 2, 0))
    W0 = WL.init_weights(wl)
    ref = run(wl, W0, 8, fused_hadamard=False)
    got = run(wl, W0, 8)
    assert got[3][:2] == [False, False] and ref[3][:2] == [True, True]
    assert_same(ref, got)


@pytest.mark.parametrize("batch,hw,chans,splits", [(4, 8, (8, 8, 16, 16), None), (8, 32, (64, 64, 128, 128, 256, 256), None),
                                                   (6, 16, (16, 24, 40, 40), {2: 4, 3: 16, 4: 8})])
def test_convolution_dx_with_fused_hadamard_bits_equal_two_kernel_form(batch, hw, chans, splits):
    """The three forms of the convolution dX kernel (pixel halo in LDS, direct-to-LDS gather, register-staged gather for a
    channel range that starts off a multiple of 8), whole and cut into channel ranges (delta' | delta'')."""
    wl = WL.vgg_small(batch=batch, hw=hw, chans=chans)
    W0 = WL.init_weights(wl)
    steps = 2 * (wl.L - 1) + 2
    ref = run(wl, W0, steps, fused_hadamard=False)
    assert np.all(np.isfinite(ref[0])) and all(ref[3][:-1])
    got = run(wl, W0, steps, splits=splits)
    # unpooled layers: masked in the dX epilogue above them; pooled layers below a convolution: masked and routed there;
    # the last pooled layer sits below the fully connected classifier and keeps its routing kernel and its dA
    assert got[3][:-1] == [i == wl.L - 2 for i in range(wl.L - 1)]
    assert_same(ref, got)
    assert_same(ref, run(wl, W0, steps, splits=splits, run_ahead=True))


def test_gelu_convolutions_look_the_derivative_up_in_both_forms():
    """A CNN with GELU: the unpooled layers' Hadamard products ride in the dX epilogues above them (convolution and fully
    connected) with f' from the table; the pooled GELU layer is routed by the stand-alone kernel (the fused routing is
    the ReLU form only).  Both forms agree bit for bit."""
    layers = (WL.Layer(WL.CONV3X3, 8, 16, WL.GELU, H=8, W=8, pool=0), WL.Layer(WL.CONV3X3, 16, 16, WL.GELU, H=8, W=8, pool=2),
              WL.Layer(WL.CONV3X3, 16, 24, WL.GELU, H=4, W=4, pool=0), WL.Layer(WL.LINEAR, 4 * 4 * 24, 40, WL.GELU),
              WL.Layer(WL.LINEAR, 40, 10, WL.IDENTITY))
    wl = WL.vgg_small(batch=6, hw=8, chans=(8, 8)).with_(layers=layers, delays=(8, 6, 4, 2, 0))
    W0 = WL.init_weights(wl)
    ref = run(wl, W0, 12, fused_hadamard=False)
    assert np.all(np.isfinite(ref[0])) and all(ref[3][:-1])
    got = run(wl, W0, 12)
    assert got[3][:-1] == [False, True, False, False]
    assert_same(ref, got)
    assert_same(ref, run(wl, W0, 12, splits={2: 8, 3: 8}, run_ahead=True))


def test_switching_the_form_between_steps_changes_no_bits():
    """lp_set_fused_hadamard may be called between steps (also under graph replay, where it drops the captured steps)."""
    wl = mlp([256, 320, 192, 136, 40], 96, WL.GELU)
    W0 = WL.init_weights(wl)
    steps = 24
    ref = run(wl, W0, steps)
    for graphs in (False, True):
        net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, graphs=graphs)
        net.set_weights(W0)
        xs = [net.to_device(WL.batch_input(wl, n)) for n in range(1, steps + 1)]
        ts = [net.to_device(WL.batch_target(wl, n), is_label=True) for n in range(1, steps + 1)]
        losses = torch.zeros(steps, dtype=torch.float32, device=DEV)
        slot = torch.zeros(1, dtype=torch.float32, device=DEV)
        torch.cuda.synchronize()
        for n in range(steps):
            if n % 5 == 3:
                lp.lp_sync(net.ctx)
                lp.lp_set_fused_hadamard(net.ctx, (n // 5) % 2 == 1)
            lp.lp_step(net.ctx, xs[n], ts[n], None, slot, net.streams)
            with torch.cuda.stream(net.streams[0]):
                losses[n:n + 1].copy_(slot)
        lp.lp_sync(net.ctx)
        torch.cuda.synchronize()
        assert np.array_equal(losses.cpu().numpy().view(np.uint32), ref[0].view(np.uint32)), graphs
        for l in range(1, wl.L + 1):
            assert np.array_equal(net.get_weights(l).view(np.uint32), ref[1][l - 1].view(np.uint32)), (graphs, l)
        net.close()
