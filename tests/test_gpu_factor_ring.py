"""Factor ring (lp_set_factor_ring): the delay elements hold (A_{l-1}, dY_l) and the delayed update forms
G_l(n - d_l) itself, applying it in the product's epilogue.  Same arithmetic as the product ring, so
weights and losses must agree bit for bit with it, in every schedule; the path is also compared with
the CPU oracle directly.  Needs a real MI355X."""
import numpy as np
import pytest
import torch

import lp_workloads as WL
import paper_2108_06629_amd as lp
from oracle import layerpipe_oracle as O
from test_gpu_parity import DEV, dev, host, one_layer_net

pytestmark = pytest.mark.gpu


def run(wl, W0, steps, **kw):
    net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, **kw)
    net.set_weights(W0)
    xs = [net.to_device(WL.batch_input(wl, n)) for n in range(1, steps + 1)]
    ts = [net.to_device(WL.batch_target(wl, n), is_label=(wl.loss == WL.SOFTMAX_CE)) for n in range(1, steps + 1)]
    losses = torch.zeros(steps, dtype=torch.float32, device=DEV)
    torch.cuda.synchronize()
    for n in range(steps):
        lp.lp_step(net.ctx, xs[n], ts[n], None, losses[n:n + 1], net.streams)
    lp.lp_sync(net.ctx)
    out = (losses.cpu().numpy().copy(), [net.get_weights(l) for l in range(1, wl.L + 1)],
           [net.tensor_np(l, lp.LP_T_WORK_W) for l in range(1, wl.L + 1)])
    net.close()
    return out


def assert_same(a, b):
    assert np.array_equal(a[0].view(np.uint32), b[0].view(np.uint32)), (a[0], b[0])
    for l, (wa, wb) in enumerate(zip(a[1], b[1]), start=1):
        assert np.array_equal(wa.view(np.uint32), wb.view(np.uint32)), "master W_%d" % l
    for l, (wa, wb) in enumerate(zip(a[2], b[2]), start=1):
        assert np.array_equal(wa, wb), "working W_%d" % l


# widths: aligned and ragged (register-staged loop), a layer wide enough for 256 x 256 tiles
@pytest.mark.parametrize("widths,batch", [([256, 320, 192, 136, 40], 96), ([77, 130, 19, 10], 33), ([512, 4096, 3072, 1000], 64)])
def test_factor_ring_bits_equal_product_ring(widths, batch):
    L = len(widths) - 1
    wl = WL.mlp_4096().with_(layers=WL._mlp(widths, WL.RELU), batch=batch, delays=tuple(2 * (L - l) for l in range(1, L + 1)))
    W0 = WL.init_weights(wl)
    ref = run(wl, W0, 11)
    assert np.all(np.isfinite(ref[0]))
    assert_same(ref, run(wl, W0, 11, factor_ring=True))
    assert_same(ref, run(wl, W0, 11, factor_ring=[1, L]))            # mixed: some layers keep the product ring
    assert_same(ref, run(wl, W0, 11, factor_ring=True, n_streams=1))


def test_factor_ring_skips_layers_whose_gradient_product_is_split_over_k():
    """Batch 2048: the G products of 512 x 512, 512 x 4096 and 4096 x 16 layers are cut into K ranges by
    lp_grad_weight; the fused update never cuts K, so "every layer" leaves those on the product ring and only the
    4096 x 4096 layer keeps its factors.  Bits equal the all-product-ring run."""
    wl = WL.mlp_4096().with_(layers=WL._mlp([512, 512, 4096, 4096, 16], WL.RELU), batch=2048, delays=(6, 4, 2, 0))
    W0 = WL.init_weights(wl)
    ref = run(wl, W0, 9)
    assert np.all(np.isfinite(ref[0])) and ref[0][0] != ref[0][-1]
    assert_same(ref, run(wl, W0, 9, factor_ring=True))
    net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, factor_ring=True)
    net.set_weights(W0)
    net.step(WL.batch_input(wl, 1), WL.batch_target(wl, 1))
    assert [net.tensor(l, lp.LP_T_G_LAST) is None for l in (1, 2, 3, 4)] == [False, False, True, False]
    net.close()
    with pytest.raises(lp.LpError) as e:
        lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, factor_ring=[1])
    assert e.value.status == 4


def test_factor_ring_with_run_ahead_graphs_and_odd_delays():
    wl = WL.mlp_4096().with_(layers=WL._mlp([256, 320, 192, 136, 40], WL.GELU), batch=96, delays=(3, 0, 1, 0))
    W0 = WL.init_weights(wl)
    ref = run(wl, W0, 30)
    assert_same(ref, run(wl, W0, 30, factor_ring=True, run_ahead=True))
    assert_same(ref, run(wl, W0, 30, factor_ring=True, graphs=True))


def test_factor_ring_per_layer_calls_and_missing_G():
    B, K, N = 64, 264, 136
    net = lp.Network((WL.Layer(WL.LINEAR, K, N, WL.RELU), WL.Layer(WL.LINEAR, N, 8, WL.IDENTITY)), B, "bf16", WL.SOFTMAX_CE, 0.05, (0, 0),
                     factor_ring=[1])
    rng = np.random.default_rng(5)
    W = [(rng.standard_normal(l.weight_shape) * 0.1).astype(np.float32) for l in net.layers]
    net.set_weights(W)
    x = rng.standard_normal((B, K)).astype(np.float32)
    dy = (rng.standard_normal((B, N)) / N).astype(np.float32)
    xd, dyd = dev(x, torch.bfloat16), dev(dy, torch.bfloat16)
    s = net.streams[0]
    lp.lp_grad_weight(net.ctx, 1, xd, dyd, None, s)        # stores the factors of step 1
    lp.lp_update(net.ctx, 1, None, s)                      # d = 0: uses them at once
    lp.lp_sync(net.ctx)
    assert net.tensor(1, lp.LP_T_G_LAST) is None
    g = O.grad_weight(O.round_bf16(x), O.round_bf16(dy))
    ref = O.store(O.delayed_sgd(W[0].astype(np.float64), g, float(np.float32(0.05))), "f32")
    w = net.get_weights(1)
    assert np.max(np.abs(w - ref)) <= 2e-4 * 0.05 * np.max(np.abs(g)) + 2.0 ** -22 * np.max(np.abs(ref))
    work = net.tensor_np(1, lp.LP_T_WORK_W).reshape(w.shape)
    assert np.array_equal(work, O.round_bf16(w))           # the working copy is the rounded master, bit for bit
    # an explicit G still goes through the stand-alone kernels
    G = torch.empty(K, N, dtype=torch.float32, device=DEV)
    lp.lp_grad_weight(net.ctx, 1, xd, dyd, G, s)
    lp.lp_sync(net.ctx)
    assert np.max(np.abs(host(G) - g)) <= 2e-4 * np.max(np.abs(g))
    net.close()


def test_factor_ring_against_oracle():
    wl = WL.mlp_4096().with_(layers=WL._mlp([512] * 5 + [1000], WL.RELU), batch=64, delays=(8, 6, 4, 2, 0))
    W0 = WL.init_weights(wl)
    net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, factor_ring=True)
    net.set_weights(W0)
    ora = O.DelayedGradientTrainer(wl.layers, W0, wl.delays, wl.lr, wl.loss, "bf16")
    for n in range(1, 13):
        x, t = WL.batch_input(wl, n), WL.batch_target(wl, n)
        loss, ref = net.step(x, t), ora.step(x, t)
        assert abs(loss - ref) <= 2e-2 * max(abs(ref), 1e-3), (n, loss, ref)
        for l in range(1, wl.L + 1):
            w, wr = net.get_weights(l), ora.W[l - 1]
            if n <= wl.delays[l - 1]:
                assert np.array_equal(w, W0[l - 1]), ("frozen", l, n)
            assert np.max(np.abs(w - wr)) <= 2e-2 * np.max(np.abs(wr)), (l, n)
    net.close()
