"""Forward run-ahead across steps (Sec. III-A): F(n+1) on its own stream, overlapping the backward
pass of step n.  The schedule changes no arithmetic, so the proof is bit-identity with the serial
lp_step on the same inputs, with the steps enqueued back to back (no host wait in between, which
is when the overlap really happens); the run-ahead path is also compared with the CPU oracle
directly.  Needs a real MI355X."""
import numpy as np
import pytest
import torch

import lp_workloads as WL
import paper_2108_06629_amd as lp
from test_gpu_parity import DEV, run_trajectory

pytestmark = pytest.mark.gpu


def enqueue_steps(wl, W0, steps, run_ahead, split=None, delays_now=None, n_streams=None):
    """All `steps` training steps enqueued without waiting; returns (losses, weights, last gradients)."""
    net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays,
                     n_streams=n_streams or (4 if run_ahead else 3), run_ahead=run_ahead)
    net.set_weights(W0)
    if split:
        for l, cols in split.items():
            lp.lp_set_delta_split(net.ctx, l, cols)
    xs = [net.to_device(WL.batch_input(wl, n)) for n in range(1, steps + 1)]
    ts = [net.to_device(WL.batch_target(wl, n), is_label=(wl.loss == WL.SOFTMAX_CE)) for n in range(1, steps + 1)]
    losses = torch.zeros(steps, dtype=torch.float32, device=DEV)
    torch.cuda.synchronize()
    for n in range(steps):
        lp.lp_step(net.ctx, xs[n], ts[n], delays_now, losses[n:n + 1], net.streams)
    lp.lp_sync(net.ctx)
    out = (losses.cpu().numpy().copy(), [net.get_weights(l) for l in range(1, wl.L + 1)],
           [net.tensor_np(l, lp.LP_T_G_LAST) for l in range(1, wl.L + 1)])
    net.close()
    return out


def assert_same_bits(a, b):
    assert np.array_equal(a[0].view(np.uint32), b[0].view(np.uint32)), (a[0], b[0])
    for l, (wa, wb) in enumerate(zip(a[1], b[1]), start=1):
        assert np.array_equal(wa.view(np.uint32), wb.view(np.uint32)), "W_%d" % l
    for l, (ga, gb) in enumerate(zip(a[2], b[2]), start=1):
        assert np.array_equal(ga.view(np.uint32), gb.view(np.uint32)), "G_%d" % l


def test_run_ahead_mlp_bits_equal_serial_schedule():
    # widths chosen so that some products split K (few tiles, long reduction) and others do not
    wl = WL.mlp_4096().with_(layers=WL._mlp([1024, 2048, 256, 1032, 520, 1000], WL.RELU), batch=160, delays=(8, 6, 4, 2, 0))
    W0 = WL.init_weights(wl)
    serial = enqueue_steps(wl, W0, 14, False)
    ahead = enqueue_steps(wl, W0, 14, True)
    assert np.all(np.isfinite(serial[0])) and serial[0][0] != serial[0][-1]
    assert_same_bits(serial, ahead)


def test_run_ahead_with_delta_split_and_odd_delays():
    # d_l = 1 makes update_l(n+1) read the gradient written one step earlier; d = 0 in the middle of the
    # network makes a forward task wait for the backward pass of the same layer
    wl = WL.mlp_4096().with_(layers=WL._mlp([256, 320, 192, 136, 40], WL.RELU), batch=96, delays=(3, 0, 1, 0))
    W0 = WL.init_weights(wl)
    serial = enqueue_steps(wl, W0, 9, False)
    ahead = enqueue_steps(wl, W0, 9, True, split={2: 64, 4: 40})
    assert_same_bits(serial, ahead)


def test_run_ahead_gelu_mse_stack():
    wl = WL.ffn_stack(d=256, hidden=1024, tokens=512, n_linear=6)
    W0 = WL.init_weights(wl)
    assert_same_bits(enqueue_steps(wl, W0, 12, False), enqueue_steps(wl, W0, 12, True))


def test_run_ahead_cnn_with_pooling():
    wl = WL.vgg_small(batch=16, hw=16, chans=(16, 16, 32, 32))
    W0 = WL.init_weights(wl)
    assert_same_bits(enqueue_steps(wl, W0, 10, False), enqueue_steps(wl, W0, 10, True))


def test_run_ahead_against_oracle():
    wl = WL.mlp_4096().with_(layers=WL._mlp([512] * 5 + [1000], WL.RELU), batch=64, delays=(8, 6, 4, 2, 0))
    run_trajectory(wl, 12, n_streams=4, run_ahead=True)


def test_run_ahead_stream_handles():
    wl = WL.mlp_4096().with_(layers=WL._mlp([64, 64, 16], WL.RELU), batch=16, delays=(2, 0))
    net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, n_streams=4, run_ahead=True)
    net.set_weights(WL.init_weights(wl))
    x, t = net.to_device(WL.batch_input(wl, 1)), net.to_device(WL.batch_target(wl, 1), True)
    with pytest.raises(lp.LpError) as e:
        lp.lp_step(net.ctx, x, t, None, net.loss_dev, net.streams[:3])
    assert e.value.status == 6     # LP_ERR_STATE: four handles are needed
    with pytest.raises(lp.LpError) as e:
        lp.lp_step(net.ctx, x, t, None, net.loss_dev, [net.streams[0], net.streams[1], net.streams[2], net.streams[0]])
    assert e.value.status == 6     # LP_ERR_STATE: the forward chain needs a stream of its own
    lp.lp_step(net.ctx, x, t, None, net.loss_dev, net.streams)
    lp.lp_sync(net.ctx)
    assert np.isfinite(float(net.loss_dev.item()))
    net.close()


@pytest.mark.parametrize("n_streams", [2, 3])
def test_run_ahead_with_shared_streams_bits_equal_serial_schedule(n_streams):
    # the G tasks and/or the updates share a stream with another role: stronger ordering, same arithmetic
    wl = WL.mlp_4096().with_(layers=WL._mlp([256, 320, 192, 136, 40], WL.RELU), batch=96, delays=(3, 0, 1, 0))
    W0 = WL.init_weights(wl)
    serial = enqueue_steps(wl, W0, 9, False)
    shared = enqueue_steps(wl, W0, 9, True, split={2: 64}, n_streams=n_streams)
    assert_same_bits(serial, shared)
