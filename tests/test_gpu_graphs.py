"""Graph replay of whole steps (lp_set_graphs): a captured step must give the bits of the same step
enqueued kernel by kernel, on every replay, with other work and host waits between the replays.
Needs a real MI355X."""
import numpy as np
import pytest
import torch

import lp_workloads as WL
import paper_2108_06629_amd as lp
from test_gpu_parity import DEV, run_trajectory
from test_gpu_run_ahead import assert_same_bits

pytestmark = pytest.mark.gpu


def run_steps(wl, W0, steps, graphs, n_streams=3, pool=3, sync_every=0, split=None):
    """Steps fed from a rotating pool of `pool` resident minibatches (as a training loop would).  Returns
    (losses, weights, last gradients, graph counters)."""
    net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, n_streams=n_streams, graphs=graphs)
    net.set_weights(W0)
    if split:
        for l, cols in split.items():
            lp.lp_set_delta_split(net.ctx, l, cols)
    xs = [net.to_device(WL.batch_input(wl, n)) for n in range(1, pool + 1)]
    ts = [net.to_device(WL.batch_target(wl, n), is_label=(wl.loss == WL.SOFTMAX_CE)) for n in range(1, pool + 1)]
    losses = torch.zeros(steps, dtype=torch.float32, device=DEV)
    loss_slot = torch.zeros(1, dtype=torch.float32, device=DEV)      # one fixed address, as a captured step needs
    scratch = torch.zeros(1 << 16, device=DEV)
    torch.cuda.synchronize()
    for n in range(steps):
        lp.lp_step(net.ctx, xs[n % pool], ts[n % pool], None, loss_slot, net.streams)
        with torch.cuda.stream(net.streams[0]):
            losses[n:n + 1].copy_(loss_slot)                           # eager work of the program between the replays
            scratch.add_(1.0)
        if sync_every and n % sync_every == sync_every - 1:
            lp.lp_sync(net.ctx)
    lp.lp_sync(net.ctx)
    torch.cuda.synchronize()
    out = (losses.cpu().numpy().copy(), [net.get_weights(l) for l in range(1, wl.L + 1)],
           [net.tensor_np(l, lp.LP_T_G_LAST) for l in range(1, wl.L + 1)])
    stats = lp.lp_graph_stats(net.ctx)
    net.close()
    return out, stats


@pytest.mark.parametrize("n_streams", [3, 1])
def test_graph_replay_mlp_bits_equal_eager_steps(n_streams):
    wl = WL.mlp_4096().with_(layers=WL._mlp([1024, 2048, 256, 1032, 520, 1000], WL.RELU), batch=160, delays=(8, 6, 4, 2, 0))
    W0 = WL.init_weights(wl)
    steps = 110       # rings of 16, 8, 4, 2, 1 slots -> period 16; pool of 3 -> 48 combinations, then replays
    eager, s0 = run_steps(wl, W0, steps, False, n_streams)
    graph, s1 = run_steps(wl, W0, steps, True, n_streams, sync_every=7)
    assert s0 == (0, 0, 0)
    captured, replayed, uncaptured = s1
    assert uncaptured == 8 + 2 and captured == 48 and replayed == steps - 10 - 48, s1
    assert np.all(np.isfinite(eager[0]))
    assert_same_bits(eager, graph)


def test_graph_replay_f32_and_delta_split():
    wl = WL.mlp_small()
    W0 = WL.init_weights(wl)
    eager, _ = run_steps(wl, W0, 40, False, pool=2)
    graph, st = run_steps(wl, W0, 40, True, pool=2, sync_every=5)
    assert st[1] > 0
    assert_same_bits(eager, graph)
    wl = WL.mlp_4096().with_(layers=WL._mlp([256, 320, 192, 136, 40], WL.RELU), batch=96, delays=(3, 0, 1, 0))
    W0 = WL.init_weights(wl)
    eager, _ = run_steps(wl, W0, 30, False, pool=2)
    graph, st = run_steps(wl, W0, 30, True, pool=2, split={2: 64, 4: 40})
    assert st[1] > 0
    assert_same_bits(eager, graph)


def test_graph_replay_cnn_and_gelu_stack():
    wl = WL.vgg_small(batch=16, hw=16, chans=(16, 16, 32, 32))
    W0 = WL.init_weights(wl)
    eager, _ = run_steps(wl, W0, 40, False, pool=2)
    graph, st = run_steps(wl, W0, 40, True, pool=2, sync_every=9)
    assert st[1] > 0
    assert_same_bits(eager, graph)
    wl = WL.ffn_stack(d=256, hidden=1024, tokens=512, n_linear=4)
    W0 = WL.init_weights(wl)
    eager, _ = run_steps(wl, W0, 36, False, pool=2)
    graph, st = run_steps(wl, W0, 36, True, pool=2)
    assert st[1] > 0
    assert_same_bits(eager, graph)


def test_graph_replay_against_oracle():
    # Network.step uploads a fresh minibatch every step; the caching allocator hands the same few
    # addresses back, so later steps replay captured graphs with new data at the old addresses
    wl = WL.mlp_4096().with_(layers=WL._mlp([256, 256, 128, 40], WL.RELU), batch=64, delays=(2, 1, 0))
    W0 = WL.init_weights(wl)
    import oracle.layerpipe_oracle as O
    net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, graphs=True)
    net.set_weights(W0)
    ora = O.DelayedGradientTrainer(wl.layers, W0, wl.delays, wl.lr, wl.loss, "bf16")
    x_dev = net.to_device(WL.batch_input(wl, 1))
    t_dev = net.to_device(WL.batch_target(wl, 1), is_label=True)
    for n in range(1, 21):
        x, t = WL.batch_input(wl, n), WL.batch_target(wl, n)
        x_dev.copy_(net.to_device(x)); t_dev.copy_(net.to_device(t, is_label=True))
        torch.cuda.synchronize()
        net.step_device(x_dev, t_dev)
        lp.lp_sync(net.ctx)
        loss, ref = float(net.loss_dev.item()), ora.step(x, t)
        assert abs(loss - ref) <= 2e-2 * max(abs(ref), 1e-3), (n, loss, ref)
    for l in range(1, wl.L + 1):
        w, wr = net.get_weights(l), ora.W[l - 1]
        assert np.max(np.abs(w - wr)) <= 2e-2 * np.max(np.abs(wr)), l
    assert lp.lp_graph_stats(net.ctx)[1] > 0
    net.close()
