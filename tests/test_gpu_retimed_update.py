"""Retimed update (lp_set_retimed_update): the delay elements of Eq. 6 sit on the weights instead of on the gradient
(Sec. III-A: retiming leaves the delays between W and its readers).  The G task applies its gradient at once in the
product's epilogue and writes a new weight version; steps read the version that is d_l + 1 steps old.  The same
gradients are applied in the same order as with the gradient ring, so the weights every step reads, the losses, and
-- d_l steps later -- the master weights must agree with it bit for bit, in every schedule; the path is also compared
with the CPU oracle directly.  Needs a real MI355X."""
import numpy as np
import pytest
import torch

import lp_workloads as WL
import paper_2108_06629_amd as lp
from oracle import layerpipe_oracle as O
from test_gpu_parity import DEV

pytestmark = pytest.mark.gpu


def make(wl, W0, **kw):
    net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, **kw)
    net.set_weights(W0)
    return net


def batches(net, wl, steps):
    xs = [net.to_device(WL.batch_input(wl, n)) for n in range(1, steps + 1)]
    ts = [net.to_device(WL.batch_target(wl, n), is_label=(wl.loss == WL.SOFTMAX_CE)) for n in range(1, steps + 1)]
    torch.cuda.synchronize()
    return xs, ts


def lockstep(wl, W0, steps, ref_kw, kw, retimed_layers):
    """Runs the gradient-ring form and the retimed form side by side: after every step the losses and the working
    weights the next step will read must hold the same bits.  The gradient-ring run goes on for max d_l more steps
    (their gradients are not applied to anything compared here); its master weights after step steps + d_l are the
    retimed master weights after `steps` steps."""
    d_max = max(wl.delays)
    ref, net = make(wl, W0, **ref_kw), make(wl, W0, **kw)
    xs, ts = batches(ref, wl, steps + d_max)
    l_ref = torch.zeros(steps + d_max, dtype=torch.float32, device=DEV)
    l_net = torch.zeros(steps, dtype=torch.float32, device=DEV)
    torch.cuda.synchronize()
    masters, ref_now = {}, {}
    retimed_only = set(retimed_layers or ()) - set(kw.get("factor_ring") or [])
    for n in range(steps + d_max):
        lp.lp_step(ref.ctx, xs[n], ts[n], None, l_ref[n:n + 1], ref.streams)
        lp.lp_sync(ref.ctx)
        for l in range(1, wl.L + 1):
            if n + 1 == steps + wl.delays[l - 1]:
                masters[l] = ref.get_weights(l)
            if n + 1 == steps:
                ref_now[l] = ref.get_weights(l)
        if n >= steps:
            continue
        lp.lp_step(net.ctx, xs[n], ts[n], None, l_net[n:n + 1], net.streams)
        lp.lp_sync(net.ctx)
        for l in range(1, wl.L + 1):
            a, b = ref.tensor(l, lp.LP_T_WORK_W), net.tensor(l, lp.LP_T_WORK_W)
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), "working W_%d after step %d" % (l, n + 1)
    losses = l_net.cpu().numpy()
    assert np.all(np.isfinite(losses)) and losses[0] != losses[-1]
    assert np.array_equal(losses.view(np.uint32), l_ref[:steps].cpu().numpy().view(np.uint32))
    if retimed_layers is None:          # whatever "every layer" selected
        retimed_layers = {l for l in range(1, wl.L + 1) if net.tensor(l, lp.LP_T_G_LAST) is None}
        retimed_only = set(retimed_layers)
        assert retimed_only
    for l in range(1, wl.L + 1):
        is_ret = net.tensor(l, lp.LP_T_G_LAST) is None
        assert is_ret == (l in retimed_layers), (l, is_ret)
        w = net.get_weights(l)
        # a retimed layer (not a factor ring, whose master weights are not ahead) holds every gradient computed so far
        want = masters[l] if l in retimed_only else ref_now[l]
        bad = w.view(np.uint32) != want.view(np.uint32)
        assert not bad.any(), "master W_%d: %d of %d differ, max %g" % (l, bad.sum(), bad.size, np.max(np.abs(w - want)))
    ref.close()
    net.close()


# widths: aligned and ragged (register-staged loop), a layer wide enough for 256 x 256 tiles
@pytest.mark.parametrize("widths,batch", [([256, 320, 192, 136, 40], 96), ([77, 130, 19, 10], 33), ([512, 4096, 3072, 1000], 64)])
def test_retimed_update_bits_equal_gradient_ring(widths, batch):
    L = len(widths) - 1
    wl = WL.mlp_4096().with_(layers=WL._mlp(widths, WL.RELU), batch=batch, delays=tuple(2 * (L - l) for l in range(1, L + 1)))
    W0 = WL.init_weights(wl)
    every = set(range(1, L + 1))
    lockstep(wl, W0, 11, {}, dict(retimed_update=True), every)
    lockstep(wl, W0, 11, {}, dict(retimed_update=[1, L]), {1, L})      # mixed: the others keep the gradient ring
    lockstep(wl, W0, 11, dict(n_streams=1), dict(retimed_update=True, n_streams=1), every)


def test_retimed_update_with_run_ahead_graphs_factor_ring_and_odd_delays():
    wl = WL.mlp_4096().with_(layers=WL._mlp([256, 320, 192, 136, 40], WL.GELU), batch=96, delays=(3, 0, 1, 0))
    W0 = WL.init_weights(wl)
    every = {1, 2, 3, 4}
    lockstep(wl, W0, 30, {}, dict(retimed_update=True, run_ahead=True), every)
    lockstep(wl, W0, 30, {}, dict(retimed_update=True, run_ahead=True, n_streams=2), every)
    lockstep(wl, W0, 30, {}, dict(retimed_update=True, graphs=True), every)
    # layers 2 and 3 on a factor ring, 1 and 4 retimed (LP_T_G_LAST is NULL for both kinds)
    lockstep(wl, W0, 30, {}, dict(retimed_update=[1, 4], factor_ring=[2, 3]), every)
    lockstep(wl, W0, 30, {}, dict(retimed_update=[1, 4], factor_ring=[2, 3], run_ahead=True), every)


@pytest.mark.parametrize("act", [WL.TANH, WL.SIGMOID, WL.GELU])
def test_retimed_update_with_other_activations_and_separate_hadamard_kernels(act):
    """tanh / sigmoid layers keep the stand-alone Hadamard kernels; GELU is run here with the fused form switched off."""
    wl = WL.mlp_4096().with_(layers=WL._mlp([136, 264, 200, 72, 24], act), batch=40, delays=(5, 2, 1, 0))
    W0 = WL.init_weights(wl)
    every = {1, 2, 3, 4}
    lockstep(wl, W0, 14, {}, dict(retimed_update=True, fused_hadamard=False), every)
    lockstep(wl, W0, 14, dict(fused_hadamard=False), dict(retimed_update=True, run_ahead=True), every)


def test_retimed_update_graph_replay_really_replays():
    wl = WL.mlp_4096().with_(layers=WL._mlp([256, 320, 192, 40], WL.RELU), batch=96, delays=(4, 2, 0))
    W0 = WL.init_weights(wl)
    ref, net = make(wl, W0), make(wl, W0, retimed_update=True, graphs=True)
    pool = 8                                   # version rings of 8, 4 and 2 slots: the buffer choice repeats every 8 steps
    xs, ts = batches(ref, wl, pool)
    steps = 40
    l_ref = torch.zeros(steps, dtype=torch.float32, device=DEV)
    slot = torch.zeros(1, dtype=torch.float32, device=DEV)
    got = []
    torch.cuda.synchronize()
    for n in range(steps):
        lp.lp_step(ref.ctx, xs[n % pool], ts[n % pool], None, l_ref[n:n + 1], ref.streams)
        lp.lp_step(net.ctx, xs[n % pool], ts[n % pool], None, slot, net.streams)
        lp.lp_sync(net.ctx)
        got.append(float(slot.item()))
    lp.lp_sync(ref.ctx)
    captured, replayed, eager = lp.lp_graph_stats(net.ctx)
    assert replayed >= 16 and captured <= 8, (captured, replayed, eager)
    assert np.array_equal(np.asarray(got, dtype=np.float32).view(np.uint32), l_ref.cpu().numpy().view(np.uint32))
    for l in range(1, wl.L + 1):
        assert torch.equal(ref.tensor(l, lp.LP_T_WORK_W).view(torch.int16), net.tensor(l, lp.LP_T_WORK_W).view(torch.int16))
    ref.close()
    net.close()


def test_retimed_update_with_delta_split():
    wl = WL.mlp_4096().with_(layers=WL._mlp([256, 320, 192, 136, 40], WL.RELU), batch=96, delays=(6, 4, 2, 0))
    W0 = WL.init_weights(wl)
    ref, net = make(wl, W0), make(wl, W0, retimed_update=True)
    lp.lp_set_delta_split(net.ctx, 3, 64)
    lp.lp_set_delta_split(net.ctx, 2, 100)
    xs, ts = batches(ref, wl, 12)
    la, lb = torch.zeros(12, dtype=torch.float32, device=DEV), torch.zeros(12, dtype=torch.float32, device=DEV)
    torch.cuda.synchronize()
    for n in range(12):
        lp.lp_step(ref.ctx, xs[n], ts[n], None, la[n:n + 1], ref.streams)
        lp.lp_step(net.ctx, xs[n], ts[n], None, lb[n:n + 1], net.streams)
    lp.lp_sync(ref.ctx)
    lp.lp_sync(net.ctx)
    assert torch.equal(la.view(torch.int32), lb.view(torch.int32))
    ref.close()
    net.close()


def test_retimed_update_where_the_gradient_product_is_split_over_k():
    """Batch 2048: the G products of the 512 x 512 and 512 x 4096 layers are cut into K ranges -- the kernel that adds
    their partial sums applies the update, K cut exactly where lp_grad_weight cuts it; the 4096 x 4096 layer runs the
    tiled GEMM and the 4096 x 16 layer the few-outputs kernel.  All four are retimed, alone and together."""
    wl = WL.mlp_4096().with_(layers=WL._mlp([512, 512, 4096, 4096, 16], WL.RELU), batch=2048, delays=(6, 4, 2, 0))
    W0 = WL.init_weights(wl)
    lockstep(wl, W0, 9, {}, dict(retimed_update=True), {1, 2, 3, 4})
    lockstep(wl, W0, 9, {}, dict(retimed_update=[1, 2]), {1, 2})
    lockstep(wl, W0, 9, {}, dict(retimed_update=True, run_ahead=True), {1, 2, 3, 4})
    # ragged: 520 x 264 outputs (the register-staged loop) over a batch of 2100
    wl = WL.mlp_4096().with_(layers=WL._mlp([520, 264, 72], WL.RELU), batch=2100, delays=(2, 0))
    lockstep(wl, WL.init_weights(wl), 6, {}, dict(retimed_update=True), {1, 2})


def test_retimed_update_in_a_network_with_convolutions():
    """A convolution applies its update in the kernel that sums the split-K partials of its G product (also the
    three-channel image layer), the ten-output classifier in the few-outputs kernel: every layer of the small VGG is
    retimed.  With a wider head on top (tiled GEMM) as well; and with only some of the layers retimed."""
    base = WL.vgg_small(batch=16)
    W0 = WL.init_weights(base)
    lockstep(base, W0, 16, {}, dict(retimed_update=True), set(range(1, base.L + 1)))
    lockstep(base, W0, 8, {}, dict(retimed_update=[2, 5, base.L]), {2, 5, base.L})
    lockstep(base, W0, 16, {}, dict(retimed_update=True, run_ahead=True), set(range(1, base.L + 1)))
    lockstep(base, W0, 20, {}, dict(retimed_update=True, graphs=True), set(range(1, base.L + 1)))   # steps past the warm-up run as captured graphs
    layers = tuple(base.layers[:-1]) + (WL.Layer(WL.LINEAR, base.layers[-1].d_in, 256, WL.RELU), WL.Layer(WL.LINEAR, 256, 64, WL.IDENTITY))
    L = len(layers)
    wl = base.with_(layers=layers, delays=tuple(2 * (L - l) for l in range(1, L + 1)))
    lockstep(wl, WL.init_weights(wl), 6, {}, dict(retimed_update=True), set(range(1, L + 1)))


def test_retimed_update_entry_points_and_errors():
    wl = WL.mlp_4096().with_(layers=WL._mlp([256, 320, 192, 40], WL.RELU), batch=96, delays=(4, 2, 0))
    W0 = WL.init_weights(wl)
    net = make(wl, W0, retimed_update=[1, 3])
    xs, ts = batches(net, wl, 2)
    # before any step: master and the working weights are the given weights and their rounding
    for l in (1, 2, 3):
        assert np.array_equal(net.get_weights(l), W0[l - 1])
        assert np.array_equal(net.tensor_np(l, lp.LP_T_WORK_W).reshape(W0[l - 1].shape), O.round_bf16(W0[l - 1]))
    with pytest.raises(lp.LpError) as e:
        lp.lp_step(net.ctx, xs[0], ts[0], [2, 2, 0], net.loss_dev, net.streams)      # layer 1 is retimed: its delay is fixed
    assert e.value.status == 5
    lp.lp_step(net.ctx, xs[0], ts[0], [4, 1, 0], net.loss_dev, net.streams)          # layer 2 has a gradient ring: free
    lp.lp_sync(net.ctx)
    G = torch.zeros(256, 320, dtype=torch.float32, device=DEV)
    torch.cuda.synchronize()
    for g in (G, None):
        with pytest.raises(lp.LpError) as e:
            lp.lp_update(net.ctx, 1, g, net.streams[0])
        assert e.value.status == 6
    lp.lp_update(net.ctx, 2, None, net.streams[0])
    lp.lp_sync(net.ctx)
    # one gradient applied to the master weights of the retimed layers; the step to come still reads version 0
    # of layer 1 (d = 4) and version 1 of layer 3 (d = 0), which is the rounded master
    w1, w3 = net.get_weights(1), net.get_weights(3)
    assert not np.array_equal(w1, W0[0]) and not np.array_equal(w3, W0[2])
    assert np.array_equal(net.tensor_np(1, lp.LP_T_WORK_W).reshape(w1.shape), O.round_bf16(W0[0]))
    assert np.array_equal(net.tensor_np(3, lp.LP_T_WORK_W).reshape(w3.shape), O.round_bf16(w3))
    # new weights in the middle of a run: every held version
    net.set_weights(W0)
    lp.lp_step(net.ctx, xs[1], ts[1], None, net.loss_dev, net.streams)
    lp.lp_sync(net.ctx)
    assert np.array_equal(net.tensor_np(1, lp.LP_T_WORK_W).reshape(w1.shape), O.round_bf16(W0[0]))
    net.close()
    with pytest.raises(lp.LpError) as e:
        lp.Network(wl.layers, wl.batch, "f32", wl.loss, wl.lr, wl.delays, retimed_update=True)
    assert e.value.status == 3
    with pytest.raises(lp.LpError) as e:
        lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, retimed_update=[2], factor_ring=[2])
    assert e.value.status == 4


def test_retimed_update_per_layer_calls():
    """Driving a step by hand: lp_grad_weight with G == NULL is the whole G task of a retimed layer."""
    from test_gpu_parity import dev, host
    B, K, N = 64, 264, 136
    net = lp.Network((WL.Layer(WL.LINEAR, K, N, WL.RELU), WL.Layer(WL.LINEAR, N, 8, WL.IDENTITY)), B, "bf16", WL.SOFTMAX_CE, 0.05, (1, 0),
                     retimed_update=[1])
    rng = np.random.default_rng(5)
    W = [(rng.standard_normal(l.weight_shape) * 0.1).astype(np.float32) for l in net.layers]
    net.set_weights(W)
    x = rng.standard_normal((B, K)).astype(np.float32)
    dy = (rng.standard_normal((B, N)) / N).astype(np.float32)
    xd, dyd = dev(x, torch.bfloat16), dev(dy, torch.bfloat16)
    s = net.streams[0]
    lp.lp_grad_weight(net.ctx, 1, xd, dyd, None, s)
    lp.lp_sync(net.ctx)
    g = O.grad_weight(O.round_bf16(x), O.round_bf16(dy))
    ref = O.store(O.delayed_sgd(W[0].astype(np.float64), g, float(np.float32(0.05))), "f32")
    w = net.get_weights(1)
    assert np.max(np.abs(w - ref)) <= 2e-4 * 0.05 * np.max(np.abs(g)) + 2.0 ** -22 * np.max(np.abs(ref))
    # d = 1: the next step (n = 2) still reads version 0, the one after it the version just written
    lp.lp_advance(net.ctx)
    assert np.array_equal(net.tensor_np(1, lp.LP_T_WORK_W).reshape(w.shape), O.round_bf16(W[0]))
    lp.lp_advance(net.ctx)
    assert np.array_equal(net.tensor_np(1, lp.LP_T_WORK_W).reshape(w.shape), O.round_bf16(w))
    # an explicit G still goes through the stand-alone kernel and leaves the weights alone
    G = torch.empty(K, N, dtype=torch.float32, device=DEV)
    lp.lp_grad_weight(net.ctx, 1, xd, dyd, G, s)
    lp.lp_sync(net.ctx)
    assert np.max(np.abs(host(G) - g)) <= 2e-4 * np.max(np.abs(g))
    assert np.array_equal(net.get_weights(1), w)
    net.close()


def test_retimed_update_against_oracle():
    """Losses against the oracle step by step; the master weights, which run d_l gradients ahead, against the oracle's
    weights d_l steps later (the oracle goes on for max d_l steps on batches whose gradients are not yet applied)."""
    wl = WL.mlp_4096().with_(layers=WL._mlp([512] * 5 + [1000], WL.RELU), batch=64, delays=(8, 6, 4, 2, 0))
    W0 = WL.init_weights(wl)
    net = make(wl, W0, retimed_update=True)
    ora = O.DelayedGradientTrainer(wl.layers, W0, wl.delays, wl.lr, wl.loss, "bf16")
    T, d_max = 12, max(wl.delays)
    for n in range(1, T + d_max + 1):
        x, t = WL.batch_input(wl, n), WL.batch_target(wl, n)
        ref = ora.step(x, t)
        if n <= T:
            loss = net.step(x, t)
            assert abs(loss - ref) <= 2e-2 * max(abs(ref), 1e-3), (n, loss, ref)
            if n == T:
                got = [net.get_weights(l) for l in range(1, wl.L + 1)]
        for l in range(1, wl.L + 1):
            if n == T + wl.delays[l - 1]:
                wr = ora.W[l - 1]
                assert np.max(np.abs(got[l - 1] - wr)) <= 2e-2 * np.max(np.abs(wr)), l
                assert not np.array_equal(got[l - 1], W0[l - 1])
    net.close()
