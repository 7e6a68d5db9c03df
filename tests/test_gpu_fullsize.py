"""Parity at the full sizes of the benchmark workloads, in the launch configuration bench.py times
(lp_step on three streams).  The three mid-size workloads run whole steps against the oracle; the
largest one (16 x 4096<->16384, 8192 tokens) is checked on sampled rows and columns of every task's
output, each recomputed by the oracle operators from the tensors that task read on the GPU.
Needs a real MI355X."""
import numpy as np
import pytest
import torch

import lp_workloads as WL
import paper_2108_06629_amd as lp
from oracle import layerpipe_oracle as O
from test_gpu_parity import relerr, run_trajectory
from test_gpu_conv import run_cnn

pytestmark = pytest.mark.gpu


# The three mid-size workloads run their delayed-gradient schedule at the benchmark's sizes against the oracle:
# every step compares loss, Z_L, every G_l (max-norm) and every W_l(n) with the oracle's trajectory, the Hadamard
# with the oracle operator on the GPU's own inputs, and every layer's delayed update (Eq. 6) with the GPU's own
# gradient of d_l steps ago; the three products and the loss are recomputed from the GPU's inputs on the listed steps.
@pytest.mark.timeout(900)
def test_mlp_4096_full_size_steps():
    wl = WL.mlp_4096()
    assert wl.batch == 256 and wl.L == 8 and wl.layers[0].d_in == 4096 and wl.layers[-1].d_out == 1000
    assert max(wl.delays) == 14
    # 17 steps: the layer with d = 14 is updated at n = 15, 16, 17
    run_trajectory(wl, 17, exact=False, product_steps={1, 2, 9, 16, 17})


@pytest.mark.timeout(900)
def test_mlp_imbalanced_full_size_step():
    wl = WL.mlp_imbalanced()
    assert wl.batch == 1024 and wl.L == 12 and wl.steps == 10
    run_trajectory(wl, wl.steps, exact=False, product_steps={1, 10})


@pytest.mark.timeout(900)
def test_vgg_small_full_size_steps():
    wl = WL.vgg_small()
    assert wl.batch == 128 and wl.gemm_dims(0) == (131072, 64, 27) and wl.steps == 20 and max(wl.delays) == 12
    run_cnn(wl, wl.steps, exact=False, product_steps={1, 2, 14, 20})


def f64(t):
    return t.to(torch.float32).cpu().numpy().astype(np.float64)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("fused", [True, False])
def test_ffn_stack_full_size_sampled(fused):
    """`fused`: the Hadamard products inside the dX products (lp_step's default) or as kernels of their own, which keeps dA.
    The largest workload for its configured 10 steps.  Layers with d_l <= 9 (the last five) receive delayed updates
    in that time; the others must stay bit-identical to their initial weights.  Every step: the update of every layer
    on a sampled 48 x 48 block of its weights against Eq. 6 with the GPU's own sampled gradient of d_l steps ago, and
    the working copy against the rounded master.  Steps 1 and 10: every task's output on sampled rows and columns,
    recomputed by the oracle operators from the tensors that task read on the GPU."""
    wl = WL.ffn_stack()
    assert wl.batch == 8192 and wl.L == 16 and wl.n_params == 16 * 4096 * 16384 and wl.steps == 10
    rng = np.random.default_rng(7)
    W0 = WL.init_weights(wl)
    net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, fused_hadamard=fused)
    net.set_weights(W0)
    B, L = wl.batch, wl.L
    rows = np.sort(rng.choice(B, 12, replace=False))
    rows[0], rows[-1] = 0, B - 1                                   # first and last tile rows
    rt = torch.from_numpy(rows).to("cuda:0")
    COLS, KIN = [], []
    for ly in wl.layers:
        cols = np.sort(rng.choice(ly.d_out, 48, replace=False)); cols[0], cols[-1] = 0, ly.d_out - 1
        kin = np.sort(rng.choice(ly.d_in, 48, replace=False)); kin[0], kin[-1] = 0, ly.d_in - 1
        COLS.append(cols); KIN.append(kin)
    W0s = [W0[l][np.ix_(KIN[l], COLS[l])].copy() for l in range(L)]
    del W0

    def view(l, which, width):
        tns = net.tensor(l, which)
        return None if tns is None else tns.view(B, width)

    def wview(l, which):
        ly = wl.layers[l - 1]
        return net.tensor(l, which).view(ly.d_in, ly.d_out)

    def wsample(l, which):
        kt, ct = torch.from_numpy(KIN[l - 1]).to("cuda:0"), torch.from_numpy(COLS[l - 1]).to("cuda:0")
        return wview(l, which)[kt][:, ct].to(torch.float32).cpu().numpy()

    G_hist = [dict() for _ in range(L)]
    eta = float(np.float32(wl.lr))
    updates_seen = 0
    for n in range(1, wl.steps + 1):
        print("ffn_stack full size: step %d" % n, flush=True)
        products = n in (1, wl.steps)
        x, t = WL.batch_input(wl, n), WL.batch_target(wl, n)
        w_before = [wsample(l, lp.LP_T_MASTER_W) for l in range(1, L + 1)]
        if products:    # the working weights F and dX of this step read: sampled columns and sampled rows
            Wc = [f64(wview(l, lp.LP_T_WORK_W)[:, torch.from_numpy(COLS[l - 1]).to("cuda:0")]) for l in range(1, L + 1)]
            Wr = [f64(wview(l, lp.LP_T_WORK_W)[torch.from_numpy(KIN[l - 1]).to("cuda:0")]) for l in range(1, L + 1)]
        xd = net.to_device(x)
        td = net.to_device(t)
        net.step_device(xd, td)
        lp.lp_sync(net.ctx)
        loss = float(net.loss_dev.item())
        A = [xd] + [view(l, lp.LP_T_A, wl.layers[l - 1].d_out) for l in range(1, L)]
        for l in range(1, L + 1):
            ly = wl.layers[l - 1]
            cols, kin = COLS[l - 1], KIN[l - 1]
            ct, kt = torch.from_numpy(cols).to("cuda:0"), torch.from_numpy(kin).to("cuda:0")
            dY = view(l, lp.LP_T_DY, ly.d_out)
            g_gpu = wsample(l, lp.LP_T_G_LAST).astype(np.float64)
            G_hist[l - 1][n] = g_gpu
            if products:
                a_rows = f64(A[l - 1][rt])                                                   # [12, d_in]
                # F (Eq. 1, Eq. 2)
                z_ref = O.store(a_rows @ Wc[l - 1], "bf16")
                zg = view(l, lp.LP_T_Z, ly.d_out)
                if zg is not None:
                    z_gpu = f64(zg[rt][:, ct])
                    assert relerr(z_gpu, z_ref) <= 2e-2, ("F/Z", l, n)
                else:
                    z_gpu = z_ref
                if l < L:
                    a_gpu = f64(A[l][rt][:, ct])
                    assert relerr(a_gpu, O.store(O.activation(z_gpu, ly.act), "bf16")) <= 2e-2, ("F/A", l, n)
                # dW (Eq. 5): G[kin, cols] = A_{l-1}[:, kin]^T . dY[:, cols], full reduction over the 8192 tokens
                g_ref = f64(A[l - 1][:, kt]).T @ f64(dY[:, ct])
                assert relerr(g_gpu, g_ref) <= 2e-4, ("dW", l, n)
                if l > 1:
                    prev = wl.layers[l - 2]
                    # dX (Eq. 4): dA_{l-1}[rows, kin] = dY[rows] . W[kin, :]^T
                    da_ref = O.store(f64(dY[rt]) @ Wr[l - 1].T, "bf16")
                    dAg = view(l - 1, lp.LP_T_DA, prev.d_out)
                    stash = view(l - 1, lp.LP_T_Z, prev.d_out)
                    stash = A[l - 1] if stash is None else stash
                    dy_prev = f64(view(l - 1, lp.LP_T_DY, prev.d_out)[rt])
                    if dAg is None:
                        # Eq. 3 was applied in the epilogue of dX_l and dA_{l-1} never stored: the two tasks together
                        assert fused and prev.act == WL.GELU, ("dA missing", l - 1, n)
                        dy_prev_ref = O.store(O.act_grad(da_ref, f64(stash[rt][:, kt]), prev.act), "bf16")
                        assert relerr(dy_prev[:, kin], dy_prev_ref) <= 2e-2, ("dX + Hadamard", l, n)
                    else:
                        assert relerr(f64(dAg[rt][:, kt]), da_ref) <= 2e-2, ("dX", l, n)
                        # the moved Hadamard (Eq. 3) on whole sampled rows
                        dy_prev_ref = O.store(O.act_grad(f64(dAg[rt]), f64(stash[rt]), prev.act), "bf16")
                        if prev.act == WL.GELU:
                            assert relerr(dy_prev, dy_prev_ref) <= 2.0 ** -7, ("Hadamard", l - 1, n)
                        else:
                            assert np.array_equal(dy_prev, dy_prev_ref), ("Hadamard", l - 1, n)
            # Eq. 6: W_l(n) = W_l(n-1) - eta G_l(n - d_l) with the GPU's own gradient of d_l steps ago
            w_gpu = wsample(l, lp.LP_T_MASTER_W)
            src = n - wl.delays[l - 1]
            if src >= 1:
                ref = O.store(O.delayed_sgd(w_before[l - 1].astype(np.float64), G_hist[l - 1].pop(src), eta), "f32")
                assert np.max(np.abs(w_gpu - ref)) <= 2.0 ** -22 * np.max(np.abs(ref)), ("update", l, n)
                assert not np.array_equal(w_gpu, w_before[l - 1]), ("update changed nothing", l, n)
                updates_seen += 1
            else:
                assert np.array_equal(w_gpu, W0s[l - 1]), ("frozen", l, n)
            assert np.array_equal(wsample(l, lp.LP_T_WORK_W), O.round_bf16(w_gpu).astype(np.float32)), ("working copy", l, n)
        if products:
            # loss and delta of the output layer on the whole tensor
            zL = f64(view(L, lp.LP_T_Z, wl.layers[-1].d_out))
            loss_ref, dy_ref = O.mse(zL, O.round_bf16(t))
            assert abs(loss - loss_ref) <= 1e-5 * loss_ref
            assert relerr(f64(view(L, lp.LP_T_DY, wl.layers[-1].d_out)), O.store(dy_ref, "bf16")) <= 2.0 ** -7
        assert np.isfinite(loss)
    assert updates_seen == sum(max(0, wl.steps - d) for d in wl.delays) == 10 + 8 + 6 + 4 + 2
    net.close()


def _run_schedule(wl, W0, steps, **kw):
    """`steps` training steps enqueued back to back from a pool of three resident minibatches; returns the
    losses and a checksum-free copy of every layer's master weights."""
    net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, **kw)
    net.set_weights(W0)
    xs = [net.to_device(WL.batch_input(wl, n)) for n in range(1, 4)]
    ts = [net.to_device(WL.batch_target(wl, n), is_label=(wl.loss == WL.SOFTMAX_CE)) for n in range(1, 4)]
    losses = torch.zeros(steps, dtype=torch.float32, device="cuda:0")
    slot = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    torch.cuda.synchronize()
    for n in range(steps):
        if kw.get("graphs"):
            # a captured step needs the same loss address every time; streams[0] carries the whole step
            lp.lp_step(net.ctx, xs[n % 3], ts[n % 3], None, slot, net.streams)
            with torch.cuda.stream(net.streams[0]):
                losses[n:n + 1].copy_(slot)
        else:
            # with run-ahead the loss of step n+1 may be written while step n still runs: one slot per step
            lp.lp_step(net.ctx, xs[n % 3], ts[n % 3], None, losses[n:n + 1], net.streams)
    lp.lp_sync(net.ctx)
    torch.cuda.synchronize()
    out = (losses.cpu().numpy().copy(), [net.get_weights(l) for l in range(1, wl.L + 1)])
    stats = lp.lp_graph_stats(net.ctx)
    net.close()
    return out, stats


@pytest.mark.parametrize("name", ["mlp_4096_bf16", "vgg_small_bf16"])
def test_full_size_schedules_and_ring_kinds_agree_bit_for_bit(name):
    """At the benchmark's shapes: serial, run-ahead, graph replay, the factor ring on top of each, and the two forms
    of the Hadamard product (inside the dX kernels, which for the CNN includes the routing of pooled gradients, or as
    kernels of their own) give the same losses and weights.  (The serial product-ring run of these workloads is the
    one the tests above compare with the oracle.)"""
    wl = WL.CONFIGS[name]()
    W0 = WL.init_weights(wl)
    steps = max(wl.delays) + 22
    ref, _ = _run_schedule(wl, W0, steps)
    assert np.all(np.isfinite(ref[0]))
    for kw in (dict(run_ahead=True), dict(graphs=True), dict(factor_ring=True), dict(factor_ring=True, run_ahead=True),
               dict(factor_ring=True, run_ahead=True, n_streams=3), dict(fused_hadamard=False), dict(fused_hadamard=False, run_ahead=True)):
        got, stats = _run_schedule(wl, W0, steps, **kw)
        assert np.array_equal(got[0].view(np.uint32), ref[0].view(np.uint32)), (kw, got[0][-4:], ref[0][-4:])
        for l, (a, b) in enumerate(zip(got[1], ref[1]), start=1):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), (kw, "W_%d" % l)
        if kw.get("graphs"):
            assert stats[0] > 0


def test_chip_filling_gradient_products_keep_the_serial_bits():
    """A layer whose G product and delta product each fill every CU with 256 x 256 tiles runs its G task behind
    dX on the critical stream instead of next to it (layers 1 and 2 here; layer 3 keeps its own stream).  The
    placement changes no arithmetic: one stream, three streams and graph replay give the same bits."""
    wl = WL.mlp_4096().with_(layers=WL._mlp([4096, 4096, 4096, 1000], WL.RELU), batch=4096, delays=(4, 2, 0))
    W0 = WL.init_weights(wl)
    ref, _ = _run_schedule(wl, W0, 9, n_streams=1)
    assert np.all(np.isfinite(ref[0])) and ref[0][0] != ref[0][-1]
    for kw in (dict(n_streams=3), dict(n_streams=3, graphs=True), dict(n_streams=3, fused_hadamard=False)):
        got, _ = _run_schedule(wl, W0, 9, **kw)
        assert np.array_equal(got[0].view(np.uint32), ref[0].view(np.uint32)), kw
        for l, (a, b) in enumerate(zip(got[1], ref[1]), start=1):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), (kw, "W_%d" % l)


@pytest.mark.timeout(600)
def test_ffn_stack_full_size_hadamard_forms_agree_bit_for_bit():
    """The largest workload, three steps in each form of the Hadamard product: every layer's dY (what the fused dX
    epilogue of 256 x 256 tiles writes for the eight GELU layers, with f' from the table) and the losses, bit for bit."""
    wl = WL.ffn_stack()
    W0 = WL.init_weights(wl)

    def run(fused):
        net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, fused_hadamard=fused)
        net.set_weights(W0)
        xs = [net.to_device(WL.batch_input(wl, n)) for n in range(1, 4)]
        ts = [net.to_device(WL.batch_target(wl, n)) for n in range(1, 4)]
        losses = torch.zeros(3, dtype=torch.float32, device="cuda:0")
        torch.cuda.synchronize()
        for n in range(3):
            lp.lp_step(net.ctx, xs[n], ts[n], None, losses[n:n + 1], net.streams)
        lp.lp_sync(net.ctx)
        has_da = [net.tensor(l, lp.LP_T_DA) is not None for l in range(1, wl.L)]
        dys = [net.tensor(l, lp.LP_T_DY).view(torch.int16).clone() for l in range(1, wl.L + 1)]
        torch.cuda.synchronize()
        out = (losses.cpu().numpy().copy(), dys, has_da)
        net.close()
        return out

    a = run(True)
    assert a[2] == [l % 2 == 0 for l in range(1, wl.L)], "dA is stored for the identity layers only"
    b = run(False)
    assert all(b[2])
    assert np.all(np.isfinite(a[0])) and np.array_equal(a[0].view(np.uint32), b[0].view(np.uint32))
    for l, (ya, yb) in enumerate(zip(a[1], b[1]), start=1):
        assert torch.equal(ya, yb), "dY_%d" % l


@pytest.mark.timeout(900)
def test_ffn_stack_full_size_retimed_update_equals_gradient_ring_bit_for_bit():
    """The largest workload in the two forms of Eq. 6, side by side for 36 steps (past the largest delay, 30, so that
    every layer reads weights that the retimed G tasks wrote): gradient rings with update tasks on three streams, and
    the retimed update on one stream, which is what bench.py times.  Losses after every step and the working weights
    of every layer at steps 1, 17 and 36, bit for bit; the retimed master weights of the last layer (d = 0) equal the
    gradient ring's."""
    wl = WL.ffn_stack()
    W0 = WL.init_weights(wl)
    ref = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, n_streams=3)
    net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, n_streams=1, retimed_update=True)
    ref.set_weights(W0)
    net.set_weights(W0)
    del W0
    pool, steps = 3, 36
    xs = [ref.to_device(WL.batch_input(wl, n)) for n in range(1, pool + 1)]
    ts = [ref.to_device(WL.batch_target(wl, n)) for n in range(1, pool + 1)]
    la = torch.zeros(steps, dtype=torch.float32, device="cuda:0")
    lb = torch.zeros(steps, dtype=torch.float32, device="cuda:0")
    torch.cuda.synchronize()
    assert all(net.tensor(l, lp.LP_T_G_LAST) is None for l in range(1, wl.L + 1))
    for n in range(steps):
        lp.lp_step(ref.ctx, xs[n % pool], ts[n % pool], None, la[n:n + 1], ref.streams)
        lp.lp_step(net.ctx, xs[n % pool], ts[n % pool], None, lb[n:n + 1], net.streams)
        if n + 1 in (1, 17, steps):
            lp.lp_sync(ref.ctx)
            lp.lp_sync(net.ctx)
            for l in range(1, wl.L + 1):
                a, b = ref.tensor(l, lp.LP_T_WORK_W), net.tensor(l, lp.LP_T_WORK_W)
                assert torch.equal(a.view(torch.int16), b.view(torch.int16)), "working W_%d after step %d" % (l, n + 1)
            print("ffn_stack full size, retimed against gradient ring: step %d of %d" % (n + 1, steps), flush=True)
    lp.lp_sync(ref.ctx)
    lp.lp_sync(net.ctx)
    losses = la.cpu().numpy()
    assert np.all(np.isfinite(losses)) and len(set(losses.tolist())) > steps // 2
    assert np.array_equal(losses.view(np.uint32), lb.cpu().numpy().view(np.uint32))
    assert torch.equal(ref.tensor(wl.L, lp.LP_T_MASTER_W).view(torch.int32), net.tensor(wl.L, lp.LP_T_MASTER_W).view(torch.int32))
    # a layer with d > 0: the retimed master weights are ahead of the gradient ring's by the gradients still in the ring
    assert not torch.equal(ref.tensor(1, lp.LP_T_MASTER_W).view(torch.int32), net.tensor(1, lp.LP_T_MASTER_W).view(torch.int32))
    ref.close()
    net.close()


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", ["mlp_4096_bf16", "mlp_imbalanced_bf16", "vgg_small_bf16"])
def test_full_size_retimed_update_equals_gradient_ring_bit_for_bit(name):
    """The mid-size workloads at their full sizes in the form bench.py times by default (retimed update on every
    layer that qualifies, three streams) against the gradient-ring form, step by step past the largest delay:
    losses and working weights of every layer after every step, and the master weights of the retimed layers
    against the gradient-ring run continued for d_l more steps, bit for bit."""
    from test_gpu_retimed_update import lockstep
    wl = WL.CONFIGS[name]()
    W0 = WL.init_weights(wl)
    lockstep(wl, W0, max(wl.delays) + 4, {}, dict(retimed_update=True), None)
