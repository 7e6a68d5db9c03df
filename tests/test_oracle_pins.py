"""Pins of the CPU oracle against things other than itself: finite differences, an independent
autograd library (torch, CPU, float64), brute-force scalar loops, closed forms and the delay
counts the paper states.  None of these tests needs a GPU."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import layerpipe_oracle as O
import lp_workloads as WL

HERE = os.path.dirname(os.path.abspath(__file__))
torch.set_num_threads(4)


# ------------------------------------------------------------------------------------------------
# helpers: an independent implementation of the same networks on torch autograd
# ------------------------------------------------------------------------------------------------
def torch_forward_loss(layers, Ws, x, target, loss):
    a = torch.as_tensor(x, dtype=torch.float64)
    for ly, w in zip(layers, Ws):
        if ly.kind == WL.LINEAR:
            if a.dim() == 4:
                a = a.reshape(a.shape[0], -1)
            z = a @ w
        else:
            # NHWC / [kh,kw,ci,co]  ->  torch's NCHW / [co,ci,kh,kw]
            z = torch.nn.functional.conv2d(a.permute(0, 3, 1, 2), w.permute(3, 2, 0, 1), padding=1).permute(0, 2, 3, 1)
        if ly.act == WL.RELU:
            a = torch.relu(z)
        elif ly.act == WL.GELU:
            a = torch.nn.functional.gelu(z)
        elif ly.act == "tanh":
            a = torch.tanh(z)
        elif ly.act == "sigmoid":
            a = torch.sigmoid(z)
        else:
            a = z
        if ly.pool == 2:
            a = torch.nn.functional.max_pool2d(a.permute(0, 3, 1, 2), 2).permute(0, 2, 3, 1)
    z = a.reshape(a.shape[0], -1)
    if loss == WL.SOFTMAX_CE:
        return torch.nn.functional.cross_entropy(z, torch.as_tensor(target, dtype=torch.long))
    return torch.nn.functional.mse_loss(z, torch.as_tensor(target, dtype=torch.float64).reshape(z.shape))


def torch_grads(layers, W_np, x, target, loss):
    Ws = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in W_np]
    E = torch_forward_loss(layers, Ws, x, target, loss)
    E.backward()
    return float(E), [w.grad.numpy().copy() for w in Ws]


def tiny_mlp(act, widths=(5, 4, 3), batch=2, loss=WL.SOFTMAX_CE):
    L = len(widths) - 1
    layers = tuple(WL.Layer(WL.LINEAR, widths[i], widths[i + 1], act if i < L - 1 else WL.IDENTITY) for i in range(L))
    return WL.Workload("tiny", layers, batch, "f32", loss, 0.05, 6, 11, 12, tuple(WL.delays_for(L)))


def tiny_cnn(batch=2):
    layers = (WL.Layer(WL.CONV3X3, 2, 3, WL.RELU, H=4, W=4, pool=0),
              WL.Layer(WL.CONV3X3, 3, 4, WL.RELU, H=4, W=4, pool=2),
              WL.Layer(WL.LINEAR, 2 * 2 * 4, 3, WL.IDENTITY))
    return WL.Workload("tinycnn", layers, batch, "f32", WL.SOFTMAX_CE, 0.05, 6, 21, 22, tuple(WL.delays_for(3)))


def loss_only(wl, W, x, t):
    tr = O.DelayedGradientTrainer(wl.layers, W, [10 ** 6] * wl.L, 0.0, wl.loss, "f64")
    return tr.step(x, t)


# ------------------------------------------------------------------------------------------------
# Eq. 1-5: central finite differences of the loss, every weight of every layer
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("act,loss", [("relu", WL.SOFTMAX_CE), ("gelu", WL.MSE), ("tanh", WL.SOFTMAX_CE), ("sigmoid", WL.MSE)])
def test_gradients_match_finite_differences_mlp(act, loss):
    wl = tiny_mlp(act, loss=loss)
    W = [w.astype(np.float64) for w in WL.init_weights(wl)]
    x, t = WL.batch_input(wl, 1).astype(np.float64), WL.batch_target(wl, 1)
    tr = O.DelayedGradientTrainer(wl.layers, W, [9] * wl.L, 0.1, wl.loss, "f64")
    tr.step(x, t)
    h = 1e-6
    for l in range(wl.L):
        num = np.zeros_like(W[l])
        for i in np.ndindex(W[l].shape):
            Wp = [w.copy() for w in W]; Wp[l][i] += h
            Wm = [w.copy() for w in W]; Wm[l][i] -= h
            num[i] = (loss_only(wl, Wp, x, t) - loss_only(wl, Wm, x, t)) / (2 * h)
        assert np.max(np.abs(num - tr.trace["G"][l])) <= 1e-6 * max(1.0, np.max(np.abs(num))), (act, l)


def test_gradients_match_finite_differences_cnn():
    wl = tiny_cnn()
    W = [w.astype(np.float64) for w in WL.init_weights(wl)]
    x, t = WL.batch_input(wl, 1).astype(np.float64), WL.batch_target(wl, 1)
    tr = O.DelayedGradientTrainer(wl.layers, W, [9] * wl.L, 0.1, wl.loss, "f64")
    tr.step(x, t)
    h = 1e-6
    for l in range(wl.L):
        num = np.zeros_like(W[l])
        for i in np.ndindex(W[l].shape):
            Wp = [w.copy() for w in W]; Wp[l][i] += h
            Wm = [w.copy() for w in W]; Wm[l][i] -= h
            num[i] = (loss_only(wl, Wp, x, t) - loss_only(wl, Wm, x, t)) / (2 * h)
        assert np.max(np.abs(num - tr.trace["G"][l])) <= 2e-6 * max(1.0, np.max(np.abs(num))), l


# ------------------------------------------------------------------------------------------------
# the whole step at zero delay is ordinary back-propagation + SGD (independent library)
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("mk", [lambda: tiny_mlp("relu", (7, 6, 5, 4), 3), lambda: tiny_mlp("gelu", (6, 8, 5), 4, WL.MSE), tiny_cnn])
def test_zero_delay_equals_standard_backprop(mk):
    wl = mk()
    W0 = [w.astype(np.float64) for w in WL.init_weights(wl)]
    tr = O.DelayedGradientTrainer(wl.layers, W0, [0] * wl.L, wl.lr, wl.loss, "f64")
    W = [w.copy() for w in W0]
    for n in range(1, 5):
        x, t = WL.batch_input(wl, n).astype(np.float64), WL.batch_target(wl, n)
        E, g = torch_grads(wl.layers, W, x, t, wl.loss)
        W = [w - wl.lr * gi for w, gi in zip(W, g)]
        assert abs(tr.step(x, t) - E) < 1e-12
        for l in range(wl.L):
            np.testing.assert_allclose(tr.trace["G"][l], g[l], rtol=1e-10, atol=1e-13)
            np.testing.assert_allclose(tr.W[l], W[l], rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------------------------------------
# Eq. 6 with per-layer delays: brute-force replay that keeps every past weight version and asks
# the autograd library for G(k) at W(k-1)
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("mk,delays", [(lambda: tiny_mlp("relu", (7, 6, 5, 4), 3), None), (tiny_cnn, None),
                                       (lambda: tiny_mlp("relu", (7, 6, 5, 4), 3), (1, 5, 0))])
def test_delayed_schedule_equals_bruteforce_replay(mk, delays):
    wl = mk()
    d = list(wl.delays if delays is None else delays)
    W0 = [w.astype(np.float64) for w in WL.init_weights(wl)]
    tr = O.DelayedGradientTrainer(wl.layers, W0, d, wl.lr, wl.loss, "f64")
    Whist = [[w.copy() for w in W0]]          # Whist[n] = weights after step n
    Ghist = [None]                            # Ghist[k] = gradients of minibatch k at W(k-1)
    T = 9
    for n in range(1, T + 1):
        x, t = WL.batch_input(wl, n).astype(np.float64), WL.batch_target(wl, n)
        _, g = torch_grads(wl.layers, Whist[n - 1], x, t, wl.loss)
        Ghist.append(g)
        Whist.append([Whist[n - 1][l] - (wl.lr * Ghist[n - d[l]][l] if n - d[l] >= 1 else 0.0) for l in range(wl.L)])
        tr.step(x, t)
        for l in range(wl.L):
            np.testing.assert_allclose(tr.W[l], Whist[n][l], rtol=1e-11, atol=1e-14)
    # a delay vector that is not all-zero must actually change the trajectory
    if any(d):
        tr0 = O.DelayedGradientTrainer(wl.layers, W0, [0] * wl.L, wl.lr, wl.loss, "f64")
        for n in range(1, T + 1):
            tr0.step(WL.batch_input(wl, n).astype(np.float64), WL.batch_target(wl, n))
        assert any(np.max(np.abs(tr0.W[l] - tr.W[l])) > 1e-8 for l in range(wl.L))


@pytest.mark.parametrize("storage", ["f64", "bf16"])
@pytest.mark.parametrize("delays", [(4, 2, 0), (1, 5, 0), (3, 0, 1)])
def test_delays_on_the_gradient_equal_delays_on_the_weights(storage, delays):
    """Retiming the update of Eq. 6 (Sec. III-A: delays may be moved from the inputs of a node to its outputs): with
    U_l(m) = U_l(m-1) - eta G_l(m), U_l(0) = W_l(0) -- every gradient applied the moment it exists -- the weights that
    step n of Eq. 6 reads are W_l(n-1) = U_l(n-1-d_l) (U_l(0) while n-1-d_l <= 0), exactly: the same numbers are
    subtracted from the same accumulator in the same order, with the same roundings of the stored master.  This is
    the identity behind the library's retimed update; it is checked here on the oracle's own trajectory."""
    wl = tiny_mlp("relu", (7, 6, 5, 4), 3)
    W0 = [w.astype(np.float64) for w in WL.init_weights(wl)]
    tr = O.DelayedGradientTrainer(wl.layers, W0, delays, wl.lr, wl.loss, storage)
    master = "f64" if storage == "f64" else "f32"
    U = [[O.store(w, master)] for w in W0]       # U[l][m]
    T = 12
    for n in range(1, T + 1):
        x, t = WL.batch_input(wl, n).astype(np.float64), WL.batch_target(wl, n)
        tr.step(x, t)
        for l in range(wl.L):
            v = max(0, n - 1 - delays[l])
            assert np.array_equal(tr.trace["Wk"][l], O.store(U[l][v], storage)), (n, l)
            U[l].append(O.store(O.delayed_sgd(U[l][n - 1], tr.trace["G"][l], tr.eta), master))
    # after T steps Eq. 6 has applied G(1..T-d_l): its master weights are U_l(T-d_l), d_l gradients behind U_l(T)
    for l in range(wl.L):
        assert np.array_equal(tr.W[l], U[l][T - delays[l]])
        if delays[l] > 0:
            assert not np.array_equal(tr.W[l], U[l][T])


def test_update_counts_closed_form_and_frozen_prefix():
    """W_l(T) = W_l(0) - eta * sum_{k=1}^{T-d_l} G_l(k); W_l(n) is bit-identical to W_l(0) for n <= d_l."""
    wl = WL.mlp_small().with_(layers=WL._mlp([20, 12, 9, 7, 5], WL.RELU), batch=4)
    assert wl.delays == (6, 4, 2, 0)
    W0 = WL.init_weights(wl)
    tr = O.DelayedGradientTrainer(wl.layers, W0, wl.delays, wl.lr, wl.loss, "f64")
    Gs = []
    for n in range(1, 9):
        tr.step(WL.batch_input(wl, n), WL.batch_target(wl, n))
        Gs.append([g.copy() for g in tr.trace["G"]])
        for l, d in enumerate(wl.delays):
            if n <= d:
                assert np.array_equal(tr.W[l], W0[l].astype(np.float64))
    for l, d in enumerate(wl.delays):
        n_upd = max(0, 8 - d)
        assert n_upd == (2, 4, 6, 8)[l]
        expect = W0[l].astype(np.float64) - wl.lr * sum(Gs[k][l] for k in range(n_upd))
        np.testing.assert_allclose(tr.W[l], expect, rtol=1e-12, atol=1e-15)


def test_gradients_independent_of_delays_until_first_update():
    wl = tiny_mlp("relu", (7, 6, 5, 4), 3)
    W0 = WL.init_weights(wl)
    big = O.DelayedGradientTrainer(wl.layers, W0, [100] * wl.L, wl.lr, wl.loss, "f64")
    some = O.DelayedGradientTrainer(wl.layers, W0, [3, 1, 0], wl.lr, wl.loss, "f64")
    for n in range(1, 4):
        x, t = WL.batch_input(wl, n), WL.batch_target(wl, n)
        big.step(x, t); some.step(x, t)
        _, g = torch_grads(wl.layers, [w.astype(np.float64) for w in W0], x.astype(np.float64), t, wl.loss)
        for l in range(wl.L):          # all delays >= T: every G(n) is the plain gradient at W(0)
            np.testing.assert_allclose(big.trace["G"][l], g[l], rtol=1e-10, atol=1e-13)
        if n == 1:                     # G(1) does not depend on the delay vector
            for l in range(wl.L):
                assert np.array_equal(big.trace["G"][l], some.trace["G"][l])


@pytest.mark.parametrize("M", [0, 1, 3, 7])
def test_scalar_dlms_recurrence(M):
    """One weight, x = 1, MSE against d:  w(n) = w(n-1) - eta * 2 (w(n-1-M) - d), brute force."""
    eta, d, w0, T = 0.1, 0.7, -0.3, 25
    layers = (WL.Layer(WL.LINEAR, 1, 1, WL.IDENTITY),)
    tr = O.DelayedGradientTrainer(layers, [np.array([[w0]])], [M], eta, WL.MSE, "f64")
    w = [w0]                       # w[n]
    for n in range(1, T + 1):
        src = n - M                # gradient of sample src was taken at w[src-1]
        w.append(w[n - 1] - (eta * 2.0 * (w[src - 1] - d) if src >= 1 else 0.0))
        tr.step(np.array([[1.0]]), np.array([[d]]))
        assert abs(tr.W[0][0, 0] - w[n]) < 1e-14
    if M == 0:                     # closed form of the undelayed recurrence
        assert abs(w[T] - (d + (w0 - d) * (1 - 2 * eta) ** T)) < 1e-13


# ------------------------------------------------------------------------------------------------
# inter-layer split: moving the Hadamard (and a column range of the product) changes no numbers
# ------------------------------------------------------------------------------------------------
def test_split_equals_unsplit_delta():
    wl = tiny_mlp("relu", (9, 8, 7, 6, 5), 4)
    W0 = WL.init_weights(wl)
    a = O.DelayedGradientTrainer(wl.layers, W0, wl.delays, wl.lr, wl.loss, "f64", split=True)
    b = O.DelayedGradientTrainer(wl.layers, W0, wl.delays, wl.lr, wl.loss, "f64", split=False)
    for n in range(1, 6):
        x, t = WL.batch_input(wl, n), WL.batch_target(wl, n)
        a.step(x, t); b.step(x, t)
        for l in range(wl.L):
            np.testing.assert_allclose(a.trace["dY"][l], b.trace["dY"][l], rtol=1e-13, atol=1e-16)
            np.testing.assert_allclose(a.W[l], b.W[l], rtol=1e-13, atol=1e-16)


def test_delta_column_partition_concatenates_to_whole():
    rng = np.random.default_rng(5)
    dy, w = rng.standard_normal((6, 7)), rng.standard_normal((9, 7))
    whole = O.grad_act(dy, w)
    parts = np.concatenate([O.grad_act(dy, w, 0, 6), O.grad_act(dy, w, 6, 9)], axis=1)   # delta' | delta''
    assert np.array_equal(whole, parts)
    dyc, wc = rng.standard_normal((2, 4, 4, 5)), rng.standard_normal((3, 3, 6, 5))
    wholec = O.grad_act(dyc, wc)
    partsc = np.concatenate([O.grad_act(dyc, wc, 0, 4), O.grad_act(dyc, wc, 4, 6)], axis=3)
    np.testing.assert_allclose(wholec, partsc, rtol=0, atol=1e-15)


# ------------------------------------------------------------------------------------------------
# single operators against definitions / library routines
# ------------------------------------------------------------------------------------------------
def test_products_against_scalar_loops():
    rng = np.random.default_rng(1)
    a, w, dy = rng.standard_normal((3, 4)), rng.standard_normal((4, 5)), rng.standard_normal((3, 5))
    z, da, g = O.forward_product(a, w), O.grad_act(dy, w), O.grad_weight(a, dy)
    for b in range(3):
        for j in range(5):
            assert abs(z[b, j] - sum(a[b, k] * w[k, j] for k in range(4))) < 1e-13
        for k in range(4):
            assert abs(da[b, k] - sum(dy[b, j] * w[k, j] for j in range(5))) < 1e-13
    for k in range(4):
        for j in range(5):
            assert abs(g[k, j] - sum(a[b, k] * dy[b, j] for b in range(3))) < 1e-13
    assert z.shape == (3, 5) and da.shape == (3, 4) and g.shape == (4, 5)


def test_conv_against_scalar_loops_and_library():
    rng = np.random.default_rng(2)
    B, H, W, C, Oc = 2, 3, 4, 2, 3
    x, w, dy = rng.standard_normal((B, H, W, C)), rng.standard_normal((3, 3, C, Oc)), rng.standard_normal((B, H, W, Oc))
    z = O.conv3x3(x, w)
    zl = np.zeros_like(z)
    for b in range(B):
        for y in range(H):
            for xx in range(W):
                for o in range(Oc):
                    s = 0.0
                    for kh in range(3):
                        for kw in range(3):
                            yy, xq = y + kh - 1, xx + kw - 1
                            if 0 <= yy < H and 0 <= xq < W:
                                for c in range(C):
                                    s += x[b, yy, xq, c] * w[kh, kw, c, o]
                    zl[b, y, xx, o] = s
    np.testing.assert_allclose(z, zl, rtol=0, atol=1e-13)
    xt = torch.tensor(x, requires_grad=True); wt = torch.tensor(w, requires_grad=True)
    zt = torch.nn.functional.conv2d(xt.permute(0, 3, 1, 2), wt.permute(3, 2, 0, 1), padding=1).permute(0, 2, 3, 1)
    np.testing.assert_allclose(z, zt.detach().numpy(), rtol=0, atol=1e-13)
    (zt * torch.tensor(dy)).sum().backward()
    np.testing.assert_allclose(O.conv3x3_grad_act(dy, w), xt.grad.numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(O.conv3x3_grad_weight(x, dy), wt.grad.numpy(), rtol=0, atol=1e-13)


def test_maxpool_first_maximum_and_library():
    a = np.zeros((1, 2, 4, 1))
    a[0, :, :, 0] = [[1.0, 1.0, 0.0, 3.0],
                     [1.0, 0.5, 3.0, 3.0]]
    p, idx = O.maxpool2x2(a)
    assert p[0, 0, :, 0].tolist() == [1.0, 3.0]
    assert idx[0, 0, :, 0].tolist() == [0, 1]        # ties -> first in (row, column) order
    da = O.maxpool2x2_backward(np.array([[[[5.0], [7.0]]]]), idx)
    assert da[0, :, :, 0].tolist() == [[5.0, 0.0, 0.0, 7.0], [0.0, 0.0, 0.0, 0.0]]
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 6, 4, 3))
    xt = torch.tensor(x, requires_grad=True)
    pt = torch.nn.functional.max_pool2d(xt.permute(0, 3, 1, 2), 2).permute(0, 2, 3, 1)
    p, idx = O.maxpool2x2(x)
    assert np.array_equal(p, pt.detach().numpy())
    dp = rng.standard_normal(p.shape)
    (pt * torch.tensor(dp)).sum().backward()
    assert np.array_equal(O.maxpool2x2_backward(dp, idx), xt.grad.numpy())


def test_activation_closed_forms():
    z = np.array([-3.0, -1.0, -0.0, 0.0, 0.5, 2.0])
    assert O.activation(z, "relu").tolist() == [0, 0, 0, 0, 0.5, 2.0]
    assert O.activation_derivative(z, "relu").tolist() == [0, 0, 0, 0, 1, 1]     # ReLU'(0) = 0
    for v in (-2.5, -0.3, 0.0, 0.7, 3.1):
        phi = 0.5 * (1 + math.erf(v / math.sqrt(2)))
        assert abs(O.activation(np.array([v]), "gelu")[0] - v * phi) < 1e-15
        pdf = math.exp(-v * v / 2) / math.sqrt(2 * math.pi)
        assert abs(O.activation_derivative(np.array([v]), "gelu")[0] - (phi + v * pdf)) < 1e-15
    zz = np.linspace(-4, 4, 41)
    for act in ("gelu", "tanh", "sigmoid", "identity"):
        h = 1e-6
        num = (O.activation(zz + h, act) - O.activation(zz - h, act)) / (2 * h)
        np.testing.assert_allclose(O.activation_derivative(zz, act), num, rtol=0, atol=1e-9)
    np.testing.assert_allclose(O.activation(zz, "gelu"), torch.nn.functional.gelu(torch.tensor(zz)).numpy(), rtol=0, atol=1e-15)


def test_softmax_ce_and_mse_closed_forms():
    C, B = 7, 5
    loss, dy = O.softmax_ce(np.zeros((B, C)), np.arange(B) % C)
    assert abs(loss - math.log(C)) < 1e-15
    rng = np.random.default_rng(4)
    z, y = rng.standard_normal((B, C)) * 30 + 500.0, rng.integers(0, C, B)      # large logits: needs max-subtraction
    loss, dy = O.softmax_ce(z, y)
    assert np.isfinite(loss) and np.max(np.abs(dy.sum(axis=1))) < 1e-15
    zt = torch.tensor(z, requires_grad=True)
    lt = torch.nn.functional.cross_entropy(zt, torch.tensor(y)); lt.backward()
    assert abs(loss - float(lt)) < 1e-10
    np.testing.assert_allclose(dy, zt.grad.numpy(), rtol=0, atol=1e-14)
    t = rng.standard_normal((B, C))
    loss, dy = O.mse(z, t)
    assert abs(loss - sum((z[b, j] - t[b, j]) ** 2 for b in range(B) for j in range(C)) / (B * C)) < 1e-9
    np.testing.assert_allclose(dy, 2 * (z - t) / (B * C), rtol=1e-15)


def test_bf16_rounding_against_library_and_ties():
    rng = np.random.default_rng(6)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** rng.integers(-20, 20, 20000).astype(np.float32),
                        np.array([0.0, -0.0, 1.0, 65504.0, 3.3895e38, 1e-40, -1e-40], dtype=np.float32)])
    ref = torch.tensor(x).to(torch.bfloat16).to(torch.float64).numpy()
    got = O.round_bf16(x)
    assert np.array_equal(got, ref)
    # exact ties: 1 + 2^-8 is halfway between bf16 neighbours 1 and 1 + 2^-7 -> even mantissa (1.0);
    # 1 + 3*2^-8 is halfway between 1 + 2^-7 and 1 + 2^-6 -> even mantissa (1 + 2^-6)
    assert O.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert O.round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert O.store(np.array([1.0 + 2.0 ** -30]), "f32")[0] == 1.0
    assert O.store(np.array([1.0 + 2.0 ** -30]), "f64")[0] != 1.0


def test_storage_rounding_is_applied_to_stored_tensors_only():
    wl = tiny_mlp("tanh", (16, 12, 8), 4)
    tr = O.DelayedGradientTrainer(wl.layers, WL.init_weights(wl), [0, 0], wl.lr, wl.loss, "bf16")
    tr.step(WL.batch_input(wl, 1), WL.batch_target(wl, 1))
    isb = lambda v: np.array_equal(O.round_bf16(v), v)
    # every tensor the HIP path keeps in bf16: activations, products, both kinds of gradient w.r.t. activations,
    # and the working copy of the weights that F and dX read
    for k in ("A", "Z", "dY", "dA", "Wk"):
        vals = [v for v in tr.trace[k] if v is not None]
        assert vals and all(isb(v) for v in vals), k
    assert not all(isb(g) for g in tr.trace["G"])                 # gradients stay unrounded
    assert all(np.array_equal(w.astype(np.float32).astype(np.float64), w) for w in tr.W)   # fp32 master
    assert not all(isb(w) for w in tr.W)                          # ... which is not the rounded copy
    # the unrounded trainer rounds none of them
    ex = O.DelayedGradientTrainer(wl.layers, WL.init_weights(wl), [0, 0], wl.lr, wl.loss, "f64")
    ex.step(WL.batch_input(wl, 1), WL.batch_target(wl, 1))
    for k in ("Z", "dY", "dA"):
        assert not all(isb(v) for v in ex.trace[k] if v is not None), k


def test_mse_target_is_rounded_to_the_stored_type():
    """A bf16 context stores the regression target in bf16: the error is taken against the rounded target.
    One identity layer with unit weights, so Z = x; targets 1.5 + 2^-8 (an exact tie: rounds to the even
    neighbour 1.5) and 3 - 2^-8 (rounds to 3).  By hand: d = (1 - 1.5, 2 - 3), E = (0.25 + 1) / 2 = 0.625,
    dY = 2 d / 2 = d.  Against the unrounded target E would be 0.62306...: the 3rd digit differs."""
    layers = (WL.Layer(WL.LINEAR, 2, 2, WL.IDENTITY),)
    x = np.array([[1.0, 2.0]])
    t = np.array([[1.5 + 2.0 ** -8, 3.0 - 2.0 ** -8]])
    tr = O.DelayedGradientTrainer(layers, [np.eye(2)], [0], 0.25, WL.MSE, "bf16")
    loss = tr.step(x, t)
    assert loss == 0.625
    assert np.array_equal(tr.trace["dY"][0], [[-0.5, -1.0]])
    unrounded = ((1.0 - t[0, 0]) ** 2 + (2.0 - t[0, 1]) ** 2) / 2
    assert abs(unrounded - 0.623062133789) < 1e-9 and abs(loss - unrounded) > 1e-3
    # G = x^T dY, W(1) = I - 0.25 G
    assert np.array_equal(tr.W[0], np.eye(2) - 0.25 * np.array([[-0.5, -1.0], [-1.0, -2.0]]))
    # an f32 context does not round it
    tr32 = O.DelayedGradientTrainer(layers, [np.eye(2)], [0], 0.25, WL.MSE, "f32")
    assert abs(tr32.step(x, t) - unrounded) < 1e-12


def test_hand_computed_bf16_step_of_a_two_layer_network():
    """One training step worked out by hand on numbers chosen so that every result is exact and every rounding to
    bf16 that the path prescribes changes a digit somewhere.  a = 1 + 2^-8 + 2^-12 is an fp32 number that rounds UP
    to 1 + 2^-7 in bf16.  Batch 1, eta = 1/2, no delay, MSE over 4 outputs (dY = (z - t) / 2).

      master W1 = [[a, 2, 1], [1, 1, 1]]                        working copy: a -> 1 + 2^-7
      x = [1, -1]        z1 = [2^-7, 1, 0]                      (with the unrounded a: 2^-8 + 2^-12)
      ReLU               a1 = [2^-7, 1, 0],  f'(z1) = [1, 1, 0]  (the unit at exactly 0 is off)
      master W2 = [[64, 0, 256 a, 0], [3, a, -2^-6, 0], [5, 7, 1, 0]]     working copy: 256 a -> 258, a -> 1 + 2^-7
      z2 = a1 . W2 = [0.5 + 3, 1 + 2^-7, 258/128 - 1/64, 0] = [3.5, 1 + 2^-7, 2, 0]
      t  = [-0.5 - 2^-10, a, 6, 0]   stored as  [-0.5, 1 + 2^-7, 6, 0]
      d  = z2 - t = [4, 0, -4, 0]     E = (16 + 0 + 16 + 0) / 4 = 8      dY2 = [2, 0, -2, 0]
      G2 = a1^T dY2 = [[2^-6, 0, -2^-6, 0], [2, 0, -2, 0], [0, 0, 0, 0]]
      dA1 = dY2 . W2^T = [128 - 516, 6 + 2^-5, 10 - 2] = [-388, 6.03125, 8]   (master 256 a instead of 258: -386.125)
      dY1 = dA1 (.) f'(z1) = [-388, 6.03125, 0]
      G1 = x^T dY1 = [[-388, 6.03125, 0], [388, -6.03125, 0]]
      W1(1) = W1 - G1 / 2,  W2(1) = W2 - G2 / 2      (on the fp32 masters)
    """
    a = 1.0 + 2.0 ** -8 + 2.0 ** -12
    assert np.float32(a) == a and O.round_bf16(np.array([a]))[0] == 1.0 + 2.0 ** -7 and O.round_bf16(np.array([256 * a]))[0] == 258.0
    layers = (WL.Layer(WL.LINEAR, 2, 3, WL.RELU), WL.Layer(WL.LINEAR, 3, 4, WL.IDENTITY))
    W1 = np.array([[a, 2.0, 1.0], [1.0, 1.0, 1.0]])
    W2 = np.array([[64.0, 0.0, 256 * a, 0.0], [3.0, a, -2.0 ** -6, 0.0], [5.0, 7.0, 1.0, 0.0]])
    x = np.array([[1.0, -1.0]])
    t = np.array([[-0.5 - 2.0 ** -10, a, 6.0, 0.0]])
    for split in (True, False):
        tr = O.DelayedGradientTrainer(layers, [W1, W2], [0, 0], 0.5, WL.MSE, "bf16", split=split)
        assert tr.step(x, t) == 8.0
        assert np.array_equal(tr.trace["Z"][0], [[2.0 ** -7, 1.0, 0.0]])
        assert np.array_equal(tr.trace["Z"][1], [[3.5, 1.0 + 2.0 ** -7, 2.0, 0.0]])
        assert np.array_equal(tr.trace["dY"][1], [[2.0, 0.0, -2.0, 0.0]])
        assert np.array_equal(tr.trace["dY"][0], [[-388.0, 6.03125, 0.0]])
        assert np.array_equal(tr.trace["G"][0], [[-388.0, 6.03125, 0.0], [388.0, -6.03125, 0.0]])
        assert np.array_equal(tr.trace["G"][1], [[2.0 ** -6, 0.0, -2.0 ** -6, 0.0], [2.0, 0.0, -2.0, 0.0], [0.0, 0.0, 0.0, 0.0]])
        assert np.array_equal(tr.W[0], [[a + 194.0, 2.0 - 3.015625, 1.0], [1.0 - 194.0, 1.0 + 3.015625, 1.0]])
        assert np.array_equal(tr.W[1], [[64.0 - 2.0 ** -7, 0.0, 256 * a + 2.0 ** -7, 0.0], [2.0, a, 1.0 - 2.0 ** -6, 0.0], [5.0, 7.0, 1.0, 0.0]])
    assert np.array_equal(tr.trace["dA"][0] if tr.trace["dA"][0] is not None else [[-388.0, 6.03125, 8.0]], [[-388.0, 6.03125, 8.0]])
    # second step: F reads the rounded copy of the UPDATED masters (a + 194 = 195.0041... is stored as 195 in bf16)
    tr = O.DelayedGradientTrainer(layers, [W1, W2], [0, 0], 0.5, WL.MSE, "bf16")
    tr.step(x, t)
    tr.step(np.array([[1.0, 0.0]]), t)
    assert np.array_equal(tr.trace["Wk"][0][0], [195.0, -1.015625, 1.0])
    assert np.array_equal(tr.trace["Z"][0], [[195.0, -1.015625, 1.0]])


# ------------------------------------------------------------------------------------------------
# delay rule: the counts the paper states for its two-layer example
# ------------------------------------------------------------------------------------------------
def test_delay_rule_golden_example():
    rows = [tuple(int(v) for v in ln.split()) for ln in open(os.path.join(HERE, "golden", "delay_rule_example.txt"))
            if ln.strip() and not ln.startswith("#")]
    assert WL.delays_for(len(rows), [r[1] for r in rows]) == [r[2] for r in rows] == [4, 2]
    assert WL.delays_for(4) == [6, 4, 2, 0]
    assert list(WL.mlp_4096().delays) == [14, 12, 10, 8, 6, 4, 2, 0]


def test_workload_shapes():
    f, dx, dw = WL.ffn_stack().flops_per_step()
    assert abs(f - 17592e9) / 17592e9 < 1e-3 and abs(dx - 16493e9) / 16493e9 < 1e-3 and f == dw
    f, dx, dw = WL.mlp_4096().flops_per_step()
    assert abs((f + dx + dw) - 178e9) / 178e9 < 5e-3
    v = WL.vgg_small()
    assert [v.gemm_dims(l) for l in range(v.L)] == [(131072, 64, 27), (131072, 64, 576), (32768, 128, 576), (32768, 128, 1152),
                                                    (8192, 256, 1152), (8192, 256, 2304), (128, 10, 4096)]
    assert WL.mlp_imbalanced().n_params == 135118848 or abs(WL.mlp_imbalanced().n_params - 135.1e6) < 1e5
    assert WL.ffn_stack().n_params == 16 * 4096 * 16384
