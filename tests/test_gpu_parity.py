"""Parity of the HIP path (called through the C-ABI) against the CPU oracle, element by element, on
the same seeded inputs.  Needs a real MI355X.

Tolerances (max |gpu - ref| / max |ref| per tensor): fp32 contexts 1e-4 per step and 1e-3 after 8
steps; bf16 contexts 2e-2.  Integer-like decisions (ReLU mask, pool routing) are compared bit-exactly
given identical inputs; the fp32 gradients of bf16 contexts are held to 2e-4 when the inputs are
identical, since only the summation order differs.
"""
import os

import numpy as np
import pytest
import torch

import lp_workloads as WL
import paper_2108_06629_amd as lp
from oracle import layerpipe_oracle as O

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def relerr(got, ref):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    den = np.max(np.abs(ref))
    return float(np.max(np.abs(got - ref)) / (den if den > 0 else 1.0))


def dev(x, dtype):
    """Host array -> device tensor.  The cast runs on torch's stream, which the library's streams are
    not ordered after: wait for it here so that a kernel enqueued next reads finished data."""
    t = torch.from_numpy(np.ascontiguousarray(x)).to(DEV).to(dtype).contiguous()
    torch.cuda.synchronize()
    return t


def synced(t):
    """A tensor torch has just filled on its own stream, safe to hand to the library: its streams are not ordered after
    torch's, so a fill still in flight could land on top of what a library kernel writes (or be read half done)."""
    torch.cuda.synchronize()
    return t


def host(t):
    return t.to(torch.float32).cpu().numpy().astype(np.float64)


def one_layer_net(d_in, d_out, batch, act="relu", dtype="bf16", seed=0):
    """Context with a single hidden layer of the given shape followed by a tiny output layer."""
    layers = (WL.Layer(WL.LINEAR, d_in, d_out, act), WL.Layer(WL.LINEAR, d_out, 8, WL.IDENTITY))
    net = lp.Network(layers, batch, dtype, WL.SOFTMAX_CE, 0.01, (0, 0))
    rng = np.random.default_rng(seed)
    W = [(rng.standard_normal(l.weight_shape) * np.sqrt(2.0 / l.d_in)).astype(np.float32) for l in layers]
    net.set_weights(W)
    return net, W, rng


# shapes: (batch, d_in, d_out).  Chosen to hit every kernel variant (>=192 tiles of 256x256, else
# 128x128, else 64x64 for unaligned shapes with few tiles; direct-to-LDS loop when every run is a
# multiple of 8, register-staged loop otherwise), ragged tails in all three dimensions, and
# degenerate sizes.
FWD_SHAPES = [(96, 200, 136), (33, 77, 19), (1, 8, 8), (7, 1, 3), (300, 520, 264), (64, 4096, 64),
              (1100, 72, 3000), (2304, 96, 5632), (256, 512, 1000), (1024, 136, 6200), (2300, 100, 5700),
              (1101, 71, 3001), (256, 2048, 512), (300, 2056, 1160), (200, 1160, 3080),
              (128, 4096, 10), (33, 264, 16), (5, 72, 1), (2048, 512, 13), (2049, 512, 10),
              (256, 4096, 3072), (512, 512, 4096)]
# (128, 4096, 10) ... (2049, 512, 10) are layers with at most 16 outputs: short-vector kernels (gemm_skinny.hip) up to batch 2048,
# MFMA tiles beyond.  The last two are skinny against a wide layer (64 and 128 tiles of 128 x 128): K cut into ranges for F and dX
# of the first, one short pass for the second.
# K is split over workgroups for F of (64, 4096, 64), (256, 2048, 512), (300, 2056, 1160) (ragged last range), for dX of
# (1100, 72, 3000), (200, 1160, 3080) and for dW of (2304, 96, 5632)


@pytest.mark.parametrize("shape", FWD_SHAPES)
@pytest.mark.parametrize("act", ["relu", "gelu"])
def test_forward_product_bf16(shape, act):
    B, K, N = shape
    if act == "gelu" and B * N > 2e6:
        pytest.skip("large shape covered with relu")
    net, W, rng = one_layer_net(K, N, B, act)
    x = rng.standard_normal((B, K)).astype(np.float32)
    xd = dev(x, torch.bfloat16)
    Z = torch.empty(B, N, dtype=torch.bfloat16, device=DEV)
    A = torch.empty(B, N, dtype=torch.bfloat16, device=DEV)
    lp.lp_forward(net.ctx, 1, xd, Z, A, net.streams[0])
    lp.lp_sync(net.ctx)
    ref_z = O.store(O.forward_product(O.round_bf16(x), O.round_bf16(W[0])), "bf16")
    assert relerr(host(Z), ref_z) <= 2e-2
    # A is defined on the stored Z: the ReLU decision must be bit-exact, GELU within a bf16 ulp
    ref_a = O.store(O.activation(host(Z), act), "bf16")
    if act == "relu":
        assert np.array_equal(host(A), ref_a)
    else:
        assert relerr(host(A), ref_a) <= 2.0 ** -7
        assert np.mean(host(A) == ref_a) > 0.98
    # Z only / A only
    A2 = torch.empty_like(A)
    lp.lp_forward(net.ctx, 1, xd, None, A2, net.streams[0])
    lp.lp_sync(net.ctx)
    assert torch.equal(A2, A)
    net.close()


def test_gelu_of_every_bf16_input_is_the_rounded_exact_value():
    """Every finite bf16 pattern as the pre-activation of a GELU layer (identity weights, so Z = X): A must be the
    fp64 GELU of the stored Z rounded to bf16, bit for bit, wherever the oracle's erf form is itself accurate to far
    below half a bf16 ulp (z > -6; beyond that 1 + erf(z / sqrt 2) cancels in fp64 and both sides are below 1e-7 in
    magnitude)."""
    n = 256
    pats = np.arange(65536, dtype=np.uint32)
    x = (pats << 16).astype(np.uint32).view(np.float32).copy()
    x[~np.isfinite(x)] = 0.0
    x = x.reshape(n, n)
    layers = (WL.Layer(WL.LINEAR, n, n, WL.GELU), WL.Layer(WL.LINEAR, n, 8, WL.IDENTITY))
    net = lp.Network(layers, n, "bf16", WL.SOFTMAX_CE, 0.01, (0, 0))
    net.set_weights([np.eye(n, dtype=np.float32), np.zeros((n, 8), dtype=np.float32)])
    xd = dev(x, torch.bfloat16)
    Z = torch.empty(n, n, dtype=torch.bfloat16, device=DEV)
    A = torch.empty(n, n, dtype=torch.bfloat16, device=DEV)
    lp.lp_forward(net.ctx, 1, xd, Z, A, net.streams[0])
    lp.lp_sync(net.ctx)
    z, a = host(Z), host(A)
    normal = np.abs(x) >= 2.0 ** -126
    assert np.array_equal(z[normal], x[normal].astype(np.float64))      # one non-zero term per sum: Z is X
    assert np.unique(z).size > 65000
    ref = O.store(O.activation(z, "gelu"), "bf16")
    accurate = z > -6.0
    assert np.array_equal(a[accurate], ref[accurate])
    assert np.all(np.signbit(a[~accurate]) | (a[~accurate] == 0.0))
    assert np.max(np.abs(a[~accurate] - ref[~accurate])) <= 1e-7
    net.close()


@pytest.mark.parametrize("shape", FWD_SHAPES)
def test_grad_act_and_column_partition_bf16(shape):
    B, K, N = shape          # layer K -> N;  dX = dY[B,N] . W[K,N]^T
    net, W, rng = one_layer_net(K, N, B)
    dy = (rng.standard_normal((B, N)) / np.sqrt(N)).astype(np.float32)
    dyd = dev(dy, torch.bfloat16)
    dX = synced(torch.full((B, K), float("nan"), dtype=torch.bfloat16, device=DEV))
    lp.lp_grad_act(net.ctx, 1, dyd, dX, 0, K, net.streams[0])
    lp.lp_sync(net.ctx)
    ref = O.store(O.grad_act(O.round_bf16(dy), O.round_bf16(W[0])), "bf16")
    assert relerr(host(dX), ref) <= 2e-2
    if K >= 2:
        # delta' | delta'': two independent calls on complementary column ranges, different streams
        cut = max(1, (K * 2) // 3)
        parts = synced(torch.full((B, K), float("nan"), dtype=torch.bfloat16, device=DEV))
        lp.lp_grad_act(net.ctx, 1, dyd, parts, 0, cut, net.streams[0])
        lp.lp_grad_act(net.ctx, 1, dyd, parts, cut, K, net.streams[1])
        lp.lp_sync(net.ctx)
        assert torch.equal(parts.view(torch.int16), dX.view(torch.int16))
        refp = np.concatenate([O.grad_act(O.round_bf16(dy), O.round_bf16(W[0]), 0, cut),
                               O.grad_act(O.round_bf16(dy), O.round_bf16(W[0]), cut, K)], axis=1)
        assert relerr(host(parts), O.store(refp, "bf16")) <= 2e-2
    net.close()


@pytest.mark.parametrize("shape", FWD_SHAPES + [(4096, 264, 520)])
def test_grad_weight_bf16(shape):
    B, K, N = shape
    net, W, rng = one_layer_net(K, N, B)
    x = rng.standard_normal((B, K)).astype(np.float32)
    dy = (rng.standard_normal((B, N)) / B).astype(np.float32)
    G = synced(torch.full((K, N), float("nan"), dtype=torch.float32, device=DEV))
    lp.lp_grad_weight(net.ctx, 1, dev(x, torch.bfloat16), dev(dy, torch.bfloat16), G, net.streams[0])
    lp.lp_sync(net.ctx)
    ref = O.grad_weight(O.round_bf16(x), O.round_bf16(dy))
    assert relerr(host(G), ref) <= 2e-4
    net.close()


# The direct-to-LDS loop refills its ring with per-lane affine offsets while whole K tiles remain and
# with bounds-checked offsets for the last (partial or empty) ones: reduction lengths around one, two,
# three and four K steps of 64, with and without a partial last step, on the 128 x 128 tiles
# (264 x 136 outputs) and on the 256 x 256 tiles (4096 x 4096 outputs).
@pytest.mark.parametrize("red", [8, 64, 72, 128, 136, 192, 200, 264])
@pytest.mark.parametrize("big", [False, True])
def test_reduction_lengths_around_the_k_step(red, big):
    if big and red not in (64, 136, 192, 264):
        pytest.skip("the large outputs take four of the lengths")
    m, n = (4096, 4096) if big else (264, 136)
    rng = np.random.default_rng(red + 1000 * big)
    # F: reduction over the layer's inputs
    net, W, _ = one_layer_net(red, n, m)
    x = rng.standard_normal((m, red)).astype(np.float32)
    Z = torch.empty(m, n, dtype=torch.bfloat16, device=DEV)
    lp.lp_forward(net.ctx, 1, dev(x, torch.bfloat16), Z, None, net.streams[0])
    lp.lp_sync(net.ctx)
    assert relerr(host(Z), O.store(O.forward_product(O.round_bf16(x), O.round_bf16(W[0])), "bf16")) <= 2e-2
    net.close()
    # dX: reduction over the layer's outputs
    net, W, _ = one_layer_net(n, red, m)
    dy = (rng.standard_normal((m, red)) / np.sqrt(red)).astype(np.float32)
    dX = synced(torch.full((m, n), float("nan"), dtype=torch.bfloat16, device=DEV))
    lp.lp_grad_act(net.ctx, 1, dev(dy, torch.bfloat16), dX, 0, n, net.streams[0])
    lp.lp_sync(net.ctx)
    assert relerr(host(dX), O.store(O.grad_act(O.round_bf16(dy), O.round_bf16(W[0])), "bf16")) <= 2e-2
    net.close()
    # dW: reduction over the batch
    net, W, _ = one_layer_net(m, n, red)
    x = rng.standard_normal((red, m)).astype(np.float32)
    dy = (rng.standard_normal((red, n)) / red).astype(np.float32)
    G = synced(torch.full((m, n), float("nan"), dtype=torch.float32, device=DEV))
    lp.lp_grad_weight(net.ctx, 1, dev(x, torch.bfloat16), dev(dy, torch.bfloat16), G, net.streams[0])
    lp.lp_sync(net.ctx)
    assert relerr(host(G), O.grad_weight(O.round_bf16(x), O.round_bf16(dy))) <= 2e-4
    net.close()


@pytest.mark.parametrize("n_feat", [8, 1000, 4099])
@pytest.mark.parametrize("act,dtype", [("relu", "bf16"), ("gelu", "bf16"), ("relu", "f32"), ("gelu", "f32"),
                                       ("tanh", "bf16"), ("sigmoid", "bf16"), ("tanh", "f32"), ("sigmoid", "f32")])
def test_act_grad_hadamard(n_feat, act, dtype):
    B = 37
    net, W, rng = one_layer_net(n_feat, n_feat, B, act, dtype)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    z = rng.standard_normal((B, n_feat)).astype(np.float32)
    z[0, :4] = [0.0, -0.0, 1e-30, -1e-30]
    da = rng.standard_normal((B, n_feat)).astype(np.float32)
    zd, dad = dev(z, td), dev(da, td)
    dY = torch.empty_like(dad)
    lp.lp_act_grad(net.ctx, 1, dad, zd, dY, net.streams[0])
    lp.lp_sync(net.ctx)
    ref = O.store(O.act_grad(host(dad), host(zd), act), "bf16" if dtype == "bf16" else "f32")
    if act == "relu":
        assert np.array_equal(host(dY), ref)              # the mask is a decision: exact
        # the stashed A (same sign as Z) serves as well
        dY2 = torch.empty_like(dad)
        ad = synced(torch.relu(zd))
        lp.lp_act_grad(net.ctx, 1, dad, ad, dY2, net.streams[0])
        lp.lp_sync(net.ctx)
        assert torch.equal(dY2, dY)
    else:
        assert relerr(host(dY), ref) <= (2.0 ** -7 if dtype == "bf16" else 1e-5)
    net.close()


def test_act_grad_hadamard_gelu_large_tensor_matches_small():
    """Tensors of 4 M elements and more take the GELU form that keeps the derivative table's live part in LDS; smaller
    ones gather from the table in memory.  Both must give the same bits, also for pre-activations outside the cached
    range (|z| >= 16, infinities, NaN) and in the scalar tail (element count not a multiple of 8)."""
    n_feat, B, Bs = 4099, 1031, 37
    assert n_feat * B >= 1 << 22 and (n_feat * B) % 8 != 0
    big, _, rng = one_layer_net(n_feat, n_feat, B, "gelu", "bf16")
    small, _, _ = one_layer_net(n_feat, n_feat, Bs, "gelu", "bf16")
    z = (rng.standard_normal((B, n_feat)) * 2.0).astype(np.float32)
    z[0, :10] = [0.0, -0.0, 1e-30, -1e-30, 15.9375, 16.0, -16.0, 300.0, -300.0, 3e38]
    z[1, :4] = [np.inf, -np.inf, np.nan, -15.9375]
    z[-1, -5:] = [17.0, -17.0, 0.5, -0.5, 4.0]            # the last five elements are the scalar tail
    da = rng.standard_normal((B, n_feat)).astype(np.float32)
    zd, dad = dev(z, torch.bfloat16), dev(da, torch.bfloat16)
    dY = synced(torch.full_like(dad, float("nan")))
    lp.lp_act_grad(big.ctx, 1, dad, zd, dY, big.streams[0])
    lp.lp_sync(big.ctx)
    for r0 in (0, B - Bs):                                 # head and tail rows through the small-tensor form
        zs, das = synced(zd[r0:r0 + Bs].clone()), synced(dad[r0:r0 + Bs].clone())
        dYs = torch.empty_like(das)
        lp.lp_act_grad(small.ctx, 1, das, zs, dYs, small.streams[0])
        lp.lp_sync(small.ctx)
        a, b = dY[r0:r0 + Bs].view(torch.int16), dYs.view(torch.int16)
        assert torch.equal(a, b)
    fin = np.isfinite(host(zd))
    ref = O.store(O.act_grad(host(dad)[fin], host(zd)[fin], "gelu"), "bf16")
    assert relerr(host(dY)[fin], ref) <= 2.0 ** -7
    big.close()
    small.close()


# row lengths: not a multiple of the 16-byte vector (scalar kernel), one / two / four / eight vectors per lane of the
# register-resident kernel, and a row too long for it
@pytest.mark.parametrize("rows,cols", [(32, 10), (256, 1000), (5, 33), (1, 1), (1024, 1000), (9, 8), (7, 2048), (6, 4096), (3, 4104), (2, 8192)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_softmax_ce(rows, cols, dtype):
    layers = (WL.Layer(WL.LINEAR, 16, cols, WL.IDENTITY),)
    net = lp.Network(layers, rows, dtype, WL.SOFTMAX_CE, 0.01, (0,))
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    rng = np.random.default_rng(rows * 7 + cols)
    z = (rng.standard_normal((rows, cols)) * 3 + 40.0).astype(np.float32)
    y = rng.integers(0, cols, rows).astype(np.int32)
    zd = dev(z, td)
    dY = torch.empty_like(zd)
    loss = synced(torch.zeros(1, dtype=torch.float32, device=DEV))
    lp.lp_loss_grad(net.ctx, zd, dev(y, torch.int32), dY, loss, net.streams[0])
    lp.lp_sync(net.ctx)
    ref_loss, ref_dy = O.softmax_ce(host(zd), y)
    tol = 2e-2 if dtype == "bf16" else 1e-4
    assert abs(float(loss) - ref_loss) <= (1e-5 * max(1.0, abs(ref_loss)))
    assert relerr(host(dY), O.store(ref_dy, "bf16" if dtype == "bf16" else "f32")) <= tol
    if dtype == "f32":
        assert np.max(np.abs(host(dY).sum(axis=1))) < 1e-6
    net.close()


# sizes: several blocks of 8192 elements, fewer elements than one vector, a ragged tail behind whole vectors
@pytest.mark.parametrize("rows,cols", [(64, 256), (3, 7), (512, 4096), (1, 3), (5, 1643), (33, 8193)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_mse(rows, cols, dtype):
    layers = (WL.Layer(WL.LINEAR, 16, cols, WL.IDENTITY),)
    net = lp.Network(layers, rows, dtype, WL.MSE, 0.01, (0,))
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    rng = np.random.default_rng(rows + cols)
    zd, tg = dev(rng.standard_normal((rows, cols)).astype(np.float32), td), dev(rng.standard_normal((rows, cols)).astype(np.float32), td)
    dY = torch.empty_like(zd)
    loss = synced(torch.zeros(1, dtype=torch.float32, device=DEV))
    lp.lp_loss_grad(net.ctx, zd, tg, dY, loss, net.streams[0])
    lp.lp_sync(net.ctx)
    ref_loss, ref_dy = O.mse(host(zd), host(tg))
    assert abs(float(loss) - ref_loss) <= 1e-5 * ref_loss
    assert relerr(host(dY), O.store(ref_dy, "bf16" if dtype == "bf16" else "f32")) <= (2.0 ** -7 if dtype == "bf16" else 1e-6)
    net.close()


@pytest.mark.parametrize("n", [1, 3, 4, 1000, 4099, 1 << 20])
def test_cast_rounds_to_nearest_even_like_the_oracle(n):
    """lp_cast is how a float input becomes an act-type tensor: bit for bit the oracle's storage rounding, including exact
    ties (both directions), values below the smallest normal and infinities; an F32 context copies."""
    layers = (WL.Layer(WL.LINEAR, 8, 8, WL.IDENTITY),)
    rng = np.random.default_rng(n)
    x = (rng.standard_normal(n) * np.exp(rng.uniform(-30, 30, n))).astype(np.float32)
    special = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 2.0 ** -130, -2.0 ** -140, 0.0, -0.0, np.inf, -np.inf,
                        3.3895314e38, 1.0 + 2.0 ** -9, 1.0 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    x[:min(n, special.size)] = special[:min(n, special.size)]
    net = lp.Network(layers, 4, "bf16", WL.MSE, 0.01, (0,))
    src = torch.from_numpy(x).to(DEV)
    dst = synced(torch.full((n,), float("nan"), dtype=torch.bfloat16, device=DEV))
    torch.cuda.synchronize()
    lp.lp_cast(net.ctx, src, dst, n, net.streams[0])
    lp.lp_sync(net.ctx)
    got = dst.view(torch.int16).cpu().numpy().view(np.uint16)
    want = (O.round_bf16(x).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    assert np.array_equal(got, want)
    assert torch.equal(net.to_device(x.reshape(1, -1)).view(torch.int16).cpu().view(-1), dst.view(torch.int16).cpu())
    net.close()
    net = lp.Network(layers, 4, "f32", WL.MSE, 0.01, (0,))
    out = synced(torch.zeros(n, dtype=torch.float32, device=DEV))
    lp.lp_cast(net.ctx, src, out, n, net.streams[0])
    lp.lp_sync(net.ctx)
    assert torch.equal(out.view(torch.int32), src.view(torch.int32))
    net.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("shape", [(8, 8), (1000, 257), (3, 5)])
def test_delayed_sgd_update(dtype, shape):
    K, N = shape
    net, W, rng = one_layer_net(K, N, 4, "relu", dtype)
    g = rng.standard_normal((K, N)).astype(np.float32)
    gd = dev(g, torch.float32)
    lp.lp_update(net.ctx, 1, gd, net.streams[0])
    lp.lp_sync(net.ctx)
    got = net.get_weights(1)
    ref = O.store(O.delayed_sgd(W[0].astype(np.float64), g.astype(np.float64), float(np.float32(0.01))), "f32")
    assert np.max(np.abs(got - ref)) <= 2.0 ** -23 * np.max(np.abs(ref))
    assert np.mean(got == ref) > 0.999
    if dtype == "bf16":   # the new working copy is the rounded master, bit for bit
        work = host(net.tensor(1, lp.LP_T_WORK_W)).reshape(K, N)
        assert np.array_equal(work, O.round_bf16(got))
    net.close()


# ------------------------------------------------------------------------------------------------
# whole training runs: the delayed-gradient schedule, every G_l and W_l(n) of every step
# ------------------------------------------------------------------------------------------------
def frob(got, ref):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


# Free-running comparison of bf16 runs with the oracle's trajectory.  The GPU (fp32 accumulation) and the oracle
# (float64 accumulation) differ in summation order only, which moves the last bf16 bit of a small fraction of the
# stored elements; a ReLU (or pool arg-max) decided on such an element may legitimately flip (measured: up to 3e-3 of
# the units of a deep layer), a flipped unit changes delta of that sample by a whole term, and every layer below it
# inherits the change: in the 7- to 12-layer ReLU networks single entries of G_l end up several per cent of the
# largest entry away from the oracle's, from step 1 on (identical weights).  Networks without such decisions (GELU,
# tanh, sigmoid, or shallow) stay below 1e-2.  So: loss, W_l and Z_L are held to the stated 2e-2 (one listed
# exception for Z_L), and every G_l to max |G_gpu - G_ref| / max |G_ref| <= 2e-2 unless the run is listed here with
# the bound measured for it (about twice the worst value seen over all layers and steps; the measured values, with
# the flip counts, are tabulated in the design notes).  The bound that does not compound is the task-by-task check
# on identical inputs (check_tasks_of_last_step): there every G_l is within 2e-4 of the oracle operator applied to
# the GPU's own tensors, at every step of every run.
G_MAXNORM_BOUND = {                                           # worst measured
    "mlp_4096_bf16_batch256_params121536512": 0.4,            # 0.185  (8 ReLU layers of 4096, 17 steps)
    "mlp_4096_bf16_batch64_params2347008": 0.3,               # 0.145  (its 512-wide replica, 18 steps)
    "mlp_4096_bf16_batch64_params1560576": 0.2,               # 0.073  (5 layers of 512)
    "mlp_imbalanced_bf16_batch1024_params135069696": 0.2,     # 0.084  (12 layers, 10 steps)
    "mlp_imbalanced_bf16_batch128_params2110464": 0.2,        # 0.077  (its 1/8-width replica)
    "vgg_small_bf16_batch128_params1185472": 0.5,             # 0.227  (6 conv + pool + FC, 20 steps)
    "vgg_small_bf16_batch8_params1185472": 0.08,              # 0.028  (the same network on 8 samples, 3 steps)
}
ZL_BOUND = {"vgg_small_bf16_batch128_params1185472": 0.05}    # 0.0218 at step 20 (the logits of a 7-layer bf16 network)

RECORDS = {}     # run key -> list of dict(n, l, g_maxnorm, g_share_over, relu_flips, relu_units, ...): what the last run measured
RECORDING = bool(os.environ.get("LP_RECORD_DIR"))   # a recording run measures the free-running figures without asserting them


def run_key(wl):
    """Names a run by its workload, batch and parameter count (scaled replicas keep the workload's name)."""
    return "%s_batch%d_params%d" % (wl.name, wl.batch, wl.n_params)


def _bound(table, wl, l, default):
    b = table.get(run_key(wl), default)
    return b.get(l, default) if isinstance(b, dict) else b


def _dump_records(name):
    """With LP_RECORD_DIR set, the per-layer per-step figures of a run are written there as JSON."""
    import json
    d = os.environ.get("LP_RECORD_DIR")
    if d and RECORDS.get(name):
        os.makedirs(d, exist_ok=True)
        with open(os.path.join(d, "free_running_%s.json" % name), "w") as f:
            json.dump(RECORDS[name], f)


def check_g_free_running(wl, l, n, g, g_ref, g_exact=None):
    """Every free-running G_l element-wise: max-norm relative to the largest entry of the oracle's G_l, and the share
    of entries beyond the stated 2e-2; the Frobenius comparison against the bf16 oracle's own distance from the
    float64 oracle is kept beside it where that oracle runs.  Returns (max-norm error, share beyond 2e-2)."""
    bf = wl.dtype == "bf16"
    g, g_ref = np.asarray(g, dtype=np.float64), np.asarray(g_ref, dtype=np.float64)
    den = np.max(np.abs(g_ref))
    den = den if den > 0 else 1.0
    err = np.abs(g - g_ref) / den
    e, share = float(err.max()), float(np.mean(err > 2e-2))
    if not bf:
        assert e <= (1e-3 if n >= 8 else 1e-4), ("G", l, n, e)
        return e, share
    if not RECORDING:
        assert e <= _bound(G_MAXNORM_BOUND, wl, l, 2e-2), ("G max-norm", run_key(wl), l, n, e)
        if g_exact is not None:
            floor = frob(g_ref, g_exact)
            ef = frob(g, g_ref)
            assert ef <= max(2e-2, floor), ("G Frobenius", l, n, ef, floor)
    return e, share


def relu_flips(net, wl, l, z_ref):
    """Number of units of ReLU layer l whose on/off decision differs between the GPU and the oracle trajectory."""
    ly = wl.layers[l - 1]
    if ly.act != "relu" or l == wl.L:
        return 0, 0
    z_gpu = net.tensor_np(l, lp.LP_T_Z)
    if z_gpu is None:                     # a ReLU layer without pool keeps A only: same sign as Z
        z_gpu = net.tensor_np(l, lp.LP_T_A)
    z_gpu = z_gpu.reshape(z_ref.shape)
    return int(np.count_nonzero((z_gpu > 0) != (z_ref > 0))), int(z_ref.size)


def check_tasks_of_last_step(net, wl, x, target, W_before, G_hist, n, products=True):
    """Task-by-task check of the step that just ran: every task's output is compared with the oracle
    operator applied to the inputs that task actually read on the GPU.  With identical inputs the
    discrete decisions (ReLU mask) are identical too, so the bound is the arithmetic one, and the
    delayed update is checked against the GPU's own gradient of d_l steps ago (the ring).
    products=False skips the recomputation of the three products and of the loss (the long runs at the
    benchmark's sizes do them on some steps only); the Hadamard, the update from the ring, the frozen
    prefix and the working copy are checked in every step."""
    bf = wl.dtype == "bf16"
    st = "bf16" if bf else "f32"
    tol = 2e-2 if bf else 1e-4
    tolG = 2e-4 if bf else 1e-4
    L = wl.L
    Wk = [O.store(w, st) for w in W_before]
    A = [O.store(x, st)] + [net.tensor_np(l, lp.LP_T_A) for l in range(1, L)]
    A = [a if a is None else a.reshape(wl.batch, -1) for a in A]
    dY = [net.tensor_np(l, lp.LP_T_DY).reshape(wl.batch, -1) for l in range(1, L + 1)]
    if products:
        for l in range(1, L + 1):
            ly = wl.layers[l - 1]
            z_ref = O.store(O.forward_product(A[l - 1], Wk[l - 1]), st)
            z_gpu = net.tensor_np(l, lp.LP_T_Z)
            if z_gpu is not None:
                z_gpu = z_gpu.reshape(z_ref.shape)
                assert relerr(z_gpu, z_ref) <= tol, ("F/Z", l, n)
            if l < L:
                a_ref = O.store(O.activation(z_gpu if z_gpu is not None else z_ref, ly.act), st)
                assert relerr(A[l], a_ref) <= tol, ("F/A", l, n)
        zL = net.tensor_np(L, lp.LP_T_Z).reshape(wl.batch, -1)
        if wl.loss == WL.SOFTMAX_CE:
            loss_ref, dyL = O.softmax_ce(zL, target)
        else:
            loss_ref, dyL = O.mse(zL, O.store(target, st).reshape(zL.shape))
        assert abs(float(net.loss_dev) - loss_ref) <= 1e-5 * max(1.0, abs(loss_ref)), ("loss", n)
        assert relerr(dY[L - 1], O.store(dyL, st)) <= tol, ("dY_L", n)
    for l in range(L, 0, -1):
        g = net.tensor_np(l, lp.LP_T_G_LAST).reshape(Wk[l - 1].shape)
        if products:
            assert relerr(g, O.grad_weight(A[l - 1], dY[l - 1])) <= tolG, ("dW", l, n)
        G_hist[l - 1][n] = g
        if l > 1:
            prev = wl.layers[l - 2]
            da = net.tensor_np(l - 1, lp.LP_T_DA)
            stash = net.tensor_np(l - 1, lp.LP_T_Z)
            stash = A[l - 1] if stash is None else stash.reshape(wl.batch, -1)
            if da is None:
                # the Hadamard product rode in the epilogue of dX_l: dA_{l-1} was never stored.  What can be compared is
                # the pair of tasks on the GPU's own dY_l, weights and stash, and the mask, which stays exact
                assert bf and prev.act in ("relu", "gelu"), ("dA missing", l - 1, n)
                if products:
                    da_ref = O.store(O.grad_act(dY[l - 1], Wk[l - 1]), st)
                    assert relerr(dY[l - 2], O.store(O.act_grad(da_ref, stash, prev.act), st)) <= tol, ("dX + Hadamard", l, n)
                if prev.act == "relu":
                    assert np.all(dY[l - 2][stash <= 0.0] == 0.0), ("ReLU mask", l - 1, n)
            else:
                da = da.reshape(wl.batch, -1)
                if products:
                    assert relerr(da, O.store(O.grad_act(dY[l - 1], Wk[l - 1]), st)) <= tol, ("dX", l, n)
                dy_ref = O.store(O.act_grad(da, stash, prev.act), st)
                if prev.act in ("relu", "identity"):
                    assert np.array_equal(dY[l - 2], dy_ref), ("Hadamard", l - 1, n)
                else:
                    assert relerr(dY[l - 2], dy_ref) <= 2.0 ** -7, ("Hadamard", l - 1, n)
        # Eq. 6 with the GPU's own G of d_l steps ago
        src = n - wl.delays[l - 1]
        w_new = net.get_weights(l)
        if src < 1:
            assert np.array_equal(w_new, W_before[l - 1]), ("frozen", l, n)
        else:
            g_old = G_hist[l - 1].pop(src)
            ref = O.store(O.delayed_sgd(W_before[l - 1].astype(np.float64), g_old, float(np.float32(wl.lr))), "f32")
            assert np.max(np.abs(w_new - ref)) <= 2.0 ** -22 * np.max(np.abs(ref)), ("update", l, n)
            if np.any(g_old != 0):
                assert not np.array_equal(w_new, W_before[l - 1]), ("update changed nothing", l, n)
        if bf:
            work = net.tensor_np(l, lp.LP_T_WORK_W).reshape(w_new.shape)
            assert np.array_equal(work, O.round_bf16(w_new)), ("working copy", l, n)


def run_trajectory(wl, steps, n_streams=3, taskwise=True, run_ahead=False, exact=True, product_steps=None, fused=True):
    """Free-running comparison with the oracle: loss, Z_L, every W_l(n) and every G_l in max-norm (for bf16 the
    bound on G_l is 2e-2 unless G_MAXNORM_BOUND lists a measured one).  With `exact`, a float64 oracle runs beside
    the bf16 one and the free-running G_l is also compared in Frobenius norm against max(2e-2, the bf16 oracle's
    own distance from the float64 oracle).  The bound that does not compound is the task-by-task check on
    identical inputs; `product_steps` (a set of step numbers, None = all) limits its recomputation of the products.
    `fused` = False runs the Hadamard products as kernels of their own, so that every dA exists and is compared."""
    bf = wl.dtype == "bf16"
    storage = "bf16" if bf else "f32"
    W0 = WL.init_weights(wl)
    net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, n_streams=n_streams, run_ahead=run_ahead, fused_hadamard=fused)
    net.set_weights(W0)
    ora = O.DelayedGradientTrainer(wl.layers, W0, wl.delays, wl.lr, wl.loss, storage)
    exact = O.DelayedGradientTrainer(wl.layers, W0, wl.delays, wl.lr, wl.loss, "f64") if (bf and exact) else None
    G_hist = [dict() for _ in range(wl.L)]
    rec = RECORDS.setdefault(run_key(wl), [])
    del rec[:]
    for n in range(1, steps + 1):
        print("run_trajectory %s step %d of %d" % (wl.name, n, steps), flush=True)
        x, t = WL.batch_input(wl, n), WL.batch_target(wl, n)
        W_before = [net.get_weights(l) for l in range(1, wl.L + 1)] if taskwise else None
        loss = net.step(x, t)
        ref = ora.step(x, t)
        if exact is not None:
            exact.step(x, t)
        tol = 2e-2 if bf else (1e-3 if n >= 8 else 1e-4)
        free = not (bf and RECORDING)
        zl = net.tensor_np(wl.L, lp.LP_T_Z).reshape(ora.trace["Z"][-1].shape)
        e_loss, e_zl = abs(loss - ref) / max(abs(ref), 1e-3), relerr(zl, ora.trace["Z"][-1])
        if free:
            assert e_loss <= tol, (n, loss, ref)
            assert e_zl <= (ZL_BOUND.get(run_key(wl), tol) if bf else tol), ("Z_L", n, e_zl)
        for l in range(1, wl.L + 1):
            g = net.tensor_np(l, lp.LP_T_G_LAST).reshape(ora.trace["G"][l - 1].shape)
            e, share = check_g_free_running(wl, l, n, g, ora.trace["G"][l - 1], None if exact is None else exact.trace["G"][l - 1])
            flips, units = relu_flips(net, wl, l, ora.trace["Z"][l - 1])
            w = net.get_weights(l)
            e_w = relerr(w, ora.W[l - 1])
            rec.append(dict(n=n, l=l, g_maxnorm=e, g_share_over=share, relu_flips=flips, relu_units=units, w_relerr=e_w, zl_relerr=e_zl,
                            loss_relerr=e_loss))
            if free:
                assert e_w <= tol, ("W", l, n)
            if n <= wl.delays[l - 1]:       # delay elements still empty: weights untouched, bit for bit
                assert np.array_equal(w, W0[l - 1]), ("frozen", l, n)
        if taskwise:
            check_tasks_of_last_step(net, wl, x, t, W_before, G_hist, n, products=(product_steps is None or n in product_steps))
    net.close()
    _dump_records(run_key(wl))


def test_trajectory_mlp_small_f32_full_config():
    wl = WL.mlp_small()
    assert wl.delays == (6, 4, 2, 0) and wl.steps == 8
    run_trajectory(wl, wl.steps)


@pytest.mark.parametrize("act", ["tanh", "sigmoid"])
@pytest.mark.parametrize("shape", [(96, 200, 136), (33, 77, 19), (300, 520, 264), (256, 2048, 512)])
def test_forward_product_saturating_activations(shape, act):
    """The activations the paper names next to ReLU (Sec. II-A), fused into the product's epilogue like the others."""
    B, K, N = shape
    for dtype, td, tol_z, tol_a in (("bf16", torch.bfloat16, 2e-2, 2.0 ** -7), ("f32", torch.float32, 1e-4, 1e-5)):
        net, W, rng = one_layer_net(K, N, B, act, dtype)
        x = rng.standard_normal((B, K)).astype(np.float32)
        Z = torch.empty(B, N, dtype=td, device=DEV)
        A = torch.empty(B, N, dtype=td, device=DEV)
        lp.lp_forward(net.ctx, 1, dev(x, td), Z, A, net.streams[0])
        lp.lp_sync(net.ctx)
        q = O.round_bf16 if dtype == "bf16" else (lambda v: v)
        assert relerr(host(Z), O.store(O.forward_product(q(x), q(W[0])), dtype)) <= tol_z
        assert relerr(host(A), O.store(O.activation(host(Z), act), dtype)) <= tol_a       # defined on the stored Z
        net.close()


@pytest.mark.parametrize("act", ["tanh", "sigmoid"])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_trajectory_saturating_activations(act, dtype):
    wl = WL.mlp_4096().with_(layers=WL._mlp([200, 264, 136, 72, 24], act), batch=48, delays=(6, 4, 2, 0), dtype=dtype, lr=0.05)
    run_trajectory(wl, 12)


# fused: the Hadamard product of layer l-1 inside the dX product of layer l (the default of lp_step), or as a kernel
# of its own, which keeps every dA in memory for the task-by-task comparison
@pytest.mark.parametrize("fused", [True, False])
def test_trajectory_mlp_bf16_scaled(fused):
    wl = WL.mlp_4096().with_(layers=WL._mlp([512] * 8 + [1000], WL.RELU), batch=64)
    assert wl.delays == tuple(range(14, -1, -2))
    run_trajectory(wl, 18, fused=fused)


@pytest.mark.parametrize("fused", [True, False])
def test_trajectory_ffn_gelu_mse_bf16_scaled(fused):
    wl = WL.ffn_stack(d=256, hidden=1024, tokens=512, n_linear=16)
    run_trajectory(wl, 10, fused=fused)


@pytest.mark.parametrize("fused", [True, False])
def test_trajectory_imbalanced_bf16_scaled(fused):
    full = WL.mlp_imbalanced()
    widths = [full.layers[0].d_in // 8] + [l.d_out // 8 for l in full.layers]   # 128, 128, 1024, 256, ... 125
    wl = full.with_(layers=WL._mlp(widths, WL.RELU), batch=128)
    run_trajectory(wl, 10, fused=fused)


def test_ragged_unaligned_network_bf16():
    wl = WL.mlp_4096().with_(layers=WL._mlp([77, 130, 45, 19, 10], WL.RELU), batch=33, delays=(6, 4, 2, 0), lr=0.01)
    run_trajectory(wl, 8)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_one_stream_and_three_streams_are_bit_identical(dtype):
    wl = WL.mlp_4096().with_(layers=WL._mlp([256, 320, 192, 136, 40], WL.RELU), batch=96, delays=(6, 4, 2, 0), dtype=dtype)
    W0 = WL.init_weights(wl)
    outs = []
    for ns in (1, 3, 2):
        net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, n_streams=ns)
        net.set_weights(W0)
        losses = [net.step(WL.batch_input(wl, n), WL.batch_target(wl, n)) for n in range(1, 10)]
        outs.append((losses, [net.get_weights(l) for l in range(1, wl.L + 1)]))
        net.close()
    for o in outs[1:]:
        assert o[0] == outs[0][0]
        assert all(np.array_equal(a, b) for a, b in zip(o[1], outs[0][1]))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_zero_delay_step_equals_textbook_order_of_per_layer_calls(dtype):
    wl = WL.mlp_4096().with_(layers=WL._mlp([128, 96, 64, 24], WL.RELU), batch=48, delays=(0, 0, 0), dtype=dtype)
    W0 = WL.init_weights(wl)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    a = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays)
    b = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays)
    a.set_weights(W0); b.set_weights(W0)
    s = b.streams[0]
    for n in range(1, 4):
        x, t = WL.batch_input(wl, n), WL.batch_target(wl, n)
        la = a.step(x, t)
        xd, tdv = b.to_device(x), b.to_device(t, is_label=True)
        torch.cuda.synchronize()
        A, Z = [xd], []
        for l, ly in enumerate(wl.layers, start=1):
            z = torch.empty(wl.batch, ly.d_out, dtype=td, device=DEV)
            act = torch.empty_like(z)
            lp.lp_forward(b.ctx, l, A[-1], z, act, s)
            Z.append(z); A.append(act)
        dY = torch.empty_like(Z[-1])
        lp.lp_loss_grad(b.ctx, Z[-1], tdv, dY, b.loss_dev, s)
        for l in range(wl.L, 0, -1):
            lp.lp_grad_weight(b.ctx, l, A[l - 1], dY, None, s)
            if l > 1:
                dA = torch.empty(wl.batch, wl.layers[l - 1].d_in, dtype=td, device=DEV)
                lp.lp_grad_act(b.ctx, l, dY, dA, 0, wl.layers[l - 1].d_in, s)
                dYp = torch.empty_like(dA)
                lp.lp_act_grad(b.ctx, l - 1, dA, Z[l - 2], dYp, s)
            lp.lp_update(b.ctx, l, None, s)
            if l > 1:
                dY = dYp
        lp.lp_advance(b.ctx)
        lp.lp_sync(b.ctx)
        assert float(b.loss_dev) == la
        for l in range(1, wl.L + 1):
            assert np.array_equal(a.get_weights(l), b.get_weights(l)), (n, l)
    assert lp.lp_step_index(a.ctx) == lp.lp_step_index(b.ctx) == 3
    a.close(); b.close()


def test_step_delay_override_and_errors():
    wl = WL.mlp_4096().with_(layers=WL._mlp([64, 48, 16], WL.RELU), batch=16, delays=(4, 0))
    W0 = WL.init_weights(wl)
    net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays)
    net.set_weights(W0)
    xd, td = net.to_device(WL.batch_input(wl, 1)), net.to_device(WL.batch_target(wl, 1), True)
    with pytest.raises(lp.LpError) as ei:
        lp.lp_step(net.ctx, xd, td, [5, 0], net.loss_dev, net.streams)      # beyond the ring the context sized
    assert ei.value.status == 5
    ora = O.DelayedGradientTrainer(wl.layers, W0, (2, 0), wl.lr, wl.loss, "bf16")
    for n in range(1, 7):
        x, t = WL.batch_input(wl, n), WL.batch_target(wl, n)
        net.step(x, t, delay=[2, 0] if n == 1 else None)
        ora.step(x, t)
    for l in (1, 2):
        assert relerr(net.get_weights(l), ora.W[l - 1]) <= 2e-2
    assert not np.array_equal(net.get_weights(1), W0[0])
    net.close()


@pytest.mark.parametrize("n_streams", [1, 3])
def test_delta_split_inside_step_changes_no_bits(n_streams):
    """delta' on the critical stream and delta'' as an independent kernel (Sec. III-B): same weights, bit for bit."""
    wl = WL.mlp_4096().with_(layers=WL._mlp([256, 320, 192, 136, 40], WL.RELU), batch=96, delays=(6, 4, 2, 0))
    W0 = WL.init_weights(wl)
    outs = []
    for splits in (None, {2: 104, 3: 1, 4: 135}):
        net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, n_streams=n_streams)
        net.set_weights(W0)
        if splits:
            for l, c in splits.items():
                lp.lp_set_delta_split(net.ctx, l, c)
        losses = [net.step(WL.batch_input(wl, n), WL.batch_target(wl, n)) for n in range(1, 9)]
        outs.append((losses, [net.get_weights(l) for l in range(1, wl.L + 1)]))
        net.close()
    assert outs[0][0] == outs[1][0]
    assert all(np.array_equal(a, b) for a, b in zip(outs[0][1], outs[1][1]))


def test_delta_split_argument_errors():
    wl = WL.mlp_4096().with_(layers=WL._mlp([64, 48, 16], WL.RELU), batch=16, delays=(2, 0))
    net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays)
    for l, c, status in ((1, 8, 4), (2, 48, 2), (2, -1, 2), (3, 1, 4)):
        with pytest.raises(lp.LpError) as ei:
            lp.lp_set_delta_split(net.ctx, l, c)
        assert ei.value.status == status
    lp.lp_set_delta_split(net.ctx, 2, 47)
    lp.lp_set_delta_split(net.ctx, 1, 0)
    net.close()


# ---- degenerate networks and the size guard ---------------------------------------------------------
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_trajectory_single_layer_network(dtype):
    """L = 1: no dX task, no Hadamard, the only layer feeds the loss (multinomial logistic regression)."""
    wl = WL.mlp_4096().with_(layers=WL._mlp([72, 10], WL.RELU), batch=40, delays=(0,), dtype=dtype, lr=0.1)
    run_trajectory(wl, 6)


def test_trajectory_batch_of_one_and_delayed_last_layer():
    """One sample per step (every product degenerates to a row), and a last layer whose own update is delayed too."""
    wl = WL.mlp_4096().with_(layers=WL._mlp([40, 24, 16, 8], WL.RELU), batch=1, delays=(5, 3, 2), dtype="f32", lr=0.05)
    run_trajectory(wl, 10)
    wl = WL.mlp_4096().with_(layers=WL._mlp([136, 72, 24], WL.GELU), batch=1, delays=(1, 1), dtype="bf16", lr=0.05)
    run_trajectory(wl, 6)


def test_operand_beyond_32_bit_offsets_is_rejected_not_launched():
    """Byte offsets inside the kernels are 32-bit; a weight matrix of 2 GiB is refused when the context is made."""
    n = 32768
    layers = (WL.Layer(WL.LINEAR, n, n, WL.IDENTITY),)
    with pytest.raises(lp.LpError) as e:
        lp.Network(layers, 8, "bf16", WL.MSE, 0.01, (0,))
    assert e.value.status == 2          # LP_ERR_SHAPE


def test_softmax_label_outside_the_classes_is_not_dereferenced():
    """A bad label gives that row the plain softmax as delta and a NaN loss; the other rows are untouched."""
    rows, cols = 6, 1000
    layers = (WL.Layer(WL.LINEAR, 16, cols, WL.IDENTITY),)
    for dtype, td in (("bf16", torch.bfloat16), ("f32", torch.float32)):
        net = lp.Network(layers, rows, dtype, WL.SOFTMAX_CE, 0.01, (0,))
        rng = np.random.default_rng(3)
        zd = dev(rng.standard_normal((rows, cols)).astype(np.float32), td)
        y = rng.integers(0, cols, rows).astype(np.int32)
        bad = y.copy(); bad[2] = cols; bad[4] = -7
        dY, dYb = torch.empty_like(zd), torch.empty_like(zd)
        loss, lossb = synced(torch.zeros(1, device=DEV)), synced(torch.zeros(1, device=DEV))
        yd, badd = dev(y, torch.int32), dev(bad, torch.int32)      # both alive until the kernels that read them have run
        lp.lp_loss_grad(net.ctx, zd, yd, dY, loss, net.streams[0])
        lp.lp_loss_grad(net.ctx, zd, badd, dYb, lossb, net.streams[0])
        lp.lp_sync(net.ctx)
        assert np.isfinite(float(loss)) and np.isnan(float(lossb))
        good = [0, 1, 3, 5]
        assert torch.equal(dY[good], dYb[good])
        p = np.exp(host(zd) - host(zd).max(axis=1, keepdims=True)); p /= p.sum(axis=1, keepdims=True)
        assert relerr(host(dYb)[[2, 4]], p[[2, 4]] / rows) <= (2e-2 if dtype == "bf16" else 1e-5)
        net.close()


def test_mfma_probe_runs_the_rounds_it_is_asked_for():
    """The calibration kernel of the matrix-core roofline: with the uniform operands every product and every
    partial sum is a small multiple of 2^-20, so the checksums are exact and linear in the number of rounds."""
    out1 = synced(torch.zeros(4 * 512, dtype=torch.float32, device=DEV))
    out2 = synced(torch.zeros(4 * 512, dtype=torch.float32, device=DEV))
    s = torch.cuda.Stream()
    lp.lp_probe_mfma(out1, 4, 100, True, s)
    lp.lp_probe_mfma(out2, 4, 200, True, s)
    s.synchronize()
    a, b = out1.cpu().numpy(), out2.cpu().numpy()
    assert np.all(a > 0) and np.array_equal(b, 2 * a)
    assert np.array_equal(a[:512], a[512:1024])                  # every workgroup holds the same uniform operands
    lp.lp_probe_mfma(out1, 4, 100, False, s)
    s.synchronize()
    r = out1.cpu().numpy()
    assert np.all(np.isfinite(r)) and not np.array_equal(r[:512], r[512:1024])   # random operands differ by workgroup
