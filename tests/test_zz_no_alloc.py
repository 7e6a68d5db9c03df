"""lp_loss_grad_static: the loss task with its partial sums in a static device array of the library instead of the
caller's workspace, for callers that cannot allocate.  Called through the C ABI on contexts that have NO workspace
bound and compared bit for bit with lp_loss_grad of a context that has one; two calls in a row, the second on a
smaller input (the array keeps the first call's contents).  Needs a real MI355X."""
import ctypes as C

import numpy as np
import pytest
import torch

import lp_workloads as WL
import paper_2108_06629_amd as lp


def synced(t):
    """A tensor torch has just filled on its own stream; the library's streams are not ordered after it."""
    torch.cuda.synchronize()
    return t


pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def bare_context(rows, cols, dtype, loss):
    """A context without workspace: lp_create only."""
    layers = (WL.Layer(WL.LINEAR, 16, cols, WL.IDENTITY),)
    return lp.lp_create(lp.make_descs(layers, (0,)), 1, rows, lp._DTYPE[dtype], lp._LOSS[loss], 0.01)


def reference(rows, cols, dtype, loss, z, target):
    layers = (WL.Layer(WL.LINEAR, 16, cols, WL.IDENTITY),)
    net = lp.Network(layers, rows, dtype, loss, 0.01, (0,))
    dY = torch.full_like(z, float("nan"))
    out = synced(torch.full((1,), float("nan"), dtype=torch.float32, device=DEV))
    lp.lp_loss_grad(net.ctx, z, target, dY, out, net.streams[0])
    lp.lp_sync(net.ctx)
    net.close()
    return dY, out


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("loss,shapes", [(WL.SOFTMAX_CE, [(1024, 1000), (96, 1000)]), (WL.SOFTMAX_CE, [(300, 10), (7, 33)]),
                                         (WL.MSE, [(512, 4096), (33, 1643)]), (WL.MSE, [(64, 256), (3, 7)])])
def test_static_scratch_loss_equals_workspace_loss_on_two_calls_in_a_row(dtype, loss, shapes):
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    stream = torch.cuda.Stream()
    rng = np.random.default_rng(11)
    for rows, cols in shapes:                 # second call: smaller input, same static array
        z = torch.from_numpy(rng.standard_normal((rows, cols)).astype(np.float32)).to(DEV).to(td)
        if loss == WL.SOFTMAX_CE:
            target = torch.from_numpy(rng.integers(0, cols, rows).astype(np.int32)).to(DEV)
        else:
            target = torch.from_numpy(rng.standard_normal((rows, cols)).astype(np.float32)).to(DEV).to(td)
        torch.cuda.synchronize()
        dY_ref, loss_ref = reference(rows, cols, dtype, loss, z, target)
        ctx = bare_context(rows, cols, dtype, loss)
        dY = torch.full_like(z, float("nan"))
        out = synced(torch.full((1,), float("nan"), dtype=torch.float32, device=DEV))
        st = lp.lib().lp_loss_grad_static(ctx, z.data_ptr(), target.data_ptr(), dY.data_ptr(), out.data_ptr(), stream.cuda_stream)
        assert st == 0, lp.lib().lp_last_error(ctx)
        stream.synchronize()
        assert torch.equal(dY.view(torch.int16 if dtype == "bf16" else torch.int32), dY_ref.view(torch.int16 if dtype == "bf16" else torch.int32))
        assert torch.equal(out.view(torch.int32), loss_ref.view(torch.int32)) and np.isfinite(float(out))
        # without the scalar loss
        dY2 = torch.full_like(z, float("nan"))
        assert lp.lib().lp_loss_grad_static(ctx, z.data_ptr(), target.data_ptr(), dY2.data_ptr(), None, stream.cuda_stream) == 0
        stream.synchronize()
        assert torch.equal(dY2.view(torch.int16 if dtype == "bf16" else torch.int32), dY_ref.view(torch.int16 if dtype == "bf16" else torch.int32))
        lp.lp_destroy(ctx)


def test_static_scratch_limit_and_argument_errors():
    ctx = bare_context(65537, 8, "bf16", WL.SOFTMAX_CE)         # one row more than the array holds partials for
    fake = 0x10000                                               # never dereferenced: the call fails in validation
    assert lp.lib().lp_loss_grad_static(ctx, fake, fake, fake, None, None) == 2
    assert b"65536" in lp.lib().lp_last_error(ctx)
    lp.lp_destroy(ctx)
    ctx = bare_context(65536, 8200, "bf16", WL.MSE)              # 65536 * 8200 elements need 65600 partials
    assert lp.lib().lp_loss_grad_static(ctx, fake, fake, fake, None, None) == 2
    assert lp.lib().lp_loss_grad_static(ctx, None, fake, fake, None, None) == 1
    assert lp.lib().lp_loss_grad_static(None, fake, fake, fake, None, None) == 1
    lp.lp_destroy(ctx)
