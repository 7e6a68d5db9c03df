#!/usr/bin/env python3
"""Benchmark of the LayerPipe hot path on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--streams S]

One "step" is one whole delayed-gradient training iteration (lp_step: F, loss, dX, the moved
Hadamard, dW and the delayed update of every layer) over one synthetic minibatch that is already
resident in HBM.  By default Eq. 6 runs in its retimed form (lp_set_retimed_update: the delays sit on
the weights, the G task applies its gradient in the product's epilogue; losses and working weights are
those of the gradient-ring form bit for bit, which --gradient-ring times instead and the default run
times beside it).  Prints ONE JSON line: training samples/s of the whole job, the roofline of the
dominant kernel (the bf16 MFMA GEMM of the forward product), per-task achieved rates, and the CPU
oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0

# Bytes the L2s request from the fabric (Infinity Cache + HBM) plus bytes written, per launch, from rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE runs of this script scaled by a 1 GiB copy.  Counters cannot be read from inside this
# process, so the figure is tied to the exact kernel it was measured on: a kernel whose name differs (any change of
# its template arguments) has no entry and reports "traffic": null until it is profiled again.
MEASURED_TRAFFIC = {
    ("ffn_stack_bf16", "gemm_bf16_dl_kernel<256,256,64,2,2,4,true,false,false>"):
        {"bytes": 1.6232e9 + 3.020e8, "profile": "profiles/hbm_traffic_ffn_stack.md"},
}
# the kernel that runs the forward product of the default workload (every layer of it takes this instantiation)
F_KERNEL = {"ffn_stack_bf16": "gemm_bf16_dl_kernel<256,256,64,2,2,4,true,false,false>"}


def task_work(wl):
    """Algorithmic work per step of each task kind: flops for the three products, HBM bytes for the
    bandwidth-bound tasks (act-type tensors 2 B for bf16 / 4 B for fp32; G and master weights 4 B)."""
    import lp_workloads as WL
    es = 2 if wl.dtype == "bf16" else 4
    f, dx, dw = wl.flops_per_step()
    had = 0.0
    for l, ly in enumerate(wl.layers[:-1]):
        if ly.act == WL.IDENTITY and not ly.pool:
            continue                         # delta == dA, no kernel
        z = 1
        for v in ly.z_shape(wl.batch):
            z *= v
        a = 1
        for v in ly.out_shape(wl.batch):
            a *= v
        had += (a + 2 * z) * es              # read dA, read stash, write dY
    last = wl.layers[-1]
    n_out = wl.batch * last.d_out
    loss = n_out * es * (3 if wl.loss == WL.MSE else 2) + (4 * wl.batch if wl.loss != WL.MSE else 0)
    per_param = 14 if wl.dtype == "bf16" else 12   # read G, read+write master (, write bf16 copy)
    return {"F": f, "dX": dx, "dW": dw, "hadamard": had, "loss": float(loss), "update_per_param": per_param}


def blas_threads():
    """(threads the BLAS behind numpy uses, what the library calls itself); the oracle's products run on them."""
    try:
        from threadpoolctl import threadpool_info
        pools = [p for p in threadpool_info() if p.get("user_api") == "blas"]
        if pools:
            return max(int(p.get("num_threads", 1)) for p in pools), ", ".join(sorted(set(str(p.get("internal_api")) for p in pools)))
    except Exception:
        pass
    return None, "unknown"


def cpu_baseline(wl):
    """The oracle as it stands, timed on a bounded sample: one training step on at most 256 samples;
    for networks above 5e8 parameters only the first two layers (one up/down block) on up to 8192 samples
    (about ten seconds of work),
    scaled to the whole network by the ratio of per-sample flops."""
    import numpy  # noqa: F401  (loads the BLAS whose thread pool is reported)
    import lp_workloads as WL
    from oracle import layerpipe_oracle as O
    threads, blas = blas_threads()
    if threads is None:
        threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)
    if wl.n_params > 5e8:
        sub = wl.with_(layers=wl.layers[:2], batch=min(wl.batch, 8192), delays=wl.delays[-2:])
        what = "the first 2 of %d layers" % wl.L
    else:
        sub = wl.with_(batch=min(wl.batch, 256))
        what = "all %d layers" % wl.L
    scale = (sum(wl.flops_per_step()) / wl.batch) / (sum(sub.flops_per_step()) / sub.batch)
    W0 = WL.init_weights(sub)
    ora = O.DelayedGradientTrainer(sub.layers, W0, sub.delays, sub.lr, sub.loss, "bf16" if wl.dtype == "bf16" else "f32")
    x, t = WL.batch_input(sub, 1), WL.batch_target(sub, 1)
    t0 = time.perf_counter()
    ora.step(x, t)
    dt = time.perf_counter() - t0
    return {"value": sub.batch / (dt * scale), "unit": "samples/s", "cores": threads, "kind": "oracle",
            "host_cpus": os.cpu_count(), "blas": blas, "omp_num_threads_env": os.environ.get("OMP_NUM_THREADS"),
            "sample": "one oracle training step (numpy float64; its products ran on %d BLAS threads (%s) of a host that shows %s CPUs) "
                      "of %s of %s at full widths on %d of the %d samples "
                      "of a minibatch took %.1f s; scaled by the per-sample flop ratio %.2f to the whole network" % (
                          threads, blas, os.cpu_count(), what, wl.name, sub.batch, wl.batch, dt, scale)}


def operand_values(reps=20):
    """F, dX and dW of one (4096 -> 16384 GELU, 16384 -> 4096) pair of ffn_stack_bf16 through the per-layer entry points, once
    on operands drawn as the benchmark draws them (N(0,1) activations and gradients, He-normal weights) and once with every
    operand element equal to 2^-7.  Kernels, addresses and bytes moved are the same in both; what differs is how many bits
    toggle in the multipliers, i.e. the energy of a multiply, which is what this chip's clock follows."""
    import numpy as np
    import torch
    import lp_workloads as WL
    import paper_2108_06629_amd as lp
    wl = WL.ffn_stack(n_linear=2)
    B, d, h = wl.batch, wl.layers[0].d_in, wl.layers[0].d_out
    rows = []
    for uniform in (False, True):
        net = lp.Network(wl.layers, B, wl.dtype, wl.loss, wl.lr, (0, 0), n_streams=1)
        W = [np.full(ly.weight_shape, 2.0 ** -7, dtype=np.float32) for ly in wl.layers] if uniform else WL.init_weights(wl)
        net.set_weights(W)
        del W
        s = net.streams[0]

        def gen(rows_, cols):
            t = torch.empty(rows_, cols, dtype=torch.bfloat16, device="cuda:0")
            return t.fill_(2.0 ** -7) if uniform else t.normal_()
        x1, dy1, x2, dy2 = gen(B, d), gen(B, h), gen(B, h), gen(B, d)
        z1, a1, z2 = torch.empty_like(dy1), torch.empty_like(dy1), torch.empty_like(dy2)
        dx1, dx2 = torch.empty_like(x1), torch.empty_like(x2)
        g = torch.empty(d * h, dtype=torch.float32, device="cuda:0")
        torch.cuda.synchronize()
        tasks = (("F up (Z and A = GELU(Z))", (B, h, d), lambda: lp.lp_forward(net.ctx, 1, x1, z1, a1, s)),
                 ("F down", (B, d, h), lambda: lp.lp_forward(net.ctx, 2, x2, z2, None, s)),
                 ("dX of the down-projection", (B, h, d), lambda: lp.lp_grad_act(net.ctx, 2, dy2, dx2, 0, h, s)),
                 ("dX of the up-projection", (B, d, h), lambda: lp.lp_grad_act(net.ctx, 1, dy1, dx1, 0, d, s)),
                 ("dW of the up-projection", (d, h, B), lambda: lp.lp_grad_weight(net.ctx, 1, x1, dy1, g, s)),
                 ("dW of the down-projection", (h, d, B), lambda: lp.lp_grad_weight(net.ctx, 2, x2, dy2, g, s)))
        for i, (name, (M, N, K), fn) in enumerate(tasks):
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(s)
            for _ in range(reps):
                fn()
            e1.record(s)
            s.synchronize()
            ms = e0.elapsed_time(e1) / reps
            tf = 2.0 * M * N * K / (ms * 1e-3) / 1e12
            if not uniform:
                rows.append({"task": name, "M_N_K": [M, N, K]})
            rows[i]["uniform" if uniform else "random"] = {"ms_per_launch": ms, "TFLOP/s": tf, "frac_of_bf16_peak": tf / PEAK_BF16_TFLOPS}
        net.close()
        del net, x1, dy1, x2, dy2, z1, a1, z2, dx1, dx2, g
        torch.cuda.empty_cache()
    return rows


def partition_report(wl, max_stages):
    """Per-layer task times measured on one stream (no overlap), fed to the library's Algorithm 1:
    T_fix = F + dW, T_flex = dX (Sec. III-C).  For each stage count: the balanced stage times, the
    delta'' fractions, and the best assignment of whole layers to contiguous stages for comparison;
    then one run with the delta'' column splits applied inside lp_step."""
    import torch
    import lp_workloads as WL
    import paper_2108_06629_amd as lp
    net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, n_streams=1)
    net.set_weights(WL.init_weights(wl))
    x = net.to_device(WL.batch_input(wl, 1))
    t = net.to_device(WL.batch_target(wl, 1), is_label=(wl.loss == WL.SOFTMAX_CE))
    for _ in range(5):
        net.step_device(x, t)
    lp.lp_sync(net.ctx)
    lp.lp_profile(net.ctx, True)
    reps = 20
    for _ in range(reps):
        net.step_device(x, t)
    lp.lp_sync(net.ctx)
    lp.lp_profile(net.ctx, False)
    per = {}
    for k, name in enumerate(lp.TASK_NAMES[:3]):
        per[name] = [lp.lp_profile_read_layer(net.ctx, k, l)[0] / reps for l in range(1, wl.L + 1)]
    net.close()
    t_fix = [f + w for f, w in zip(per["F"], per["dW"])]
    t_flex = per["dX"]
    tot = [a + b for a, b in zip(t_fix, t_flex)]

    def best_whole_layers(n):       # minimise the bottleneck over contiguous whole-layer stages (dynamic programme)
        L = len(tot)
        pre = [0.0]
        for v in tot:
            pre.append(pre[-1] + v)
        INF = float("inf")
        dp = [[INF] * (L + 1) for _ in range(n + 1)]
        dp[0][0] = 0.0
        for s in range(1, n + 1):
            for j in range(1, L + 1):
                for i in range(s - 1, j):
                    dp[s][j] = min(dp[s][j], max(dp[s - 1][i], pre[j] - pre[i]))
        return min(dp[s][L] for s in range(1, n + 1))

    rows = []
    for n in range(2, max_stages + 1):
        r = lp.lp_partition(t_fix, t_flex, n, 1.01)
        rows.append({"stages": n, "balanced_bottleneck_ms": max(r["stage_time"]), "whole_layer_bottleneck_ms": best_whole_layers(n),
                     "speedup_vs_1": sum(tot) / max(r["stage_time"]), "whole_layer_speedup_vs_1": sum(tot) / best_whole_layers(n),
                     "stage_fix": r["stage_fix"], "borrowed_frac": [round(v, 4) for v in r["borrowed_frac"]],
                     "stage_time_ms": [round(v, 4) for v in r["stage_time"]]})
    # apply the last partition's delta'' fractions as column splits and time the step
    r = lp.lp_partition(t_fix, t_flex, max_stages, 1.01)
    times = {}
    for label, use in (("unsplit", False), ("split", True)):
        net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, n_streams=3)
        net.set_weights(WL.init_weights(wl))
        if use:
            for l in range(2, wl.L + 1):
                cols = int(round(r["borrowed_frac"][l - 1] * wl.layers[l - 1].d_in / 8.0)) * 8
                lp.lp_set_delta_split(net.ctx, l, min(max(cols, 0), wl.layers[l - 1].d_in - 8))
        x = net.to_device(WL.batch_input(wl, 1))
        t = net.to_device(WL.batch_target(wl, 1), is_label=(wl.loss == WL.SOFTMAX_CE))
        for _ in range(5):
            net.step_device(x, t)
        lp.lp_sync(net.ctx)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(20):
            net.step_device(x, t)
        lp.lp_sync(net.ctx)
        torch.cuda.synchronize()
        times[label] = (time.perf_counter() - t0) / 20 * 1e3
        net.close()
    return {"workload": wl.name, "per_layer_ms": {k: [round(v, 4) for v in vals] for k, vals in per.items()},
            "partitions": rows, "step_ms_three_streams": times}


RETIMED_UPDATE = True    # --gradient-ring clears it; lp_set_retimed_update on every layer that qualifies (bf16 contexts)
FUSED_HADAMARD = True   # --separate-hadamard clears it: Eq. 3 then runs as a kernel of its own after every dX product


def fills_chip(wl):
    """Every product of every layer covers the chip with 256 x 256 tiles on its own (one per CU at least)."""
    import lp_workloads as WL
    t = lambda m, n: -(-m // 256) * -(-n // 256)
    return all(ly.kind == WL.LINEAR and t(wl.batch, ly.d_out) >= 256 and t(wl.batch, ly.d_in) >= 256 and t(ly.d_in, ly.d_out) >= 256
               for ly in wl.layers)


def default_streams(wl, retimed):
    """Streams of the serial schedule when --streams is not given: three, on which small kernels run side by side and the
    delayed updates overlap the products -- but one for a network whose every product fills the chip alone once the
    retimed update has removed the update tasks: nothing is left to run beside the products, and the forks and joins
    of a step only cost (ffn_stack: 44.43 ms on three streams, 44.22 ms on one, same box); and one for a network so
    small that the host's enqueue time bounds its step."""
    if sum(wl.flops_per_step()) < 1e10:
        # a step of a few microseconds of GPU work is bound by the host's enqueue time, and cross-stream waits are the
        # expensive part of that (mlp_small: 0.13 ms per step on one stream, 0.22 ms on three)
        return 1
    return 1 if (retimed and wl.dtype == "bf16" and fills_chip(wl)) else 3


def run_workload(wl, steps, warmup, n_streams, profile=True, weights=None, run_ahead=False, factor_ring=False, retimed=None):
    import numpy as np
    import torch
    import lp_workloads as WL
    import paper_2108_06629_amd as lp

    dev = torch.device("cuda:0")
    net = lp.Network(wl.layers, wl.batch, wl.dtype, wl.loss, wl.lr, wl.delays, device="cuda:0", n_streams=n_streams,
                     run_ahead=run_ahead, factor_ring=(True if factor_ring else None), fused_hadamard=FUSED_HADAMARD,
                     retimed_update=(True if (RETIMED_UPDATE if retimed is None else retimed) and wl.dtype == "bf16" and not factor_ring else None))
    net.set_weights(WL.init_weights(wl) if weights is None else weights)
    # a small pool of resident minibatches, reused round-robin
    pool = 4
    xs = [net.to_device(WL.batch_input(wl, n)) for n in range(1, pool + 1)]
    ts = [net.to_device(WL.batch_target(wl, n), is_label=(wl.loss == WL.SOFTMAX_CE)) for n in range(1, pool + 1)]
    torch.cuda.synchronize(dev)
    s0 = net.streams[0]
    for i in range(warmup):
        net.step_device(xs[i % pool], ts[i % pool])
    lp.lp_sync(net.ctx)
    torch.cuda.synchronize(dev)
    n0 = lp.lp_step_index(net.ctx)
    if profile:
        lp.lp_profile(net.ctx, True)
    t0 = time.perf_counter()
    for i in range(steps):
        net.step_device(xs[i % pool], ts[i % pool])
    lp.lp_sync(net.ctx)
    torch.cuda.synchronize(dev)
    dt = time.perf_counter() - t0
    loss = float(net.loss_dev.item())
    prof = {}
    if profile:
        lp.lp_profile(net.ctx, False)
        for k, name in enumerate(lp.TASK_NAMES):
            ms, cnt = lp.lp_profile_read(net.ctx, k, reset=True)
            prof[name] = (ms, cnt)
    # how many layer updates ran in the timed steps (layers with n <= d_l are still frozen; a layer with the retimed
    # update -- it keeps no gradients, like a factor ring, which this script never combines with it -- applies one in every step)
    applies_at_once = [not factor_ring and net.tensor(l, lp.LP_T_G_LAST) is None for l in range(1, wl.L + 1)]
    upd_params = 0
    for n in range(n0 + 1, n0 + steps + 1):
        upd_params += sum(ly.n_params for ly, d, now in zip(wl.layers, wl.delays, applies_at_once) if now or n - d >= 1)
    net.close()
    del net
    torch.cuda.empty_cache()
    return dt, loss, prof, upd_params


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--workload", default="ffn_stack_bf16")
    ap.add_argument("--streams", type=int, default=None,
                    help="streams of the serial schedule (default: 3; 1 for a network whose every product fills the chip, with the retimed update)")
    ap.add_argument("--no-task-timing", action="store_true", help="no per-task events in the timed steps (they cost host time; roofline and tasks are then empty)")
    ap.add_argument("--ra-streams", type=int, default=4, help="distinct streams of the run-ahead schedule (2, 3 or 4)")
    ap.add_argument("--run-ahead", action="store_true",
                    help="forward run-ahead across steps (lp_set_run_ahead): F(n+1) on a fourth stream next to the backward pass of step n")
    ap.add_argument("--factor-ring", action="store_true",
                    help="keep (A, dY) pairs instead of G in the delay elements and fuse the product into the delayed update (lp_set_factor_ring)")
    ap.add_argument("--gradient-ring", action="store_true",
                    help="Eq. 6 as printed: G_l(n) into a ring of d_l + 1 gradients, a delayed update task per layer and step.  Default is its retimed form "
                         "(lp_set_retimed_update: the G task applies its gradient in the product's epilogue, steps read weight versions d_l + 1 steps old; "
                         "same losses and working weights bit for bit, no gradient ring, no update task)")
    ap.add_argument("--separate-hadamard", action="store_true",
                    help="run the Hadamard products f'(S) (.) dA as kernels of their own instead of inside the dX products (lp_set_fused_hadamard 0)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the short runs of the other workloads")
    ap.add_argument("--partition", type=int, default=0, metavar="NP",
                    help="instead of the benchmark line: measure every layer's task times, run Algorithm 1 for 2..NP stages and "
                         "print the balanced stage times next to the best whole-layer (PipeDream-style) assignment")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run five 1 GiB device-to-device copy kernels (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--calibrate-operands", action="store_true",
                    help="time the three products of one ffn_stack layer pair on the benchmark's random operands and on operands that all "
                         "hold one small value: same kernels and bytes, different switching activity in the multipliers")
    ap.add_argument("--calibrate-mfma", action="store_true",
                    help="only run the matrix-instruction-only kernel (lp_probe_mfma) with one and with two workgroups per CU and "
                         "print what it sustains: the practical ceiling of the bf16 MFMA roofline on this machine")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one MI355X per box, no collectives); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    global FUSED_HADAMARD, RETIMED_UPDATE
    FUSED_HADAMARD = not args.separate_hadamard
    RETIMED_UPDATE = not args.gradient_ring and not args.factor_ring

    import torch
    import lp_workloads as WL
    import paper_2108_06629_amd as lp
    lp.load_library()          # fails loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    if args.calibrate_copy:
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": {"bytes_read": src.numel() * 2, "bytes_written": src.numel() * 2, "copies": 5}}))
        return

    def mfma_only(per_cu, uniform, reps):
        """lp_probe_mfma with `per_cu` workgroups per CU: (workgroups, rounds, ms per launch, TFLOP/s, a checksum)."""
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        wgs, iters = cus * per_cu, 20000 // per_cu
        out = torch.empty(wgs * 512, dtype=torch.float32, device="cuda:0")
        s = torch.cuda.Stream()
        lp.lp_probe_mfma(out, wgs, 200, uniform, s)
        s.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(s)
        for _ in range(reps):
            lp.lp_probe_mfma(out, wgs, iters, uniform, s)
        e1.record(s)
        s.synchronize()
        ms = e0.elapsed_time(e1) / reps
        return wgs, iters, ms, wgs * 8 * iters * 8 * 32768.0 / (ms * 1e-3) / 1e12, float(out[0].item())

    if args.calibrate_mfma:
        rows = []
        for per_cu, uniform in ((1, False), (2, False), (1, True)):     # 1: two waves per SIMD, as in the 256 x 256 GEMM; 2: four
            wgs, iters, ms, tf, chk = mfma_only(per_cu, uniform, 8)
            rows.append({"workgroups": wgs, "iters": iters, "operands": "uniform small values" if uniform else "pseudo-random in [-1, 1)",
                         "ms_per_launch": ms, "TFLOP/s": tf, "frac_of_bf16_peak": tf / PEAK_BF16_TFLOPS, "checksum": chk})
        print(json.dumps({"calibrate_mfma": rows}))
        return

    if args.calibrate_operands:
        print(json.dumps({"calibrate_operands": operand_values()}))
        return

    wl = WL.CONFIGS[args.workload]()
    streams_given = args.streams is not None
    if not streams_given:
        args.streams = default_streams(wl, RETIMED_UPDATE)
    if args.partition:
        print(json.dumps(partition_report(wl, args.partition)))
        return
    work = task_work(wl)
    weights = WL.init_weights(wl)
    dt, loss, prof, upd_params = run_workload(wl, args.steps, args.warmup, args.ra_streams if args.run_ahead else args.streams, not args.no_task_timing, weights, args.run_ahead, args.factor_ring)
    del weights
    retimed_here = RETIMED_UPDATE and wl.dtype == "bf16"
    ms_per_step = dt / args.steps * 1e3
    value = wl.batch * args.steps / dt

    def task_rates(prof, steps, upd_params, factor_ring, retimed=None):
        retimed = retimed_here if retimed is None else retimed
        out = {}
        for name in ("F", "dX", "dW"):
            ms, cnt = prof.get(name, (0.0, 0))
            if name == "dW" and factor_ring:
                # the G task only copies its factors; the product runs inside the update
                ums, ucnt = prof.get("update", (0.0, 0))
                if ucnt:
                    tf = work["dW"] * steps / (ums * 1e-3) / 1e12
                    out["update+dW"] = {"launches": ucnt, "avg_ms": ums / ucnt, "TFLOP/s": tf, "frac_of_bf16_peak": tf / PEAK_BF16_TFLOPS}
                continue
            if cnt:
                tf = work[name] * steps / (ms * 1e-3) / 1e12
                out[name] = {"launches": cnt, "avg_ms": ms / cnt, "TFLOP/s": tf, "frac_of_bf16_peak": tf / PEAK_BF16_TFLOPS}
                if name == "dW" and retimed:
                    out[name]["note"] = ("retimed update: the epilogue of this product applies Eq. 6 to the master weights and writes the next bf16 weight "
                                         "version (10 B per parameter on top of the product's operands); the flops counted are the product's alone")
        for name in ("hadamard", "loss"):
            ms, cnt = prof.get(name, (0.0, 0))
            if cnt and ms > 0:
                gbs = work[name] * steps / (ms * 1e-3) / 1e9
                out[name] = {"launches": cnt, "avg_ms": ms / cnt, "GB/s": gbs, "frac_of_hbm_peak": gbs / PEAK_HBM_GBS}
            elif name == "hadamard" and work[name] > 0:
                out[name] = {"launches": 0, "note": "applied in the epilogue of the dX products (its time is part of dX; --separate-hadamard times it alone)"}
        ms, cnt = prof.get("update", (0.0, 0))
        if cnt and ms > 0 and not factor_ring:
            gbs = upd_params * work["update_per_param"] / (ms * 1e-3) / 1e9
            out["update"] = {"launches": cnt, "avg_ms": ms / cnt, "GB/s": gbs, "frac_of_hbm_peak": gbs / PEAK_HBM_GBS}
            if retimed:
                out["update"]["note"] = "layers that keep a gradient ring (linear layers whose G product is split over K, convolutions whose G product is not); the others update inside dW"
        elif retimed and not factor_ring:
            out["update"] = {"launches": 0, "note": "applied in the epilogue of the dW products (its time is part of dW; --gradient-ring times it alone)"}
        return out

    tasks = task_rates(prof, args.steps, upd_params, args.factor_ring)
    # The same tasks with nothing running next to them (one stream, 4 steps): each kernel's own rate.  In the timed
    # region above dX and dW share the GPU and the updates run next to F, so those durations include the sharing.
    # On one stream the timed region is that measurement.
    tasks_alone = None
    if not args.run_ahead and args.streams == 1:
        tasks_alone = tasks
    elif not args.no_others and not args.run_ahead:
        _, _, prof1, upd1 = run_workload(wl, 4, args.warmup, 1, True, None, False, args.factor_ring)
        tasks_alone = task_rates(prof1, 4, upd1, args.factor_ring)
    # Eq. 6 as printed, for comparison: gradient rings and one delayed update task per layer on three streams
    ring_form = None
    if retimed_here and not args.no_others and not args.run_ahead:
        gdt, gloss, gprof, gupd = run_workload(wl, args.steps, args.warmup, 3, True, None, False, False, retimed=False)
        ring_form = {"streams": 3, "ms_per_step": gdt / args.steps * 1e3, "value": wl.batch * args.steps / gdt, "final_loss": gloss,
                     "updated_params_per_step": gupd / args.steps, "tasks": task_rates(gprof, args.steps, gupd, False, retimed=False)}
        # ... and its kernels' own rates (one stream, 4 steps): the stand-alone update kernel is the HBM-bound one
        _, _, gprof1, gupd1 = run_workload(wl, 4, args.warmup, 1, True, None, False, False, retimed=False)
        ring_form["tasks_one_stream"] = task_rates(gprof1, 4, gupd1, False, retimed=False)

    # dominant kernel: the bf16 MFMA GEMM of the forward products (same instantiation for all layers
    # of the default workload)
    roofline = None
    if "F" in tasks and wl.dtype == "bf16":
        flops_per_launch = work["F"] / wl.L
        avg_s = tasks["F"]["avg_ms"] * 1e-3
        ach = flops_per_launch / avg_s / 1e12
        kernel = F_KERNEL.get(wl.name)
        traffic = MEASURED_TRAFFIC.get((wl.name, kernel))
        roofline = {"bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS,
                    "traffic": traffic["bytes"] if traffic else None,
                    "traffic_source": traffic["profile"] if traffic else None,
                    "kernel": ("%s (forward product F)" % kernel if kernel
                               else "bf16 MFMA GEMM of the forward product F (tile and K split chosen per layer shape)"),
                    "flops_per_launch": flops_per_launch,
                    "avg_launch_ms": tasks["F"]["avg_ms"]}
        # context, measured now on this machine: the matrix instruction alone on random register operands (the chip lowers
        # its clock with the energy the work draws, so this, not the nominal peak, is what dense bf16 work can reach)
        if not args.no_others:
            roofline["mfma_only_TFLOP/s_on_random_operands"] = mfma_only(1, False, 4)[3]
            if wl.name == "ffn_stack_bf16":
                # ... and this very kernel, stand-alone, on the benchmark's operands and on operands that all hold one value
                # (same bytes, same schedule, fewer bits toggling): the gap is the clock the chip gives up to power
                f_up = operand_values(reps=10)[0]
                roofline["F_kernel_alone_frac_random_vs_uniform_operands"] = [f_up["random"]["frac_of_bf16_peak"], f_up["uniform"]["frac_of_bf16_peak"]]
    elif "F" in tasks:
        flops_per_launch = work["F"] / wl.L
        ach = flops_per_launch / (tasks["F"]["avg_ms"] * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": ach, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_FP32_MFMA_TFLOPS,
                    "traffic": None, "kernel": "gemm_f32_kernel (forward product F)", "flops_per_launch": flops_per_launch,
                    "avg_launch_ms": tasks["F"]["avg_ms"]}

    others = {}
    if not args.no_others:
        for name, mk in WL.CONFIGS.items():
            if name == wl.name:
                continue
            o = mk()
            try:
                o_streams = args.streams if streams_given else default_streams(o, RETIMED_UPDATE)
                odt, oloss, _, _ = run_workload(o, o.steps, 3, o_streams, False)
                others[name] = {"samples_per_s": o.batch * o.steps / odt, "ms_per_step": odt / o.steps * 1e3, "steps": o.steps,
                                "final_loss": oloss}
                if o.n_params < 5e8:
                    # steady state: every layer's delayed update is active (n > max d_l) in all timed steps
                    ydt, _, _, _ = run_workload(o, 100, max(o.delays) + 2, o_streams, False)
                    others[name]["steady_state_ms_per_step"] = ydt / 100 * 1e3
                if o.dtype == "bf16" and RETIMED_UPDATE and o.n_params < 5e8:
                    gdt, gloss, _, _ = run_workload(o, o.steps, 3, 3, False, retimed=False)
                    ydt, _, _, _ = run_workload(o, 100, max(o.delays) + 2, 3, False, retimed=False)
                    others[name]["gradient_ring"] = {"samples_per_s": o.batch * o.steps / gdt, "ms_per_step": gdt / o.steps * 1e3,
                                                     "steady_state_ms_per_step": ydt / 100 * 1e3, "final_loss": gloss}
                if o.n_params < 5e8:
                    # one stream: a third of the host's enqueue time (no cross-stream waits), best for launch-bound networks
                    sdt, sloss, _, _ = run_workload(o, o.steps, 3, 1, False)
                    others[name]["one_stream"] = {"samples_per_s": o.batch * o.steps / sdt, "ms_per_step": sdt / o.steps * 1e3,
                                                  "final_loss": sloss}
                if o.dtype == "bf16" and o.n_params < 5e8:
                    for label, kw in (("run_ahead", dict(run_ahead=True)), ("factor_ring", dict(factor_ring=True)),
                                      ("factor_ring+run_ahead", dict(run_ahead=True, factor_ring=True)),
                                      ("factor_ring+run_ahead_3_streams", dict(run_ahead=True, factor_ring=True, ns=3))):
                        ns = kw.pop("ns", args.ra_streams if "run_ahead" in kw else o_streams)
                        rdt, rloss, _, _ = run_workload(o, o.steps, 3, ns, False, **kw)
                        ydt, _, _, _ = run_workload(o, 100, max(o.delays) + 2, ns, False, **kw)
                        others[name][label] = {"samples_per_s": o.batch * o.steps / rdt, "ms_per_step": rdt / o.steps * 1e3,
                                               "steady_state_ms_per_step": ydt / 100 * 1e3, "final_loss": rloss}
            except Exception as e:  # a workload this build cannot run yet is reported, not hidden
                others[name] = {"error": str(e)[:200]}

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(wl)

    # Steady state of the headline workload: a layer is not updated while n <= d_l (Eq. 6 with empty delay elements),
    # so timed steps that start before step max d_l + 1 carry fewer updates.  When the requested warm-up is that short,
    # the same number of steps is timed once more behind a warm-up of max d_l + 1 steps.
    d_max = max(wl.delays)
    full_steps = sum(1 for n in range(args.warmup + 1, args.warmup + args.steps + 1) if n > d_max)
    if upd_params == wl.n_params * args.steps:
        full_steps = args.steps    # every layer has the retimed update: its G task applies a gradient in every step, from the first
    steady = None
    if full_steps < args.steps and not args.run_ahead:
        sdt, _, _, supd = run_workload(wl, args.steps, d_max + 1, args.streams, False, None, False, args.factor_ring)
        steady = {"warmup": d_max + 1, "steps": args.steps, "ms_per_step": sdt / args.steps * 1e3, "value": wl.batch * args.steps / sdt,
                  "unit": "samples/s", "updated_params_per_step": supd / args.steps}

    out = {
        "metric": "training samples/sec (1 GPU)", "value": value, "unit": "samples/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": "%s: %d layers, batch %d, delays %s, %s loss, lr %g, %d stream%s; %d of the %d timed steps update every layer%s" % (
            wl.name, wl.L, wl.batch, list(wl.delays), wl.loss, wl.lr, args.ra_streams if args.run_ahead else args.streams,
            "" if (args.ra_streams if args.run_ahead else args.streams) == 1 else "s",
            full_steps, args.steps, "" if retimed_here else " (step number > max delay %d)" % d_max) + (
                ", forward run-ahead" if args.run_ahead else "") + (", factor ring" if args.factor_ring else "") + (
                ", Hadamard products as separate kernels" if args.separate_hadamard else "") + (
                ", retimed update (Eq. 6 with its delays on the weights: weight versions in place of gradient rings, the dW launches apply the updates; "
                "same losses bit for bit, see gradient_ring)" if retimed_here else ", gradient rings"),
            "params": wl.n_params, "flops_per_step": sum(wl.flops_per_step()),
            "updated_params_per_step": upd_params / args.steps},
        "steady_state": steady,
        "roofline": roofline, "cpu_baseline": cpu, "tasks": tasks, "tasks_one_stream": tasks_alone, "gradient_ring": ring_form,
        "other_workloads": others,
        "final_loss": loss,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
