"""Algorithm 1 (balanced pipeline partitioning): the oracle against the paper's worked example
(Table II -> Table III), and the library's host-side lp_partition against the oracle."""
import ctypes as C
import os
import random

import pytest

from oracle import partition_oracle as P
import paper_2108_06629_amd as lp

HERE = os.path.dirname(os.path.abspath(__file__))


def golden():
    layers, procs, pd, imp = [], [], None, None
    for ln in open(os.path.join(HERE, "golden", "sample_network_partition.txt")):
        t = ln.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "layer":
            layers.append(tuple(float(v) for v in t[2:]))
        elif t[0] == "proc":
            procs.append(tuple(float(v) for v in t[2:]))
        elif t[0] == "pipedream":
            pd = [float(v) for v in t[1:]]
        elif t[0] == "improvement_percent":
            imp = float(t[1])
    return layers, procs, pd, imp


def close(a, b, rel=0.011):      # the tables print three significant digits
    return abs(a - b) <= rel * max(abs(a), abs(b), 1.0)


def test_oracle_reproduces_table_iii():
    layers, procs, pd, imp = golden()
    t_fix = [fp + g for fp, g, d in layers]          # forward + weight gradient: immovable
    t_flex = [d for fp, g, d in layers]              # delta: movable to the next layer's processor
    r = P.partition(t_fix, t_flex, 3)
    assert r["stage_fix"] == [0, 1, 2, 2]            # layers 1 | 2 | 3+4, as in the paper's Sec. IV-B
    assert r["stage_delta_rest"] == [0, 1, 2, 2]
    for s, (assigned, borrowed, total) in enumerate(procs):
        assert close(r["stage_time"][s], total), (s, r["stage_time"][s], total)
    # borrowed computation: processor 2 borrows from layer 1, processor 3 from layer 2
    assert close(r["borrowed_frac"][0] * t_flex[0], procs[1][1])
    assert close(r["borrowed_frac"][1] * t_flex[1], procs[2][1])
    assert r["borrowed_frac"][2] == 0.0 and r["borrowed_frac"][3] == 0.0     # layers 3 and 4 share a processor; nothing after layer 4
    # assigned = own delta' + own fixed part (+ whole layers)
    own = [t_fix[0] + (1 - r["borrowed_frac"][0]) * t_flex[0], t_fix[1] + (1 - r["borrowed_frac"][1]) * t_flex[1],
           t_fix[2] + t_flex[2] + t_fix[3] + t_flex[3]]
    for s in range(3):
        assert close(own[s], procs[s][0]), (s, own[s], procs[s][0])
    # PipeDream's whole-layer assignment and the quoted improvement of the bottleneck stage
    tot = [a + b for a, b in zip(t_fix, t_flex)]
    stages = P.pipedream_like(tot, [1, 2])
    for got, want in zip(stages, pd):
        assert close(got, want)
    assert abs((1 - max(r["stage_time"]) / max(stages)) * 100 - imp) < 1.0


def test_oracle_invariants_on_random_inputs():
    rng = random.Random(3)
    for trial in range(300):
        L = rng.randint(1, 12)
        n_proc = rng.randint(1, 8)
        t_fix = [rng.uniform(0.1, 5.0) for _ in range(L)]
        t_flex = [rng.uniform(0.0, 20.0) for _ in range(L)]
        r = P.partition(t_fix, t_flex, n_proc, alpha=1.05)
        assert abs(sum(r["stage_time"]) - (sum(t_fix) + sum(t_flex))) < 1e-9 * (sum(t_fix) + sum(t_flex))      # nothing lost
        st, dr = r["stage_fix"], r["stage_delta_rest"]
        assert all(0 <= s < n_proc for s in st) and all(a <= b for a, b in zip(st, st[1:]))                  # contiguous, ordered stages
        assert all(0.0 <= f <= 1.0 for f in r["borrowed_frac"]) and r["borrowed_frac"][-1] == 0.0
        for l in range(L):
            assert st[l] <= dr[l] <= (st[l + 1] if l < L - 1 else n_proc - 1)     # delta' sits between its layer and the borrower
            if r["borrowed_frac"][l] > 0:
                assert st[l + 1] > st[l]                                          # only another (the next layer's) processor borrows
        assert r["t_p"] >= (sum(t_fix) + sum(t_flex)) / n_proc - 1e-12
    one = P.partition([1.0, 2.0, 3.0], [4.0, 5.0, 6.0], 1)
    assert one["stage_fix"] == [0, 0, 0] and abs(one["stage_time"][0] - 21.0) < 1e-12 and one["borrowed_frac"] == [0.0, 0.0, 0.0]


def lib_partition(t_fix, t_flex, n_proc, alpha):
    L = len(t_fix)
    arr = C.c_double * L
    st, dr, bf, tt, tp = (C.c_int * L)(), (C.c_int * L)(), arr(), (C.c_double * n_proc)(), C.c_double()
    rc = lp.lib().lp_partition(arr(*t_fix), arr(*t_flex), L, n_proc, alpha, st, dr, bf, tt, C.byref(tp))
    assert rc == 0
    return dict(stage_fix=list(st), stage_delta_rest=list(dr), borrowed_frac=list(bf), stage_time=list(tt), t_p=tp.value)


def test_library_partition_matches_oracle_and_table_iii():
    layers, procs, pd, imp = golden()
    t_fix = [fp + g for fp, g, d in layers]
    t_flex = [d for fp, g, d in layers]
    got = lib_partition(t_fix, t_flex, 3, 1.01)
    want = P.partition(t_fix, t_flex, 3, 1.01)
    assert got["stage_fix"] == want["stage_fix"] == [0, 1, 2, 2] and got["stage_delta_rest"] == want["stage_delta_rest"]
    for k in ("borrowed_frac", "stage_time"):
        assert all(abs(a - b) <= 1e-12 * max(1.0, abs(b)) for a, b in zip(got[k], want[k])), k
    rng = random.Random(5)
    for trial in range(300):
        L, n_proc = rng.randint(1, 16), rng.randint(1, 9)
        t_fix = [rng.uniform(0.1, 5.0) for _ in range(L)]
        t_flex = [rng.uniform(0.0, 20.0) for _ in range(L)]
        got, want = lib_partition(t_fix, t_flex, n_proc, 1.05), P.partition(t_fix, t_flex, n_proc, 1.05)
        assert got["stage_fix"] == want["stage_fix"] and got["stage_delta_rest"] == want["stage_delta_rest"], trial
        assert abs(got["t_p"] - want["t_p"]) <= 1e-12 * want["t_p"]
        for k in ("borrowed_frac", "stage_time"):
            assert all(abs(a - b) <= 1e-9 * max(1.0, abs(b)) for a, b in zip(got[k], want[k])), (trial, k)


# ------------------------------------------------------------------------------------------------
# brute force, written from the text of Sec. III-C rather than from the listing's arithmetic
# ------------------------------------------------------------------------------------------------
def unit_walk(t_fix, t_flex, n_proc, cap):
    """All times are whole numbers of unit jobs.  Processors are filled one after the other, last layer first, each up
    to `cap` units.  A layer's delta task is a pile of independent unit jobs (the delta computation is parallel over
    channels): each unit goes to the processor being filled; the first unit that finds it full opens the next
    processor, and the rest of the pile follows it there (the task is cut once, into delta'' and delta').  The fixed
    part of a layer is one indivisible job: it opens a fresh processor unless all of it fits.  Returns None if that
    takes more than n_proc processors, else (processor of each fixed part, units of each delta task per processor,
    load per processor), processors numbered from the back of the network."""
    L = len(t_fix)
    load = [0]
    fix_on = [None] * L
    flex_on = [dict() for _ in range(L)]
    for l in reversed(range(L)):
        cut = False
        for _ in range(t_flex[l]):
            if not cut and load[-1] + 1 > cap:
                load.append(0)
                cut = True
            load[-1] += 1
            flex_on[l][len(load) - 1] = flex_on[l].get(len(load) - 1, 0) + 1
        if load[-1] + t_fix[l] > cap:
            load.append(0)
        load[-1] += t_fix[l]
        fix_on[l] = len(load) - 1
    return None if len(load) > n_proc else (fix_on, flex_on, load)


def brute_force_partition(t_fix, t_flex, n_proc, alpha):
    cap = (sum(t_fix) + sum(t_flex)) // n_proc
    while True:
        r = unit_walk(t_fix, t_flex, n_proc, cap)
        if r is not None:
            return cap, r
        cap *= alpha


@pytest.mark.parametrize("which", ["oracle", "library"])
def test_partition_against_unit_by_unit_brute_force(which):
    """Whole-number task times, a total divisible by N_p and alpha = 2 keep the target load a whole number, so the
    unit-by-unit walk and Algorithm 1 must agree exactly: stage of every fixed part, units of every delta task that
    the next layer's stage borrows, load of every stage.  Delta tasks no longer than the first target load: a pile
    longer than a whole processor is outside what the text describes (the listing would overfill one processor)."""
    rng = random.Random(11)
    done = 0
    while done < 400:
        L, n_proc = rng.randint(1, 5), rng.randint(1, 4)
        t_fix = [rng.randint(0, 12) for _ in range(L)]
        t_flex = [rng.randint(0, 30) for _ in range(L)]
        tot = sum(t_fix) + sum(t_flex)
        t_fix[0] += (-tot) % n_proc                      # total divisible by N_p
        tot = sum(t_fix) + sum(t_flex)
        if tot == 0 or max(t_flex) > tot // n_proc:
            continue
        done += 1
        cap, (fix_on, flex_on, load) = brute_force_partition(t_fix, t_flex, n_proc, 2)
        used = len(load)
        f = [float(v) for v in t_fix], [float(v) for v in t_flex]
        got = P.partition(f[0], f[1], n_proc, 2.0) if which == "oracle" else lib_partition(f[0], f[1], n_proc, 2.0)
        case = (t_fix, t_flex, n_proc)
        assert got["t_p"] == cap, case
        assert got["stage_fix"] == [used - 1 - q for q in fix_on], case
        assert got["stage_time"] == [float(v) for v in reversed(load)] + [0.0] * (n_proc - used), case
        for l in range(L):
            # units of layer l's delta task that run on the stage of layer l+1's fixed part while layer l's own fixed part
            # sits elsewhere = the borrowed part (delta'')
            borrowed = 0
            if l < L - 1 and fix_on[l + 1] != fix_on[l]:
                borrowed = flex_on[l].get(fix_on[l + 1], 0)
            assert abs(got["borrowed_frac"][l] * t_flex[l] - borrowed) < 1e-9, (case, l)
            rest = [q for q in flex_on[l] if not (l < L - 1 and q == fix_on[l + 1] and fix_on[l + 1] != fix_on[l])]
            if t_flex[l] > 0 and rest:
                assert got["stage_delta_rest"][l] == used - 1 - max(rest), (case, l)


def test_library_partition_rejects_bad_arguments():
    L = lp.lib()
    one = (C.c_double * 1)(1.0)
    st, dr, bf, tt, tp = (C.c_int * 1)(), (C.c_int * 1)(), (C.c_double * 1)(), (C.c_double * 1)(), C.c_double()
    assert L.lp_partition(None, one, 1, 1, 1.05, st, dr, bf, tt, C.byref(tp)) == 1
    assert L.lp_partition(one, one, 0, 1, 1.05, st, dr, bf, tt, C.byref(tp)) == 2
    assert L.lp_partition(one, one, 1, 0, 1.05, st, dr, bf, tt, C.byref(tp)) == 2
    assert L.lp_partition(one, one, 1, 1, 1.0, st, dr, bf, tt, C.byref(tp)) == 2
    neg = (C.c_double * 1)(-1.0)
    assert L.lp_partition(neg, one, 1, 1, 1.05, st, dr, bf, tt, C.byref(tp)) == 2
