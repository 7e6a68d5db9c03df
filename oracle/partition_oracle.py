"""CPU oracle of the balanced-pipeline partitioner (Algorithm 1, Sec. III-C).  TEST INFRASTRUCTURE ONLY.

Inputs: per-layer fixed time T_fix[l] (forward + weight-gradient task, immovable) and flexible time
T_flex[l] (the delta task, which only the processor of layer l+1 may borrow), the number of
processors N_p and the relaxation factor alpha.  The walk goes over the layers in reverse, filling
one processor after the other up to the target T_p = T_tot / N_p; a delta task that does not fit the
room left in the current processor is cut into delta'' (fills that room, stays with layer l+1's
processor) and delta' (goes to the next processor, together with layer l's fixed part).  If more
processors are needed than exist, T_p is multiplied by alpha and the walk restarts.

Readings where the printed algorithm is ambiguous (also listed in the design notes):
  * when the fixed part does not fit and moves to the next processor, that processor starts empty
    (its room is T_p), although the listing does not reset the room explicitly;
  * processors are counted from the back of the network during the walk and renumbered at the end so
    that stage 0 holds the first layers, as in Table III;
  * "more processors than available" means the walk opened more than N_p processors;
  * comparisons use a relative slack of 1e-9 so that a part that fits exactly (as the last fixed
    part of the paper's own example does, to the table's rounding) is not pushed out by rounding.

Pinned by the paper's worked example (Table II -> Table III) in tests/test_partition.py.
"""
from __future__ import annotations


def partition(t_fix, t_flex, n_proc, alpha=1.01, max_rounds=100000):
    """Returns dict(t_p, stage_fix, stage_delta_rest, borrowed_frac, stage_time, rounds).

    stage_fix[l]         stage that holds layer l's fixed part (forward + weight gradient)
    borrowed_frac[l]     fraction of layer l's delta task that stays with the stage of layer l+1 (delta'');
                         0 for the last layer and whenever layers l and l+1 share a stage
    stage_delta_rest[l]  stage that runs the rest of layer l's delta task (delta')
    stage_time[s]        total time assigned to stage s
    """
    L = len(t_fix)
    assert L == len(t_flex) and L >= 1 and n_proc >= 1 and alpha > 1.0
    t_tot = sum(t_fix) + sum(t_flex)
    t_p = t_tot / n_proc
    eps = 1e-9
    for rounds in range(1, max_rounds + 1):
        p = 0
        idle = t_p
        proc_fix = [0] * L
        proc_first = [0] * L      # processor that receives the first (or only) part of the delta task
        proc_rest = [0] * L       # processor that receives delta'
        first_frac = [1.0] * L
        load = [0.0]
        for l in range(L - 1, -1, -1):
            flex = t_flex[l]
            proc_first[l] = p
            if flex <= idle * (1 + eps):
                load[p] += flex                  # the whole delta task fits in the room that is left
                idle -= flex
                proc_rest[l] = p
            else:
                d2 = max(idle, 0.0)              # delta'': what still fits
                d1 = flex - d2                   # delta': the rest moves on
                load[p] += d2
                first_frac[l] = d2 / flex
                p += 1
                load.append(d1)
                idle = t_p - d1
                proc_rest[l] = p
            if t_fix[l] > idle * (1 + eps) + eps * t_p:
                p += 1
                load.append(0.0)
                idle = t_p
            load[p] += t_fix[l]
            idle -= t_fix[l]
            proc_fix[l] = p
        if p + 1 > n_proc:
            t_p *= alpha
            continue
        used = p + 1
        stage = lambda q: used - 1 - q
        borrowed, rest = [0.0] * L, [0] * L
        for l in range(L):
            rest[l] = stage(proc_rest[l])
            if l < L - 1 and proc_first[l] == proc_fix[l + 1] and proc_fix[l + 1] != proc_fix[l] and t_flex[l] > 0:
                borrowed[l] = first_frac[l]
        return dict(t_p=t_p, stage_fix=[stage(q) for q in proc_fix], stage_delta_rest=rest, borrowed_frac=borrowed,
                    stage_time=list(reversed(load)) + [0.0] * (n_proc - used), rounds=rounds)
    raise RuntimeError("partition did not converge")


def pipedream_like(t_total_per_layer, cuts):
    """Per-stage time when whole layers are assigned to stages; cuts = index of the first layer of every stage but the first."""
    bounds = [0] + list(cuts) + [len(t_total_per_layer)]
    return [sum(t_total_per_layer[a:b]) for a, b in zip(bounds[:-1], bounds[1:])]
