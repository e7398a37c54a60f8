"""Plain-Python checker of a swap plan (TEST INFRASTRUCTURE, like the rest of oracle/).

It takes what the library exports about a plan - the tensor table, the per-step read and
write lists (the global memory-object access pattern of Sec. 3.2) and the instruction list
for the three streams of Sec. 5 - and re-derives from the paper's definitions, with no code
shared with the planner:

  * the memory model, Eq. 4: at every instant the bytes allocated minus the bytes released
    stay within the budget, and no two live objects overlap;
  * that every step finds its data on the GPU (what t_ready of Algorithm 1 stands for),
    that a block is only written again after the last use of its previous content has
    finished (a happens-before relation over streams and events), and that what an offload
    wrote to the host is what the matching prefetch reads;
  * the timing recurrences of the three streams (Algorithm 1 with releases made explicit):
    an instruction starts when its stream is free and everything it waits for has ended;
    t_ready[j] is the latest end among the things step j waits for; Eq. 6 holds for step j
    iff t_ready[j] <= end of step j-1.
"""
from typing import Dict, List

LOAD, COMPUTE, OFFLOAD, PREFETCH = 0, 1, 2, 3
S_COMPUTE, S_OUT, S_IN = 0, 1, 2
STREAM_OF = {LOAD: S_IN, COMPUTE: S_COMPUTE, OFFLOAD: S_OUT, PREFETCH: S_IN}


class PlanError(AssertionError):
    pass


def gather(ctx) -> dict:
    """Everything the checker needs, read through the C ABI."""
    nt, ns = ctx.tensor_count(), ctx.step_count()
    return dict(tensors=[ctx.tensor_info(t) for t in range(nt)],
                steps=[ctx.step_info(j) for j in range(ns)],
                io=[ctx.step_io(j) for j in range(ns)],
                instrs=ctx.instructions())


def _overlap(a0, a1, b0, b1):
    return a0 < b1 and b0 < a1


def check_plan(plan: dict, budget: int, static_bytes: int) -> dict:
    """Raises PlanError on the first violation; returns summary figures."""
    T, io, instrs = plan["tensors"], plan["io"], plan["instrs"]
    ns = len(plan["steps"])
    # position of every instruction on its own stream
    pos = []
    counters = [0, 0, 0]
    for ins in instrs:
        s = STREAM_OF[ins["op"]]
        counters[s] += 1
        pos.append(counters[s])
    # vector clocks: clock[s][t] = how far stream s is known to be behind stream t
    clock = [[0, 0, 0] for _ in range(3)]
    ev_step: Dict[int, List[int]] = {}
    ev_d2h: Dict[int, List[int]] = {}
    ev_h2d: Dict[int, List[int]] = {}

    where = {}            # tensor -> current device range (lo, hi)
    owner = []            # list of (lo, hi, tensor): who owns which device bytes now
    host_owner = []       # same for the pinned arena
    accesses = []         # (lo, hi, is_write, stream, stream_pos, what)
    loaded = set()        # tensors that went through offload
    peak, live = 0, 0
    live_ranges = {}      # tensor -> (lo, hi) while it is alive (for Eq. 4)
    steps_seen = 0
    n_swapped = 0

    def ordered_before(acc, s_now):
        _, _, _, s_then, p_then, _ = acc
        return s_then == s_now or clock[s_now][s_then] >= p_then

    def touch(lo, hi, is_write, s, p, what):
        if lo < static_bytes or hi > budget:
            raise PlanError(f"{what}: bytes [{lo},{hi}) outside the dynamic part of the budget")
        for acc in accesses:
            if _overlap(lo, hi, acc[0], acc[1]) and (is_write or acc[2]) and not ordered_before(acc, s):
                raise PlanError(f"{what}: races with {acc[5]} on [{max(lo, acc[0])},{min(hi, acc[1])})")
        accesses.append((lo, hi, is_write, s, p, what))

    def claim(lo, hi, t):
        owner[:] = [o for o in owner if not _overlap(lo, hi, o[0], o[1]) or o[2] == t]
        owner.append((lo, hi, t))

    def owns(lo, hi, t):
        return any(o[2] == t and o[0] <= lo and hi <= o[1] for o in owner)

    def begin_life(t, lo, hi):
        nonlocal live, peak
        for u, (a, b) in live_ranges.items():
            if u != t and _overlap(lo, hi, a, b):
                raise PlanError(f"tensor {t} placed over live tensor {u}")
        live_ranges[t] = (lo, hi)
        live += hi - lo
        peak = max(peak, live)

    def end_life(t):
        nonlocal live
        if t in live_ranges:
            lo, hi = live_ranges.pop(t)
            live -= hi - lo

    for idx, ins in enumerate(instrs):
        op, arg = ins["op"], ins["arg"]
        s, p = STREAM_OF[op], pos[idx]
        # waits merge the clocks of what is waited for
        for key, table in (("wait_step", ev_step), ("wait_d2h", ev_d2h), ("wait_h2d", ev_h2d)):
            w = ins[key]
            if w >= 0:
                if w not in table:
                    raise PlanError(f"instruction {idx} waits for an event that was never recorded ({key}={w})")
                clock[s] = [max(a, b) for a, b in zip(clock[s], table[w])]
        clock[s][s] = p
        if op == LOAD:
            t = T[arg]
            lo, hi = t["offset"], t["offset"] + t["bytes"]
            begin_life(arg, lo, hi)
            touch(lo, hi, True, s, p, f"load of tensor {arg}")
            claim(lo, hi, arg)
            where[arg] = (lo, hi)
            ev_h2d[ins["seq"]] = list(clock[s])
        elif op == COMPUTE:
            if arg != steps_seen:
                raise PlanError(f"compute steps out of order: {arg} after {steps_seen - 1}")
            steps_seen += 1
            reads, writes = io[arg]
            for t in writes:
                if t not in where:
                    lo, hi = T[t]["offset"], T[t]["offset"] + T[t]["bytes"]
                    begin_life(t, lo, hi)
                    where[t] = (lo, hi)
            for t in reads:
                if t not in where:
                    raise PlanError(f"step {arg} reads tensor {t}, which is not on the GPU")
                lo, hi = where[t]
                if not owns(lo, hi, t):
                    raise PlanError(f"step {arg} reads tensor {t}, whose bytes were overwritten")
                touch(lo, hi, False, s, p, f"step {arg} reading tensor {t}")
            for t in writes:
                lo, hi = where[t]
                touch(lo, hi, True, s, p, f"step {arg} writing tensor {t}")
                claim(lo, hi, t)
            if ins["record"]:
                ev_step[arg] = list(clock[s])
            # release: objects whose last use this was
            for t in set(reads) | set(writes):
                if T[t]["last_step"] == arg and t in where:
                    del where[t]
                    end_life(t)
        elif op == OFFLOAD:
            t = T[arg]
            if arg not in where:
                raise PlanError(f"offload of tensor {arg}, which is not on the GPU")
            if not t["swapped"] or ins["wait_step"] < t["last_fwd_step"]:
                raise PlanError(f"offload of tensor {arg} does not wait for its last forward use")
            lo, hi = where[arg]
            if not owns(lo, hi, arg):
                raise PlanError(f"offload of tensor {arg}, whose bytes were overwritten")
            touch(lo, hi, False, s, p, f"offload of tensor {arg}")
            h0, h1 = t["host_offset"], t["host_offset"] + t["bytes"]
            for o in host_owner:
                if _overlap(h0, h1, o[0], o[1]):
                    raise PlanError(f"host slot of tensor {arg} overlaps that of tensor {o[2]}")
            host_owner.append((h0, h1, arg))
            ev_d2h[ins["seq"]] = list(clock[s])
            del where[arg]
            end_life(arg)
            loaded.add(arg)
            n_swapped += 1
        elif op == PREFETCH:
            t = T[arg]
            if arg not in loaded:
                raise PlanError(f"prefetch of tensor {arg} before its offload")
            # the host copy must be complete: the prefetch has to be ordered after the offload
            off_acc = [a for a in accesses if a[5] == f"offload of tensor {arg}"][0]
            if not ordered_before(off_acc, s):
                raise PlanError(f"prefetch of tensor {arg} is not ordered after its offload")
            lo, hi = t["offset2"], t["offset2"] + t["bytes"]
            begin_life(arg, lo, hi)
            touch(lo, hi, True, s, p, f"prefetch of tensor {arg}")
            claim(lo, hi, arg)
            where[arg] = (lo, hi)
            ev_h2d[ins["seq"]] = list(clock[s])
        else:
            raise PlanError(f"unknown op {op}")
    if steps_seen != ns:
        raise PlanError(f"{steps_seen} of {ns} steps in the instruction list")
    if where:
        raise PlanError(f"tensors never released: {sorted(where)}")
    return dict(peak_dynamic_bytes=peak, n_swapped=n_swapped)


def replay_times(plan: dict, step_seconds: List[float], d2h_bps: float, h2d_bps: float,
                 copy_latency_s: float) -> dict:
    """Three-stream timing: start = max(stream free, ends of everything waited for)."""
    T, instrs = plan["tensors"], plan["instrs"]
    ns = len(plan["steps"])
    free = [0.0, 0.0, 0.0]
    end_step = [0.0] * ns
    start_step = [0.0] * ns
    t_ready = [0.0] * ns
    end_d2h, end_h2d = {}, {}
    floor = [0.0, 0.0, 0.0]          # a stream never runs before something it has waited for
    for ins in instrs:
        op, arg = ins["op"], ins["arg"]
        s = STREAM_OF[op]
        if ins["wait_step"] >= 0:
            floor[s] = max(floor[s], end_step[ins["wait_step"]])
        if ins["wait_d2h"] >= 0:
            floor[s] = max(floor[s], end_d2h[ins["wait_d2h"]])
        if ins["wait_h2d"] >= 0:
            floor[s] = max(floor[s], end_h2d[ins["wait_h2d"]])
        start = max(free[s], floor[s])
        if op == COMPUTE:
            t_ready[arg] = floor[s]
            start_step[arg] = start
            end = start + step_seconds[arg]
            end_step[arg] = end
        elif op == OFFLOAD:
            end = start + copy_latency_s + T[arg]["bytes"] / d2h_bps
            end_d2h[ins["seq"]] = end
        else:
            end = start + copy_latency_s + T[arg]["bytes"] / h2d_bps
            end_h2d[ins["seq"]] = end
        free[s] = end
    stall = sum(max(0.0, start_step[j] - (end_step[j - 1] if j else 0.0)) for j in range(ns))
    no_stall = all(t_ready[j] <= (end_step[j - 1] if j else 0.0) + 1e-12 for j in range(ns))
    return dict(t_ready=t_ready, t_start=start_step, t_end=end_step, t_iter=max(free), t_stall=stall,
                eq6_holds=no_stall)
