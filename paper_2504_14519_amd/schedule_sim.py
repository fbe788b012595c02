"""Slice-wise 1F1B pipeline schedule of the paper (Sec. 4.1.2, Fig. slim_schedule) as a host-side discrete
simulation: per-device pass order, a timeline under given per-slice forward/backward times (measured
kernel times can be fed in), accumulated activation in slices, bubble fraction, and the effect of the
attention context exchange (Sec. 4.2) on the imbalance bubbles.  Plain Python, no GPU work; the
non-interleaved form (one stage per device) only.

Notation of the paper: p pipeline devices, n slices per sequence, m microbatches.  Slices and
microbatches are 0-based here."""
from .planner import redistribute_pairwise, redistribute_balanced


def device_order(p, n, m, rank):
    """Pass order on device `rank` (0 = first stage): [('F'|'B', microbatch, slice)].

    Forward passes go in sequence order; the backward passes of one microbatch go in reverse slice order
    (last in, first out, so the newest part of the key-value cache is released first).  Device `rank`
    runs n + 2(p-1-rank) forward passes before its first backward pass -- the extra forward passes that
    the paper puts ahead so that forward meets forward and backward meets backward across devices --
    then alternates one backward, one forward."""
    total = n * m
    fwd = [("F", f // n, f % n) for f in range(total)]
    bwd = [("B", b // n, n - 1 - b % n) for b in range(total)]
    warm = min(total, n + 2 * (p - 1 - rank))
    order = fwd[:warm]
    fi, bi = warm, 0
    while bi < total:
        order.append(bwd[bi]); bi += 1
        if fi < total:
            order.append(fwd[fi]); fi += 1
    return order


def accumulated_slices(p, n, m, rank):
    """Largest number of slices whose activations device `rank` holds at once (forward done, backward not
    yet finished), counted over its pass order."""
    live = peak = 0
    for kind, _, _ in device_order(p, n, m, rank):
        if kind == "F":
            live += 1
            peak = max(peak, live)
        else:
            live -= 1          # released when the backward pass has finished
    return peak


def accumulated_fraction(p, n, m=None, rank=0):
    """Accumulated activation of device `rank` as a fraction of M_a, the activation of one whole microbatch
    over all stages: a slice on one of p stages holds M_a / (n p).  With enough microbatches this is
    (1 + 2(p-1)/n) / p on the first device (Sec. 4.1.3, Eq. 1)."""
    if m is None:
        m = 2 * p
    return accumulated_slices(p, n, m, rank) / float(n * p)


def exchange_groups(p, n, m):
    """Which passes run at the same moment in the aligned schedule: forward pass number f (= microbatch*n +
    slice) on device r meets forward pass f-1 on device r+1, backward pass number b on device r meets b+1 on
    r+1.  -> {('F', f + r) | ('B', b + p-1-r): [(rank, microbatch, slice)]}.  Within a group the slice
    indices form the arithmetic progression of Sec. 4.2.1 (broken at the juncture of two microbatches)."""
    groups = {}
    total = n * m
    for r in range(p):
        for f in range(total):
            groups.setdefault(("F", f + r), []).append((r, f // n, f % n))
        for b in range(total):
            groups.setdefault(("B", b + (p - 1 - r)), []).append((r, b // n, n - 1 - b % n))
    return groups


def exchanged_loads(p, n, m, mode="pairwise"):
    """{(kind, rank, microbatch, slice): key-value slices that device computes after the context exchange}.
    Before the exchange the load of a pass is slice + 1.  mode: 'pairwise' and 'balanced' move whole
    key-value slices as the planner decides; 'ideal' gives every device of a group the group's mean (a
    fractional load: the limit of ever finer pieces)."""
    plan = {"pairwise": redistribute_pairwise, "balanced": redistribute_balanced, "ideal": None}[mode]
    out = {}
    for (kind, _), members in exchange_groups(p, n, m).items():
        before = [i + 1 for _, _, i in members]
        after = plan(before)[1] if plan else [sum(before) / float(len(before))] * len(before)
        for (r, k, i), load in zip(members, after):
            out[(kind, r, k, i)] = load
    return out


def pass_time(table, load):
    """Time of a pass over `load` key-value slices from table[L-1] (L = 1..n), linear between whole slices."""
    lo = int(load)
    if lo == load:
        return table[lo - 1]
    return table[lo - 1] + (load - lo) * (table[lo] - table[lo - 1])


def simulate(p, n, m, t_fwd, t_bwd, exchange=None, t_other_fwd=0.0, t_other_bwd=0.0, t_send=0.0):
    """Run the schedule.  t_fwd[L-1], t_bwd[L-1]: time of the attention forward / backward pass of one slice
    that attends to L key-value slices (L = 1..n; for slice i without exchange L = i + 1); t_other_*: the
    part of a pass that does not depend on the slice index (linear layers); t_send: stage-to-stage latency.
    exchange: None, 'pairwise', 'balanced' or 'ideal' -- the passes that run at the same moment share
    their attention work (see exchanged_loads) and each costs the time of its load after the exchange.
    Devices that have no pass of that kind at that moment (warm-up, cool-down) do not help.

    A forward pass starts when the device is free and the previous stage has finished the same slice; a
    backward pass when the next stage has finished the backward of the same slice.

    -> dict(makespan, busy[rank], bubble_fraction, timeline[rank] = [(kind, k, i, start, end)],
            peak_slices[rank]).  bubble_fraction = (makespan - ideal) / ideal with ideal = all work spread evenly
    over the p devices, the definition under which default 1F1B has (p-1)/m."""
    loads = exchanged_loads(p, n, m, exchange) if exchange else None
    orders = [device_order(p, n, m, r) for r in range(p)]
    pos = [0] * p
    free = [0.0] * p
    done = {}
    timeline = [[] for _ in range(p)]
    remaining = sum(len(o) for o in orders)
    while remaining:
        progressed = False
        for r in range(p):
            while pos[r] < len(orders[r]):
                kind, k, i = orders[r][pos[r]]
                if kind == "F":
                    dep = ("F", r - 1, k, i) if r > 0 else None
                else:
                    dep = ("B", r + 1, k, i) if r < p - 1 else ("F", r, k, i)
                if dep is not None and dep not in done:
                    break
                ready = done[dep] + (t_send if dep is not None and dep[1] != r else 0.0) if dep is not None else 0.0
                load = loads[(kind, r, k, i)] if loads else i + 1
                dur = (pass_time(t_fwd, load) + t_other_fwd) if kind == "F" else (pass_time(t_bwd, load) + t_other_bwd)
                start = max(free[r], ready)
                end = start + dur
                free[r] = end
                done[(kind, r, k, i)] = end
                timeline[r].append((kind, k, i, start, end))
                pos[r] += 1
                remaining -= 1
                progressed = True
        if not progressed:
            raise RuntimeError("schedule deadlock: p=%d n=%d m=%d" % (p, n, m))
    makespan = max(free)
    busy = [sum(e - s for _, _, _, s, e in tl) for tl in timeline]
    ideal = sum(busy) / p
    return dict(makespan=makespan, busy=busy, bubble_fraction=(makespan - ideal) / ideal, timeline=timeline,
                peak_slices=[accumulated_slices(p, n, m, r) for r in range(p)])


def simulate_lockstep(p, n, m, t_fwd, t_bwd, exchange=None, partial_columns=False, t_other_fwd=0.0, t_other_bwd=0.0):
    """The schedule as the paper draws it: passes that stand in one column (exchange_groups) start together and
    the column lasts as long as its slowest pass.  This is the model behind the closed forms of Sec. 4.1.3: a
    device's bubble is the sum of the columns in which it has no pass (p-1 forward columns and p-1 backward
    columns), plus what it waits inside the columns it shares.

    exchange: None, or 'pairwise' / 'balanced' / 'ideal' as in `simulate`; it is applied to the columns in which
    all p devices have a pass (the situation of the paper's picture) and, with partial_columns, also among the
    devices of the incomplete columns of the warm-up and cool-down.  With pass time proportional to the load
    the paper's long-context bubble figure (p-1)p/((n+1)nm) lies between the last device's bubble in the two
    variants: it charges the columns the last device is absent from at their heaviest pass, and nothing for the
    incomplete columns it takes part in.

    -> dict(makespan, busy[rank], bubble[rank], ideal, bubble_fraction[rank]) with ideal = all work spread evenly
    over the p devices and bubble_fraction = bubble / ideal."""
    plan = {None: None, "pairwise": redistribute_pairwise, "balanced": redistribute_balanced, "ideal": "ideal"}[exchange]
    busy = [0.0] * p
    makespan = 0.0
    for (kind, _), members in exchange_groups(p, n, m).items():
        loads = [i + 1 for _, _, i in members]
        if plan is not None and (len(members) == p or partial_columns):
            loads = [sum(loads) / float(len(loads))] * len(loads) if plan == "ideal" else plan(loads)[1]
        table, other = (t_fwd, t_other_fwd) if kind == "F" else (t_bwd, t_other_bwd)
        times = [pass_time(table, load) + other for load in loads]
        makespan += max(times)
        for (r, _, _), t in zip(members, times):
            busy[r] += t
    ideal = sum(busy) / p
    bubble = [makespan - b for b in busy]
    return dict(makespan=makespan, busy=busy, bubble=bubble, ideal=ideal, bubble_fraction=[b / ideal for b in bubble])
