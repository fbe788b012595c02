"""Slice-wise 1F1B pipeline schedule of the paper (Sec. 4.1.2, Fig. slim_schedule) as a host-side discrete
simulation: per-device pass order, a timeline under given per-slice forward/backward times (measured
kernel times can be fed in), accumulated activation in slices, bubble fraction, and the effect of the
attention context exchange (Sec. 4.2) on the imbalance bubbles.  Plain Python, no GPU work.  The functions
whose names end in `_interleaved` cover the interleaving form (v stages per device, Fig. interleaved_slim_schedule,
the SlimPipe row of Table sched-comparison); the others are its v = 1 case.

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


def simulate_lockstep(p, n, m, t_fwd, t_bwd, exchange=None, partial_columns=False, t_other_fwd=0.0, t_other_bwd=0.0, v=1):
    """The schedule as the paper draws it: passes that stand in one column (exchange_groups) start together and
    the column lasts as long as its slowest pass.  This is the model behind the closed forms of Sec. 4.1.3 and of
    Table sched-comparison: a device's bubble is the sum of the columns in which it has no pass (p-1 forward columns
    and p-1 backward columns), plus what it waits inside the columns it shares.  v > 1: the interleaving form (columns
    of exchange_groups_interleaved, a pass through one of a device's v stages takes 1/v of the device's time).

    exchange: None, or 'pairwise' / 'balanced' / 'ideal' as in `simulate`; it is applied to the columns in which
    all p devices have a pass (the situation of the paper's picture) and, with partial_columns, also among the
    devices of the incomplete columns of the warm-up and cool-down.

    `absent_fraction[rank]` is the part of the bubble that the paper's closed forms count: the columns the device has
    no pass in, each at the length of its slowest pass, over the ideal time.  For the last device it is (p-1)/(nvm)
    when pass times do not depend on the slice, and (p-1)p/((n+1)nvm) when they are proportional to the attended
    key-value length (the first p-1 forward columns hold slices 1..p-1 only, the last p-1 backward columns
    likewise): the paper's two figures.  What the device waits INSIDE shared incomplete columns comes on top in
    `bubble_fraction` unless the exchange also runs there (partial_columns).

    -> dict(makespan, busy[rank], bubble[rank], ideal, bubble_fraction[rank], absent_fraction[rank]) with ideal = all
    work spread evenly over the p devices and bubble_fraction = bubble / ideal."""
    plan = {None: None, "pairwise": redistribute_pairwise, "balanced": redistribute_balanced, "ideal": "ideal"}[exchange]
    busy = [0.0] * p
    absent = [0.0] * p
    makespan = 0.0
    for (kind, _), members in exchange_groups_interleaved(p, n, m, v).items():
        loads = [mem[2] + 1 for mem in members]
        if plan is not None and (len(members) == p or partial_columns):
            loads = [sum(loads) / float(len(loads))] * len(loads) if plan == "ideal" else plan(loads)[1]
        table, other = (t_fwd, t_other_fwd) if kind == "F" else (t_bwd, t_other_bwd)
        times = [(pass_time(table, load) + other) / v for load in loads]
        makespan += max(times)
        present = set()
        for mem, t in zip(members, times):
            busy[mem[0]] += t
            present.add(mem[0])
        for r in range(p):
            if r not in present:
                absent[r] += max(times)
    ideal = sum(busy) / p
    bubble = [makespan - b for b in busy]
    return dict(makespan=makespan, busy=busy, bubble=bubble, ideal=ideal, bubble_fraction=[b / ideal for b in bubble],
                absent_fraction=[a / ideal for a in absent])


# ---- the interleaving form (Sec. 4.1.2 last paragraph, Fig. interleaved_slim_schedule, Table sched-comparison) ----
# Every device holds v small stages: stage c * p + r (c = 0..v-1) sits on device r, so a slice crosses the devices v
# times.  A pass is (kind, microbatch, slice, c).  As drawn: a device takes the slices of a microbatch in groups of p;
# a group goes through the device's first stage, then the same group through its second stage, ..., then the next
# group; backward passes run the other way round (last group first, last stage first, last slice first).

def unit_sequences_interleaved(p, n, m, v):
    """(forward passes, backward passes) of any device in its own order: lists of (microbatch, slice, c)."""
    if n % p != 0:
        raise ValueError("the interleaving form takes the slices in groups of p: n must be a multiple of p")
    fwd = [(k, g * p + j, c) for k in range(m) for g in range(n // p) for c in range(v) for j in range(p)]
    bwd = [(k, g * p + j, c) for k in range(m) for g in reversed(range(n // p)) for c in reversed(range(v))
           for j in reversed(range(p))]
    return fwd, bwd


def device_order_interleaved(p, n, m, v, rank):
    """Pass order on device `rank`: [('F'|'B', microbatch, slice, c)].  The device runs n v + 2(p-1-rank) forward
    passes before its first backward pass (the v = 1 rule with n v passes per microbatch), then alternates one
    backward, one forward."""
    fwd, bwd = unit_sequences_interleaved(p, n, m, v)
    total = len(fwd)
    warm = min(total, n * v + 2 * (p - 1 - rank))
    order = [("F",) + u for u in fwd[:warm]]
    fi, bi = warm, 0
    while bi < total:
        order.append(("B",) + bwd[bi]); bi += 1
        if fi < total:
            order.append(("F",) + fwd[fi]); fi += 1
    return order


def accumulated_units_interleaved(p, n, m, v, rank):
    """Largest number of (slice, stage) activations device `rank` holds at once; one is M_a / (n v p)."""
    live = peak = 0
    for o in device_order_interleaved(p, n, m, v, rank):
        live += 1 if o[0] == "F" else -1
        peak = max(peak, live)
    return peak


def accumulated_fraction_interleaved(p, n, v, m=None, rank=0):
    """Accumulated activation of device `rank` as a fraction of M_a; on the first device, with enough microbatches,
    1/p + 2(p-1)/(n v p) (Table sched-comparison, SlimPipe row)."""
    if m is None:
        m = 2 * p
    return accumulated_units_interleaved(p, n, m, v, rank) / float(n * v * p)


def exchange_groups_interleaved(p, n, m, v):
    """Passes that stand in one column of the aligned schedule: the u-th forward pass of device r with the (u-1)-th of
    device r+1, the u-th backward pass of device r with the (u+1)-th of device r+1.
    -> {('F'|'B', column): [(rank, microbatch, slice, c)]}."""
    fwd, bwd = unit_sequences_interleaved(p, n, m, v)
    groups = {}
    for r in range(p):
        for u, unit in enumerate(fwd):
            groups.setdefault(("F", u + r), []).append((r,) + unit)
        for u, unit in enumerate(bwd):
            groups.setdefault(("B", u + (p - 1 - r)), []).append((r,) + unit)
    return groups


def simulate_interleaved(p, n, m, v, t_fwd, t_bwd, exchange=None, t_other_fwd=0.0, t_other_bwd=0.0, t_send=0.0):
    """`simulate` for v stages per device.  t_fwd[L-1], t_bwd[L-1] (and t_other_*) are the times of a pass through ALL
    layers of a device; a pass through one of its v stages takes 1/v of that.  A forward pass of stage c * p + r waits
    for the same slice on stage c * p + r - 1 (device r-1, or device p-1 with c-1), a backward pass for stage
    c * p + r + 1; the last stage's backward pass follows its own forward pass.  exchange as in `simulate`, over the
    columns of exchange_groups_interleaved.
    -> dict(makespan, busy[rank], bubble_fraction, timeline[rank] = [(kind, k, i, c, start, end)], peak_units[rank])."""
    loads = None
    if exchange:
        plan = {"pairwise": redistribute_pairwise, "balanced": redistribute_balanced, "ideal": None}[exchange]
        loads = {}
        for (kind, _), members in exchange_groups_interleaved(p, n, m, v).items():
            before = [i + 1 for _, _, i, _ in members]
            after = plan(before)[1] if plan else [sum(before) / float(len(before))] * len(before)
            for (r, k, i, c), load in zip(members, after):
                loads[(kind, r, k, i, c)] = load
    orders = [device_order_interleaved(p, n, m, v, r) for r in range(p)]
    pos, free, done = [0] * p, [0.0] * p, {}
    timeline = [[] for _ in range(p)]
    remaining = sum(len(o) for o in orders)
    while remaining:
        progressed = False
        for r in range(p):
            while pos[r] < len(orders[r]):
                kind, k, i, c = orders[r][pos[r]]
                if kind == "F":
                    dep = ("F", r - 1, k, i, c) if r > 0 else (("F", p - 1, k, i, c - 1) if c > 0 else None)
                else:
                    dep = ("B", r + 1, k, i, c) if r < p - 1 else (("B", 0, k, i, c + 1) if c < v - 1 else ("F", r, k, i, c))
                if dep is not None and dep not in done:
                    break
                ready = 0.0 if dep is None else done[dep] + (t_send if dep[1] != r else 0.0)
                load = loads[(kind, r, k, i, c)] if loads else i + 1
                dur = ((pass_time(t_fwd, load) + t_other_fwd) if kind == "F" else (pass_time(t_bwd, load) + t_other_bwd)) / v
                start = max(free[r], ready)
                free[r] = start + dur
                done[(kind, r, k, i, c)] = free[r]
                timeline[r].append((kind, k, i, c, start, free[r]))
                pos[r] += 1
                remaining -= 1
                progressed = True
        if not progressed:
            raise RuntimeError("schedule deadlock: p=%d n=%d m=%d v=%d" % (p, n, m, v))
    makespan = max(free)
    busy = [sum(x[5] - x[4] for x in tl) for tl in timeline]
    ideal = sum(busy) / p
    return dict(makespan=makespan, busy=busy, bubble_fraction=(makespan - ideal) / ideal, timeline=timeline,
                peak_units=[accumulated_units_interleaved(p, n, m, v, r) for r in range(p)])
