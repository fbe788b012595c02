"""The slice-wise 1F1B schedule simulator against what the paper fixes: the pass order drawn in
Fig. slim_schedule, the accumulated activation of Eq. 1 and the bubble fractions, both with the values
plotted in Fig. memory_dec, and the direction of the imbalance-bubble claims of Sec. 4.2.  CPU only."""
import json
import os

import pytest

from paper_2504_14519_amd.schedule_sim import (device_order, accumulated_slices, accumulated_fraction, exchange_groups,
                                               exchanged_loads, simulate, pass_time)

with open(os.path.join(os.path.dirname(__file__), "golden", "slim_schedule.json")) as f:
    FIG = json.load(f)


def test_pass_order_of_the_figure():
    p, n = FIG["p"], FIG["n"]
    for dev in range(1, p + 1):
        order = device_order(p, n, 5, dev - 1)
        warm = FIG["forward_passes_before_first_backward"][dev - 1]
        assert [o[0] for o in order[:warm]] == ["F"] * warm and order[warm][0] == "B"
        assert order[:warm] == [("F", f // n, f % n) for f in range(warm)]
        drawn = [(kind, k - 1, i - 1) for kind, k, i in FIG["passes_after_warmup"][str(dev)]]
        assert order[warm:warm + len(drawn)] == drawn


def test_every_pass_once_and_backward_after_forward():
    for p, n, m in [(1, 1, 1), (2, 2, 1), (4, 8, 3), (8, 8, 2), (4, 12, 5)]:
        for r in range(p):
            order = device_order(p, n, m, r)
            assert sorted(order) == sorted([(kd, k, i) for kd in "FB" for k in range(m) for i in range(n)])
            at = {o: j for j, o in enumerate(order)}
            for k in range(m):
                for i in range(n):
                    assert at[("F", k, i)] < at[("B", k, i)]
                    if i + 1 < n:          # last in, first out inside a microbatch
                        assert at[("B", k, i + 1)] < at[("B", k, i)] and at[("F", k, i)] < at[("F", k, i + 1)]


def test_aligned_moments_of_the_figure():
    p, n = FIG["p"], FIG["n"]
    groups = exchange_groups(p, n, 3)
    def group_of(kind, dev, k, i):
        for key, members in groups.items():
            if key[0] == kind and (dev - 1, k - 1, i - 1) in members:
                return key
    fw = {group_of("F", *x) for x in FIG["aligned_moment"]["forward"]}
    bw = {group_of("B", *x) for x in FIG["aligned_moment"]["backward"]}
    assert len(fw) == 1 and len(bw) == 1 and None not in fw | bw
    # away from the junctures the loads of a full group are a progression of step one, heaviest on device 1
    members = sorted(groups[("F", 2 * n + p)])
    assert [i for _, _, i in members] == [p - 1 - r + (2 * n + p - (p - 1)) % n for r in range(p)]


@pytest.mark.parametrize("p", [4, 8, 16])
def test_accumulated_activation_plotted_values(p):
    for x, percent in FIG["accumulated_percent_of_Ma"][str(p)].items():
        n = int(x) * p
        assert accumulated_slices(p, n, 2 * p, 0) == n + 2 * (p - 1)
        got = 100.0 * accumulated_fraction(p, n)
        assert abs(got - percent) < 6e-3, (p, n, got, percent)                 # plotted with 3 decimals
        assert abs(got - 100.0 * (1 + 2.0 * (p - 1) / n) / p) < 1e-9            # Eq. 1
    # later stages hold less
    assert [accumulated_slices(p, 2 * p, 2 * p, r) for r in range(p)] == [2 * p + 2 * (p - 1 - r) for r in range(p)]


@pytest.mark.parametrize("m", [2, 4, 8])
def test_bubble_fraction_plotted_values(m):
    p = 4
    for x, frac in FIG["bubble_fraction_p4"][str(m)].items():
        n = max(1, int(float(x) * p))
        for tf, tb in ((1.0, 2.0), (0.7, 1.9)):
            r = simulate(p, n, m, [tf] * n, [tb] * n)
            assert abs(r["bubble_fraction"] - frac) < 1e-9, (m, n, r["bubble_fraction"], frac)
            assert abs(r["makespan"] - (m * n + p - 1) * (tf + tb)) < 1e-9


def test_attention_dominated_bubbles():
    # pass time proportional to the attended key-value length (Sec. 4.2.1), backward twice the forward
    for p, n, m in [(4, 8, 4), (4, 16, 4), (8, 32, 4)]:
        tf = [float(L) for L in range(1, n + 1)]
        tb = [2.0 * L for L in range(1, n + 1)]
        plain = simulate(p, n, m, tf, tb)
        pair = simulate(p, n, m, tf, tb, exchange="pairwise")
        bal = simulate(p, n, m, tf, tb, exchange="balanced")
        ideal = simulate(p, n, m, tf, tb, exchange="ideal")
        # the exchange moves work, it does not create any
        for r in (pair, bal, ideal):
            assert abs(sum(r["busy"]) - sum(plain["busy"])) < 1e-6
        # imbalance bubbles: without the exchange the bubble is far above the warm-up/cool-down bound ...
        bound = (p - 1.0) / (n * m)
        assert plain["bubble_fraction"] > 2 * bound
        # ... the exchange removes most of it, finer balancing more, and perfectly equal loads reach the bound
        assert pair["bubble_fraction"] < 0.5 * plain["bubble_fraction"]
        assert ideal["bubble_fraction"] <= min(pair["bubble_fraction"], bal["bubble_fraction"]) + 1e-12
        assert abs(ideal["bubble_fraction"] - bound) < 1e-9
        # and never goes below the paper's long-context figure
        assert ideal["bubble_fraction"] >= (p - 1.0) * p / ((n + 1.0) * n * m)


def test_exchange_conserves_blocks_and_dependencies_hold():
    p, n, m = 4, 8, 3
    for mode in ("pairwise", "balanced", "ideal"):
        loads = exchanged_loads(p, n, m, mode)
        assert abs(sum(loads.values()) - 2 * p * m * n * (n + 1) / 2) < 1e-9
    r = simulate(p, n, m, [1.0 + 0.3 * L for L in range(n)], [2.0 + 0.8 * L for L in range(n)], exchange="pairwise",
                 t_other_fwd=0.5, t_other_bwd=1.0, t_send=0.1)
    end = {(kd, d, k, i): e for d in range(p) for kd, k, i, s, e in r["timeline"][d]}
    start = {(kd, d, k, i): s for d in range(p) for kd, k, i, s, e in r["timeline"][d]}
    for d in range(p):
        t = 0.0
        for kd, k, i, s, e in r["timeline"][d]:
            assert s >= t - 1e-12 and e > s          # one pass at a time
            t = e
            if kd == "F" and d > 0:
                assert s >= end[("F", d - 1, k, i)] + 0.1 - 1e-12
            if kd == "B" and d < p - 1:
                assert s >= end[("B", d + 1, k, i)] + 0.1 - 1e-12
            if kd == "B":
                assert s >= end[("F", d, k, i)]
    assert r["peak_slices"] == [n + 2 * (p - 1 - d) for d in range(p)]


def test_pass_time_interpolates():
    t = [1.0, 3.0, 7.0]
    assert pass_time(t, 2) == 3.0 and pass_time(t, 2.0) == 3.0 and abs(pass_time(t, 2.25) - 4.0) < 1e-12


def test_lockstep_model_and_the_long_context_figure():
    """Columns of aligned passes, each as long as its slowest pass: exact (p-1)/(nm) on every device for
    slice-independent times; for pass time proportional to the attended key-value length the paper's
    (p-1)p/((n+1)nm) is bracketed by the last device's bubble with and without the exchange in the incomplete
    columns of warm-up and cool-down."""
    from paper_2504_14519_amd.schedule_sim import simulate_lockstep
    for p, n, m in [(2, 2, 1), (4, 8, 4), (4, 16, 2), (8, 32, 8), (8, 64, 2), (16, 64, 3)]:
        u = simulate_lockstep(p, n, m, [0.7] * n, [1.9] * n)
        for frac in u["bubble_fraction"]:
            assert abs(frac - (p - 1.0) / (n * m)) < 1e-12
        assert abs(u["makespan"] - (n * m + p - 1) * 2.6) < 1e-9
        tf = [float(L) for L in range(1, n + 1)]
        tb = [2.0 * L for L in range(1, n + 1)]
        paper = (p - 1.0) * p / ((n + 1.0) * n * m)
        full_only = simulate_lockstep(p, n, m, tf, tb, exchange="ideal")
        everywhere = simulate_lockstep(p, n, m, tf, tb, exchange="ideal", partial_columns=True)
        lo, hi = everywhere["bubble_fraction"][-1], full_only["bubble_fraction"][-1]
        assert lo <= paper + 1e-12 and paper <= hi + 1e-12, (p, n, m, lo, paper, hi)
        # the figure itself: the columns the last device has no pass in (slices 1..p-1 only), nothing else
        assert abs(full_only["absent_fraction"][-1] - paper) < 1e-12
        # the two ends in closed form: columns without the last device at their mean / heaviest pass, and the
        # waits of the last device in the incomplete columns it shares
        assert abs(lo - (p - 1.0) * (p + 2) / (2.0 * m * n * (n + 1))) < 1e-12
        waits = sum(j * (1.0 + 2.0) for j in range(1, p - 1))          # it is j slices lighter than the heaviest
        assert abs(hi - (paper + waits / (m * 3.0 * n * (n + 1) / 2.0))) < 1e-12
        # the exchange conserves work; without it the columns last as long as their heaviest pass
        plain = simulate_lockstep(p, n, m, tf, tb)
        assert abs(sum(plain["busy"]) - sum(full_only["busy"])) < 1e-6
        assert plain["makespan"] > full_only["makespan"] or p == 1
        if n >= 2 * p:
            assert plain["bubble_fraction"][-1] > 3 * hi


# ---- the interleaving form: Fig. interleaved_slim_schedule and the SlimPipe row of Table sched-comparison ----
with open(os.path.join(os.path.dirname(__file__), "golden", "interleaved_slim_schedule.json")) as f:
    IFIG = json.load(f)


def drawn_passes(dev):
    """[(kind, microbatch, slice, stage, drawn start)] of a device, 0-based, from the figure's boxes (forward boxes are
    one unit wide, backward boxes two; the microbatch is the occurrence count of the box's label)."""
    x, seen, out = 0, {}, []
    for kind, stage, num in IFIG["drawn"][str(dev)]:
        if kind == "-":
            x += num
            continue
        k = seen.get((kind, stage, num), 0)
        seen[(kind, stage, num)] = k + 1
        out.append((kind, k, num - 1, stage - 1, x))
        x += 1 if kind == "F" else 2
    return out, x


def test_interleaved_pass_order_of_the_figure():
    from paper_2504_14519_amd.schedule_sim import device_order_interleaved, simulate_interleaved
    p, n, m, v = IFIG["p"], IFIG["n"], IFIG["m"], IFIG["v"]
    widths = []
    for dev in range(1, p + 1):
        drawn, width = drawn_passes(dev)
        widths.append(width)
        assert len(drawn) == 2 * n * m * v
        assert [d[:4] for d in drawn] == device_order_interleaved(p, n, m, v, dev - 1)      # every pass of the figure
    # the timeline under the figure's box widths (a forward pass of one stage 1 unit, a backward pass 2)
    r = simulate_interleaved(p, n, m, v, [1.0 * v] * n, [2.0 * v] * n)
    assert r["makespan"] == max(widths) == 105
    assert abs(r["bubble_fraction"] - 9.0 / 96.0) < 1e-12 and 9.0 / 96.0 == (p - 1.0) / (n * v * m)
    for dev in range(1, p + 1):
        drawn, _ = drawn_passes(dev)
        starts = [t[4] for t in r["timeline"][dev - 1]]
        # the last device is drawn exactly as simulated; the others never start a pass later than drawn (the figure
        # shifts some warm-up forward passes to the right to line them up with the other devices' passes)
        if dev == p:
            assert starts == [float(d[4]) for d in drawn]
        assert all(s <= d[4] for s, d in zip(starts, drawn))
        assert r["timeline"][dev - 1][-1][5] <= widths[dev - 1]


def test_interleaved_table_closed_forms():
    from paper_2504_14519_amd.schedule_sim import (device_order_interleaved, accumulated_units_interleaved,
                                                   accumulated_fraction_interleaved, simulate_interleaved, simulate_lockstep)
    for p, n, m, v in [(4, 8, 2, 2), (4, 8, 4, 2), (8, 16, 4, 3), (4, 12, 3, 1), (8, 8, 2, 5), (2, 4, 3, 4), (16, 32, 2, 2)]:
        # activation memory: 1/p + 2(p-1)/(nvp) of M_a on the first device, less on the later ones
        if m * n * v >= n * v + 2 * (p - 1):
            assert accumulated_units_interleaved(p, n, m, v, 0) == n * v + 2 * (p - 1)
            assert abs(accumulated_fraction_interleaved(p, n, v, m) - (1.0 / p + 2.0 * (p - 1) / (n * v * p))) < 1e-12
            assert [accumulated_units_interleaved(p, n, m, v, r) for r in range(p)] == [n * v + 2 * (p - 1 - r) for r in range(p)]
        # bubble fraction (p-1)/(nvm) for slice-independent pass times: event simulation and lockstep columns
        for tf, tb in ((1.0, 2.0), (0.7, 1.9)):
            r = simulate_interleaved(p, n, m, v, [tf] * n, [tb] * n)
            assert abs(r["bubble_fraction"] - (p - 1.0) / (n * v * m)) < 1e-9
            assert abs(r["makespan"] - (m * n * v + p - 1) * (tf + tb) / v) < 1e-9
            u = simulate_lockstep(p, n, m, [tf] * n, [tb] * n, v=v)
            assert all(abs(f - (p - 1.0) / (n * v * m)) < 1e-12 for f in u["bubble_fraction"])
            assert abs(u["absent_fraction"][-1] - (p - 1.0) / (n * v * m)) < 1e-12
        # "extremely long context": pass time proportional to the attended key-value length.  The columns the last
        # device is absent from hold slices 1..p-1 only: (p-1)p/((n+1)nvm), the table's footnote, exactly
        tf = [float(L) for L in range(1, n + 1)]
        tb = [2.0 * L for L in range(1, n + 1)]
        u = simulate_lockstep(p, n, m, tf, tb, exchange="ideal", v=v)
        assert abs(u["absent_fraction"][-1] - (p - 1.0) * p / ((n + 1.0) * n * v * m)) < 1e-12
        assert u["absent_fraction"][-1] < (p - 1.0) / (n * v * m) or n == p == 1
        # every pass once, backward after forward, and v = 1 is the plain schedule
        for rank in (0, p - 1):
            order = device_order_interleaved(p, n, m, v, rank)
            assert sorted(order) == sorted((kd, k, i, c) for kd in "FB" for k in range(m) for i in range(n) for c in range(v))
            at = {o: j for j, o in enumerate(order)}
            assert all(at[("F", k, i, c)] < at[("B", k, i, c)] for k in range(m) for i in range(n) for c in range(v))
            if v == 1:
                assert [o[:3] for o in order] == device_order(p, n, m, rank)
    # v = 1: same timeline as the plain simulator, with the context exchange
    p, n, m = 4, 8, 3
    tf, tb = [1.0 + 0.3 * L for L in range(n)], [2.0 + 0.8 * L for L in range(n)]
    for mode in (None, "pairwise", "balanced", "ideal"):
        a = simulate(p, n, m, tf, tb, exchange=mode, t_other_fwd=0.5, t_other_bwd=1.0, t_send=0.1)
        b = simulate_interleaved(p, n, m, 1, tf, tb, exchange=mode, t_other_fwd=0.5, t_other_bwd=1.0, t_send=0.1)
        assert abs(a["makespan"] - b["makespan"]) < 1e-9 and abs(a["bubble_fraction"] - b["bubble_fraction"]) < 1e-12


def test_interleaved_dependencies_and_exchange():
    from paper_2504_14519_amd.schedule_sim import simulate_interleaved
    p, n, m, v = 4, 8, 2, 2
    tf = [float(L) for L in range(1, n + 1)]
    tb = [2.0 * L for L in range(1, n + 1)]
    plain = simulate_interleaved(p, n, m, v, tf, tb)
    for mode in ("pairwise", "balanced", "ideal"):
        r = simulate_interleaved(p, n, m, v, tf, tb, exchange=mode, t_send=0.05)
        assert abs(sum(r["busy"]) - sum(plain["busy"])) < 1e-6          # the exchange moves work, it creates none
        assert r["bubble_fraction"] < plain["bubble_fraction"]
        end = {(kd, d, k, i, c): e for d in range(p) for kd, k, i, c, s, e in r["timeline"][d]}
        for d in range(p):
            t = 0.0
            for kd, k, i, c, s, e in r["timeline"][d]:
                assert s >= t - 1e-12 and e > s
                t = e
                stage = c * p + d
                if kd == "F" and stage > 0:
                    prev = (stage - 1) % p, (stage - 1) // p
                    assert s >= end[("F", prev[0], k, i, prev[1])] + (0.05 if prev[0] != d else 0.0) - 1e-12
                if kd == "B":
                    assert s >= end[("F", d, k, i, c)]
                    if stage < p * v - 1:
                        nxt = (stage + 1) % p, (stage + 1) // p
                        assert s >= end[("B", nxt[0], k, i, nxt[1])] + (0.05 if nxt[0] != d else 0.0) - 1e-12
