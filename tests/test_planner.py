"""Host-side planner of the attention context exchange (paper Sec. 4.2.2) against what the paper fixes:
the worked picture (Fig. attn_balance), the claim that loads end within one key-value slice of each other, the slice counts that enter the
communication-volume formula and its bound.  CPU only."""
import json
import os

import pytest

from paper_2504_14519_amd.planner import (redistribute_pairwise, redistribute_balanced, piece_key_range,
                                          exchange_volume_slices, visible_pairs_upto)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def figure():
    with open(os.path.join(GOLDEN, "attn_balance.json")) as f:
        return json.load(f)


@pytest.mark.parametrize("plan", [redistribute_pairwise, redistribute_balanced])
def test_reproduces_the_papers_picture(plan):
    fig = figure()
    pieces, after = plan(fig["loads_before"])
    assert after == fig["loads_after"]
    # the same pieces as drawn: (owner query, helper device, blocks)
    drawn = sorted((r["query"], d["device"], r["blocks"][0], r["blocks"][-1]) for d in fig["devices"] for r in d["remote"])
    query_of = {i: d["query"] for i, d in enumerate(fig["devices"])}
    dev_of = {i: d["device"] for i, d in enumerate(fig["devices"])}
    got = sorted((query_of[o], dev_of[h], a, b) for o, h, a, b in pieces)
    assert got == drawn
    # what stays local is what the figure keeps solid
    for i, d in enumerate(fig["devices"]):
        given = sum(b - a + 1 for o, h, a, b in pieces if o == i)
        assert list(range(1, fig["loads_before"][i] - given + 1)) == d["local"]


@pytest.mark.parametrize("p", [2, 3, 4, 6, 8, 16])
def test_steady_state_progressions_end_within_one_block(p):
    # away from the junctures the loads of the p devices form an arithmetic progression of step 1
    for heaviest in range(p, 3 * p):
        loads = [heaviest - d for d in range(p)]
        for plan in (redistribute_pairwise, redistribute_balanced):
            pieces, after = plan(loads)
            assert sum(after) == sum(loads)
            assert max(after) - min(after) <= 1
            # no device hands away more key-value slices than the paper counts: floor((p-1)/2)
            for d in range(p):
                assert sum(b - a + 1 for o, h, a, b in pieces if o == d) <= (p - 1) // 2
            # pieces are the owner's LAST blocks, contiguous, and never reach below block 1
            for o, h, a, b in pieces:
                assert 1 <= a <= b <= loads[o] and o != h


def test_junctures():
    # at the juncture of two microbatches some devices are already on the first slices of the next one
    p, n = 4, 8
    for shift in range(1, p):
        loads = [((n - 1 - d + shift) % n) + 1 for d in range(p)]          # e.g. [1, 8, 7, 6]
        pieces, after = redistribute_pairwise(loads)
        assert sum(after) == sum(loads)
        heavy = max(range(p), key=lambda d: loads[d])
        # the heaviest device hands away at most floor((n-1)/2) key-value slices (the paper's juncture term)
        assert sum(b - a + 1 for o, h, a, b in pieces if o == heavy) <= (n - 1) // 2
        pieces, after = redistribute_balanced(loads)
        assert sum(after) == sum(loads) and max(after) - min(after) <= 1
        # every block of every query is computed exactly once
        for d in range(p):
            kept = loads[d] - sum(b - a + 1 for o, h, a, b in pieces if o == d)
            blocks = list(range(1, kept + 1)) + [x for o, h, a, b in pieces if o == d for x in range(a, b + 1)]
            assert sorted(blocks) == list(range(1, loads[d] + 1))


def test_balanced_handles_arbitrary_loads():
    import random
    rng = random.Random(5)
    for _ in range(200):
        p = rng.randint(1, 12)
        loads = [rng.randint(1, 40) for _ in range(p)]
        pieces, after = redistribute_balanced(loads)
        assert sum(after) == sum(loads) and max(after) - min(after) <= 1
        for d in range(p):
            recomputed = loads[d] - sum(b - a + 1 for o, h, a, b in pieces if o == d) + sum(b - a + 1 for o, h, a, b in pieces if h == d)
            assert recomputed == after[d]
        for o, h, a, b in pieces:
            assert 1 <= a <= b <= loads[o] and loads[o] > loads[h]


@pytest.mark.parametrize("p,n", [(2, 2), (4, 8), (4, 16), (8, 8), (8, 32), (16, 64)])
def test_exchange_volume_bound(p, n):
    # Theta = (2n + 2(n-p+1) floor((p-1)/2) + 2(p-1) floor((n-1)/2)) * L*M_h/(p*n)  <=  (2 - (p-1)/n) * L*M_h
    qo, kv, kvj = exchange_volume_slices(p, n)
    theta_over_lmh = (qo + kv + kvj) / (p * n)
    assert theta_over_lmh <= 2 - (p - 1) / n + 1e-12
    assert theta_over_lmh <= 2
    # without the round-downs the bound is attained
    exact = (2 * n + 2 * (n - p + 1) * (p - 1) / 2 + 2 * (p - 1) * (n - 1) / 2) / (p * n)
    assert abs(exact - (2 - (p - 1) / n)) < 1e-12


def test_piece_key_range_and_cost():
    s = 512
    pieces, _ = redistribute_pairwise([7, 6, 5, 4, 3, 2])
    by_owner = {o: (a, b) for o, h, a, b in pieces}
    assert piece_key_range((0, 5) + by_owner[0], s) == (5 * s, 7 * s)
    # the cost model behind "load = number of blocks": a full block costs s*s pairs, the diagonal one about half
    q_off = 6 * s
    full = visible_pairs_upto(s, q_off, 6 * s) - visible_pairs_upto(s, q_off, 5 * s)
    diag = visible_pairs_upto(s, q_off, 7 * s) - visible_pairs_upto(s, q_off, 6 * s)
    assert full == s * s and diag == s * (s + 1) // 2


def test_plan_in_key_units():
    from paper_2504_14519_amd.planner import plan_context_exchange
    s = 1024
    plan = plan_context_exchange([6, 5, 4, 3, 2, 1], s)
    assert sorted(plan) == [(4, 1, 5, 5 * s, 6 * s), (5, 0, 6, 5 * s, 7 * s)]
    # the piece that is handed away contains the causal diagonal block: its end is the end of the query slice
    for h, o, qs, a, b in plan:
        assert b == (qs + 1) * s
