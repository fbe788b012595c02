"""Host-side integer helpers for splitting one slice's attention into key ranges of equal work.

A slice of s query rows at offset q_offset sees keys [0, q_offset + s).  The number of visible
(query, key) pairs with key < e is  C(e) = s*e  for e <= q_offset and
s*q_offset + x*s - x*(x-1)/2  with x = e - q_offset  beyond (the causal triangle of the diagonal
block).  Cutting at equal C gives ranges of equal attention cost, which is what the paper's
attention context exchange balances (Sec. 4.2.1: cost proportional to attended key-value length;
Sec. 4.2.2: portions of key-value handed to another device).
"""


def visible_pairs_upto(s, q_offset, e):
    """Visible (row, key) pairs with key < e for one causal query slice (per head)."""
    e = max(0, min(e, q_offset + s))
    if e <= q_offset:
        return s * e
    x = e - q_offset
    return s * q_offset + x * s - x * (x - 1) // 2


def equal_flop_cuts(s, q_offset, parts, align=128):
    """Cut points 0 = c_0 < c_1 <= ... <= c_parts = q_offset + s, interior ones multiples of `align`,
    each the smallest aligned key index whose pair count reaches k/parts of the total."""
    end = q_offset + s
    total = visible_pairs_upto(s, q_offset, end)
    cuts = [0]
    for k in range(1, parts):
        target = (k * total + parts - 1) // parts
        lo, hi = 0, (end + align - 1) // align
        while lo < hi:                                   # smallest m with C(m*align) >= target
            mid = (lo + hi) // 2
            if visible_pairs_upto(s, q_offset, mid * align) >= target:
                hi = mid
            else:
                lo = mid + 1
        cuts.append(min(max(lo * align, cuts[-1]), end))
    cuts.append(end)
    return cuts


# ---------------------------------------------------------------------------------------------------
# Attention context exchange (paper Sec. 4.2.2): which device computes which (query slice, key-value
# blocks) piece so that the attention workloads of the pipeline devices at one moment are as equal as
# possible.  A device's load is the number of key-value slices ("blocks") its query slice attends to:
# blocks 1..load, the last one being the causal diagonal block.  Devices with more blocks hand their
# LAST blocks, together with the query, to devices with fewer; the partial outputs come back and are
# merged by the online-softmax rule (slimpipe_attn_merge).

def redistribute_pairwise(loads):
    """The scheme of the paper's picture: the k-th heaviest device is paired with the k-th lightest and
    hands it floor((heavy - light) / 2) of its last blocks, one helper per device.

    loads[d] -> (pieces, loads_after); pieces = [(owner, helper, first_block, last_block)], blocks 1-based
    and inclusive as in the paper's figure."""
    p = len(loads)
    order = sorted(range(p), key=lambda d: (-loads[d], d))          # heaviest first, ties by device
    after = list(loads)
    pieces = []
    for k in range(p // 2):
        heavy, light = order[k], order[p - 1 - k]
        move = (loads[heavy] - loads[light]) // 2
        if move > 0:
            pieces.append((heavy, light, loads[heavy] - move + 1, loads[heavy]))
            after[heavy] -= move
            after[light] += move
    return pieces, after


def redistribute_balanced(loads):
    """Loads equal up to one block for ANY load vector (also at the juncture of two microbatches, where
    pairwise exchange leaves a spread): every device ends at floor or ceil of the mean, the devices that
    were heaviest keeping the larger share; a heavy device may feed several helpers, last blocks first
    to the lightest helper.  Same output format as redistribute_pairwise."""
    p = len(loads)
    total = sum(loads)
    base, extra = divmod(total, p)
    order = sorted(range(p), key=lambda d: (-loads[d], d))
    target = {d: base + (1 if rank < extra else 0) for rank, d in enumerate(order)}
    # a device never takes on work when it is above the mean and never gives when it is below it
    donors = [d for d in order if loads[d] > target[d]]
    takers = [d for d in reversed(order) if loads[d] < target[d]]           # lightest first
    after = list(loads)
    pieces = []
    ti = 0
    for d in donors:
        give = loads[d] - target[d]
        last = loads[d]
        while give > 0:
            t = takers[ti]
            n = min(give, target[t] - after[t])
            pieces.append((d, t, last - n + 1, last))
            last -= n
            give -= n
            after[d] -= n
            after[t] += n
            if after[t] == target[t]:
                ti += 1
    return pieces, after


def piece_key_range(piece, slice_len):
    """(owner, helper, first_block, last_block) -> (kv_begin, kv_end) in keys, for the library calls."""
    return (piece[2] - 1) * slice_len, piece[3] * slice_len


def exchange_volume_slices(p, n):
    """Exchanged context per microbatch per device in units of one slice of one tensor, the three terms of
    the paper's communication-volume formula (Sec. 4.2.2): query + output, key + value away from the
    junctures of two microbatches, key + value at the junctures (p - 1 of the n passes)."""
    return 2 * n, 2 * (n - p + 1) * ((p - 1) // 2), 2 * (p - 1) * ((n - 1) // 2)


def plan_context_exchange(slice_index, slice_len, balanced=False):
    """slice_index[d] = index (0-based) of the query slice device d works on at this moment, each within its
    own microbatch -> list of (helper device, owner device, owner's query slice, kv_begin, kv_end): the
    helper computes attention of the owner's query slice over keys [kv_begin, kv_end) of the owner's
    microbatch and returns (out, lse); the owner keeps keys [0, first kv_begin it gave away)."""
    loads = [i + 1 for i in slice_index]
    pieces, _ = (redistribute_balanced if balanced else redistribute_pairwise)(loads)
    return [(h, o, slice_index[o]) + piece_key_range((o, h, a, b), slice_len) for o, h, a, b in pieces]
