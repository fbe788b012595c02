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
