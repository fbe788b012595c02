"""Plain fp64 definition of slice-wise causal attention, its gradient and the
log-sum-exp merge.  TEST INFRASTRUCTURE: slow, unblocked, written to be checked
against the paper by eye.  It shares no code with the HIP path.

What it follows (SlimPipe paper):
  * Sec. 4.1.2 "Slice-wise Scheduling": the queries of slice i attend causally to
    the cached keys/values of slices 0..i; the same K/V are kept for backward.
  * Sec. 4.1.1: causality means a later query sees earlier keys, never the reverse.
  * Sec. 4.2.2 "Exchange the Context": a (query slice, K/V portion) pair is computed
    elsewhere and its output is folded into the local one by the online-softmax
    rule; Sec. 5 "Commutated Context Parallelism": what travels with an output is
    the softmax normaliser.
The paper fixes no formula beyond "causal attention"; the textbook definition is
written out here.  Readings taken where the paper is silent: the normaliser is one
number per row, lse = ln sum_j exp(scale * q.k_j) (natural log, scale inside);
key j is visible to row r iff kv_begin <= j < kv_end and (not causal or
j <= q_offset + r); query head h reads KV head h // (Hq // Hkv); a row that sees
no key has out = 0 and lse = -inf.

Pins (tests/test_oracle_pins.py): a stock fp64 scaled-dot-product routine and its
autograd on unsliced sequences, central finite differences, closed forms that can
be counted by hand, scalar brute force, split/merge identities and the block
pattern of Fig. "attn_balance".

Layouts: q, out, dout, dq [B, s, Hq, D]; k, v, dk, dv [B, Nkv, Hkv, D] where row j
is global position j; lse [B, Hq, s].  All float64 numpy arrays.
"""
import numpy as np


def _visible(s, q_offset, kv_begin, kv_end, causal):
    """Boolean [s, kv_end-kv_begin]: is key kv_begin+c visible to row r."""
    j = np.arange(kv_begin, kv_end)[None, :]
    if causal:
        t = (q_offset + np.arange(s))[:, None]
        return j <= t
    return np.ones((s, kv_end - kv_begin), dtype=bool)


def attn_fwd(q, k, v, q_offset, kv_begin, kv_end, causal, scale):
    """(out, lse) of the query slice against keys [kv_begin, kv_end).  Sec. 4.1.2, 4.2.2."""
    B, s, Hq, D = q.shape
    Hkv = k.shape[2]
    G = Hq // Hkv
    out = np.zeros((B, s, Hq, D), dtype=np.float64)
    lse = np.full((B, Hq, s), -np.inf, dtype=np.float64)
    if kv_end <= kv_begin:
        return out, lse
    vis = _visible(s, q_offset, kv_begin, kv_end, causal)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            kk = k[b, kv_begin:kv_end, g, :]
            vv = v[b, kv_begin:kv_end, g, :]
            sc = scale * (q[b, :, h, :] @ kk.T)
            sc = np.where(vis, sc, -np.inf)
            m = sc.max(axis=1)
            has = np.isfinite(m)
            m_safe = np.where(has, m, 0.0)
            e = np.exp(sc - m_safe[:, None])          # exp(-inf) = 0 for hidden keys
            l = e.sum(axis=1)
            row_lse = np.where(has, m_safe + np.log(np.where(has, l, 1.0)), -np.inf)
            p = np.where(has[:, None], e / np.where(has, l, 1.0)[:, None], 0.0)
            out[b, :, h, :] = p @ vv
            lse[b, h, :] = row_lse
    return out, lse


def attn_merge(outs, lses):
    """Online-softmax merge of partial results over disjoint key sets.  Sec. 4.2.2.

    outs: list of [B, s, Hq, D]; lses: list of [B, Hq, s].
    lse = ln sum_r exp(lse_r);  out = sum_r exp(lse_r - lse) * out_r.
    """
    L = np.stack(lses, axis=0)                        # [R, B, Hq, s]
    m = L.max(axis=0)
    has = np.isfinite(m)
    m_safe = np.where(has, m, 0.0)
    tot = np.exp(L - m_safe[None]).sum(axis=0)
    lse = np.where(has, m_safe + np.log(np.where(has, tot, 1.0)), -np.inf)
    out = np.zeros_like(outs[0], dtype=np.float64)
    for o, l in zip(outs, lses):
        w = np.where(has, np.exp(l - np.where(has, lse, 0.0)), 0.0)   # [B, Hq, s]
        out += np.transpose(w, (0, 2, 1))[..., None] * o
    return out, lse


def attn_bwd(q, k, v, out, dout, lse, q_offset, kv_begin, kv_end, causal, scale):
    """Gradient of sum(out * dout) restricted to keys [kv_begin, kv_end).

    `out` and `lse` are the rows' final (merged, whole visible set) values, so a
    call over a sub-range yields the exact partial gradient of that range:
    dq parts add up over ranges, dk/dv rows outside the range stay zero.
    Sec. 4.1.2 (backward per slice, K/V kept for it), Sec. 4.2.2.
      p_ij  = exp(scale q_i.k_j - lse_i) for visible j, else 0
      delta = sum_d dout_i,d out_i,d
      dv_j  = sum_{h in group} sum_i p_ij dout_i
      ds_ij = p_ij (dout_i.v_j - delta_i)
      dq_i  = scale sum_j ds_ij k_j ;  dk_j = scale sum_{h in group} sum_i ds_ij q_i
    """
    B, s, Hq, D = q.shape
    Hkv = k.shape[2]
    G = Hq // Hkv
    dq = np.zeros_like(q, dtype=np.float64)
    dk = np.zeros_like(k, dtype=np.float64)
    dv = np.zeros_like(v, dtype=np.float64)
    if kv_end <= kv_begin:
        return dq, dk, dv
    vis = _visible(s, q_offset, kv_begin, kv_end, causal)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            kk = k[b, kv_begin:kv_end, g, :]
            vv = v[b, kv_begin:kv_end, g, :]
            row_lse = lse[b, h, :]
            has = np.isfinite(row_lse)
            sc = scale * (q[b, :, h, :] @ kk.T)
            p = np.exp(np.where(vis & has[:, None], sc - np.where(has, row_lse, 0.0)[:, None], -np.inf))
            do = dout[b, :, h, :]
            delta = (do * out[b, :, h, :]).sum(axis=1)
            dp = do @ vv.T
            ds = p * (dp - delta[:, None])
            dq[b, :, h, :] = scale * (ds @ kk)
            dk[b, kv_begin:kv_end, g, :] += scale * (ds.T @ q[b, :, h, :])
            dv[b, kv_begin:kv_end, g, :] += p.T @ do
    return dq, dk, dv
