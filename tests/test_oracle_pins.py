"""Pins of the fp64 oracle against things other than itself (no GPU).

  * a stock fp64 scaled-dot-product-attention routine and its autograd (library special case:
    unsliced causal attention, and rectangular slices via an explicit boolean mask);
  * central finite differences of the forward oracle;
  * closed forms that are fixed by counting (zero queries, one visible key, equal keys, key shift);
  * scalar brute force with exact summation on tiny inputs (index/transposition/GQA mistakes);
  * structural identities of the method: slices + cached prefix == unsliced sequence (Sec. 4.1.2),
    merged partial ranges == whole range (Sec. 4.2.2), incl. the block pattern of Fig. attn_balance.
"""
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import attn_fwd, attn_bwd, attn_merge

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rnd(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def torch_causal_full(q, k, v, scale, G):
    """Unsliced causal attention and its gradients from the stock routine + autograd (fp64)."""
    tq = torch.tensor(q, dtype=torch.float64, requires_grad=True)
    tk = torch.tensor(k, dtype=torch.float64, requires_grad=True)
    tv = torch.tensor(v, dtype=torch.float64, requires_grad=True)
    kk = tk.repeat_interleave(G, dim=2)
    vv = tv.repeat_interleave(G, dim=2)
    o = torch.nn.functional.scaled_dot_product_attention(
        tq.permute(0, 2, 1, 3), kk.permute(0, 2, 1, 3), vv.permute(0, 2, 1, 3), is_causal=True, scale=scale)
    return tq, tk, tv, o.permute(0, 2, 1, 3)


# ---------------------------------------------------------------- library special case
@pytest.mark.parametrize("n,s,Hq,Hkv,D", [(4, 7, 4, 2, 8), (3, 5, 2, 1, 4), (1, 16, 3, 3, 6)])
def test_slices_equal_unsliced_library_fwd_and_bwd(n, s, Hq, Hkv, D):
    N, B, G = n * s, 2, Hq // Hkv
    scale = 0.37
    q, k, v, do = rnd((B, N, Hq, D), 1), rnd((B, N, Hkv, D), 2), rnd((B, N, Hkv, D), 3), rnd((B, N, Hq, D), 4)
    tq, tk, tv, o_ref = torch_causal_full(q, k, v, scale, G)
    (o_ref * torch.tensor(do)).sum().backward()
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for i in range(n):
        sl = slice(i * s, (i + 1) * s)
        o, lse = attn_fwd(q[:, sl], k, v, i * s, 0, (i + 1) * s, True, scale)
        np.testing.assert_allclose(o, o_ref.detach().numpy()[:, sl], rtol=0, atol=1e-12)
    for i in reversed(range(n)):                      # backward in reverse slice order
        sl = slice(i * s, (i + 1) * s)
        o, lse = attn_fwd(q[:, sl], k, v, i * s, 0, (i + 1) * s, True, scale)
        dq_i, dk_i, dv_i = attn_bwd(q[:, sl], k, v, o, do[:, sl], lse, i * s, 0, (i + 1) * s, True, scale)
        np.testing.assert_allclose(dq_i, tq.grad.numpy()[:, sl], rtol=0, atol=1e-12)
        dk += dk_i
        dv += dv_i
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=0, atol=1e-12)


def test_rectangular_slice_vs_library_with_explicit_mask_and_lse():
    B, s, Hq, Hkv, D, Nkv = 1, 6, 4, 2, 8, 29
    q_offset, kv_begin, kv_end, scale = 17, 3, 21, 0.5
    q, k, v = rnd((B, s, Hq, D), 5), rnd((B, Nkv, Hkv, D), 6), rnd((B, Nkv, Hkv, D), 7)
    o, lse = attn_fwd(q, k, v, q_offset, kv_begin, kv_end, True, scale)
    j = torch.arange(Nkv)[None, :]
    t = (q_offset + torch.arange(s))[:, None]
    mask = (j >= kv_begin) & (j < kv_end) & (j <= t)
    tq = torch.tensor(q).permute(0, 2, 1, 3)
    tk = torch.tensor(k).repeat_interleave(2, dim=2).permute(0, 2, 1, 3)
    tv = torch.tensor(v).repeat_interleave(2, dim=2).permute(0, 2, 1, 3)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=scale)
    np.testing.assert_allclose(o, ref.permute(0, 2, 1, 3).numpy(), atol=1e-12)
    sc = scale * (tq @ tk.transpose(-1, -2))
    ref_lse = torch.logsumexp(sc.masked_fill(~mask, -math.inf), dim=-1)   # [B,Hq,s]
    np.testing.assert_allclose(lse, ref_lse.numpy(), atol=1e-12)


def test_noncausal_full_range_is_plain_softmax_attention():
    B, s, H, D, Nkv = 1, 5, 2, 4, 9
    q, k, v = rnd((B, s, H, D), 8), rnd((B, Nkv, H, D), 9), rnd((B, Nkv, H, D), 10)
    o, _ = attn_fwd(q, k, v, 0, 0, Nkv, False, 0.7)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.tensor(q).permute(0, 2, 1, 3), torch.tensor(k).permute(0, 2, 1, 3),
        torch.tensor(v).permute(0, 2, 1, 3), scale=0.7)
    np.testing.assert_allclose(o, ref.permute(0, 2, 1, 3).numpy(), atol=1e-12)


# ---------------------------------------------------------------- finite differences
def test_bwd_matches_central_finite_differences_incl_gqa_and_split():
    B, s, Hq, Hkv, D = 1, 5, 2, 1, 4
    n = 3
    Nkv = n * s
    scale = 0.6
    i = 2
    q_off = i * s
    q, k, v, do = rnd((B, s, Hq, D), 11), rnd((B, Nkv, Hkv, D), 12), rnd((B, Nkv, Hkv, D), 13), rnd((B, s, Hq, D), 14)

    def loss(q_, k_, v_):
        o, _ = attn_fwd(q_, k_, v_, q_off, 0, Nkv, True, scale)
        return float((o * do).sum())

    o, lse = attn_fwd(q, k, v, q_off, 0, Nkv, True, scale)
    dq, dk, dv = attn_bwd(q, k, v, o, do, lse, q_off, 0, Nkv, True, scale)
    # the same gradient as the sum of two partial-range calls that use the merged (out, lse)
    cut = 12                                           # inside the diagonal block
    dq1, dk1, dv1 = attn_bwd(q, k, v, o, do, lse, q_off, 0, cut, True, scale)
    dq2, dk2, dv2 = attn_bwd(q, k, v, o, do, lse, q_off, cut, Nkv, True, scale)
    np.testing.assert_allclose(dq1 + dq2, dq, atol=1e-13)
    np.testing.assert_allclose(dk1 + dk2, dk, atol=1e-13)
    np.testing.assert_allclose(dv1 + dv2, dv, atol=1e-13)
    assert np.all(dk1[:, cut:] == 0) and np.all(dv2[:, :cut] == 0)
    h = 1e-6
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            xp, xm = x.copy(), x.copy()
            xp[idx] += h
            xm[idx] -= h
            args_p = dict(q=q, k=k, v=v)
            args_m = dict(q=q, k=k, v=v)
            args_p[name], args_m[name] = xp, xm
            num[idx] = (loss(args_p["q"], args_p["k"], args_p["v"]) - loss(args_m["q"], args_m["k"], args_m["v"])) / (2 * h)
        rel = np.linalg.norm(num - g) / np.linalg.norm(num)
        assert rel < 1e-6, (name, rel)


# ---------------------------------------------------------------- closed forms
def test_zero_queries_count_visible_keys_exactly():
    B, s, Hq, Hkv, D, Nkv = 1, 9, 2, 2, 4, 40
    k, v = rnd((B, Nkv, Hkv, D), 15), rnd((B, Nkv, Hkv, D), 16)
    q = np.zeros((B, s, Hq, D))
    for (q_off, a, b, causal) in [(20, 0, 29, True), (20, 5, 24, True), (20, 22, 40, True), (3, 7, 30, True),
                                  (0, 0, 40, False), (20, 23, 23, True), (10, 12, 18, True)]:
        o, lse = attn_fwd(q, k, v, q_off, a, b, causal, 1.3)
        for r in range(s):
            hi = min(b, q_off + r + 1) if causal else b
            cnt = max(0, hi - a)
            for h in range(Hq):
                if cnt == 0:
                    assert lse[0, h, r] == -np.inf and np.all(o[0, r, h] == 0)
                else:
                    assert abs(lse[0, h, r] - math.log(cnt)) < 1e-13
                    np.testing.assert_allclose(o[0, r, h], v[0, a:hi, h].mean(axis=0), atol=1e-13)


def test_single_visible_key_returns_its_value_and_score():
    B, s, Hq, Hkv, D, Nkv = 1, 3, 4, 2, 5, 10
    q, k, v = rnd((B, s, Hq, D), 17), rnd((B, Nkv, Hkv, D), 18), rnd((B, Nkv, Hkv, D), 19)
    scale = 0.45
    o, lse = attn_fwd(q, k, v, 0, 0, Nkv, True, scale)       # row 0 sees key 0 only
    for h in range(Hq):
        g = h // 2
        np.testing.assert_allclose(o[0, 0, h], v[0, 0, g], atol=1e-14)
        assert abs(lse[0, h, 0] - scale * float(q[0, 0, h] @ k[0, 0, g])) < 1e-13
    o, lse = attn_fwd(q, k, v, 2, 6, 7, False, scale)         # range of one key
    for h in range(Hq):
        np.testing.assert_allclose(o[0, :, h], np.broadcast_to(v[0, 6, h // 2], (s, D)), atol=1e-14)
        np.testing.assert_allclose(lse[0, h], scale * (q[0, :, h] @ k[0, 6, h // 2]), atol=1e-13)


def test_equal_keys_give_mean_value_and_shift_invariance():
    B, s, H, D, Nkv = 1, 4, 2, 6, 12
    q, v = rnd((B, s, H, D), 20), rnd((B, Nkv, H, D), 21)
    k1 = rnd((B, 1, H, D), 22)
    k = np.repeat(k1, Nkv, axis=1)
    scale = 0.8
    o, lse = attn_fwd(q, k, v, 8, 0, Nkv, True, scale)
    for r in range(s):
        cnt = 8 + r + 1
        for h in range(H):
            np.testing.assert_allclose(o[0, r, h], v[0, :cnt, h].mean(axis=0), atol=1e-13)
            assert abs(lse[0, h, r] - (scale * float(q[0, r, h] @ k1[0, 0, h]) + math.log(cnt))) < 1e-12
    # adding one vector u to every key leaves out unchanged, shifts lse by scale*q.u
    k2 = rnd((B, Nkv, H, D), 23)
    u = rnd((D,), 24)
    o_a, lse_a = attn_fwd(q, k2, v, 8, 2, Nkv, True, scale)
    o_b, lse_b = attn_fwd(q, k2 + u, v, 8, 2, Nkv, True, scale)
    np.testing.assert_allclose(o_a, o_b, atol=1e-12)
    np.testing.assert_allclose(lse_b - lse_a, scale * np.einsum("bshd,d->bhs", q, u), atol=1e-12)


def test_rows_of_p_sum_to_one_and_rows_of_ds_to_zero():
    B, s, Hq, Hkv, D, Nkv = 1, 6, 2, 1, 4, 18
    q, k, do = rnd((B, s, Hq, D), 25), rnd((B, Nkv, Hkv, D), 26), rnd((B, s, Hq, D), 27)
    ones = np.ones((B, Nkv, Hkv, D))
    o, lse = attn_fwd(q, k, ones, 12, 0, Nkv, True, 0.5)
    np.testing.assert_allclose(o, 1.0, atol=1e-13)                    # sum_j p_ij = 1
    # sum_j dS_ij = 0  <=>  dq.(any u) = 0 when every key is shifted by u ... check via k = const rows:
    v = rnd((B, Nkv, Hkv, D), 28)
    o, lse = attn_fwd(q, k, v, 12, 0, Nkv, True, 0.5)
    dq, dk, dv = attn_bwd(q, k, v, o, do, lse, 12, 0, Nkv, True, 0.5)
    # loss is invariant to a common shift of all keys along q_i's direction only in lse, not out:
    # d/du loss = sum_j dk_j = scale * sum_h sum_i (sum_j dS_ij) q_i = 0
    np.testing.assert_allclose(dk.sum(axis=1), 0.0, atol=1e-12)


# ---------------------------------------------------------------- scalar brute force
def test_scalar_brute_force_fwd_bwd_tiny():
    B, s, Hq, Hkv, D, Nkv = 2, 3, 4, 2, 3, 11
    G = Hq // Hkv
    q_off, a, b_, scale = 6, 2, 10, 0.9
    q, k, v, do = rnd((B, s, Hq, D), 29), rnd((B, Nkv, Hkv, D), 30), rnd((B, Nkv, Hkv, D), 31), rnd((B, s, Hq, D), 32)
    o, lse = attn_fwd(q, k, v, q_off, a, b_, True, scale)
    dq, dk, dv = attn_bwd(q, k, v, o, do, lse, q_off, a, b_, True, scale)
    dq_ref, dk_ref, dv_ref = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            for r in range(s):
                J = [j for j in range(Nkv) if a <= j < b_ and j <= q_off + r]
                sc = {j: scale * math.fsum(q[b, r, h, d] * k[b, j, g, d] for d in range(D)) for j in J}
                Z = math.fsum(math.exp(sc[j]) for j in J)
                assert abs(lse[b, h, r] - math.log(Z)) < 1e-12
                p = {j: math.exp(sc[j]) / Z for j in J}
                orow = [math.fsum(p[j] * v[b, j, g, d] for j in J) for d in range(D)]
                np.testing.assert_allclose(o[b, r, h], orow, atol=1e-13)
                delta = math.fsum(do[b, r, h, d] * orow[d] for d in range(D))
                for j in J:
                    dp = math.fsum(do[b, r, h, d] * v[b, j, g, d] for d in range(D))
                    ds = p[j] * (dp - delta)
                    for d in range(D):
                        dv_ref[b, j, g, d] += p[j] * do[b, r, h, d]
                        dq_ref[b, r, h, d] += scale * ds * k[b, j, g, d]
                        dk_ref[b, j, g, d] += scale * ds * q[b, r, h, d]
    np.testing.assert_allclose(dq, dq_ref, atol=1e-12)
    np.testing.assert_allclose(dk, dk_ref, atol=1e-12)
    np.testing.assert_allclose(dv, dv_ref, atol=1e-12)


# ---------------------------------------------------------------- split / merge identities
@pytest.mark.parametrize("cuts", [[0, 12, 30], [0, 7, 7, 19, 30], [0, 25, 27, 30], [0, 1, 2, 3, 4, 5, 6, 30], [0, 30]])
def test_merge_of_any_split_equals_unsplit(cuts):
    B, s, Hq, Hkv, D = 2, 6, 4, 2, 8
    q_off, Nkv, scale = 24, 30, 0.35
    q, k, v, do = rnd((B, s, Hq, D), 33), rnd((B, Nkv, Hkv, D), 34), rnd((B, Nkv, Hkv, D), 35), rnd((B, s, Hq, D), 36)
    o, lse = attn_fwd(q, k, v, q_off, 0, Nkv, True, scale)
    parts = [attn_fwd(q, k, v, q_off, a, b, True, scale) for a, b in zip(cuts[:-1], cuts[1:])]
    om, lm = attn_merge([p[0] for p in parts], [p[1] for p in parts])
    np.testing.assert_allclose(om, o, atol=1e-12)
    np.testing.assert_allclose(lm, lse, atol=1e-12)
    dq, dk, dv = attn_bwd(q, k, v, o, do, lse, q_off, 0, Nkv, True, scale)
    acc = [np.zeros_like(dq), np.zeros_like(dk), np.zeros_like(dv)]
    for a, b in zip(cuts[:-1], cuts[1:]):
        for t, g_ in zip(acc, attn_bwd(q, k, v, om, do, lm, q_off, a, b, True, scale)):
            t += g_
    for t, ref in zip(acc, (dq, dk, dv)):
        np.testing.assert_allclose(t, ref, atol=1e-12)


def test_merge_weights_closed_form_and_all_empty():
    # two parts with lse ln(1), ln(3) -> weights 1/4, 3/4 and lse ln(4)
    o1, o2 = np.full((1, 1, 1, 2), 2.0), np.full((1, 1, 1, 2), 6.0)
    l1, l2 = np.full((1, 1, 1), 0.0), np.full((1, 1, 1), math.log(3.0))
    o, l = attn_merge([o1, o2], [l1, l2])
    np.testing.assert_allclose(o, 5.0, atol=1e-14)
    np.testing.assert_allclose(l, math.log(4.0), atol=1e-14)
    ninf = np.full((1, 1, 1), -np.inf)
    o, l = attn_merge([o1, o2], [ninf, l2])
    np.testing.assert_allclose(o, 6.0, atol=1e-14)
    o, l = attn_merge([np.zeros_like(o1), np.zeros_like(o1)], [ninf, ninf])
    assert np.all(o == 0) and np.all(l == -np.inf)


def test_fig_attn_balance_block_pattern():
    with open(os.path.join(GOLDEN, "attn_balance.json")) as f:
        fig = json.load(f)
    devs = fig["devices"]
    assert [len(d["blocks_before"]) for d in devs] == fig["loads_before"]
    after = [len(d["local"]) + sum(len(r["blocks"]) for r in d["remote"]) for d in devs]
    assert after == fig["loads_after"] and max(after) - min(after) <= 1
    s, Hq, Hkv, D, scale = 4, 2, 1, 4, 0.5
    nblk = 7
    k, v = rnd((1, nblk * s, Hkv, D), 37), rnd((1, nblk * s, Hkv, D), 38)
    for d in devs:
        qi = d["query"]                              # 1-based slice index; its diagonal block is block qi
        q = rnd((1, s, Hq, D), 100 + qi)
        q_off = (qi - 1) * s
        whole = attn_fwd(q, k, v, q_off, 0, qi * s, True, scale)
        pieces = [d["local"]] + [r["blocks"] for dd in devs for r in dd["remote"] if r["query"] == qi]
        assert sorted(b for p in pieces for b in p) == d["blocks_before"]
        parts = [attn_fwd(q, k, v, q_off, (p[0] - 1) * s, p[-1] * s, True, scale) for p in pieces]
        om, lm = attn_merge([p[0] for p in parts], [p[1] for p in parts])
        np.testing.assert_allclose(om, whole[0], atol=1e-12)
        np.testing.assert_allclose(lm, whole[1], atol=1e-12)
