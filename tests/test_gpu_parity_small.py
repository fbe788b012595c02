"""HIP path vs fp64 oracle, element by element, at sizes the oracle finishes in seconds.
Everything goes through the C ABI (via the ctypes binding)."""
import math

import numpy as np
import pytest

from oracle import attn_fwd, attn_bwd, attn_merge
from synth_inputs import CONFIGS, normal_bf16, bf16_bits_to_f64
from gpu_util import say, dev_bf16, host_f64, rel_l2, max_abs, out_err, TOL_OUT, TOL_LSE, TOL_GRAD

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    import torch
    assert torch.cuda.is_available(), "needs the MI355X"
    import paper_2504_14519_amd as sp_
    return sp_


def check_fwd(name, o_gpu, lse_gpu, o_ref, lse_ref, bf16_out=True):
    eo, n_big = out_err(host_f64(o_gpu), o_ref, bf16_out)
    el = max_abs(host_f64(lse_gpu), lse_ref)       # also fails on NaN and on a differing -inf pattern
    say("%s: out max-abs %.3e  lse max-abs %.3e  (|out|>=4 elements held to half a bf16 ulp: %d)" % (name, eo, el, n_big))
    assert eo <= TOL_OUT, name
    assert el <= TOL_LSE, name


def check_grad(name, g_gpu, g_ref):
    e = rel_l2(host_f64(g_gpu), g_ref)
    say("%s: rel-L2 %.3e" % (name, e))
    assert e <= TOL_GRAD, name


def run_sliced(sp, cfg_id, B, N, n, Hq, Hkv, D, splits=()):
    import torch
    s = N // n
    scale = 1.0 / math.sqrt(D)
    qb, kb, vb, dob = (normal_bf16((B, N, H, D), cfg_id, t) for t, H in (("q", Hq), ("k", Hkv), ("v", Hkv), ("do", Hq)))
    q64, k64, v64, do64 = (bf16_bits_to_f64(x) for x in (qb, kb, vb, dob))
    q, k, v, do = (dev_bf16(x) for x in (qb, kb, vb, dob))
    dk_acc = torch.zeros((B, N, Hkv, D), device="cuda:0", dtype=torch.float32)
    dv_acc = torch.zeros_like(dk_acc)
    outs, lses = {}, {}
    for i in range(n):
        say("cfg%d fwd slice %d" % (cfg_id, i))
        o, l = sp.slimpipe_attn_fwd(q[:, i * s:(i + 1) * s], k, v, i * s, 0, (i + 1) * s, True, scale)
        torch.cuda.synchronize()
        o_ref, l_ref = attn_fwd(q64[:, i * s:(i + 1) * s], k64, v64, i * s, 0, (i + 1) * s, True, scale)
        check_fwd("cfg%d fwd slice %d" % (cfg_id, i), o, l, o_ref, l_ref)
        outs[i], lses[i] = (o, l), (o_ref, l_ref)
    dk_ref = np.zeros((B, N, Hkv, D))
    dv_ref = np.zeros((B, N, Hkv, D))
    dk_e2e = np.zeros((B, N, Hkv, D))
    dv_e2e = np.zeros((B, N, Hkv, D))
    for i in reversed(range(n)):
        say("cfg%d bwd slice %d" % (cfg_id, i))
        sl = slice(i * s, (i + 1) * s)
        o, l = outs[i]
        dq = sp.slimpipe_attn_bwd(q[:, sl], k, v, o, do[:, sl], l, i * s, 0, (i + 1) * s, dk_acc, dv_acc, True, scale,
                                  dq_dtype=sp.F32, dkv_accumulate=True)
        torch.cuda.synchronize()
        # (1) the call's own contract: the oracle gets exactly what the kernel got, the bf16 out and fp32 lse of the forward
        dq_r, dk_r, dv_r = attn_bwd(q64[:, sl], k64, v64, host_f64(o), do64[:, sl], host_f64(l), i * s, 0, (i + 1) * s, True, scale)
        check_grad("cfg%d dq slice %d" % (cfg_id, i), dq, dq_r)
        dk_ref += dk_r
        dv_ref += dv_r
        # (2) end to end: GPU forward -> GPU backward against oracle forward -> oracle backward (nothing of the GPU's enters)
        o_ref, l_ref = lses[i]
        dq_e, dk_e, dv_e = attn_bwd(q64[:, sl], k64, v64, o_ref, do64[:, sl], l_ref, i * s, 0, (i + 1) * s, True, scale)
        check_grad("cfg%d dq slice %d, oracle-only chain" % (cfg_id, i), dq, dq_e)
        dk_e2e += dk_e
        dv_e2e += dv_e
    check_grad("cfg%d dk (all slices)" % cfg_id, dk_acc, dk_ref)
    check_grad("cfg%d dv (all slices)" % cfg_id, dv_acc, dv_ref)
    check_grad("cfg%d dk (all slices), oracle-only chain" % cfg_id, dk_acc, dk_e2e)
    check_grad("cfg%d dv (all slices), oracle-only chain" % cfg_id, dv_acc, dv_e2e)
    dk_b = sp.slimpipe_attn_finalize_bf16(dk_acc)
    check_grad("cfg%d dk finalized bf16" % cfg_id, dk_b, dk_ref)
    check_grad("cfg%d dk finalized bf16, oracle-only chain" % cfg_id, dk_b, dk_e2e)

    i = n - 1
    sl = slice(i * s, (i + 1) * s)
    for cuts in splits:
        say("cfg%d split of last slice at %s" % (cfg_id, cuts))
        edges = [0] + list(cuts) + [N]
        parts = [sp.slimpipe_attn_fwd(q[:, sl], k, v, i * s, a, b, True, scale, out_dtype=sp.F32) for a, b in zip(edges[:-1], edges[1:])]
        om, lm = sp.slimpipe_attn_merge([p[0] for p in parts], [p[1] for p in parts])
        torch.cuda.synchronize()
        for (po, pl), a, b in zip(parts, edges[:-1], edges[1:]):
            r_o, r_l = attn_fwd(q64[:, sl], k64, v64, i * s, a, b, True, scale)
            check_fwd("  part [%d,%d)" % (a, b), po, pl, r_o, r_l, bf16_out=False)
        check_fwd("  merged", om, lm, lses[i][0], lses[i][1])
        # oracle merge of the oracle parts equals the unsplit oracle result (identity of the method)
        # backward per part with the merged (out, lse); dq summed, dk/dv placed per range
        dk2 = torch.zeros_like(dk_acc)
        dv2 = torch.zeros_like(dk_acc)
        dq2 = torch.zeros((B, s, Hq, D), device="cuda:0", dtype=torch.float32)
        for a, b in zip(edges[:-1], edges[1:]):
            sp.slimpipe_attn_bwd(q[:, sl], k, v, om, do[:, sl], lm, i * s, a, b, dk2, dv2, True, scale,
                                 dq=dq2, dq_dtype=sp.F32, dq_accumulate=True, dkv_accumulate=False)
        torch.cuda.synchronize()
        dq_r, dk_r, dv_r = attn_bwd(q64[:, sl], k64, v64, host_f64(om), do64[:, sl], host_f64(lm), i * s, 0, N, True, scale)
        check_grad("  split dq", dq2, dq_r)
        check_grad("  split dk", dk2, dk_r)
        check_grad("  split dv", dv2, dv_r)
        # oracle-only chain of the split: oracle parts -> oracle merge -> oracle backward per part, dq summed
        po = [attn_fwd(q64[:, sl], k64, v64, i * s, a, b, True, scale) for a, b in zip(edges[:-1], edges[1:])]
        om_r, lm_r = attn_merge([x[0] for x in po], [x[1] for x in po])
        dq_e, dk_e, dv_e = np.zeros_like(dq_r), np.zeros_like(dk_r), np.zeros_like(dv_r)
        for a, b in zip(edges[:-1], edges[1:]):
            g = attn_bwd(q64[:, sl], k64, v64, om_r, do64[:, sl], lm_r, i * s, a, b, True, scale)
            dq_e += g[0]; dk_e += g[1]; dv_e += g[2]
        check_grad("  split dq, oracle-only chain", dq2, dq_e)
        check_grad("  split dk, oracle-only chain", dk2, dk_e)
        check_grad("  split dv, oracle-only chain", dv2, dv_e)


def test_config_tiny_full(sp):
    c = CONFIGS[0]
    run_sliced(sp, 0, 1, c["N"], c["n"], c["Hq"], c["Hkv"], c["D"], splits=[(1024,), (1500,), (1800,), (512, 1537, 2000)])


def test_d128_gqa_sliced_full(sp):
    run_sliced(sp, 5, 1, 1536, 3, 8, 2, 128, splits=[(700,), (1100, 1300)])


@pytest.mark.parametrize("D", [64, 128])
def test_ragged_unaligned_strided(sp, D):
    """s_q, the range ends and q_offset are not multiples of any tile; batch 2; GQA; q/k/v are views
    with padded strides; covers range starting inside / ending inside the diagonal block."""
    import torch
    B, s, Hq, Hkv, Nkv = 2, 200, 4, 2, 777
    scale = 0.11
    qb = normal_bf16((B, s, Hq, D + 8), 6, "q", salt=D)
    kb = normal_bf16((B, Nkv, Hkv + 1, D), 6, "k", salt=D)
    vb = normal_bf16((B, Nkv, Hkv + 1, D), 6, "v", salt=D)
    dob = normal_bf16((B, s, Hq, D), 6, "do", salt=D)
    q = dev_bf16(qb)[..., :D]
    k = dev_bf16(kb)[:, :, :Hkv]
    v = dev_bf16(vb)[:, :, :Hkv]
    do = dev_bf16(dob)
    q64, k64, v64, do64 = bf16_bits_to_f64(qb)[..., :D], bf16_bits_to_f64(kb)[:, :, :Hkv], bf16_bits_to_f64(vb)[:, :, :Hkv], bf16_bits_to_f64(dob)
    cases = [(500, 13, 650, True), (500, 0, 777, True), (500, 601, 777, True), (0, 0, 200, True), (3, 1, 777, False),
             (500, 700, 777, True), (100, 290, 310, True)]
    for (q_off, a, b, causal) in cases:
        name = "ragged D%d q_off %d range [%d,%d) causal %d" % (D, q_off, a, b, causal)
        say(name)
        o, l = sp.slimpipe_attn_fwd(q, k, v, q_off, a, b, causal, scale, out_dtype=sp.F32)
        torch.cuda.synchronize()
        o_ref, l_ref = attn_fwd(q64, k64, v64, q_off, a, b, causal, scale)
        check_fwd(name, o, l, o_ref, l_ref, bf16_out=False)
        ob = o.to(torch.bfloat16)
        dk_acc = torch.full((B, Nkv, Hkv + 1, D), 7.0, device="cuda:0", dtype=torch.float32)[:, :, :Hkv]
        dv_acc = torch.full((B, Nkv, Hkv + 1, D), 7.0, device="cuda:0", dtype=torch.float32)[:, :, :Hkv]
        dq = torch.empty((B, s, Hq, D + 8), device="cuda:0", dtype=torch.bfloat16)[..., :D]
        sp.slimpipe_attn_bwd(q, k, v, ob, do, l, q_off, a, b, dk_acc, dv_acc, causal, scale, dq=dq, dq_dtype=sp.BF16,
                             dkv_accumulate=False)
        torch.cuda.synchronize()
        dq_r, dk_r, dv_r = attn_bwd(q64, k64, v64, host_f64(ob), do64, host_f64(l), q_off, a, b, causal, scale)
        if np.linalg.norm(dq_r) > 0:
            check_grad(name + " dq", dq, dq_r)
            check_grad(name + " dk", dk_acc[:, a:b], dk_r[:, a:b])
            check_grad(name + " dv", dv_acc[:, a:b], dv_r[:, a:b])
        else:
            assert float(dq.float().abs().max()) == 0.0
        # rows outside the range are untouched
        hk = host_f64(dk_acc)
        assert np.all(hk[:, :a] == 7.0) and np.all(hk[:, b:] == 7.0), name
        hv = host_f64(dv_acc)
        assert np.all(hv[:, :a] == 7.0) and np.all(hv[:, b:] == 7.0), name


def test_empty_range_and_rows_without_keys(sp):
    import torch
    B, s, Hq, Hkv, D, Nkv = 1, 96, 2, 1, 128, 256
    qb, kb, vb, dob = normal_bf16((B, s, Hq, D), 7, "q"), normal_bf16((B, Nkv, Hkv, D), 7, "k"), normal_bf16((B, Nkv, Hkv, D), 7, "v"), normal_bf16((B, s, Hq, D), 7, "do")
    q, k, v, do = dev_bf16(qb), dev_bf16(kb), dev_bf16(vb), dev_bf16(dob)
    for (q_off, a, b) in [(100, 50, 50), (100, 230, 256), (100, 150, 256)]:
        say("empty/partly empty: q_off %d range [%d,%d)" % (q_off, a, b))
        o, l = sp.slimpipe_attn_fwd(q, k, v, q_off, a, b, True, 0.09, out_dtype=sp.F32)
        torch.cuda.synchronize()
        o_ref, l_ref = attn_fwd(bf16_bits_to_f64(qb), bf16_bits_to_f64(kb), bf16_bits_to_f64(vb), q_off, a, b, True, 0.09)
        check_fwd("empty case", o, l, o_ref, l_ref, bf16_out=False)
        assert not np.isnan(host_f64(o)).any()
        dk_acc = torch.zeros((B, Nkv, Hkv, D), device="cuda:0")
        dv_acc = torch.zeros_like(dk_acc)
        dq = sp.slimpipe_attn_bwd(q, k, v, o.to(torch.bfloat16), do, l, q_off, a, b, dk_acc, dv_acc, True, 0.09, dq_dtype=sp.F32)
        torch.cuda.synchronize()
        for t in (dq, dk_acc, dv_acc):
            assert not torch.isnan(t).any()
        dq_r, dk_r, dv_r = attn_bwd(bf16_bits_to_f64(qb), bf16_bits_to_f64(kb), bf16_bits_to_f64(vb), host_f64(o.to(torch.bfloat16)),
                                    bf16_bits_to_f64(dob), host_f64(l), q_off, a, b, True, 0.09)
        assert max_abs(host_f64(dq), dq_r) < 1e-2 * max(1.0, np.abs(dq_r).max())
        rows_empty = np.isneginf(l_ref[0, 0])
        assert np.all(host_f64(dq)[0, rows_empty] == 0)


def test_dkdv_bit_reproducible(sp):
    import torch
    B, s, Hq, Hkv, D, Nkv = 1, 512, 8, 1, 128, 1024
    qb, kb, vb, dob = normal_bf16((B, s, Hq, D), 8, "q"), normal_bf16((B, Nkv, Hkv, D), 8, "k"), normal_bf16((B, Nkv, Hkv, D), 8, "v"), normal_bf16((B, s, Hq, D), 8, "do")
    q, k, v, do = dev_bf16(qb), dev_bf16(kb), dev_bf16(vb), dev_bf16(dob)
    o, l = sp.slimpipe_attn_fwd(q, k, v, 512, 0, 1024, True, None)
    res = []
    for rep in range(3):
        say("determinism run %d" % rep)
        dk_acc = torch.zeros((B, Nkv, Hkv, D), device="cuda:0")
        dv_acc = torch.zeros_like(dk_acc)
        dq = sp.slimpipe_attn_bwd(q, k, v, o, do, l, 512, 0, 1024, dk_acc, dv_acc, True, None, dq_dtype=sp.F32)
        torch.cuda.synchronize()
        res.append((dk_acc.cpu(), dv_acc.cpu(), dq.cpu()))
    for r in res[1:]:
        assert torch.equal(r[0], res[0][0]) and torch.equal(r[1], res[0][1]) and torch.equal(r[2], res[0][2])


def test_more_work_items_than_compute_units_d64(sp):
    """head_dim 64 at a size where all three attention kernels have more work items than the GPU has compute units, so
    that workgroups take their items from the counter in the workspace:
    every element against the oracle, and two runs bit-equal although workgroups and items pair up differently."""
    import torch
    B, s, Hq, Hkv, D, q_off = 1, 1100, 56, 56, 64, 256
    Nkv = q_off + s
    scale = 1.0 / math.sqrt(D)
    qb, kb, vb, dob = normal_bf16((B, s, Hq, D), 11, "q"), normal_bf16((B, Nkv, Hkv, D), 11, "k"), normal_bf16((B, Nkv, Hkv, D), 11, "v"), normal_bf16((B, s, Hq, D), 11, "do")
    q64, k64, v64, do64 = (bf16_bits_to_f64(x) for x in (qb, kb, vb, dob))
    q, k, v, do = dev_bf16(qb), dev_bf16(kb), dev_bf16(vb), dev_bf16(dob)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert (s + 255) // 256 * Hq * B > cus and (Nkv + 255) // 256 * Hkv * B > cus, "this shape is meant to exceed the compute units"
    p = sp.make_params(q, k, q, q_off, 0, Nkv, True, scale)
    fws = torch.empty(sp.slimpipe_attn_workspace_bytes(p, False), device="cuda:0", dtype=torch.uint8)
    bws = torch.empty(sp.slimpipe_attn_workspace_bytes(p, True), device="cuda:0", dtype=torch.uint8)
    runs = []
    for rep in range(2):
        say("more items than compute units, D 64: run %d" % rep)
        o, l = sp.slimpipe_attn_fwd(q, k, v, q_off, 0, Nkv, True, scale, workspace=fws)
        dk_acc = torch.zeros((B, Nkv, Hkv, D), device="cuda:0")
        dv_acc = torch.zeros_like(dk_acc)
        dq = sp.slimpipe_attn_bwd(q, k, v, o, do, l, q_off, 0, Nkv, dk_acc, dv_acc, True, scale, dq_dtype=sp.F32,
                                  dkv_accumulate=False, workspace=bws)
        torch.cuda.synchronize()
        runs.append((o, l, dq, dk_acc, dv_acc))
    for a, b in zip(runs[0], runs[1]):
        assert torch.equal(a, b)
    o, l, dq, dk_acc, dv_acc = runs[0]
    say("oracle")
    o_ref, l_ref = attn_fwd(q64, k64, v64, q_off, 0, Nkv, True, scale)
    check_fwd("D 64, counter-driven forward", o, l, o_ref, l_ref)
    dq_r, dk_r, dv_r = attn_bwd(q64, k64, v64, o_ref, do64, l_ref, q_off, 0, Nkv, True, scale)
    check_grad("D 64, counter-driven dq, oracle-only chain", dq, dq_r)
    check_grad("D 64, counter-driven dk, oracle-only chain", dk_acc, dk_r)
    check_grad("D 64, counter-driven dv, oracle-only chain", dv_acc, dv_r)


def test_dkdv_split_query_stream(sp):
    """Few key tiles and a long query stream: the dk/dv kernel cuts the stream of every key tile into
    chunks (partial sums + reduce kernel).  Checked against the oracle, against the unsplit path
    (workspace too small for partial sums) and for bit-reproducibility, with and without accumulation."""
    import torch
    B, s, Hq, Hkv, D, Nkv, q_off = 1, 2048, 4, 2, 128, 2304, 256
    scale = 1.0 / math.sqrt(D)
    qb, kb, vb, dob = normal_bf16((B, s, Hq, D), 9, "q"), normal_bf16((B, Nkv, Hkv, D), 9, "k"), normal_bf16((B, Nkv, Hkv, D), 9, "v"), normal_bf16((B, s, Hq, D), 9, "do")
    q64, k64, v64, do64 = (bf16_bits_to_f64(x) for x in (qb, kb, vb, dob))
    q, k, v, do = dev_bf16(qb), dev_bf16(kb), dev_bf16(vb), dev_bf16(dob)
    kv_end = q_off + s - 100            # ragged end: the last key tile is partial, the last rows see all keys
    p = sp.make_params(q, k, q, q_off, 0, kv_end, True, scale)
    need = sp.slimpipe_attn_workspace_bytes(p, True)
    stats_only = 2 * (((B * Hq * s * 4) + 255) // 256 * 256)
    assert need > stats_only, "this shape is meant to ask for a split"
    o, l = sp.slimpipe_attn_fwd(q, k, v, q_off, 0, kv_end, True, scale)
    torch.cuda.synchronize()
    o_ref, l_ref = attn_fwd(q64, k64, v64, q_off, 0, kv_end, True, scale)
    dq_ref, dk_ref, dv_ref = attn_bwd(q64, k64, v64, host_f64(o), do64, host_f64(l), q_off, 0, kv_end, True, scale)
    res = {}
    for name, ws_bytes in (("split", need), ("split again", need), ("unsplit", stats_only)):
        say("dk/dv %s: workspace %d bytes" % (name, ws_bytes))
        ws = torch.empty(ws_bytes, device="cuda:0", dtype=torch.uint8)
        dk_acc = torch.full((B, Nkv, Hkv, D), 0.5, device="cuda:0")
        dv_acc = torch.full((B, Nkv, Hkv, D), -0.25, device="cuda:0")
        sp.slimpipe_attn_bwd(q, k, v, o, do, l, q_off, 0, kv_end, dk_acc, dv_acc, True, scale, dq_dtype=sp.F32,
                             dkv_accumulate=True, workspace=ws)
        torch.cuda.synchronize()
        res[name] = (dk_acc.cpu(), dv_acc.cpu())
        dk_g, dv_g = host_f64(dk_acc), host_f64(dv_acc)
        check_grad("dk (%s)" % name, dk_acc[:, :kv_end] - 0.5, dk_ref[:, :kv_end])
        check_grad("dv (%s)" % name, dv_acc[:, :kv_end] + 0.25, dv_ref[:, :kv_end])
        # rows outside [kv_begin, kv_end) are untouched
        assert np.all(dk_g[:, kv_end:] == 0.5) and np.all(dv_g[:, kv_end:] == -0.25)
    assert torch.equal(res["split"][0], res["split again"][0]) and torch.equal(res["split"][1], res["split again"][1])
    # the split only changes the order of fp32 additions
    assert torch.allclose(res["split"][0], res["unsplit"][0], rtol=1e-4, atol=1e-4)
    assert torch.allclose(res["split"][1], res["unsplit"][1], rtol=1e-4, atol=1e-4)


@pytest.mark.parametrize("kv_begin,kv_end", [(0, 2048), (300, 1900)])
def test_chunked_kv(sp, kv_begin, kv_end):
    """K/V (and the dK/dV accumulators) as a list of slice-sized chunks that are separate allocations:
    same results as the oracle on the concatenated prefix; with an aligned range bit-identical to the
    contiguous calls (the tile walk is the same), with an unaligned one within the tolerances."""
    import torch
    B, s, Hq, Hkv, D, chunk, nch = 1, 512, 4, 2, 128, 512, 4
    N, q_off = chunk * nch, 1536
    scale = 1.0 / math.sqrt(D)
    qb, kb, vb, dob = normal_bf16((B, s, Hq, D), 10, "q"), normal_bf16((B, N, Hkv, D), 10, "k"), normal_bf16((B, N, Hkv, D), 10, "v"), normal_bf16((B, s, Hq, D), 10, "do")
    q64, k64, v64, do64 = (bf16_bits_to_f64(x) for x in (qb, kb, vb, dob))
    q, k, v, do = dev_bf16(qb), dev_bf16(kb), dev_bf16(vb), dev_bf16(dob)
    # separate allocations in shuffled order, with something else allocated in between
    order = [2, 0, 3, 1]
    kc, vc, pad = [None] * nch, [None] * nch, []
    for i in order:
        kc[i] = k[:, i * chunk:(i + 1) * chunk].clone()
        pad.append(torch.empty(4096 + 512 * i, device="cuda:0"))
        vc[i] = v[:, i * chunk:(i + 1) * chunk].clone()
    say("chunked fwd [%d, %d)" % (kv_begin, kv_end))
    o_c, l_c = sp.slimpipe_attn_fwd_chunked(q, kc, vc, q_off, kv_begin, kv_end, True, scale)
    o_f, l_f = sp.slimpipe_attn_fwd(q, k, v, q_off, kv_begin, kv_end, True, scale)
    torch.cuda.synchronize()
    o_ref, l_ref = attn_fwd(q64, k64, v64, q_off, kv_begin, kv_end, True, scale)
    check_fwd("chunked fwd", o_c, l_c, o_ref, l_ref)
    dq_ref, dk_ref, dv_ref = attn_bwd(q64, k64, v64, host_f64(o_c), do64, host_f64(l_c), q_off, kv_begin, kv_end, True, scale)
    dkc = [torch.full((B, chunk, Hkv, D), 1.0, device="cuda:0") for _ in range(nch)]
    dvc = [torch.full((B, chunk, Hkv, D), -2.0, device="cuda:0") for _ in range(nch)]
    say("chunked bwd")
    dq_c = sp.slimpipe_attn_bwd_chunked(q, kc, vc, o_c, do, l_c, q_off, kv_begin, kv_end, dkc, dvc, True, scale, dq_dtype=sp.F32,
                                        dkv_accumulate=True)
    dk_f = torch.full((B, N, Hkv, D), 1.0, device="cuda:0")
    dv_f = torch.full((B, N, Hkv, D), -2.0, device="cuda:0")
    dq_f = sp.slimpipe_attn_bwd(q, k, v, o_c, do, l_c, q_off, kv_begin, kv_end, dk_f, dv_f, True, scale, dq_dtype=sp.F32,
                                dkv_accumulate=True)
    torch.cuda.synchronize()
    dk_c, dv_c = torch.cat(dkc, dim=1), torch.cat(dvc, dim=1)
    check_grad("chunked dq", dq_c, dq_ref)
    check_grad("chunked dk", dk_c[:, kv_begin:kv_end] - 1.0, dk_ref[:, kv_begin:kv_end])
    check_grad("chunked dv", dv_c[:, kv_begin:kv_end] + 2.0, dv_ref[:, kv_begin:kv_end])
    # rows outside the range are untouched
    outside = torch.ones(N, dtype=torch.bool); outside[kv_begin:kv_end] = False
    assert torch.all(dk_c.cpu()[:, outside] == 1.0) and torch.all(dv_c.cpu()[:, outside] == -2.0)
    if kv_begin % 256 == 0:
        assert torch.equal(o_c, o_f) and torch.equal(l_c, l_f) and torch.equal(dq_c, dq_f)
        assert torch.equal(dk_c, dk_f) and torch.equal(dv_c, dv_f)
    else:
        assert torch.allclose(dq_c, dq_f, rtol=1e-3, atol=1e-3) and torch.allclose(dk_c, dk_f, rtol=1e-3, atol=1e-3)
        assert torch.allclose(dv_c, dv_f, rtol=1e-3, atol=1e-3)
    del pad


@pytest.mark.parametrize("s,Nkv,q_off,Hq,Hkv,D", [(1, 1, 0, 1, 1, 128), (1, 300, 299, 2, 1, 64), (5, 3, 0, 3, 3, 128), (33, 65, 32, 2, 2, 64)])
def test_smallest_shapes(sp, s, Nkv, q_off, Hq, Hkv, D):
    """One query row, one key, fewer rows than a wave owns: every tile is a ragged tail."""
    import torch
    B = 1
    scale = 1.0 / math.sqrt(D)
    qb, kb, vb, dob = normal_bf16((B, s, Hq, D), 15, "q", salt=s), normal_bf16((B, Nkv, Hkv, D), 15, "k", salt=s), normal_bf16((B, Nkv, Hkv, D), 15, "v", salt=s), normal_bf16((B, s, Hq, D), 15, "do", salt=s)
    q64, k64, v64, do64 = (bf16_bits_to_f64(x) for x in (qb, kb, vb, dob))
    q, k, v, do = dev_bf16(qb), dev_bf16(kb), dev_bf16(vb), dev_bf16(dob)
    name = "smallest s=%d Nkv=%d q_off=%d" % (s, Nkv, q_off)
    say(name)
    o, l = sp.slimpipe_attn_fwd(q, k, v, q_off, 0, Nkv, True, scale, out_dtype=sp.F32)
    torch.cuda.synchronize()
    o_ref, l_ref = attn_fwd(q64, k64, v64, q_off, 0, Nkv, True, scale)
    check_fwd(name, o, l, o_ref, l_ref, bf16_out=False)
    ob = o.to(torch.bfloat16)
    dk_acc = torch.zeros((B, Nkv, Hkv, D), device="cuda:0")
    dv_acc = torch.zeros_like(dk_acc)
    dq = sp.slimpipe_attn_bwd(q, k, v, ob, do, l, q_off, 0, Nkv, dk_acc, dv_acc, True, scale, dq_dtype=sp.F32, dkv_accumulate=False)
    torch.cuda.synchronize()
    dq_r, dk_r, dv_r = attn_bwd(q64, k64, v64, host_f64(ob), do64, host_f64(l), q_off, 0, Nkv, True, scale)
    check_grad(name + " dq", dq, dq_r)
    check_grad(name + " dk", dk_acc, dk_r)
    check_grad(name + " dv", dv_acc, dv_r)
