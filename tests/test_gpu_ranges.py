"""Several key ranges of one query slice in one launch (the pieces of the paper's context exchange, Sec. 4.2.2)
and the automatic cut of a short slice over a long cache: HIP path vs the fp64 oracle through the C ABI."""
import math

import numpy as np
import pytest

from oracle import attn_fwd, attn_merge
from synth_inputs import normal_bf16, bf16_bits_to_f64
from gpu_util import say, dev_bf16, host_f64, max_abs, TOL_OUT, TOL_LSE
from test_gpu_parity_small import check_fwd

pytestmark = pytest.mark.gpu


def _inputs(B, s, N, Hq, Hkv, D, cfg):
    qb, kb, vb = normal_bf16((B, s, Hq, D), cfg, "q"), normal_bf16((B, N, Hkv, D), cfg, "k"), normal_bf16((B, N, Hkv, D), cfg, "v")
    return (bf16_bits_to_f64(qb), bf16_bits_to_f64(kb), bf16_bits_to_f64(vb)), (dev_bf16(qb), dev_bf16(kb), dev_bf16(vb))


@pytest.mark.parametrize("D,chunked", [(128, False), (128, True), (64, False)])
def test_ranges_in_one_launch(D, chunked):
    import torch
    import paper_2504_14519_amd as sp
    B, s, N, Hq, Hkv = 2, 320, 2048, 4, 2
    q_off = N - s
    scale = 1.0 / math.sqrt(D)
    (q64, k64, v64), (q, k, v) = _inputs(B, s, N, Hq, Hkv, D, 12)
    kk, vv = (k, v) if not chunked else ([k[:, i:i + 512].clone() for i in range(0, N, 512)], [v[:, i:i + 512].clone() for i in range(0, N, 512)])
    # a partition with an empty piece and unaligned cuts, then overlapping / gappy ranges (parts only)
    partition = [(0, 1000), (1000, 1000), (1000, q_off + 70), (q_off + 70, N)]
    say("fwd_ranges D=%d chunked=%s partition %s" % (D, chunked, partition))
    po, pl, om, lm = sp.slimpipe_attn_fwd_ranges(q, kk, vv, q_off, partition, True, scale, merged=True, out_dtype=sp.F32)
    torch.cuda.synchronize()
    refs = [attn_fwd(q64, k64, v64, q_off, a, b, True, scale) for a, b in partition]
    for r, (a, b) in enumerate(partition):
        check_fwd("  part [%d,%d)" % (a, b), po[r], pl[r], refs[r][0], refs[r][1], bf16_out=False)
    o_ref, l_ref = attn_fwd(q64, k64, v64, q_off, 0, N, True, scale)
    check_fwd("  merged", om, lm, o_ref, l_ref, bf16_out=False)
    # the merged result is what the merge entry point makes of the same parts, bit for bit
    om2, lm2 = sp.slimpipe_attn_merge([po[r] for r in range(len(partition))], [pl[r] for r in range(len(partition))], out_dtype=sp.F32)
    torch.cuda.synchronize()
    assert torch.equal(om, om2) and torch.equal(lm, lm2)
    # each part is what the one-range call returns, bit for bit
    for r, (a, b) in enumerate(partition):
        if chunked:
            o1, l1 = sp.slimpipe_attn_fwd_chunked(q, kk, vv, q_off, a, b, True, scale, out_dtype=sp.F32)
        else:
            o1, l1 = sp.slimpipe_attn_fwd(q, k, v, q_off, a, b, True, scale, out_dtype=sp.F32)
        torch.cuda.synchronize()
        assert torch.equal(o1, po[r]) and torch.equal(l1, pl[r]), (a, b)
    loose = [(300, 1900), (0, N), (1500, 1700), (N - 1, N)]
    say("fwd_ranges loose ranges %s" % loose)
    po, pl, none_o, none_l = sp.slimpipe_attn_fwd_ranges(q, kk, vv, q_off, loose, True, scale, merged=False)
    torch.cuda.synchronize()
    assert none_o is None and none_l is None
    for r, (a, b) in enumerate(loose):
        o_r, l_r = attn_fwd(q64, k64, v64, q_off, a, b, True, scale)
        check_fwd("  range [%d,%d)" % (a, b), po[r], pl[r], o_r, l_r, bf16_out=False)


def test_short_slice_over_long_cache_is_cut_into_ranges():
    import torch
    import paper_2504_14519_amd as sp
    B, s, N, Hq, Hkv, D = 1, 512, 8192, 4, 1, 128
    q_off = N - s - 100                    # the last 100 keys lie beyond every query
    kv_begin, kv_end = 200, N
    scale = 1.0 / math.sqrt(D)
    (q64, k64, v64), (q, k, v) = _inputs(B, s, N, Hq, Hkv, D, 13)
    out = torch.empty((B, s, Hq, D), device="cuda:0", dtype=torch.bfloat16)
    p = sp.make_params(q, k, out, q_off, kv_begin, kv_end, True, scale)
    need = sp.slimpipe_attn_workspace_bytes(p, False)
    per_range = B * s * Hq * D * 4 + B * Hq * s * 4
    ticket = 256          # the workspace starts with the counter the workgroups take their work items from
    assert need > ticket and (need - ticket) % per_range == 0, "8 workgroups on 256 compute units: the call is meant to ask for ranges"
    say("auto ranges: workspace %d bytes = counter + %d ranges" % (need, (need - ticket) // per_range))
    o_ref, l_ref = attn_fwd(q64, k64, v64, q_off, kv_begin, kv_end, True, scale)
    o0, l0 = sp.slimpipe_attn_fwd(q, k, v, q_off, kv_begin, kv_end, True, scale)
    res = []
    for nbytes in (need, need, ticket + 2 * per_range, ticket + per_range):
        ws = torch.full((nbytes,), 0xff, device="cuda:0", dtype=torch.uint8)       # NaN patterns: nothing stale may be read
        o, l = sp.slimpipe_attn_fwd(q, k, v, q_off, kv_begin, kv_end, True, scale, workspace=ws)
        torch.cuda.synchronize()
        check_fwd("  workspace %d" % nbytes, o, l, o_ref, l_ref)
        res.append((o, l))
    assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1])
    # room for one range only: the undivided computation, bit for bit
    assert torch.equal(res[3][0], o0) and torch.equal(res[3][1], l0)
    # the cut only reorders fp32 additions
    assert max_abs(host_f64(res[0][0]), host_f64(o0)) <= 2 ** -7 and max_abs(host_f64(res[0][1]), host_f64(l0)) <= 1e-5
    # a strided output (heads padded to 160 elements, rows interleaved with something else): same values
    big = torch.zeros((B, s, 2, Hq, 160), device="cuda:0", dtype=torch.bfloat16)
    view = big[:, :, 1, :, 16:16 + D]
    ws = torch.empty(need, device="cuda:0", dtype=torch.uint8)
    o_s, l_s = sp.slimpipe_attn_fwd(q, k, v, q_off, kv_begin, kv_end, True, scale, out=view, workspace=ws)
    torch.cuda.synchronize()
    assert o_s.data_ptr() == view.data_ptr() and torch.equal(view, res[0][0]) and torch.equal(l_s, res[0][1])
    assert float(big[:, :, 0].abs().max()) == 0.0 and float(big[..., :16].abs().max()) == 0.0 and float(big[..., 16 + D:].abs().max()) == 0.0
    # chunked cache, same call
    kc, vc = [k[:, i:i + 1024].clone() for i in range(0, N, 1024)], [v[:, i:i + 1024].clone() for i in range(0, N, 1024)]
    ws = torch.empty(need, device="cuda:0", dtype=torch.uint8)
    oc, lc = sp.slimpipe_attn_fwd_chunked(q, kc, vc, q_off, kv_begin, kv_end, True, scale, workspace=ws)
    torch.cuda.synchronize()
    check_fwd("  chunked", oc, lc, o_ref, l_ref)


@pytest.mark.parametrize("dq_dtype_name,accumulate", [("F32", True), ("BF16", False)])
def test_backward_of_a_short_slice_cuts_dq_into_key_ranges(dq_dtype_name, accumulate):
    import torch
    import paper_2504_14519_amd as sp
    from oracle import attn_bwd
    from gpu_util import rel_l2, TOL_GRAD
    B, s, N, Hq, Hkv, D = 2, 384, 4096, 2, 1, 128
    q_off, kv_begin, kv_end = N - s, 100, N - 37
    scale = 1.0 / math.sqrt(D)
    dq_dtype = getattr(sp, dq_dtype_name)
    (q64, k64, v64), (q, k, v) = _inputs(B, s, N, Hq, Hkv, D, 14)
    dob = normal_bf16((B, s, Hq, D), 14, "do")
    do64, do = bf16_bits_to_f64(dob), dev_bf16(dob)
    o, l = sp.slimpipe_attn_fwd(q, k, v, q_off, kv_begin, kv_end, True, scale)
    torch.cuda.synchronize()
    dq_ref, dk_ref, dv_ref = attn_bwd(q64, k64, v64, host_f64(o), do64, host_f64(l), q_off, kv_begin, kv_end, True, scale)
    p = sp.make_params(q, k, q, q_off, kv_begin, kv_end, True, scale)
    need = sp.slimpipe_attn_workspace_bytes(p, True)
    stats_only = 2 * (((B * Hq * s * 4) + 255) // 256 * 256)
    dq_part = B * s * Hq * D * 4
    assert need >= stats_only + 2 * dq_part, "4 query blocks on 256 compute units: the call is meant to ask for dq ranges"
    res = {}
    for name, nbytes in (("ranges", need), ("ranges again", need), ("undivided", stats_only)):
        say("dq %s (%s, accumulate %s): workspace %d bytes" % (name, dq_dtype_name, accumulate, nbytes))
        ws = torch.full((nbytes,), 0xff, device="cuda:0", dtype=torch.uint8)
        dk = torch.zeros((B, N, Hkv, D), device="cuda:0")
        dv = torch.zeros_like(dk)
        dq = torch.full((B, s, Hq, D), 0.25, device="cuda:0", dtype=torch.float32 if dq_dtype == sp.F32 else torch.bfloat16)
        sp.slimpipe_attn_bwd(q, k, v, o, do, l, q_off, kv_begin, kv_end, dk, dv, True, scale, dq=dq, dq_dtype=dq_dtype,
                             dq_accumulate=accumulate, dkv_accumulate=False, workspace=ws)
        torch.cuda.synchronize()
        got = host_f64(dq) - (0.25 if accumulate else 0.0)
        e = rel_l2(got, dq_ref)
        say("  dq rel-L2 %.3e" % e)
        assert e <= TOL_GRAD
        assert rel_l2(host_f64(dk), dk_ref) <= TOL_GRAD and rel_l2(host_f64(dv), dv_ref) <= TOL_GRAD
        res[name] = dq.float().cpu()
    assert torch.equal(res["ranges"], res["ranges again"])
    assert torch.allclose(res["ranges"], res["undivided"], rtol=2e-2 if dq_dtype == sp.BF16 else 1e-4, atol=1e-2 if dq_dtype == sp.BF16 else 1e-4)
