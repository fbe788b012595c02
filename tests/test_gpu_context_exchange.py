"""The attention context exchange (paper Sec. 4.2.2) executed on one GPU: the planner's pieces of the
paper's picture (six devices, queries 7..2) are computed one by one as a helper device would, merged
with the owner's local part, and compared with the fp64 oracle of the undivided attention; backward
per piece with the merged (out, lse).  Everything on the GPU goes through the C ABI."""
import math

import numpy as np
import pytest

from oracle import attn_fwd, attn_bwd
from synth_inputs import normal_bf16, bf16_bits_to_f64
from gpu_util import say, dev_bf16, host_f64
from test_gpu_parity_small import check_fwd, check_grad

pytestmark = pytest.mark.gpu


def test_planned_pieces_merge_to_the_undivided_result():
    import torch
    import paper_2504_14519_amd as sp
    from paper_2504_14519_amd.planner import redistribute_pairwise, piece_key_range
    loads = [7, 6, 5, 4, 3, 2]
    B, s, Hq, Hkv, D = 1, 160, 4, 2, 128           # 160: slices that are no multiple of any tile
    N = max(loads) * s
    scale = 1.0 / math.sqrt(D)
    pieces, after = redistribute_pairwise(loads)
    assert after == [5, 5, 5, 4, 4, 4]
    kb, vb = normal_bf16((B, N, Hkv, D), 11, "k"), normal_bf16((B, N, Hkv, D), 11, "v")
    k64, v64 = bf16_bits_to_f64(kb), bf16_bits_to_f64(vb)
    k, v = dev_bf16(kb), dev_bf16(vb)
    for dev, load in enumerate(loads):
        qb, dob = normal_bf16((B, s, Hq, D), 11, "q", salt=dev), normal_bf16((B, s, Hq, D), 11, "do", salt=dev)
        q64, do64 = bf16_bits_to_f64(qb), bf16_bits_to_f64(dob)
        q, do = dev_bf16(qb), dev_bf16(dob)
        q_off = (load - 1) * s
        given = [pc for pc in pieces if pc[0] == dev]
        kept = load - sum(pc[3] - pc[2] + 1 for pc in given)
        ranges = [(0, kept * s)] + [piece_key_range(pc, s) for pc in given]
        say("device %d: query %d, key ranges %s" % (dev + 1, load, ranges))
        parts = [sp.slimpipe_attn_fwd(q, k, v, q_off, a, b, True, scale, out_dtype=sp.F32) for a, b in ranges]
        if len(parts) > 1:
            om, lm = sp.slimpipe_attn_merge([x[0] for x in parts], [x[1] for x in parts])
        else:
            om, lm = parts[0]
        torch.cuda.synchronize()
        o_ref, l_ref = attn_fwd(q64, k64, v64, q_off, 0, load * s, True, scale)
        check_fwd("device %d merged" % (dev + 1), om, lm, o_ref, l_ref, bf16_out=False)
        dk = torch.zeros((B, N, Hkv, D), device="cuda:0")
        dv = torch.zeros_like(dk)
        dq = torch.zeros((B, s, Hq, D), device="cuda:0")
        ob = om.to(torch.bfloat16)
        for a, b in ranges:
            sp.slimpipe_attn_bwd(q, k, v, ob, do, lm, q_off, a, b, dk, dv, True, scale, dq=dq, dq_dtype=sp.F32,
                                 dq_accumulate=True, dkv_accumulate=False)
        torch.cuda.synchronize()
        dq_r, dk_r, dv_r = attn_bwd(q64, k64, v64, host_f64(ob), do64, host_f64(lm), q_off, 0, load * s, True, scale)
        check_grad("device %d dq" % (dev + 1), dq, dq_r)
        check_grad("device %d dk" % (dev + 1), dk, dk_r)
        check_grad("device %d dv" % (dev + 1), dv, dv_r)
        assert np.all(host_f64(dk)[:, load * s:] == 0)
