"""Every output of the library sits inside a larger allocation whose other bytes are poisoned; after the calls the
poison must be intact: no kernel writes before or behind out, lse, dq, the dk/dv accumulators (nor into their rows
outside the key range), the workspace or the merge outputs.  Ragged shapes, so that every tile has a tail."""
import math

import pytest

from synth_inputs import normal_bf16
from gpu_util import say, dev_bf16

pytestmark = pytest.mark.gpu

GUARD = 4096          # elements of poison on either side


class Guarded:
    """A tensor of `shape` carved out of the middle of a poisoned 1-D allocation."""
    def __init__(self, torch, shape, dtype, poison):
        n = 1
        for x in shape:
            n *= x
        self.raw = torch.full((n + 2 * GUARD,), poison, device="cuda:0", dtype=dtype)
        self.view = self.raw[GUARD:GUARD + n].view(*shape)
        self.n, self.poison, self.torch = n, poison, torch

    def intact(self):
        t = self.torch
        ref = t.full((GUARD,), self.poison, device="cuda:0", dtype=self.raw.dtype)
        as_int = {2: t.int16, 4: t.int32, 1: t.uint8}[self.raw.element_size()]
        return bool(t.equal(self.raw[:GUARD].view(as_int), ref.view(as_int)) and
                    t.equal(self.raw[GUARD + self.n:].view(as_int), ref.view(as_int)))


@pytest.mark.parametrize("D", [64, 128])
def test_no_write_outside_the_outputs(D):
    import torch
    import paper_2504_14519_amd as sp
    B, s, Hq, Hkv, Nkv = 2, 203, 4, 2, 1531
    scale = 1.0 / math.sqrt(D)
    mk = lambda shape, t: dev_bf16(normal_bf16(shape, 18, t, salt=D))
    q, k, v, do = mk((B, s, Hq, D), "q"), mk((B, Nkv, Hkv, D), "k"), mk((B, Nkv, Hkv, D), "v"), mk((B, s, Hq, D), "do")
    for (q_off, a, b) in [(1300, 0, 1531), (1200, 77, 1403), (0, 0, 203), (1328, 1200, 1531)]:
        for out_dtype, tdt in ((sp.BF16, torch.bfloat16), (sp.F32, torch.float32)):
            name = "guards D%d q_off %d keys [%d,%d) out %s" % (D, q_off, a, b, "bf16" if out_dtype == sp.BF16 else "f32")
            say(name)
            out = Guarded(torch, (B, s, Hq, D), tdt, 7.0)
            lse = Guarded(torch, (B, Hq, s), torch.float32, 7.0)
            p = sp.make_params(q, k, out.view, q_off, a, b, True, scale, out_dtype)
            fws = Guarded(torch, (max(256, sp.slimpipe_attn_workspace_bytes(p, False)),), torch.uint8, 0x5A)
            sp.slimpipe_attn_fwd(q, k, v, q_off, a, b, True, scale, out_dtype=out_dtype, out=out.view, lse=lse.view, workspace=fws.view)
            torch.cuda.synchronize()
            assert out.intact() and lse.intact() and fws.intact(), name + ": forward wrote outside its outputs"
            assert not torch.isnan(out.view.float()).any()
            if out_dtype == sp.F32:
                continue
            for dq_dtype, qdt in ((sp.BF16, torch.bfloat16), (sp.F32, torch.float32)):
                dq = Guarded(torch, (B, s, Hq, D), qdt, 7.0)
                dk = Guarded(torch, (B, Nkv, Hkv, D), torch.float32, 7.0)
                dv = Guarded(torch, (B, Nkv, Hkv, D), torch.float32, 7.0)
                dk.view.fill_(3.0)
                dv.view.fill_(-3.0)
                pb = sp.make_params(q, k, out.view, q_off, a, b, True, scale)
                ws = Guarded(torch, (sp.slimpipe_attn_workspace_bytes(pb, True),), torch.uint8, 0x5A)
                sp.slimpipe_attn_bwd(q, k, v, out.view, do, lse.view, q_off, a, b, dk.view, dv.view, True, scale, dq=dq.view,
                                     dq_dtype=dq_dtype, dkv_accumulate=False, workspace=ws.view)
                torch.cuda.synchronize()
                assert dq.intact() and dk.intact() and dv.intact() and ws.intact(), name + ": backward wrote outside its outputs"
                assert out.intact() and lse.intact(), name + ": backward wrote next to its inputs"
                # rows of the accumulators outside [a, b) keep what they held
                assert bool((dk.view[:, :a] == 3.0).all() and (dk.view[:, b:] == 3.0).all())
                assert bool((dv.view[:, :a] == -3.0).all() and (dv.view[:, b:] == -3.0).all())
                assert torch.isfinite(dq.view.float()).all() and torch.isfinite(dk.view).all() and torch.isfinite(dv.view).all()


def test_no_write_outside_ranges_merge_and_finalize():
    import torch
    import paper_2504_14519_amd as sp
    B, s, Hq, Hkv, D, Nkv, q_off = 1, 333, 4, 1, 128, 2049, 1716
    mk = lambda shape, t: dev_bf16(normal_bf16(shape, 19, t))
    q, k, v = mk((B, s, Hq, D), "q"), mk((B, Nkv, Hkv, D), "k"), mk((B, Nkv, Hkv, D), "v")
    ranges = [(0, 700), (700, 1500), (1500, 2049)]
    say("guards: three ranges in one launch, parts + merged")
    po, pl, om, lm = sp.slimpipe_attn_fwd_ranges(q, k, v, q_off, ranges, True, None)
    # the same through guarded buffers: parts one call each, then the merge and the final rounding
    parts = []
    for a, b in ranges:
        o = Guarded(torch, (B, s, Hq, D), torch.float32, 7.0)
        l = Guarded(torch, (B, Hq, s), torch.float32, 7.0)
        sp.slimpipe_attn_fwd(q, k, v, q_off, a, b, True, None, out_dtype=sp.F32, out=o.view, lse=l.view)
        parts.append((o, l))
    mo = Guarded(torch, (B, s, Hq, D), torch.bfloat16, 7.0)
    ml = Guarded(torch, (B, Hq, s), torch.float32, 7.0)
    sp.slimpipe_attn_merge([x[0].view for x in parts], [x[1].view for x in parts], out=mo.view, lse=ml.view)
    acc = torch.randn((Nkv * D + 3,), device="cuda:0")
    fin = Guarded(torch, (Nkv * D + 3,), torch.bfloat16, 7.0)
    sp.slimpipe_attn_finalize_bf16(acc, fin.view)
    torch.cuda.synchronize()
    assert all(o.intact() and l.intact() for o, l in parts) and mo.intact() and ml.intact() and fin.intact()
    assert torch.equal(mo.view, om) and torch.equal(ml.view, lm)
    assert torch.equal(fin.view, acc.to(torch.bfloat16))
