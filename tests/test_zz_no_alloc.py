"""The backward entry point that allocates nothing (its row statistics live in a fixed device array of the library)
against the ordinary backward entry point given a workspace of the minimum size: same kernels, same plan, so the
results agree bit for bit, well inside the gradient tolerance.  Two calls in a row, the second with a smaller
input, so that what the first call left in the fixed array cannot leak into the second."""
import math

import pytest

from synth_inputs import normal_bf16
from gpu_util import say, dev_bf16, host_f64, rel_l2, TOL_GRAD

pytestmark = pytest.mark.gpu


def one_case(sp, salt, B, s, N, Hq, Hkv, D, q_off, kv_begin, kv_end):
    import torch
    scale = 1.0 / math.sqrt(D)
    mk = lambda shape, t: dev_bf16(normal_bf16(shape, 17, t, salt=salt))
    q, k, v, do = mk((B, s, Hq, D), "q"), mk((B, N, Hkv, D), "k"), mk((B, N, Hkv, D), "v"), mk((B, s, Hq, D), "do")
    out, lse = sp.slimpipe_attn_fwd(q, k, v, q_off, kv_begin, kv_end, True, scale)
    stats_only = 2 * (((B * Hq * s * 4) + 255) // 256 * 256)
    ws = torch.empty(stats_only, device="cuda:0", dtype=torch.uint8)
    res = {}
    for name in ("workspace", "noalloc"):
        dk = torch.full((B, N, Hkv, D), 0.25, device="cuda:0", dtype=torch.float32)
        dv = torch.full((B, N, Hkv, D), -0.5, device="cuda:0", dtype=torch.float32)
        dq = torch.full((B, s, Hq, D), float("nan"), device="cuda:0", dtype=torch.float32)
        torch.cuda.synchronize()
        say("no-alloc case %d (%s): s=%d keys [%d,%d) heads %d/%d D=%d" % (salt, name, s, kv_begin, kv_end, Hq, Hkv, D))
        if name == "workspace":
            sp.slimpipe_attn_bwd(q, k, v, out, do, lse, q_off, kv_begin, kv_end, dk, dv, True, scale, dq=dq, dq_dtype=sp.F32,
                                 dkv_accumulate=True, workspace=ws)
        else:
            sp.slimpipe_attn_bwd_noalloc(q, k, v, out, do, lse, q_off, kv_begin, kv_end, dq, dk, dv, True, scale,
                                         dkv_accumulate=True)
        torch.cuda.synchronize()
        res[name] = (dq, dk, dv)
    for nm, a, b in zip(("dq", "dk", "dv"), res["noalloc"], res["workspace"]):
        assert torch.isfinite(a).all(), nm
        e = rel_l2(host_f64(a), host_f64(b))
        say("  %s: no-alloc vs workspace entry point rel-L2 %.3e, bit-equal %s" % (nm, e, bool(torch.equal(a, b))))
        assert e <= TOL_GRAD, nm
        assert torch.equal(a, b), nm + ": same kernels and plan, so the bits agree"


def test_noalloc_backward_matches_workspace_backward_twice():
    import torch
    assert torch.cuda.is_available(), "needs the MI355X"
    import paper_2504_14519_amd as sp
    # first call: more work items than compute units in the dq and the dk/dv kernel, so that the no-alloc path hands
    # them out through the counters it keeps in the fixed array (the workspace of the minimum size has no room for
    # counters: there the workgroup index is the item; the bits agree all the same)
    one_case(sp, 0, 1, 4352, 4608, 16, 16, 64, 256, 0, 4608)
    # then 1024 rows, 8/2 heads, range cutting the diagonal block; last call: smaller in every dimension
    one_case(sp, 1, 1, 1024, 3072, 8, 2, 128, 2048, 100, 2900)
    one_case(sp, 2, 1, 200, 777, 4, 4, 64, 500, 0, 650)


def test_noalloc_rejects_what_does_not_fit():
    import torch
    import paper_2504_14519_amd as sp
    B, s, Hq, D = 1, 65536 + 256, 8, 64          # 8 * 65792 rows of statistics: more than the fixed array holds
    q = torch.zeros((B, s, Hq, D), device="cuda:0", dtype=torch.bfloat16)
    k = torch.zeros((B, 256, 1, D), device="cuda:0", dtype=torch.bfloat16)
    lse = torch.zeros((B, Hq, s), device="cuda:0", dtype=torch.float32)
    dq = torch.zeros((B, s, Hq, D), device="cuda:0", dtype=torch.float32)
    dk = torch.zeros((B, 256, 1, D), device="cuda:0", dtype=torch.float32)
    with pytest.raises(sp.SlimpipeError) as e:
        sp.slimpipe_attn_bwd_noalloc(q, k, k, q, q, lse, 0, 0, 256, dq, dk, dk.clone())
    assert "-8" in str(e.value)
