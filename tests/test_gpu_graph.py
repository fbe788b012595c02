"""The hot path under HIP graph capture: the library allocates nothing and synchronises nothing, so one forward
and one backward call (six kernels) can be captured once and replayed.  Every replay is checked against the eager
result on fresh inputs, with eager work and synchronisations between the replays.  The second test does the same
in a process of its own whose FIRST use of the library is the capture, after slimpipe_attn_init()."""
import math
import os
import subprocess
import sys

import pytest

from synth_inputs import normal_bf16
from gpu_util import say, dev_bf16

pytestmark = pytest.mark.gpu


def test_forward_backward_replayed_from_a_graph():
    capture_and_replay(eager_warmup=True)


def test_capture_is_the_first_use_after_init():
    """A fresh process: slimpipe_attn_init(), then the capture, with no eager launch before it."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = ("import sys; sys.path.insert(0, %r); sys.path.insert(0, %r); import test_gpu_graph as t; "
            "t.capture_and_replay(eager_warmup=False); print('child ok', flush=True)") % (root, os.path.join(root, "tests"))
    r = subprocess.run([sys.executable, "-u", "-c", code], capture_output=True, text=True, timeout=300)
    say("child process: rc %d\n%s%s" % (r.returncode, r.stdout[-2000:], r.stderr[-2000:]))
    assert r.returncode == 0 and "child ok" in r.stdout


def capture_and_replay(eager_warmup):
    import torch
    import paper_2504_14519_amd as sp
    B, s, N, Hq, Hkv, D = 1, 512, 2048, 4, 1, 128
    q_off = N - s
    scale = 1.0 / math.sqrt(D)
    dev = "cuda:0"
    mk = lambda shape, t, salt: dev_bf16(normal_bf16(shape, 16, t, salt=salt))
    # static buffers the graph reads and writes
    q, k, v, do = mk((B, s, Hq, D), "q", 0), mk((B, N, Hkv, D), "k", 0), mk((B, N, Hkv, D), "v", 0), mk((B, s, Hq, D), "do", 0)
    out = torch.empty((B, s, Hq, D), device=dev, dtype=torch.bfloat16)
    lse = torch.empty((B, Hq, s), device=dev, dtype=torch.float32)
    dq = torch.empty((B, s, Hq, D), device=dev, dtype=torch.float32)
    dk = torch.zeros((B, N, Hkv, D), device=dev, dtype=torch.float32)
    dv = torch.zeros_like(dk)
    p = sp.make_params(q, k, out, q_off, 0, N, True, scale)
    fws = torch.empty(max(sp.slimpipe_attn_workspace_bytes(p, False), 256), device=dev, dtype=torch.uint8)
    ws = torch.empty(sp.slimpipe_attn_workspace_bytes(p, True), device=dev, dtype=torch.uint8)

    def step():
        sp.slimpipe_attn_fwd(q, k, v, q_off, 0, N, True, scale, out=out, lse=lse, workspace=fws)
        sp.slimpipe_attn_bwd(q, k, v, out, do, lse, q_off, 0, N, dk, dv, True, scale, dq=dq, dq_dtype=sp.F32,
                             dkv_accumulate=False, workspace=ws)

    if eager_warmup:
        say("graph: eager warm-up")
        step()
        torch.cuda.synchronize()
    else:
        say("graph: slimpipe_attn_init(), no eager launch")
        sp.slimpipe_attn_init()
    say("graph: capture")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    for rep in range(3):
        say("graph: replay %d" % rep)
        # fresh inputs into the static buffers, eager reference first
        q.copy_(mk((B, s, Hq, D), "q", rep + 1)); do.copy_(mk((B, s, Hq, D), "do", rep + 1))
        k.copy_(mk((B, N, Hkv, D), "k", rep + 1)); v.copy_(mk((B, N, Hkv, D), "v", rep + 1))
        step()
        torch.cuda.synchronize()
        ref = [t.clone() for t in (out, lse, dq, dk, dv)]
        for t in (out, lse, dq, dk, dv):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("out", "lse", "dq", "dk", "dv"), (out, lse, dq, dk, dv), ref):
            assert torch.equal(a, b), "replay %d: %s differs from the eager result" % (rep, name)
