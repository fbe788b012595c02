"""Two host threads make their FIRST calls into the library at the same time, each on its own stream with its own
buffers (a fresh process, so that the per-device preparation really happens under contention); both must get what a
single-threaded run gets, bit for bit."""
import math
import os
import subprocess
import sys
import threading

import pytest

from synth_inputs import normal_bf16
from gpu_util import say, dev_bf16

pytestmark = pytest.mark.gpu


def run_two_threads():
    import torch
    import paper_2504_14519_amd as sp
    B, s, N, Hq, Hkv, D = 1, 384, 1536, 4, 2, 128
    scale = 1.0 / math.sqrt(D)
    jobs = []
    for t in range(2):
        mk = lambda shape, name: dev_bf16(normal_bf16(shape, 20, name, salt=t))
        jobs.append(dict(q=mk((B, s, Hq, D), "q"), k=mk((B, N, Hkv, D), "k"), v=mk((B, N, Hkv, D), "v"), do=mk((B, s, Hq, D), "do"),
                         stream=torch.cuda.Stream(), res=None, err=None))
    torch.cuda.synchronize()
    gate = threading.Barrier(2)

    def work(job):
        try:
            gate.wait()
            with torch.cuda.stream(job["stream"]):
                out, lse = sp.slimpipe_attn_fwd(job["q"], job["k"], job["v"], N - s, 0, N, True, scale)
                dk = torch.zeros((B, N, Hkv, D), device="cuda:0")
                dv = torch.zeros_like(dk)
                dq = sp.slimpipe_attn_bwd(job["q"], job["k"], job["v"], out, job["do"], lse, N - s, 0, N, dk, dv, True, scale,
                                          dq_dtype=sp.F32, dkv_accumulate=False)
            job["stream"].synchronize()
            job["res"] = (out, lse, dq, dk, dv)
        except Exception as e:          # reported by the main thread
            job["err"] = e

    threads = [threading.Thread(target=work, args=(j,)) for j in jobs]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    for j in jobs:
        assert j["err"] is None, j["err"]
    # the same two jobs one after the other on the default stream
    for j in jobs:
        out, lse = sp.slimpipe_attn_fwd(j["q"], j["k"], j["v"], N - s, 0, N, True, scale)
        dk = torch.zeros((B, N, Hkv, D), device="cuda:0")
        dv = torch.zeros_like(dk)
        dq = sp.slimpipe_attn_bwd(j["q"], j["k"], j["v"], out, j["do"], lse, N - s, 0, N, dk, dv, True, scale, dq_dtype=sp.F32,
                                  dkv_accumulate=False)
        torch.cuda.synchronize()
        for name, a, b in zip(("out", "lse", "dq", "dk", "dv"), j["res"], (out, lse, dq, dk, dv)):
            assert torch.isfinite(a.float()).all(), name
            assert torch.equal(a, b), name + " differs between the threaded and the sequential run"


def test_first_calls_from_two_threads():
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = ("import sys; sys.path.insert(0, %r); sys.path.insert(0, %r); import test_gpu_threads as t; "
            "t.run_two_threads(); print('child ok', flush=True)") % (root, os.path.join(root, "tests"))
    r = subprocess.run([sys.executable, "-u", "-c", code], capture_output=True, text=True, timeout=300)
    say("child process: rc %d\n%s%s" % (r.returncode, r.stdout[-2000:], r.stderr[-2000:]))
    assert r.returncode == 0 and "child ok" in r.stdout
