"""HIP path vs fp64 oracle at the full sizes of the workload configurations, in the launch shape the
benchmark times.  The oracle cannot evaluate a whole call at these sizes, so:

  * forward out / lse and dq are compared on sampled query rows (random blocks of 8 rows, the first
    and last rows of the slice, rows next to tile boundaries): the oracle is called on each block as
    an 8-row slice at that block's global position, which is the same definition;
  * dk / dv of a full-shape launch are compared at EVERY key by making the upstream gradient zero
    outside the sampled rows: the sum of the oracle's one-row backward calls is then the exact answer;
  * one dense-gradient backward per configuration runs on a reduced number of query rows of a late
    slice, with all heads, where the oracle still finishes in seconds.
"""
import math

import numpy as np
import pytest

from oracle import attn_fwd, attn_bwd
from synth_inputs import CONFIGS, normal_bf16, bf16_bits_to_f64
from gpu_util import say, dev_bf16, host_f64, rel_l2, max_abs, out_err, TOL_OUT, TOL_LSE, TOL_GRAD

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    import torch
    assert torch.cuda.is_available(), "needs the MI355X"
    import paper_2504_14519_amd as sp_
    return sp_


BLK = 8   # sampled rows come in blocks of 8 consecutive rows: one oracle call per block


def sample_rows(s, n_blocks, seed):
    """Row indices: the first and last 8 rows, blocks straddling tile boundaries, random blocks."""
    rng = np.random.default_rng(seed)
    starts = {0, s - BLK, 252, s // 2 - 4, s // 2 + 28}
    starts |= set(int(x) for x in rng.integers(0, s - BLK, size=n_blocks))
    starts = sorted(x for x in starts if 0 <= x <= s - BLK)
    keep, last = [], -BLK
    for x in starts:                       # no overlapping blocks
        if x >= last + BLK:
            keep.append(x)
            last = x
    return np.concatenate([np.arange(x, x + BLK) for x in keep]).astype(np.int64)


def oracle_rows_fwd(q64, k64, v64, rows, q_offset, kv_begin, kv_end, scale):
    """Oracle out/lse of the sampled rows: each block of 8 rows is a slice of its own at its global position."""
    Hq, D = q64.shape[2], q64.shape[3]
    out = np.zeros((len(rows), Hq, D))
    lse = np.zeros((Hq, len(rows)))
    for n in range(0, len(rows), BLK):
        r0 = int(rows[n])
        o, l = attn_fwd(q64[:, r0:r0 + BLK], k64, v64, q_offset + r0, kv_begin, kv_end, True, scale)
        out[n:n + BLK] = o[0]
        lse[:, n:n + BLK] = l[0]
    return out, lse


def check_fwd_rows(name, o_gpu, l_gpu, rows, o_ref, l_ref):
    og = host_f64(o_gpu[0, rows.tolist()])
    lg = host_f64(l_gpu[0][:, rows.tolist()])
    el = max_abs(lg, l_ref)                  # fails on NaN / on a differing -inf pattern
    # elements with |out| >= 4 (rows that see a handful of keys) are held to half a bf16 ulp + 2e-3 and counted
    eo, n_big = out_err(og, o_ref, True)
    say("%s: %d rows, out max-abs %.3e, lse max-abs %.3e, |out|>=4 elements: %d" % (name, len(rows), eo, el, n_big))
    assert eo <= TOL_OUT and el <= TOL_LSE, name


def sparse_bwd_check(sp, name, q, k, v, do_bits_rows, rows, q64, k64, v64, q_offset, kv_end, scale, out, lse, ranges=None):
    """Full-shape backward launch with d_out zero outside `rows`; oracle = sum of one-row calls.  With `ranges`
    (key ranges that tile [0, kv_end)) the backward runs once per range with the same (out, lse), dq summed and
    dk/dv placed per range, and the oracle does the same, range by range."""
    import torch
    B, s, Hq, D = q.shape
    Hkv = k.shape[2]
    ranges = [(0, kv_end)] if ranges is None else list(ranges)
    do = torch.zeros((B, s, Hq, D), device="cuda:0", dtype=torch.bfloat16)
    do[0, rows.tolist()] = dev_bf16(do_bits_rows)
    do64_rows = bf16_bits_to_f64(do_bits_rows)
    dk = torch.zeros((B, kv_end, Hkv, D), device="cuda:0", dtype=torch.float32)
    dv = torch.zeros_like(dk)
    kk, vv = k[:, :kv_end], v[:, :kv_end]
    dq = torch.zeros((B, s, Hq, D), device="cuda:0", dtype=torch.float32)
    for a, b in ranges:
        sp.slimpipe_attn_bwd(q, kk, vv, out, do, lse, q_offset, a, b, dk, dv, True, scale, dq=dq, dq_dtype=sp.F32,
                             dq_accumulate=True, dkv_accumulate=False)
    torch.cuda.synchronize()
    out64 = host_f64(out[0, rows.tolist()])
    lse64 = host_f64(lse[0][:, rows.tolist()])
    dq_ref = np.zeros((len(rows), Hq, D))
    dk_ref = np.zeros((kv_end, Hkv, D))
    dv_ref = np.zeros((kv_end, Hkv, D))
    k64c, v64c = k64[:, :kv_end], v64[:, :kv_end]
    for n in range(0, len(rows), BLK):
        r0 = int(rows[n])
        for a, b in ranges:
            dq_r, dk_r, dv_r = attn_bwd(q64[:, r0:r0 + BLK], k64c, v64c, out64[n:n + BLK][None], do64_rows[n:n + BLK][None],
                                        lse64[:, n:n + BLK][None], q_offset + r0, a, b, True, scale)
            dq_ref[n:n + BLK] += dq_r[0]
            dk_ref += dk_r[0]
            dv_ref += dv_r[0]
    e_q = rel_l2(host_f64(dq[0, rows.tolist()]), dq_ref)
    e_k = rel_l2(host_f64(dk[0]), dk_ref)
    e_v = rel_l2(host_f64(dv[0]), dv_ref)
    others = np.ones(s, dtype=bool)
    others[rows] = False
    dq_other = float(dq[0, torch.from_numpy(np.nonzero(others)[0]).to("cuda:0")].abs().max()) if others.any() else 0.0
    say("%s: sparse-dO backward%s, %d rows: dq rel-L2 %.3e, dk %.3e, dv %.3e (all %d keys); |dq| on zero-dO rows %.1e"
        % (name, "" if len(ranges) == 1 else " in %d key ranges" % len(ranges), len(rows), e_q, e_k, e_v, kv_end, dq_other))
    assert e_q <= TOL_GRAD and e_k <= TOL_GRAD and e_v <= TOL_GRAD, name
    assert dq_other == 0.0


def dense_bwd_check(sp, name, q, k, v, do, q64, k64, v64, do64, row_lo, nrows, q_offset_slice, scale, key_ranges=None):
    """Dense-gradient backward of `nrows` consecutive rows of a slice (all heads) as its own call: forward over the
    whole prefix, then backward over the whole prefix, or - where the oracle could not finish that in minutes (a
    million keys) - one backward call per key range of `key_ranges`, each with the rows' final (out, lse) as the
    call defines it, compared range by range with the oracle's backward over that range (partial dq of the range,
    dk/dv rows of the range)."""
    import torch
    q_off = q_offset_slice + row_lo
    kv_end = q_off + nrows
    rs = slice(row_lo, row_lo + nrows)
    kk, vv = k[:, :kv_end], v[:, :kv_end]
    k64c, v64c = k64[:, :kv_end], v64[:, :kv_end]
    o, l = sp.slimpipe_attn_fwd(q[:, rs], kk, vv, q_off, 0, kv_end, True, scale)
    torch.cuda.synchronize()
    o64, l64 = host_f64(o), host_f64(l)
    if key_ranges is None:
        o_ref, l_ref = attn_fwd(q64[:, rs], k64c, v64c, q_off, 0, kv_end, True, scale)
        eo, n_big = out_err(o64, o_ref, True)
        el = max_abs(l64, l_ref)
        say("%s: forward of %d rows vs %d keys: out %.3e lse %.3e" % (name, nrows, kv_end, eo, el))
        assert eo <= TOL_OUT and el <= TOL_LSE
    for a, b in ([(0, kv_end)] if key_ranges is None else key_ranges):
        dk = torch.zeros((1, kv_end, k.shape[2], k.shape[3]), device="cuda:0", dtype=torch.float32)
        dv = torch.zeros_like(dk)
        dq = sp.slimpipe_attn_bwd(q[:, rs], kk, vv, o, do[:, rs], l, q_off, a, b, dk, dv, True, scale,
                                  dq_dtype=sp.BF16 if key_ranges is None else sp.F32, dkv_accumulate=False)
        torch.cuda.synchronize()
        dq_r, dk_r, dv_r = attn_bwd(q64[:, rs], k64c, v64c, o64, do64[:, rs], l64, q_off, a, b, True, scale)
        e_q, e_k, e_v = rel_l2(host_f64(dq), dq_r), rel_l2(host_f64(dk), dk_r), rel_l2(host_f64(dv), dv_r)
        say("%s: dense backward of %d rows, keys [%d, %d) of %d: dq %.3e dk %.3e dv %.3e" % (name, nrows, a, b, kv_end, e_q, e_k, e_v))
        assert e_q <= TOL_GRAD and e_k <= TOL_GRAD and e_v <= TOL_GRAD, name
        del dk, dv, dq


def run_config(sp, cfg_id, slices_fwd, slice_sparse, n_rows, dense=(1, 0, 1024), dense_key_ranges=None):
    import torch
    c = CONFIGS[cfg_id]
    N, n, Hq, Hkv, D = c["N"], c["n"], c["Hq"], c["Hkv"], c["D"]
    s = N // n
    scale = 1.0 / math.sqrt(D)
    say("config %s: generating inputs" % c["name"])
    kb, vb = normal_bf16((1, N, Hkv, D), cfg_id, "k"), normal_bf16((1, N, Hkv, D), cfg_id, "v")
    k, v = dev_bf16(kb), dev_bf16(vb)
    k64 = v64 = None
    for i in slices_fwd:
        qb = normal_bf16((1, s, Hq, D), cfg_id, "q", salt=i + 1)
        q = dev_bf16(qb)
        kv_end = (i + 1) * s
        say("config %s slice %d: forward launch (s=%d, kv=%d, %d/%d heads)" % (c["name"], i, s, kv_end, Hq, Hkv))
        out, lse = sp.slimpipe_attn_fwd(q, k[:, :kv_end], v[:, :kv_end], i * s, 0, kv_end, True, scale)
        torch.cuda.synchronize()
        rows = sample_rows(s, n_rows, seed=1000 * cfg_id + i)
        if k64 is None:
            k64, v64 = bf16_bits_to_f64(kb), bf16_bits_to_f64(vb)
        q64 = bf16_bits_to_f64(qb)
        o_ref, l_ref = oracle_rows_fwd(q64, k64[:, :kv_end], v64[:, :kv_end], rows, i * s, 0, kv_end, scale)
        check_fwd_rows("config %s slice %d fwd" % (c["name"], i), out, lse, rows, o_ref, l_ref)
        if i == slice_sparse:
            do_rows = normal_bf16((len(rows), Hq, D), cfg_id, "do", salt=i + 1)
            sparse_bwd_check(sp, "config %s slice %d" % (c["name"], i), q, k, v, do_rows, rows, q64, k64, v64, i * s, kv_end,
                             scale, out, lse)
        if dense is not None and i == dense[0]:
            dob = normal_bf16((1, s, Hq, D), cfg_id, "do", salt=100 + i)
            dense_bwd_check(sp, "config %s slice %d" % (c["name"], i), q, k, v, dev_bf16(dob), q64, k64, v64,
                            bf16_bits_to_f64(dob), dense[1], dense[2], i * s, scale, key_ranges=dense_key_ranges)
        del q, out, lse
    del k, v
    torch.cuda.empty_cache()


def test_llama13b_share(sp):
    # 32768 = 8 x 4096, 40 MHA heads: forward of slices 0, 3, 7; sparse-dO backward on slice 7
    run_config(sp, 1, slices_fwd=[0, 3, 7], slice_sparse=7, n_rows=4, dense=(3, 2048, 512))


def test_llama70b_tp8_share(sp):
    # 262144 = 16 x 16384, 8 q heads / 1 kv head: the benchmark's launch shape
    run_config(sp, 2, slices_fwd=[0, 1, 15], slice_sparse=15, n_rows=8, dense=(1, 8192, 2048))


def test_longest_share(sp):
    # 1048576 = 64 x 16384: the final slice attends to ~1M keys (64-bit indexing).  The dense-gradient block is 1024
    # rows of the final slice as their own call against 1,047,552 keys; its backward is checked on the first 12288
    # keys and on the last 20480 (the causal diagonal of the rows among them): 3.4e7 (row, key) pairs per head in the
    # oracle.  (Every key of a full-shape launch is covered by the sparse-gradient check of the same slice.)
    N, s = CONFIGS[4]["N"], CONFIGS[4]["N"] // CONFIGS[4]["n"]
    kv_end = 63 * s + 15360
    run_config(sp, 4, slices_fwd=[56, 63], slice_sparse=63, n_rows=1, dense=(63, 14336, 1024),
               dense_key_ranges=[(0, 12288), (kv_end - 20480, kv_end)])


def test_redistribution_split_merge(sp):
    """Slices 16..31 of the 131072-token sequence split into equal-FLOP key ranges whose count grows with
    the slice index, computed separately and merged; compared with the unsplit launch and the oracle."""
    import torch
    from paper_2504_14519_amd.planner import equal_flop_cuts
    cfg_id = 3
    c = CONFIGS[cfg_id]
    N, n, Hq, Hkv, D = c["N"], c["n"], c["Hq"], c["Hkv"], c["D"]
    s = N // n
    scale = 1.0 / math.sqrt(D)
    kb, vb = normal_bf16((1, N, Hkv, D), cfg_id, "k"), normal_bf16((1, N, Hkv, D), cfg_id, "v")
    k, v = dev_bf16(kb), dev_bf16(vb)
    k64, v64 = bf16_bits_to_f64(kb), bf16_bits_to_f64(vb)
    for i in (16, 23, 27, 31):
        parts = 2 + (i - 16) // 4
        cuts = equal_flop_cuts(s, i * s, parts)
        say("redistribution slice %d: %d parts, cuts %s" % (i, parts, cuts))
        qb = normal_bf16((1, s, Hq, D), cfg_id, "q", salt=i + 1)
        dob = normal_bf16((1, s, Hq, D), cfg_id, "do", salt=i + 1)
        q, do = dev_bf16(qb), dev_bf16(dob)
        kv_end = (i + 1) * s
        kk, vv = k[:, :kv_end], v[:, :kv_end]
        o_u, l_u = sp.slimpipe_attn_fwd(q, kk, vv, i * s, 0, kv_end, True, scale)
        ps = [sp.slimpipe_attn_fwd(q, kk, vv, i * s, a, b, True, scale, out_dtype=sp.F32) for a, b in zip(cuts[:-1], cuts[1:])]
        o_m, l_m = sp.slimpipe_attn_merge([p[0] for p in ps], [p[1] for p in ps])
        torch.cuda.synchronize()
        d_o = float((o_m.float() - o_u.float()).abs().max())
        d_l = float((l_m - l_u).abs().max())
        say("  merged vs unsplit on the GPU: out max-abs %.3e, lse max-abs %.3e" % (d_o, d_l))
        assert d_o <= TOL_OUT and d_l <= TOL_LSE
        rows = sample_rows(s, 3, seed=7000 + i)
        q64 = bf16_bits_to_f64(qb)
        o_ref, l_ref = oracle_rows_fwd(q64, k64[:, :kv_end], v64[:, :kv_end], rows, i * s, 0, kv_end, scale)
        check_fwd_rows("  merged vs oracle", o_m, l_m, rows, o_ref, l_ref)
        # backward per part with the merged (out, lse): dq summed, dk/dv placed per range == unsplit backward
        dk_u = torch.zeros((1, kv_end, Hkv, D), device="cuda:0")
        dv_u = torch.zeros_like(dk_u)
        dq_u = sp.slimpipe_attn_bwd(q, kk, vv, o_m, do, l_m, i * s, 0, kv_end, dk_u, dv_u, True, scale, dq_dtype=sp.F32,
                                    dkv_accumulate=False)
        dk_s = torch.zeros_like(dk_u)
        dv_s = torch.zeros_like(dk_u)
        dq_s = torch.zeros_like(dq_u)
        for a, b in zip(cuts[:-1], cuts[1:]):
            sp.slimpipe_attn_bwd(q, kk, vv, o_m, do, l_m, i * s, a, b, dk_s, dv_s, True, scale, dq=dq_s, dq_dtype=sp.F32,
                                 dq_accumulate=True, dkv_accumulate=False)
        torch.cuda.synchronize()
        for nm, x, y in (("dq", dq_s, dq_u), ("dk", dk_s, dk_u), ("dv", dv_s, dv_u)):
            e = float((x - y).norm() / y.norm())
            say("  split vs unsplit backward %s: rel-L2 %.3e" % (nm, e))
            assert e <= TOL_GRAD
        # the split backward against the oracle: upstream gradient on the sampled rows only, one backward call per
        # key range with the merged (out, lse), dq summed, dk/dv placed per range; the oracle does the same range by range
        do_rows = normal_bf16((len(rows), Hq, D), cfg_id, "do", salt=200 + i)
        sparse_bwd_check(sp, "  slice %d split" % i, q, k, v, do_rows, rows, q64, k64, v64, i * s, kv_end, scale, o_m, l_m,
                         ranges=list(zip(cuts[:-1], cuts[1:])))
        del q, do, o_u, l_u, ps, o_m, l_m, dk_u, dv_u, dq_u, dk_s, dv_s, dq_s


def test_llama70b_chunked_matches_contiguous(sp):
    """The benchmark's launch shape with the cache as 16 slice-sized allocations: forward and backward
    of the last slice equal the contiguous calls bit for bit (same tile walk, same order of sums), and
    the contiguous calls are the ones checked against the oracle above."""
    import torch
    cfg_id = 2
    c = CONFIGS[cfg_id]
    N, n, Hq, Hkv, D = c["N"], c["n"], c["Hq"], c["Hkv"], c["D"]
    s = N // n
    i = n - 1
    say("config %s chunked: generating inputs" % c["name"])
    k, v = dev_bf16(normal_bf16((1, N, Hkv, D), cfg_id, "k")), dev_bf16(normal_bf16((1, N, Hkv, D), cfg_id, "v"))
    q = dev_bf16(normal_bf16((1, s, Hq, D), cfg_id, "q", salt=i + 1))
    do = dev_bf16(normal_bf16((1, s, Hq, D), cfg_id, "do", salt=100 + i))
    kc = [k[:, j * s:(j + 1) * s].clone() for j in range(n)]
    vc = [v[:, j * s:(j + 1) * s].clone() for j in range(n)]
    say("forward, contiguous and chunked")
    o_f, l_f = sp.slimpipe_attn_fwd(q, k, v, i * s, 0, N, True, None)
    o_c, l_c = sp.slimpipe_attn_fwd_chunked(q, kc, vc, i * s, 0, N, True, None)
    torch.cuda.synchronize()
    assert torch.equal(o_f, o_c) and torch.equal(l_f, l_c)
    say("backward, contiguous")
    dk_f = torch.zeros((1, N, Hkv, D), device="cuda:0")
    dv_f = torch.zeros_like(dk_f)
    dq_f = sp.slimpipe_attn_bwd(q, k, v, o_f, do, l_f, i * s, 0, N, dk_f, dv_f, True, None, dkv_accumulate=False)
    say("backward, chunked")
    dkc = [torch.zeros((1, s, Hkv, D), device="cuda:0") for _ in range(n)]
    dvc = [torch.zeros((1, s, Hkv, D), device="cuda:0") for _ in range(n)]
    dq_c = sp.slimpipe_attn_bwd_chunked(q, kc, vc, o_f, do, l_f, i * s, 0, N, dkc, dvc, True, None, dkv_accumulate=False)
    torch.cuda.synchronize()
    assert torch.equal(dq_f, dq_c)
    assert torch.equal(dk_f, torch.cat(dkc, dim=1)) and torch.equal(dv_f, torch.cat(dvc, dim=1))


def test_redistribution_key_ranges_in_one_launch(sp):
    """The 4096-row slices of the 131072-token workload leave half the compute units idle, so the library
    cuts the forward and the dq kernel into key ranges when it has the workspace (the launch shape bench.py
    times for this workload): forward and backward against the oracle on sampled rows, the one-launch
    multi-range forward against the one-range calls."""
    import torch
    from paper_2504_14519_amd.planner import equal_flop_cuts
    cfg_id = 3
    c = CONFIGS[cfg_id]
    N, n, Hq, Hkv, D = c["N"], c["n"], c["Hq"], c["Hkv"], c["D"]
    s = N // n
    scale = 1.0 / math.sqrt(D)
    kb, vb = normal_bf16((1, N, Hkv, D), cfg_id, "k"), normal_bf16((1, N, Hkv, D), cfg_id, "v")
    k, v = dev_bf16(kb), dev_bf16(vb)
    k64, v64 = bf16_bits_to_f64(kb), bf16_bits_to_f64(vb)
    for i in (5, 31):
        qb = normal_bf16((1, s, Hq, D), cfg_id, "q", salt=i + 1)
        q, q64 = dev_bf16(qb), bf16_bits_to_f64(qb)
        kv_end = (i + 1) * s
        kk, vv = k[:, :kv_end], v[:, :kv_end]
        out = torch.empty((1, s, Hq, D), device="cuda:0", dtype=torch.bfloat16)
        need = sp.slimpipe_attn_workspace_bytes(sp.make_params(q, kk, out, i * s, 0, kv_end, True, scale), False)
        assert need > 256          # more than the ticket counter: room for key ranges
        ws = torch.empty(need, device="cuda:0", dtype=torch.uint8)
        say("redistribution slice %d: forward cut into key ranges (workspace %d bytes)" % (i, need))
        o_r, l_r = sp.slimpipe_attn_fwd(q, kk, vv, i * s, 0, kv_end, True, scale, out=out, workspace=ws)
        torch.cuda.synchronize()
        rows = sample_rows(s, 3, seed=7100 + i)
        o_ref, l_ref = oracle_rows_fwd(q64, k64[:, :kv_end], v64[:, :kv_end], rows, i * s, 0, kv_end, scale)
        check_fwd_rows("  ranges vs oracle", o_r, l_r, rows, o_ref, l_ref)
        # backward with the library's own workspace request: dq in key ranges, dk/dv with a split query stream
        do_rows = normal_bf16((len(rows), Hq, D), cfg_id, "do", salt=i + 1)
        sparse_bwd_check(sp, "  slice %d" % i, q, k, v, do_rows, rows, q64, k64, v64, i * s, kv_end, scale, o_r, l_r)
        # several ranges in one launch == the same ranges one call each, bit for bit
        cuts = equal_flop_cuts(s, i * s, 3)
        ranges = list(zip(cuts[:-1], cuts[1:]))
        po, pl, om, lm = sp.slimpipe_attn_fwd_ranges(q, kk, vv, i * s, ranges, True, scale)
        for r, (a, b) in enumerate(ranges):
            o1, l1 = sp.slimpipe_attn_fwd(q, kk, vv, i * s, a, b, True, scale, out_dtype=sp.F32)
            torch.cuda.synchronize()
            assert torch.equal(o1, po[r]) and torch.equal(l1, pl[r])
        check_fwd_rows("  three ranges merged vs oracle", om, lm, rows, o_ref, l_ref)
        del q, out, ws, o_r, l_r, po, pl, om, lm
