"""ctypes binding of libslimpipe_attn.so: argument marshalling only.

Same entry-point names as the C header.  Tensors are torch tensors on the GPU; torch supplies
device memory and the current stream, every step of the computation runs in the library's kernels.
There is no fallback: if the shared library is missing the import fails.
"""
import ctypes
import math
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libslimpipe_attn.so")

BF16, F32 = 0, 1


class SlimpipeError(RuntimeError):
    pass


class AttnParams(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("s_q", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("causal", ctypes.c_int32),
        ("kv_capacity", ctypes.c_int64), ("q_offset", ctypes.c_int64), ("kv_begin", ctypes.c_int64),
        ("kv_end", ctypes.c_int64), ("scale", ctypes.c_float), ("out_dtype", ctypes.c_int32),
        ("q_stride_b", ctypes.c_int64), ("q_stride_s", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
        ("kv_stride_b", ctypes.c_int64), ("kv_stride_s", ctypes.c_int64), ("kv_stride_h", ctypes.c_int64),
        ("o_stride_b", ctypes.c_int64), ("o_stride_s", ctypes.c_int64), ("o_stride_h", ctypes.c_int64),
        ("do_stride_b", ctypes.c_int64), ("do_stride_s", ctypes.c_int64), ("do_stride_h", ctypes.c_int64),
    ]


def library_path():
    return _LIB_PATH


def _load():
    if not os.path.exists(_LIB_PATH):
        # nothing built yet: compile the HIP library now (hipcc cross-compiles without a GPU).  There is no
        # fallback path: if that fails, so does the import.
        try:
            from .build import build as _build
            _build()
        except Exception as e:
            raise ImportError("libslimpipe_attn.so is not built and building it failed (%s): run "
                              "`python paper_2504_14519_amd/build.py`" % e)
    # torch first: the tensors and streams handed to the library come from torch's HIP runtime, so that runtime has
    # to be the one already in the process when the library's dependency on libamdhip64 is resolved (loaded the other
    # way round, the library can end up on a second runtime instance that sees no device)
    import torch  # noqa: F401
    L = ctypes.CDLL(_LIB_PATH)
    P = ctypes.POINTER(AttnParams)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    L.slimpipe_attn_init.argtypes = []
    L.slimpipe_attn_init.restype = ctypes.c_int
    L.slimpipe_attn_validate.argtypes = [P, ctypes.c_int]
    L.slimpipe_attn_validate.restype = ctypes.c_int
    L.slimpipe_attn_workspace_bytes.argtypes = [P, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
    L.slimpipe_attn_workspace_bytes.restype = ctypes.c_int
    L.slimpipe_attn_fwd.argtypes = [P, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    L.slimpipe_attn_fwd.restype = ctypes.c_int
    L.slimpipe_attn_bwd.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, i32, vp, ctypes.c_size_t, vp]
    L.slimpipe_attn_bwd.restype = ctypes.c_int
    L.slimpipe_attn_bwd_noalloc.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, i32, vp]
    L.slimpipe_attn_bwd_noalloc.restype = ctypes.c_int
    L.slimpipe_attn_noalloc_max_rows.argtypes = []
    L.slimpipe_attn_noalloc_max_rows.restype = ctypes.c_int
    pp = ctypes.POINTER(vp)
    L.slimpipe_attn_fwd_chunked.argtypes = [P, vp, pp, pp, i32, i64, vp, vp, vp, ctypes.c_size_t, vp]
    L.slimpipe_attn_fwd_chunked.restype = ctypes.c_int
    L.slimpipe_attn_bwd_chunked.argtypes = [P, vp, pp, pp, i32, i64, vp, vp, vp, vp, i32, i32, pp, pp, i32, vp, ctypes.c_size_t, vp]
    L.slimpipe_attn_bwd_chunked.restype = ctypes.c_int
    L.slimpipe_attn_fwd_ranges.argtypes = [P, vp, pp, pp, i32, i64, i32, ctypes.POINTER(i64), ctypes.POINTER(i64), vp, vp, vp, vp, vp]
    L.slimpipe_attn_fwd_ranges.restype = ctypes.c_int
    L.slimpipe_attn_merge.argtypes = [i32, ctypes.POINTER(vp), ctypes.POINTER(vp), i32, i32, i32, i32, i32, vp, i32, vp, vp]
    L.slimpipe_attn_merge.restype = ctypes.c_int
    L.slimpipe_attn_finalize_bf16.argtypes = [vp, vp, i64, vp]
    L.slimpipe_attn_finalize_bf16.restype = ctypes.c_int
    L.slimpipe_attn_mfma_rate.argtypes = [ctypes.c_int, vp, ctypes.POINTER(ctypes.c_double), vp]
    L.slimpipe_attn_mfma_rate.restype = ctypes.c_int
    L.slimpipe_attn_dq_atomic_probe.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
    L.slimpipe_attn_dq_atomic_probe.restype = ctypes.c_int
    L.slimpipe_attn_xcd_rate.argtypes = [i32, i32, vp, vp, vp, vp]
    L.slimpipe_attn_xcd_rate.restype = ctypes.c_int
    L.slimpipe_attn_profile_enable.argtypes = [ctypes.c_int]
    L.slimpipe_attn_profile_enable.restype = ctypes.c_int
    L.slimpipe_attn_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    L.slimpipe_attn_profile_read.restype = ctypes.c_int
    L.slimpipe_attn_strerror.argtypes = [ctypes.c_int]
    L.slimpipe_attn_strerror.restype = ctypes.c_char_p
    return L


lib = _load()


def slimpipe_attn_strerror(code):
    return lib.slimpipe_attn_strerror(int(code)).decode()


def _check(rc, what):
    if rc != 0:
        raise SlimpipeError("%s failed: %d (%s)" % (what, rc, slimpipe_attn_strerror(rc)))


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _same_strides(a, b):
    """Equal shapes and equal strides on every dimension longer than one."""
    return a.shape == b.shape and all(sa == sb for n, sa, sb in zip(a.shape, a.stride(), b.stride()) if n > 1)


def make_params(q, k, out_like, q_offset, kv_begin, kv_end, causal, scale, out_dtype=BF16):
    """Fill the parameter block from tensor shapes/strides.  q [B,s,Hq,D], k [B,Nkv,Hkv,D]."""
    B, s, Hq, D = q.shape
    p = AttnParams()
    p.batch, p.s_q, p.n_q_heads, p.n_kv_heads, p.head_dim = B, s, Hq, k.shape[2], D
    p.causal = 1 if causal else 0
    p.kv_capacity, p.q_offset, p.kv_begin, p.kv_end = k.shape[1], q_offset, kv_begin, kv_end
    p.scale = float(scale) if scale is not None else 1.0 / math.sqrt(D)
    p.out_dtype = out_dtype
    p.q_stride_b, p.q_stride_s, p.q_stride_h = q.stride(0), q.stride(1), q.stride(2)
    p.kv_stride_b, p.kv_stride_s, p.kv_stride_h = k.stride(0), k.stride(1), k.stride(2)
    p.o_stride_b, p.o_stride_s, p.o_stride_h = out_like.stride(0), out_like.stride(1), out_like.stride(2)
    p.do_stride_b, p.do_stride_s, p.do_stride_h = p.o_stride_b, p.o_stride_s, p.o_stride_h   # backward overrides
    return p


def slimpipe_attn_init():
    """Prepare the current device for launches (needed once per device before a HIP graph capture)."""
    _check(lib.slimpipe_attn_init(), "slimpipe_attn_init")


def slimpipe_attn_validate(params, is_bwd=False):
    return lib.slimpipe_attn_validate(ctypes.byref(params), 1 if is_bwd else 0)


def slimpipe_attn_workspace_bytes(params, is_bwd):
    n = ctypes.c_size_t(0)
    _check(lib.slimpipe_attn_workspace_bytes(ctypes.byref(params), 1 if is_bwd else 0, ctypes.byref(n)), "workspace_bytes")
    return n.value


def _ws(workspace):
    return (workspace.data_ptr(), workspace.numel()) if workspace is not None else (None, 0)


def slimpipe_attn_fwd(q_slice, k_prefix, v_prefix, q_offset, kv_begin, kv_end, causal=True, scale=None,
                      out_dtype=BF16, out=None, lse=None, workspace=None):
    """-> (out, lse).  out [B,s,Hq,D] (bf16 or fp32), lse [B,Hq,s] fp32.  workspace: uint8 tensor the library may
    use to cut a short slice over a long cache into key ranges (slimpipe_attn_workspace_bytes(p, False))."""
    import torch
    B, s, Hq, D = q_slice.shape
    if out is None:
        out = torch.empty((B, s, Hq, D), device=q_slice.device, dtype=torch.float32 if out_dtype == F32 else torch.bfloat16)
    if lse is None:
        lse = torch.empty((B, Hq, s), device=q_slice.device, dtype=torch.float32)
    p = make_params(q_slice, k_prefix, out, q_offset, kv_begin, kv_end, causal, scale, out_dtype)
    _check(lib.slimpipe_attn_fwd(ctypes.byref(p), q_slice.data_ptr(), k_prefix.data_ptr(), v_prefix.data_ptr(),
                                 out.data_ptr(), lse.data_ptr(), *_ws(workspace), _stream()), "slimpipe_attn_fwd")
    return out, lse


def slimpipe_attn_bwd(q_slice, k_prefix, v_prefix, out, d_out, lse, q_offset, kv_begin, kv_end, dk_acc, dv_acc,
                      causal=True, scale=None, dq=None, dq_dtype=BF16, dq_accumulate=False, dkv_accumulate=True,
                      workspace=None):
    """-> dq.  dk_acc/dv_acc (fp32, shaped like k_prefix) get rows [kv_begin, kv_end) written or incremented."""
    import torch
    if dq is None:
        dq = torch.empty_like(q_slice, dtype=torch.float32 if dq_dtype == F32 else torch.bfloat16)
    if not (_same_strides(dq, q_slice) and _same_strides(dk_acc, k_prefix) and _same_strides(dv_acc, k_prefix)):
        raise SlimpipeError("dq must have the strides of q; dk_acc/dv_acc those of k")
    p = make_params(q_slice, k_prefix, out, q_offset, kv_begin, kv_end, causal, scale)
    p.do_stride_b, p.do_stride_s, p.do_stride_h = d_out.stride(0), d_out.stride(1), d_out.stride(2)
    need = slimpipe_attn_workspace_bytes(p, True)
    if workspace is None:
        workspace = torch.empty(need, device=q_slice.device, dtype=torch.uint8)
    _check(lib.slimpipe_attn_bwd(ctypes.byref(p), q_slice.data_ptr(), k_prefix.data_ptr(), v_prefix.data_ptr(),
                                 out.data_ptr(), d_out.data_ptr(), lse.data_ptr(), dq.data_ptr(), dq_dtype,
                                 1 if dq_accumulate else 0, dk_acc.data_ptr(), dv_acc.data_ptr(),
                                 1 if dkv_accumulate else 0, workspace.data_ptr(), workspace.numel(), _stream()),
           "slimpipe_attn_bwd")
    return dq


def slimpipe_attn_bwd_noalloc(q_slice, k_prefix, v_prefix, out, d_out, lse, q_offset, kv_begin, kv_end, dq, dk_acc, dv_acc,
                              causal=True, scale=None, dq_accumulate=False, dkv_accumulate=True):
    """slimpipe_attn_bwd without a workspace and without any allocation (the binding allocates nothing either: dq is
    the caller's, float32 or bf16 by its dtype).  -> the status code's check; results in dq, dk_acc, dv_acc."""
    import torch
    if not (_same_strides(dq, q_slice) and _same_strides(dk_acc, k_prefix) and _same_strides(dv_acc, k_prefix)):
        raise SlimpipeError("dq must have the strides of q; dk_acc/dv_acc those of k")
    p = make_params(q_slice, k_prefix, out, q_offset, kv_begin, kv_end, causal, scale)
    p.do_stride_b, p.do_stride_s, p.do_stride_h = d_out.stride(0), d_out.stride(1), d_out.stride(2)
    _check(lib.slimpipe_attn_bwd_noalloc(ctypes.byref(p), q_slice.data_ptr(), k_prefix.data_ptr(), v_prefix.data_ptr(),
                                         out.data_ptr(), d_out.data_ptr(), lse.data_ptr(), dq.data_ptr(),
                                         F32 if dq.dtype == torch.float32 else BF16, 1 if dq_accumulate else 0,
                                         dk_acc.data_ptr(), dv_acc.data_ptr(), 1 if dkv_accumulate else 0, _stream()),
           "slimpipe_attn_bwd_noalloc")
    return dq


def _chunk_table(chunks):
    """list of tensors -> ctypes array of device pointers (all chunks share shape and strides)."""
    c0 = chunks[0]
    for c in chunks:
        if c.shape != c0.shape or not _same_strides(c, c0):
            raise SlimpipeError("chunks must share shape and strides")
    return (ctypes.c_void_p * len(chunks))(*[c.data_ptr() for c in chunks])


class _ChunkedKV:
    """What make_params needs to know of a chunk list: the shape and strides of the virtual prefix."""
    def __init__(self, chunks):
        c0 = chunks[0]
        self.shape = (c0.shape[0], len(chunks) * c0.shape[1], c0.shape[2], c0.shape[3])
        self._strides = c0.stride()

    def stride(self, i):
        return self._strides[i]


def slimpipe_attn_fwd_chunked(q_slice, k_chunks, v_chunks, q_offset, kv_begin, kv_end, causal=True, scale=None,
                              out_dtype=BF16, out=None, lse=None, workspace=None):
    """As slimpipe_attn_fwd with K/V given as lists of equally shaped chunks [B, chunk_len, Hkv, D]."""
    import torch
    B, s, Hq, D = q_slice.shape
    if out is None:
        out = torch.empty((B, s, Hq, D), device=q_slice.device, dtype=torch.float32 if out_dtype == F32 else torch.bfloat16)
    if lse is None:
        lse = torch.empty((B, Hq, s), device=q_slice.device, dtype=torch.float32)
    p = make_params(q_slice, _ChunkedKV(k_chunks), out, q_offset, kv_begin, kv_end, causal, scale, out_dtype)
    _check(lib.slimpipe_attn_fwd_chunked(ctypes.byref(p), q_slice.data_ptr(), _chunk_table(k_chunks), _chunk_table(v_chunks),
                                         len(k_chunks), k_chunks[0].shape[1], out.data_ptr(), lse.data_ptr(), *_ws(workspace),
                                         _stream()),
           "slimpipe_attn_fwd_chunked")
    return out, lse


def slimpipe_attn_fwd_ranges(q_slice, k_chunks, v_chunks, q_offset, ranges, causal=True, scale=None, merged=True,
                             out_dtype=BF16, out=None, lse=None):
    """One launch over several key ranges [(kv_begin, kv_end), ...] of one query slice; k_chunks / v_chunks: a list
    of chunks, or one tensor.  -> (part_out [R,B,s,Hq,D] fp32, part_lse [R,B,Hq,s], out, lse); out and lse are the
    merged result, or None with merged=False."""
    import torch
    if not isinstance(k_chunks, (list, tuple)):
        k_chunks, v_chunks = [k_chunks], [v_chunks]
    B, s, Hq, D = q_slice.shape
    R = len(ranges)
    part_out = torch.empty((R, B, s, Hq, D), device=q_slice.device, dtype=torch.float32)
    part_lse = torch.empty((R, B, Hq, s), device=q_slice.device, dtype=torch.float32)
    if merged:
        if out is None:
            out = torch.empty((B, s, Hq, D), device=q_slice.device, dtype=torch.float32 if out_dtype == F32 else torch.bfloat16)
        if lse is None:
            lse = torch.empty((B, Hq, s), device=q_slice.device, dtype=torch.float32)
    else:
        out = lse = None
    kv = _ChunkedKV(k_chunks)
    p = make_params(q_slice, kv, out if merged else part_out[0], q_offset, 0, kv.shape[1], causal, scale, out_dtype)
    begins = (ctypes.c_int64 * R)(*[int(a) for a, _ in ranges])
    ends = (ctypes.c_int64 * R)(*[int(b) for _, b in ranges])
    _check(lib.slimpipe_attn_fwd_ranges(ctypes.byref(p), q_slice.data_ptr(), _chunk_table(k_chunks), _chunk_table(v_chunks),
                                        len(k_chunks), k_chunks[0].shape[1], R, begins, ends, part_out.data_ptr(), part_lse.data_ptr(),
                                        out.data_ptr() if merged else None, lse.data_ptr() if merged else None, _stream()),
           "slimpipe_attn_fwd_ranges")
    return part_out, part_lse, out, lse


def slimpipe_attn_bwd_chunked(q_slice, k_chunks, v_chunks, out, d_out, lse, q_offset, kv_begin, kv_end, dk_chunks, dv_chunks,
                              causal=True, scale=None, dq=None, dq_dtype=BF16, dq_accumulate=False, dkv_accumulate=True,
                              workspace=None):
    """As slimpipe_attn_bwd with K/V and the fp32 dK/dV accumulators given as lists of chunks."""
    import torch
    if dq is None:
        dq = torch.empty_like(q_slice, dtype=torch.float32 if dq_dtype == F32 else torch.bfloat16)
    if not _same_strides(dq, q_slice):
        raise SlimpipeError("dq must have the strides of q")
    for c in list(dk_chunks) + list(dv_chunks):
        if not _same_strides(c, k_chunks[0]):
            raise SlimpipeError("dk/dv chunks must have the strides of the k chunks")
    p = make_params(q_slice, _ChunkedKV(k_chunks), out, q_offset, kv_begin, kv_end, causal, scale)
    p.do_stride_b, p.do_stride_s, p.do_stride_h = d_out.stride(0), d_out.stride(1), d_out.stride(2)
    need = slimpipe_attn_workspace_bytes(p, True)
    if workspace is None:
        workspace = torch.empty(need, device=q_slice.device, dtype=torch.uint8)
    _check(lib.slimpipe_attn_bwd_chunked(ctypes.byref(p), q_slice.data_ptr(), _chunk_table(k_chunks), _chunk_table(v_chunks),
                                         len(k_chunks), k_chunks[0].shape[1], out.data_ptr(), d_out.data_ptr(), lse.data_ptr(),
                                         dq.data_ptr(), dq_dtype, 1 if dq_accumulate else 0, _chunk_table(dk_chunks),
                                         _chunk_table(dv_chunks), 1 if dkv_accumulate else 0, workspace.data_ptr(),
                                         workspace.numel(), _stream()),
           "slimpipe_attn_bwd_chunked")
    return dq


def slimpipe_attn_merge(outs, lses, out_dtype=BF16, out=None, lse=None):
    """Merge partial (out, lse) pairs over disjoint key sets -> (out, lse)."""
    import torch
    n = len(outs)
    B, s, Hq, D = outs[0].shape
    part_dtype = F32 if outs[0].dtype == torch.float32 else BF16
    for o in outs:
        if not o.is_contiguous():
            raise SlimpipeError("partial outputs must be contiguous")
    if out is None:
        out = torch.empty((B, s, Hq, D), device=outs[0].device, dtype=torch.float32 if out_dtype == F32 else torch.bfloat16)
    if lse is None:
        lse = torch.empty((B, Hq, s), device=outs[0].device, dtype=torch.float32)
    op = (ctypes.c_void_p * n)(*[o.data_ptr() for o in outs])
    lp = (ctypes.c_void_p * n)(*[l.data_ptr() for l in lses])
    _check(lib.slimpipe_attn_merge(n, op, lp, part_dtype, B, s, Hq, D, out.data_ptr(), out_dtype, lse.data_ptr(), _stream()),
           "slimpipe_attn_merge")
    return out, lse


def slimpipe_attn_finalize_bf16(acc, dst=None):
    import torch
    if dst is None:
        dst = torch.empty(acc.shape, device=acc.device, dtype=torch.bfloat16)
    _check(lib.slimpipe_attn_finalize_bf16(acc.data_ptr(), dst.data_ptr(), acc.numel(), _stream()), "finalize_bf16")
    return dst


KERNEL_KINDS = ("fwd", "delta", "dq", "dkdv", "merge", "finalize", "dkdv_reduce", "dq_reduce")


def slimpipe_attn_mfma_rate(random_operands):
    """-> TFLOP/s of a pure bf16 MFMA stream on this GPU (constant or random operands)."""
    import torch
    sink = torch.zeros(4, device="cuda", dtype=torch.float32)
    tf = ctypes.c_double(0.0)
    _check(lib.slimpipe_attn_mfma_rate(1 if random_operands else 0, sink.data_ptr(), ctypes.byref(tf), _stream()), "mfma_rate")
    return tf.value


def slimpipe_attn_dq_atomic_probe(s_q, heads, key_tiles, rows_per_step, placement, rotate, filler_mfma, with_atomics):
    """-> (ms, every element of dq holds the expected count, workgroups not on XCD w % 8 [placement 1 only])."""
    import torch
    dq = torch.zeros((s_q, heads, 128), device="cuda", dtype=torch.float32)
    mism = torch.zeros(1, device="cuda", dtype=torch.int32)
    ms = ctypes.c_double(0.0)
    torch.cuda.synchronize()
    rc = lib.slimpipe_attn_dq_atomic_probe(dq.data_ptr(), s_q, heads, key_tiles, rows_per_step, placement, rotate, filler_mfma,
                                           1 if with_atomics else 0, mism.data_ptr(), ctypes.byref(ms), _stream())
    _check(rc, "dq_atomic_probe (step/HIP error %s)" % ms.value)
    want = float(key_tiles * (64 // rows_per_step)) if with_atomics else 0.0
    ok = bool((dq == want).all())
    return ms.value, ok, int(mism.item())


def slimpipe_attn_xcd_rate(iters=20000, rounds=4):
    """-> {xcd: (workgroups, mean workgroup ms, last end ms)} for `rounds` workgroups of equal matrix work per compute unit."""
    import torch
    n = rounds * torch.cuda.get_device_properties(0).multi_processor_count
    t0 = torch.zeros(n, device="cuda", dtype=torch.int64)
    t1 = torch.zeros(n, device="cuda", dtype=torch.int64)
    xcc = torch.zeros(n, device="cuda", dtype=torch.int32)
    for _ in range(2):          # the second launch is the one reported (clocks settled)
        _check(lib.slimpipe_attn_xcd_rate(iters, n, t0.data_ptr(), t1.data_ptr(), xcc.data_ptr(), _stream()), "xcd_rate")
    t0, t1, xcc = t0.cpu(), t1.cpu(), xcc.cpu()
    base = int(t0.min())
    out = {}
    for x in sorted(set(xcc.tolist())):
        sel = xcc == x
        out[int(x)] = (int(sel.sum()), float((t1[sel] - t0[sel]).double().mean()) / 1e5, float(int(t1[sel].max()) - base) / 1e5)
    return out


def slimpipe_attn_profile_enable(enable):
    _check(lib.slimpipe_attn_profile_enable(1 if enable else 0), "profile_enable")


def slimpipe_attn_profile_read():
    """-> {kernel kind: (total ms, launches)} since the last read (waits for the recorded events)."""
    ms = (ctypes.c_double * len(KERNEL_KINDS))()
    n = (ctypes.c_int64 * len(KERNEL_KINDS))()
    _check(lib.slimpipe_attn_profile_read(ms, n), "profile_read")
    return {k: (ms[i], n[i]) for i, k in enumerate(KERNEL_KINDS)}
