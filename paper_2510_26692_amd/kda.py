"""ctypes binding for libkda.so (see include/kda.h for the contract).

Argument marshalling only.  Tensors are torch tensors used as device-memory
handles (``data_ptr()``), the stream is torch's current HIP stream.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# KDA_LIBRARY_PATH lets a developer point the binding at another build of the same library.
_LIB_PATH = os.environ.get("KDA_LIBRARY_PATH") or os.path.join(_HERE, "libkda.so")
_lib = None

KDA_F32, KDA_BF16 = 0, 1
_DTYPE_CODE = {torch.float32: KDA_F32, torch.bfloat16: KDA_BF16}


class KdaError(RuntimeError):
    """A libkda entry point returned a non-zero status."""

    def __init__(self, status, detail):
        super().__init__("libkda status %d (%s): %s" % (status, kda_status_string(status), detail))
        self.status = status
        self.detail = detail


class KdaDims(ctypes.Structure):
    """Mirror of ``kda_dims``."""
    _fields_ = [("batch", ctypes.c_int32), ("seqlen", ctypes.c_int64), ("heads", ctypes.c_int32),
                ("dk", ctypes.c_int32), ("dv", ctypes.c_int32), ("chunk", ctypes.c_int32),
                ("num_seqs", ctypes.c_int32), ("in_dtype", ctypes.c_int), ("out_dtype", ctypes.c_int),
                ("scale", ctypes.c_float), ("max_seqlen", ctypes.c_int64)]


class KdaPrologue(ctypes.Structure):
    """Mirror of ``kda_prologue``."""
    _fields_ = [("l2norm_eps", ctypes.c_float), ("a_scale", ctypes.c_void_p), ("dt_bias", ctypes.c_void_p)]


class KdaEpilogue(ctypes.Structure):
    """Mirror of ``kda_epilogue``."""
    _fields_ = [("rms_eps", ctypes.c_float), ("gate", ctypes.c_void_p), ("norm_weight", ctypes.c_void_p)]


def library_path():
    return _LIB_PATH


def load_library():
    """Load libkda.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError("libkda.so is not built: run `python -m paper_2510_26692_amd.build` "
                           "(there is no CPU or PyTorch fallback for the KDA kernels)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    dp = ctypes.POINTER(KdaDims)
    lib.kda_version.restype = ctypes.c_char_p
    lib.kda_last_error.restype = ctypes.c_char_p
    lib.kda_status_string.restype = ctypes.c_char_p
    lib.kda_status_string.argtypes = [ctypes.c_int]
    lib.kda_chunk_fwd_workspace_size.restype = sz
    lib.kda_chunk_fwd_workspace_size.argtypes = [dp]
    lib.kda_chunk_fwd_min_workspace_size.restype = sz
    lib.kda_chunk_fwd_min_workspace_size.argtypes = [dp]
    lib.kda_chunk_fwd.restype = ctypes.c_int
    lib.kda_chunk_fwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kda_chunk_fwd_check.restype = ctypes.c_int
    lib.kda_chunk_fwd_check.argtypes = [dp, vp, sz, vp]
    lib.kda_chunk_bwd_workspace_size.restype = sz
    lib.kda_chunk_bwd_workspace_size.argtypes = [dp]
    lib.kda_chunk_bwd.restype = ctypes.c_int
    lib.kda_chunk_bwd.argtypes = [dp] + [vp] * 15 + [vp, sz, vp]
    lib.kda_static_scratch_size.restype = ctypes.c_size_t
    lib.kda_static_scratch_size.argtypes = []
    lib.kda_chunk_fwd_static_scratch.restype = ctypes.c_int
    lib.kda_chunk_fwd_static_scratch.argtypes = [ctypes.POINTER(KdaDims)] + [ctypes.c_void_p] * 10
    lib.kda_debug_set_producers.restype = None
    lib.kda_debug_set_producers.argtypes = [ctypes.c_int]
    lib.kda_debug_set_wait_limit.restype = None
    lib.kda_debug_set_wait_limit.argtypes = [ctypes.c_ulonglong]
    lib.kda_debug_chunk_fwd_plan.restype = ctypes.c_int
    lib.kda_debug_chunk_fwd_plan.argtypes = [ctypes.POINTER(KdaDims), ctypes.c_size_t, ctypes.c_int,
                                             ctypes.POINTER(ctypes.c_int64)]
    lib.kda_debug_chunk_fwd_status.restype = ctypes.c_int
    lib.kda_debug_chunk_fwd_status.argtypes = [ctypes.POINTER(KdaDims), vp, sz, vp, ctypes.POINTER(ctypes.c_uint)]
    lib.kda_debug_stream_probe.restype = ctypes.c_int
    lib.kda_debug_stream_probe.argtypes = [ctypes.c_int, vp, sz, vp]
    lib.kda_debug_prefill_traffic_probe.restype = ctypes.c_int
    lib.kda_debug_prefill_traffic_probe.argtypes = [vp, sz, ctypes.POINTER(ctypes.c_size_t), vp]
    lib.kda_debug_mfma_probe.restype = ctypes.c_int
    lib.kda_debug_mfma_probe.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double), vp]
    lib.kda_debug_set_time_split.restype = None
    lib.kda_debug_set_time_split.argtypes = [ctypes.c_int]
    lib.kda_recurrent_step.restype = ctypes.c_int
    lib.kda_recurrent_step.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.kda_recurrent_steps_pooled.restype = ctypes.c_int
    lib.kda_recurrent_steps_pooled.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    pp, ep = ctypes.POINTER(KdaPrologue), ctypes.POINTER(KdaEpilogue)
    lib.kda_chunk_fwd_fused.restype = ctypes.c_int
    lib.kda_chunk_fwd_fused.argtypes = [dp, pp, ep, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kda_chunk_fwd_fused_workspace_size.restype = sz
    lib.kda_chunk_fwd_fused_workspace_size.argtypes = [dp, ep]
    lib.kda_chunk_fwd_fused_min_workspace_size.restype = sz
    lib.kda_chunk_fwd_fused_min_workspace_size.argtypes = [dp, ep]
    lib.kda_chunk_fwd_scalar_gate.restype = ctypes.c_int
    lib.kda_chunk_fwd_scalar_gate.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kda_recurrent_steps_pooled_scalar_gate.restype = ctypes.c_int
    lib.kda_recurrent_steps_pooled_scalar_gate.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.kda_recurrent_steps_fused.restype = ctypes.c_int
    lib.kda_recurrent_steps_fused.argtypes = [dp, pp, ep, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    _lib = lib
    return lib


def kda_version():
    return load_library().kda_version().decode()


def kda_last_error():
    return load_library().kda_last_error().decode()


def kda_debug_set_producers(enabled):
    """Fault injection (kda_debug.h): 0 makes the per-chunk workgroups of later prefill calls do nothing."""
    load_library().kda_debug_set_producers(int(bool(enabled)))


def kda_debug_set_wait_limit(ticks):
    """Ticks of the 100 MHz device clock a sequential workgroup waits for one slot (default 200 000 000)."""
    load_library().kda_debug_set_wait_limit(int(ticks))


def kda_debug_chunk_fwd_plan(dims, workspace_bytes, output_gate=False):
    """(chunk indices per time segment, time segments, ranges of the time-split scan, chunks in the first
    range, chunks in each other range) for a kda_chunk_fwd call with this workspace size."""
    out = (ctypes.c_int64 * 5)()
    st = load_library().kda_debug_chunk_fwd_plan(ctypes.byref(dims), ctypes.c_size_t(int(workspace_bytes)),
                                                 int(bool(output_gate)), out)
    if st != 0:
        raise KdaError(st, kda_last_error())
    return tuple(int(x) for x in out)


def kda_debug_chunk_fwd_status(dims, workspace):
    """The raw status word the bf16 prefill call that used `workspace` with `dims` left behind (waits for the
    current stream): bits 1, 2, 4 failures, 256 / 512 the way the time-split scan took (kda_debug.h)."""
    word = ctypes.c_uint(0)
    st = load_library().kda_debug_chunk_fwd_status(ctypes.byref(dims), _ptr(workspace),
                                                   ctypes.c_size_t(workspace.numel() * workspace.element_size()),
                                                   _stream_ptr(workspace.device), ctypes.byref(word))
    if st != 0:
        raise KdaError(st, kda_last_error())
    return int(word.value)


def kda_debug_stream_probe(mode, buffer):
    """One streaming pass over the fp32 device tensor `buffer` (a multiple of 65536 bytes, overwritten) on the
    current stream: mode 0 reads, 1 writes, 2 reads, modifies and writes in place.  Returns the bytes of the buffer."""
    _check_dev(buffer)
    assert buffer.dtype == torch.float32 and buffer.is_contiguous()
    nbytes = buffer.numel() * 4
    st = load_library().kda_debug_stream_probe(int(mode), _ptr(buffer), ctypes.c_size_t(nbytes), _stream_ptr(buffer.device))
    if st != 0:
        raise KdaError(st, kda_last_error())
    return nbytes


def kda_debug_prefill_traffic_probe(buffer):
    """One launch of the prefill traffic probe over the uint8 device tensor `buffer` (a multiple of 172032 bytes,
    overwritten) on the current stream; returns (items, bytes moved)."""
    _check_dev(buffer)
    nbytes = buffer.numel() * buffer.element_size()
    moved = ctypes.c_size_t(0)
    st = load_library().kda_debug_prefill_traffic_probe(_ptr(buffer), ctypes.c_size_t(nbytes), ctypes.byref(moved),
                                                        _stream_ptr(buffer.device))
    if st != 0:
        raise KdaError(st, kda_last_error())
    return nbytes // 172032, int(moved.value)


def kda_debug_mfma_probe(sink, workgroups, iters):
    """One launch of the matrix-core probe on the current stream; returns its floating-point operations."""
    _check_dev(sink)
    flops = ctypes.c_double(0.0)
    st = load_library().kda_debug_mfma_probe(_ptr(sink), int(workgroups), int(iters), ctypes.byref(flops), _stream_ptr(sink.device))
    if st != 0:
        raise KdaError(st, kda_last_error())
    return flops.value


def kda_debug_set_time_split(mode):
    """0 = off, 1 = on (the library estimates whether and how far to split), 2..32 = that many ranges
    (at most) whatever the estimate says."""
    load_library().kda_debug_set_time_split(int(mode))


def kda_status_string(status):
    return load_library().kda_status_string(int(status)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _check_dev(*tensors):
    dev = None
    for t in tensors:
        if t is None:
            continue
        if not t.is_cuda:
            raise ValueError("libkda takes device tensors only")
        if not t.is_contiguous():
            raise ValueError("libkda takes contiguous tensors only")
        dev = dev or t.device
        if t.device != dev:
            raise ValueError("all tensors must live on one device")
    return dev


def _stream_ptr(dev):
    return ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream)


def _out_dtype(o, out_dtype):
    """torch dtype of o: that of a tensor passed in, else `out_dtype`, else fp32."""
    dt = o.dtype if o is not None else (out_dtype or torch.float32)
    if out_dtype is not None and dt != out_dtype:
        raise ValueError("o has dtype %s but out_dtype is %s" % (dt, out_dtype))
    if dt not in _DTYPE_CODE:
        raise ValueError("unsupported output dtype %s" % dt)
    return dt


def make_chunk_dims(q, v, cu_seqlens=None, scale=1.0, max_seqlen=0, out_dtype=torch.float32):
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    N = B if cu_seqlens is None else cu_seqlens.numel() - 1
    return KdaDims(batch=B, seqlen=T, heads=H, dk=dk, dv=dv, chunk=64, num_seqs=N,
                   in_dtype=_DTYPE_CODE[q.dtype], out_dtype=_DTYPE_CODE[out_dtype], scale=float(scale),
                   max_seqlen=int(max_seqlen))


def kda_chunk_fwd_workspace_size(dims, output_gate=False):
    """Bytes for a single-segment call; output_gate=True: for kda_chunk_fwd_fused with an output gate."""
    if not output_gate:
        return int(load_library().kda_chunk_fwd_workspace_size(ctypes.byref(dims)))
    return int(load_library().kda_chunk_fwd_fused_workspace_size(ctypes.byref(dims), ctypes.byref(KdaEpilogue())))


def kda_chunk_fwd_min_workspace_size(dims, output_gate=False):
    if not output_gate:
        return int(load_library().kda_chunk_fwd_min_workspace_size(ctypes.byref(dims)))
    return int(load_library().kda_chunk_fwd_fused_min_workspace_size(ctypes.byref(dims), ctypes.byref(KdaEpilogue())))


def kda_chunk_fwd_check(dims, workspace):
    """Waits for the current stream and raises KdaError if the kda_chunk_fwd call that used
    `workspace` with `dims` reported a failed wait (see kda_chunk_fwd_check in kda.h)."""
    if workspace is None:
        return
    st = load_library().kda_chunk_fwd_check(ctypes.byref(dims), _ptr(workspace),
                                            ctypes.c_size_t(workspace.numel() * workspace.element_size()),
                                            _stream_ptr(workspace.device))
    if st != 0:
        raise KdaError(st, kda_last_error())


def _make_prologue(H, dk, l2norm_eps, a_scale, dt_bias):
    for t, shape, name in ((a_scale, (H,), "a_scale"), (dt_bias, (H, dk), "dt_bias")):
        if t is not None and (t.dtype != torch.float32 or tuple(t.shape) != shape or not t.is_cuda
                              or not t.is_contiguous()):
            raise ValueError("%s must be a contiguous fp32 device tensor of shape %r" % (name, shape))
    return KdaPrologue(l2norm_eps=float(l2norm_eps),
                       a_scale=None if a_scale is None else a_scale.data_ptr(),
                       dt_bias=None if dt_bias is None else dt_bias.data_ptr())


def _make_epilogue(v, out_gate, norm_weight, rms_eps):
    if out_gate is None:
        return None
    if out_gate.shape != v.shape or out_gate.dtype != v.dtype or not out_gate.is_cuda or not out_gate.is_contiguous():
        raise ValueError("out_gate must be a contiguous device tensor with the shape and dtype of v")
    if norm_weight is not None and (norm_weight.dtype != torch.float32 or tuple(norm_weight.shape) != (v.shape[-1],)
                                    or not norm_weight.is_cuda or not norm_weight.is_contiguous()):
        raise ValueError("norm_weight must be a contiguous fp32 device tensor of shape (dv,)")
    return KdaEpilogue(rms_eps=float(rms_eps), gate=out_gate.data_ptr(),
                       norm_weight=None if norm_weight is None else norm_weight.data_ptr())


def kda_chunk_fwd_fused(q, k, v, gate, beta, prologue=True, l2norm_eps=1e-6, a_scale=None, dt_bias=None,
                        out_gate=None, norm_weight=None, rms_eps=1e-6, **kw):
    """kda_chunk_fwd with the fused stages of kda.h.  prologue=True: q, k, beta and gate are raw
    projections (L2Norm, Sigmoid and log_alpha = -a_scale[h] softplus(gate + dt_bias[h]) run inside
    the kernel; a_scale fp32 [H], dt_bias fp32 [H,dk] on the device, or None); prologue=False: they
    are taken as kda_chunk_fwd takes them (gate = log_alpha).  out_gate (shape and dtype of v) turns
    on the output gate o <- Sigmoid(out_gate) * RMSNorm(o) * norm_weight (fp32 [dv] or None).
    Other arguments and the result as for kda_chunk_fwd."""
    pro = _make_prologue(q.shape[2], q.shape[3], l2norm_eps, a_scale, dt_bias) if prologue else None
    return kda_chunk_fwd(q, k, v, gate, beta, _fused=(pro, _make_epilogue(v, out_gate, norm_weight, rms_eps)), **kw)


def kda_chunk_fwd(q, k, v, log_alpha, beta, h0=None, cu_seqlens=None, scale=1.0, o=None,
                  hT=None, want_hT=True, workspace=None, max_seqlen=0, check=False, out_dtype=None,
                  _fused=None, _scalar_gate=False):
    """Chunkwise prefill.  q,k,log_alpha [B,T,H,dk]; v [B,T,H,dv]; beta [B,T,H];
    h0 [N,H,dk,dv] fp32 or None; cu_seqlens int32 [N+1] on device or None.
    Returns (o [B,T,H,dv], hT fp32 [N,H,dk,dv] or None); o is fp32 unless out_dtype (or the `o`
    passed in) is torch.bfloat16, which bf16 inputs allow.  `o`, `hT` and
    `workspace` (a uint8 device tensor) may be passed in to avoid allocation.
    check=True synchronises and runs kda_chunk_fwd_check before returning."""
    lib = load_library()
    dev = _check_dev(q, k, v, log_alpha, beta, h0, cu_seqlens, o, hT, workspace)
    if not (q.dtype == k.dtype == v.dtype == log_alpha.dtype == beta.dtype):
        raise ValueError("q, k, v, log_alpha, beta must share one dtype")
    if q.dtype not in _DTYPE_CODE:
        raise ValueError("unsupported input dtype %s" % q.dtype)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    if k.shape != q.shape or log_alpha.shape != ((B, T, H) if _scalar_gate else q.shape) \
            or v.shape != (B, T, H, dv) or beta.shape != (B, T, H):
        raise ValueError("inconsistent input shapes")
    odt = _out_dtype(o, out_dtype)
    dims = make_chunk_dims(q, v, cu_seqlens, scale, max_seqlen, odt)
    N = dims.num_seqs
    if o is not None and o.shape != (B, T, H, dv):
        raise ValueError("o must have shape [B,T,H,dv]")
    if h0 is not None and (h0.dtype != torch.float32 or h0.shape != (N, H, dk, dv)):
        raise ValueError("h0 must be fp32 [N,H,dk,dv]")
    if cu_seqlens is not None and cu_seqlens.dtype != torch.int32:
        raise ValueError("cu_seqlens must be int32")
    if o is None:
        o = torch.zeros(B, T, H, dv, dtype=odt, device=dev)
    if hT is None and want_hT:
        hT = torch.empty(N, H, dk, dv, dtype=torch.float32, device=dev)
    if workspace is None:
        need = kda_chunk_fwd_workspace_size(dims, output_gate=_fused is not None and _fused[1] is not None)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev) if need else None
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    tail = (_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(beta), _ptr(h0), _ptr(cu_seqlens), _ptr(o),
            _ptr(hT), _ptr(workspace), ctypes.c_size_t(ws_bytes), _stream_ptr(dev))
    if _scalar_gate:
        st = lib.kda_chunk_fwd_scalar_gate(ctypes.byref(dims), *tail)
    elif _fused is None:
        st = lib.kda_chunk_fwd(ctypes.byref(dims), *tail)
    else:
        st = lib.kda_chunk_fwd_fused(ctypes.byref(dims), *[None if f is None else ctypes.byref(f) for f in _fused],
                                     *tail)
    if st != 0:
        raise KdaError(st, kda_last_error())
    if check:
        kda_chunk_fwd_check(dims, workspace)
    return o, hT


def kda_static_scratch_size():
    return int(load_library().kda_static_scratch_size())


def kda_chunk_fwd_static_scratch(q, k, v, log_alpha, beta, o, hT=None, h0=None, cu_seqlens=None, scale=1.0, max_seqlen=0):
    """kda_chunk_fwd on the library's static scratch array: nothing is allocated, so `o` (and `hT`, if the
    final states are wanted) must be passed in.  Returns (o, hT)."""
    lib = load_library()
    dev = _check_dev(q, k, v, log_alpha, beta, h0, cu_seqlens, o, hT)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    if not (q.dtype == k.dtype == v.dtype == log_alpha.dtype == beta.dtype) or q.dtype not in _DTYPE_CODE:
        raise ValueError("q, k, v, log_alpha, beta must share a supported dtype")
    if k.shape != q.shape or log_alpha.shape != q.shape or v.shape != (B, T, H, dv) or beta.shape != (B, T, H) \
            or o.shape != (B, T, H, dv) or o.dtype not in _DTYPE_CODE:
        raise ValueError("inconsistent shapes")
    dims = make_chunk_dims(q, v, cu_seqlens, scale, max_seqlen, o.dtype)
    N = dims.num_seqs
    for name, t in (("hT", hT), ("h0", h0)):
        if t is not None and (t.dtype != torch.float32 or t.shape != (N, H, dk, dv)):
            raise ValueError("%s must be fp32 [N,H,dk,dv]" % name)
    st = lib.kda_chunk_fwd_static_scratch(ctypes.byref(dims), _ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(beta),
                                          _ptr(h0), _ptr(cu_seqlens), _ptr(o), _ptr(hT), _stream_ptr(dev))
    if st != 0:
        raise KdaError(st, kda_last_error())
    return o, hT


def kda_chunk_bwd_workspace_size(dims):
    return int(load_library().kda_chunk_bwd_workspace_size(ctypes.byref(dims)))


def kda_chunk_bwd(q, k, v, log_alpha, beta, do, dhT=None, h0=None, cu_seqlens=None, scale=1.0,
                  want_dh0=True, workspace=None, max_seqlen=0, out=None):
    """Backward pass of kda_chunk_fwd.  Inputs as there; do [B,T,H,dv] fp32, or bf16 with bf16 inputs;
    dhT fp32 [N,H,dk,dv] or None.  Returns a dict of fp32 tensors dq, dk, dlog_alpha [B,T,H,dk], dv [B,T,H,dv], dbeta [B,T,H]
    and dh0 [N,H,dk,dv] (None unless want_dh0); rows of tokens that belong to no sequence are zero
    (this wrapper allocates the gradients zero-filled; the library leaves such rows untouched).  `out`:
    the dict an earlier call returned, to be written in place instead of allocating."""
    lib = load_library()
    dev = _check_dev(q, k, v, log_alpha, beta, do, dhT, h0, cu_seqlens, workspace)
    if not (q.dtype == k.dtype == v.dtype == log_alpha.dtype == beta.dtype) or q.dtype not in _DTYPE_CODE:
        raise ValueError("q, k, v, log_alpha, beta must share a supported dtype")
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    if k.shape != q.shape or log_alpha.shape != q.shape or v.shape != (B, T, H, dv) or beta.shape != (B, T, H):
        raise ValueError("inconsistent input shapes")
    if do.dtype not in _DTYPE_CODE or do.shape != (B, T, H, dv):
        raise ValueError("do must be fp32 or bf16 [B,T,H,dv]")
    dims = make_chunk_dims(q, v, cu_seqlens, scale, max_seqlen, do.dtype)        # do has the dtype o had
    N = dims.num_seqs
    for name, t in (("dhT", dhT), ("h0", h0)):
        if t is not None and (t.dtype != torch.float32 or t.shape != (N, H, dk, dv)):
            raise ValueError("%s must be fp32 [N,H,dk,dv]" % name)
    if cu_seqlens is not None and cu_seqlens.dtype != torch.int32:
        raise ValueError("cu_seqlens must be int32")
    f32 = dict(dtype=torch.float32, device=dev)
    shapes = {"dq": (B, T, H, dk), "dk": (B, T, H, dk), "dv": (B, T, H, dv), "dlog_alpha": (B, T, H, dk),
              "dbeta": (B, T, H), "dh0": (N, H, dk, dv)}
    if out is None:
        out = {n_: torch.zeros(*sh, **f32) for n_, sh in shapes.items() if n_ != "dh0"}
        out["dh0"] = torch.empty(*shapes["dh0"], **f32) if want_dh0 else None
    else:                                   # the dict of an earlier call with the same shapes, written in place
        for n_, sh in shapes.items():
            t = out.get(n_)
            if t is None and n_ == "dh0":
                continue
            if t is None or t.dtype != torch.float32 or tuple(t.shape) != sh or not t.is_contiguous():
                raise ValueError("out[%r] must be a contiguous fp32 tensor of shape %r" % (n_, sh))
        _check_dev(q, *[t for t in out.values() if t is not None])
    if workspace is None:
        need = kda_chunk_bwd_workspace_size(dims)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev) if need else None
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib.kda_chunk_bwd(ctypes.byref(dims), _ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(beta), _ptr(h0),
                           _ptr(cu_seqlens), _ptr(do), _ptr(dhT), _ptr(out["dq"]), _ptr(out["dk"]),
                           _ptr(out["dv"]), _ptr(out["dlog_alpha"]), _ptr(out["dbeta"]), _ptr(out["dh0"]),
                           _ptr(workspace), ctypes.c_size_t(ws_bytes), _stream_ptr(dev))
    if st != 0:
        raise KdaError(st, kda_last_error())
    return out


def kda_chunk_fwd_scalar_gate(q, k, v, log_alpha_head, beta, **kw):
    """kda_chunk_fwd with one decay per (token, head): log_alpha_head [B,T,H] (the scalar-gate case
    of Eq. (1)); other arguments and the result as for kda_chunk_fwd."""
    return kda_chunk_fwd(q, k, v, log_alpha_head, beta, _scalar_gate=True, **kw)


def kda_recurrent_step(q, k, v, log_alpha, beta, S, scale=1.0, o=None, out_dtype=None):
    """One decode step.  q,k,log_alpha [N,H,dk]; v [N,H,dv]; beta [N,H];
    S fp32 [N,H,dk,dv], updated in place.  Returns o [N,H,dv] (fp32, or bf16 on request as in
    kda_chunk_fwd)."""
    lib = load_library()
    dev = _check_dev(q, k, v, log_alpha, beta, S, o)
    N, H, dk = q.shape
    dv = v.shape[-1]
    if S.dtype != torch.float32 or S.shape != (N, H, dk, dv):
        raise ValueError("S must be fp32 [N,H,dk,dv]")
    if q.dtype not in _DTYPE_CODE or not (q.dtype == k.dtype == v.dtype == log_alpha.dtype == beta.dtype):
        raise ValueError("q, k, v, log_alpha, beta must share a supported dtype")
    odt = _out_dtype(o, out_dtype)
    if o is None:
        o = torch.empty(N, H, dv, dtype=odt, device=dev)
    elif o.shape != (N, H, dv):
        raise ValueError("o must have shape [N,H,dv]")
    dims = KdaDims(batch=N, seqlen=1, heads=H, dk=dk, dv=dv, chunk=64, num_seqs=N,
                   in_dtype=_DTYPE_CODE[q.dtype], out_dtype=_DTYPE_CODE[odt], scale=float(scale), max_seqlen=0)
    st = lib.kda_recurrent_step(ctypes.byref(dims), _ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha),
                                _ptr(beta), _ptr(S), _ptr(o), _stream_ptr(dev))
    if st != 0:
        raise KdaError(st, kda_last_error())
    return o


def kda_recurrent_steps_fused(q, k, v, gate, beta, S_pool, state_indices=None, prologue=True, l2norm_eps=1e-6,
                              a_scale=None, dt_bias=None, out_gate=None, norm_weight=None, rms_eps=1e-6, **kw):
    """kda_recurrent_steps_pooled with the fused stages (see kda_chunk_fwd_fused)."""
    pro = _make_prologue(q.shape[2], q.shape[3], l2norm_eps, a_scale, dt_bias) if prologue else None
    return kda_recurrent_steps_pooled(q, k, v, gate, beta, S_pool, state_indices,
                                      _fused=(pro, _make_epilogue(v, out_gate, norm_weight, rms_eps)), **kw)


def kda_recurrent_steps_pooled_scalar_gate(q, k, v, log_alpha_head, beta, S_pool, state_indices=None, **kw):
    """kda_recurrent_steps_pooled with one decay per (token, head): log_alpha_head [N,Tq,H]."""
    return kda_recurrent_steps_pooled(q, k, v, log_alpha_head, beta, S_pool, state_indices, _scalar_gate=True, **kw)


def kda_recurrent_steps_pooled(q, k, v, log_alpha, beta, S_pool, state_indices=None, scale=1.0, o=None,
                               out_dtype=None, _fused=None, _scalar_gate=False):
    """Decode over a state pool.  q,k,log_alpha [N,Tq,H,dk]; v [N,Tq,H,dv]; beta [N,Tq,H];
    S_pool fp32 [P,H,dk,dv], the addressed states updated in place; state_indices int32 [N] on the
    device (negative = skip) or None for 0..N-1.  Returns o [N,Tq,H,dv] (fp32, or bf16 on request as in
    kda_chunk_fwd)."""
    lib = load_library()
    dev = _check_dev(q, k, v, log_alpha, beta, S_pool, state_indices, o)
    N, Tq, H, dk = q.shape
    dv = v.shape[-1]
    if S_pool.dtype != torch.float32 or S_pool.dim() != 4 or S_pool.shape[1:] != (H, dk, dv):
        raise ValueError("S_pool must be fp32 [P,H,dk,dv]")
    if q.dtype not in _DTYPE_CODE or not (q.dtype == k.dtype == v.dtype == log_alpha.dtype == beta.dtype):
        raise ValueError("q, k, v, log_alpha, beta must share a supported dtype")
    if k.shape != q.shape or log_alpha.shape != ((N, Tq, H) if _scalar_gate else q.shape) \
            or v.shape != (N, Tq, H, dv) or beta.shape != (N, Tq, H):
        raise ValueError("inconsistent input shapes")
    if state_indices is None:
        if S_pool.shape[0] < N:
            raise ValueError("S_pool holds fewer states than there are sequences")
    elif state_indices.dtype != torch.int32 or state_indices.shape != (N,):
        raise ValueError("state_indices must be int32 [N]")
    odt = _out_dtype(o, out_dtype)
    if o is None:
        o = torch.zeros(N, Tq, H, dv, dtype=odt, device=dev)
    elif o.shape != (N, Tq, H, dv):
        raise ValueError("o must have shape [N,Tq,H,dv]")
    dims = KdaDims(batch=N, seqlen=Tq, heads=H, dk=dk, dv=dv, chunk=64, num_seqs=N,
                   in_dtype=_DTYPE_CODE[q.dtype], out_dtype=_DTYPE_CODE[odt], scale=float(scale), max_seqlen=0)
    tail = (_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(beta), _ptr(S_pool), _ptr(state_indices), _ptr(o),
            _stream_ptr(dev))
    if _scalar_gate:
        st = lib.kda_recurrent_steps_pooled_scalar_gate(ctypes.byref(dims), *tail)
    elif _fused is None:
        st = lib.kda_recurrent_steps_pooled(ctypes.byref(dims), *tail)
    else:
        st = lib.kda_recurrent_steps_fused(ctypes.byref(dims),
                                           *[None if f is None else ctypes.byref(f) for f in _fused], *tail)
    if st != 0:
        raise KdaError(st, kda_last_error())
    return o
