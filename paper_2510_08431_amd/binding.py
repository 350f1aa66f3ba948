"""ctypes binding of the attn_jvp C-ABI library: argument marshalling only.

PyTorch supplies device memory (`data_ptr()`) and the current HIP stream; every step of
the computation runs inside the library's kernels.  There is no CPU or eager fallback:
if the shared library is missing, loading raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libattn_jvp.so")

KERNEL_AUTO, KERNEL_FP32, KERNEL_MFMA = 0, 1, 2
LAYOUT_BHLD = 0   # tensors are [B, H, L, d]
LAYOUT_BLHD = 1   # tensors are [B, L, H, d] (lse stays [B, H, Lq])
FLAG_FAST = 1     # MFMA kernel: P~ and H~ as single bf16 terms (6 matrix products per key block; not tolerance-safe)
FLAG_F16_ALWAYS = 4   # MFMA kernel: fp16 value path also for short key sequences (given a workspace)
FLAG_NO_LOCKSTEP = 8   # MFMA kernel, running-reference fp16 tier: no lock-step start of the tiles of an XCD
FLAG_NO_RESIDENT = 16   # MFMA kernel: one workgroup per query tile instead of resident workgroups
FLAG_NO_F16 = 2   # MFMA kernel: hi + lo bf16 pairs (9 products) even when a workspace is available
_DTYPE_CODE = {torch.bfloat16: 0, torch.float32: 1}


class AttnJvpOpts(ctypes.Structure):
    _fields_ = [("in_dtype", ctypes.c_int), ("out_dtype", ctypes.c_int), ("stream", ctypes.c_void_p),
                ("kernel", ctypes.c_int), ("flags", ctypes.c_int), ("workspace", ctypes.c_void_p),
                ("workspace_bytes", ctypes.c_size_t), ("timing_events", ctypes.c_void_p * 2),
                ("layout", ctypes.c_int), ("reserved", ctypes.c_int)]


class AttnJvpError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"attn_jvp error {code}: {message}")
        self.code = code


_lib = None


def load_library():
    """Load libattn_jvp.so (built in-tree by __graft_entry__.build()) and declare its symbols."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build the HIP library first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    common = [vp] * 9 + [ci] * 5 + [cf]
    lib.attn_jvp_fwd.argtypes = common
    lib.attn_jvp_fwd.restype = ci
    lib.attn_jvp_fwd_ex.argtypes = common + [ctypes.POINTER(AttnJvpOpts)]
    lib.attn_jvp_fwd_ex.restype = ci
    lib.attn_jvp_fwd_static.argtypes = common + [ctypes.POINTER(AttnJvpOpts)]
    lib.attn_jvp_fwd_static.restype = ci
    lib.attn_jvp_static_scratch_bytes.argtypes = []
    lib.attn_jvp_static_scratch_bytes.restype = ctypes.c_size_t
    lib.attn_jvp_strerror.argtypes = [ci]
    lib.attn_jvp_strerror.restype = ctypes.c_char_p
    lib.attn_jvp_version.argtypes = []
    lib.attn_jvp_version.restype = ci
    lib.attn_jvp_rmsnorm_fwd.argtypes = [vp] * 5 + [ctypes.c_longlong, ci, ctypes.c_float, ci, vp]
    lib.attn_jvp_rmsnorm_fwd.restype = ci
    lib.attn_jvp_mfma_rate_probe.argtypes = [vp, vp, ci, ci, vp, ctypes.POINTER(ctypes.c_longlong), ctypes.POINTER(ci)]
    lib.attn_jvp_mfma_rate_probe.restype = ci
    lib.attn_jvp_workspace_bytes.argtypes = [ci] * 5
    lib.attn_jvp_workspace_bytes.restype = ctypes.c_size_t
    _lib = lib
    return lib


def attn_jvp_strerror(code):
    return load_library().attn_jvp_strerror(int(code)).decode()


def attn_jvp_version():
    return load_library().attn_jvp_version()


def attn_jvp_workspace_bytes(B, H, Lq, Lkv, d):
    return int(load_library().attn_jvp_workspace_bytes(B, H, Lq, Lkv, d))


_workspaces = {}


def _workspace(device, stream, nbytes):
    """A scratch tensor from torch's allocator per (device, stream), grown on demand and reused across calls.

    Calls enqueued on one stream run in order, so they can share scratch; calls on different streams may overlap
    and get separate buffers.  Callers that want to own the memory pass their own `workspace`."""
    key = (device, stream.cuda_stream)
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < nbytes:
        with torch.cuda.stream(stream):      # so that torch's caching allocator ties the block to this stream
            ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    return ws


def _ptr(t):
    return t.data_ptr() if t is not None else None


def _check_inputs(q, k, v, tq, tk, tv, layout=LAYOUT_BHLD):
    if q.dim() != 4 or k.dim() != 4:
        raise ValueError("q and k must be [B, H, L, d] (or [B, L, H, d] with layout=LAYOUT_BLHD)")
    if layout == LAYOUT_BLHD:
        B, Lq, H, d = q.shape
        Lkv = k.shape[1]
        shape = lambda L: (B, L, H, d)
    elif layout == LAYOUT_BHLD:
        B, H, Lq, d = q.shape
        Lkv = k.shape[2]
        shape = lambda L: (B, H, L, d)
    else:
        raise ValueError(f"unknown layout {layout}")
    if (tk is None) != (tv is None):
        raise ValueError("tk and tv must both be given or both be None (zero key/value tangents)")
    if tq is None and tk is not None:
        raise ValueError("tq=None means no tangents at all: tk and tv must be None too")
    for name, t, L in (("q", q, Lq), ("tq", tq, Lq), ("k", k, Lkv), ("v", v, Lkv), ("tk", tk, Lkv), ("tv", tv, Lkv)):
        if t is None:
            continue
        if tuple(t.shape) != shape(L):
            raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {shape(L)}")
        if t.dtype != q.dtype or t.device != q.device:
            raise ValueError(f"{name}: dtype/device differ from q")
        if not t.is_contiguous():
            raise ValueError(f"{name} must be contiguous")
    if q.dtype not in _DTYPE_CODE:
        raise ValueError(f"unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("tensors must live on the GPU; there is no CPU path")
    return B, H, Lq, Lkv, d


def attn_jvp_fwd_ex(q, k, v, tq, tk, tv, scale, out=None, out_dtype=torch.float32, kernel=KERNEL_AUTO, stream=None,
                    flags=0, workspace="auto", timing_events=None, layout=LAYOUT_BHLD):
    """Enqueue O, tO, lse = attention forward + JVP on the current (or given) stream.

    q, tq: [B, H, Lq, d]; k, v, tk, tv: [B, H, Lkv, d]; bf16 or fp32, contiguous, on the GPU.  tk and tv may both be
    None: zero key/value tangents (cross-attention onto a context without tangent); tq, tk, tv all None: plain
    attention forward, the returned `to` is None.
    out: optional (o, to, lse) to write into.  workspace: "auto" (a cached per-device torch buffer), None (no
    scratch: the kernel then uses its bf16-pair path), a uint8 CUDA tensor, or "static" (the C entry point
    attn_jvp_fwd_static: the library's own static device array; with `out` given the call allocates nothing).  layout=LAYOUT_BLHD: all eight
    tensors are [B, L, H, d] instead (lse stays [B, H, Lq]).  timing_events: optional pair of
    torch.cuda.Event(enable_timing=True) that the library records right before and after the main kernel.
    Returns (o, to, lse); asynchronous.
    """
    lib = load_library()
    B, H, Lq, Lkv, d = _check_inputs(q, k, v, tq, tk, tv, layout)
    if out is None:
        o = torch.empty(q.shape, dtype=out_dtype, device=q.device)     # same layout as q
        to = torch.empty_like(o) if tq is not None else None
        lse = torch.empty(B, H, Lq, dtype=torch.float32, device=q.device)
    else:
        o, to, lse = out
        out_dtype = o.dtype
        if (tuple(o.shape) != tuple(q.shape) or tuple(lse.shape) != (B, H, Lq)
                or (to is not None and tuple(to.shape) != tuple(q.shape)) or (to is None and tq is not None)):
            raise ValueError("out must be (o, to, lse) with o, to shaped like q and lse [B, H, Lq]")
    if out_dtype not in (torch.float32, q.dtype):
        raise ValueError("out_dtype must be float32 or the input dtype")
    opts = AttnJvpOpts()
    opts.in_dtype = _DTYPE_CODE[q.dtype]
    opts.out_dtype = 0 if out_dtype == torch.float32 else 1
    if stream is None:
        stream = torch.cuda.current_stream(q.device)
    opts.stream = stream.cuda_stream
    opts.kernel = int(kernel)
    opts.flags = int(flags)
    opts.layout = int(layout)
    entry = lib.attn_jvp_fwd_ex
    if isinstance(workspace, str) and workspace == "static":
        entry = lib.attn_jvp_fwd_static
        workspace = None
    if isinstance(workspace, str) and workspace == "auto":
        need = lib.attn_jvp_workspace_bytes(B, H, Lq, Lkv, d) if q.dtype == torch.bfloat16 else 0
        workspace = _workspace(q.device, stream, need) if need else None
    if workspace is not None:
        opts.workspace = workspace.data_ptr()
        opts.workspace_bytes = workspace.numel() * workspace.element_size()
    if timing_events is not None:
        for i, ev in enumerate(timing_events):
            if not ev.cuda_event:      # torch creates the HIP event lazily, at its first record
                ev.record(stream)
            opts.timing_events[i] = ev.cuda_event
    with torch.cuda.device(q.device):
        rc = entry(q.data_ptr(), k.data_ptr(), v.data_ptr(), _ptr(tq), _ptr(tk), _ptr(tv),
                   o.data_ptr(), _ptr(to), lse.data_ptr(), B, H, Lq, Lkv, d, float(scale), ctypes.byref(opts))
    if rc != 0:
        raise AttnJvpError(rc, attn_jvp_strerror(rc))
    return o, to, lse


def attn_jvp_static_scratch_bytes():
    return int(load_library().attn_jvp_static_scratch_bytes())


def attn_jvp_fwd_static(q, k, v, tq, tk, tv, scale, out, **kw):
    """The C entry point `attn_jvp_fwd_static`: as attn_jvp_fwd_ex, with the library's static device scratch in
    place of a workspace.  `out` = (o, to, lse) is required, so that nothing is allocated on the way."""
    if out is None:
        raise ValueError("attn_jvp_fwd_static writes into caller-provided outputs: pass out=(o, to, lse)")
    return attn_jvp_fwd_ex(q, k, v, tq, tk, tv, scale, out=out, workspace="static", **kw)


def attn_jvp_rmsnorm_fwd(x, tx, w, eps, out=None, stream=None):
    """Enqueue y, ty = RMS normalisation with gain w and its JVP over the last dimension.

    x, tx: [..., d] bf16 or fp32, contiguous, on the GPU; w: [d] float32.  out: optional (y, ty) to write into
    (may be (x, tx) themselves).  Returns (y, ty); asynchronous."""
    lib = load_library()
    if x.dtype not in _DTYPE_CODE or tx.dtype != x.dtype or tuple(tx.shape) != tuple(x.shape):
        raise ValueError("x and tx must have the same shape and dtype (bf16 or fp32)")
    if not (x.is_cuda and tx.is_cuda and w.is_cuda):
        raise ValueError("tensors must live on the GPU; there is no CPU path")
    if not (x.is_contiguous() and tx.is_contiguous() and w.is_contiguous()):
        raise ValueError("x, tx and w must be contiguous")
    d = x.shape[-1]
    if w.dtype != torch.float32 or tuple(w.shape) != (d,):
        raise ValueError("w must be a float32 vector of length d")
    rows = x.numel() // d
    if out is None:
        y, ty = torch.empty_like(x), torch.empty_like(tx)
    else:
        y, ty = out
        if y.dtype != x.dtype or ty.dtype != x.dtype or tuple(y.shape) != tuple(x.shape) or tuple(ty.shape) != tuple(x.shape):
            raise ValueError("out must be (y, ty) shaped and typed like x")
    if stream is None:
        stream = torch.cuda.current_stream(x.device)
    with torch.cuda.device(x.device):
        rc = lib.attn_jvp_rmsnorm_fwd(x.data_ptr(), tx.data_ptr(), w.data_ptr(), y.data_ptr(), ty.data_ptr(),
                                      rows, d, float(eps), _DTYPE_CODE[x.dtype], stream.cuda_stream)
    if rc != 0:
        raise AttnJvpError(rc, attn_jvp_strerror(rc))
    return y, ty


def attn_jvp_mfma_rate_probe(operands, out, f16, iters, stream=None):
    """Enqueue the library's back-to-back MFMA loop on the operand values given (measurement aid).

    operands: uint8/int tensor of 8 * 256 * 16 bytes on the GPU (bf16 or fp16 bit patterns); out: float32 tensor with
    at least 256 elements per compute unit.  Returns the number of floating-point operations the launch performs;
    the caller times it."""
    lib = load_library()
    if not (operands.is_cuda and out.is_cuda and operands.is_contiguous() and out.is_contiguous()):
        raise ValueError("operands and out must be contiguous GPU tensors")
    if operands.numel() * operands.element_size() < 8 * 256 * 16:
        raise ValueError("operands must hold 8 x 256 x 16 bytes")
    cus = torch.cuda.get_device_properties(out.device).multi_processor_count
    if out.dtype != torch.float32 or out.numel() < 256 * cus:
        raise ValueError("out must be float32 with 256 elements per compute unit")
    if stream is None:
        stream = torch.cuda.current_stream(out.device)
    per_wave, waves = ctypes.c_longlong(0), ctypes.c_int(0)
    with torch.cuda.device(out.device):
        rc = lib.attn_jvp_mfma_rate_probe(operands.data_ptr(), out.data_ptr(), int(bool(f16)), int(iters),
                                          stream.cuda_stream, ctypes.byref(per_wave), ctypes.byref(waves))
    if rc != 0:
        raise AttnJvpError(rc, attn_jvp_strerror(rc))
    return 32768.0 * per_wave.value * waves.value


def attn_jvp_fwd(q, k, v, tq, tk, tv, scale, out=None):
    """The C entry point `attn_jvp_fwd`: bf16 inputs, fp32 outputs, no workspace, the default stream.

    When torch's current stream is not the default stream the same kernel is enqueued there through
    `attn_jvp_fwd_ex` instead (no workspace either)."""
    lib = load_library()
    B, H, Lq, Lkv, d = _check_inputs(q, k, v, tq, tk, tv)
    if q.dtype != torch.bfloat16:
        raise ValueError("attn_jvp_fwd takes bf16 inputs; use attn_jvp_fwd_ex for fp32")
    if torch.cuda.current_stream(q.device).cuda_stream != 0:
        return attn_jvp_fwd_ex(q, k, v, tq, tk, tv, scale, out=out, workspace=None)
    if out is None:
        o = torch.empty(B, H, Lq, d, dtype=torch.float32, device=q.device)
        to = torch.empty_like(o) if tq is not None else None
        lse = torch.empty(B, H, Lq, dtype=torch.float32, device=q.device)
    else:
        o, to, lse = out
    with torch.cuda.device(q.device):
        rc = lib.attn_jvp_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), _ptr(tq), _ptr(tk), _ptr(tv),
                              o.data_ptr(), _ptr(to), lse.data_ptr(), B, H, Lq, Lkv, d, float(scale))
    if rc != 0:
        raise AttnJvpError(rc, attn_jvp_strerror(rc))
    return o, to, lse
