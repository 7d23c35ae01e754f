"""ctypes binding of libvardrop.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/vardrop.h).  Tensors
are torch tensors on the GPU; torch provides device memory and the current HIP stream,
nothing else.  There is no fallback: if the shared library is missing, loading fails.
"""
import ctypes
import os

import torch

F32 = 0
BF16 = 1
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

_c_int = ctypes.c_int
_c_i64 = ctypes.c_int64
_c_u32 = ctypes.c_uint32
_c_u64 = ctypes.c_uint64
_c_size = ctypes.c_size_t
_ptr = ctypes.c_void_p

_SIGNATURES = {
    "vardrop_create": (_c_int, [ctypes.POINTER(_ptr), _c_int]),
    "vardrop_destroy": (None, [_ptr]),
    "vardrop_strerror": (ctypes.c_char_p, [_c_int]),
    "vardrop_last_hip_error": (_c_int, [_ptr]),
    "vardrop_hash_strided_workspace_bytes": (ctypes.c_size_t, [_c_int, _c_int, _c_int]),
    "vardrop_hash_default_cutoff": (_c_int, [_c_int]),
    "vardrop_profile_select": (_c_int, [_ptr, _c_int]),
    "vardrop_profile_read": (_c_int, [_ptr, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(_c_int)]),
    "vardrop_profile_stride": (_c_int, [_ptr, _c_int]),
    "vardrop_signal_after": (_c_int, [_ptr, _c_int, _ptr]),
    "vardrop_profile_read_all": (_c_int, [_ptr, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(_c_int)]),
    "vardrop_kernel_name": (ctypes.c_char_p, [_c_int]),
    "vardrop_hash_workspace_bytes": (_c_size, [_c_int] * 6),
    "vardrop_hash": (_c_int, [_ptr, _ptr, _c_int, _c_int, _c_int, _c_i64, _c_i64, _c_i64, _c_int, _c_int, _c_int,
                              _ptr, _ptr, _ptr, _ptr, _c_size, _ptr]),
    "vardrop_sample_workspace_bytes": (_c_size, [_c_int]),
    "vardrop_sample": (_c_int, [_ptr, _ptr, _c_int, _c_u32, _c_u32, _c_u32, _c_u64, _c_u64,
                                _ptr, _ptr, _ptr, _ptr, _ptr, _c_size, _ptr]),
    "vardrop_sample_dev": (_c_int, [_ptr, _ptr, _c_int, _c_u32, _c_u32, _c_u32, _c_u64, _ptr, _c_int,
                                    _ptr, _ptr, _ptr, _ptr, _c_size, _ptr]),
    "vardrop_sample_nearest_workspace_bytes": (_c_size, [_c_int, _c_int]),
    "vardrop_sample_nearest": (_c_int, [_ptr, _ptr, _ptr, _c_int, _c_int, _c_u32, _c_u32, _c_u32,
                                        _ptr, _ptr, _ptr, _ptr, _ptr, _c_size, _ptr]),
    "vardrop_sample_nearest_noalloc": (_c_int, [_ptr, _ptr, _ptr, _c_int, _c_int, _c_u32, _c_u32, _c_u32,
                                                _ptr, _ptr, _ptr, _ptr]),
    "vardrop_gather": (_c_int, [_ptr, _ptr, _c_int, _c_int, _c_int, _c_int, _ptr, _c_int, _ptr, _ptr]),
    "vardrop_scatter": (_c_int, [_ptr, _ptr, _c_int, _c_int, _c_int, _c_int, _ptr, _c_int, _ptr, _ptr]),
    "vardrop_gather_dev": (_c_int, [_ptr, _ptr, _c_int, _c_int, _c_int, _c_int, _ptr, _ptr, _c_int, _ptr, _ptr, _ptr]),
    "vardrop_scatter_dev": (_c_int, [_ptr, _ptr, _c_int, _c_int, _c_int, _c_int, _ptr, _ptr, _c_int, _ptr, _ptr, _ptr]),
    "vardrop_embed_saved_bytes": (_c_size, [_c_int] * 4),
    "vardrop_embed_workspace_bytes": (_c_size, [_c_int] * 5),
    "vardrop_embed_fwd": (_c_int, [_ptr, _ptr, _c_int, _c_int, _c_int, _c_i64, _c_i64, _ptr, _c_int, _c_int,
                                   _ptr, _ptr, _c_int, _c_int, _ptr, _ptr, _ptr]),
    "vardrop_embed_bwd": (_c_int, [_ptr, _ptr, _c_int, _c_int, _c_int, _c_int, _c_int, _ptr, _ptr, _ptr,
                                   _ptr, _c_size, _ptr]),
    "vardrop_embed_fwd_dev": (_c_int, [_ptr, _ptr, _c_int, _c_int, _c_int, _c_i64, _c_i64, _ptr, _ptr, _c_int, _ptr, _c_int,
                                       _ptr, _ptr, _c_int, _c_int, _ptr, _ptr, _ptr]),
    "vardrop_embed_bwd_dev": (_c_int, [_ptr, _ptr, _c_int, _ptr, _c_int, _c_int, _c_int, _c_int, _ptr, _ptr, _ptr,
                                       _ptr, _c_size, _ptr]),
    "vardrop_attn_fwd_dev": (_c_int, [_ptr, _ptr, _c_int, _ptr, _c_int, _ptr, _c_int, _c_int, _c_int] + [_ptr] * 8 +
                             [_ptr, _ptr, _ptr, _c_size, _ptr]),
    "vardrop_attn_saved_bytes": (_c_size, [_c_int] * 5),
    "vardrop_attn_workspace_bytes": (_c_size, [_c_int] * 5),
    "vardrop_attn_fwd": (_c_int, [_ptr, _ptr, _c_int, _c_int, _c_int, _c_int, _c_int] + [_ptr] * 8 +
                         [_ptr, _ptr, _ptr, _c_size, _ptr]),
    "vardrop_gather_attn_fwd": (_c_int, [_ptr, _ptr, _c_int, _c_int, _ptr, _c_int, _c_int, _c_int, _c_int] + [_ptr] * 8 +
                                [_ptr, _ptr, _ptr, _ptr, _c_size, _ptr]),
    "vardrop_attn_bwd": (_c_int, [_ptr, _ptr, _ptr, _c_int, _c_int, _c_int, _c_int, _c_int] + [_ptr] * 4 +
                         [_ptr] + [_ptr] * 9 + [_ptr, _c_size, _ptr]),
    "vardrop_gather_attn_fwd_dev": (_c_int, [_ptr, _ptr, _c_int, _c_int, _ptr, _ptr, _c_int, _ptr, _c_int, _c_int, _c_int] +
                                    [_ptr] * 8 + [_ptr, _ptr, _ptr, _ptr, _c_size, _ptr]),
    "vardrop_attn_bwd_dev": (_c_int, [_ptr, _ptr, _ptr, _c_int, _ptr, _c_int, _ptr, _c_int, _c_int, _c_int] + [_ptr] * 4 +
                             [_ptr] + [_ptr] * 9 + [_ptr, _c_size, _ptr]),
}


class VarDropError(RuntimeError):
    def __init__(self, code, where, detail=""):
        self.code = code
        super().__init__("%s failed: %s (%d)%s" % (where, _strerror(code), code, detail))


def library_path():
    return os.path.join(_HERE, "libvardrop.so")


def load_library():
    """Loads libvardrop.so (built by paper_2501_14183_amd/build.py) and declares its signatures."""
    global _LIB
    if _LIB is None:
        path = library_path()
        if not os.path.exists(path):
            raise ImportError("libvardrop.so is not built: run `python -m paper_2501_14183_amd.build` "
                              "(there is no fallback implementation)")
        lib = ctypes.CDLL(path)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _LIB = lib
    return _LIB


def _strerror(code):
    return load_library().vardrop_strerror(code).decode()


def _p(t):
    return None if t is None else t.data_ptr()


def _stream(t, stream=None):
    """Raw hipStream_t: `stream` (an integer handle, e.g. torch.cuda.Stream.cuda_stream) or torch's current one."""
    return torch.cuda.current_stream(t.device).cuda_stream if stream is None else stream


def _own_buffers(stream, what, **bufs):
    """Temporaries come from torch's allocator, which hands freed memory to work on torch's current stream: with a
    raw `stream` handle the caller has to own every buffer the call uses."""
    if stream is not None:
        missing = [k for k, v in bufs.items() if v is None]
        if missing:
            raise TypeError("%s on a raw stream needs caller-owned %s" % (what, ", ".join(missing)))


def _dtype_code(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("tokens and weights must be float32 or bfloat16")


class Context:
    """Owns a vardrop_ctx on one device."""

    def __init__(self, device=0):
        self._lib = load_library()
        self.device = torch.device("cuda", device) if isinstance(device, int) else torch.device(device)
        h = ctypes.c_void_p()
        rc = self._lib.vardrop_create(ctypes.byref(h), self.device.index or 0)
        if rc != 0:
            raise VarDropError(rc, "vardrop_create")
        self.handle = h

    def check(self, rc, where):
        if rc != 0:
            detail = ""
            if rc == -3:
                detail = " hipError=%d" % self._lib.vardrop_last_hip_error(self.handle)
            raise VarDropError(rc, where, detail)

    def close(self):
        if getattr(self, "handle", None):
            self._lib.vardrop_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def vardrop_kernel_name(kid):
    name = load_library().vardrop_kernel_name(kid)
    return None if name is None else name.decode()


def vardrop_profile_select(ctx, kid):
    """Brackets every launch of kernel `kid` with HIP events (-1: off)."""
    ctx.check(ctx._lib.vardrop_profile_select(ctx.handle, kid), "vardrop_profile_select")


def vardrop_profile_stride(ctx, stride):
    """Bracket only every `stride`-th launch of the selected kernel (takes effect at the next select)."""
    ctx.check(ctx._lib.vardrop_profile_stride(ctx.handle, stride), "vardrop_profile_stride")


def vardrop_signal_after(ctx, kid, event):
    """The next launch of kernel `kid` carries `event` (a raw hipEvent_t handle, e.g. torch.cuda.Event.cuda_event of
    an event that has been recorded once; None cancels) as the completion event of its own dispatch."""
    ctx.check(ctx._lib.vardrop_signal_after(ctx.handle, kid, ctypes.c_void_p(event) if event else None), "vardrop_signal_after")


def vardrop_profile_read(ctx):
    """-> (summed duration in ms, number of launches) since the last read or select."""
    ms = ctypes.c_double()
    n = _c_int()
    ctx.check(ctx._lib.vardrop_profile_read(ctx.handle, ctypes.byref(ms), ctypes.byref(n)), "vardrop_profile_read")
    return ms.value, n.value


K_ALL = -2          # vardrop_profile_select: every kernel


def vardrop_profile_read_all(ctx):
    """-> {kernel name: (summed duration in ms, launches)} since the last read or select, for the kernels that ran."""
    n = 0
    while load_library().vardrop_kernel_name(n) is not None:
        n += 1
    ms = (ctypes.c_double * n)()
    cnt = (_c_int * n)()
    ctx.check(ctx._lib.vardrop_profile_read_all(ctx.handle, ms, cnt), "vardrop_profile_read_all")
    return {vardrop_kernel_name(k): (ms[k], cnt[k]) for k in range(n) if cnt[k]}


def vardrop_hash(ctx, x, k, f_min=1, f_max=None, want_abar=False, out=None, stream=None, ws=None):
    """x float32 [B, N, L] (any strides) -> (topk int32 [N, k], hash int64 [N] (the uint64 bits), abar or None).

    out: optional (topk, hash) tensors to write into instead of allocating.
    ws:  optional uint8 workspace for inputs whose time stride is not 1 (allocated when missing)."""
    if x.dtype != torch.float32 or x.dim() != 3:
        raise TypeError("x must be float32 [B, N, L]")
    B, N, L = x.shape
    if f_max is None:
        f_max = ctx._lib.vardrop_hash_default_cutoff(L)      # the paper's default cut-off (the library's rule)
    if out is not None:
        topk, hsh = out
    else:
        topk = torch.empty((N, k), dtype=torch.int32, device=x.device)
        hsh = torch.empty((N,), dtype=torch.int64, device=x.device)
    abar = torch.empty((N, f_max - f_min + 1), dtype=torch.float32, device=x.device) if want_abar else None
    sb, sn, st = x.stride()
    if st != 1:
        _own_buffers(stream, "vardrop_hash of a strided batch", ws=ws)
    if st != 1 and ws is None:
        ws = torch.empty(ctx._lib.vardrop_hash_strided_workspace_bytes(B, N, L), dtype=torch.uint8, device=x.device)
    rc = ctx._lib.vardrop_hash(ctx.handle, _p(x), B, N, L, sb, sn, st, k, f_min, f_max,
                               _p(topk), _p(hsh), _p(abar), _p(ws), 0 if ws is None else ws.numel(),
                               _stream(x, stream))
    ctx.check(rc, "vardrop_hash")
    return topk, hsh, abar


def vardrop_sample(ctx, hsh, gs, ratio_num, ratio_den, seed, step, counts_host=None, out=None, stream=None):
    """hash int64 [N] -> (group_id int32 [N], sel int32 [N] (first N' valid), counts int32 [2] = {N', G}).

    counts_host: optional pinned int32 [2] CPU tensor that receives the counts asynchronously.
    out: optional (group_id, sel, counts) tensors to write into instead of allocating.
    """
    N = hsh.shape[0]
    if out is not None:
        gid, sel, counts = out
    else:
        gid = torch.empty((N,), dtype=torch.int32, device=hsh.device)
        sel = torch.empty((N,), dtype=torch.int32, device=hsh.device)
        counts = torch.empty((2,), dtype=torch.int32, device=hsh.device)
    rc = ctx._lib.vardrop_sample(ctx.handle, _p(hsh), N, gs, ratio_num, ratio_den, seed, step,
                                 _p(gid), _p(sel), _p(counts), _p(counts_host), None, 0, _stream(hsh, stream))
    ctx.check(rc, "vardrop_sample")
    return gid, sel, counts


def vardrop_gather(ctx, tokens, sel, n_sel, out=None, stream=None):
    """tokens [B, N, d], sel int32 -> [B, n_sel, d] (written into `out` when given)."""
    B, N, d = tokens.shape
    if out is None:
        out = torch.empty((B, n_sel, d), dtype=tokens.dtype, device=tokens.device)
    rc = ctx._lib.vardrop_gather(ctx.handle, _p(tokens), B, N, d, _dtype_code(tokens), _p(sel), n_sel, _p(out),
                                 _stream(tokens, stream))
    ctx.check(rc, "vardrop_gather")
    return out


def vardrop_scatter(ctx, dxs, sel, n_sel, N, stream=None):
    """dxs [B, n_sel, d] -> dtokens [B, N, d] with zeros at dropped variates."""
    B, _, d = dxs.shape
    out = torch.empty((B, N, d), dtype=dxs.dtype, device=dxs.device)
    rc = ctx._lib.vardrop_scatter(ctx.handle, _p(dxs), B, N, d, _dtype_code(dxs), _p(sel), n_sel, _p(out),
                                  _stream(dxs, stream))
    ctx.check(rc, "vardrop_scatter")
    return out


def vardrop_attn_fwd(ctx, xs, Wq, Wk, Wv, Wo, H, bq=None, bk=None, bv=None, bo=None, saved=None, out=None, stream=None):
    """xs [B, n, d] -> (y [B, n, d], saved uint8 buffer for the backward); y is written into `out` when given."""
    B, n, d = xs.shape
    code = _dtype_code(xs)
    nbytes = ctx._lib.vardrop_attn_saved_bytes(B, n, d, H, code)
    if saved is None or saved.numel() < nbytes:
        saved = torch.empty((max(nbytes, 256),), dtype=torch.uint8, device=xs.device)
    y = torch.empty_like(xs) if out is None else out
    rc = ctx._lib.vardrop_attn_fwd(ctx.handle, _p(xs), B, n, d, H, code, _p(Wq), _p(Wk), _p(Wv), _p(Wo),
                                   _p(bq), _p(bk), _p(bv), _p(bo), _p(y), _p(saved), None, 0, _stream(xs, stream))
    ctx.check(rc, "vardrop_attn_fwd")
    return y, saved


def vardrop_gather_attn_fwd(ctx, tokens, sel, n_sel, Wq, Wk, Wv, Wo, H, bq=None, bk=None, bv=None, bo=None,
                            saved=None, out=None, stream=None):
    """tokens [B, N, d], sel int32 (first n_sel entries: the kept rows) -> (xs [B, n_sel, d], y [B, n_sel, d], saved):
    the gather and the attention forward in one call.  `out`, when given, is the pair (xs, y) to write into."""
    B, N, d = tokens.shape
    code = _dtype_code(tokens)
    nbytes = ctx._lib.vardrop_attn_saved_bytes(B, n_sel, d, H, code)
    if saved is None or saved.numel() < nbytes:
        saved = torch.empty((max(nbytes, 256),), dtype=torch.uint8, device=tokens.device)
    if out is not None:
        xs, y = out
    else:
        xs = torch.empty((B, n_sel, d), dtype=tokens.dtype, device=tokens.device)
        y = torch.empty_like(xs)
    rc = ctx._lib.vardrop_gather_attn_fwd(ctx.handle, _p(tokens), B, N, _p(sel), n_sel, d, H, code,
                                          _p(Wq), _p(Wk), _p(Wv), _p(Wo), _p(bq), _p(bk), _p(bv), _p(bo),
                                          _p(xs), _p(y), _p(saved), None, 0, _stream(tokens, stream))
    ctx.check(rc, "vardrop_gather_attn_fwd")
    return xs, y, saved


def vardrop_attn_bwd(ctx, dy, xs, Wq, Wk, Wv, Wo, H, saved, bias_grads=False, ws=None, out=None, stream=None):
    """-> (dxs, dWq, dWk, dWv, dWo) or, with bias_grads, (..., dbq, dbk, dbv, dbo); weight grads are float32.
    `out`, when given, is that tuple of preallocated tensors."""
    B, n, d = xs.shape
    code = _dtype_code(xs)
    nbytes = ctx._lib.vardrop_attn_workspace_bytes(B, n, d, H, code)
    _own_buffers(stream, "vardrop_attn_bwd", ws=ws, out=out)
    if ws is None or ws.numel() < nbytes:
        ws = torch.empty((max(nbytes, 256),), dtype=torch.uint8, device=xs.device)
    if out is not None:
        dxs, dW = out[0], list(out[1:5])
        db = list(out[5:9]) if bias_grads else [None] * 4
    else:
        dxs = torch.empty_like(xs)
        dW = [torch.empty((d, d), dtype=torch.float32, device=xs.device) for _ in range(4)]
        db = [torch.empty((d,), dtype=torch.float32, device=xs.device) if bias_grads else None for _ in range(4)]
    rc = ctx._lib.vardrop_attn_bwd(ctx.handle, _p(dy), _p(xs), B, n, d, H, code, _p(Wq), _p(Wk), _p(Wv), _p(Wo),
                                   _p(saved), _p(dxs), *[_p(t) for t in dW], *[_p(t) for t in db],
                                   _p(ws), ws.numel(), _stream(xs, stream))
    ctx.check(rc, "vardrop_attn_bwd")
    return (dxs, *dW, *db) if bias_grads else (dxs, *dW)


def vardrop_embed_fwd(ctx, x, sel, n_sel, We, be=None, standardise=True, saved=None, out=None, stream=None):
    """x float32 [B, N, L] (time contiguous), sel int32, We [L, d] -> (xs [B, n_sel, d] in We's dtype, saved)."""
    if x.dtype != torch.float32 or x.dim() != 3 or x.stride(2) != 1:
        raise TypeError("x must be float32 [B, N, L] with contiguous time")
    B, N, L = x.shape
    d = We.shape[1]
    dt = _dtype_code(We)
    if saved is None:
        saved = torch.empty(ctx._lib.vardrop_embed_saved_bytes(B, n_sel, L, dt), dtype=torch.uint8, device=x.device)
    xs = out if out is not None else torch.empty((B, n_sel, d), dtype=We.dtype, device=x.device)
    rc = ctx._lib.vardrop_embed_fwd(ctx.handle, _p(x), B, N, L, x.stride(0), x.stride(1), _p(sel), n_sel,
                                    1 if standardise else 0, _p(We), _p(be), d, dt, _p(xs), _p(saved),
                                    _stream(x, stream))
    ctx.check(rc, "vardrop_embed_fwd")
    return xs, saved


def vardrop_embed_bwd(ctx, dxs, L, saved, want_bias=True, ws=None, out=None, stream=None):
    """dxs [B, n_sel, d], saved from vardrop_embed_fwd -> (dWe float32 [L, d], dbe float32 [d] or None).
    `out`, when given, is that pair of preallocated tensors."""
    B, n_sel, d = dxs.shape
    dt = _dtype_code(dxs)
    _own_buffers(stream, "vardrop_embed_bwd", ws=ws, out=out)
    if ws is None:
        ws = torch.empty(max(ctx._lib.vardrop_embed_workspace_bytes(B, n_sel, L, d, dt), 256), dtype=torch.uint8,
                         device=dxs.device)
    if out is not None:
        dWe, dbe = out
    else:
        dWe = torch.empty((L, d), dtype=torch.float32, device=dxs.device)
        dbe = torch.empty((d,), dtype=torch.float32, device=dxs.device) if want_bias else None
    rc = ctx._lib.vardrop_embed_bwd(ctx.handle, _p(dxs), B, n_sel, L, d, dt, _p(saved), _p(dWe), _p(dbe),
                                    _p(ws), ws.numel(), _stream(dxs, stream))
    ctx.check(rc, "vardrop_embed_bwd")
    return dWe, dbe


def vardrop_sample_nearest(ctx, hsh, abar, gs, ratio_num, ratio_den, stream=None):
    """hash int64 [N], abar float32 [N, F] -> (group_id int32 [N], sel int32 [N] (first N' valid), counts int32 [2]):
    every group keeps the members closest to its mean spectrum."""
    N, F = abar.shape
    dev = hsh.device
    if stream is not None:
        raise TypeError("vardrop_sample_nearest allocates its workspace: call it on torch's current stream")
    gid = torch.empty((N,), dtype=torch.int32, device=dev)
    sel = torch.empty((N,), dtype=torch.int32, device=dev)
    counts = torch.empty((2,), dtype=torch.int32, device=dev)
    ws = torch.empty(max(ctx._lib.vardrop_sample_nearest_workspace_bytes(N, F), 256), dtype=torch.uint8, device=dev)
    rc = ctx._lib.vardrop_sample_nearest(ctx.handle, _p(hsh), _p(abar), N, F, gs, ratio_num, ratio_den,
                                         _p(gid), _p(sel), _p(counts), None, _p(ws), ws.numel(), _stream(hsh, stream))
    ctx.check(rc, "vardrop_sample_nearest")
    return gid, sel, counts



# ---------------------------------------------------------------- device-side token count
def vardrop_sample_dev(ctx, hsh, gs, ratio_num, ratio_den, seed, step_dev, advance, out, stream=None):
    """vardrop_sample with the step counter in device memory (step_dev: int64 [1]); out = (group_id, sel, counts)."""
    N = hsh.shape[0]
    gid, sel, counts = out
    rc = ctx._lib.vardrop_sample_dev(ctx.handle, _p(hsh), N, gs, ratio_num, ratio_den, seed, _p(step_dev), 1 if advance else 0,
                                     _p(gid), _p(sel), _p(counts), None, 0, _stream(hsh, stream))
    ctx.check(rc, "vardrop_sample_dev")
    return gid, sel, counts


def vardrop_gather_dev(ctx, tokens, sel, n_dev, n_max, out, status=None, stream=None):
    """tokens [B, N, d], sel int32, n_dev int32 [1] on the device -> out (>= B * n_max * d elements), packed [B, N', d]."""
    B, N, d = tokens.shape
    rc = ctx._lib.vardrop_gather_dev(ctx.handle, _p(tokens), B, N, d, _dtype_code(tokens), _p(sel), _p(n_dev), n_max,
                                     _p(status), _p(out), _stream(tokens, stream))
    ctx.check(rc, "vardrop_gather_dev")
    return out


def vardrop_scatter_dev(ctx, dxs, sel, n_dev, n_max, out, status=None, stream=None):
    """dxs packed [B, N', d] -> out [B, N, d] with zeros at dropped variates; N' read from n_dev on the device."""
    B, N, d = out.shape
    rc = ctx._lib.vardrop_scatter_dev(ctx.handle, _p(dxs), B, N, d, _dtype_code(out), _p(sel), _p(n_dev), n_max,
                                      _p(status), _p(out), _stream(out, stream))
    ctx.check(rc, "vardrop_scatter_dev")
    return out


def vardrop_gather_attn_fwd_dev(ctx, tokens, sel, n_dev, n_max, Wq, Wk, Wv, Wo, H, xs, y, saved,
                                bq=None, bk=None, bv=None, bo=None, status=None, stream=None):
    """Gather + attention forward with N' read on the device from n_dev (int32 [1]); xs, y hold >= B * n_max * d
    elements and receive [B, N', d] packed; saved holds vardrop_attn_saved_bytes(B, n_max, d, H) bytes."""
    B, N, d = tokens.shape
    rc = ctx._lib.vardrop_gather_attn_fwd_dev(ctx.handle, _p(tokens), B, N, _p(sel), _p(n_dev), n_max, _p(status), d, H,
                                              _dtype_code(tokens), _p(Wq), _p(Wk), _p(Wv), _p(Wo),
                                              _p(bq), _p(bk), _p(bv), _p(bo), _p(xs), _p(y), _p(saved), None, 0,
                                              _stream(tokens, stream))
    ctx.check(rc, "vardrop_gather_attn_fwd_dev")
    return xs, y, saved


def vardrop_attn_bwd_dev(ctx, dy, xs, n_dev, n_max, Wq, Wk, Wv, Wo, H, saved, ws, out, status=None, stream=None):
    """Attention backward with N' read on the device; out = (dxs, dWq, dWk, dWv, dWo[, dbq, dbk, dbv, dbo]);
    B is taken from the weights' caller: dy, xs, dxs are flat or [B, n_max, d] buffers, so B = out[0].shape[0]."""
    B = out[0].shape[0]
    d = Wq.shape[0]
    dxs, dW = out[0], list(out[1:5])
    db = list(out[5:9]) if len(out) >= 9 else [None] * 4
    rc = ctx._lib.vardrop_attn_bwd_dev(ctx.handle, _p(dy), _p(xs), B, _p(n_dev), n_max, _p(status), d, H, _dtype_code(Wq),
                                       _p(Wq), _p(Wk), _p(Wv), _p(Wo), _p(saved), _p(dxs), *[_p(t) for t in dW],
                                       *[_p(t) for t in db], _p(ws), ws.numel(), _stream(Wq, stream))
    ctx.check(rc, "vardrop_attn_bwd_dev")
    return out


def vardrop_sample_nearest_noalloc(ctx, hsh, abar, gs, ratio_num, ratio_den, out, stream=None):
    """vardrop_sample_nearest on the library's static scratch (allocates nothing); out = (group_id, sel, counts)."""
    N, F = abar.shape
    gid, sel, counts = out
    rc = ctx._lib.vardrop_sample_nearest_noalloc(ctx.handle, _p(hsh), _p(abar), N, F, gs, ratio_num, ratio_den,
                                                 _p(gid), _p(sel), _p(counts), _stream(hsh, stream))
    ctx.check(rc, "vardrop_sample_nearest_noalloc")
    return gid, sel, counts


def vardrop_attn_fwd_dev(ctx, xs, n_dev, n_max, Wq, Wk, Wv, Wo, H, y, saved, bq=None, bk=None, bv=None, bo=None,
                         status=None, stream=None):
    """Attention forward on packed tokens xs ([B, n_max, d] buffer holding [B, N', d]) with N' read on the device."""
    B, d = xs.shape[0], Wq.shape[0]
    rc = ctx._lib.vardrop_attn_fwd_dev(ctx.handle, _p(xs), B, _p(n_dev), n_max, _p(status), d, H, _dtype_code(Wq),
                                       _p(Wq), _p(Wk), _p(Wv), _p(Wo), _p(bq), _p(bk), _p(bv), _p(bo),
                                       _p(y), _p(saved), None, 0, _stream(xs, stream))
    ctx.check(rc, "vardrop_attn_fwd_dev")
    return y, saved


def vardrop_embed_fwd_dev(ctx, x, sel, n_dev, n_max, We, be, xs, saved, standardise=True, status=None, stream=None):
    """Embedding of the kept windows with their count read on the device; xs: [B, n_max, d] buffer, packed [B, N', d]."""
    B, N, L = x.shape
    rc = ctx._lib.vardrop_embed_fwd_dev(ctx.handle, _p(x), B, N, L, x.stride(0), x.stride(1), _p(sel), _p(n_dev), n_max,
                                        _p(status), 1 if standardise else 0, _p(We), _p(be), We.shape[1], _dtype_code(We),
                                        _p(xs), _p(saved), _stream(x, stream))
    ctx.check(rc, "vardrop_embed_fwd_dev")
    return xs, saved


def vardrop_embed_bwd_dev(ctx, dxs, n_dev, n_max, L, saved, ws, out, stream=None):
    """Weight gradients of the embedding with the count read on the device; out = (dWe, dbe or None)."""
    B, d = dxs.shape[0], dxs.shape[-1]
    dWe, dbe = out
    rc = ctx._lib.vardrop_embed_bwd_dev(ctx.handle, _p(dxs), B, _p(n_dev), n_max, L, d, _dtype_code(dxs), _p(saved),
                                        _p(dWe), _p(dbe), _p(ws), ws.numel(), _stream(dxs, stream))
    ctx.check(rc, "vardrop_embed_bwd_dev")
    return dWe, dbe
