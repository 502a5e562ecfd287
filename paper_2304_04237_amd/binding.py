"""ctypes binding of libslide_attn.so: argument marshalling only.

Function names match the C ABI (include/slide_attn.h).  Tensors must be
contiguous CUDA(HIP) tensors; activations float32 or bfloat16 [B, C, H, W],
kernels / bias float32.  Work is enqueued on torch's current stream.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libslide_attn.so")
_lib = None

SLIDE_F32, SLIDE_BF16 = 0, 1
_vp = ctypes.c_void_p


class SlideAttnError(RuntimeError):
    pass


def lib_path():
    return _LIB_PATH


def load_library():
    """Load the built HIP library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise SlideAttnError(
            "libslide_attn.so is not built: run `python -m paper_2304_04237_amd.build` "
            "(there is no CPU or PyTorch fallback)")
    lib = ctypes.CDLL(_LIB_PATH)
    i, sz = ctypes.c_int, ctypes.c_size_t
    lib.slide_status_string.restype = ctypes.c_char_p
    lib.slide_status_string.argtypes = [i]
    lib.slide_reparam.restype = i
    lib.slide_reparam.argtypes = [_vp, _vp, i, i, _vp]
    lib.slide_attn_workspace_bytes.restype = sz
    lib.slide_attn_workspace_bytes.argtypes = [i] * 8
    lib.slide_attn_fwd_path.restype = i
    lib.slide_attn_fwd_path.argtypes = [i] * 7
    lib.slide_attn_fwd_variant.restype = i
    lib.slide_attn_fwd_variant.argtypes = [i] * 8
    lib.slide_attn_bwd_variant.restype = i
    lib.slide_attn_bwd_variant.argtypes = [i] * 8
    lib.slide_attn_fwd.restype = i
    lib.slide_attn_fwd.argtypes = [_vp] * 8 + [i] * 7 + [_vp, sz, _vp]
    lib.slide_attn_fwd_noalloc.restype = i
    lib.slide_attn_fwd_noalloc.argtypes = [_vp] * 8 + [i] * 7 + [_vp]
    lib.slide_attn_fwd_shift.restype = i
    lib.slide_attn_fwd_shift.argtypes = [_vp] * 6 + [i] * 7 + [_vp]
    lib.slide_attn_fwd_nhwc.restype = i
    lib.slide_attn_fwd_nhwc.argtypes = [_vp] * 8 + [i] * 7 + [_vp]
    lib.slide_attn_bwd_nhwc_workspace_bytes.restype = sz
    lib.slide_attn_bwd_nhwc_workspace_bytes.argtypes = [i] * 7
    lib.slide_attn_bwd_nhwc.restype = i
    lib.slide_attn_bwd_nhwc.argtypes = [_vp] * 13 + [i] * 9 + [_vp, sz, _vp]
    lib.slide_attn_fwd_traffic_probe.restype = i
    lib.slide_attn_fwd_traffic_probe.argtypes = [_vp] * 4 + [i] * 6 + [_vp]
    lib.slide_attn_bwd.restype = i
    lib.slide_attn_bwd.argtypes = [_vp] * 15 + [i] * 7 + [_vp, sz, _vp]
    lib.slide_attn_fwd_two_branch.restype = i
    lib.slide_attn_fwd_two_branch.argtypes = [_vp] * 8 + [i] * 7 + [_vp, sz, _vp]
    lib.slide_attn_bwd_two_branch.restype = i
    lib.slide_attn_bwd_two_branch.argtypes = [_vp] * 15 + [i] * 8 + [_vp, sz, _vp]
    _lib = lib
    return lib


def slide_status_string(status):
    return load_library().slide_status_string(int(status)).decode()


def _check(status):
    if status != 0:
        raise SlideAttnError(slide_status_string(status))


def _dtype_code(t):
    if t.dtype == torch.float32:
        return SLIDE_F32
    if t.dtype == torch.bfloat16:
        return SLIDE_BF16
    raise SlideAttnError("activations must be float32 or bfloat16, got %s" % t.dtype)


def _dev(t, name, dtype=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise SlideAttnError("%s must live on the GPU" % name)
    if not t.is_contiguous():
        raise SlideAttnError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise SlideAttnError("%s must be %s" % (name, dtype))
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def slide_attn_workspace_bytes(B, H, W, C, heads, ksize, dtype, backward):
    code = dtype if isinstance(dtype, int) else (SLIDE_F32 if dtype == torch.float32 else SLIDE_BF16)
    return int(load_library().slide_attn_workspace_bytes(B, H, W, C, heads, ksize, code, int(bool(backward))))


def slide_attn_fwd_path(B, H, W, C, heads, ksize, dtype):
    code = dtype if isinstance(dtype, int) else (SLIDE_F32 if dtype == torch.float32 else SLIDE_BF16)
    return int(load_library().slide_attn_fwd_path(B, H, W, C, heads, ksize, code))


def slide_attn_fwd_variant(B, H, W, C, heads, ksize, dtype, aligned16=True):
    code = dtype if isinstance(dtype, int) else (SLIDE_F32 if dtype == torch.float32 else SLIDE_BF16)
    return int(load_library().slide_attn_fwd_variant(B, H, W, C, heads, ksize, code, int(bool(aligned16))))


def slide_attn_bwd_variant(B, H, W, C, heads, ksize, dtype, aligned16=True):
    code = dtype if isinstance(dtype, int) else (SLIDE_F32 if dtype == torch.float32 else SLIDE_BF16)
    return int(load_library().slide_attn_bwd_variant(B, H, W, C, heads, ksize, code, int(bool(aligned16))))


def _check_params(q, wk, wv, bias, heads, ksize):
    """Shapes of the kernels and the bias against the activations (a mismatch must not
    reach a kernel as an out-of-bounds access)."""
    if q.dim() != 4:
        raise SlideAttnError("activations must be [B, C, H, W]")
    C = q.shape[1]
    S = ksize * ksize
    for t, n in ((wk, "wk"), (wv, "wv")):
        if tuple(t.shape) != (C, S, ksize, ksize):
            raise SlideAttnError("%s must be [C, k*k, k, k] = %s, got %s" % (n, (C, S, ksize, ksize), tuple(t.shape)))
    if bias is not None and tuple(bias.shape) != (heads, S):
        raise SlideAttnError("bias must be [heads, k*k] = %s, got %s" % ((heads, S), tuple(bias.shape)))


def slide_reparam(w_learned, w_merged=None):
    """w_merged = one-hot shift kernels + w_learned, float32 [C, k*k, k, k]."""
    lib = load_library()
    C, S, kh, kw = w_learned.shape
    if kh != kw or S != kh * kw:
        raise SlideAttnError("kernel must be [C, k*k, k, k]")
    if w_merged is None:
        w_merged = torch.empty_like(w_learned)
    elif w_merged.shape != w_learned.shape:
        raise SlideAttnError("w_merged must have the shape of w_learned")
    _check(lib.slide_reparam(_dev(w_learned, "w_learned", torch.float32),
                             _dev(w_merged, "w_merged", torch.float32), C, kh, _stream()))
    return w_merged


def slide_attn_fwd(q, k, v, wk, wv, bias, heads, ksize, out=None, workspace=None, lse=None):
    """out = slide attention of (q, k, v) with MERGED kernels wk, wv and per-head bias.

    lse: optional float32 [B, heads, H, W] tensor that receives the log of the softmax
    denominator per pixel and head."""
    return _fwd(load_library().slide_attn_fwd, q, k, v, wk, wv, bias, heads, ksize, out, workspace, lse)


def slide_attn_fwd_noalloc(q, k, v, wk, wv, bias, heads, ksize, out, lse=None):
    """slide_attn_fwd through the entry point that allocates nothing: `out` must be given,
    the kernels' scratch is the library's own fixed array."""
    lib = load_library()
    _check_params(q, wk, wv, bias, heads, ksize)
    B, C, H, W = q.shape
    code = _dtype_code(q)
    for t, n in ((k, "k"), (v, "v"), (out, "out")):
        if t.shape != q.shape or t.dtype != q.dtype:
            raise SlideAttnError("%s must match q in shape and dtype" % n)
    if lse is not None and tuple(lse.shape) != (B, heads, H, W):
        raise SlideAttnError("lse must be [B, heads, H, W]")
    _check(lib.slide_attn_fwd_noalloc(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"),
                                      _dev(wk, "wk", torch.float32), _dev(wv, "wv", torch.float32),
                                      _dev(bias, "bias", torch.float32), _dev(out, "out", q.dtype),
                                      _dev(lse, "lse", torch.float32),
                                      B, H, W, C, heads, ksize, code, _stream()))
    return out


def slide_attn_fwd_shift(q, k, v, bias, heads, ksize, out=None, lse=None):
    """Plain-shift forward: local attention over the window with no learned kernels."""
    if q.dim() != 4:
        raise SlideAttnError("activations must be [B, C, H, W]")
    B, C, H, W = q.shape
    code = _dtype_code(q)
    for t, n in ((k, "k"), (v, "v")):
        if t.shape != q.shape or t.dtype != q.dtype:
            raise SlideAttnError("%s must match q in shape and dtype" % n)
    if bias is not None and tuple(bias.shape) != (heads, ksize * ksize):
        raise SlideAttnError("bias must be [heads, k*k] = %s, got %s" % ((heads, ksize * ksize), tuple(bias.shape)))
    if out is None:
        out = torch.empty_like(q)
    elif out.shape != q.shape or out.dtype != q.dtype:
        raise SlideAttnError("out must match q in shape and dtype")
    if lse is not None and tuple(lse.shape) != (B, heads, H, W):
        raise SlideAttnError("lse must be [B, heads, H, W]")
    _check(load_library().slide_attn_fwd_shift(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"),
                                               _dev(bias, "bias", torch.float32), _dev(out, "out"),
                                               _dev(lse, "lse", torch.float32),
                                               B, H, W, C, heads, ksize, code, _stream()))
    return out


def slide_attn_fwd_nhwc(q, k, v, wk, wv, bias, heads, ksize, out=None, lse=None):
    """Forward for channels-last activations [B, H, W, C]; lse, if given, is [B, heads, H, W]."""
    if q.dim() != 4:
        raise SlideAttnError("activations must be [B, H, W, C]")
    B, H, W, C = q.shape
    S = ksize * ksize
    for t, n in ((wk, "wk"), (wv, "wv")):
        if tuple(t.shape) != (C, S, ksize, ksize):
            raise SlideAttnError("%s must be [C, k*k, k, k] = %s, got %s" % (n, (C, S, ksize, ksize), tuple(t.shape)))
    if bias is not None and tuple(bias.shape) != (heads, S):
        raise SlideAttnError("bias must be [heads, k*k] = %s, got %s" % ((heads, S), tuple(bias.shape)))
    code = _dtype_code(q)
    for t, n in ((k, "k"), (v, "v")):
        if t.shape != q.shape or t.dtype != q.dtype:
            raise SlideAttnError("%s must match q in shape and dtype" % n)
    if out is None:
        out = torch.empty_like(q)
    elif out.shape != q.shape or out.dtype != q.dtype:
        raise SlideAttnError("out must match q in shape and dtype")
    if lse is not None and tuple(lse.shape) != (B, heads, H, W):
        raise SlideAttnError("lse must be [B, heads, H, W]")
    _check(load_library().slide_attn_fwd_nhwc(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"),
                                              _dev(wk, "wk", torch.float32), _dev(wv, "wv", torch.float32),
                                              _dev(bias, "bias", torch.float32), _dev(out, "out"),
                                              _dev(lse, "lse", torch.float32),
                                              B, H, W, C, heads, ksize, code, _stream()))
    return out


def slide_attn_bwd_nhwc(dout, q, k, v, wk, wv, bias, heads, ksize, workspace=None, outputs=None,
                        two_branch=False, accumulate=False):
    """Backward for channels-last activations [B, H, W, C]: returns (dq, dk, dv, dwk, dwv, dbias),
    the first three [B, H, W, C].  two_branch: wk, wv are the learned kernels; accumulate: the
    parameter gradients are added to what `outputs` holds."""
    lib = load_library()
    if q.dim() != 4:
        raise SlideAttnError("activations must be [B, H, W, C]")
    B, H, W, C = q.shape
    S = ksize * ksize
    for t, n in ((wk, "wk"), (wv, "wv")):
        if tuple(t.shape) != (C, S, ksize, ksize):
            raise SlideAttnError("%s must be [C, k*k, k, k] = %s, got %s" % (n, (C, S, ksize, ksize), tuple(t.shape)))
    if bias is not None and tuple(bias.shape) != (heads, S):
        raise SlideAttnError("bias must be [heads, k*k] = %s, got %s" % ((heads, S), tuple(bias.shape)))
    code = _dtype_code(q)
    for t, n in ((k, "k"), (v, "v"), (dout, "dout")):
        if t.shape != q.shape or t.dtype != q.dtype:
            raise SlideAttnError("%s must match q in shape and dtype" % n)
    if outputs is None:
        dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
        dwk, dwv = torch.empty_like(wk), torch.empty_like(wv)
        dbias = torch.empty_like(bias) if bias is not None else None
    else:
        dq, dk, dv, dwk, dwv, dbias = outputs
        for t, n in ((dq, "dq"), (dk, "dk"), (dv, "dv")):
            if t.shape != q.shape or t.dtype != q.dtype:
                raise SlideAttnError("%s must match q in shape and dtype" % n)
        for t, n, like in ((dwk, "dwk", wk), (dwv, "dwv", wv), (dbias, "dbias", bias)):
            if (t is None) != (like is None) or (t is not None and t.shape != like.shape):
                raise SlideAttnError("%s must have the shape of the parameter it is the gradient of" % n)
    need = lib.slide_attn_bwd_nhwc_workspace_bytes(B, H, W, C, heads, ksize, code)
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=q.device)
    elif not workspace.is_cuda:
        raise SlideAttnError("workspace must live on the GPU")
    _check(lib.slide_attn_bwd_nhwc(_dev(dout, "dout"), _dev(q, "q"), _dev(k, "k"), _dev(v, "v"),
                                   _dev(wk, "wk", torch.float32), _dev(wv, "wv", torch.float32),
                                   _dev(bias, "bias", torch.float32),
                                   _dev(dq, "dq", q.dtype), _dev(dk, "dk", q.dtype), _dev(dv, "dv", q.dtype),
                                   _dev(dwk, "dwk", torch.float32), _dev(dwv, "dwv", torch.float32),
                                   _dev(dbias, "dbias", torch.float32),
                                   int(bool(two_branch)), int(bool(accumulate)),
                                   B, H, W, C, heads, ksize, code,
                                   workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream()))
    return dq, dk, dv, dwk, dwv, dbias


def slide_attn_fwd_traffic_probe(q, k, v, out, heads, mode):
    """The forward's bytes without its arithmetic (mode 0: flat copy, 1: the streaming kernel's pattern)."""
    B, C, H, W = q.shape
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (out, "out")):
        if t.shape != q.shape or t.dtype != torch.bfloat16:
            raise SlideAttnError("%s must be bfloat16 [B, C, H, W]" % n)
    _check(load_library().slide_attn_fwd_traffic_probe(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(out, "out"),
                                                       B, H, W, C, heads, int(mode), _stream()))
    return out


def slide_attn_fwd_two_branch(q, k, v, wk_learned, wv_learned, bias, heads, ksize, out=None,
                              workspace=None, lse=None):
    """The same with the LEARNED kernels of the training form (shift path added inside)."""
    return _fwd(load_library().slide_attn_fwd_two_branch, q, k, v, wk_learned, wv_learned, bias, heads,
                ksize, out, workspace, lse)


def _fwd(entry, q, k, v, wk, wv, bias, heads, ksize, out, workspace, lse):
    lib = load_library()
    _check_params(q, wk, wv, bias, heads, ksize)
    B, C, H, W = q.shape
    code = _dtype_code(q)
    for t, n in ((k, "k"), (v, "v")):
        if t.shape != q.shape or t.dtype != q.dtype:
            raise SlideAttnError("%s must match q in shape and dtype" % n)
    if out is None:
        out = torch.empty_like(q)
    elif out.shape != q.shape or out.dtype != q.dtype:
        raise SlideAttnError("out must match q in shape and dtype")
    if lse is not None and tuple(lse.shape) != (B, heads, H, W):
        raise SlideAttnError("lse must be [B, heads, H, W]")
    need = lib.slide_attn_workspace_bytes(B, H, W, C, heads, ksize, code, 0)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    if workspace is not None and not workspace.is_cuda:
        raise SlideAttnError("workspace must live on the GPU")
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(entry(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"),
                 _dev(wk, "wk", torch.float32), _dev(wv, "wv", torch.float32),
                 _dev(bias, "bias", torch.float32), _dev(out, "out", q.dtype),
                 _dev(lse, "lse", torch.float32),
                 B, H, W, C, heads, ksize, code, ws_ptr, ws_bytes, _stream()))
    return out


def slide_attn_bwd(dout, q, k, v, wk, wv, bias, heads, ksize, workspace=None, outputs=None,
                   out=None, lse=None):
    """Returns (dq, dk, dv, dwk, dwv, dbias); dbias is None when bias is None.

    out, lse: the forward's results, if the caller kept them (optional; passed through)."""
    return _bwd(False, False, dout, q, k, v, wk, wv, bias, heads, ksize, workspace, outputs, out, lse)


def slide_attn_bwd_two_branch(dout, q, k, v, wk_learned, wv_learned, bias, heads, ksize, workspace=None,
                              outputs=None, out=None, lse=None, accumulate=False):
    """Backward of the training form.  accumulate: add dwk, dwv, dbias to what `outputs` holds."""
    if accumulate and outputs is None:
        raise SlideAttnError("accumulate needs the gradient tensors in `outputs`")
    return _bwd(True, accumulate, dout, q, k, v, wk_learned, wv_learned, bias, heads, ksize, workspace,
                outputs, out, lse)


def _bwd(two_branch, accumulate, dout, q, k, v, wk, wv, bias, heads, ksize, workspace, outputs, out, lse):
    lib = load_library()
    _check_params(q, wk, wv, bias, heads, ksize)
    B, C, H, W = q.shape
    code = _dtype_code(q)
    for t, n in ((k, "k"), (v, "v"), (dout, "dout")):
        if t.shape != q.shape or t.dtype != q.dtype:
            raise SlideAttnError("%s must match q in shape and dtype" % n)
    if outputs is None:
        dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
        dwk, dwv = torch.empty_like(wk), torch.empty_like(wv)
        dbias = torch.empty_like(bias) if bias is not None else None
    else:
        dq, dk, dv, dwk, dwv, dbias = outputs
        for t, n in ((dq, "dq"), (dk, "dk"), (dv, "dv")):
            if t.shape != q.shape or t.dtype != q.dtype:
                raise SlideAttnError("%s must match q in shape and dtype" % n)
        for t, n, like in ((dwk, "dwk", wk), (dwv, "dwv", wv), (dbias, "dbias", bias)):
            if (t is None) != (like is None) or (t is not None and t.shape != like.shape):
                raise SlideAttnError("%s must have the shape of the parameter it is the gradient of" % n)
    for t, n in ((out, "out"), ):
        if t is not None and (t.shape != q.shape or t.dtype != q.dtype):
            raise SlideAttnError("%s must match q in shape and dtype" % n)
    if lse is not None and tuple(lse.shape) != (B, heads, H, W):
        raise SlideAttnError("lse must be [B, heads, H, W]")
    need = lib.slide_attn_workspace_bytes(B, H, W, C, heads, ksize, code, 1)
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=q.device)
    elif not workspace.is_cuda:
        raise SlideAttnError("workspace must live on the GPU")
    ptrs = (_dev(dout, "dout"), _dev(q, "q"), _dev(k, "k"), _dev(v, "v"),
            _dev(wk, "wk", torch.float32), _dev(wv, "wv", torch.float32),
            _dev(bias, "bias", torch.float32),
            _dev(out, "out", q.dtype), _dev(lse, "lse", torch.float32),
            _dev(dq, "dq", q.dtype), _dev(dk, "dk", q.dtype), _dev(dv, "dv", q.dtype),
            _dev(dwk, "dwk", torch.float32), _dev(dwv, "dwv", torch.float32),
            _dev(dbias, "dbias", torch.float32))
    tail = (B, H, W, C, heads, ksize, code,
            workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream())
    if two_branch:
        _check(lib.slide_attn_bwd_two_branch(*ptrs, int(bool(accumulate)), *tail))
    else:
        _check(lib.slide_attn_bwd(*ptrs, *tail))
    return dq, dk, dv, dwk, dwv, dbias
