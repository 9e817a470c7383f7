"""Python binding of the HIPPO hot-path library for MI355X (``libhippo.so``, C ABI in include/hippo.h).

Argument marshalling only: every step runs in the HIP kernels.  torch supplies device memory and
the current stream; nothing here computes.  If the shared library is missing the calls raise -- there
is no fallback path.
"""
from __future__ import annotations

import contextlib
import ctypes as C
import os
from typing import Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhippo.so")

DTYPE_F32, DTYPE_BF16, DTYPE_FP8_E4M3 = 0, 1, 2
CALL_SCORE_TOKENS, CALL_SELECT_GATHER_KV, CALL_DRAFT_ATTENTION, CALL_VERIFY_ATTENTION = 0, 1, 2, 3
SCORE_ATTN, SCORE_TEMP, SCORE_SPA, SCORE_ALL, SCORE_ACCUMULATE_ONLY = 1, 2, 4, 7, 8
(OK, ERR_NULL_ARG, ERR_BAD_SHAPE, ERR_BAD_DTYPE, ERR_BAD_ALIGN, ERR_WORKSPACE_TOO_SMALL, ERR_HIP,
 ERR_STATIC_SCRATCH_LIMIT) = range(8)

EXPORTS = ("hippo_status_string", "hippo_workspace_bytes", "hippo_score_tokens",
           "hippo_score_layers_workspace_bytes", "hippo_score_tokens_layers",
           "hippo_select_gather_kv", "hippo_verify_attention", "hippo_draft_attention",
           "hippo_static_scratch_bytes", "hippo_static_scratch_init", "hippo_verify_attention_static",
           "hippo_verify_attention_append", "hippo_draft_attention_append",
           "hippo_verify_attention_paged", "hippo_draft_attention_paged",
           "hippo_verify_attention_fp8kv", "hippo_draft_attention_fp8kv",
           "hippo_quantize_kv_workspace_bytes", "hippo_quantize_kv_e4m3",
           "hippo_spec_verify_workspace_bytes", "hippo_spec_verify", "hippo_vpsd_prefill_buffer",
           "hippo_vpsd_init", "hippo_vpsd_plan", "hippo_vpsd_commit", "hippo_vpsd_simulate")
VPSD_CONSERVATIVE, VPSD_OPTIMISTIC = 0, 1
POLICY_AUTOREGRESSIVE, POLICY_SERIAL_SD, POLICY_VPSD = 0, 1, 2


class VpsdState(C.Structure):
    _fields_ = [("gamma", C.c_int32), ("mode", C.c_int32), ("n_pending", C.c_int32), ("reserved", C.c_int32),
                ("n_emitted", C.c_int64), ("n_rounds", C.c_int64), ("n_target_calls", C.c_int64),
                ("n_draft_tokens", C.c_int64), ("n_draft_wasted", C.c_int64), ("n_mode_switches", C.c_int64)]


class VpsdRound(C.Structure):
    _fields_ = [("mode", C.c_int32), ("draft_serial", C.c_int32), ("verify_len", C.c_int32),
                ("draft_parallel", C.c_int32)]


class VpsdResult(C.Structure):
    _fields_ = [("time", C.c_double), ("speedup", C.c_double), ("n_emitted", C.c_int64), ("n_rounds", C.c_int64),
                ("n_target_calls", C.c_int64), ("n_draft_tokens", C.c_int64), ("n_draft_wasted", C.c_int64),
                ("n_mode_switches", C.c_int64), ("n_flags_used", C.c_int64)]


class PagedKvDesc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("dtype", C.c_int32), ("page_size", C.c_int32),
                ("max_pages", C.c_int32), ("n_pool_pages", C.c_int32),
                ("stride_page", C.c_int64), ("stride_n", C.c_int64), ("stride_h", C.c_int64)]


class KvDesc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("dtype", C.c_int32),
                ("stride_b", C.c_int64), ("stride_h", C.c_int64), ("stride_n", C.c_int64)]


class VideoDesc(C.Structure):
    _fields_ = [("n_frames", C.c_int32), ("grid_h", C.c_int32), ("grid_w", C.c_int32),
                ("vis_offset", C.c_int32), ("crop_h", C.c_int32), ("crop_w", C.c_int32)]


class HippoError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__("%s failed: status %d (%s)" % (what, status, status_string(status)))
        self.status = status


_lib = None


def load():
    """dlopen libhippo.so and declare the signatures.  Raises if the library has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libhippo.so is not built: run `python -m paper_2601_08273_amd.build` "
                           "(there is no fallback implementation)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, u32, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_float, C.c_size_t
    kvp, vdp = C.POINTER(KvDesc), C.POINTER(VideoDesc)
    lib.hippo_status_string.argtypes = [C.c_int]
    lib.hippo_status_string.restype = C.c_char_p
    lib.hippo_workspace_bytes.argtypes = [i32, kvp, vdp, i32, i32, i32, i32]
    lib.hippo_workspace_bytes.restype = sz
    lib.hippo_score_tokens.argtypes = [vp, i32, vp, kvp, i32, vdp, vp, i32, i64, u32, vp, vp, vp, vp, sz, vp]
    lib.hippo_score_tokens.restype = C.c_int
    lib.hippo_score_layers_workspace_bytes.argtypes = [kvp, vdp, i32, i32]
    lib.hippo_score_layers_workspace_bytes.restype = C.c_size_t
    lib.hippo_score_tokens_layers.argtypes = [i32, vp, i32, vp, i32, kvp, i32, vdp, vp, i32, i64, u32, vp, vp, vp, vp,
                                              sz, vp]
    lib.hippo_score_tokens_layers.restype = C.c_int
    lib.hippo_select_gather_kv.argtypes = [vp, i32, vp, vp, kvp, i32, vdp, vp, vp, kvp, vp, vp, sz, vp]
    lib.hippo_select_gather_kv.restype = C.c_int
    for fn in (lib.hippo_verify_attention, lib.hippo_draft_attention):
        fn.argtypes = [vp, i32, vp, vp, kvp, i32, f32, i32, vp, vp, vp, sz, vp]
        fn.restype = C.c_int
    lib.hippo_static_scratch_bytes.argtypes = []
    lib.hippo_static_scratch_bytes.restype = sz
    lib.hippo_static_scratch_init.argtypes = []
    lib.hippo_static_scratch_init.restype = C.c_int
    lib.hippo_verify_attention_static.argtypes = [vp, i32, vp, vp, kvp, i32, f32, i32, vp, vp, vp]
    lib.hippo_verify_attention_static.restype = C.c_int
    for fn in (lib.hippo_verify_attention_paged, lib.hippo_draft_attention_paged):
        fn.argtypes = [vp, i32, vp, vp, vp, C.POINTER(PagedKvDesc), i32, f32, i32, vp, vp, vp, sz, vp]
        fn.restype = C.c_int
    for fn in (lib.hippo_verify_attention_append, lib.hippo_draft_attention_append,
               lib.hippo_verify_attention_fp8kv, lib.hippo_draft_attention_fp8kv):
        fn.argtypes = [vp, i32, vp, vp, vp, vp, kvp, i32, f32, i32, vp, vp, vp, sz, vp]
        fn.restype = C.c_int
    lib.hippo_quantize_kv_workspace_bytes.argtypes = [kvp, i32]
    lib.hippo_quantize_kv_workspace_bytes.restype = C.c_size_t
    lib.hippo_quantize_kv_e4m3.argtypes = [vp, vp, kvp, i32, vp, vp, kvp, vp, vp, vp, sz, vp]
    lib.hippo_quantize_kv_e4m3.restype = C.c_int
    f64 = C.c_double
    lib.hippo_vpsd_prefill_buffer.argtypes = [f64, f64, f64]
    lib.hippo_vpsd_prefill_buffer.restype = C.c_int32
    lib.hippo_vpsd_init.argtypes = [C.POINTER(VpsdState), i32, i32]
    lib.hippo_vpsd_plan.argtypes = [C.POINTER(VpsdState), C.POINTER(VpsdRound)]
    lib.hippo_vpsd_commit.argtypes = [C.POINTER(VpsdState), C.POINTER(VpsdRound), i32, i32]
    lib.hippo_vpsd_simulate.argtypes = [i32, i32, f64, f64, i32, vp, i64, i64, C.POINTER(VpsdResult)]
    for fn in (lib.hippo_vpsd_init, lib.hippo_vpsd_plan, lib.hippo_vpsd_commit, lib.hippo_vpsd_simulate):
        fn.restype = C.c_int
    lib.hippo_spec_verify_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.hippo_spec_verify_workspace_bytes.restype = C.c_size_t
    lib.hippo_spec_verify.argtypes = [vp, vp, i32, i64, i64, vp, vp, vp, i32, i32, i32, f32, vp, vp, vp, vp, sz, vp]
    lib.hippo_spec_verify.restype = C.c_int
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().hippo_status_string(int(status)).decode()


# ---------------------------------------------------------------------------------------------
# torch plumbing (device memory + streams)
# ---------------------------------------------------------------------------------------------

def _torch():
    import torch
    return torch


def _dtype_code(t) -> int:
    torch = _torch()
    if t.dtype == torch.float32:
        return DTYPE_F32
    if t.dtype == torch.bfloat16:
        return DTYPE_BF16
    if t.dtype in (torch.uint8, torch.float8_e4m3fn):       # E4M3 cache codes
        return DTYPE_FP8_E4M3
    raise TypeError("unsupported dtype %s (fp32, bf16, or uint8 / float8_e4m3fn cache codes)" % t.dtype)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def kv_desc(cache, n_q_heads: int) -> KvDesc:
    """Descriptor of a [B, H_kv, N, d] cache tensor (any strides with unit stride on d)."""
    assert cache.dim() == 4 and cache.stride(3) == 1
    B, Hkv, _, d = cache.shape
    return KvDesc(B, n_q_heads, Hkv, d, _dtype_code(cache), cache.stride(0), cache.stride(1), cache.stride(2))


def video_desc(n_frames, grid_h, grid_w, vis_offset, crop_h=5, crop_w=5) -> VideoDesc:
    return VideoDesc(n_frames, grid_h, grid_w, vis_offset, crop_h, crop_w)


def workspace_bytes(call: int, kv: KvDesc, vid: Optional[VideoDesc], n_rows: int, seq_len: int,
                    k: int = 0, num_splits: int = 0) -> int:
    return int(load().hippo_workspace_bytes(call, C.byref(kv), C.byref(vid) if vid is not None else None,
                                            n_rows, seq_len, k, num_splits))


def _on(stream):
    """Context in which the wrapper allocates what the caller did not pass (workspace, outputs): the
    stream the kernels are enqueued on.  torch's caching allocator ties a block to the stream that was
    current when it was allocated and may hand it out again, on that stream, as soon as the tensor is
    dropped; allocated under another stream than the kernels', a workspace could be recycled while they
    still use it."""
    return _torch().cuda.stream(stream) if stream is not None else contextlib.nullcontext()


def _allocates_on_its_stream(fn):
    """Run the marshalling of `fn` with its `stream=` argument as the current stream (see _on)."""
    import functools
    import inspect
    sig = inspect.signature(fn)

    @functools.wraps(fn)
    def wrapper(*args, **kwargs):
        stream = sig.bind(*args, **kwargs).arguments.get("stream")
        with _on(stream):
            return fn(*args, **kwargs)
    return wrapper


def _workspace(nbytes: int, device, workspace=None):
    torch = _torch()
    if workspace is not None:
        return workspace
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def _check(status: int, what: str):
    if status != OK:
        raise HippoError(status, what)


# ---------------------------------------------------------------------------------------------
# the four entry points
# ---------------------------------------------------------------------------------------------

@_allocates_on_its_stream
def hippo_score_tokens(q_txt, k_cache, vid: VideoDesc, emb=None, flags: int = SCORE_ALL,
                       attn_mass_inout=None, want_components: bool = False, scores_out=None, workspace=None,
                       stream=None):
    """q_txt [B,L,H,d], k_cache [B,Hkv,N,d] -> scores [B,N_v] fp32 (and components [3,B,N_v])."""
    torch = _torch()
    lib = load()
    assert q_txt.is_contiguous() and q_txt.dim() == 4
    B, L, H, d = q_txt.shape
    kv = kv_desc(k_cache, H)
    n_vis = vid.n_frames * vid.grid_h * vid.grid_w
    nbytes = workspace_bytes(CALL_SCORE_TOKENS, kv, vid, L, k_cache.shape[2])
    ws = _workspace(nbytes, q_txt.device, workspace)
    acc_only = bool(flags & SCORE_ACCUMULATE_ONLY)
    scores = scores_out
    if scores is None and not acc_only:
        scores = torch.empty((B, n_vis), dtype=torch.float32, device=q_txt.device)
    comps = torch.zeros((3, B, n_vis), dtype=torch.float32, device=q_txt.device) if want_components else None
    emb_dim, emb_stride = (0, 0) if emb is None else (emb.shape[2], emb.stride(1))
    if emb is not None:
        assert emb.dim() == 3 and emb.stride(2) == 1 and emb.stride(0) == emb.shape[1] * emb.stride(1)
    st = lib.hippo_score_tokens(_ptr(q_txt), L, _ptr(k_cache), C.byref(kv), k_cache.shape[2], C.byref(vid),
                                _ptr(emb), emb_dim, emb_stride, flags, _ptr(attn_mass_inout), _ptr(scores),
                                _ptr(comps), _ptr(ws), ws.numel(), _stream(stream))
    _check(st, "hippo_score_tokens")
    return (scores, comps) if want_components else scores


@_allocates_on_its_stream
def hippo_score_tokens_layers(q_txt_layers, k_cache_layers, vid: VideoDesc, emb_layer: int = 0, emb=None,
                              flags: int = SCORE_ALL, attn_mass_inout=None, want_components: bool = False,
                              scores_out=None, workspace=None, stream=None):
    """Eq. 2 with its sum over layers inside one call: lists of per-layer q_txt [B,L,H,d] and
    k_cache [B,Hkv,N,d] (same shapes and strides) -> scores [B,N_v] fp32 (and components)."""
    torch = _torch()
    lib = load()
    n_layers = len(q_txt_layers)
    assert n_layers == len(k_cache_layers) and n_layers >= 1
    q0, k0 = q_txt_layers[0], k_cache_layers[0]
    B, L, H, d = q0.shape
    for q, k in zip(q_txt_layers, k_cache_layers):
        assert q.is_contiguous() and q.shape == q0.shape and k.shape == k0.shape and k.stride() == k0.stride()
    kv = kv_desc(k0, H)
    n_vis = vid.n_frames * vid.grid_h * vid.grid_w
    nbytes = int(lib.hippo_score_layers_workspace_bytes(C.byref(kv), C.byref(vid), L, n_layers))
    ws = _workspace(nbytes, q0.device, workspace)
    acc_only = bool(flags & SCORE_ACCUMULATE_ONLY)
    scores = scores_out
    if scores is None and not acc_only:
        scores = torch.empty((B, n_vis), dtype=torch.float32, device=q0.device)
    comps = torch.zeros((3, B, n_vis), dtype=torch.float32, device=q0.device) if want_components else None
    emb_dim, emb_stride = (0, 0) if emb is None else (emb.shape[2], emb.stride(1))
    qs = (C.c_void_p * n_layers)(*[q.data_ptr() for q in q_txt_layers])
    ks = (C.c_void_p * n_layers)(*[k.data_ptr() for k in k_cache_layers])
    st = lib.hippo_score_tokens_layers(n_layers, C.cast(qs, C.c_void_p), L, C.cast(ks, C.c_void_p), emb_layer,
                                       C.byref(kv), k0.shape[2], C.byref(vid), _ptr(emb), emb_dim, emb_stride, flags,
                                       _ptr(attn_mass_inout), _ptr(scores), _ptr(comps), _ptr(ws), ws.numel(),
                                       _stream(stream))
    _check(st, "hippo_score_tokens_layers")
    return (scores, comps) if want_components else scores


@_allocates_on_its_stream
def hippo_select_gather_kv(scores, k: int, k_src, v_src, vid: VideoDesc, n_q_heads: Optional[int] = None,
                           gather: bool = True, idx_out=None, k_dst=None, v_dst=None, workspace=None, stream=None):
    """scores [B,N_v] fp32 -> (idx [B,k] int32, k_dst, v_dst [B,Hkv,N-N_v+k,d]).
    idx_out / k_dst / v_dst: optional preallocated outputs (k_dst, v_dst may be strided views)."""
    torch = _torch()
    lib = load()
    assert scores.dtype == torch.float32 and scores.is_contiguous()
    B, Hkv, N, d = k_src.shape
    n_vis = vid.n_frames * vid.grid_h * vid.grid_w
    H = n_q_heads or Hkv
    src = kv_desc(k_src, H)
    assert v_src.stride() == k_src.stride() and v_src.shape == k_src.shape
    idx = idx_out if idx_out is not None else torch.empty((B, k), dtype=torch.int32, device=scores.device)
    dst = None
    if gather:
        n_dst = N - n_vis + k
        if k_dst is None:
            k_dst = torch.empty((B, Hkv, max(n_dst, 0), d), dtype=k_src.dtype, device=k_src.device)
            v_dst = torch.empty_like(k_dst)
        assert k_dst.shape == (B, Hkv, n_dst, d) and v_dst.shape == k_dst.shape and v_dst.stride() == k_dst.stride()
        dst = kv_desc(k_dst, H)
    else:
        k_dst = v_dst = None
    ws = _workspace(256, scores.device, workspace)
    st = lib.hippo_select_gather_kv(_ptr(scores), k, _ptr(k_src), _ptr(v_src), C.byref(src), N, C.byref(vid),
                                    _ptr(k_dst), _ptr(v_dst), C.byref(dst) if dst is not None else None,
                                    _ptr(idx), _ptr(ws), ws.numel(), _stream(stream))
    _check(st, "hippo_select_gather_kv")
    return idx, k_dst, v_dst


@_allocates_on_its_stream
def _attention(fn_name, call, q, k_cache, v_cache, ctx_len, softmax_scale, num_splits, want_lse, out,
               workspace, stream, k_new=None, v_new=None):
    torch = _torch()
    lib = load()
    assert q.is_contiguous() and q.dim() == 4
    B, q_len, H, d = q.shape
    kv = kv_desc(k_cache, H)
    assert v_cache.stride() == k_cache.stride() and v_cache.shape == k_cache.shape
    nbytes = workspace_bytes(call, kv, None, q_len, ctx_len + q_len, 0, num_splits)
    ws = _workspace(nbytes, q.device, workspace)
    if out is None:
        out = torch.empty_like(q)
    lse = torch.empty((B, H, q_len), dtype=torch.float32, device=q.device) if want_lse else None
    if k_new is not None:
        fn_name += "_append"
        Hkv = k_cache.shape[1]
        for t in (k_new, v_new):
            assert t.shape == (B, q_len, Hkv, d) and t.is_contiguous() and t.dtype == k_cache.dtype
        st = getattr(lib, fn_name)(_ptr(q), q_len, _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                   C.byref(kv), ctx_len, float(softmax_scale or 0.0), num_splits, _ptr(out),
                                   _ptr(lse), _ptr(ws), ws.numel(), _stream(stream))
        _check(st, fn_name)
        return (out, lse) if want_lse else out
    st = getattr(lib, fn_name)(_ptr(q), q_len, _ptr(k_cache), _ptr(v_cache), C.byref(kv), ctx_len,
                               float(softmax_scale or 0.0), num_splits, _ptr(out), _ptr(lse), _ptr(ws),
                               ws.numel(), _stream(stream))
    _check(st, fn_name)
    return (out, lse) if want_lse else out


def hippo_verify_attention(q, k_cache, v_cache, ctx_len: int, softmax_scale: float = 0.0, num_splits: int = 0,
                           want_lse: bool = False, out=None, workspace=None, stream=None, k_new=None, v_new=None):
    """q [B,q_len,H,d]; caches hold ctx_len+q_len rows; row i attends to [0, ctx_len+i].
    With k_new / v_new [B,q_len,Hkv,d] the new rows are taken from there and appended to the caches
    by the same launch (hippo_verify_attention_append)."""
    return _attention("hippo_verify_attention", CALL_VERIFY_ATTENTION, q, k_cache, v_cache, ctx_len,
                      softmax_scale, num_splits, want_lse, out, workspace, stream, k_new, v_new)


def hippo_draft_attention(q, k_cache, v_cache, ctx_len: int, softmax_scale: float = 0.0, num_splits: int = 0,
                          want_lse: bool = False, out=None, workspace=None, stream=None, k_new=None, v_new=None):
    return _attention("hippo_draft_attention", CALL_DRAFT_ATTENTION, q, k_cache, v_cache, ctx_len,
                      softmax_scale, num_splits, want_lse, out, workspace, stream, k_new, v_new)


@_allocates_on_its_stream
def hippo_verify_attention_static(q, k_cache, v_cache, ctx_len: int, softmax_scale: float = 0.0, num_splits: int = 0,
                                  lse_out=None, out=None, stream=None):
    """hippo_verify_attention without a workspace: the split partials live in the library's own static
    device array (calls on one GPU must not overlap).  Pass `out` (and `lse_out`) to keep the whole call
    free of allocations."""
    torch = _torch()
    lib = load()
    assert q.is_contiguous() and q.dim() == 4
    B, q_len, H, d = q.shape
    kv = kv_desc(k_cache, H)
    assert v_cache.stride() == k_cache.stride() and v_cache.shape == k_cache.shape
    if out is None:
        out = torch.empty_like(q)
    st = lib.hippo_verify_attention_static(_ptr(q), q_len, _ptr(k_cache), _ptr(v_cache), C.byref(kv), ctx_len,
                                           float(softmax_scale or 0.0), num_splits, _ptr(out), _ptr(lse_out),
                                           _stream(stream))
    _check(st, "hippo_verify_attention_static")
    return out


@_allocates_on_its_stream
def _attention_fp8kv(fn_name, call, q, k_codes, v_codes, k_scale, v_scale, ctx_len, softmax_scale, num_splits,
                     want_lse, out, workspace, stream):
    torch = _torch()
    lib = load()
    assert q.is_contiguous() and q.dim() == 4 and q.dtype == torch.bfloat16
    B, q_len, H, d = q.shape
    assert k_codes.dim() == 4 and k_codes.stride(3) == 1 and k_codes.dtype in (torch.uint8, torch.float8_e4m3fn)
    assert v_codes.shape == k_codes.shape and v_codes.stride() == k_codes.stride() and v_codes.dtype == k_codes.dtype
    Hkv = k_codes.shape[1]
    for t in (k_scale, v_scale):
        assert t.shape == (B, Hkv) and t.is_contiguous() and t.dtype == torch.float32
    kv = KvDesc(B, H, Hkv, d, DTYPE_FP8_E4M3, k_codes.stride(0), k_codes.stride(1), k_codes.stride(2))
    nbytes = workspace_bytes(call, kv, None, q_len, ctx_len + q_len, 0, num_splits)
    ws = _workspace(nbytes, q.device, workspace)
    if out is None:
        out = torch.empty_like(q)
    lse = torch.empty((B, H, q_len), dtype=torch.float32, device=q.device) if want_lse else None
    st = getattr(lib, fn_name)(_ptr(q), q_len, _ptr(k_codes), _ptr(v_codes), _ptr(k_scale), _ptr(v_scale),
                               C.byref(kv), ctx_len, float(softmax_scale or 0.0), num_splits, _ptr(out), _ptr(lse),
                               _ptr(ws), ws.numel(), _stream(stream))
    _check(st, fn_name)
    return (out, lse) if want_lse else out


def hippo_verify_attention_fp8kv(q, k_codes, v_codes, k_scale, v_scale, ctx_len: int, softmax_scale: float = 0.0,
                                 num_splits: int = 0, want_lse: bool = False, out=None, workspace=None,
                                 stream=None):
    """q [B,q_len,H,d] bf16; k_codes / v_codes [B,Hkv,N,d] E4M3 bytes; k_scale / v_scale [B,Hkv] fp32."""
    return _attention_fp8kv("hippo_verify_attention_fp8kv", CALL_VERIFY_ATTENTION, q, k_codes, v_codes, k_scale,
                            v_scale, ctx_len, softmax_scale, num_splits, want_lse, out, workspace, stream)


def hippo_draft_attention_fp8kv(q, k_codes, v_codes, k_scale, v_scale, ctx_len: int, softmax_scale: float = 0.0,
                                num_splits: int = 0, want_lse: bool = False, out=None, workspace=None,
                                stream=None):
    return _attention_fp8kv("hippo_draft_attention_fp8kv", CALL_DRAFT_ATTENTION, q, k_codes, v_codes, k_scale,
                            v_scale, ctx_len, softmax_scale, num_splits, want_lse, out, workspace, stream)


@_allocates_on_its_stream
def hippo_quantize_kv_e4m3(k_src, v_src, n_rows: Optional[int] = None, k_codes=None, v_codes=None, workspace=None,
                           stream=None):
    """k_src / v_src [B,Hkv,N,d] bf16 or fp32 -> (k_codes, v_codes uint8 [B,Hkv,n_rows,d], k_scale, v_scale
    fp32 [B,Hkv]): the cache format of the *_fp8kv attention calls."""
    torch = _torch()
    lib = load()
    B, Hkv, N, d = k_src.shape
    n_rows = N if n_rows is None else n_rows
    assert v_src.shape == k_src.shape and v_src.stride() == k_src.stride() and 1 <= n_rows <= N
    src = kv_desc(k_src, Hkv)
    if k_codes is None:
        k_codes = torch.empty((B, Hkv, n_rows, d), dtype=torch.uint8, device=k_src.device)
        v_codes = torch.empty_like(k_codes)
    assert k_codes.shape[:2] == (B, Hkv) and k_codes.shape[3] == d and k_codes.shape[2] >= n_rows
    assert v_codes.shape == k_codes.shape and v_codes.stride() == k_codes.stride()
    dst = kv_desc(k_codes, Hkv)
    k_scale = torch.empty((B, Hkv), dtype=torch.float32, device=k_src.device)
    v_scale = torch.empty_like(k_scale)
    ws = _workspace(int(lib.hippo_quantize_kv_workspace_bytes(C.byref(src), n_rows)), k_src.device, workspace)
    st = lib.hippo_quantize_kv_e4m3(_ptr(k_src), _ptr(v_src), C.byref(src), n_rows, _ptr(k_codes), _ptr(v_codes),
                                    C.byref(dst), _ptr(k_scale), _ptr(v_scale), _ptr(ws), ws.numel(), _stream(stream))
    _check(st, "hippo_quantize_kv_e4m3")
    return k_codes, v_codes, k_scale, v_scale


@_allocates_on_its_stream
def _attention_paged(fn_name, call, q, k_pool, v_pool, block_table, ctx_len, softmax_scale, num_splits, want_lse,
                     out, workspace, stream):
    torch = _torch()
    lib = load()
    assert q.is_contiguous() and q.dim() == 4 and k_pool.dim() == 4 and k_pool.stride(3) == 1
    B, q_len, H, d = q.shape
    n_pages, page_size, Hkv, _ = k_pool.shape
    assert v_pool.shape == k_pool.shape and v_pool.stride() == k_pool.stride()
    assert block_table.dtype == torch.int32 and block_table.is_contiguous() and block_table.shape[0] == B
    pd = PagedKvDesc(B, H, Hkv, d, _dtype_code(k_pool), page_size, block_table.shape[1], n_pages,
                     k_pool.stride(0), k_pool.stride(1), k_pool.stride(2))
    flat = KvDesc(B, H, Hkv, d, _dtype_code(k_pool), 0, k_pool.stride(2), k_pool.stride(1))
    nbytes = workspace_bytes(call, flat, None, q_len, ctx_len + q_len, 0, num_splits)
    ws = _workspace(nbytes, q.device, workspace)
    if out is None:
        out = torch.empty_like(q)
    lse = torch.empty((B, H, q_len), dtype=torch.float32, device=q.device) if want_lse else None
    st = getattr(lib, fn_name)(_ptr(q), q_len, _ptr(k_pool), _ptr(v_pool), _ptr(block_table), C.byref(pd), ctx_len,
                               float(softmax_scale or 0.0), num_splits, _ptr(out), _ptr(lse), _ptr(ws), ws.numel(),
                               _stream(stream))
    _check(st, fn_name)
    return (out, lse) if want_lse else out


def hippo_verify_attention_paged(q, k_pool, v_pool, block_table, ctx_len: int, softmax_scale: float = 0.0,
                                 num_splits: int = 0, want_lse: bool = False, out=None, workspace=None, stream=None):
    """Pools [n_pages, page_size, Hkv, d]; block_table [B, max_pages] int32 on the device."""
    return _attention_paged("hippo_verify_attention_paged", CALL_VERIFY_ATTENTION, q, k_pool, v_pool, block_table,
                            ctx_len, softmax_scale, num_splits, want_lse, out, workspace, stream)


def hippo_draft_attention_paged(q, k_pool, v_pool, block_table, ctx_len: int, softmax_scale: float = 0.0,
                                num_splits: int = 0, want_lse: bool = False, out=None, workspace=None, stream=None):
    return _attention_paged("hippo_draft_attention_paged", CALL_DRAFT_ATTENTION, q, k_pool, v_pool, block_table,
                            ctx_len, softmax_scale, num_splits, want_lse, out, workspace, stream)


@_allocates_on_its_stream
def hippo_spec_verify(p_logits, q_logits, draft_tokens, u_accept, u_sample, temperature: float,
                      want_alpha: bool = False, n_accept_out=None, next_token_out=None, workspace=None,
                      stream=None):
    """p_logits [B,gamma+1,V] (rows may be padded: stride(1) >= V), q_logits [B,gamma,V] or None
    (greedy), draft_tokens [B,gamma] int32, u_accept [B,gamma] fp32, u_sample [B] fp32 ->
    (n_accept [B] int32, next_token [B] int32[, alpha [B,gamma] fp32])."""
    torch = _torch()
    lib = load()
    assert p_logits.dim() == 3 and p_logits.stride(2) == 1
    B, g1, V = p_logits.shape
    gamma = g1 - 1
    assert B == 1 or p_logits.stride(0) == g1 * p_logits.stride(1)
    q_stride = 0
    if gamma == 0:
        q_logits = draft_tokens = u_accept = None       # nothing to verify: a plain draw from p_0
    if q_logits is not None:
        assert q_logits.shape == (B, gamma, V) and q_logits.stride(2) == 1 and q_logits.dtype == p_logits.dtype
        assert B == 1 or q_logits.stride(0) == gamma * q_logits.stride(1)
        q_stride = q_logits.stride(1)
    for t, dt in ((draft_tokens, torch.int32), (u_accept, torch.float32), (u_sample, torch.float32)):
        assert t is None or (t.dtype == dt and t.is_contiguous())
    dev = p_logits.device
    n_acc = n_accept_out if n_accept_out is not None else torch.empty(B, dtype=torch.int32, device=dev)
    nxt = next_token_out if next_token_out is not None else torch.empty(B, dtype=torch.int32, device=dev)
    alpha = torch.empty((B, gamma), dtype=torch.float32, device=dev) if want_alpha else None
    code = _dtype_code(p_logits)
    ws = _workspace(int(lib.hippo_spec_verify_workspace_bytes(B, gamma, V, code)), dev, workspace)
    st = lib.hippo_spec_verify(_ptr(p_logits), _ptr(q_logits), code, p_logits.stride(1), q_stride,
                               _ptr(draft_tokens), _ptr(u_accept), _ptr(u_sample), B, gamma, V,
                               float(temperature), _ptr(n_acc), _ptr(nxt), _ptr(alpha), _ptr(ws), ws.numel(),
                               _stream(stream))
    _check(st, "hippo_spec_verify")
    return (n_acc, nxt, alpha) if want_alpha else (n_acc, nxt)


# ---------------------------------------------------------------------------------------------
# host-side control of video parallel speculative decoding (no GPU involved)
# ---------------------------------------------------------------------------------------------

def vpsd_prefill_buffer(t_prefill_target: float, t_prefill_draft: float, t_draft_token: float) -> int:
    return int(load().hippo_vpsd_prefill_buffer(t_prefill_target, t_prefill_draft, t_draft_token))


def vpsd_init(gamma: int, n_prefill_buffer: int = 0) -> VpsdState:
    s = VpsdState()
    _check(load().hippo_vpsd_init(C.byref(s), gamma, n_prefill_buffer), "hippo_vpsd_init")
    return s


def vpsd_plan(state: VpsdState) -> VpsdRound:
    r = VpsdRound()
    _check(load().hippo_vpsd_plan(C.byref(state), C.byref(r)), "hippo_vpsd_plan")
    return r


def vpsd_commit(state: VpsdState, rnd: VpsdRound, n_accept: int, n_drafted_parallel: Optional[int] = None) -> None:
    n = rnd.draft_parallel if n_drafted_parallel is None else n_drafted_parallel
    _check(load().hippo_vpsd_commit(C.byref(state), C.byref(rnd), n_accept, n), "hippo_vpsd_commit")


def vpsd_simulate(policy: int, gamma: int, t_draft: float, t_target: float, accept, n_tokens: int,
                  n_prefill_buffer: int = 0) -> VpsdResult:
    flags = bytes(bytearray(1 if a else 0 for a in accept))
    res = VpsdResult()
    buf = C.create_string_buffer(flags, len(flags)) if flags else None
    _check(load().hippo_vpsd_simulate(policy, gamma, t_draft, t_target, n_prefill_buffer,
                                      C.cast(buf, C.c_void_p) if buf is not None else None, len(flags), n_tokens,
                                      C.byref(res)), "hippo_vpsd_simulate")
    return res
