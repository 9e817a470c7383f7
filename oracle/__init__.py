"""ctypes front end of the CPU oracle (``hippo_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this package.  It never touches the HIP library and the HIP binding never touches it.

For the paper's own path the wrapper does argument marshalling only, plus the two input
re-arrangements the boundary defines (the "embedding = visual keys concatenated over KV heads"
default, and slicing the visual span out of a cache); that arithmetic is in the C file.  The 8-bit
cache format, which the paper does not mention, is written out here in numpy (float64):
`e4m3_decode`, `quantize_e4m3`, and `attention_fp8kv` over the dequantised cache through a dense
restatement of the attention definition (`_attention64`).  Pins: tests/test_oracle_pins.py,
tests/test_oracle_sd_pins.py, tests/test_oracle_fp8_pins.py; nothing here is "parity unpinned"
except against the authors' own code, which does not exist in public form.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hippo_oracle.c")
_LIB = os.path.join(_HERE, "libhippo_oracle.so")

FLAG_ATTN, FLAG_TEMP, FLAG_SPA = 1, 2, 4
FLAG_ALL = 7


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (float64, OpenMP over independent items)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
                               "-fno-fast-math", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


_I, _I64, _VP, _D, _U = C.c_int, C.c_int64, C.c_void_p, C.c_double, C.c_uint
_SIGS = {
    "hippo_oracle_s_attn": [_VP, _I, _I, _I, _I, _I, _VP, _I64, _I64, _I, _VP],
    "hippo_oracle_s_temp": [_VP, _I, _I, _I, _I, _I64, _I64, _VP],
    "hippo_oracle_s_spa": [_VP, _I, _I, _I, _I, _I, _I, _I, _I64, _I64, _VP],
    "hippo_oracle_fuse": [_VP, _VP, _VP, _U, _I, _I, _I, _VP],
    "hippo_oracle_topk": [_VP, _I, _I, _I, _VP],
    "hippo_oracle_gather": [_VP, _I, _I, _I, _I, _I, _I, _VP, _I, _VP],
    "hippo_oracle_attention": [_VP, _I, _I, _I, _I, _I, _VP, _VP, _I64, _I64, _I, _D, _VP, _VP],
    "hippo_oracle_spec_verify": [_VP, _VP, _VP, _VP, _VP, _I, _I, _I, _D, _VP, _VP, _VP],
}


def _L():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        for name, sig in _SIGS.items():
            fn = getattr(lib, name)
            fn.argtypes = sig
            fn.restype = None
        lib.hippo_oracle_threads.restype = C.c_int
        _lib = lib
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _i(x) -> int:
    return int(x)


def threads() -> int:
    return int(_L().hippo_oracle_threads())


def s_attn(q_txt: np.ndarray, k_cache: np.ndarray, vis_off: int, n_vis: int) -> np.ndarray:
    """Eq. 2.  q_txt [B,L,H,d], k_cache [B,Hkv,N,d] -> [B,N_v] float64."""
    q_txt, k_cache = _f32(q_txt), _f32(k_cache)
    B, L, H, d = q_txt.shape
    _, Hkv, N, _ = k_cache.shape
    k_vis = np.ascontiguousarray(k_cache[:, :, vis_off:vis_off + n_vis, :])
    out = np.zeros((B, n_vis), dtype=np.float64)
    _L().hippo_oracle_s_attn(_p(q_txt), B, L, H, Hkv, d, _p(k_vis),
                             C.c_int64(Hkv * n_vis * d), C.c_int64(n_vis * d), n_vis, _p(out))
    return out


def keys_as_embedding(k_cache: np.ndarray, vis_off: int, n_vis: int) -> np.ndarray:
    """The boundary's default embedding: token j's vector is its keys of all KV heads,
    concatenated in head order.  [B,Hkv,N,d] -> [B,N_v,Hkv*d]."""
    k_cache = _f32(k_cache)
    B, Hkv, N, d = k_cache.shape
    kv = k_cache[:, :, vis_off:vis_off + n_vis, :]
    return np.ascontiguousarray(kv.transpose(0, 2, 1, 3)).reshape(B, n_vis, Hkv * d)


def s_temp(emb: np.ndarray, n_frames: int) -> np.ndarray:
    """Eq. 3-4.  emb [B,N_v,de] -> [B,N_v] float64."""
    emb = _f32(emb)
    B, Nv, de = emb.shape
    P = Nv // n_frames
    out = np.zeros((B, Nv), dtype=np.float64)
    _L().hippo_oracle_s_temp(_p(emb), B, n_frames, P, de, C.c_int64(Nv * de), C.c_int64(de), _p(out))
    return out


def s_spa(emb: np.ndarray, n_frames: int, grid_h: int, grid_w: int, crop_h: int = 5,
          crop_w: int = 5) -> np.ndarray:
    """Eq. 5-6.  emb [B,N_v,de] -> [B,N_v] float64."""
    emb = _f32(emb)
    B, Nv, de = emb.shape
    assert Nv == n_frames * grid_h * grid_w
    out = np.zeros((B, Nv), dtype=np.float64)
    _L().hippo_oracle_s_spa(_p(emb), B, _i(n_frames), _i(grid_h), _i(grid_w), _i(crop_h), _i(crop_w), de,
                            C.c_int64(Nv * de), C.c_int64(de), _p(out))
    return out


def fuse(sa: np.ndarray, st: np.ndarray, ss: np.ndarray, n_frames: int,
         flags: int = FLAG_ALL) -> np.ndarray:
    """Eq. 7.  three [B,N_v] float64 -> [B,N_v] float64."""
    sa = np.ascontiguousarray(sa, dtype=np.float64)
    st = np.ascontiguousarray(st, dtype=np.float64)
    ss = np.ascontiguousarray(ss, dtype=np.float64)
    B, Nv = sa.shape
    out = np.zeros((B, Nv), dtype=np.float64)
    _L().hippo_oracle_fuse(_p(sa), _p(st), _p(ss), C.c_uint(flags), B, n_frames, Nv // n_frames, _p(out))
    return out


def score_tokens(q_txt, k_cache, vis_off, n_frames, grid_h, grid_w, crop_h=5, crop_w=5,
                 emb: Optional[np.ndarray] = None, flags: int = FLAG_ALL
                 ) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 2-7 end to end.  Returns (scores [B,N_v], components [3,B,N_v]) in float64."""
    n_vis = n_frames * grid_h * grid_w
    if emb is None:
        emb = keys_as_embedding(k_cache, vis_off, n_vis)
    sa = s_attn(q_txt, k_cache, vis_off, n_vis)
    st = s_temp(emb, n_frames)
    ss = s_spa(emb, n_frames, grid_h, grid_w, crop_h, crop_w)
    return fuse(sa, st, ss, n_frames, flags), np.stack([sa, st, ss])


def topk(scores: np.ndarray, k: int) -> np.ndarray:
    """Top-k of fp32 scores, ties to the lower index, output ascending.  [B,N] -> [B,k] int32."""
    scores = _f32(scores)
    B, N = scores.shape
    idx = np.full((B, k), -1, dtype=np.int32)
    _L().hippo_oracle_topk(_p(scores), B, N, k, _p(idx))
    return idx


def gather(src: np.ndarray, vis_off: int, n_vis: int, idx: np.ndarray) -> np.ndarray:
    """[B,Hkv,N,d] -> [B,Hkv,N-N_v+k,d] (prefix | kept visual rows | rest), bit copy."""
    src = _f32(src)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    B, Hkv, N, d = src.shape
    k = idx.shape[1]
    dst = np.empty((B, Hkv, N - n_vis + k, d), dtype=np.float32)
    _L().hippo_oracle_gather(_p(src), B, Hkv, N, d, vis_off, n_vis, _p(idx), k, _p(dst))
    return dst


def attention(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, ctx_len: int,
              scale: Optional[float] = None) -> Tuple[np.ndarray, np.ndarray]:
    """q [B,q_len,H,d]; caches [B,Hkv,>=ctx_len+q_len,d].  Row i sees entries [0, ctx_len+i].
    Returns (out [B,q_len,H,d], lse [B,H,q_len]) in float64."""
    q, k_cache, v_cache = _f32(q), _f32(k_cache), _f32(v_cache)
    B, q_len, H, d = q.shape
    _, Hkv, N, _ = k_cache.shape
    assert N >= ctx_len + q_len and v_cache.shape == k_cache.shape
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.zeros((B, q_len, H, d), dtype=np.float64)
    lse = np.zeros((B, H, q_len), dtype=np.float64)
    _L().hippo_oracle_attention(_p(q), B, q_len, H, Hkv, d, _p(k_cache), _p(v_cache),
                                C.c_int64(Hkv * N * d), C.c_int64(N * d), ctx_len,
                                C.c_double(scale), _p(out), _p(lse))
    return out, lse


def _attention64(q: np.ndarray, k: np.ndarray, v: np.ndarray, ctx_len: int,
                 scale: Optional[float]) -> Tuple[np.ndarray, np.ndarray]:
    """The same definition as `attention` for float64 caches, as dense numpy operations:
    per head, z = scale * q K^T, entries beyond ctx_len + i masked for row i, softmax, times V."""
    B, q_len, H, d = q.shape
    _, Hkv, N, _ = k.shape
    assert N >= ctx_len + q_len and v.shape == k.shape and H % Hkv == 0
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    n = ctx_len + q_len
    visible = np.arange(n)[None, :] <= ctx_len + np.arange(q_len)[:, None]
    out = np.zeros((B, q_len, H, d), dtype=np.float64)
    lse = np.zeros((B, H, q_len), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            hk = h // (H // Hkv)
            z = scale * (q[b, :, h, :] @ k[b, hk, :n, :].T)
            z = np.where(visible, z, -np.inf)
            zmax = z.max(axis=1, keepdims=True)
            w = np.exp(z - zmax)
            denom = w.sum(axis=1, keepdims=True)
            out[b, :, h, :] = (w / denom) @ v[b, hk, :n, :]
            lse[b, h, :] = (zmax + np.log(denom))[:, 0]
    return out, lse


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    """8-bit floating-point codes, 1 sign / 4 exponent / 3 mantissa bits, exponent bias 7, the
    finite-only variant (OCP 8-bit floating point specification, E4M3: no infinities; exponent 15
    with mantissa 7 is NaN; exponent 0 is subnormal) -> float64, written out from that definition.
    A format the paper does not mention: it serves the fp8 cache variant of the attention calls."""
    c = np.ascontiguousarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c >> 7 == 1, -1.0, 1.0)
    e = (c >> 3) & 15
    m = (c & 7).astype(np.float64)
    normal = (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))
    subnormal = (m / 8.0) * 2.0 ** -6
    val = np.where(e == 0, subnormal, normal)
    val = np.where((e == 15) & (m == 7), np.nan, val)
    return sign * val


def quantize_e4m3(x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """[B,Hkv,N,d] -> (E4M3 codes uint8 of the same shape, multipliers float32 [B,Hkv]).
    Per (batch element, KV head): multiplier = max|x| / 448 in float32 (1 when the maximum is 0);
    code = the E4M3 value nearest to x / multiplier (float32 division), ties to the even code
    (the rule of IEEE 754 applied to the format's 3-bit mantissa).  Written out as a search over the
    decoded magnitudes, whose order is the order of their codes."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    amax = np.abs(x).max(axis=(2, 3)).astype(np.float32)
    mult = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    y = (x / mult[:, :, None, None]).astype(np.float32)
    mags = e4m3_decode(np.arange(127, dtype=np.uint8))          # 0 .. 448, increasing
    a = np.abs(y).astype(np.float64)
    hi = np.clip(np.searchsorted(mags, a, side="left"), 1, 126)
    lo = hi - 1
    d_lo, d_hi = a - mags[lo], mags[hi] - a
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    code = np.where(a >= 448.0, np.uint8(126), code)             # the maximum maps to the largest code
    return (code | (np.signbit(y).astype(np.uint8) << 7)).astype(np.uint8), mult


def attention_fp8kv(q: np.ndarray, k_codes: np.ndarray, v_codes: np.ndarray, k_scale: np.ndarray,
                    v_scale: np.ndarray, ctx_len: int, scale: Optional[float] = None
                    ) -> Tuple[np.ndarray, np.ndarray]:
    """The attention call over a cache stored as E4M3 codes with one fp32 multiplier per (batch
    element, KV head): the cache entry is multiplier * decoded code, and the result is `attention`
    (paper: Preliminaries, "Speculative Decoding") of those entries.  k_codes / v_codes
    [B,Hkv,N,d] uint8, k_scale / v_scale [B,Hkv]."""
    ks = np.asarray(k_scale, dtype=np.float64)[:, :, None, None]
    vs = np.asarray(v_scale, dtype=np.float64)[:, :, None, None]
    k = e4m3_decode(k_codes) * ks
    v = e4m3_decode(v_codes) * vs
    # every product of a code value (4 significant bits) and an fp32 multiplier is exact in float64;
    # `attention` takes float32 caches, so feed it through the float64 entry below
    return _attention64(np.asarray(q, dtype=np.float64), k, v, ctx_len, scale)


def spec_verify(p_logits: np.ndarray, q_logits: Optional[np.ndarray], tokens: np.ndarray,
                u_accept: np.ndarray, u_sample: np.ndarray, temperature: float
                ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Eq. 1 + resampling.  p_logits [B,gamma+1,V], q_logits [B,gamma,V] (None allowed when
    temperature == 0), tokens [B,gamma] int32, u_accept [B,gamma], u_sample [B].
    Returns (n_accept [B] int32, next_token [B] int32, alpha [B,gamma] float64)."""
    p_logits = _f32(p_logits)
    B, g1, V = p_logits.shape
    gamma = g1 - 1
    tokens = np.ascontiguousarray(tokens, dtype=np.int32).reshape(B, gamma)
    assert tokens.min(initial=0) >= 0 and tokens.max(initial=0) < V
    if q_logits is not None:
        q_logits = _f32(q_logits)
        assert q_logits.shape == (B, gamma, V)
    else:
        assert temperature == 0
    u_accept = _f32(u_accept).reshape(B, gamma)
    u_sample = _f32(u_sample).reshape(B)
    n_acc = np.zeros(B, dtype=np.int32)
    nxt = np.full(B, -1, dtype=np.int32)
    alpha = np.zeros((B, gamma), dtype=np.float64)
    _L().hippo_oracle_spec_verify(_p(p_logits), None if q_logits is None else _p(q_logits), _p(tokens),
                                  _p(u_accept), _p(u_sample), B, gamma, V, C.c_double(temperature),
                                  _p(n_acc), _p(nxt), _p(alpha))
    return n_acc, nxt, alpha
